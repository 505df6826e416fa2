// bf16 MFMA main loop of the linear predictors (Sect. 3.2 of the AQUA-KV paper) on a tile of 64 token rows x ALL 1024
// outputs (8 kv heads x 128), for eight wavefronts: wave h owns head h.  This is the shape the encoder needs when the
// rotation group is the whole token (Sect. 4.1: groups of 1024): scale and the butterfly stages across the heads want
// all 8 heads of a token in one workgroup.
//
// Same instruction (v_mfma_f32_32x32x16_bf16), operand orientation and K order per output as gemm_core.h, hence the
// same bits.  What differs: a k-tile is 32 wide (64-byte LDS rows, 4 chunks of 16 bytes) so that the 1024 rows of W
// plus the 64 token rows are 68 KiB and two stages fit; every workgroup streams the whole of W from L2 (about 68 bytes
// per clock and CU at full matrix rate, which is what a CU can take from L2), so the loop is as much an L2 as a matrix
// loop; a wave reads 2 + 4 operand fragments per 8 MFMAs.
//
// W is read from a re-tiled copy (retile_w_kernel in fused_wide_encode.hip writes it into the call's workspace; a
// few microseconds for 2 - 4 MiB): k-tile after k-tile, each the 64 KiB image of its LDS tile, swizzle included.  A load
// instruction of a wave then copies 1 KiB of consecutive bytes, whole 128-byte lines, instead of sixteen 64-byte
// pieces 2 or 4 KiB apart (half lines, which halve what L2 delivers per request).
#pragma once
#include "gemm_core.h"

namespace aquakv {

constexpr int kSlabRows = 64;                          // token rows of a tile
constexpr int kSlabCols = 1024;                        // outputs of a tile = 8 heads x 128
constexpr int kSlabBK = 32;
constexpr int kSlabRowBytes = kSlabBK * 2;             // 64 B of bf16 per LDS row
constexpr int kSlabATileBytes = kSlabRows * kSlabRowBytes;            // 4 KiB
constexpr int kSlabStageBytes = (kSlabRows + kSlabCols) * kSlabRowBytes;   // 68 KiB
constexpr int kSlabLdsBytes = 2 * kSlabStageBytes;                    // 136 KiB
constexpr int kSlabWaves = 8;
constexpr int kSlabBTileBytes = kSlabCols * kSlabRowBytes;              // 64 KiB: one k-tile of W, in LDS and in the re-tiled copy

// 16-byte chunk `ch` (0..3) of LDS row `row`.  A row is 64 B = a quarter of the 64 banks, so rows 4 apart would meet in
// the same banks; the chunk is XOR-ed with (row / 4) % 4, and the 16 lanes served together by a 128-bit fragment read
// (16 consecutive rows, same chunk) touch all 64 banks once.
__device__ __forceinline__ int slab_lds_off(int row, int ch) { return row * kSlabRowBytes + ((ch ^ ((row >> 2) & 3)) << 4); }

// acc[i][j]: the 32 x 32 block at token rows 32 i, outputs 128 wave + 32 j of the tile; inside it the lane holds output
// column lane % 32 and rows 8 blk + 4 (lane / 32) + r in register 4 blk + r (as gemm_core.h).
// `lds_base` points at kSlabLdsBytes bytes of LDS.  The last barrier comes after the last LDS read, so the caller may
// reuse the LDS at once.  Requires K = d0 + d1 a multiple of 128, d0 of 64.  `Wt`: the re-tiled copy of the 1024 x K weights.
// `before_drain()` is called once, when the last operand loads are out.
//
// Schedule.  k-tile t lives in stage t % 2 and is multiplied in two steps of 16 k (8 MFMAs per wave each) from two
// fragment buffers:
//   MFMAs (t, 0)   + fragment reads (t, 1)
//   barrier B_{t+1}: tile t + 1 complete in LDS, every wave done reading tile t
//   MFMAs (t, 1)   + fragment reads (t + 1, 0) + the loads of tile t + 2 (into the stage tile t leaves)
// A wave loads the 128 rows of W it multiplies itself (8 load instructions per k-tile); waves 0..3 add the 64 token rows.
template <typename BeforeDrain>
__device__ __forceinline__ void gemm_mainloop_token_slab(unsigned char* lds_base, const bf16_t* __restrict__ x0, int d0,
                                                         const bf16_t* __restrict__ x1, int d1,
                                                         const bf16_t* __restrict__ Wt, int64_t T, int64_t m0,
                                                         f32x16 (&acc)[2][4], BeforeDrain&& before_drain) {
  constexpr int MI = 2;
  constexpr int kBLoads = 128 / 16;                // load instructions per wave and k-tile for its rows of W (16 rows each)
  constexpr int kFragPieces = MI + 4;
  constexpr int kMma = MI * 4;
  typedef __attribute__((address_space(3))) unsigned char* lptr_t;
  typedef const __attribute__((address_space(1))) char* gptr_t;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int K = d0 + d1;
  const int nk = K / kSlabBK;
  const bool loads_x = wave < kSlabRows / 16;      // waves 0..3: 16 token rows each

  struct Frag { bf16x8 v[kFragPieces]; };

  // One load instruction of a wave fills 1 KiB of LDS = 16 rows of 64 B: lane l -> row l / 4, slot l % 4, and fetches
  // from global memory the chunk that belongs in its slot.
  const int lrow = lane >> 2;                                        // 0..15
  const int chunk = (lane & 3) ^ ((lrow >> 2) & 3);                  // rows of a piece start at a multiple of 16
  const int last = (int)((T - 1 - m0) < (kSlabRows - 1) ? (T - 1 - m0) : (kSlabRows - 1));
  const int xrow = (wave * 16 + lrow) < last ? (wave * 16 + lrow) : last;        // token row of this lane (waves 0..3), clamped
  const uint32_t offW = (uint32_t)(wave * 128 * kSlabRowBytes + lane * 16);      // + pc KiB: the image of the wave's rows
  const char* const wbase = reinterpret_cast<const char*>(Wt);
  const auto uniform_ptr = [](const char* p) {
    const uint64_t u = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)u);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(u >> 32));
    return (gptr_t)(((uint64_t)hi << 32) | lo);
  };
  const lptr_t lds3 = (lptr_t)lds_base;
  // piece pc of tile kt: pc < 8: rows 128 wave + 16 pc ... of W; pc == 8 (waves 0..3): token rows 16 wave ...
  auto load_piece = [&](int kt, int stage_off, int pc) {
    const int k0 = kt * kSlabBK;
    if (pc < kBLoads) {
      const lptr_t dst = lds3 + (stage_off + kSlabATileBytes + (wave * 128 + pc * 16) * kSlabRowBytes);
      const gptr_t base = uniform_ptr(wbase + (int64_t)kt * kSlabBTileBytes);
      __builtin_amdgcn_global_load_lds(base + (offW + (uint32_t)pc * 1024u), dst, 16, 0, 0);
    } else {
      const lptr_t dst = lds3 + (stage_off + wave * 16 * kSlabRowBytes);
      const bool second = k0 >= d0;
      const int ld2 = __builtin_amdgcn_readfirstlane((second ? d1 : d0) * 2);
      const gptr_t base = uniform_ptr(reinterpret_cast<const char*>(second ? x1 : x0) +
                                      (m0 * ld2 + (int64_t)(second ? k0 - d0 : k0) * 2));
      __builtin_amdgcn_global_load_lds(base + ((uint32_t)__umul24(xrow, ld2) + chunk * 16), dst, 16, 0, 0);
    }
  };
  auto load_tile = [&](int kt, int stage_off) {
#pragma unroll
    for (int pc = 0; pc < kBLoads; ++pc) load_piece(kt, stage_off, pc);
    if (loads_x) load_piece(kt, stage_off, kBLoads);
  };
  const int frow = lane & 31;
  const int fk = lane >> 5;
  auto frag_piece = [&](int stage_off, int ks, Frag& f, int pc) {
    const int off = pc < MI ? slab_lds_off(pc * 32 + frow, ks * 2 + fk)
                            : kSlabATileBytes + slab_lds_off(wave * 128 + (pc - MI) * 32 + frow, ks * 2 + fk);
    f.v[pc] = *reinterpret_cast<const bf16x8*>(lds_base + stage_off + off);
  };

#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  auto mma8 = [&](const Frag& f, auto&& extra) {
#pragma unroll
    for (int m = 0; m < kMma; ++m) {
      const int i = m >> 2, j = m & 3;
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.v[i], f.v[MI + j], acc[i][j], 0, 0, 0);
      extra(m);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  auto spread = [&](int m, int n, auto&& item) {
    if (2 * m < n) item(2 * m);
    if (2 * m + 1 < n) item(2 * m + 1);
  };
  auto publish = [&] {
    __builtin_amdgcn_s_waitcnt(0x0070);                    // vmcnt(0) lgkmcnt(0)
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
  };

  Frag f[2];
  load_tile(0, 0);
  load_tile(1, kSlabStageBytes);                           // nk >= 4
  // tile 0 has landed when at most this wave's loads of tile 1 are still in flight
  if (loads_x) __builtin_amdgcn_s_waitcnt(0x0070 | (kBLoads + 1));
  else __builtin_amdgcn_s_waitcnt(0x0070 | kBLoads);
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
#pragma unroll
  for (int pc = 0; pc < kFragPieces; ++pc) frag_piece(0, 0, f[0], pc);
  __builtin_amdgcn_sched_barrier(0);

  // tile t in the stage at `cur`; `next_tile`: tile t + 1 exists; `do_load`: tile t + 2 exists
  auto tile = [&](int t, int cur, bool next_tile, bool do_load) {
    mma8(f[0], [&](int m) { spread(m, kFragPieces, [&](int e) { frag_piece(cur, 1, f[1], e); }); });
    publish();
    mma8(f[1], [&](int m) {
      spread(m, kFragPieces + kBLoads + 1, [&](int e) {
        if (e < kFragPieces) { if (next_tile) frag_piece(cur ^ kSlabStageBytes, 0, f[0], e); }
        else if (do_load && (e - kFragPieces < kBLoads || loads_x)) load_piece(t + 2, cur, e - kFragPieces);
      });
    });
  };

  int cur = 0, t = 0;
  for (; t + 2 < nk; ++t) {
    tile(t, cur, true, true);
    cur ^= kSlabStageBytes;
  }
  before_drain();
  __builtin_amdgcn_sched_barrier(0);
  tile(t, cur, true, false);                               // the last two tiles: nothing left to load
  cur ^= kSlabStageBytes;
  tile(t + 1, cur, false, false);
}

}  // namespace aquakv
