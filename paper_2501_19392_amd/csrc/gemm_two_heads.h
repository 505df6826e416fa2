// bf16 MFMA main loop of the linear predictors (Sect. 3.2 of the AQUA-KV paper) on a tile of
// 256 token rows x 256 outputs = TWO kv heads, for eight wavefronts (two per SIMD).
//
// Same instruction (v_mfma_f32_32x32x16_bf16), same operand layout in LDS, same direct-to-LDS loads and the same
// K order per output as gemm_core.h, hence the same bits; what changes is the shape.  Wave w owns the 64 token rows
// 64 (w / 2) ... and the 128 outputs of head w % 2: per 16 k it reads 2 + 4 operand fragments for 8 MFMAs
// (0.75 reads per MFMA against 1.25 for 32 rows x 128 outputs), and a k-tile brings (256 + 256) rows into LDS for
// 65536 outputs (against 384 rows for 32768), a third less traffic from L2 per output.  The price is LDS: a k-tile is
// 64 KiB, so the ring has two stages, and a wave holds 128 accumulator registers.
#pragma once
#include "gemm_core.h"

namespace aquakv {

constexpr int BM2 = 256, BN2 = 256;                  // block tile; BK as in gemm_core.h
constexpr int kATile2Bytes = BM2 * kRowBytes;        // 32 KiB
constexpr int kStage2Bytes = (BM2 + BN2) * kRowBytes;   // 64 KiB
constexpr int kMainLoop2LdsBytes = 2 * kStage2Bytes; // 128 KiB
constexpr int kWaves2 = 8;

// acc[i][j]: the 32 x 32 block at token rows 64 (wave / 2) + 32 i, outputs 128 (wave % 2) + 32 j of the tile; inside
// it the lane holds output column lane % 32 and rows 8 blk + 4 (lane / 32) + r in register 4 blk + r (as gemm_core.h).
// `lds_base` points at kMainLoop2LdsBytes bytes of LDS.  The last barrier comes after the last LDS read, so the caller
// may reuse the LDS at once.  Requires
// K = d0 + d1 a multiple of 128, d0 of 64.  `before_drain()` is called once, when the last operand loads are out.
//
// Schedule.  k-tile t lives in stage t % 2 and is multiplied in four steps of 16 k (8 MFMAs per wave each) from two
// fragment buffers: a step's MFMAs run while the next step's fragments are read.  Per tile t:
//   MFMAs (t, 0)   + fragment reads (t, 1)
//   MFMAs (t, 1)   + fragment reads (t, 2)
//   MFMAs (t, 2)   + fragment reads (t, 3)
//   barrier B_{t+1}: tile t + 1 complete in LDS, every wave done reading tile t
//   MFMAs (t, 3)   + fragment reads (t + 1, 0) + the 8 loads of tile t + 2 (into the stage tile t leaves)
// so a load has a whole tile of both waves of a SIMD (about 1 us) to land, the matrix pipe keeps running across the
// barrier, and the fragments take 48 registers beside the 128 accumulators.
template <typename BeforeDrain>
__device__ __forceinline__ void gemm_mainloop_two_heads(unsigned char* lds_base, const bf16_t* __restrict__ x0, int d0,
                                                        const bf16_t* __restrict__ x1, int d1,
                                                        const bf16_t* __restrict__ W, int64_t T, int64_t m0, int n0,
                                                        f32x16 (&acc)[2][4], BeforeDrain&& before_drain) {
  constexpr int kThreadsW = kWaves2 * 64;
  constexpr int MI = 2;
  constexpr int kAChunks = BM2 * 8 / kThreadsW;    // 4 load instructions per thread and k-tile for x
  constexpr int kBChunks = BN2 * 8 / kThreadsW;    // 4 for W
  constexpr int kPieces = kAChunks + kBChunks;
  constexpr int kPieceBytes = kThreadsW * 16;      // 8 KiB = 64 tile rows
  constexpr int kFragPieces = MI + 4;
  constexpr int kMma = MI * 4;
  typedef __attribute__((address_space(3))) unsigned char* lptr_t;
  typedef const __attribute__((address_space(1))) char* gptr_t;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ws = wave >> 1, wh = wave & 1;
  const int K = d0 + d1;
  const int nk = K / BK;

  struct Frag { bf16x8 v[kFragPieces]; };

  const int ch16 = ((tid & 7) ^ ((tid >> 4) & 7)) * 16;
  int rowc[kAChunks];
  uint32_t offB[kBChunks];
  {
    const int last = (int)((T - 1 - m0) < (BM2 - 1) ? (T - 1 - m0) : (BM2 - 1));
#pragma unroll
    for (int pc = 0; pc < kAChunks; ++pc) {
      const int row = (tid >> 3) + pc * (kThreadsW / 8);
      rowc[pc] = row < last ? row : last;
    }
#pragma unroll
    for (int pc = 0; pc < kBChunks; ++pc)
      offB[pc] = (uint32_t)((tid >> 3) + pc * (kThreadsW / 8)) * (uint32_t)(K * 2) + ch16;
  }
  const char* const wbase = reinterpret_cast<const char*>(W) + (int64_t)n0 * K * 2;
  const auto uniform_ptr = [](const char* p) {
    const uint64_t u = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)u);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(u >> 32));
    return (gptr_t)(((uint64_t)hi << 32) | lo);
  };
  const lptr_t lds3 = (lptr_t)lds_base;
  auto load_piece = [&](int kt, int stage_off, int pc) {
    const int k0 = kt * BK;
    const lptr_t dst = lds3 + (stage_off + pc * kPieceBytes + wave * 1024);   // x pieces fill the A tile, W pieces follow
    if (pc < kAChunks) {
      const bool second = k0 >= d0;
      const int ld2 = __builtin_amdgcn_readfirstlane((second ? d1 : d0) * 2);
      const gptr_t base = uniform_ptr(reinterpret_cast<const char*>(second ? x1 : x0) +
                                      (m0 * ld2 + (int64_t)(second ? k0 - d0 : k0) * 2));
      const uint32_t off = (uint32_t)__umul24(rowc[pc], ld2) + ch16;
      __builtin_amdgcn_global_load_lds(base + off, dst, 16, 0, 0);
    } else {
      const gptr_t base = uniform_ptr(wbase + (int64_t)k0 * 2);
      __builtin_amdgcn_global_load_lds(base + offB[pc - kAChunks], dst, 16, 0, 0);
    }
  };
  const int frow = lane & 31;
  const int fk = lane >> 5;
  auto frag_piece = [&](int stage_off, int ks, Frag& f, int pc) {
    const int off = pc < MI ? lds_off(ws * (MI * 32) + pc * 32 + frow, ks * 2 + fk)
                            : kATile2Bytes + lds_off(wh * 128 + (pc - MI) * 32 + frow, ks * 2 + fk);
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
  // publish a k-tile: this wave's loads have landed, its LDS reads have returned; then meet the other waves
  auto publish = [&] {
    __builtin_amdgcn_s_waitcnt(0x0070);                    // vmcnt(0) lgkmcnt(0)
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
  };

  Frag f[2];
#pragma unroll
  for (int pc = 0; pc < kPieces; ++pc) load_piece(0, 0, pc);
#pragma unroll
  for (int pc = 0; pc < kPieces; ++pc) load_piece(1, kStage2Bytes, pc);          // nk >= 2
  __builtin_amdgcn_s_waitcnt(0x0070 | (kPieces & 15) | ((kPieces >> 4) << 14));  // tile 0 has landed, tile 1 may be in flight
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
#pragma unroll
  for (int pc = 0; pc < kFragPieces; ++pc) frag_piece(0, 0, f[0], pc);
  __builtin_amdgcn_sched_barrier(0);

  // tile t in the stage at `cur`; `next_tile`: tile t + 1 exists; `do_load`: tile t + 2 exists
  auto tile = [&](int t, int cur, bool next_tile, bool do_load) {
    mma8(f[0], [&](int m) { spread(m, kFragPieces, [&](int e) { frag_piece(cur, 1, f[1], e); }); });
    mma8(f[1], [&](int m) { spread(m, kFragPieces, [&](int e) { frag_piece(cur, 2, f[0], e); }); });
    mma8(f[0], [&](int m) { spread(m, kFragPieces, [&](int e) { frag_piece(cur, 3, f[1], e); }); });
    publish();
    mma8(f[1], [&](int m) {
      spread(m, kFragPieces + kPieces, [&](int e) {
        if (e < kFragPieces) { if (next_tile) frag_piece(cur ^ kStage2Bytes, 0, f[0], e); }
        else if (do_load) load_piece(t + 2, cur, e - kFragPieces);
      });
    });
  };

  int cur = 0, t = 0;
  for (; t + 2 < nk; ++t) {
    tile(t, cur, true, true);
    cur ^= kStage2Bytes;
  }
  before_drain();
  __builtin_amdgcn_sched_barrier(0);
  tile(t, cur, true, false);                               // the last two tiles: nothing left to load
  cur ^= kStage2Bytes;
  tile(t + 1, cur, false, false);
}

}  // namespace aquakv
