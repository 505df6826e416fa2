// bf16 MFMA main loop of the linear predictors (Sect. 3.2 of the AQUA-KV paper):
// acc[256 x 128 tile] = [x0 | x1] W^T for one workgroup, shared by the stand-alone
// predictor kernel and by the fused encode / decode / scoring kernels.
//
// v_mfma_f32_32x32x16_bf16, fp32 accumulate.  Both operands are K-contiguous (x is [T, K],
// W is [D, K]), so A and B fragments are 128-bit LDS reads.  Every output accumulates K in
// ascending order in one accumulator, whatever the number of rows in the call: a row's
// prediction does not depend on its neighbours, which is what lets decode reproduce encode.
#pragma once
#include "device_utils.h"

namespace aquakv {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 f16x8;

constexpr int BM = 256, BN = 128, BK = 64;       // block tile; the waves are stacked in M
constexpr int kRowBytes = BK * 2;                // 128 B of bf16 per LDS row
constexpr int kATileBytes = BM * kRowBytes;      // 32 KiB
constexpr int kBTileBytes = BN * kRowBytes;      // 16 KiB
constexpr int kStageBytes = kATileBytes + kBTileBytes;   // 48 KiB
constexpr int kStages = 3;                       // LDS ring of k-tiles
constexpr int kMainLoopLdsBytes = kStages * kStageBytes;
// The tile is worked on by WAVES = 4 or 8 wavefronts (one or two per SIMD); wave w owns rows
// (256 / WAVES) * w ... of the tile and all 128 columns.  Both shapes run the same MFMAs in the
// same K order per output element, so they give identical bits.
constexpr int kGemmThreads = 256;                // the 4-wave shape (stand-alone predictor kernel)

// 16-byte chunk `ch` (0..7) of LDS row `row`.  A row is 128 B = half of the 64 banks, so even
// and odd rows already sit in different bank halves; the chunk is XOR-swizzled with row/2 so
// that the 16 lanes served together by a 128-bit fragment read (16 consecutive rows, same
// chunk) touch all 64 banks exactly once.
__device__ __forceinline__ int lds_off(int row, int ch) { return row * kRowBytes + ((ch ^ ((row >> 1) & 7)) << 4); }

// XCD-aware tile order: consecutive workgroup ids land on different XCDs, so
// give each XCD a contiguous range of tiles (n fastest): the column tiles of
// a row tile then share that XCD's L2 copy of the x rows.
__device__ __forceinline__ int remap_block(int bid, int nblocks) {
  constexpr int kXcd = 8;
  if (nblocks % kXcd != 0) return bid;
  return (bid % kXcd) * (nblocks / kXcd) + bid / kXcd;
}

// The workgroup's accumulator tile: wave w owns rows (256/WAVES)*w ... of the 256, all 128 columns;
// acc[i][j] is the 32 x 32 block at rows 32i, columns 32j of the wave's rows; inside it the lane
// holds column lane%32 and rows 8*blk + 4*(lane/32) + r4 in register 4*blk + r4.
// `lds_base` points at kMainLoopLdsBytes bytes of LDS.  Ends with a barrier after the last LDS
// read, so the caller may reuse the LDS at once.  Requires K = d0 + d1 a multiple of 128, d0 of 64.
// `before_drain()` is called once, when the last operand loads have been issued and about two
// k-tiles of MFMA work remain: the place to request what the caller's epilogue reads.
//
// Operands go from global memory straight into LDS (global_load_lds_dwordx4): no staging
// registers, no ds_write instructions.  One such instruction of a wave fills 1 KiB of LDS,
// lane l at byte 16 l, i.e. 8 consecutive tile rows with lane l -> row l/8, slot l%8.  The LDS
// layout is swizzled (lds_off), so the lane fetches from global memory the chunk that belongs
// in its slot.  The compiler does not track these writes to LDS: completion is awaited with an
// explicit vmcnt before the barrier that publishes a k-tile (loads complete in issue order, so
// waiting until at most one tile's worth is outstanding means every older tile has landed).
template <int WAVES, typename BeforeDrain>
__device__ __forceinline__ void gemm_mainloop(unsigned char* lds_base, const bf16_t* __restrict__ x0, int d0,
                                              const bf16_t* __restrict__ x1, int d1, const bf16_t* __restrict__ W,
                                              int64_t T, int64_t m0, int n0, f32x16 (&acc)[BM / WAVES / 32][4],
                                              BeforeDrain&& before_drain) {
  static_assert(WAVES == 4 || WAVES == 8, "one or two waves per SIMD");
  constexpr int kThreadsW = WAVES * 64;
  constexpr int MI = BM / WAVES / 32;              // 32-row blocks per wave (2 or 1)
  constexpr int kAChunks = BM * 8 / kThreadsW;     // load instructions per thread and k-tile for x (8 or 4)
  constexpr int kBChunks = BN * 8 / kThreadsW;     // for W (4 or 2)
  constexpr int kPieces = kAChunks + kBChunks;     // 12 or 6
  constexpr int kPieceBytes = kThreadsW * 16;      // LDS filled by one load instruction of the workgroup
  constexpr int kFragPieces = MI + 4;              // a[0..MI), b[0..4)
  constexpr int kMma = MI * 4;                     // MFMAs per step of 16 k
  static_assert(kPieces <= 63, "vmcnt range");
  typedef __attribute__((address_space(3))) unsigned char* lptr_t;
  typedef const __attribute__((address_space(1))) char* gptr_t;          // global address space
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int K = d0 + d1;
  const int nk = K / BK;

  // Software pipeline (one block per CU and at most two waves per SIMD, so the overlap has to be
  // built into the instruction stream).  k-tile t lives in LDS stage t % 3 and is multiplied in
  // four steps of 16 k.  Between barrier B_t (tile t complete in LDS) and B_{t+1}:
  //   MFMAs (t-1, step 2)   + fragment reads (t, 0)   + half of the loads of tile t+2
  //   MFMAs (t-1, step 3)   + fragment reads (t, 1)   + the other half
  //   MFMAs (t,   step 0)   + fragment reads (t, 2)
  //   MFMAs (t,   step 1)   + fragment reads (t, 3)
  // (8 MFMAs per step and wave with 4 waves, 4 with 8 waves.)  Tile t+2 overwrites the stage of
  // tile t-1, whose last fragment reads have returned before B_t.  At most two memory
  // instructions sit in the shadow of one MFMA, every fragment is requested at least one step
  // before its use, the matrix pipe keeps running across the barrier, and a load has almost two
  // iterations to land.  Loads use a scalar base (per k-tile) plus a per-thread byte offset.
  // sched_barrier(0) after each MFMA keeps the compiler from regrouping the stream.
  struct Frag { bf16x8 v[kFragPieces]; };

  const int ch16 = ((tid & 7) ^ ((tid >> 4) & 7)) * 16;   // byte offset in a tile row of the chunk for this lane's slot
  int rowc[kAChunks];                                      // tile-local x row of piece pc, clamped to the last valid row
  uint32_t offB[kBChunks];                                 // byte offset of piece pc in W relative to (n0, k0)
  {
    const int last = (int)((T - 1 - m0) < (BM - 1) ? (T - 1 - m0) : (BM - 1));
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

  // wave-uniform values are pinned to scalar registers so that the loads take the
  // "scalar base + 32-bit vector offset" form
  const auto uniform_ptr = [](const char* p) {
    const uint64_t u = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)u);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(u >> 32));
    return (gptr_t)(((uint64_t)hi << 32) | lo);
  };
  const lptr_t lds3 = (lptr_t)lds_base;
  auto load_piece = [&](int kt, int stage_off, int pc) {   // piece pc of tile kt: global -> LDS stage at byte stage_off
    const int k0 = kt * BK;
    const lptr_t dst = lds3 + (stage_off + pc * kPieceBytes + wave * 1024);   // x pieces fill the A tile, W pieces follow
    if (pc < kAChunks) {
      const bool second = k0 >= d0;                        // which K-panel of the concatenated input
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
  const int frow = lane & 31;       // row (A) / column (B) inside a 32-wide fragment
  const int fk = lane >> 5;         // which half of the 16 k values
  auto frag_piece = [&](int stage_off, int ks, Frag& f, int pc) {  // LDS -> MFMA operand registers
    const int off = pc < MI ? lds_off(wave * (MI * 32) + pc * 32 + frow, ks * 2 + fk)
                            : kATileBytes + lds_off((pc - MI) * 32 + frow, ks * 2 + fk);
    f.v[pc] = *reinterpret_cast<const bf16x8*>(lds_base + stage_off + off);
  };

#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // the MFMAs of one step on fragment f; extra(m) is issued right after MFMA m
  auto mma8 = [&](const Frag& f, auto&& extra) {
#pragma unroll
    for (int m = 0; m < kMma; ++m) {
      const int i = m >> 2, j = m & 3;
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.v[i], f.v[MI + j], acc[i][j], 0, 0, 0);
      extra(m);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // memory work attached to MFMA slot m of a step: the step's share of a list of n items is
  // spread two per slot from slot 0 on (n <= 2 * kMma)
  auto spread = [&](int m, int n, auto&& item) {
    if (2 * m < n) item(2 * m);
    if (2 * m + 1 < n) item(2 * m + 1);
  };
  // Publish a k-tile: wait until at most `outstanding` of this wave's loads are in flight (older
  // ones have landed in LDS) and its own LDS reads have returned, then meet the other waves.
  // The empty asm statements keep the compiler from moving LDS accesses across the barrier.
  auto publish = [&](bool more_in_flight) {
    if (more_in_flight) __builtin_amdgcn_s_waitcnt(0x0070 | (kPieces & 15) | ((kPieces >> 4) << 14));   // vmcnt(kPieces) lgkmcnt(0)
    else __builtin_amdgcn_s_waitcnt(0x0070);                                                            // vmcnt(0) lgkmcnt(0)
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
  };

  Frag f[4];                                               // one buffer per step of a tile
  constexpr int kHalf = kPieces / 2;
#pragma unroll
  for (int pc = 0; pc < kPieces; ++pc) load_piece(0, 0, pc);
#pragma unroll
  for (int pc = 0; pc < kPieces; ++pc) load_piece(1, kStageBytes, pc);  // nk >= 2
  publish(true);                                                        // B_0

  // iteration t (see the table above): tile t is in the stage at s0; tile t+2 goes to the stage at s2
  auto iteration = [&](int t, int s0, int s2, bool first, bool do_load) {
    if (!first) {
      mma8(f[2], [&](int m) {
        spread(m, kFragPieces + kHalf, [&](int e) {
          if (e < kFragPieces) frag_piece(s0, 0, f[0], e);
          else if (do_load) load_piece(t + 2, s2, e - kFragPieces);
        });
      });
      mma8(f[3], [&](int m) {
        spread(m, kFragPieces + kHalf, [&](int e) {
          if (e < kFragPieces) frag_piece(s0, 1, f[1], e);
          else if (do_load) load_piece(t + 2, s2, kHalf + e - kFragPieces);
        });
      });
    } else {
#pragma unroll
      for (int pc = 0; pc < kFragPieces; ++pc) { frag_piece(s0, 0, f[0], pc); frag_piece(s0, 1, f[1], pc); }
      if (do_load) {
#pragma unroll
        for (int pc = 0; pc < kPieces; ++pc) load_piece(t + 2, s2, pc);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    mma8(f[0], [&](int m) { spread(m, kFragPieces, [&](int e) { frag_piece(s0, 2, f[2], e); }); });
    mma8(f[1], [&](int m) { spread(m, kFragPieces, [&](int e) { frag_piece(s0, 3, f[3], e); }); });
  };
  const auto next_stage = [](int s) { return s + kStageBytes == kMainLoopLdsBytes ? 0 : s + kStageBytes; };

  // nk is even and >= 2 (K is a multiple of 128)
  int s0 = 0, s2 = 2 * kStageBytes;
  iteration(0, s0, s2, true, nk > 2);
  publish(nk > 2);                                                      // B_1
  s0 = next_stage(s0); s2 = next_stage(s2);
  int t = 1;
  for (; t + 2 < nk; ++t) {                          // steady state: tile t+2 is still to be requested
    iteration(t, s0, s2, false, true);
    publish(true);
    s0 = next_stage(s0); s2 = next_stage(s2);
  }
  before_drain();
  __builtin_amdgcn_sched_barrier(0);
  for (; t < nk; ++t) {                              // drain: the last two tiles (one if nk == 2), nothing left to load
    iteration(t, s0, s2, false, false);
    publish(false);
    s0 = next_stage(s0); s2 = next_stage(s2);
  }
  mma8(f[2], [&](int) {});                           // (nk-1, steps 2 and 3)
  mma8(f[3], [&](int) {});
}

}  // namespace aquakv
