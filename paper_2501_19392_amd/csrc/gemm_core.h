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

constexpr int BM = 256, BN = 128, BK = 64;       // block tile; 4 waves stacked in M, wave tile 64 x 128
constexpr int kGemmThreads = 256;
constexpr int kRowBytes = BK * 2;                // 128 B of bf16 per LDS row
constexpr int kATileBytes = BM * kRowBytes;      // 32 KiB
constexpr int kBTileBytes = BN * kRowBytes;      // 16 KiB
constexpr int kStageBytes = kATileBytes + kBTileBytes;
constexpr int kAChunks = BM * 8 / kGemmThreads;  // 16-byte chunks per thread and k-tile (8)
constexpr int kBChunks = BN * 8 / kGemmThreads;  // (4)

// 16-byte chunk `ch` (0..7) of LDS row `row`, XOR-swizzled so that the 32 lanes
// of a fragment read (32 consecutive rows, same chunk) spread over all banks.
__device__ __forceinline__ int lds_off(int row, int ch) { return row * kRowBytes + ((ch ^ (row & 7)) << 4); }

// XCD-aware tile order: consecutive workgroup ids land on different XCDs, so
// give each XCD a contiguous range of tiles (n fastest): the column tiles of
// a row tile then share that XCD's L2 copy of the x rows.
__device__ __forceinline__ int remap_block(int bid, int nblocks) {
  constexpr int kXcd = 8;
  if (nblocks % kXcd != 0) return bid;
  return (bid % kXcd) * (nblocks / kXcd) + bid / kXcd;
}

// The workgroup's accumulator tile: wave w owns rows 64w .. 64w+63 of the 256, all 128 columns;
// acc[i][j] is the 32 x 32 block at rows 32i, columns 32j; inside it the lane holds column
// lane%32 and rows 8*blk + 4*(lane/32) + r4 in register 4*blk + r4.
// `lds_base` points at 2 * kStageBytes bytes of LDS.  Ends with a barrier after the last LDS read,
// so the caller may reuse the LDS at once.  Requires K = d0 + d1 a multiple of 128, d0 of 64.
__device__ __forceinline__ void gemm_mainloop(unsigned char* lds_base, const bf16_t* __restrict__ x0, int d0,
                                              const bf16_t* __restrict__ x1, int d1, const bf16_t* __restrict__ W,
                                              int64_t T, int64_t m0, int n0, f32x16 (&acc)[2][4]) {
  unsigned char (*lds)[kStageBytes] = reinterpret_cast<unsigned char (*)[kStageBytes]>(lds_base);
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int K = d0 + d1;
  const int nk = K / BK;

  // Software pipeline (one block per CU, one wave per SIMD, so the overlap has to be built
  // into the instruction stream).  For k-tile t, living in LDS stage t&1:
  //   barrier B_t                       -- tile t is completely in LDS, stage (t+1)&1 is free
  //   fragment reads (t, step 0)
  //   8 MFMAs of (t-1, step 3)          + the 12 LDS writes of tile t+1 into stage (t+1)&1
  //   8 MFMAs of (t, step 0)            + fragment reads (t, 1) + the 12 global loads of tile t+3
  //   8 MFMAs of (t, step 1)            + fragment reads (t, 2)
  //   8 MFMAs of (t, step 2)            + fragment reads (t, 3)
  // Every memory instruction is issued in the shadow of an MFMA, the matrix pipe runs across
  // the barrier, and a global load has two iterations to land (two register sets).
  // sched_barrier(0) after each MFMA keeps the compiler from regrouping the stream.
  struct Regs { u32x4 v[kAChunks + kBChunks]; };
  struct Frag { bf16x8 v[6]; };      // a[0], a[1], b[0..3]

  auto load_piece = [&](int kt, Regs& r, int pc) {         // piece pc of tile kt: global -> registers
    const int k0 = kt * BK;
    const int id = tid + (pc < kAChunks ? pc : pc - kAChunks) * kGemmThreads;
    const int row = id >> 3, ch = id & 7;
    if (pc < kAChunks) {
      const bf16_t* xa;
      int ld, kk;
      if (k0 < d0) { xa = x0; ld = d0; kk = k0; } else { xa = x1; ld = d1; kk = k0 - d0; }
      int64_t gr = m0 + row;
      gr = gr < T ? gr : T - 1;
      r.v[pc] = *reinterpret_cast<const u32x4*>(xa + gr * ld + kk + ch * 8);
    } else {
      r.v[pc] = *reinterpret_cast<const u32x4*>(W + (int64_t)(n0 + row) * K + k0 + ch * 8);
    }
  };
  auto store_piece = [&](int stage, const Regs& r, int pc) {   // registers -> LDS
    const int id = tid + (pc < kAChunks ? pc : pc - kAChunks) * kGemmThreads;
    const int base = pc < kAChunks ? 0 : kATileBytes;
    *reinterpret_cast<u32x4*>(&lds[stage][base + lds_off(id >> 3, id & 7)]) = r.v[pc];
  };
  const int frow = lane & 31;       // row (A) / column (B) inside a 32-wide fragment
  const int fk = lane >> 5;         // which half of the 16 k values
  auto frag_piece = [&](int stage, int ks, Frag& f, int pc) {  // LDS -> MFMA operand registers
    const int off = pc < 2 ? lds_off(wave * 64 + pc * 32 + frow, ks * 2 + fk)
                           : kATileBytes + lds_off((pc - 2) * 32 + frow, ks * 2 + fk);
    f.v[pc] = *reinterpret_cast<const bf16x8*>(&lds[stage][off]);
  };

#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // 8 MFMAs on fragment f; extra(m) is issued right after MFMA m
  auto mma8 = [&](const Frag& f, auto&& extra) {
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      const int i = m >> 2, j = m & 3;
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.v[i], f.v[2 + j], acc[i][j], 0, 0, 0);
      extra(m);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  Regs rs[2];
  Frag f0, f1, carry;
  constexpr int kPieces = kAChunks + kBChunks;   // 12
#pragma unroll
  for (int pc = 0; pc < kPieces; ++pc) load_piece(0, rs[0], pc);
#pragma unroll
  for (int pc = 0; pc < kPieces; ++pc) store_piece(0, rs[0], pc);
#pragma unroll
  for (int pc = 0; pc < kPieces; ++pc) load_piece(1, rs[1], pc);        // nk >= 2
#pragma unroll
  for (int pc = 0; pc < kPieces; ++pc)
    if (nk > 2) load_piece(2, rs[0], pc);
  __syncthreads();                                                      // B_0

  // iteration t; `first`: no (t-1, 3) to finish; write/load flags for the drain
  auto iteration = [&](int t, Regs& rw, bool first, bool do_store, bool do_load) {
    const int stage = t & 1;
#pragma unroll
    for (int pc = 0; pc < 6; ++pc) frag_piece(stage, 0, f0, pc);
    __builtin_amdgcn_sched_barrier(0);
    if (!first) {
      mma8(carry, [&](int m) {
        if (do_store) {
          if (m < 4) { store_piece(stage ^ 1, rw, 2 * m); store_piece(stage ^ 1, rw, 2 * m + 1); }
          else store_piece(stage ^ 1, rw, 4 + m);
        }
      });
    } else if (do_store) {
#pragma unroll
      for (int pc = 0; pc < kPieces; ++pc) store_piece(stage ^ 1, rw, pc);
      __builtin_amdgcn_sched_barrier(0);
    }
    mma8(f0, [&](int m) {
      if (m < 6) frag_piece(stage, 1, f1, m);
      if (do_load) {
        if (m < 4) { load_piece(t + 3, rw, 2 * m); load_piece(t + 3, rw, 2 * m + 1); }
        else load_piece(t + 3, rw, 4 + m);
      }
    });
    mma8(f1, [&](int m) { if (m < 6) frag_piece(stage, 2, f0, m); });
    mma8(f0, [&](int m) { if (m < 6) frag_piece(stage, 3, carry, m); });
    __syncthreads();                                                    // B_{t+1}
  };

  // nk is even and >= 2 (K is a multiple of 128)
  iteration(0, rs[1], true, true, nk > 3);
  int t = 1;
  for (; t + 3 < nk; t += 2) {                       // steady state, unrolled x2 over the register sets
    iteration(t, rs[0], false, true, true);
    iteration(t + 1, rs[1], false, true, true);
  }
  if (nk >= 4) {                                     // drain: t = nk-3 (odd), nk-2; nothing left to load
    iteration(nk - 3, rs[0], false, true, false);
    iteration(nk - 2, rs[1], false, true, false);
  }
  iteration(nk - 1, rs[0], false, false, false);
  mma8(carry, [&](int) {});                          // (nk-1, step 3)

}

}  // namespace aquakv
