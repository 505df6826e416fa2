// Linear predictors of Sect. 3.2 of the AQUA-KV paper:  P = [x0 | x1] W^T + b.
//
// bf16 path: a dense contraction, so it runs on the gfx950 matrix cores
// (v_mfma_f32_32x32x16_bf16, fp32 accumulate).  Both operands are K-contiguous
// (x is [T, K], W is [D, K]), so A and B fragments are 128-bit LDS reads.
// Every output accumulates K in ascending order in one accumulator, whatever
// the tile shape or the number of rows: a row's prediction does not depend on
// how many rows are in the call, which is what lets decode reproduce encode.
//
// fp32 path: plain FMA tiles (parity mode for the small fp32 configuration).
#include "device_utils.h"
#include "kernels.h"

namespace aquakv {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int BM = 128, BN = 128, BK = 64;       // block tile; 4 waves as 2 x 2, wave tile 64 x 64
constexpr int kGemmThreads = 256;
constexpr int kRowBytes = BK * 2;                // 128 B of bf16 per LDS row
constexpr int kTileBytes = BM * kRowBytes;       // 16 KiB per operand per stage

// 16-byte chunk `ch` (0..7) of LDS row `row`, XOR-swizzled so that the 32 lanes
// of a fragment read (32 consecutive rows, same chunk) spread over all banks.
__device__ __forceinline__ int lds_off(int row, int ch) { return row * kRowBytes + ((ch ^ (row & 7)) << 4); }

// XCD-aware tile order: consecutive workgroup ids land on different XCDs, so
// give each XCD a contiguous range of tiles (n fastest): the 8 column tiles of
// a row tile then share that XCD's L2 copy of the x rows.
__device__ __forceinline__ int remap_block(int bid, int nblocks) {
  constexpr int kXcd = 8;
  if (nblocks % kXcd != 0) return bid;
  return (bid % kXcd) * (nblocks / kXcd) + bid / kXcd;
}

__global__ __launch_bounds__(kGemmThreads) void predict_bf16_kernel(
    const bf16_t* __restrict__ x0, int d0, const bf16_t* __restrict__ x1, int d1, const bf16_t* __restrict__ W,
    const float* __restrict__ bias, float* __restrict__ P, int64_t T, int D) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[2][2][kTileBytes];   // [stage][A|B]

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int n_tiles = D / BN;
  const int logical = remap_block(blockIdx.x, gridDim.x);
  const int tile_m = logical / n_tiles, tile_n = logical % n_tiles;
  const int64_t m0 = (int64_t)tile_m * BM;
  const int n0 = tile_n * BN;
  const int K = d0 + d1;
  const int nk = K / BK;

  // global -> register staging: 4 chunks of A and 4 of B per thread and k-tile
  uint4 ra[4], rb[4];
  auto load_tile = [&](int kt) {
    const int k0 = kt * BK;
    const bf16_t* xa;
    int ld, kk;
    if (k0 < d0) { xa = x0; ld = d0; kk = k0; } else { xa = x1; ld = d1; kk = k0 - d0; }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int id = tid + i * kGemmThreads;
      const int row = id >> 3, ch = id & 7;
      int64_t gr = m0 + row;
      gr = gr < T ? gr : T - 1;
      ra[i] = *reinterpret_cast<const uint4*>(xa + gr * ld + kk + ch * 8);
      rb[i] = *reinterpret_cast<const uint4*>(W + (int64_t)(n0 + row) * K + k0 + ch * 8);
    }
  };
  auto store_tile = [&](int stage) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int id = tid + i * kGemmThreads;
      const int row = id >> 3, ch = id & 7;
      *reinterpret_cast<uint4*>(&lds[stage][0][lds_off(row, ch)]) = ra[i];
      *reinterpret_cast<uint4*>(&lds[stage][1][lds_off(row, ch)]) = rb[i];
    }
  };

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  load_tile(0);
  store_tile(0);
  __syncthreads();

  const int frow = lane & 31;       // row (A) / column (B) inside a 32-wide fragment
  const int fk = lane >> 5;         // which half of the 16 k values
  for (int kt = 0; kt < nk; ++kt) {
    const int stage = kt & 1;
    if (kt + 1 < nk) load_tile(kt + 1);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 a[2], b[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int row = wm * 64 + i * 32 + frow;
        a[i] = *reinterpret_cast<const bf16x8*>(&lds[stage][0][lds_off(row, ks * 2 + fk)]);
        const int col = wn * 64 + i * 32 + frow;
        b[i] = *reinterpret_cast<const bf16x8*>(&lds[stage][1][lds_off(col, ks * 2 + fk)]);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) store_tile(stage ^ 1);
    __syncthreads();
  }

  // accumulator layout of the 32x32 tile: lane holds column lane%32 and rows
  // 8*blk + 4*(lane/32) + j for register 4*blk + j.
#pragma unroll
  for (int i = 0; i < 2; ++i) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int col = n0 + wn * 64 + j * 32 + frow;
      const float bv = bias != nullptr ? bias[col] : 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t row = m0 + wm * 64 + i * 32 + (r >> 2) * 8 + fk * 4 + (r & 3);
        if (row < T) P[row * D + col] = acc[i][j][r] + bv;
      }
    }
  }
}

// fp32 reference-precision path: 64 x 64 tile, each thread 4 x 4 outputs, K ascending.
constexpr int FM = 64, FN = 64, FK = 16;
__global__ __launch_bounds__(256) void predict_fp32_kernel(const float* __restrict__ x0, int d0,
                                                           const float* __restrict__ x1, int d1,
                                                           const float* __restrict__ W, const float* __restrict__ bias,
                                                           float* __restrict__ P, int64_t T, int D) {
  __shared__ float sa[FK][FM + 1];
  __shared__ float sb[FK][FN + 1];
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;
  const int n_tiles = D / FN;
  const int tile_m = blockIdx.x / n_tiles, tile_n = blockIdx.x % n_tiles;
  const int64_t m0 = (int64_t)tile_m * FM;
  const int n0 = tile_n * FN;
  const int K = d0 + d1;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += FK) {
    const float* xa;
    int ld, kk;
    if (k0 < d0) { xa = x0; ld = d0; kk = k0; } else { xa = x1; ld = d1; kk = k0 - d0; }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int id = tid + i * 256;
      const int row = id >> 4, k = id & 15;
      int64_t gr = m0 + row;
      gr = gr < T ? gr : T - 1;
      sa[k][row] = xa[gr * ld + kk + k];
      sb[k][row] = W[(int64_t)(n0 + row) * K + k0 + k];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < FK; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = sa[k][ty * 4 + i]; b[i] = sb[k][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = __fmaf_rn(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t row = m0 + ty * 4 + i;
    if (row >= T) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int col = n0 + tx * 4 + j;
      P[row * D + col] = acc[i][j] + (bias != nullptr ? bias[col] : 0.f);
    }
  }
}

}  // namespace

hipError_t launch_predict(int dtype, const void* x0, int d0, const void* x1, int d1, const void* W, const float* bias,
                          float* P, int64_t T, int D, hipStream_t stream) {
  if (T == 0) return hipSuccess;
  if (dtype == kBF16) {
    const int64_t blocks = ((T + BM - 1) / BM) * (D / BN);
    predict_bf16_kernel<<<(unsigned)blocks, kGemmThreads, 0, stream>>>(
        static_cast<const bf16_t*>(x0), d0, static_cast<const bf16_t*>(x1), d1, static_cast<const bf16_t*>(W), bias, P,
        T, D);
  } else {
    const int64_t blocks = ((T + FM - 1) / FM) * (D / FN);
    predict_fp32_kernel<<<(unsigned)blocks, 256, 0, stream>>>(static_cast<const float*>(x0), d0,
                                                              static_cast<const float*>(x1), d1,
                                                              static_cast<const float*>(W), bias, P, T, D);
  }
  return hipGetLastError();
}

}  // namespace aquakv
