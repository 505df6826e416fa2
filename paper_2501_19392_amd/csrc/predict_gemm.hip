// Linear predictors of Sect. 3.2 of the AQUA-KV paper as a stand-alone stage:
// P = [x0 | x1] W^T + b written to memory in fp32.
//
// bf16 path: a dense contraction, so it runs on the gfx950 matrix cores (main loop in
// gemm_core.h).  fp32 path: plain FMA tiles (parity mode for the small fp32 configuration).
#include "gemm_core.h"
#include "kernels.h"

namespace aquakv {
namespace {

__global__ __launch_bounds__(kGemmThreads) void predict_bf16_kernel(
    const bf16_t* __restrict__ x0, int d0, const bf16_t* __restrict__ x1, int d1, const bf16_t* __restrict__ W,
    const float* __restrict__ bias, float* __restrict__ P, int64_t T, int D) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[kMainLoopLdsBytes];

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int n_tiles = D / BN;
  const int logical = remap_block(blockIdx.x, gridDim.x);
  const int tile_m = logical / n_tiles, tile_n = logical % n_tiles;
  const int64_t m0 = (int64_t)tile_m * BM;
  const int n0 = tile_n * BN;
  const int frow = lane & 31, fk = lane >> 5;

  f32x16 acc[2][4];
  gemm_mainloop<4>(lds, x0, d0, x1, d1, W, T, m0, n0, acc, [] {});

  // accumulator layout of the 32x32 tile: lane holds column lane%32 and rows
  // 8*blk + 4*(lane/32) + j for register 4*blk + j.
#pragma unroll
  for (int i = 0; i < 2; ++i) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int col = n0 + j * 32 + frow;
      const float bv = bias != nullptr ? bias[col] : 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t row = m0 + wave * 64 + i * 32 + (r >> 2) * 8 + fk * 4 + (r & 3);
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
