// Linear predictors of Sect. 3.2 of the AQUA-KV paper as a stand-alone stage:
// P = [x0 | x1] W^T + b written to memory in fp32.
//
// bf16 path: a dense contraction, so it runs on the gfx950 matrix cores (main loop in
// gemm_team.h).  fp32 path: plain FMA tiles (parity mode for the small fp32 configuration).
#include "gemm_core.h"
#include "gemm_team.h"
#include "kernels.h"

namespace aquakv {
namespace {

// Four-wave main loop with swapped operands (gemm_team.h): a lane holds 64 consecutive outputs of one token, so the
// stores are 16 bytes each and 256 contiguous bytes per lane.
__global__ __launch_bounds__(kTeamThreads) void predict_bf16_kernel(
    const bf16_t* __restrict__ x0, int d0, const bf16_t* __restrict__ x1, int d1, const bf16_t* __restrict__ W,
    const float* __restrict__ bias, float* __restrict__ P, int64_t T, int D) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[kMainLoopLdsBytes + sizeof(TeamFlags)];
  TeamFlags& flags = *reinterpret_cast<TeamFlags*>(lds + kMainLoopLdsBytes);
  if (threadIdx.x < sizeof(TeamFlags) / 4) reinterpret_cast<uint32_t*>(&flags)[threadIdx.x] = 0;
  __syncthreads();
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int n_tiles = D / BN;
  const int logical = remap_block(blockIdx.x, gridDim.x);
  const int tile_m = logical / n_tiles, tile_n = logical % n_tiles;
  const int64_t m0 = (int64_t)tile_m * BM;
  const int n0 = tile_n * BN;
  f32x16 acc[4][2];
  uint32_t epoch = 0;
  gemm_team_mainloop(lds, flags.arrive, epoch, x0, d0, x1, d1, W, T, m0, n0, acc, [] {});
  const int tok = lane & 31, hf = lane >> 5;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int64_t row = m0 + wave * 64 + i * 32 + tok;
    if (row >= T) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int blk = 0; blk < 4; ++blk) {
        const int col = n0 + 64 * hf + 16 * j + 4 * blk;
        f32x4 o;
        o.x = acc[j][i][4 * blk] + (bias != nullptr ? bias[col] : 0.f);
        o.y = acc[j][i][4 * blk + 1] + (bias != nullptr ? bias[col + 1] : 0.f);
        o.z = acc[j][i][4 * blk + 2] + (bias != nullptr ? bias[col + 2] : 0.f);
        o.w = acc[j][i][4 * blk + 3] + (bias != nullptr ? bias[col + 3] : 0.f);
        *reinterpret_cast<f32x4*>(P + row * D + col) = o;
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
    predict_bf16_kernel<<<(unsigned)blocks, kTeamThreads, 0, stream>>>(
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
