// Least-squares fit of a linear predictor (Alg. "Calibration" of the AQUA-KV paper, Sect. 3.2):
//   W = argmin || [x0 | x1] W^T - Y ||^2 + lambda ||W||^2,   lambda = rate * trace(X^T X) / d_in,
// through the normal equations in fp64:  G = X^T X + lambda I,  C = X^T Y,  G = L L^T (Cholesky),
// L Z = C, L^T S = Z, W = S^T rounded to the storage dtype.  With an intercept, X and Y are centred first (the Gram
// products of the centred data are those of the raw data minus T mean mean^T) and b = mean(Y) - W mean(X).
//
// Everything is tiled in 64 x 64 blocks of doubles.  The two Gram products stream the tokens once per output tile
// (tokens in ascending order in one accumulator per output: the result does not depend on the launch shape) on the
// fp64 matrix cores; the factorisation and the two triangular solves are right-looking block algorithms in plain
// fp64 FMA arithmetic, one small launch per block step and kind (diagonal block / panel / trailing update), so
// that the trailing updates use the whole chip.  Calibration runs once per model, its cost is the Gram products,
// and fp64 keeps the solution within rounding of the definition.
#include "device_utils.h"
#include "kernels.h"

namespace aquakv {
namespace {

constexpr int kNb = 64;                      // block size of every tile
constexpr int kFitThreads = 256;             // 16 x 16 threads, 4 x 4 outputs each

typedef double f64x4 __attribute__((ext_vector_type(4)));

// 8 consecutive storage elements (16-byte aligned) -> doubles
__device__ __forceinline__ void load8(const float* p, double (&v)[8]) {
  const f32x4 a = reinterpret_cast<const f32x4*>(p)[0], b = reinterpret_cast<const f32x4*>(p)[1];
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ __forceinline__ void load8(const bf16_t* p, double (&v)[8]) {
  float f[8];
  unpack_bf16x8(*reinterpret_cast<const u32x4*>(p), f);
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = f[e];
}

// ------------------------------------------------------------------ Gram products
// blockIdx.x = tile index: the first nd (nd + 1) / 2 tiles are the lower triangle of the symmetric
// G(i, j) = sum_t X[t, 64 i ...] X[t, 64 j ...], j <= i (the tile is also stored mirrored at (j, i)), the following
// nd * no tiles are C(i, j) = sum_t X[t, 64 i ...] Y[t, 64 j ...].  X is the concatenation [x0 | x1]; d0 is a
// multiple of 64, so a tile's 64 columns come from one of the two.
template <typename T>
__global__ __launch_bounds__(kFitThreads) void gram_kernel(const T* __restrict__ x0, int d0, const T* __restrict__ x1,
                                                           int d1, const T* __restrict__ Y, int d_out, int64_t tokens,
                                                           double* __restrict__ G, double* __restrict__ C) {
  constexpr int kChunk = 32;                 // tokens per LDS chunk
  // rows 80 doubles apart: the 4 token rows a fragment read touches start 32 banks apart
  __shared__ double As[kChunk][kNb + 16], Bs[kChunk][kNb + 16];
  const int d_in = d0 + d1;
  const int nd = d_in / kNb, no = d_out / kNb;
  int tile = blockIdx.x;
  const int n_sym = nd * (nd + 1) / 2;
  const bool is_c = tile >= n_sym;
  int ti, tj;
  if (is_c) {
    tile -= n_sym;
    ti = tile / no; tj = tile % no;
  } else {
    ti = 0;
    while (tile > ti) { tile -= ti + 1; ++ti; }          // row ti of the triangle holds ti + 1 tiles
    tj = tile;
  }
  // column sources of the two operands
  const int ca = ti * kNb;
  const T* pa = ca < d0 ? x0 + ca : x1 + (ca - d0);
  const int lda = ca < d0 ? d0 : d1;
  const T* pb;
  int ldb;
  if (is_c) {
    pb = Y + tj * kNb; ldb = d_out;
  } else {
    const int cb = tj * kNb;
    pb = cb < d0 ? x0 + cb : x1 + (cb - d0);
    ldb = cb < d0 ? d0 : d1;
  }
  // fp64 matrix cores (v_mfma_f64_16x16x4_f64: D[16 x 16] += A[16 x 4] B[4 x 16], lane l holds A[l % 16][l / 16] and
  // B[l / 16][l % 16], i.e. one double each, and D[4 v + l / 16][l % 16] in register v).  With the tokens as the
  // contracted index both operands are read from the token-major LDS chunk as they lie.  Wave w owns the 32 x 32
  // quarter at rows 32 (w / 2), columns 32 (w % 2) of the tile: 2 x 2 blocks.
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int fr = lane & 15, fk = lane >> 4;
  const int ra = 32 * (wave >> 1), cbq = 32 * (wave & 1);
  f64x4 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = f64x4{0.0, 0.0, 0.0, 0.0};
  for (int64_t t0 = 0; t0 < tokens; t0 += kChunk) {
    // 32 tokens x 64 columns per operand: 8 elements per thread, a thread reads 8 consecutive columns of one token
    {
      const int r = threadIdx.x >> 3, c8 = (threadIdx.x & 7) * 8;
      const int64_t t = t0 + r;
      double va[8] = {}, vb[8] = {};
      if (t < tokens) {
        load8(pa + t * lda + c8, va);
        load8(pb + t * ldb + c8, vb);
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) { As[r][c8 + e] = va[e]; Bs[r][c8 + e] = vb[e]; }
    }
    __syncthreads();
#pragma unroll
    for (int k0 = 0; k0 < kChunk; k0 += 4) {
      double a[2], b[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) { a[i] = As[k0 + fk][ra + 16 * i + fr]; b[i] = Bs[k0 + fk][cbq + 16 * i + fr]; }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
  }
  double* out = is_c ? C : G;
  const int ldo = is_c ? d_out : d_in;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int row = ti * kNb + ra + 16 * i + 4 * v + fk, col = tj * kNb + cbq + 16 * j + fr;
        out[(int64_t)row * ldo + col] = acc[i][j][v];
        if (!is_c && ti != tj) out[(int64_t)col * ldo + row] = acc[i][j][v];
      }
}

// ------------------------------------------------------------------ intercept (centred regression)
// Column means of [X | Y]: blockIdx.x = 64-column block (the first d_in / 64 blocks are X, the rest Y); 4 strands of
// tokens per column, added in a fixed order.
template <typename T>
__global__ __launch_bounds__(kFitThreads) void column_mean_kernel(const T* __restrict__ x0, int d0, const T* __restrict__ x1,
                                                                  int d1, const T* __restrict__ Y, int d_out, int64_t tokens,
                                                                  double* __restrict__ mean) {
  __shared__ double part[4][kNb];
  const int d_in = d0 + d1;
  const int c0 = blockIdx.x * kNb;
  const T* p;
  int ld;
  if (c0 < d0) { p = x0 + c0; ld = d0; }
  else if (c0 < d_in) { p = x1 + (c0 - d0); ld = d1; }
  else { p = Y + (c0 - d_in); ld = d_out; }
  const int c = threadIdx.x & 63, strand = threadIdx.x >> 6;
  double s = 0.0;
  for (int64_t t = strand; t < tokens; t += 4) s += (double)static_cast<float>(p[t * ld + c]);
  part[strand][c] = s;
  __syncthreads();
  if (strand == 0) mean[c0 + c] = (((part[0][c] + part[1][c]) + part[2][c]) + part[3][c]) / (double)tokens;
}

// G -= T mx mx^T, C -= T mx my^T: the Gram products of the centred data from those of the raw data
__global__ void centre_kernel(double* __restrict__ G, double* __restrict__ C, const double* __restrict__ mean, int d_in,
                              int d_out, double tokens) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t ng = (int64_t)d_in * d_in;
  if (e < ng) {
    const int i = (int)(e / d_in), j = (int)(e % d_in);
    G[e] -= tokens * mean[i] * mean[j];
  } else if (e < ng + (int64_t)d_in * d_out) {
    const int64_t f = e - ng;
    const int i = (int)(f / d_out), o = (int)(f % d_out);
    C[f] -= tokens * mean[i] * mean[d_in + o];
  }
}

// b[o] = my[o] - sum_i S[i][o] mx[i] (i ascending), fp32 out; NaN after a failed factorisation
__global__ void intercept_kernel(const double* __restrict__ S, const double* __restrict__ mean, int d_in, int d_out,
                                 float* __restrict__ bias, const int* __restrict__ status) {
  const int o = blockIdx.x * blockDim.x + threadIdx.x;
  if (o >= d_out) return;
  double b = mean[d_in + o];
  for (int i = 0; i < d_in; ++i) b -= S[(int64_t)i * d_out + o] * mean[i];
  bias[o] = *status != 0 ? __uint_as_float(0x7fc00000u) : (float)b;
}

// G[i][i] += rate * trace(G) / d (one block; the trace is summed in a fixed order); clears the status word
__global__ __launch_bounds__(kFitThreads) void ridge_kernel(double* __restrict__ G, int d, double rate, int* status) {
  __shared__ double part[kFitThreads];
  if (threadIdx.x == 0) *status = 0;
  double s = 0.0;
  for (int i = threadIdx.x; i < d; i += kFitThreads) s += G[(int64_t)i * d + i];
  part[threadIdx.x] = s;
  __syncthreads();
  for (int w = kFitThreads / 2; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
    __syncthreads();
  }
  const double lam = rate * part[0] / d;
  for (int i = threadIdx.x; i < d; i += kFitThreads) G[(int64_t)i * d + i] += lam;
}

// ------------------------------------------------------------------ block kernels (all tiles 64 x 64, fp64)
// Cholesky of the diagonal block (k, k) in LDS; the strict upper triangle of the block is zeroed.
// `status` (device int): set to k + 1 if a pivot is not positive (the matrix is not positive definite).
__global__ __launch_bounds__(kFitThreads) void potrf_block_kernel(double* __restrict__ G, int d, int k, int* status) {
  __shared__ double A[kNb][kNb + 1];
  double* base = G + ((int64_t)k * kNb) * d + k * kNb;
  for (int e = threadIdx.x; e < kNb * kNb; e += kFitThreads) A[e >> 6][e & 63] = base[(int64_t)(e >> 6) * d + (e & 63)];
  __syncthreads();
  for (int c = 0; c < kNb; ++c) {
    const double piv = A[c][c];
    if (!(piv > 0.0)) {
      if (threadIdx.x == 0) *status = k + 1;
      return;                                             // uniform: every thread reads the same pivot
    }
    const double r = sqrt(piv);
    __syncthreads();
    if (threadIdx.x < kNb) {
      const int i = threadIdx.x;
      if (i == c) A[c][c] = r;
      else if (i > c) A[i][c] = A[i][c] / r;
    }
    __syncthreads();
    // trailing update of the block: A[i][j] -= A[i][c] A[j][c] for c < j <= i
    for (int e = threadIdx.x; e < kNb * kNb; e += kFitThreads) {
      const int i = e >> 6, j = e & 63;
      if (j > c && i >= j) A[i][j] -= A[i][c] * A[j][c];
    }
    __syncthreads();
  }
  for (int e = threadIdx.x; e < kNb * kNb; e += kFitThreads) {
    const int i = e >> 6, j = e & 63;
    base[(int64_t)i * d + j] = j <= i ? A[i][j] : 0.0;
  }
}

// Panel below the diagonal block: G(i, k) <- G(i, k) L_kk^-T for block rows i = k + 1 + blockIdx.x.
// One row of the block per thread (64 active threads), forward substitution along the row.
__global__ __launch_bounds__(kNb) void trsm_panel_kernel(double* __restrict__ G, int d, int k) {
  __shared__ double L[kNb][kNb + 1];
  __shared__ double X[kNb][kNb];                          // X[c][thread]: element c of the thread's row
  const double* lkk = G + ((int64_t)k * kNb) * d + k * kNb;
  for (int e = threadIdx.x; e < kNb * kNb; e += kNb) L[e >> 6][e & 63] = lkk[(int64_t)(e >> 6) * d + (e & 63)];
  __syncthreads();
  const int i = k + 1 + blockIdx.x;
  const int tid = threadIdx.x;
  double* row = G + ((int64_t)i * kNb + tid) * d + k * kNb;
  for (int c = 0; c < kNb; ++c) X[c][tid] = row[c];
  for (int c = 0; c < kNb; ++c) {
    double s = X[c][tid];
    for (int m = 0; m < c; ++m) s -= X[m][tid] * L[c][m];
    X[c][tid] = s / L[c][c];
  }
  for (int c = 0; c < kNb; ++c) row[c] = X[c][tid];
}

// Triangular solve with the diagonal block on block row k of the right-hand sides R [d, nrhs]:
// forward: R(k, r) <- L_kk^-1 R(k, r); backward: R(k, r) <- L_kk^-T R(k, r).  One column per thread, r = blockIdx.x.
template <bool BACKWARD>
__global__ __launch_bounds__(kNb) void trsm_diag_kernel(const double* __restrict__ G, int d, double* __restrict__ R,
                                                        int nrhs, int k) {
  __shared__ double L[kNb][kNb + 1];
  const double* lkk = G + ((int64_t)k * kNb) * d + k * kNb;
  for (int e = threadIdx.x; e < kNb * kNb; e += kNb) L[e >> 6][e & 63] = lkk[(int64_t)(e >> 6) * d + (e & 63)];
  __syncthreads();
  __shared__ double X[kNb][kNb];                          // X[c][thread]: element c of the thread's column
  const int tid = threadIdx.x;
  double* col = R + ((int64_t)k * kNb) * nrhs + blockIdx.x * kNb + tid;      // element c at col[c * nrhs]
  for (int c = 0; c < kNb; ++c) X[c][tid] = col[(int64_t)c * nrhs];
  if (!BACKWARD) {
    for (int c = 0; c < kNb; ++c) {
      double s = X[c][tid];
      for (int m = 0; m < c; ++m) s -= L[c][m] * X[m][tid];
      X[c][tid] = s / L[c][c];
    }
  } else {
    for (int c = kNb - 1; c >= 0; --c) {
      double s = X[c][tid];
      for (int m = c + 1; m < kNb; ++m) s -= L[m][c] * X[m][tid];      // (L^T)[c][m] = L[m][c]
      X[c][tid] = s / L[c][c];
    }
  }
  for (int c = 0; c < kNb; ++c) col[(int64_t)c * nrhs] = X[c][tid];
}

// Tile update  Cm(ci, cj) -= op(A) * op(B)  with 64 x 64 x 64 products; the tile pair comes from blockIdx.x.
//   kind 0 (factorisation): for k < j <= i: G(i, j) -= G(i, k) G(j, k)^T;  blockIdx.x enumerates the pairs
//   kind 1 (forward solve): for i > k: R(i, r) -= G(i, k) R(k, r)
//   kind 2 (backward solve): for i < k: R(i, r) -= G(k, i)^T R(k, r)
__global__ __launch_bounds__(kFitThreads) void block_update_kernel(double* __restrict__ G, int d,
                                                                   double* __restrict__ R, int nrhs, int k, int kind) {
  __shared__ double As[kNb][kNb + 1], Bs[kNb][kNb + 1];      // As[m][kk], Bs[kk][n]
  int bi, bj;                                                 // block coordinates of the updated tile
  if (kind == 0) {
    // pairs (i, j), k < j <= i < nb, row by row
    int p = blockIdx.x, i = k + 1;
    while (p >= i - k) { p -= i - k; ++i; }
    bi = i; bj = k + 1 + p;
  } else {
    const int nr = nrhs / kNb;
    const int ii = blockIdx.x / nr;
    bj = blockIdx.x % nr;
    bi = kind == 1 ? k + 1 + ii : ii;
  }
  for (int e = threadIdx.x; e < kNb * kNb; e += kFitThreads) {
    const int r = e >> 6, c = e & 63;
    if (kind == 0) {
      As[r][c] = G[((int64_t)bi * kNb + r) * d + k * kNb + c];            // G(i, k)[m][kk]
      Bs[c][r] = G[((int64_t)bj * kNb + r) * d + k * kNb + c];            // G(j, k)^T: Bs[kk][n] = G(j, k)[n][kk]
    } else if (kind == 1) {
      As[r][c] = G[((int64_t)bi * kNb + r) * d + k * kNb + c];            // G(i, k)[m][kk]
      Bs[r][c] = R[((int64_t)k * kNb + r) * nrhs + bj * kNb + c];         // R(k, r)[kk][n]
    } else {
      As[c][r] = G[((int64_t)k * kNb + r) * d + bi * kNb + c];            // G(k, i)^T: As[m][kk] = G(k, i)[kk][m]
      Bs[r][c] = R[((int64_t)k * kNb + r) * nrhs + bj * kNb + c];
    }
  }
  __syncthreads();
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  double acc[4][4] = {};
#pragma unroll 4
  for (int kk = 0; kk < kNb; ++kk) {
    double a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) { a[i] = As[4 * ty + i][kk]; b[i] = Bs[kk][4 * tx + i]; }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = __fma_rn(a[i], b[j], acc[i][j]);
  }
  double* out = kind == 0 ? G + ((int64_t)bi * kNb) * d + bj * kNb : R + ((int64_t)bi * kNb) * nrhs + bj * kNb;
  const int ldo = kind == 0 ? d : nrhs;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) out[(int64_t)(4 * ty + i) * ldo + 4 * tx + j] -= acc[i][j];
}

// fp64 -> storage dtype with one rounding (nearest even).  bf16: the double is first taken to fp32 towards zero with
// the discarded bits ORed into the last place (round to odd), which the final rounding to 8 bits cannot see.
template <typename T> __device__ __forceinline__ T round_from_double(double v);
template <> __device__ __forceinline__ float round_from_double<float>(double v) { return (float)v; }
template <> __device__ __forceinline__ bf16_t round_from_double<bf16_t>(double v) {
  float f = __double2float_rz(v);
  if ((double)f != v && f == f) f = __uint_as_float(__float_as_uint(f) | 1u);
  return static_cast<bf16_t>(f);
}

// W[o][i] = S[i][o] rounded to the storage dtype; W64 (nullable) receives the unrounded solution in the same
// layout.  A failed factorisation (status != 0) yields NaNs.
template <typename T>
__global__ void transpose_round_kernel(const double* __restrict__ S, int d_in, int d_out, T* __restrict__ W,
                                       double* __restrict__ W64, const int* __restrict__ status) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= (int64_t)d_in * d_out) return;
  const int o = (int)(e / d_in), i = (int)(e % d_in);
  const double v = *status != 0 ? __longlong_as_double(0x7ff8000000000000ll) : S[(int64_t)i * d_out + o];
  W[e] = round_from_double<T>(v);
  if (W64 != nullptr) W64[e] = v;
}

}  // namespace

size_t fit_workspace_bytes(int d_in, int d_out) {
  // G, C / solution, column means of [X | Y], status word
  return ((size_t)d_in * d_in + (size_t)d_in * d_out + d_in + d_out) * sizeof(double) + 16;
}

hipError_t launch_fit_predictor(int dtype, int64_t tokens, const void* x0, int d0, const void* x1, int d1, const void* Y,
                                int d_out, double rate, void* W, double* W64, float* bias, void* workspace,
                                hipStream_t stream) {
  const int d = d0 + d1;
  const int nb = d / kNb, nr = d_out / kNb;
  double* G = static_cast<double*>(workspace);
  double* C = G + (size_t)d * d;
  double* mean = C + (size_t)d * d_out;
  int* status = reinterpret_cast<int*>(mean + d + d_out);
  const unsigned tiles = (unsigned)(nb * (nb + 1) / 2 + nb * nr);
  if (dtype == kBF16)
    gram_kernel<bf16_t><<<tiles, kFitThreads, 0, stream>>>(static_cast<const bf16_t*>(x0), d0, static_cast<const bf16_t*>(x1),
                                                           d1, static_cast<const bf16_t*>(Y), d_out, tokens, G, C);
  else
    gram_kernel<float><<<tiles, kFitThreads, 0, stream>>>(static_cast<const float*>(x0), d0, static_cast<const float*>(x1), d1,
                                                          static_cast<const float*>(Y), d_out, tokens, G, C);
  if (bias != nullptr) {       // intercept: regress the centred Y on the centred X
    if (dtype == kBF16)
      column_mean_kernel<bf16_t><<<nb + nr, kFitThreads, 0, stream>>>(static_cast<const bf16_t*>(x0), d0,
                                                                      static_cast<const bf16_t*>(x1), d1,
                                                                      static_cast<const bf16_t*>(Y), d_out, tokens, mean);
    else
      column_mean_kernel<float><<<nb + nr, kFitThreads, 0, stream>>>(static_cast<const float*>(x0), d0,
                                                                     static_cast<const float*>(x1), d1,
                                                                     static_cast<const float*>(Y), d_out, tokens, mean);
    const int64_t ne = (int64_t)d * d + (int64_t)d * d_out;
    centre_kernel<<<(unsigned)((ne + 255) / 256), 256, 0, stream>>>(G, C, mean, d, d_out, (double)tokens);
  }
  ridge_kernel<<<1, kFitThreads, 0, stream>>>(G, d, rate, status);
  // G = L L^T, block column by block column
  for (int k = 0; k < nb; ++k) {
    potrf_block_kernel<<<1, kFitThreads, 0, stream>>>(G, d, k, status);
    const int below = nb - 1 - k;
    if (below > 0) {
      trsm_panel_kernel<<<below, kNb, 0, stream>>>(G, d, k);
      block_update_kernel<<<below * (below + 1) / 2, kFitThreads, 0, stream>>>(G, d, nullptr, 0, k, 0);
    }
  }
  // L Z = C
  for (int k = 0; k < nb; ++k) {
    trsm_diag_kernel<false><<<nr, kNb, 0, stream>>>(G, d, C, d_out, k);
    if (nb - 1 - k > 0) block_update_kernel<<<(nb - 1 - k) * nr, kFitThreads, 0, stream>>>(G, d, C, d_out, k, 1);
  }
  // L^T S = Z
  for (int k = nb - 1; k >= 0; --k) {
    trsm_diag_kernel<true><<<nr, kNb, 0, stream>>>(G, d, C, d_out, k);
    if (k > 0) block_update_kernel<<<k * nr, kFitThreads, 0, stream>>>(G, d, C, d_out, k, 2);
  }
  if (bias != nullptr) intercept_kernel<<<(d_out + 255) / 256, 256, 0, stream>>>(C, mean, d, d_out, bias, status);
  const int64_t n = (int64_t)d * d_out;
  const unsigned blocks = (unsigned)((n + 255) / 256);
  if (dtype == kBF16) transpose_round_kernel<bf16_t><<<blocks, 256, 0, stream>>>(C, d, d_out, static_cast<bf16_t*>(W), W64, status);
  else transpose_round_kernel<float><<<blocks, 256, 0, stream>>>(C, d, d_out, static_cast<float*>(W), W64, status);
  return hipGetLastError();
}

}  // namespace aquakv
