// Value side of attention over the decoded cache (Alg. "Inference" of the AQUA-KV paper: the block call attends
// over the recovered keys and values; its output is the weighted sum of the values): soft-max of score rows, the
// weighted sum over values that already sit in memory (plain weights, or raw scores with the soft-max taken per
// chunk), the merge of the per-chunk results that both that kernel and the fused decode kernel leave behind, and the
// attention over tokens held in the storage dtype (sinks, recent buffer) with its merge into a running result.
// All sums run in a fixed order, so a call gives the same bits every time.
#include "device_utils.h"
#include "kernels.h"

namespace aquakv {
namespace {

constexpr int kThreads = 256;

// Block-wide reduction in a fixed tree order; every thread gets the result.
template <bool MAX> __device__ __forceinline__ float block_reduce(float x, float* buf) {
  buf[threadIdx.x] = x;
  __syncthreads();
#pragma unroll
  for (int s = kThreads / 2; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) {
      const float a = buf[threadIdx.x], b = buf[threadIdx.x + s];
      buf[threadIdx.x] = MAX ? fmaxf(a, b) : a + b;
    }
    __syncthreads();
  }
  const float r = buf[0];
  __syncthreads();
  return r;
}

// One workgroup per row: p = exp(s - max) / sum exp(s - max).  Any row length; three passes over the row.
__global__ __launch_bounds__(kThreads) void softmax_rows_kernel(const float* scores, float* probs, int64_t n) {
  __shared__ float buf[kThreads];
  const float* s = scores + (int64_t)blockIdx.x * n;
  float* p = probs + (int64_t)blockIdx.x * n;
  float m = -INFINITY;
  for (int64_t i = threadIdx.x; i < n; i += kThreads) m = fmaxf(m, s[i]);
  m = block_reduce<true>(m, buf);
  float sum = 0.f;
  for (int64_t i = threadIdx.x; i < n; i += kThreads) sum += expf(s[i] - m);
  sum = block_reduce<false>(sum, buf);
  const float inv = 1.0f / sum;
  for (int64_t i = threadIdx.x; i < n; i += kThreads) p[i] = expf(s[i] - m) * inv;
}

// The same for rows of up to 1024 * 4 * VEC values with n % 4 == 0: 1024 threads hold the row in registers
// (VEC 16-byte pieces each), so it is read once, and the two reductions go through the wavefronts' lanes
// and then 16 partial results in LDS.
constexpr int kWideThreads = 1024;
template <bool MAX> __device__ __forceinline__ float wide_reduce(float x, float* buf) {
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) {
    const float y = __shfl_xor(x, m);
    x = MAX ? fmaxf(x, y) : x + y;
  }
  if ((threadIdx.x & 63) == 0) buf[threadIdx.x >> 6] = x;
  __syncthreads();
  float r = buf[0];
#pragma unroll
  for (int w = 1; w < kWideThreads / 64; ++w) r = MAX ? fmaxf(r, buf[w]) : r + buf[w];
  __syncthreads();
  return r;
}
template <int VEC>
__global__ __launch_bounds__(kWideThreads) void softmax_rows_regs_kernel(const float* scores, float* probs, int n4) {
  __shared__ float buf[kWideThreads / 64];
  const f32x4* s = reinterpret_cast<const f32x4*>(scores) + (int64_t)blockIdx.x * n4;
  f32x4* p = reinterpret_cast<f32x4*>(probs) + (int64_t)blockIdx.x * n4;
  f32x4 v[VEC];
  float m = -INFINITY;
#pragma unroll
  for (int k = 0; k < VEC; ++k) {
    const int i = threadIdx.x + k * kWideThreads;
    if (i < n4) {
      v[k] = s[i];
      m = fmaxf(fmaxf(m, fmaxf(v[k].x, v[k].y)), fmaxf(v[k].z, v[k].w));
    }
  }
  m = wide_reduce<true>(m, buf);
  float sum = 0.f;
#pragma unroll
  for (int k = 0; k < VEC; ++k) {
    const int i = threadIdx.x + k * kWideThreads;
    if (i < n4) {
      v[k].x = expf(v[k].x - m); v[k].y = expf(v[k].y - m); v[k].z = expf(v[k].z - m); v[k].w = expf(v[k].w - m);
      sum += (v[k].x + v[k].y) + (v[k].z + v[k].w);
    }
  }
  sum = wide_reduce<false>(sum, buf);
  const float inv = 1.0f / sum;
#pragma unroll
  for (int k = 0; k < VEC; ++k) {
    const int i = threadIdx.x + k * kWideThreads;
    if (i < n4) {
      f32x4 o;
      o.x = v[k].x * inv; o.y = v[k].y * inv; o.z = v[k].z * inv; o.w = v[k].w * inv;
      p[i] = o;
    }
  }
}

// 8 consecutive values of a row as they lie in memory, and their fp32 form
template <typename T> struct Raw8;
template <> struct Raw8<float> {
  f32x4 a, b;
  __device__ __forceinline__ void load(const float* p) { a = reinterpret_cast<const f32x4*>(p)[0]; b = reinterpret_cast<const f32x4*>(p)[1]; }
  __device__ __forceinline__ void get(float (&v)[8]) const {
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
};
template <> struct Raw8<bf16_t> {
  u32x4 a;
  __device__ __forceinline__ void load(const bf16_t* p) { a = *reinterpret_cast<const u32x4*>(p); }
  __device__ __forceinline__ void get(float (&v)[8]) const { unpack_bf16x8(a, v); }
};

// One workgroup per (sequence, chunk of 256 tokens, kv head).  Thread (tsub = tid / 16, l = tid % 16) owns tokens
// tsub, tsub + 16, ... of the chunk and dims 8 l .. 8 l + 7; it reads its 16 row pieces once (all loads in flight
// together), keeps them in registers for the query heads of the group, and the 16 token classes are added through
// LDS.  This is the path for what the fused kernel does not cover (no predictor, fp32, groups of 1024, ragged
// sequences).
// pstats (nullable): soft-max form, `weights` holds raw scores: the weights are exp(score - chunk maximum), and the
// chunk's maximum and weight sum are written to pstats[chunk, qh, 2].
template <typename T>
__global__ __launch_bounds__(kThreads) void weighted_values_kernel(const T* __restrict__ Vhat, const float* __restrict__ weights,
                                                                   float* __restrict__ part, float* __restrict__ pstats,
                                                                   int seq_len, int H, int q_heads, int chunks_per_seq) {
  __shared__ float red[16][kGroup];
  __shared__ float buf[kThreads];
  constexpr int kIters = kWeightedChunk / 16;
  const int b = blockIdx.x / chunks_per_seq, chunk = blockIdx.x % chunks_per_seq, head = blockIdx.y;
  const int rep = q_heads / H;
  const int tsub = threadIdx.x >> 4, l = threadIdx.x & 15;
  const int t0 = chunk * kWeightedChunk + tsub;
  const T* vbase = Vhat + ((int64_t)b * seq_len * H + head) * kGroup + l * 8;
  Raw8<T> rows[kIters];
#pragma unroll
  for (int it = 0; it < kIters; ++it) {
    const int t = t0 + it * 16;
    rows[it].load(vbase + (int64_t)(t < seq_len ? t : seq_len - 1) * H * kGroup);     // beyond the end: weight 0 below
  }
  for (int r = 0; r < rep; ++r) {
    const int qh = head * rep + r;
    const float* w = weights + ((int64_t)b * q_heads + qh) * seq_len;
    float wt[kIters];
#pragma unroll
    for (int it = 0; it < kIters; ++it) {
      const int t = t0 + it * 16;
      wt[it] = t < seq_len ? w[t] : (pstats != nullptr ? -INFINITY : 0.f);
    }
    if (pstats != nullptr) {
      float mx = wt[0];
#pragma unroll
      for (int it = 1; it < kIters; ++it) mx = fmaxf(mx, wt[it]);
      const float shift = block_reduce<true>(mx, buf);
      float wsum = 0.f;
#pragma unroll
      for (int it = 0; it < kIters; ++it) {
        wt[it] = expf(wt[it] - shift);                       // exp(-inf) = 0 for tokens beyond the end
        wsum += wt[it];
      }
      const float total = block_reduce<false>(l == 0 ? wsum : 0.f, buf);      // every token counted once
      if (threadIdx.x == 0) {
        pstats[((int64_t)blockIdx.x * q_heads + qh) * 2] = shift;
        pstats[((int64_t)blockIdx.x * q_heads + qh) * 2 + 1] = total;
      }
    }
    float acc[8] = {};
#pragma unroll
    for (int it = 0; it < kIters; ++it) {
      float v[8];
      rows[it].get(v);
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] = __fmaf_rn(wt[it], v[i], acc[i]);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) red[tsub][l * 8 + i] = acc[i];
    __syncthreads();
    if (threadIdx.x < kGroup) {
      float sum = 0.f;
#pragma unroll
      for (int k = 0; k < 16; ++k) sum += red[k][threadIdx.x];
      part[((int64_t)blockIdx.x * q_heads + qh) * kGroup + threadIdx.x] = sum;
    }
    __syncthreads();
  }
}

// out[b, qh, d] = sum of the chunk sums, in a fixed order.  A workgroup owns 32 consecutive outputs; thread
// (k = tid / 32, j = tid % 32) adds the chunks c = k, k + 8, ... of output j (so every load of a wavefront is
// two full 128-byte lines and the loads of a thread do not wait for each other), and the 8 running sums are
// added in k order through LDS.
__global__ __launch_bounds__(kThreads) void combine_weighted_kernel(const float* __restrict__ part, float* __restrict__ out,
                                                                    int chunks_per_seq, int row, int64_t total) {
  __shared__ float red[8][32];
  const int k = threadIdx.x >> 5, j32 = threadIdx.x & 31;
  const int64_t i = (int64_t)blockIdx.x * 32 + j32;                     // index into out[batch][row], row = q_heads * 128
  float acc = 0.f;
  if (i < total) {
    const int64_t b = i / row, j = i % row;
    const float* src = part + b * chunks_per_seq * row + j;
    int c = k;
    for (; c + 24 < chunks_per_seq; c += 32) {
      const float a0 = src[(int64_t)c * row], a1 = src[(int64_t)(c + 8) * row], a2 = src[(int64_t)(c + 16) * row],
                  a3 = src[(int64_t)(c + 24) * row];
      acc = (((acc + a0) + a1) + a2) + a3;
    }
    for (; c < chunks_per_seq; c += 8) acc += src[(int64_t)c * row];
  }
  red[k][j32] = acc;
  __syncthreads();
  if (k == 0 && i < total) {
    float sum = red[0][j32];
#pragma unroll
    for (int w = 1; w < 8; ++w) sum += red[w][j32];
    out[i] = sum;
  }
}

// Soft-max form: chunk c carries sums taken with weights exp(score - m_c), its maximum m_c and weight sum l_c.
// out = sum_c e^(m_c - M) part_c / sum_c e^(m_c - M) l_c with M = max_c m_c; row_stats (nullable) receives M and the
// denominator.  Same thread layout as above; the three reductions over the chunks go through LDS in a fixed order.
__global__ __launch_bounds__(kThreads) void combine_softmax_kernel(const float* __restrict__ part, const float* __restrict__ pstats,
                                                                   float* __restrict__ out, float* __restrict__ row_stats,
                                                                   int chunks_per_seq, int q_heads) {
  __shared__ float red[8][32];
  __shared__ float den[8];
  const int row = q_heads * kGroup;
  const int k = threadIdx.x >> 5, j32 = threadIdx.x & 31;
  const int64_t i = (int64_t)blockIdx.x * 32 + j32;                     // the grid covers batch * q_heads * 128 outputs exactly
  const int64_t b = i / row, j = i % row;
  const int qh = (int)(j / kGroup);                                     // the same for the 32 outputs of a workgroup
  const float* src = part + b * chunks_per_seq * row + j;
  const float* st = pstats + (b * chunks_per_seq * q_heads + qh) * 2;
  float mx = -INFINITY;
  for (int c = k; c < chunks_per_seq; c += 8) mx = fmaxf(mx, st[(int64_t)c * q_heads * 2]);
  red[k][j32] = mx;
  __syncthreads();
  float M = red[0][j32];
#pragma unroll
  for (int w = 1; w < 8; ++w) M = fmaxf(M, red[w][j32]);
  __syncthreads();
  float acc = 0.f, l = 0.f;
  for (int c = k; c < chunks_per_seq; c += 8) {
    const float e = expf(st[(int64_t)c * q_heads * 2] - M);
    acc = __fmaf_rn(e, src[(int64_t)c * row], acc);
    l = __fmaf_rn(e, st[(int64_t)c * q_heads * 2 + 1], l);
  }
  red[k][j32] = acc;
  if (j32 == 0) den[k] = l;
  __syncthreads();
  if (k == 0) {
    float sum = red[0][j32], d = den[0];
#pragma unroll
    for (int w = 1; w < 8; ++w) { sum += red[w][j32]; d += den[w]; }
    out[i] = sum / d;
    if (row_stats != nullptr && j % kGroup == 0) {
      row_stats[(b * q_heads + qh) * 2] = M;
      row_stats[(b * q_heads + qh) * 2 + 1] = d;
    }
  }
}

// Attention of one query per sequence and query head over `tokens` keys / values held in the storage dtype (the
// attention sinks and the recent-token buffer of Sect. 3.3, which are not quantized), merged into a running result.
// rope_cos / rope_sin (nullable, fp32 [tokens, 64]: the angles of this call's tokens): the cache holds keys from
// before the rotary embedding (Sect. 3.3), so key t is rotated by its position first, coordinate d paired with d + 64.
// One workgroup per (sequence, query head): scores s_t = scale * q . k_t (a wave per token, lane l holds the
// coordinate pair (l, l + 64)), their
// maximum m and l = sum exp(s_t - m) through the block reductions, o = sum exp(s_t - m) v_t (thread = dim and token
// parity).  accumulate == 0: out = o / l, stats = (m, l).  Otherwise (out, stats) hold a result over other tokens,
// out normalised by its own L: M' = max(M, m), L' = L e^(M - M') + l e^(m - M'),
// out' = (out L e^(M - M') + o e^(m - M')) / L'.
constexpr int kRawMaxTokens = kAttendRawMaxTokens;
template <typename T>
__global__ __launch_bounds__(kThreads) void attend_raw_kernel(const T* __restrict__ K, const T* __restrict__ V,
                                                              const T* __restrict__ q, const float* __restrict__ rope_cos,
                                                              const float* __restrict__ rope_sin, float scale, float* out,
                                                              float* stats, int tokens, int H, int q_heads, int accumulate) {
  __shared__ float sc[kRawMaxTokens];
  __shared__ float buf[kThreads];
  __shared__ float half_sum[kGroup];
  const int b = blockIdx.x / q_heads, qh = blockIdx.x % q_heads;
  const int head = qh / (q_heads / H);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const T* qp = q + ((int64_t)b * q_heads + qh) * kGroup;
  const float q0 = static_cast<float>(qp[lane]), q1 = static_cast<float>(qp[lane + 64]);
  const T* kb = K + ((int64_t)b * tokens * H + head) * kGroup;
  const T* vb = V + ((int64_t)b * tokens * H + head) * kGroup;
  for (int t = wave; t < tokens; t += kThreads / 64) {
    const T* kp = kb + (int64_t)t * H * kGroup;
    float k0 = static_cast<float>(kp[lane]), k1 = static_cast<float>(kp[lane + 64]);
    if (rope_cos != nullptr) {
      const float cs = rope_cos[t * 64 + lane], sn = rope_sin[t * 64 + lane];
      const float r0 = __fmaf_rn(k0, cs, -(k1 * sn)), r1 = __fmaf_rn(k1, cs, k0 * sn);
      k0 = r0; k1 = r1;
    }
    float d = __fmaf_rn(q1, k1, q0 * k0);
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) d += __shfl_xor(d, m);
    if (lane == 0) sc[t] = d * scale;
  }
  __syncthreads();
  float mx = -INFINITY;
  for (int t = threadIdx.x; t < tokens; t += kThreads) mx = fmaxf(mx, sc[t]);
  const float m = block_reduce<true>(mx, buf);
  float ls = 0.f;
  for (int t = threadIdx.x; t < tokens; t += kThreads) {
    const float e = expf(sc[t] - m);
    sc[t] = e;                                  // each entry is touched by one thread only
    ls += e;
  }
  const float l = block_reduce<false>(ls, buf);       // its barriers also publish the exponentials
  const int d = threadIdx.x & (kGroup - 1), par = threadIdx.x >> 7;
  float o = 0.f;
  for (int t = par; t < tokens; t += 2) o = __fmaf_rn(sc[t], static_cast<float>(vb[(int64_t)t * H * kGroup + d]), o);
  if (par == 1) half_sum[d] = o;
  float* st = stats + ((int64_t)b * q_heads + qh) * 2;
  float M = 0.f, L = 0.f;
  if (accumulate) { M = st[0]; L = st[1]; }     // read by every thread before the barrier, rewritten after it
  __syncthreads();
  if (par == 0) {
    o += half_sum[d];
    float* op = out + ((int64_t)b * q_heads + qh) * kGroup + d;
    float M2 = m, L2 = l, res = o / l;
    if (accumulate) {
      M2 = fmaxf(M, m);
      const float ea = expf(M - M2), eb = expf(m - M2);
      L2 = __fmaf_rn(L, ea, l * eb);
      res = __fmaf_rn(*op * L, ea, o * eb) / L2;
    }
    *op = res;
    if (d == 0) { st[0] = M2; st[1] = L2; }
  }
}

}  // namespace

hipError_t launch_softmax_rows(const float* scores, float* probs, int64_t rows, int64_t n, hipStream_t stream) {
  if (rows == 0 || n == 0) return hipSuccess;
  const bool vec = n % 4 == 0 && n <= 4 * 4 * kWideThreads;
  if (vec && n <= 4 * kWideThreads)
    softmax_rows_regs_kernel<1><<<(unsigned)rows, kWideThreads, 0, stream>>>(scores, probs, (int)(n / 4));
  else if (vec && n <= 2 * 4 * kWideThreads)
    softmax_rows_regs_kernel<2><<<(unsigned)rows, kWideThreads, 0, stream>>>(scores, probs, (int)(n / 4));
  else if (vec)
    softmax_rows_regs_kernel<4><<<(unsigned)rows, kWideThreads, 0, stream>>>(scores, probs, (int)(n / 4));
  else
    softmax_rows_kernel<<<(unsigned)rows, kThreads, 0, stream>>>(scores, probs, n);
  return hipGetLastError();
}

hipError_t launch_weighted_values(int dtype, const void* Vhat, const float* weights, float* part, float* pstats, int batch,
                                  int seq_len, int H, int q_heads, hipStream_t stream) {
  if (batch == 0 || seq_len == 0) return hipSuccess;
  const int chunks = (seq_len + kWeightedChunk - 1) / kWeightedChunk;
  const dim3 grid((unsigned)batch * chunks, (unsigned)H);
  if (dtype == kBF16)
    weighted_values_kernel<bf16_t><<<grid, kThreads, 0, stream>>>(static_cast<const bf16_t*>(Vhat), weights, part, pstats,
                                                                  seq_len, H, q_heads, chunks);
  else
    weighted_values_kernel<float><<<grid, kThreads, 0, stream>>>(static_cast<const float*>(Vhat), weights, part, pstats,
                                                                 seq_len, H, q_heads, chunks);
  return hipGetLastError();
}

hipError_t launch_combine_weighted(const float* part, const float* pstats, float* out, float* row_stats, int batch,
                                   int seq_len, int q_heads, hipStream_t stream) {
  if (batch == 0) return hipSuccess;
  const int chunks = (seq_len + kWeightedChunk - 1) / kWeightedChunk;
  const int row = q_heads * kGroup;
  const int64_t total = (int64_t)batch * row;
  if (pstats != nullptr) {
    combine_softmax_kernel<<<(unsigned)(total / 32), kThreads, 0, stream>>>(part, pstats, out, row_stats, chunks, q_heads);
    return hipGetLastError();
  }
  combine_weighted_kernel<<<(unsigned)((total + 31) / 32), kThreads, 0, stream>>>(part, out, chunks, row, total);
  return hipGetLastError();
}

hipError_t launch_attend_raw(int dtype, const void* K, const void* V, const void* q, const float* rope_cos,
                             const float* rope_sin, float scale, float* out, float* stats, int batch, int tokens, int H,
                             int q_heads, int accumulate, hipStream_t stream) {
  if (batch == 0 || tokens == 0) return hipSuccess;
  const unsigned grid = (unsigned)batch * q_heads;
  if (dtype == kBF16)
    attend_raw_kernel<bf16_t><<<grid, kThreads, 0, stream>>>(static_cast<const bf16_t*>(K), static_cast<const bf16_t*>(V),
                                                             static_cast<const bf16_t*>(q), rope_cos, rope_sin, scale, out, stats,
                                                             tokens, H, q_heads, accumulate);
  else
    attend_raw_kernel<float><<<grid, kThreads, 0, stream>>>(static_cast<const float*>(K), static_cast<const float*>(V),
                                                            static_cast<const float*>(q), rope_cos, rope_sin, scale, out, stats,
                                                            tokens, H, q_heads, accumulate);
  return hipGetLastError();
}

}  // namespace aquakv
