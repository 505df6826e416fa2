// Streaming kernels of the backbone quantizer (Sect. 2 "Vector Quantization" of
// the AQUA-KV paper, HIGGS-style): quantize (residual -> RHT -> group scale ->
// nearest grid point -> packed codes, plus the reconstruction), dequantize, and
// dequantize fused with grouped-query q.k scoring.
//
// Work decomposition: one rotation group (128 values of one token and kv head)
// is held by 16 lanes x 8 consecutive values, so every global access is a
// 128-bit load/store and a wavefront covers 4 groups.  The Walsh-Hadamard
// butterfly runs 3 stages in registers and 4 stages over DPP row operations.
#include "device_utils.h"
#include "kernels.h"

namespace aquakv {
namespace {

constexpr int kThreads = 256;
constexpr int kGroupsPerBlock = kThreads / kLanesPerGroup;   // 16

template <int NCW> struct CodeBits;
template <> struct CodeBits<16> { static constexpr int c = 4; };
template <> struct CodeBits<64> { static constexpr int c = 6; };
template <> struct CodeBits<256> { static constexpr int c = 8; };

// Grid in LDS as (a, b, -(a^2+b^2)/2, unused): argmin ||y - C||^2 = argmax y.C - |C|^2/2.
template <int NCW>
__device__ __forceinline__ void load_codebook(const float* __restrict__ codebook, float4* cb) {
  for (int j = threadIdx.x; j < NCW; j += kThreads) {
    const float a = codebook[2 * j], b = codebook[2 * j + 1];
    cb[j] = make_float4(a, b, -0.5f * (a * a + b * b), 0.f);
  }
  __syncthreads();
}

// Nearest grid point for the 4 pairs a lane holds; lowest index wins ties.
template <int NCW>
__device__ __forceinline__ void search4(const float (&y)[8], const float4* cb, int (&idx)[4]) {
  float best[4];
  {
    const float4 c0 = cb[0];
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      best[m] = __fmaf_rn(y[2 * m], c0.x, __fmaf_rn(y[2 * m + 1], c0.y, c0.z));
      idx[m] = 0;
    }
  }
#pragma unroll 4
  for (int j = 1; j < NCW; ++j) {
    const float4 cj = cb[j];
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      const float s = __fmaf_rn(y[2 * m], cj.x, __fmaf_rn(y[2 * m + 1], cj.y, cj.z));
      const bool better = s > best[m];
      best[m] = better ? s : best[m];
      idx[m] = better ? j : idx[m];
    }
  }
}

// 4 codes of c bits per lane -> the group's little-endian bit string.
template <int NCW>
__device__ __forceinline__ void store_codes(uint8_t* __restrict__ codes, int64_t gid, int sub, const int (&idx)[4],
                                            bool active) {
  constexpr int c = CodeBits<NCW>::c;
  const uint32_t w = (uint32_t)idx[0] | ((uint32_t)idx[1] << c) | ((uint32_t)idx[2] << (2 * c)) |
                     ((uint32_t)idx[3] << (3 * c));
  uint8_t* base = codes + gid * (kGroup / 2 * c / 8);
  if constexpr (c == 4) {
    const uint32_t other = lane_xor_u32<1>(w);                 // odd neighbour's 16 bits
    if (active && (sub & 1) == 0) *reinterpret_cast<uint32_t*>(base + sub * 2) = w | (other << 16);
  } else if constexpr (c == 6) {
    // a quad of lanes owns 96 bits = 3 dwords; lane q < 3 builds dword q from w_q and w_{q+1}
    const uint32_t next = __float_as_uint(__int_as_float(
        __builtin_amdgcn_update_dpp(0, (int)w, 0xF9 /* quad_perm [1,2,3,3] */, 0xF, 0xF, false)));
    const int q = sub & 3;
    const uint32_t d = (w >> (8 * q)) | (next << (24 - 8 * q));
    if (active && q < 3) *reinterpret_cast<uint32_t*>(base + (sub >> 2) * 12 + q * 4) = d;
  } else {
    if (active) *reinterpret_cast<uint32_t*>(base + sub * 4) = w;
  }
}

template <int NCW>
__device__ __forceinline__ void load_codes(const uint8_t* __restrict__ codes, int64_t gid, int sub, int (&idx)[4]) {
  constexpr int c = CodeBits<NCW>::c;
  const uint8_t* base = codes + gid * (kGroup / 2 * c / 8);
  uint32_t w;
  if constexpr (c == 4) {
    w = *reinterpret_cast<const uint16_t*>(base + sub * 2);
  } else if constexpr (c == 6) {
    const int q = sub & 3;
    const uint32_t own = *reinterpret_cast<const uint32_t*>(base + (sub >> 2) * 12 + (q < 2 ? q : 2) * 4);
    const uint32_t prev = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)own, 0x90 /* quad_perm [0,0,1,2] */, 0xF, 0xF,
                                                                 false);
    if (q == 0) w = own;
    else if (q == 3) w = own >> 8;
    else w = (prev >> (32 - 8 * q)) | (own << (8 * q));
  } else {
    w = *reinterpret_cast<const uint32_t*>(base + sub * 4);
  }
  constexpr uint32_t mask = (1u << c) - 1;
#pragma unroll
  for (int m = 0; m < 4; ++m) idx[m] = (w >> (m * c)) & mask;
}

__device__ __forceinline__ float half_bits_to_float(uint16_t h) {
  return static_cast<float>(__builtin_bit_cast(_Float16, h));
}

// ------------------------------------------------------------------ quantize
template <typename T, int NCW>
__global__ __launch_bounds__(kThreads) void quantize_kernel(const T* __restrict__ X, const float* __restrict__ P,
                                                            const int8_t* __restrict__ signs,
                                                            const float* __restrict__ codebook,
                                                            uint8_t* __restrict__ codes, uint16_t* __restrict__ scales,
                                                            T* Xhat, int64_t n_groups, int H) {
  __shared__ float4 cb[NCW];
  load_codebook<NCW>(codebook, cb);

  const int sub = threadIdx.x & 15;
  int64_t gid = (int64_t)blockIdx.x * kGroupsPerBlock + (threadIdx.x >> 4);
  const bool active = gid < n_groups;
  if (!active) gid = n_groups - 1;                      // keep every lane in the DPP exchanges
  const int head = (int)(gid % H);
  const int64_t off = gid * kGroup + sub * kValsPerLane;

  float x[8], p[8], v[8];
  uint32_t sb[8];
  Storage<T>::load8(X + off, x);
  if (P != nullptr) {
    Storage<float>::load8(P + off, p);
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) p[i] = 0.f;
  }
  load_sign_bits(signs, head, sub, sb);

#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = __uint_as_float(__float_as_uint(x[i] - p[i]) ^ sb[i]);   // s * (x - p)
  wht128(v, sub);                                         // w = H u (unnormalised)

  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) ss = __fmaf_rn(v[i], v[i], ss);
  ss = group_sum16(ss);
  // z = w / sqrt(g)  =>  rms(z) = sqrt(sum w^2) / g
  float sigma = __fsqrt_rn(ss) * (1.0f / kGroup);
  sigma = fminf(sigma, 65504.0f);
  const _Float16 s16h = static_cast<_Float16>(sigma);     // round to nearest even
  const float s16 = static_cast<float>(s16h);
  const float inv = s16 > 0.f ? __fdiv_rn(kRsqrtG, s16) : 0.f;
  float y[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) y[i] = v[i] * inv;

  int idx[4];
  search4<NCW>(y, cb, idx);
  store_codes<NCW>(codes, gid, sub, idx, active);
  if (active && sub == 0) scales[gid] = __builtin_bit_cast(uint16_t, s16h);

  if (Xhat != nullptr) {
    float z[8];
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      const float4 cw = cb[idx[m]];
      z[2 * m] = cw.x * s16;
      z[2 * m + 1] = cw.y * s16;
    }
    reconstruct(z, sub, sb, p);
    if (active) Storage<T>::store8(Xhat + off, z);
  }
}

// ------------------------------------------------------------------ dequantize
template <typename T, int NCW>
__global__ __launch_bounds__(kThreads) void dequantize_kernel(const uint8_t* __restrict__ codes,
                                                              const uint16_t* __restrict__ scales,
                                                              const float* __restrict__ P,
                                                              const int8_t* __restrict__ signs,
                                                              const float* __restrict__ codebook, T* __restrict__ Xhat,
                                                              int64_t n_groups, int H) {
  __shared__ float4 cb[NCW];
  load_codebook<NCW>(codebook, cb);

  const int sub = threadIdx.x & 15;
  int64_t gid = (int64_t)blockIdx.x * kGroupsPerBlock + (threadIdx.x >> 4);
  const bool active = gid < n_groups;
  if (!active) gid = n_groups - 1;
  const int head = (int)(gid % H);
  const int64_t off = gid * kGroup + sub * kValsPerLane;

  float p[8], z[8];
  uint32_t sb[8];
  int idx[4];
  load_codes<NCW>(codes, gid, sub, idx);
  const float s16 = half_bits_to_float(scales[gid]);
  if (P != nullptr) {
    Storage<float>::load8(P + off, p);
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) p[i] = 0.f;
  }
  load_sign_bits(signs, head, sub, sb);
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    const float4 cw = cb[idx[m]];
    z[2 * m] = cw.x * s16;
    z[2 * m + 1] = cw.y * s16;
  }
  reconstruct(z, sub, sb, p);
  if (active) Storage<T>::store8(Xhat + off, z);
}

// ------------------------------------------------------------------ dequantize + q.k
// Group gid = row * H + head of the chunk; row = b * seq_len + t (global row = row0 + row).
template <typename T, int NCW>
__global__ __launch_bounds__(kThreads) void attn_scores_kernel(
    const uint8_t* __restrict__ codes, const uint16_t* __restrict__ scales, const float* __restrict__ P,
    const int8_t* __restrict__ signs, const float* __restrict__ codebook, const T* __restrict__ q, float score_scale,
    float* __restrict__ scores, T* __restrict__ Khat_out, int64_t row0, int64_t n_groups, int seq_len, int H,
    int q_heads) {
  __shared__ float4 cb[NCW];
  load_codebook<NCW>(codebook, cb);

  const int sub = threadIdx.x & 15;
  int64_t gid = (int64_t)blockIdx.x * kGroupsPerBlock + (threadIdx.x >> 4);
  const bool active = gid < n_groups;
  if (!active) gid = n_groups - 1;
  const int head = (int)(gid % H);
  const int64_t row = row0 + gid / H;
  const int64_t b = row / seq_len;
  const int64_t t = row % seq_len;
  const int64_t off = gid * kGroup + sub * kValsPerLane;

  float p[8], z[8];
  uint32_t sb[8];
  int idx[4];
  load_codes<NCW>(codes, gid, sub, idx);
  const float s16 = half_bits_to_float(scales[gid]);
  if (P != nullptr) {
    Storage<float>::load8(P + off, p);
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) p[i] = 0.f;
  }
  load_sign_bits(signs, head, sub, sb);
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    const float4 cw = cb[idx[m]];
    z[2 * m] = cw.x * s16;
    z[2 * m + 1] = cw.y * s16;
  }
  reconstruct(z, sub, sb, p);
  if (Khat_out != nullptr && active) Storage<T>::store8(Khat_out + off, z);
#pragma unroll
  for (int i = 0; i < 8; ++i) z[i] = Storage<T>::round(z[i]);      // score the stored keys

  const int rep = q_heads / H;
  for (int r = 0; r < rep; ++r) {
    const int qh = head * rep + r;
    float qv[8];
    Storage<T>::load8(q + ((int64_t)b * q_heads + qh) * kGroup + sub * kValsPerLane, qv);
    float acc = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) acc = __fmaf_rn(qv[i], z[i], acc);
    acc = group_sum16(acc);
    if (active && sub == 0) scores[((int64_t)b * q_heads + qh) * seq_len + t] = acc * score_scale;
  }
}

inline unsigned blocks_for(int64_t n_groups) {
  return (unsigned)((n_groups + kGroupsPerBlock - 1) / kGroupsPerBlock);
}

}  // namespace

#define AQUAKV_DISPATCH(DT, NCW, CALL)                                                  \
  do {                                                                                  \
    if ((DT) == kBF16) {                                                                \
      typedef bf16_t T;                                                                 \
      if ((NCW) == 16) { constexpr int N = 16; CALL; }                                  \
      else if ((NCW) == 64) { constexpr int N = 64; CALL; }                             \
      else { constexpr int N = 256; CALL; }                                             \
    } else {                                                                            \
      typedef float T;                                                                  \
      if ((NCW) == 16) { constexpr int N = 16; CALL; }                                  \
      else if ((NCW) == 64) { constexpr int N = 64; CALL; }                             \
      else { constexpr int N = 256; CALL; }                                             \
    }                                                                                   \
  } while (0)

hipError_t launch_quantize(int dtype, int n_codewords, const void* X, const float* P, const int8_t* signs,
                           const float* codebook, uint8_t* codes, uint16_t* scales, void* Xhat, int64_t T_, int H,
                           hipStream_t stream) {
  const int64_t n_groups = T_ * H;
  if (n_groups == 0) return hipSuccess;
  AQUAKV_DISPATCH(dtype, n_codewords,
                  (quantize_kernel<T, N><<<blocks_for(n_groups), kThreads, 0, stream>>>(
                      static_cast<const T*>(X), P, signs, codebook, codes, scales, static_cast<T*>(Xhat), n_groups, H)));
  return hipGetLastError();
}

hipError_t launch_dequantize(int dtype, int n_codewords, const uint8_t* codes, const uint16_t* scales, const float* P,
                             const int8_t* signs, const float* codebook, void* Xhat, int64_t T_, int H,
                             hipStream_t stream) {
  const int64_t n_groups = T_ * H;
  if (n_groups == 0) return hipSuccess;
  AQUAKV_DISPATCH(dtype, n_codewords,
                  (dequantize_kernel<T, N><<<blocks_for(n_groups), kThreads, 0, stream>>>(
                      codes, scales, P, signs, codebook, static_cast<T*>(Xhat), n_groups, H)));
  return hipGetLastError();
}

hipError_t launch_attn_scores(int dtype, int n_codewords, const uint8_t* codes, const uint16_t* scales, const float* P,
                              const int8_t* signs, const float* codebook, const void* q, float score_scale,
                              float* scores, void* Khat_out, int64_t row0, int64_t rows, int seq_len, int H,
                              int q_heads, hipStream_t stream) {
  const int64_t n_groups = rows * H;
  if (n_groups == 0) return hipSuccess;
  AQUAKV_DISPATCH(dtype, n_codewords,
                  (attn_scores_kernel<T, N><<<blocks_for(n_groups), kThreads, 0, stream>>>(
                      codes, scales, P, signs, codebook, static_cast<const T*>(q), score_scale, scores,
                      static_cast<T*>(Khat_out), row0, n_groups, seq_len, H, q_heads)));
  return hipGetLastError();
}

}  // namespace aquakv
