// Streaming kernels of the backbone quantizer (Sect. 2 "Vector Quantization" of
// the AQUA-KV paper, HIGGS-style): quantize (residual -> RHT -> group scale ->
// nearest grid point -> packed codes, plus the reconstruction), dequantize, and
// dequantize fused with grouped-query q.k scoring; plus the builder of the
// nearest-grid-point search table.
//
// One rotation group is held by a quad of lanes x 32 values (see device_utils.h);
// a 256-thread block covers 64 groups per pass.
//
// Nearest grid point.  The definition is a search over all n grid points.  The
// kernels reach the same answer with a 64 x 64 table of square cells over
// [-4, 4]^2 (border cells are unbounded outwards): each cell
// lists, in ascending order, every grid point that can be nearest to some point
// of the (slightly enlarged) cell -- at most 4, else the cell is marked and the
// lane falls back to the full search.  Only the listed points are scored, with
// the same fp32 expression and the same lowest-index tie rule as the full
// search, so both give identical codes.
#include "device_utils.h"
#include "kernels.h"

namespace aquakv {
namespace {

constexpr int kThreads = 256;
constexpr int kGroupsPerBlock = kThreads / kLanesPerGroup;   // 64
constexpr int kCells = 64;                   // table is kCells x kCells
constexpr float kCellHalfRange = 4.0f;       // cells tile [-4, 4]^2
constexpr float kCellScale = kCells / (2.0f * kCellHalfRange);   // 8 cells per unit
constexpr uint32_t kCellFull = 0xffffffffu;  // too many candidates for the list: full search

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
}

__device__ __forceinline__ float score(float y0, float y1, const float4 c) {
  return __fmaf_rn(y0, c.x, __fmaf_rn(y1, c.y, c.z));
}

// Full search over all grid points; lowest index wins ties.
template <int NCW>
__device__ __forceinline__ int search_full(float y0, float y1, const float4* cb) {
  float best = score(y0, y1, cb[0]);
  int idx = 0;
#pragma unroll 8
  for (int j = 1; j < NCW; ++j) {
    const float s = score(y0, y1, cb[j]);
    const bool better = s > best;
    best = better ? s : best;
    idx = better ? j : idx;
  }
  return idx;
}

// Table search: score the (up to 4, ascending, last one repeated) candidates of the cell.
template <int NCW>
__device__ __forceinline__ int search_cell(float y0, float y1, const float4* cb, const uint32_t* table) {
  const float fx = __builtin_amdgcn_fmed3f(__fmaf_rn(y0, kCellScale, 0.5f * kCells), 0.0f, kCells - 0.5f);
  const float fy = __builtin_amdgcn_fmed3f(__fmaf_rn(y1, kCellScale, 0.5f * kCells), 0.0f, kCells - 0.5f);
  const uint32_t e = table[(int)fy * kCells + (int)fx];
  int idx = e & 0xff;
  float best = score(y0, y1, cb[idx]);
  constexpr int kCand = NCW == 16 ? 3 : 4;       // 16 grid points never need more than 3 per cell
#pragma unroll
  for (int k = 1; k < kCand; ++k) {
    const int j = (e >> (8 * k)) & 0xff;
    const float s = score(y0, y1, cb[j]);
    const bool better = s > best;                // duplicates of the last candidate never win
    best = better ? s : best;
    idx = better ? j : idx;
  }
  if (__builtin_expect(e == kCellFull, 0)) idx = search_full<NCW>(y0, y1, cb);   // crowded cell
  return idx;
}

// 16 codes of c bits per lane = 4c contiguous bytes of the group's little-endian bit string.
template <int NCW>
__device__ __forceinline__ void store_codes(uint8_t* __restrict__ codes, int64_t gid, int q, const int (&idx)[16]) {
  constexpr int c = CodeBits<NCW>::c;
  uint32_t* dst = reinterpret_cast<uint32_t*>(codes + gid * (kGroup / 2 * c / 8) + q * (2 * c));
  if constexpr (c == 4) {
    uint32_t d[2] = {0, 0};
#pragma unroll
    for (int m = 0; m < 16; ++m) d[m >> 3] |= (uint32_t)idx[m] << (4 * (m & 7));
    u32x2 v; v.x = d[0]; v.y = d[1];
    *reinterpret_cast<u32x2*>(dst) = v;
  } else if constexpr (c == 6) {
    uint32_t d[3] = {0, 0, 0};
#pragma unroll
    for (int m = 0; m < 16; ++m) {
      const int bit = 6 * m, w = bit >> 5, sh = bit & 31;
      d[w] |= (uint32_t)idx[m] << sh;
      if (sh > 26) d[w + 1] |= (uint32_t)idx[m] >> (32 - sh);
    }
    dst[0] = d[0]; dst[1] = d[1]; dst[2] = d[2];
  } else {
    u32x4 v;
    uint32_t d[4];
#pragma unroll
    for (int w = 0; w < 4; ++w)
      d[w] = (uint32_t)idx[4 * w] | ((uint32_t)idx[4 * w + 1] << 8) | ((uint32_t)idx[4 * w + 2] << 16) |
             ((uint32_t)idx[4 * w + 3] << 24);
    v.x = d[0]; v.y = d[1]; v.z = d[2]; v.w = d[3];
    *reinterpret_cast<u32x4*>(dst) = v;
  }
}

template <int NCW>
__device__ __forceinline__ void load_codes(const uint8_t* __restrict__ codes, int64_t gid, int q, int (&idx)[16]) {
  constexpr int c = CodeBits<NCW>::c;
  const uint32_t* src = reinterpret_cast<const uint32_t*>(codes + gid * (kGroup / 2 * c / 8) + q * (2 * c));
  if constexpr (c == 4) {
    const u32x2 v = *reinterpret_cast<const u32x2*>(src);
    const uint32_t d[2] = {v.x, v.y};
#pragma unroll
    for (int m = 0; m < 16; ++m) idx[m] = (d[m >> 3] >> (4 * (m & 7))) & 15;
  } else if constexpr (c == 6) {
    const uint32_t d[3] = {src[0], src[1], src[2]};
#pragma unroll
    for (int m = 0; m < 16; ++m) {
      const int bit = 6 * m, w = bit >> 5, sh = bit & 31;
      uint32_t x = d[w] >> sh;
      if (sh > 26) x |= d[w + 1] << (32 - sh);
      idx[m] = x & 63;
    }
  } else {
    const u32x4 v = *reinterpret_cast<const u32x4*>(src);
    const uint32_t d[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int m = 0; m < 16; ++m) idx[m] = (d[m >> 2] >> (8 * (m & 3))) & 255;
  }
}

__device__ __forceinline__ float half_bits_to_float(uint16_t h) {
  return static_cast<float>(__builtin_bit_cast(_Float16, h));
}

// codes + scale of one lane's part of a group -> zhat (rotated, scaled by sigma16)
__device__ __forceinline__ void gather_zhat(const int (&idx)[16], float s16, const float4* cb, float (&z)[32]) {
#pragma unroll
  for (int m = 0; m < 16; ++m) {
    const float4 cw = cb[idx[m]];
    z[2 * m] = cw.x * s16;
    z[2 * m + 1] = cw.y * s16;
  }
}

struct Lds {
  float4 cb[256];
  uint32_t table[kCells * kCells];
};

template <int NCW>
__device__ __forceinline__ void stage_lds(Lds& lds, const float* __restrict__ codebook,
                                          const uint32_t* __restrict__ table) {
  load_codebook<NCW>(codebook, lds.cb);
  if (table != nullptr) {
    const u32x4* src = reinterpret_cast<const u32x4*>(table);
    u32x4* dst = reinterpret_cast<u32x4*>(lds.table);
    for (int i = threadIdx.x; i < kCells * kCells / 4; i += kThreads) dst[i] = src[i];
  }
  __syncthreads();
}

// ------------------------------------------------------------------ quantize
template <typename T, int NCW>
__global__ __launch_bounds__(kThreads) void quantize_kernel(const T* X, const float* __restrict__ P,
                                                            const int8_t* __restrict__ signs,
                                                            const float* __restrict__ codebook,
                                                            const uint32_t* __restrict__ table,
                                                            uint8_t* __restrict__ codes, uint16_t* __restrict__ scales,
                                                            T* Xhat, int64_t n_groups, int H) {
  __shared__ Lds lds;
  stage_lds<NCW>(lds, codebook, table);
  const int q = threadIdx.x & 3;
  for (int64_t g0 = (int64_t)blockIdx.x * kGroupsPerBlock; g0 < n_groups; g0 += (int64_t)gridDim.x * kGroupsPerBlock) {
    int64_t gid = g0 + (threadIdx.x >> 2);
    const bool active = gid < n_groups;
    if (!active) gid = n_groups - 1;                      // keep every lane in the DPP exchanges
    const int head = (int)(gid % H);
    const int64_t off = gid * kGroup + q * kValsPerLane;

    float v[32], p[32];
    uint32_t sb[32];
    Storage<T>::load32(X + off, v);
    if (P != nullptr) {
      load32_f32(P + off, p);
    } else {
#pragma unroll
      for (int r = 0; r < 32; ++r) p[r] = 0.f;
    }
    load_sign_bits(signs, head, q, sb);
#pragma unroll
    for (int r = 0; r < 32; ++r) v[r] = __uint_as_float(__float_as_uint(v[r] - p[r]) ^ sb[r]);   // s * (x - p)
    wht128(v, q);                                           // w = H u (unnormalised)

    float ss = 0.f;
#pragma unroll
    for (int r = 0; r < 32; ++r) ss = __fmaf_rn(v[r], v[r], ss);
    ss = quad_sum(ss);
    // z = w / sqrt(g)  =>  rms(z) = sqrt(sum w^2) / g
    float sigma = __fsqrt_rn(ss) * (1.0f / kGroup);
    sigma = fminf(sigma, 65504.0f);
    const _Float16 s16h = static_cast<_Float16>(sigma);     // round to nearest even
    const float s16 = static_cast<float>(s16h);
    const float inv = s16 > 0.f ? __fdiv_rn(kRsqrtG, s16) : 0.f;

    int idx[16];
#pragma unroll
    for (int m = 0; m < 16; ++m) {
      const float y0 = v[2 * m] * inv, y1 = v[2 * m + 1] * inv;
      idx[m] = table != nullptr ? search_cell<NCW>(y0, y1, lds.cb, lds.table) : search_full<NCW>(y0, y1, lds.cb);
    }
    if (active) {
      store_codes<NCW>(codes, gid, q, idx);
      if (q == 0) scales[gid] = __builtin_bit_cast(uint16_t, s16h);
    }
    if (Xhat != nullptr) {
      gather_zhat(idx, s16, lds.cb, v);
      reconstruct(v, q, sb, p);
      if (active) Storage<T>::store32(Xhat + off, v);
    }
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
  __syncthreads();
  const int q = threadIdx.x & 3;
  for (int64_t g0 = (int64_t)blockIdx.x * kGroupsPerBlock; g0 < n_groups; g0 += (int64_t)gridDim.x * kGroupsPerBlock) {
    int64_t gid = g0 + (threadIdx.x >> 2);
    const bool active = gid < n_groups;
    if (!active) gid = n_groups - 1;
    const int head = (int)(gid % H);
    const int64_t off = gid * kGroup + q * kValsPerLane;

    float p[32], z[32];
    uint32_t sb[32];
    int idx[16];
    load_codes<NCW>(codes, gid, q, idx);
    const float s16 = half_bits_to_float(scales[gid]);
    if (P != nullptr) {
      load32_f32(P + off, p);
    } else {
#pragma unroll
      for (int r = 0; r < 32; ++r) p[r] = 0.f;
    }
    load_sign_bits(signs, head, q, sb);
    gather_zhat(idx, s16, cb, z);
    reconstruct(z, q, sb, p);
    if (active) Storage<T>::store32(Xhat + off, z);
  }
}

// ------------------------------------------------------------------ dequantize + q.k
// Group gid = row * H + head of the chunk; row = b * seq_len + t (global row = row0 + row).
template <typename T, int NCW>
__global__ __launch_bounds__(kThreads) void attn_scores_kernel(
    const uint8_t* __restrict__ codes, const uint16_t* __restrict__ scales, const float* __restrict__ P,
    const int8_t* __restrict__ signs, const float* __restrict__ codebook, const T* __restrict__ qv_,
    float score_scale, float* __restrict__ scores, T* __restrict__ Khat_out, int64_t row0, int64_t n_groups,
    int seq_len, int H, int q_heads) {
  __shared__ float4 cb[NCW];
  load_codebook<NCW>(codebook, cb);
  __syncthreads();
  const int q = threadIdx.x & 3;
  const int rep = q_heads / H;
  for (int64_t g0 = (int64_t)blockIdx.x * kGroupsPerBlock; g0 < n_groups; g0 += (int64_t)gridDim.x * kGroupsPerBlock) {
    int64_t gid = g0 + (threadIdx.x >> 2);
    const bool active = gid < n_groups;
    if (!active) gid = n_groups - 1;
    const int head = (int)(gid % H);
    const int64_t row = row0 + gid / H;
    const int64_t b = row / seq_len;
    const int64_t t = row % seq_len;
    const int64_t off = gid * kGroup + q * kValsPerLane;

    float p[32], z[32];
    uint32_t sb[32];
    int idx[16];
    load_codes<NCW>(codes, gid, q, idx);
    const float s16 = half_bits_to_float(scales[gid]);
    if (P != nullptr) {
      load32_f32(P + off, p);
    } else {
#pragma unroll
      for (int r = 0; r < 32; ++r) p[r] = 0.f;
    }
    load_sign_bits(signs, head, q, sb);
    gather_zhat(idx, s16, cb, z);
    reconstruct(z, q, sb, p);
    if (Khat_out != nullptr && active) Storage<T>::store32(Khat_out + off, z);
#pragma unroll
    for (int r = 0; r < 32; ++r) z[r] = Storage<T>::round(z[r]);      // score the stored keys

    for (int r = 0; r < rep; ++r) {
      const int qh = head * rep + r;
      float qv[32];
      Storage<T>::load32(qv_ + ((int64_t)b * q_heads + qh) * kGroup + q * kValsPerLane, qv);
      float acc = 0.f;
#pragma unroll
      for (int i = 0; i < 32; ++i) acc = __fmaf_rn(qv[i], z[i], acc);
      acc = quad_sum(acc);
      if (active && q == 0) scores[((int64_t)b * q_heads + qh) * seq_len + t] = acc * score_scale;
    }
  }
}

// ------------------------------------------------------------------ search table builder
// One thread per cell.  Grid point j is dropped from a cell only if some single other point i
// is closer by more than `eps` everywhere in the enlarged cell.  d_j(y) - d_i(y) =
// -2 y.(C_j - C_i) + |C_j|^2 - |C_i|^2 is linear in y, so its minimum over the rectangle sits at
// a corner; border cells reach out to +-1e30 (a clamped scale lets |y| grow without bound).
// The list is a superset of the points that can win anywhere in the cell, also under the
// kernels' fp32 rounding.
__global__ void build_table_kernel(const float* __restrict__ codebook, int n, uint32_t* __restrict__ table) {
  const int cell = blockIdx.x * blockDim.x + threadIdx.x;
  if (cell >= kCells * kCells) return;
  const int cx = cell % kCells, cy = cell / kCells;
  const double far = 1e30;
  const double delta = 1e-4, eps = 1e-3;
  const double h = 2.0 * kCellHalfRange / kCells;
  double x0 = cx == 0 ? -far : -kCellHalfRange + cx * h, x1 = cx == kCells - 1 ? far : -kCellHalfRange + (cx + 1) * h;
  double y0 = cy == 0 ? -far : -kCellHalfRange + cy * h, y1 = cy == kCells - 1 ? far : -kCellHalfRange + (cy + 1) * h;
  x0 -= delta; y0 -= delta; x1 += delta; y1 += delta;
  const double cxs[4] = {x0, x1, x0, x1}, cys[4] = {y0, y0, y1, y1};
  uint32_t entry = 0;
  int count = 0, last = 0;
  for (int j = 0; j < n; ++j) {
    const double aj = codebook[2 * j], bj = codebook[2 * j + 1];
    bool dominated = false;
    for (int i = 0; i < n && !dominated; ++i) {
      if (i == j) continue;
      const double ai = codebook[2 * i], bi = codebook[2 * i + 1];
      const double gx = -2.0 * (aj - ai), gy = -2.0 * (bj - bi);
      const double c0 = (aj * aj + bj * bj) - (ai * ai + bi * bi);
      double mn = 1e300;
      for (int k = 0; k < 4; ++k) mn = fmin(mn, gx * cxs[k] + gy * cys[k] + c0);
      dominated = mn > eps;
    }
    if (!dominated) {
      if (count < 4) entry |= (uint32_t)j << (8 * count);
      last = j;
      ++count;
    }
  }
  if (count > (n == 16 ? 3 : 4)) {      // more than the kernels score per cell
    entry = kCellFull;
  } else {
    for (int k = count; k < 4; ++k) entry |= (uint32_t)last << (8 * k);   // repeat the last candidate
  }
  table[cell] = entry;
}

inline unsigned blocks_for(int64_t n_groups) {
  const int64_t need = (n_groups + kGroupsPerBlock - 1) / kGroupsPerBlock;
  const int64_t cap = 256 * 16;           // a few resident waves per SIMD on 256 CUs; the kernels grid-stride
  return (unsigned)(need < cap ? need : cap);
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

hipError_t launch_build_search_table(const float* codebook, int n_codewords, void* table, hipStream_t stream) {
  build_table_kernel<<<kCells * kCells / 64, 64, 0, stream>>>(codebook, n_codewords, static_cast<uint32_t*>(table));
  return hipGetLastError();
}

hipError_t launch_quantize(int dtype, int n_codewords, const void* X, const float* P, const int8_t* signs,
                           const float* codebook, const void* table, uint8_t* codes, uint16_t* scales, void* Xhat,
                           int64_t T_, int H, hipStream_t stream) {
  const int64_t n_groups = T_ * H;
  if (n_groups == 0) return hipSuccess;
  AQUAKV_DISPATCH(dtype, n_codewords,
                  (quantize_kernel<T, N><<<blocks_for(n_groups), kThreads, 0, stream>>>(
                      static_cast<const T*>(X), P, signs, codebook, static_cast<const uint32_t*>(table), codes, scales,
                      static_cast<T*>(Xhat), n_groups, H)));
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
