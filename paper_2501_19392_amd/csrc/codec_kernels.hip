// Streaming kernels of the backbone quantizer (Sect. 2 "Vector Quantization" of
// the AQUA-KV paper, HIGGS-style): quantize (residual -> RHT -> group scale ->
// nearest grid point -> packed codes, plus the reconstruction), dequantize, and
// dequantize fused with grouped-query q.k scoring; plus the builder of the
// nearest-grid-point search table.  These are the stand-alone forms (prediction
// read from memory, or absent); the fused forms live in fused_kernels.hip.
//
// One head group (128 values) is held by a quad of lanes x 32 values (see device_utils.h);
// a 256-thread block covers 64 head groups = 8 tokens of 8 heads per pass.  WIDE = true selects
// rotation groups of 1024 = the whole token (the grouping of the paper's experiments, Sect. 4.1):
// the 8 quads of a token (32 consecutive lanes) then share three more butterfly stages and one scale.
#include "codec_core.h"
#include "kernels.h"

namespace aquakv {
namespace {

constexpr int kThreads = 256;
constexpr int kGroupsPerBlock = kThreads / kLanesPerGroup;   // 64

// ------------------------------------------------------------------ quantize
template <typename T, int NCW, bool WIDE>
__global__ __launch_bounds__(kThreads) void quantize_kernel(const T* X, const float* __restrict__ P,
                                                            const int8_t* __restrict__ signs,
                                                            const float* __restrict__ codebook,
                                                            const uint32_t* __restrict__ table,
                                                            uint8_t* __restrict__ codes, uint16_t* __restrict__ scales,
                                                            T* Xhat, int64_t n_groups, int H) {
  __shared__ Lds lds;
  stage_lds<NCW>(lds, codebook, table);
  const int q = threadIdx.x & 3;
  // A thread meets the same head in every round of the grid-stride loop when the stride is a multiple of H (it is
  // for the power-of-two head counts in use): the signs are then fetched once.
  float sf[32] = {};
  const bool fixed_head = kGroupsPerBlock % H == 0;
  if constexpr (!is_rtn(NCW)) {
    if (fixed_head) load_signs(signs, (int)((blockIdx.x * (unsigned)kGroupsPerBlock + (threadIdx.x >> 2)) % (unsigned)H), q, sf);
  }
  // The rows (and the fp32 prediction) of the next round are requested before the current round is worked on: with two
  // waves per SIMD nothing else hides the latency of these loads.
  constexpr int kXQuads = sizeof(T) == 2 ? 4 : 8;
  struct Rows { u32x4 x[kXQuads]; f32x4 p[8]; };
  const auto request = [&](int64_t g0, Rows& r) {
    int64_t gid = g0 + (threadIdx.x >> 2);
    gid = gid < n_groups ? gid : n_groups - 1;
    const int64_t off = gid * kGroup + q * kValsPerLane;
    const u32x4* src = reinterpret_cast<const u32x4*>(X + off);
#pragma unroll
    for (int k = 0; k < kXQuads; ++k) r.x[k] = src[k];
    if (P != nullptr) {
#pragma unroll
      for (int k = 0; k < 8; ++k) r.p[k] = reinterpret_cast<const f32x4*>(P + off)[k];
    }
  };
  const int64_t stride = (int64_t)gridDim.x * kGroupsPerBlock;
  Rows cur;
  if ((int64_t)blockIdx.x * kGroupsPerBlock < n_groups) request((int64_t)blockIdx.x * kGroupsPerBlock, cur);
  for (int64_t g0 = (int64_t)blockIdx.x * kGroupsPerBlock; g0 < n_groups; g0 += stride) {
    Rows nxt;
    if (g0 + stride < n_groups) request(g0 + stride, nxt);
    int64_t gid = g0 + (threadIdx.x >> 2);
    const bool active = gid < n_groups;
    if (!active) gid = n_groups - 1;                      // keep every lane in the DPP exchanges
    const int64_t off = gid * kGroup + q * kValsPerLane;

    float v[32], p[32];
    if constexpr (sizeof(T) == 2) {
#pragma unroll
      for (int k = 0; k < 4; ++k) unpack_bf16x8(cur.x[k], &v[8 * k]);
    } else {
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        v[4 * k] = __uint_as_float(cur.x[k].x); v[4 * k + 1] = __uint_as_float(cur.x[k].y);
        v[4 * k + 2] = __uint_as_float(cur.x[k].z); v[4 * k + 3] = __uint_as_float(cur.x[k].w);
      }
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const f32x4 a = P != nullptr ? cur.p[k] : f32x4{0.f, 0.f, 0.f, 0.f};
      p[4 * k] = a.x; p[4 * k + 1] = a.y; p[4 * k + 2] = a.z; p[4 * k + 3] = a.w;
    }
    if constexpr (!is_rtn(NCW)) {
      if (!fixed_head) load_signs(signs, (int)(gid % H), q, sf);     // (a 64-bit remainder: kept off the common path)
    }
    quantize_group<NCW, WIDE>(v, p, sf, WIDE ? (int)(threadIdx.x & 31) : q, lds.cb, table != nullptr ? lds.table : nullptr,
                              active, gid, codes, scales, Xhat != nullptr);
    if (Xhat != nullptr && active) Storage<T>::store32(Xhat + off, v);
    cur = nxt;
  }
}

// ------------------------------------------------------------------ dequantize
template <typename T, int NCW, bool WIDE>
__global__ __launch_bounds__(kThreads) void dequantize_kernel(const uint8_t* __restrict__ codes,
                                                              const uint16_t* __restrict__ scales,
                                                              const float* __restrict__ P,
                                                              const int8_t* __restrict__ signs,
                                                              const float* __restrict__ codebook, T* __restrict__ Xhat,
                                                              int64_t n_groups, int H) {
  __shared__ float4 cb[is_rtn(NCW) ? 1 : NCW];
  load_codebook<NCW>(codebook, cb);
  __syncthreads();
  const int q = threadIdx.x & 3;
  // A thread meets the same head in every round of the grid-stride loop when the stride is a multiple of H (it is
  // for the power-of-two head counts in use): the signs are then fetched once.
  float sf[32] = {};
  const bool fixed_head = kGroupsPerBlock % H == 0;
  if constexpr (!is_rtn(NCW)) {
    if (fixed_head) load_signs(signs, (int)((blockIdx.x * (unsigned)kGroupsPerBlock + (threadIdx.x >> 2)) % (unsigned)H), q, sf);
  }
  // the code and scale words of the next round are requested before the current round is worked on
  const auto request = [&](int64_t g0) {
    int64_t gid = g0 + (threadIdx.x >> 2);
    gid = gid < n_groups ? gid : n_groups - 1;
    return request_words<NCW, WIDE>(codes, scales, gid, q);
  };
  const int64_t stride = (int64_t)gridDim.x * kGroupsPerBlock;
  CodeWords cur = {};
  if ((int64_t)blockIdx.x * kGroupsPerBlock < n_groups) cur = request((int64_t)blockIdx.x * kGroupsPerBlock);
  for (int64_t g0 = (int64_t)blockIdx.x * kGroupsPerBlock; g0 < n_groups; g0 += stride) {
    CodeWords nxt = {};
    if (g0 + stride < n_groups) nxt = request(g0 + stride);
    int64_t gid = g0 + (threadIdx.x >> 2);
    const bool active = gid < n_groups;
    if (!active) gid = n_groups - 1;
    const int64_t off = gid * kGroup + q * kValsPerLane;

    float p[32], z[32];
    if (P != nullptr) {
      load32_f32(P + off, p);
    } else {
#pragma unroll
      for (int r = 0; r < 32; ++r) p[r] = 0.f;
    }
    if constexpr (!is_rtn(NCW)) {
      if (!fixed_head) load_signs(signs, (int)(gid % H), q, sf);     // (a 64-bit remainder: kept off the common path)
    }
    dequantize_words<NCW, WIDE>(cur, p, sf, WIDE ? (int)(threadIdx.x & 31) : q, cb, z);
    if (active) Storage<T>::store32(Xhat + off, z);
    cur = nxt;
  }
}

// ------------------------------------------------------------------ dequantize + q.k
// Group gid = row * H + head of the chunk; row = b * seq_len + t (global row = row0 + row).
template <typename T, int NCW, bool WIDE>
__global__ __launch_bounds__(kThreads) void attn_scores_kernel(
    const uint8_t* __restrict__ codes, const uint16_t* __restrict__ scales, const float* __restrict__ P,
    const int8_t* __restrict__ signs, const float* __restrict__ codebook, const T* __restrict__ qv_,
    float score_scale, float* __restrict__ scores, T* __restrict__ Khat_out, int64_t row0, int64_t n_groups,
    int seq_len, int H, int q_heads, const float* __restrict__ rope_cos, const float* __restrict__ rope_sin) {
  __shared__ float4 cb[is_rtn(NCW) ? 1 : NCW];
  load_codebook<NCW>(codebook, cb);
  __syncthreads();
  const int q = threadIdx.x & 3;
  // A thread meets the same head in every round of the grid-stride loop when the stride is a multiple of H (it is
  // for the power-of-two head counts in use): the signs are then fetched once.
  float sf[32] = {};
  const bool fixed_head = kGroupsPerBlock % H == 0;
  if constexpr (!is_rtn(NCW)) {
    if (fixed_head) load_signs(signs, (int)((blockIdx.x * (unsigned)kGroupsPerBlock + (threadIdx.x >> 2)) % (unsigned)H), q, sf);
  }
  const int rep = q_heads / H;
  const auto request = [&](int64_t g0) {
    int64_t gid = g0 + (threadIdx.x >> 2);
    gid = gid < n_groups ? gid : n_groups - 1;
    return request_words<NCW, WIDE>(codes, scales, gid, q);
  };
  const int64_t stride = (int64_t)gridDim.x * kGroupsPerBlock;
  CodeWords cur = {};
  if ((int64_t)blockIdx.x * kGroupsPerBlock < n_groups) cur = request((int64_t)blockIdx.x * kGroupsPerBlock);
  for (int64_t g0 = (int64_t)blockIdx.x * kGroupsPerBlock; g0 < n_groups; g0 += stride) {
    CodeWords nxt = {};
    if (g0 + stride < n_groups) nxt = request(g0 + stride);
    int64_t gid = g0 + (threadIdx.x >> 2);
    const bool active = gid < n_groups;
    if (!active) gid = n_groups - 1;
    const int head = (int)(gid % H);
    const int64_t row = row0 + gid / H;
    const int64_t b = row / seq_len;
    const int64_t t = row % seq_len;
    const int64_t off = gid * kGroup + q * kValsPerLane;

    float p[32], z[32];
    if (P != nullptr) {
      load32_f32(P + off, p);
    } else {
#pragma unroll
      for (int r = 0; r < 32; ++r) p[r] = 0.f;
    }
    if constexpr (!is_rtn(NCW)) {
      if (!fixed_head) load_signs(signs, (int)(gid % H), q, sf);     // (a 64-bit remainder: kept off the common path)
    }
    dequantize_words<NCW, WIDE>(cur, p, sf, WIDE ? (int)(threadIdx.x & 31) : q, cb, z);
    cur = nxt;
    if (Khat_out != nullptr && active) Storage<T>::store32(Khat_out + off, z);
#pragma unroll
    for (int r = 0; r < 32; ++r) z[r] = Storage<T>::round(z[r]);      // score the stored keys
    if (rope_cos != nullptr) rope128(z, q, rope_cos + t * (kGroup / 2), rope_sin + t * (kGroup / 2));   // cached before RoPE

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
// Grid point j is dropped from a cell only if some single other point i is closer by more than `eps` everywhere in
// the enlarged cell.  d_j(y) - d_i(y) = -2 y.(C_j - C_i) + |C_j|^2 - |C_i|^2 is linear in y, so its minimum over the
// rectangle sits at a corner; border cells reach out to +-1e30 (a clamped scale lets |y| grow without bound).
// The list is a superset of the points that can win anywhere in the cell, also under the kernels' fp32 rounding.
// Returns the number of candidates; the first kOvfCand of them (indices, ascending) go to cand[].
__device__ int cell_candidates(const float* __restrict__ codebook, int n, int cell, int (&cand)[kOvfCand]) {
  const int cx = cell % kCells, cy = cell / kCells;
  const double far = 1e30;
  const double delta = 1e-4, eps = 1e-3;
  const double R = cell_half_range(n);
  const double h = 2.0 * R / kCells;
  double x0 = cx == 0 ? -far : -R + cx * h, x1 = cx == kCells - 1 ? far : -R + (cx + 1) * h;
  double y0 = cy == 0 ? -far : -R + cy * h, y1 = cy == kCells - 1 ? far : -R + (cy + 1) * h;
  x0 -= delta; y0 -= delta; x1 += delta; y1 += delta;
  const double cxs[4] = {x0, x1, x0, x1}, cys[4] = {y0, y0, y1, y1};
  int count = 0;
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
#pragma unroll
      for (int k = 0; k < kOvfCand; ++k)
        if (k == count) cand[k] = j;
      ++count;
    }
  }
  return count;
}

// candidates -> `bytes` slot bytes, ascending, the last one repeated (little-endian into 32-bit words)
__device__ void pack_candidates(const int (&cand)[kOvfCand], int count, int shift, int bytes, uint32_t (&w)[2]) {
  w[0] = w[1] = 0;
#pragma unroll
  for (int k = 0; k < kOvfCand; ++k) {
    int c = 0;
#pragma unroll
    for (int t = 0; t < kOvfCand; ++t)
      if (t == (k < count ? k : count - 1)) c = cand[t];
    if (k < bytes) w[k >> 2] |= (uint32_t)(c << shift) << (8 * (k & 3));
  }
}

// First pass, one thread per cell: the ordinary entries; cells that need an overflow list of their own are left marked
// "full search".  With 256 points the cells that list nothing but point 255 name the shared list 0.
__global__ void build_table_kernel(const float* __restrict__ codebook, int n, uint32_t* __restrict__ table) {
  const int cell = blockIdx.x * blockDim.x + threadIdx.x;
  if (cell >= kCellWords) return;
  int cand[kOvfCand];
  const int count = cell_candidates(codebook, n, cell, cand);
  uint32_t w[2];
  pack_candidates(cand, count < 4 ? count : 4, slot_shift(n), 4, w);
  const bool ordinary = count <= (n == 16 ? 3 : 4) && w[0] < crowded_threshold(n);
  const bool only_last = n == 256 && count == 1 && cand[0] == n - 1;
  table[cell] = ordinary ? w[0] : crowded_entry(n, only_last ? 0u : slot_top(n));
}

// Second pass, one workgroup: the marked cells get overflow lists in cell order (a fixed table for a given grid).  A cell
// with more than kOvfCand candidates, or one that finds no list left, stays "full search".
__global__ __launch_bounds__(1024) void build_overflow_kernel(const float* __restrict__ codebook, int n,
                                                              uint32_t* __restrict__ table) {
  __shared__ int offs[1024];
  constexpr int kPer = kCellWords / 1024;
  const uint32_t marked = crowded_entry(n, slot_top(n));
  int mine = 0;
  for (int k = 0; k < kPer; ++k) mine += table[threadIdx.x * kPer + k] == marked;
  offs[threadIdx.x] = mine;
  __syncthreads();
  for (int d = 1; d < 1024; d <<= 1) {                    // inclusive scan
    const int add = (int)threadIdx.x >= d ? offs[threadIdx.x - d] : 0;
    __syncthreads();
    offs[threadIdx.x] += add;
    __syncthreads();
  }
  const int first = n == 256 ? 1 : 0;                     // list 0 of the 256-point grid: point 255 alone
  int list = first + offs[threadIdx.x] - mine;            // lists before this thread's cells
  // unused lists name point 0; the shared list names the last point in every byte
  for (int k = threadIdx.x; k < 2 * kOvfLists; k += 1024) table[kCellWords + k] = (first && k < 2) ? 0xFFFFFFFFu : 0u;
  __syncthreads();
  for (int k = 0; k < kPer; ++k) {
    const int cell = threadIdx.x * kPer + k;
    if (table[cell] != marked) continue;
    int cand[kOvfCand];
    const int count = cell_candidates(codebook, n, cell, cand);
    if (count <= kOvfCand && list < ovf_capacity(n)) {
      uint32_t w[2];
      pack_candidates(cand, count, slot_shift(n), kOvfCand, w);
      table[kCellWords + 2 * list] = w[0];
      table[kCellWords + 2 * list + 1] = w[1];
      table[cell] = crowded_entry(n, (uint32_t)list << slot_shift(n));
    }
    ++list;
  }
}

// Workgroups per CU (256 CUs), the kernels grid-stride.  The quantizer holds two workgroups per CU (registers) and stages
// 21 KiB of grid and cell table per workgroup, more than the 16 KiB of rows of one round: with exactly the resident
// number of workgroups the staging is paid once and the request of the next round's rows has a next round to run ahead
// of (measured at 32768 tokens: 52 us against 67 us with 16 per CU).  The inverse stages 256 B and runs four waves per
// SIMD; four workgroups per CU were the best of 2 / 4 / 8 / 16 at 32768 tokens (25.7 against 29 us with 16).
constexpr int kQuantizeWgPerCu = 2;
constexpr int kDequantizeWgPerCu = 4;
inline unsigned blocks_for(int64_t n_groups, int per_cu) {
  const int64_t need = (n_groups + kGroupsPerBlock - 1) / kGroupsPerBlock;
  const int64_t cap = 256 * per_cu;
  return (unsigned)(need < cap ? need : cap);
}

}  // namespace

#define AQUAKV_DISPATCH_GRID(NCW, CALL)                                                 \
  do {                                                                                  \
    if ((NCW) == 16) { constexpr int N = 16; CALL; }                                    \
    else if ((NCW) == 64) { constexpr int N = 64; CALL; }                               \
    else { constexpr int N = 256; CALL; }                                               \
  } while (0)
#define AQUAKV_DISPATCH_N(NCW, CALL)                                                    \
  do {                                                                                  \
    if ((NCW) == kRtn2) { constexpr int N = kRtn2; CALL; }                              \
    else if ((NCW) == kRtn4) { constexpr int N = kRtn4; CALL; }                         \
    else AQUAKV_DISPATCH_GRID(NCW, CALL);                                               \
  } while (0)
// binds T (storage type), N (quantizer id: grid size, or kRtn2 / kRtn4) and W (groups of 1024 = the whole token)
// as compile-time names for CALL
#define AQUAKV_DISPATCH(DT, NCW, WIDE_, CALL)                                           \
  do {                                                                                  \
    if ((DT) == kBF16) {                                                                \
      typedef bf16_t T;                                                                 \
      if (WIDE_) { constexpr bool W = true; AQUAKV_DISPATCH_N(NCW, CALL); }             \
      else { constexpr bool W = false; AQUAKV_DISPATCH_N(NCW, CALL); }                  \
    } else {                                                                            \
      typedef float T;                                                                  \
      if (WIDE_) { constexpr bool W = true; AQUAKV_DISPATCH_N(NCW, CALL); }             \
      else { constexpr bool W = false; AQUAKV_DISPATCH_N(NCW, CALL); }                  \
    }                                                                                   \
  } while (0)

hipError_t launch_build_search_table(const float* codebook, int n_codewords, void* table, hipStream_t stream) {
  build_table_kernel<<<kCellWords / 64, 64, 0, stream>>>(codebook, n_codewords, static_cast<uint32_t*>(table));
  build_overflow_kernel<<<1, 1024, 0, stream>>>(codebook, n_codewords, static_cast<uint32_t*>(table));
  return hipGetLastError();
}

hipError_t launch_quantize(int dtype, int n_codewords, const void* X, const float* P, const int8_t* signs,
                           const float* codebook, const void* table, uint8_t* codes, uint16_t* scales, void* Xhat,
                           int64_t T_, int H, bool wide, hipStream_t stream) {
  const int64_t n_groups = T_ * H;
  if (n_groups == 0) return hipSuccess;
  AQUAKV_DISPATCH(dtype, n_codewords, wide,
                  (quantize_kernel<T, N, W><<<blocks_for(n_groups, kQuantizeWgPerCu), kThreads, 0, stream>>>(
                      static_cast<const T*>(X), P, signs, codebook, static_cast<const uint32_t*>(table), codes, scales,
                      static_cast<T*>(Xhat), n_groups, H)));
  return hipGetLastError();
}

hipError_t launch_dequantize(int dtype, int n_codewords, const uint8_t* codes, const uint16_t* scales, const float* P,
                             const int8_t* signs, const float* codebook, void* Xhat, int64_t T_, int H, bool wide,
                             hipStream_t stream) {
  const int64_t n_groups = T_ * H;
  if (n_groups == 0) return hipSuccess;
  AQUAKV_DISPATCH(dtype, n_codewords, wide,
                  (dequantize_kernel<T, N, W><<<blocks_for(n_groups, kDequantizeWgPerCu), kThreads, 0, stream>>>(
                      codes, scales, P, signs, codebook, static_cast<T*>(Xhat), n_groups, H)));
  return hipGetLastError();
}

hipError_t launch_attn_scores(int dtype, int n_codewords, const uint8_t* codes, const uint16_t* scales, const float* P,
                              const int8_t* signs, const float* codebook, const void* q, float score_scale,
                              float* scores, void* Khat_out, int64_t row0, int64_t rows, int seq_len, int H,
                              int q_heads, const float* rope_cos, const float* rope_sin, bool wide, hipStream_t stream) {
  const int64_t n_groups = rows * H;
  if (n_groups == 0) return hipSuccess;
  AQUAKV_DISPATCH(dtype, n_codewords, wide,
                  (attn_scores_kernel<T, N, W><<<blocks_for(n_groups, kDequantizeWgPerCu), kThreads, 0, stream>>>(
                      codes, scales, P, signs, codebook, static_cast<const T*>(q), score_scale, scores,
                      static_cast<T*>(Khat_out), row0, n_groups, seq_len, H, q_heads, rope_cos, rope_sin)));
  return hipGetLastError();
}

}  // namespace aquakv
