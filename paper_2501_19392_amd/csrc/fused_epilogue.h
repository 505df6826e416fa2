// Pieces of the epilogue that the fused predictor kernels share (fused_kernels.hip: tiles of 256 tokens x one kv
// head; fused_two_heads.hip: x two heads): the layout of a parked block of predictions in LDS, and the tails of
// Alg. "decode" of the AQUA-KV paper on one rotation group per quad of lanes (groups of one head).  One copy of
// each, so that both tiles produce the same bits by construction.
#pragma once
#include "codec_core.h"
#include "gemm_core.h"

namespace aquakv {

constexpr int kLdP = kGroup + 4;                    // padded fp32 row of a parked block
// Position of column `col` inside a parked row.  A quad reads 16-byte slot 8q + k of a row in
// its k-th load; q and q+2 would be 128 B = half the banks apart and collide with the next
// rows, so the upper half of the row has its slots XOR-ed by 4: the 16 lanes served together
// (4 rows x 4 lanes) then touch all 64 banks once.
__device__ __forceinline__ constexpr int park_col(int col) {
  const int slot = col >> 2;
  return (((slot & 16) ? (slot ^ 4) : slot) << 2) | (col & 3);
}

// One 32 x 128 block of a wave's accumulators (+ bias) -> rows 0..31 at `dst` (row stride kLdP floats).  acc[j]: the
// 32 x 32 block of columns 32 j; the lane holds column lane % 32 and rows 8 b + 4 (lane / 32) + r in register 4 b + r.
__device__ __forceinline__ void park_block(float* dst, const f32x16 (&acc)[4], const float (&bv)[4], int lane) {
  const int frow = lane & 31, fk = lane >> 5;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int lrow = (r >> 2) * 8 + fk * 4 + (r & 3);
      dst[lrow * kLdP + park_col(j * 32 + frow)] = acc[j][r] + bv[j];
    }
}

// the 32 predictions of quad position q of a parked row
__device__ __forceinline__ void read_parked(const float* rowp, int q, float (&p)[32]) {
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const f32x4 a = *reinterpret_cast<const f32x4*>(rowp + park_col(q * kValsPerLane + 4 * k));
    p[4 * k] = a.x; p[4 * k + 1] = a.y; p[4 * k + 2] = a.z; p[4 * k + 3] = a.w;
  }
}

// Rotation groups of 1024 = the whole token of 8 heads (Sect. 4.1), decoded by a quad that holds ONE head of the token:
// the code words of the lane's 16 sub-vector slots in each of the 8 heads ...
template <int NCW> struct WideCodes { u32x4 h[8]; };
template <int NCW>
__device__ __forceinline__ void request_wide_codes(const uint8_t* __restrict__ codes, int64_t row, int q, WideCodes<NCW>& wc) {
#pragma unroll
  for (int hh = 0; hh < 8; ++hh) wc.h[hh] = request_codes<NCW>(codes, row * 8 + hh, q);
}
// ... and Q^-1 + p from them (grids): the grid points of the 8 heads, added as the stages across the heads of the
// 1024-point transform add them for head `head`, ((0 +- 1) +- (2 +- 3)) +- ((4 +- 5) +- (6 +- 7)), minus where the
// head's bit of that level is set (the tree of Rot<true>::iwht, so the same bits as the stand-alone kernels), then the
// quad's own 128-point stages, sign and prediction.  scale_word: the token's fp16 scale.
template <int NCW>
__device__ __forceinline__ void dequantize_across_heads(const WideCodes<NCW>& wc, uint32_t scale_word, int head, int q,
                                                        const float (&p)[32], const float (&sf)[32], const float4* cb,
                                                        float (&v)[32]) {
  const float s16 = recon_scale<true>(half_bits_to_float((uint16_t)scale_word), q);   // the quad's two lane bits only
  const float g0 = (head & 1) ? -1.0f : 1.0f, g1 = (head & 2) ? -1.0f : 1.0f, g2 = (head & 4) ? -1.0f : 1.0f;
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    const auto zhat_half = [&](int hh, float (&z)[16]) {
      int idx[16];
      unpack_codes<NCW>(wc.h[hh], idx);
#pragma unroll
      for (int m = 0; m < 8; ++m) {
        const float2 cw = *reinterpret_cast<const float2*>(&cb[idx[8 * half + m]]);
        z[2 * m] = cw.x * s16;
        z[2 * m + 1] = cw.y * s16;
      }
    };
    const auto pair_of = [&](int hh, float (&t)[16]) {        // z[hh] +- z[hh + 1]
      float b[16];
      zhat_half(hh, t);
      zhat_half(hh + 1, b);
#pragma unroll
      for (int i = 0; i < 16; ++i) t[i] = __fmaf_rn(b[i], g0, t[i]);
    };
    float u0[16], u1[16], t[16];
    pair_of(0, u0);
    pair_of(2, t);
#pragma unroll
    for (int i = 0; i < 16; ++i) u0[i] = __fmaf_rn(t[i], g1, u0[i]);
    pair_of(4, u1);
    pair_of(6, t);
#pragma unroll
    for (int i = 0; i < 16; ++i) u1[i] = __fmaf_rn(t[i], g1, u1[i]);
#pragma unroll
    for (int i = 0; i < 16; ++i) v[16 * half + i] = __fmaf_rn(u1[i], g2, u0[i]);
  }
  wht128<true>(v, q);
#pragma unroll
  for (int r = 0; r < 32; ++r) v[r] = __fmaf_rn(v[r], sf[r], p[r]);
}

// Grouped-query scores of one decoded key row of kv head `head` (the quad's 4 x 32 values in v, unrounded):
//   scores[b, qh, t] = score_scale * sum_d q[b, qh, d] * round_bf16(v)[d]   for the q_heads / H query heads of the head,
// the key rotated by its position t first when rope_cos is given (caches that hold keys from before the rotary
// embedding, Sect. 3.3).  Row index rowc = b * seq_len + t.
// q_lds (nullable): the queries of this row's sequence for the query heads of `head`, staged by the caller as fp32,
// kQueryLdsStride floats per query head, quad position q at float q * kQueryLdsQuad (stage_queries below); the same
// values as in memory, so the same bits either way.
constexpr int kQueryLdsQuad = kValsPerLane + 4;          // 144-byte steps: the four quad positions fall on disjoint banks
constexpr int kQueryLdsStride = 4 * kQueryLdsQuad;
// The queries a tile scores against, on their way to LDS: when the tile's rows [m0, m0 + rows) lie inside one sequence, the
// n_qh query heads from first_qh on (adjacent in memory: the query heads of the tile's kv heads) are requested early, 4
// values per thread, and stored as fp32 once the LDS is free; the epilogue then reads them from LDS instead of waiting
// for memory once per query head and pass.  n_qh <= 16.
struct QueryStage {
  u32x2 regs;
  bool staged;
  __device__ __forceinline__ void request(const bf16_t* __restrict__ qv, int64_t m0, int rows, int64_t T, int seq_len,
                                          int q_heads, int first_qh, int n_qh) {
    const int64_t last = m0 + rows - 1 < T ? m0 + rows - 1 : T - 1;
    const int64_t b = m0 / seq_len;
    regs = u32x2{0, 0};
    staged = last / seq_len == b && n_qh * kGroup <= 4 * (int)blockDim.x;
    if (staged && (int)threadIdx.x * 4 < n_qh * kGroup)
      regs = *reinterpret_cast<const u32x2*>(qv + (b * q_heads + first_qh) * kGroup + threadIdx.x * 4);
  }
  __device__ __forceinline__ void store(float* q_lds, int n_qh) const {
    if (staged && (int)threadIdx.x * 4 < n_qh * kGroup) {
      const int e = threadIdx.x * 4, qh = e / kGroup, d = e % kGroup;       // 4 consecutive values of one quad position
      f32x4 f;
      f.x = __uint_as_float(regs.x << 16); f.y = __uint_as_float(regs.x & 0xffff0000u);
      f.z = __uint_as_float(regs.y << 16); f.w = __uint_as_float(regs.y & 0xffff0000u);
      *reinterpret_cast<f32x4*>(q_lds + qh * kQueryLdsStride + (d / kValsPerLane) * kQueryLdsQuad + d % kValsPerLane) = f;
    }
  }
};

__device__ __forceinline__ void score_row(float (&v)[32], int q, int head, int H, int q_heads, int seq_len, int64_t rowc,
                                          bool active, const bf16_t* __restrict__ qv, float score_scale,
                                          float* __restrict__ scores, const float* __restrict__ rope_cos,
                                          const float* __restrict__ rope_sin, const float* q_lds = nullptr) {
#pragma unroll
  for (int r = 0; r < 32; ++r) v[r] = Storage<bf16_t>::round(v[r]);      // score the stored keys
  const int rep = q_heads / H;
  const int64_t b = rowc / seq_len, t = rowc % seq_len;
  if (rope_cos != nullptr) rope128(v, q, rope_cos + t * (kGroup / 2), rope_sin + t * (kGroup / 2));
  for (int r = 0; r < rep; ++r) {
    const int qh = head * rep + r;
    float qf[32];
    if (q_lds != nullptr) {
      const float* src = q_lds + r * kQueryLdsStride + q * kQueryLdsQuad;
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const f32x4 a = *reinterpret_cast<const f32x4*>(src + 4 * k);
        qf[4 * k] = a.x; qf[4 * k + 1] = a.y; qf[4 * k + 2] = a.z; qf[4 * k + 3] = a.w;
      }
    } else {
      Storage<bf16_t>::load32(qv + (b * q_heads + qh) * kGroup + q * kValsPerLane, qf);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 32; ++i) s = __fmaf_rn(qf[i], v[i], s);
    s = quad_sum(s);
    if (active && q == 0) scores[(b * q_heads + qh) * seq_len + t] = s * score_scale;
  }
}

}  // namespace aquakv
