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
__device__ __forceinline__ void score_row(float (&v)[32], int q, int head, int H, int q_heads, int seq_len, int64_t rowc,
                                          bool active, const bf16_t* __restrict__ qv, float score_scale,
                                          float* __restrict__ scores, const float* __restrict__ rope_cos,
                                          const float* __restrict__ rope_sin) {
#pragma unroll
  for (int r = 0; r < 32; ++r) v[r] = Storage<bf16_t>::round(v[r]);      // score the stored keys
  const int rep = q_heads / H;
  const int64_t b = rowc / seq_len, t = rowc % seq_len;
  if (rope_cos != nullptr) rope128(v, q, rope_cos + t * (kGroup / 2), rope_sin + t * (kGroup / 2));
  for (int r = 0; r < rep; ++r) {
    const int qh = head * rep + r;
    float qf[32];
    Storage<bf16_t>::load32(qv + (b * q_heads + qh) * kGroup + q * kValsPerLane, qf);
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 32; ++i) s = __fmaf_rn(qf[i], v[i], s);
    s = quad_sum(s);
    if (active && q == 0) scores[(b * q_heads + qh) * seq_len + t] = s * score_scale;
  }
}

}  // namespace aquakv
