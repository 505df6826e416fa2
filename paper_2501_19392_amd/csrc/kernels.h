// Host-side launchers of the gfx950 kernels (one per stage).  Arguments are
// validated by the C-ABI layer before these are called.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace aquakv {

enum Dtype : int { kBF16 = 0, kFP32 = 1 };

// P[T, D] = [x0 (T x d0) | x1 (T x d1)] W^T + bias, W is [D, d0 + d1] row-major.
hipError_t launch_predict(int dtype, const void* x0, int d0, const void* x1, int d1, const void* W,
                          const float* bias, float* P, int64_t T, int D, hipStream_t stream);

// Q(X - P): codes, scales and (optionally) the reconstruction.  rows = T, H heads of 128.
// wide: rotation groups of 1024 = the whole token (H must be 8), scales [T] instead of [T, H].
// `table` (nullable): nearest-grid-point search table from launch_build_search_table.
hipError_t launch_quantize(int dtype, int n_codewords, const void* X, const float* P, const int8_t* signs,
                           const float* codebook, const void* table, uint8_t* codes, uint16_t* scales, void* Xhat,
                           int64_t T, int H, bool wide, hipStream_t stream);

// 64 x 64 cells x 4 candidate bytes = 16 KiB, and 128 overflow lists of 8 candidate bytes.
constexpr size_t kSearchTableBytes = (64 * 64 + 2 * 128) * 4;     // cell entries + overflow lists (codec_core.h)
hipError_t launch_build_search_table(const float* codebook, int n_codewords, void* table, hipStream_t stream);

hipError_t launch_dequantize(int dtype, int n_codewords, const uint8_t* codes, const uint16_t* scales, const float* P,
                             const int8_t* signs, const float* codebook, void* Xhat, int64_t T, int H, bool wide,
                             hipStream_t stream);

// scores[b, qh, t] for rows [row0, row0 + rows) of the flattened [batch*seq_len] axis.
// codes/scales/P/Khat_out point at row `row0`; q and scores at their tensor bases.
// rope_cos / rope_sin (nullable, fp32 [seq_len, 64]): rotate the decoded key of token t by position t first.
hipError_t launch_attn_scores(int dtype, int n_codewords, const uint8_t* codes, const uint16_t* scales, const float* P,
                              const int8_t* signs, const float* codebook, const void* q, float score_scale,
                              float* scores, void* Khat_out, int64_t row0, int64_t rows, int seq_len, int H,
                              int q_heads, const float* rope_cos, const float* rope_sin, bool wide, hipStream_t stream);

// Fused bf16 forms: prediction [x0 | x1] W^T + bias on the matrix cores, consumed in the same
// kernel by the quantizer (encode), its inverse (decode) or its inverse plus q.k (scores).
// wide (decode, scores, weighted; D = 1024): rotation groups of 1024 = the whole token, one scale per token.
hipError_t launch_fused_encode(int n_codewords, const void* x0, int d0, const void* x1, int d1, const void* W,
                               const float* bias, const int8_t* signs, const float* codebook, const void* table,
                               const void* X, uint8_t* codes, uint16_t* scales, void* Xhat, int64_t T, int D,
                               hipStream_t stream);
// The same for rotation groups of 1024 (8 heads): a workgroup owns 64 tokens x all heads.  `w_retiled`: device scratch of
// 1024 * (d0 + d1) * 2 bytes, 16-byte aligned, that the call fills with the weights in the order its main loop reads them.
hipError_t launch_fused_encode_wide(int n_codewords, const void* x0, int d0, const void* x1, int d1, const void* W,
                                    void* w_retiled, const float* bias, const int8_t* signs, const float* codebook,
                                    const void* table, const void* X, uint8_t* codes, uint16_t* scales, void* Xhat,
                                    int64_t T, int D, hipStream_t stream);
hipError_t launch_fused_decode(int n_codewords, const void* x0, int d0, const void* x1, int d1, const void* W,
                               const float* bias, const int8_t* signs, const float* codebook, const uint8_t* codes,
                               const uint16_t* scales, void* Xhat, int64_t T, int D, bool wide, hipStream_t stream);
hipError_t launch_fused_scores(int n_codewords, const void* x0, int d0, const void* W, const float* bias,
                               const int8_t* signs, const float* codebook, const uint8_t* codes,
                               const uint16_t* scales, const void* q, float score_scale, float* scores, void* Khat_out,
                               int seq_len, int q_heads, int64_t T, int D, const float* rope_cos, const float* rope_sin,
                               bool wide, hipStream_t stream);

// The same on tiles of 256 tokens x two heads (D a multiple of 256; wide: decode only): same bits, a faster main
// loop, half as many workgroups.  launch_fused_decode / launch_fused_scores take this form by themselves when
// two_heads_pays(T, D): when the larger tile costs no extra round over the CUs.
bool two_heads_pays(int64_t T, int D);
hipError_t launch_fused_encode_two_heads(int n_codewords, const void* x0, int d0, const void* x1, int d1, const void* W,
                                         const float* bias, const int8_t* signs, const float* codebook, const void* table,
                                         const void* X, uint8_t* codes, uint16_t* scales, void* Xhat, int64_t T, int D,
                                         hipStream_t stream);
hipError_t launch_fused_decode_two_heads(int n_codewords, const void* x0, int d0, const void* x1, int d1, const void* W,
                                         const float* bias, const int8_t* signs, const float* codebook,
                                         const uint8_t* codes, const uint16_t* scales, void* Xhat, int64_t T, int D,
                                         bool wide, hipStream_t stream);
hipError_t launch_fused_scores_two_heads(int n_codewords, const void* x0, int d0, const void* W, const float* bias,
                                         const int8_t* signs, const float* codebook, const uint8_t* codes,
                                         const uint16_t* scales, const void* q, float score_scale, float* scores,
                                         void* Khat_out, int seq_len, int q_heads, int64_t T, int D,
                                         const float* rope_cos, const float* rope_sin, hipStream_t stream);

// Value side of attention.  The sums over tokens are taken per chunk of kWeightedChunk tokens of one sequence
// (part[batch * chunks_per_seq, q_heads, 128] fp32, chunks_per_seq = ceil(seq_len / kWeightedChunk)) and then added in
// chunk order by launch_combine_weighted: out[b, qh, :] = sum_t weights[b, qh, t] * Vhat[b * seq_len + t, qh / rep, :].
// Soft-max form (pstats given, [batch * chunks_per_seq, q_heads, 2] fp32): `weights` holds raw scores, a chunk's sums are
// taken with exp(score - chunk maximum), pstats receives that maximum and the chunk's weight sum, and the combine step
// rescales the chunks to the row maximum and divides by the row's weight sum (row_stats, nullable, [batch, q_heads, 2]:
// row maximum and that denominator).
constexpr int kWeightedChunk = 256;
// decode of the values with the chunk sums taken in the epilogue (bf16, seq_len a multiple of kWeightedChunk); Xhat nullable
hipError_t launch_fused_weighted(int n_codewords, const void* x0, int d0, const void* x1, int d1, const void* W,
                                 const float* bias, const int8_t* signs, const float* codebook, const uint8_t* codes,
                                 const uint16_t* scales, void* Xhat, const float* weights, float* part, float* pstats,
                                 int seq_len, int q_heads, int64_t T, int D, bool wide, hipStream_t stream);
// chunk sums over values already decoded to memory (any dtype, any seq_len)
hipError_t launch_weighted_values(int dtype, const void* Vhat, const float* weights, float* part, float* pstats, int batch,
                                  int seq_len, int H, int q_heads, hipStream_t stream);
hipError_t launch_combine_weighted(const float* part, const float* pstats, float* out, float* row_stats, int batch,
                                   int seq_len, int q_heads, hipStream_t stream);
// Attention of one query per sequence over `tokens` (<= kAttendRawMaxTokens) keys / values in the storage dtype
// ([batch * tokens, H, 128]), written to or merged into (accumulate != 0) out [batch, q_heads, 128] and the row
// statistics [batch, q_heads, 2] (maximum, sum of exp(score - maximum)) that launch_combine_weighted hands out.
constexpr int kAttendRawMaxTokens = 4096;
// rope_cos / rope_sin (nullable, fp32 [tokens, 64]): rotate key t by its position before the dot product.
hipError_t launch_attend_raw(int dtype, const void* K, const void* V, const void* q, const float* rope_cos,
                             const float* rope_sin, float scale, float* out, float* stats, int batch, int tokens, int H,
                             int q_heads, int accumulate, hipStream_t stream);
// probs[r, :] = softmax(scores[r, :]) for `rows` rows of length n (in place allowed)
hipError_t launch_softmax_rows(const float* scores, float* probs, int64_t rows, int64_t n, hipStream_t stream);

// Scores with the key predictor folded into the query (bf16, 8 kv heads, 1024 predictor inputs,
// q_heads <= 64): reads Khat_prev and the codes once per 4 query heads of a kv head (one pass up to 32 query
// heads, two up to 64).  `workspace`: folded_scores_workspace_bytes(batch, q_heads).
// bytes of folded query operands per batch entry and pass: u as bf16 high / low MFMA operands (8 waves x 2 x 8 k
// steps x 1 KiB), the rotated queries [32][128] fp32, q . b [32] fp32
constexpr size_t kFoldedBytesPerBatch = (size_t)8 * 2 * 8 * 1024 + 32 * 128 * 4 + 32 * 4;
bool folded_scores_supported(int kv_heads, int d_in_k, int q_heads);
size_t folded_scores_workspace_bytes(int batch, int q_heads);
hipError_t launch_folded_scores(int n_codewords, const void* Khat_prev, const void* W, const float* bias,
                                const int8_t* signs, const float* codebook, const uint8_t* codes,
                                const uint16_t* scales, const void* q, float score_scale, float* scores, void* workspace,
                                int batch, int seq_len, int q_heads, hipStream_t stream);

// Ridge least-squares fit of a predictor, W [d_out, d0 + d1] = argmin || [x0 | x1] W^T - Y ||^2 + lambda ||W||^2 with
// lambda = rate * trace(X^T X) / d_in, in fp64 through the normal equations.  d0, d1, d_out multiples of 64.
// `workspace`: fit_workspace_bytes(d0 + d1, d_out).  W64 (nullable): the unrounded solution [d_out, d_in].
// bias (nullable, fp32 [d_out]): fit an intercept as well (centred regression).
size_t fit_workspace_bytes(int d_in, int d_out);
hipError_t launch_fit_predictor(int dtype, int64_t tokens, const void* x0, int d0, const void* x1, int d1, const void* Y,
                                int d_out, double rate, void* W, double* W64, float* bias, void* workspace,
                                hipStream_t stream);

}  // namespace aquakv
