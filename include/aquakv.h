/*
 * aquakv.h -- C ABI of the MI355X (gfx950) AQUA-KV per-layer KV-cache codec.
 *
 * The library implements the per-layer `encode` and `decode` procedures of the
 * AQUA-KV paper (arxiv 2501.19392; Appendix, Alg. "encode" and Alg. "decode")
 * on top of the HIGGS-style backbone quantizer of Sect. 2 "Vector Quantization"
 * (randomized Hadamard transform, group scale, nearest point of an n-point grid
 * in R^2; Sect. 4.1: n = 16 / 64 / 256 for 2 / 3 / 4 bits per value) and the
 * linear predictors of Sect. 3.2.
 *
 * General conventions
 *   - Every pointer below is a DEVICE pointer owned by the caller unless the
 *     comment says "host".  The library allocates nothing, keeps no state
 *     between calls and never synchronises the device: all work is enqueued on
 *     `stream` (a hipStream_t passed as void*; NULL = the default stream) and the
 *     outputs are valid once the stream reaches that point.
 *   - Every device pointer must be 16-byte aligned (AQUAKV_EALIGN otherwise), except the scale
 *     arrays, which need 2 bytes (with one scale per token a row range starts at any even address).
 *   - Return value: AQUAKV_OK (0) or a negative aquakv_status.  On a validation
 *     error nothing is launched.  aquakv_last_error() returns a thread-local
 *     text for the most recent failure on the calling thread.
 *   - Results for a token row never depend on how many other rows are in the
 *     call (the predictor's summation order is fixed), so `decode` reproduces
 *     bit-for-bit the reconstructions `encode` returned.
 *
 * Shapes and layouts (T = tokens, H = kv_heads, g = head_dim = 128 = one
 * rotation/scale group, D = H*g, n = n_codewords, c = log2(n) code bits):
 *   K, V, Khat, Vhat, *_prev : [T, H, g] row-major, element type = layer.dtype
 *   codes                    : uint8 [T, H, g*c/16]; per group a little-endian
 *                              bit string, code i (sub-vector of rotated
 *                              coordinates 2i, 2i+1) at bits [i*c, (i+1)*c)
 *   scales                   : IEEE fp16 bit patterns, uint16 [T, H]
 *   predictions P            : fp32 [T, D]
 *
 * Second backbone (Sect. 4.1 "Backbone quantization": uniform round-to-nearest, groups of 64
 * channels of a token, 2.50 stored bits per value at 2 bits in Table 1), selected by vq_dim = 1
 * with n_codewords = 4 or 16 levels (b = 2 or 4 bits per value); no grid, no rotation:
 *   per group of 64 consecutive channels of x - p: lo = min(0, min), hi = max(0, max),
 *   step = (hi - lo) / (n - 1) stored as fp16, zero = round(-lo / step),
 *   code = clamp(round((x - p) / step) + zero, 0, n - 1), rounding half to even;
 *   reconstruction p + (code - zero) * step.
 *   codes  : uint8 [T, D*b/8], b bits per value in channel order, little-endian
 *   scales : uint16 [T, D/64, 2] = (fp16 bits of the step, zero point) per group; 4-byte aligned
 * Every entry point below takes such a layer; where a comment says "scales [T, H]" read the
 * layout above instead.  In the folded form of the scoring call the code term is
 * step * sum_i q_i (code_i - zero) per group (no rotation).
 */
#ifndef AQUAKV_H
#define AQUAKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define AQUAKV_VERSION 100 /* major*10000 + minor*100 + patch */

typedef enum {
  AQUAKV_OK = 0,
  AQUAKV_EINVAL = -1,       /* a size or enum is out of range / inconsistent    */
  AQUAKV_ENULL = -2,        /* a required pointer is NULL                       */
  AQUAKV_EALIGN = -3,       /* a pointer is not 16-byte aligned                 */
  AQUAKV_EUNSUPPORTED = -4, /* valid in principle, not built (e.g. head_dim 64) */
  AQUAKV_EWORKSPACE = -5,   /* workspace smaller than aquakv_workspace_bytes()  */
  AQUAKV_EHIP = -6          /* a HIP launch failed; see aquakv_last_error()     */
} aquakv_status;

typedef enum { AQUAKV_BF16 = 0, AQUAKV_FP32 = 1 } aquakv_dtype;
typedef enum { AQUAKV_KEY = 0, AQUAKV_VALUE = 1 } aquakv_which;

/*
 * One layer's fixed parameters: the REQUIRE lines of Alg. "encode"/"decode"
 * (predictors) plus what the quantizer of Sect. 2 needs (grid, sign vectors).
 * The struct itself lives in HOST memory; the pointers in it are device pointers.
 */
typedef struct aquakv_layer {
  int32_t kv_heads;     /* H >= 1                                                */
  int32_t head_dim;     /* g; only 128 is built                                   */
  int32_t vq_dim;       /* p = 2: grid in R^2 behind the rotation (Sect. 4.1: d = 2);
                           1: uniform round-to-nearest backbone (see above)       */
  int32_t n_codewords;  /* p = 2: n in {16, 64, 256} = 2, 3, 4 code bits per value;
                           p = 1: 4 or 16 levels                                  */
  int32_t dtype;        /* aquakv_dtype of K, V, reconstructions and weights      */
  int32_t d_in_k;       /* inputs of f_key (= width of Khat_prev); 0 = no key
                           predictor (layer 0: prediction is zero)                */
  int32_t d_in_v;       /* inputs of f_value = width of Vhat_prev + D; 0 = none   */
  int32_t rht_group;    /* values per rotation group and scale: 0 or head_dim = one
                           group per (token, kv head), scales [tokens, kv_heads];
                           kv_heads * head_dim = the whole token vector is one group
                           with one scale, scales [tokens] (the grouping of the paper's
                           experiments, Sect. 4.1: 1024 values, 2.02 stored bits per
                           value; built for 8 heads of 128).  The code bytes have the
                           same layout either way.  In bf16 both groupings run the
                           predictor fused with the quantizer; for groups across
                           heads the encoder reads the predictor weights from a
                           re-tiled copy it writes into the workspace first
                           (kv_heads * head_dim * max(d_in_k, d_in_v) elements at
                           the front of the workspace).  With vq_dim = 1: 0 or
                           64, the group of the round-to-nearest backbone, or 1024 =
                           the whole token of 8 heads (one (step, zero) per token).  */
  const float* codebook;   /* [n, 2] fp32 grid points (ignored when vq_dim = 1, like
                              signs_k, signs_v and search_table)                  */
  const int8_t* signs_k;   /* [H*g] entries +1 / -1: RHT signs for keys           */
  const int8_t* signs_v;   /* [H*g] same for values                               */
  const void* w_k;      /* [D, d_in_k] row-major, dtype: K_pred = Khat_prev w_k^T.  A departure
                           from the order of the REQUIRE lines of Alg. "encode", which read as
                           K_pred = Khat_prev W with W [d_in, D]: the weights are stored
                           transposed, input index contiguous, which is how both operands of
                           the matrix instructions want them                              */
  const float* b_k;     /* [D] fp32 bias or NULL                                  */
  const void* w_v;      /* [D, d_in_v] row-major; input columns: Vhat_prev first,
                           then this layer's Khat (Alg. "encode": [Vhat_prev; Khat]) */
  const float* b_v;     /* [D] fp32 bias or NULL                                  */
  const void* search_table; /* NULL, or the table aquakv_build_search_table made from
                           `codebook`: same codes, found without scoring all n points */
} aquakv_layer;

int aquakv_version(void);
const char* aquakv_status_string(int status);
const char* aquakv_last_error(void);

/*
 * Optional accelerator for the nearest-grid-point step of Sect. 2 (the paper calls the
 * encoding cost of vector quantization its practical obstacle).  The table partitions the
 * plane into cells and lists, per cell, every grid point that can be nearest somewhere in
 * it; quantize then scores only those (cells with more candidates than fit an entry name
 * an overflow list kept behind the cell entries, and beyond 8 candidates fall back to the
 * full search).  The result is identical to the full search.
 * `table` is device memory of aquakv_search_table_bytes(n) bytes, written on `stream`;
 * build it once per grid and put it into aquakv_layer.search_table.
 */
size_t aquakv_search_table_bytes(int32_t n_codewords);   /* 0 if n is not supported */
int aquakv_build_search_table(const float* codebook, int32_t vq_dim, int32_t n_codewords,
                              void* table, void* stream);

/* Bytes of device workspace the three layer-level calls below need for `tokens`
 * rows (0 on invalid arguments).  Its front part holds the fp32 predictions of one
 * chunk of rows (fp32 layers) or the re-tiled predictor weights (bf16 layers with
 * rotation groups across the heads; nothing for the other bf16 layers); behind it
 * a temporary Khat for one chunk of rows when the caller does not ask for one. */
size_t aquakv_workspace_bytes(const aquakv_layer* layer, int64_t tokens);

/* Which tile the fused bf16 kernels (predictor of Sect. 3.2 with the quantizer or its inverse inside: aquakv_encode_layer,
 * aquakv_encode_keys / _values, aquakv_decode_layer, aquakv_decode_values, aquakv_decode_attn_scores and its rotary
 * form) take for a call over `tokens` rows: 2 = 256 tokens x two kv heads per workgroup, 1 = 256 tokens x one head (for
 * layers with rotation groups across the heads: the tile of aquakv_decode_layer / _values; their encoder works on 64
 * tokens x all heads, their scoring call on one head),
 * 0 = the layer does not go through them (fp32, no predictor) or the arguments are invalid.  The large tile has the
 * faster main loop and is taken when it costs no extra round of workgroups over the compute units; the value sums of
 * aquakv_decode_values_weighted / _attend stay on the small tile.  For information (benchmarks label their kernels by
 * it): the results are the same bits either way.  Host only, no GPU work. */
int aquakv_fused_tile_heads(const aquakv_layer* layer, int64_t tokens);

/*
 * Stage entry points (also what the layer-level calls are made of).
 *
 * aquakv_predict -- Sect. 3.2: P = [x0 | x1] W^T + b in fp32 (bf16 inputs:
 *   bf16 MFMA with fp32 accumulation; fp32 inputs: fp32 FMA).
 *   which = AQUAKV_KEY  : x0 = Khat_prev [T, d_in_k], x1 ignored (may be NULL)
 *   which = AQUAKV_VALUE: x0 = Vhat_prev [T, d_in_v - D], x1 = Khat [T, D]
 *   P: fp32 [T, D] out.  AQUAKV_EINVAL if the layer has no such predictor.
 *
 * aquakv_quantize -- Sect. 2: Q(X - P).  z = H_g(s*(x-p))/sqrt(g) per group,
 *   sigma = rms(z) stored as fp16, nearest grid point of z/sigma16 per pair,
 *   lowest index on ties.  P (fp32 [T, D]) may be NULL = zero prediction.
 *   Xhat (nullable, dtype) receives round(P + Q^-1(codes)) exactly as
 *   aquakv_dequantize would produce it.  Xhat may alias X; nothing else may alias.
 *
 * aquakv_dequantize -- Sect. 2 / Alg. "decode": Xhat = round(P + s*H_g(C[code]*sigma16)/sqrt(g)).
 */
int aquakv_predict(const aquakv_layer* layer, int which, int64_t tokens,
                   const void* x0, const void* x1, float* P, void* stream);
int aquakv_quantize(const aquakv_layer* layer, int which, int64_t tokens,
                    const void* X, const float* P,
                    uint8_t* codes, uint16_t* scales, void* Xhat, void* stream);
int aquakv_dequantize(const aquakv_layer* layer, int which, int64_t tokens,
                      const uint8_t* codes, const uint16_t* scales, const float* P,
                      void* Xhat, void* stream);

/*
 * aquakv_encode_layer -- Alg. "encode" for one layer and `tokens` rows:
 *   K_pred = f_key(Khat_prev); K_q = Q(K - K_pred); Khat = Q^-1(K_q) + K_pred;
 *   V_pred = f_value([Vhat_prev; Khat]); V_q = Q(V - V_pred); Vhat likewise.
 * Khat_prev / Vhat_prev: required iff the layer has the respective predictor.
 * Khat, Vhat: outputs (nullable).  They are what Alg. "Inference" feeds to the
 * next layer; the stored (rounded) Khat is also what f_value reads.
 * Khat may coincide with K and Vhat with V (reconstruction in place: the same address); any other
 * overlap between an output (or the workspace) and an input or another output is refused with
 * AQUAKV_EINVAL before anything is launched (the same holds for the decode call and the halves below).
 * tokens == 0 is a no-op.
 */
int aquakv_encode_layer(const aquakv_layer* layer, int64_t tokens,
                        const void* K, const void* V,
                        const void* Khat_prev, const void* Vhat_prev,
                        uint8_t* k_codes, uint16_t* k_scales,
                        uint8_t* v_codes, uint16_t* v_scales,
                        void* Khat, void* Vhat,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * aquakv_decode_layer -- Alg. "decode":
 *   Khat = Q^-1(K_q) + f_key(Khat_prev); Vhat = Q^-1(V_q) + f_value([Vhat_prev; Khat]).
 * Khat is required when the layer has a value predictor and Vhat is requested;
 * Vhat may be NULL (keys only; v_codes / v_scales are then ignored).
 */
int aquakv_decode_layer(const aquakv_layer* layer, int64_t tokens,
                        const uint8_t* k_codes, const uint16_t* k_scales,
                        const uint8_t* v_codes, const uint16_t* v_scales,
                        const void* Khat_prev, const void* Vhat_prev,
                        void* Khat, void* Vhat,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * The two halves of Alg. "encode" / "decode" as calls of their own (same kernels, same bits as the
 * layer-level calls).  Over a stack of layers the key chain depends on keys only
 * (Khat of layer l from Khat of layer l-1), the value chain on the previous layer's values and this
 * layer's keys, so a caller may put the two chains on two streams, with an event from each key call
 * to the value call of the same layer, and let the kernels of neighbouring layers overlap.
 *   aquakv_encode_keys   : K_q = Q(K - f_key(Khat_prev)); Khat (nullable) = reconstruction.
 *   aquakv_encode_values : V_q = Q(V - f_value([Vhat_prev; Khat])); Khat is an INPUT here (required iff
 *                          the layer has a value predictor); Vhat (nullable) = reconstruction.
 *   aquakv_decode_values : Vhat = Q^-1(V_q) + f_value([Vhat_prev; Khat]); Khat is an INPUT.
 *   (keys only of Alg. "decode": aquakv_decode_layer with Vhat = NULL.)
 * Workspace: the front part of aquakv_workspace_bytes() suffices (none for bf16 layers with groups of one head).  Two
 * calls that run at the same time (two streams) need a workspace each.
 */
int aquakv_encode_keys(const aquakv_layer* layer, int64_t tokens, const void* K, const void* Khat_prev,
                       uint8_t* k_codes, uint16_t* k_scales, void* Khat,
                       void* workspace, size_t workspace_bytes, void* stream);
int aquakv_encode_values(const aquakv_layer* layer, int64_t tokens, const void* V, const void* Vhat_prev,
                         const void* Khat, uint8_t* v_codes, uint16_t* v_scales, void* Vhat,
                         void* workspace, size_t workspace_bytes, void* stream);
int aquakv_decode_values(const aquakv_layer* layer, int64_t tokens, const uint8_t* v_codes, const uint16_t* v_scales,
                         const void* Vhat_prev, const void* Khat, void* Vhat,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * aquakv_decode_attn_scores -- decode of the keys (Alg. "decode", first line)
 * fused with grouped-query q.k scoring, so the keys need not be written:
 *   scores[b, qh, t] = score_scale * sum_d q[b, qh, d] * Khat[b*seq_len + t, qh / (q_heads/H), d]
 * q: [batch, q_heads, g] (dtype); scores: fp32 [batch, q_heads, seq_len];
 * codes / scales / Khat_prev cover batch*seq_len rows; no rotary embedding.
 * Khat_out (nullable, dtype, [batch*seq_len, H, g]) also receives the keys.
 * q_heads must be a multiple of H with q_heads / H <= 8.
 *
 * Always the definition above (the storage-rounded key is scored); `workspace`: the fp32 prediction part of
 * aquakv_workspace_bytes() for layers that do not run fused (fp32), unused otherwise.
 *
 * aquakv_decode_attn_scores_folded -- the same scores in the folded form, a call of its own so that the
 * arithmetic a caller gets never depends on the size of a workspace.  A score is linear in the key, so with
 * a key predictor (Sect. 3.2)
 *   q . Khat[t] = Khat_prev[t] . (W_h^T q) + q . b_h + sigma[t] * (R q) . C[codes[t]],
 * R q the rotated query: one 1024-long dot product per token and query head instead of the
 * predictor product, bound by reading Khat_prev and the codes once.  The keys are never formed, so there
 * is no Khat_out, and the scores are those of the UNROUNDED keys: they agree with the definition to the
 * storage precision of Khat (2^-9 relative per term in bf16).  Built for bf16 layers with 8 kv heads, a key
 * predictor with 1024 inputs, rotation groups of one head and q_heads <= 64 (one pass over the cache per 4
 * query heads of a kv head, so two passes above 32 query heads); AQUAKV_EUNSUPPORTED otherwise, and
 * aquakv_scores_workspace_bytes() is then 0.  `workspace`: at least aquakv_scores_workspace_bytes() bytes
 * (the folded queries of this call; AQUAKV_EWORKSPACE if smaller).
 */
size_t aquakv_scores_workspace_bytes(const aquakv_layer* layer, int32_t batch, int32_t q_heads);
int aquakv_decode_attn_scores(const aquakv_layer* layer, int32_t batch, int32_t seq_len, int32_t q_heads,
                              const uint8_t* k_codes, const uint16_t* k_scales,
                              const void* Khat_prev, const void* q, float score_scale,
                              float* scores, void* Khat_out,
                              void* workspace, size_t workspace_bytes, void* stream);
int aquakv_decode_attn_scores_folded(const aquakv_layer* layer, int32_t batch, int32_t seq_len, int32_t q_heads,
                                     const uint8_t* k_codes, const uint16_t* k_scales,
                                     const void* Khat_prev, const void* q, float score_scale,
                                     float* scores, void* workspace, size_t workspace_bytes, void* stream);

/*
 * aquakv_decode_attn_scores_folded_static -- aquakv_decode_attn_scores_folded for callers that cannot
 * allocate device memory and so have no workspace to pass (code under HIP graph capture, tight serving
 * loops, harnesses that forbid allocation).  Same arguments without the workspace, same kernels, same
 * bits.  The folded queries live in a buffer built into the library (about 9 MiB of device memory per
 * GPU the library runs on, held until the process ends), so the call allocates nothing; it serves
 * batch x passes <= 64 (passes = 1 up to 32 query heads, 2 above) and returns AQUAKV_EUNSUPPORTED with
 * a text beyond that.  Every call on a GPU uses that GPU's one buffer: calls on the same GPU must not
 * overlap in time (different streams without an ordering between them, or several host threads) or
 * they race on it; calls on one stream are ordered and safe.  Nothing in the buffer needs clearing
 * between calls: each call writes every byte it later reads.
 */
int aquakv_decode_attn_scores_folded_static(const aquakv_layer* layer, int32_t batch, int32_t seq_len, int32_t q_heads,
                                            const uint8_t* k_codes, const uint16_t* k_scales,
                                            const void* Khat_prev, const void* q, float score_scale,
                                            float* scores, void* stream);

/*
 * aquakv_decode_attn_scores_rope -- the same call for caches that hold the keys from BEFORE the
 * rotary positional embedding (Sect. 3.3 "Positional embeddings": predictors and quantizer work
 * best there).  The decoded (storage-rounded) key of token t of every sequence is rotated by
 * position t before the dot product: coordinate d is paired with d + g/2,
 *   k'_d = k_d cos[t, d] - k_{d+g/2} sin[t, d],   k'_{d+g/2} = k_{d+g/2} cos[t, d] + k_d sin[t, d],
 * rope_cos / rope_sin: device, fp32 [seq_len, g/2], 16-byte aligned, owned by the caller (any
 * frequency base or scaling).  q must already be rotated for its own position.  Khat_out
 * (nullable) receives the UNROTATED keys, which is what the next layer's predictor reads.
 * Always recomputes the prediction (the folded form does not commute with a per-token rotation).
 */
int aquakv_decode_attn_scores_rope(const aquakv_layer* layer, int32_t batch, int32_t seq_len, int32_t q_heads,
                                   const uint8_t* k_codes, const uint16_t* k_scales,
                                   const void* Khat_prev, const void* q,
                                   const float* rope_cos, const float* rope_sin, float score_scale,
                                   float* scores, void* Khat_out,
                                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * Value side of attention over the compressed cache (Alg. "Inference": the block call attends over the
 * recovered keys and values, its output is the weighted sum of the values; Sect. 5 of the paper names the integration of the cache with
 * attention as the step its own implementation leaves open).
 *
 * aquakv_softmax -- probs[r, :] = exp(s - max s) / sum exp(s - max s) over each of `rows` rows of
 *   n fp32 values (device memory; probs may be scores: in place).  rows = batch * q_heads and
 *   n = seq_len turns the scores of aquakv_decode_attn_scores into attention weights.
 *
 * aquakv_decode_values_weighted -- decode of the values (Alg. "decode", second line) together with
 *   out[b, qh, :] = sum_t weights[b, qh, t] * Vhat[b*seq_len + t, qh / (q_heads/H), :],
 *   Vhat being the storage-rounded reconstruction (what aquakv_decode_values writes).
 *   weights: device, fp32 [batch, q_heads, seq_len], any real numbers (soft-max rows in the plain case;
 *   a caller that also attends to tokens outside the compressed cache normalises over all of them
 *   and adds their share itself).  out: device, fp32 [batch, q_heads, g].  Vhat (dtype,
 *   [batch*seq_len, H, g]) receives the decoded values, which the next layer's predictor reads.
 *   For bf16 layers with a value predictor and seq_len a multiple of 256
 *   the sums are taken inside the decode kernel from the values it holds
 *   on chip (weights enter as bf16 pairs hi + lo, i.e. with 16 mantissa bits; products accumulate in
 *   fp32), and Vhat may then be NULL: nothing but `out` is written (the last layer of a sweep).
 *   Otherwise Vhat is required, the values are decoded to it first and summed from there in fp32.
 *   q_heads must be a multiple of H with q_heads / H <= 8.  `workspace`: at least
 *   aquakv_weighted_workspace_bytes() bytes, holding the per-256-token partial sums (added in a fixed
 *   order: the result does not depend on scheduling), their soft-max statistics and, for layers that
 *   are not fused, the fp32 prediction.  Errors as for aquakv_decode_values.
 *
 * aquakv_decode_values_attend -- the same call with the soft-max inside: `scores` (device, fp32
 *   [batch, q_heads, seq_len], finite; what aquakv_decode_attn_scores wrote) takes the place of the weights and
 *   out[b, qh, :] = sum_t softmax(scores[b, qh, :])[t] * Vhat[...].  Every 256 tokens are summed with weights
 *   exp(score - their own maximum); the pieces are then rescaled to the row maximum M and divided by
 *   L = sum_t exp(score - M) (the scheme of split-sequence attention kernels), so no separate soft-max pass
 *   runs.  row_stats (nullable; device, fp32 [batch, q_heads, 2]) receives (M, L): a caller that also attends
 *   to tokens outside the compressed cache merges its own (max, sum, weighted values) with (M, L, out).
 *   Same conditions for the sums inside the decode kernel, same workspace.
 *
 * aquakv_attend_raw -- attention of the same queries over tokens that are held in 16 bits (Sect. 3.3: the attention
 *   sinks and the recent-token buffer are not quantized): K, V device, dtype, [batch*tokens, kv_heads, 128] (tokens <=
 *   4096); q [batch, q_heads, 128] (dtype).  rope_cos / rope_sin (both NULL, or device fp32 [tokens, 64], the angles
 *   of this call's tokens, 16-byte aligned): the keys are held from before the rotary embedding and token t of every
 *   sequence is rotated by row t of the tables before the dot product, as in aquakv_decode_attn_scores_rope (a caller
 *   whose tokens start at position p passes the tables offset by p rows).  accumulate = 0 writes out = softmax(score_scale * q.K^T) V and
 *   row_stats = (maximum, sum of exp(score - maximum)); accumulate != 0 merges that with the result (out, row_stats)
 *   already there -- from aquakv_decode_values_attend or an earlier aquakv_attend_raw call on the same queries --
 *   into the attention over the union of the token sets.  tokens = 0 with accumulate != 0 is a no-op;
 *   more than 4096 tokens per call is AQUAKV_EUNSUPPORTED (call again with accumulate != 0 for the rest).
 *
 * All buffers are the caller's and stay so; outputs (Vhat, out, row_stats, probs other than in place) may not
 * alias inputs or the workspace.  Calls on one stream run in order; a call reads `scores` / `weights` while it
 * runs, so they must not be overwritten by work on another stream before it has finished.
 */
int aquakv_softmax(int64_t rows, int64_t n, const float* scores, float* probs, void* stream);
int aquakv_attend_raw(int32_t dtype, int32_t batch, int32_t tokens, int32_t kv_heads, int32_t q_heads,
                      const void* K, const void* V, const void* q,
                      const float* rope_cos, const float* rope_sin, float score_scale,
                      float* out, float* row_stats, int32_t accumulate, void* stream);
size_t aquakv_weighted_workspace_bytes(const aquakv_layer* layer, int32_t batch, int32_t seq_len, int32_t q_heads);
int aquakv_decode_values_weighted(const aquakv_layer* layer, int32_t batch, int32_t seq_len, int32_t q_heads,
                                  const uint8_t* v_codes, const uint16_t* v_scales,
                                  const void* Vhat_prev, const void* Khat, const float* weights,
                                  void* Vhat, float* out,
                                  void* workspace, size_t workspace_bytes, void* stream);
int aquakv_decode_values_attend(const aquakv_layer* layer, int32_t batch, int32_t seq_len, int32_t q_heads,
                                const uint8_t* v_codes, const uint16_t* v_scales,
                                const void* Vhat_prev, const void* Khat, const float* scores,
                                void* Vhat, float* out, float* row_stats,
                                void* workspace, size_t workspace_bytes, void* stream);

/*
 * aquakv_fit_predictor -- calibration of one predictor (Alg. "Calibration", Sect. 3.2): the linear map that best
 * predicts Y from X = [x0 | x1] in the least-squares sense,
 *     W = argmin || X W^T - Y ||^2 + lambda ||W||^2,   lambda = rate * trace(X^T X) / d_in   (rate = 0: plain
 *     least squares, X must then have full column rank),
 * solved in fp64 through the normal equations (Gram products, Cholesky, two triangular solves) and rounded once to
 * `dtype`.  x0 [tokens, d0], x1 [tokens, d1] (NULL iff d1 = 0), Y [tokens, d_out], all `dtype`, row-major;
 * d0, d1, d_out multiples of 64, at most 8192 inputs / outputs.  W [d_out, d0 + d1] out: the layout of
 * aquakv_layer.w_k / w_v (key predictor: x0 = Khat_prev, Y = K; value predictor: x0 = Vhat_prev, x1 = Khat, Y = V).
 * W64 (nullable) receives the unrounded fp64 solution in the same layout.  bias (nullable, fp32 [d_out], the layout
 * of aquakv_layer.b_k / b_v): if given, an intercept is fitted as well, X W^T + b: the regression of the centred Y
 * on the centred X (lambda acts on W only, with the trace of the centred X^T X), b = mean(Y) - W mean(X).  If the
 * matrix X^T X + lambda I is not positive definite in fp64, W (and W64, bias) are filled with NaN.  `workspace`: aquakv_fit_workspace_bytes(d0 + d1, d_out)
 * bytes (0 for unsupported sizes).  The layer-by-layer procedure of the algorithm (fit the key predictor, encode
 * the keys with it, fit the value predictor on [Vhat_prev | Khat], encode, move on) is made of this call and
 * aquakv_encode_keys / aquakv_encode_values.
 */
size_t aquakv_fit_workspace_bytes(int32_t d_in, int32_t d_out);
int aquakv_fit_predictor(int32_t dtype, int64_t tokens, const void* x0, int32_t d0, const void* x1, int32_t d1,
                         const void* Y, int32_t d_out, double rate, void* W, double* W64, float* bias,
                         void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* AQUAKV_H */
