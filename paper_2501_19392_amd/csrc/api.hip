// C-ABI layer: argument validation, workspace layout, chunking and dispatch.
// No HIP call is made before validation has passed.
#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <mutex>

#include "../../include/aquakv.h"
#include "kernels.h"

namespace {

thread_local char g_err[512] = "";

int fail(int status, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return status;
}

// Rows handled per pass of the layer-level calls.  bf16 layers run the fused kernels, which
// need no prediction buffer (the chunk only bounds the temporary Khat).  fp32 layers run
// predictor and quantizer as separate kernels: the fp32 predictions of one chunk
// (chunk * D * 4 bytes) then stay close to the caches between the two.
constexpr int64_t kChunkRowsFused = 65536;
constexpr int64_t kChunkRowsSplit = 16384;

inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }
inline size_t elem_bytes(int dtype) { return dtype == AQUAKV_BF16 ? 2 : 4; }
// Sect. 4.1 "Backbone quantization": vq_dim 2 = grid in R^2 behind a Hadamard rotation, vq_dim 1 = uniform
// round-to-nearest on groups of 64 channels
inline bool is_rtn(const aquakv_layer* L) { return L->vq_dim == 1; }
constexpr int kRtnGroup = 64;
// what the kernels are instantiated on: the grid size, or the bits per value of the round-to-nearest backbone
inline int quantizer_id(const aquakv_layer* L) { return is_rtn(L) ? (L->n_codewords == 4 ? 2 : 4) : L->n_codewords; }
// code bits per pair of values
inline int code_bits(const aquakv_layer* L) {
  if (is_rtn(L)) return L->n_codewords == 4 ? 4 : 8;
  return L->n_codewords == 16 ? 4 : L->n_codewords == 64 ? 6 : 8;
}

int check_layer(const aquakv_layer* L) {
  if (L == nullptr) return fail(AQUAKV_ENULL, "layer is NULL");
  if (L->kv_heads < 1 || L->kv_heads > 4096) return fail(AQUAKV_EINVAL, "kv_heads=%d out of range", L->kv_heads);
  if (L->head_dim < 1 || (L->head_dim & (L->head_dim - 1)))
    return fail(AQUAKV_EINVAL, "head_dim=%d is not a power of two", L->head_dim);
  if (L->head_dim != 128) return fail(AQUAKV_EUNSUPPORTED, "head_dim=%d: only 128 is built", L->head_dim);
  if (L->vq_dim < 1) return fail(AQUAKV_EINVAL, "vq_dim=%d", L->vq_dim);
  if (L->vq_dim > 2) return fail(AQUAKV_EUNSUPPORTED, "vq_dim=%d: only 1 and 2 are built", L->vq_dim);
  const bool pow2 = L->n_codewords >= 2 && !(L->n_codewords & (L->n_codewords - 1));
  if (is_rtn(L)) {
    if (L->n_codewords != 4 && L->n_codewords != 16)
      return fail(pow2 ? AQUAKV_EUNSUPPORTED : AQUAKV_EINVAL, "n_codewords=%d: vq_dim 1 is built for 4 or 16 levels", L->n_codewords);
    if (L->rht_group != 0 && L->rht_group != kRtnGroup && !(L->rht_group == 1024 && L->kv_heads * L->head_dim == 1024))
      return fail(AQUAKV_EUNSUPPORTED, "rht_group=%d: vq_dim 1 is built for groups of %d, and of 1024 = the whole token of 8 heads",
                  L->rht_group, kRtnGroup);
  } else if (L->n_codewords != 16 && L->n_codewords != 64 && L->n_codewords != 256) {
    return fail(pow2 ? AQUAKV_EUNSUPPORTED : AQUAKV_EINVAL, "n_codewords=%d: must be 16, 64 or 256", L->n_codewords);
  }
  if (L->dtype != AQUAKV_BF16 && L->dtype != AQUAKV_FP32) return fail(AQUAKV_EINVAL, "dtype=%d", L->dtype);
  const int D = L->kv_heads * L->head_dim;
  if (!is_rtn(L) && L->rht_group != 0 && L->rht_group != L->head_dim) {
    if (L->rht_group != D) return fail(AQUAKV_EINVAL, "rht_group=%d must be 0, head_dim or kv_heads * head_dim", L->rht_group);
    if (D != 1024) return fail(AQUAKV_EUNSUPPORTED, "rht_group=%d: groups across heads are built for 8 heads of 128", L->rht_group);
  }
  if (L->d_in_k < 0 || L->d_in_k % 128) return fail(AQUAKV_EINVAL, "d_in_k=%d must be a non-negative multiple of 128", L->d_in_k);
  if (L->d_in_v < 0 || L->d_in_v % 128) return fail(AQUAKV_EINVAL, "d_in_v=%d must be a non-negative multiple of 128", L->d_in_v);
  if (L->d_in_v != 0 && L->d_in_v <= D)
    return fail(AQUAKV_EINVAL, "d_in_v=%d must exceed D=%d (inputs are [Vhat_prev | Khat])", L->d_in_v, D);
  if (!is_rtn(L)) {      // the round-to-nearest backbone has neither grid nor rotation; the three pointers are ignored
    if (L->codebook == nullptr) return fail(AQUAKV_ENULL, "codebook is NULL");
    if (L->signs_k == nullptr || L->signs_v == nullptr) return fail(AQUAKV_ENULL, "signs_k / signs_v is NULL");
  }
  if (L->d_in_k && L->w_k == nullptr) return fail(AQUAKV_ENULL, "w_k is NULL but d_in_k=%d", L->d_in_k);
  if (L->d_in_v && L->w_v == nullptr) return fail(AQUAKV_ENULL, "w_v is NULL but d_in_v=%d", L->d_in_v);
  const void* used[] = {L->w_k, L->b_k, L->w_v, L->b_v};
  for (const void* p : used)
    if (p != nullptr && misaligned(p)) return fail(AQUAKV_EALIGN, "a pointer in aquakv_layer is not 16-byte aligned");
  if (!is_rtn(L)) {      // ignored (never read, whatever they hold) by the round-to-nearest backbone
    const void* grid[] = {L->codebook, L->signs_k, L->signs_v, L->search_table};
    for (const void* p : grid)
      if (p != nullptr && misaligned(p)) return fail(AQUAKV_EALIGN, "a pointer in aquakv_layer is not 16-byte aligned");
  }
  return AQUAKV_OK;
}

// rotation group = the whole token vector (Sect. 4.1 of the paper) instead of one head
inline bool is_wide(const aquakv_layer* L) {
  if (is_rtn(L)) return L->rht_group == 1024;
  return L->rht_group != 0 && L->rht_group != L->head_dim;
}
// bytes of scales per token row: one fp16 per rotation group, or (fp16 step, 16-bit zero point) per group of 64
inline size_t scale_row_bytes(const aquakv_layer* L) {
  if (is_rtn(L)) return (is_wide(L) ? 1 : (size_t)L->kv_heads * (L->head_dim / kRtnGroup)) * 2 * sizeof(uint16_t);
  return (is_wide(L) ? 1 : (size_t)L->kv_heads) * sizeof(uint16_t);
}

int check_ptr(const void* p, const char* name, bool required) {
  if (p == nullptr) return required ? fail(AQUAKV_ENULL, "%s is NULL", name) : AQUAKV_OK;
  if (misaligned(p)) return fail(AQUAKV_EALIGN, "%s is not 16-byte aligned", name);
  return AQUAKV_OK;
}

// scales are read and written one fp16 at a time: with one scale per token a row range of the cache starts at
// any even address
// (the round-to-nearest backbone stores a step and a zero point together as one 4-byte word)
int check_scales(const aquakv_layer* L, const void* p, const char* name, bool required) {
  if (p == nullptr) return required ? fail(AQUAKV_ENULL, "%s is NULL", name) : AQUAKV_OK;
  const unsigned need = is_rtn(L) ? 4u : 2u;
  if (reinterpret_cast<uintptr_t>(p) & (need - 1u)) return fail(AQUAKV_EALIGN, "%s is not %u-byte aligned", name, need);
  return AQUAKV_OK;
}

// Byte ranges [p, p + n) of the buffers of one call.  The kernels of a call read whole rows of their inputs
// while other workgroups write outputs for the same rows, so an output that overlaps an input it may not
// alias (or another output, or the workspace) is a race; it is refused before anything is launched.
struct Range { const void* p; size_t n; const char* name; };
inline bool overlap(const Range& a, const Range& b) {
  if (a.p == nullptr || b.p == nullptr || a.n == 0 || b.n == 0) return false;
  const uintptr_t a0 = reinterpret_cast<uintptr_t>(a.p), b0 = reinterpret_cast<uintptr_t>(b.p);
  return a0 < b0 + b.n && b0 < a0 + a.n;
}
// every output against every input and against the other outputs; `inplace` (nullable, one entry per output)
// names the one input an output may coincide with exactly (reconstruction in place)
int check_no_alias(const Range* outs, int n_out, const Range* ins, int n_in, const void* const* inplace = nullptr) {
  for (int i = 0; i < n_out; ++i) {
    for (int j = 0; j < n_in; ++j) {
      if (inplace != nullptr && inplace[i] != nullptr && inplace[i] == ins[j].p && outs[i].p == ins[j].p) continue;
      if (overlap(outs[i], ins[j])) return fail(AQUAKV_EINVAL, "%s overlaps %s", outs[i].name, ins[j].name);
    }
    for (int j = i + 1; j < n_out; ++j)
      if (overlap(outs[i], outs[j])) return fail(AQUAKV_EINVAL, "%s overlaps %s", outs[i].name, outs[j].name);
  }
  return AQUAKV_OK;
}

#define CHECK(expr)                      \
  do {                                   \
    const int s_ = (expr);               \
    if (s_ != AQUAKV_OK) return s_;      \
  } while (0)

#define HIP_TRY(expr)                                                                     \
  do {                                                                                    \
    const hipError_t e_ = (expr);                                                         \
    if (e_ != hipSuccess) return fail(AQUAKV_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

struct Plan {
  int D;
  size_t eb;          // bytes per element of the storage dtype
  size_t code_row;    // bytes of codes per token row
  int64_t chunk;      // rows per pass
  bool fused;         // bf16: predictor fused with the quantizer kernels
  bool fused_dec;     // bf16: predictor fused with the inverse quantizer (also for groups across the 8 heads)
  size_t p_bytes;     // front of the workspace: fp32 predictions of one chunk, or re-tiled predictor weights
  size_t khat_bytes;  // temporary Khat of one chunk
};

Plan make_plan(const aquakv_layer* L, int64_t tokens) {
  Plan pl;
  pl.D = L->kv_heads * L->head_dim;
  pl.eb = elem_bytes(L->dtype);
  pl.code_row = (size_t)L->kv_heads * (L->head_dim / 2) * code_bits(L) / 8;
  pl.fused = L->dtype == AQUAKV_BF16;                  // predictor fused with the quantizer (groups of one head: a tile of one
                                                       // head; groups across the 8 heads: a slab of 64 tokens x all heads)
  pl.fused_dec = L->dtype == AQUAKV_BF16;              // decoding needs no statistic of the whole group
  const int64_t cap = pl.fused ? kChunkRowsFused : kChunkRowsSplit;
  pl.chunk = tokens < cap ? tokens : cap;
  // front of the workspace: the fp32 predictions of a chunk (split path), or (bf16, groups across the heads) the
  // predictor weights re-tiled for the encoder's main loop
  const int d_in_max = L->d_in_k > L->d_in_v ? L->d_in_k : L->d_in_v;
  pl.p_bytes = !pl.fused ? (size_t)pl.chunk * pl.D * sizeof(float) : (is_wide(L) ? (size_t)pl.D * d_in_max * pl.eb : 0);
  pl.khat_bytes = (size_t)pl.chunk * pl.D * pl.eb;
  return pl;
}

inline const void* at(const void* base, int64_t row, size_t row_bytes) {
  return base == nullptr ? nullptr : static_cast<const unsigned char*>(base) + row * row_bytes;
}
inline void* at(void* base, int64_t row, size_t row_bytes) {
  return base == nullptr ? nullptr : static_cast<unsigned char*>(base) + row * row_bytes;
}

// ---- one chunk of rows [r0, r0 + n) of one tensor; pointers are the tensors' bases -------------------------------
// keys of Alg. "encode":  K_pred = f_key(Khat_prev);  K_q = Q(K - K_pred);  khat_dst (chunk-local, nullable) = Q^-1(K_q) + K_pred
int encode_keys_chunk(const aquakv_layer* L, const Plan& pl, int64_t r0, int64_t n, const void* K, const void* Khat_prev,
                      uint8_t* k_codes, uint16_t* k_scales, void* khat_dst, float* Pbuf, hipStream_t stream) {
  const bool has_k = L->d_in_k != 0;
  const size_t row = (size_t)pl.D * pl.eb, srow = scale_row_bytes(L);
  if (has_k && pl.fused) {
    const void* x0 = at(Khat_prev, r0, (size_t)L->d_in_k * pl.eb);
    uint8_t* const kc = static_cast<uint8_t*>(at(k_codes, r0, pl.code_row));
    uint16_t* const ks = static_cast<uint16_t*>(at(k_scales, r0, srow));
    if (is_wide(L))
      HIP_TRY(aquakv::launch_fused_encode_wide(quantizer_id(L), x0, L->d_in_k, nullptr, 0, L->w_k, Pbuf, L->b_k, L->signs_k,
                                               L->codebook, L->search_table, at(K, r0, row), kc, ks, khat_dst, n, pl.D, stream));
    else
      HIP_TRY(aquakv::launch_fused_encode(quantizer_id(L), x0, L->d_in_k, nullptr, 0, L->w_k, L->b_k, L->signs_k, L->codebook,
                                          L->search_table, at(K, r0, row), kc, ks, khat_dst, n, pl.D, stream));
    return AQUAKV_OK;
  }
  if (has_k)
    HIP_TRY(aquakv::launch_predict(L->dtype, at(Khat_prev, r0, (size_t)L->d_in_k * pl.eb), L->d_in_k, nullptr, 0, L->w_k,
                                   L->b_k, Pbuf, n, pl.D, stream));
  HIP_TRY(aquakv::launch_quantize(L->dtype, quantizer_id(L), at(K, r0, row), has_k ? Pbuf : nullptr, L->signs_k, L->codebook,
                                  L->search_table, static_cast<uint8_t*>(at(k_codes, r0, pl.code_row)),
                                  static_cast<uint16_t*>(at(k_scales, r0, srow)), khat_dst, n, L->kv_heads, is_wide(L),
                                  stream));
  return AQUAKV_OK;
}

// values of Alg. "encode":  V_pred = f_value([Vhat_prev; Khat]);  V_q = Q(V - V_pred);  khat_src is chunk-local
int encode_values_chunk(const aquakv_layer* L, const Plan& pl, int64_t r0, int64_t n, const void* V, const void* Vhat_prev,
                        const void* khat_src, uint8_t* v_codes, uint16_t* v_scales, void* Vhat, float* Pbuf,
                        hipStream_t stream) {
  const bool has_v = L->d_in_v != 0;
  const int D = pl.D;
  const size_t row = (size_t)D * pl.eb, srow = scale_row_bytes(L);
  if (has_v && pl.fused) {
    const void* x0 = at(Vhat_prev, r0, (size_t)(L->d_in_v - D) * pl.eb);
    uint8_t* const vc = static_cast<uint8_t*>(at(v_codes, r0, pl.code_row));
    uint16_t* const vs = static_cast<uint16_t*>(at(v_scales, r0, srow));
    if (is_wide(L))
      HIP_TRY(aquakv::launch_fused_encode_wide(quantizer_id(L), x0, L->d_in_v - D, khat_src, D, L->w_v, Pbuf, L->b_v,
                                               L->signs_v, L->codebook, L->search_table, at(V, r0, row), vc, vs,
                                               at(Vhat, r0, row), n, D, stream));
    else
      HIP_TRY(aquakv::launch_fused_encode(quantizer_id(L), x0, L->d_in_v - D, khat_src, D, L->w_v, L->b_v, L->signs_v,
                                          L->codebook, L->search_table, at(V, r0, row), vc, vs, at(Vhat, r0, row), n, D, stream));
    return AQUAKV_OK;
  }
  if (has_v)
    HIP_TRY(aquakv::launch_predict(L->dtype, at(Vhat_prev, r0, (size_t)(L->d_in_v - D) * pl.eb), L->d_in_v - D, khat_src, D,
                                   L->w_v, L->b_v, Pbuf, n, D, stream));
  HIP_TRY(aquakv::launch_quantize(L->dtype, quantizer_id(L), at(V, r0, row), has_v ? Pbuf : nullptr, L->signs_v, L->codebook,
                                  L->search_table, static_cast<uint8_t*>(at(v_codes, r0, pl.code_row)),
                                  static_cast<uint16_t*>(at(v_scales, r0, srow)), at(Vhat, r0, row), n, L->kv_heads,
                                  is_wide(L), stream));
  return AQUAKV_OK;
}

// keys of Alg. "decode":  Khat = Q^-1(K_q) + f_key(Khat_prev)
int decode_keys_chunk(const aquakv_layer* L, const Plan& pl, int64_t r0, int64_t n, const uint8_t* k_codes,
                      const uint16_t* k_scales, const void* Khat_prev, void* Khat, float* Pbuf, hipStream_t stream) {
  const bool has_k = L->d_in_k != 0;
  const size_t row = (size_t)pl.D * pl.eb, srow = scale_row_bytes(L);
  if (has_k && pl.fused_dec) {
    HIP_TRY(aquakv::launch_fused_decode(quantizer_id(L), at(Khat_prev, r0, (size_t)L->d_in_k * pl.eb), L->d_in_k, nullptr, 0,
                                        L->w_k, L->b_k, L->signs_k, L->codebook,
                                        static_cast<const uint8_t*>(at(k_codes, r0, pl.code_row)),
                                        static_cast<const uint16_t*>(at(k_scales, r0, srow)), at(Khat, r0, row), n, pl.D,
                                        is_wide(L), stream));
    return AQUAKV_OK;
  }
  if (has_k)
    HIP_TRY(aquakv::launch_predict(L->dtype, at(Khat_prev, r0, (size_t)L->d_in_k * pl.eb), L->d_in_k, nullptr, 0, L->w_k,
                                   L->b_k, Pbuf, n, pl.D, stream));
  HIP_TRY(aquakv::launch_dequantize(L->dtype, quantizer_id(L), static_cast<const uint8_t*>(at(k_codes, r0, pl.code_row)),
                                    static_cast<const uint16_t*>(at(k_scales, r0, srow)), has_k ? Pbuf : nullptr, L->signs_k,
                                    L->codebook, at(Khat, r0, row), n, L->kv_heads, is_wide(L), stream));
  return AQUAKV_OK;
}

// values of Alg. "decode":  Vhat = Q^-1(V_q) + f_value([Vhat_prev; Khat])
int decode_values_chunk(const aquakv_layer* L, const Plan& pl, int64_t r0, int64_t n, const uint8_t* v_codes,
                        const uint16_t* v_scales, const void* Vhat_prev, const void* Khat, void* Vhat, float* Pbuf,
                        hipStream_t stream) {
  const bool has_v = L->d_in_v != 0;
  const int D = pl.D;
  const size_t row = (size_t)D * pl.eb, srow = scale_row_bytes(L);
  if (has_v && pl.fused_dec) {
    HIP_TRY(aquakv::launch_fused_decode(quantizer_id(L), at(Vhat_prev, r0, (size_t)(L->d_in_v - D) * pl.eb), L->d_in_v - D,
                                        at(Khat, r0, row), D, L->w_v, L->b_v, L->signs_v, L->codebook,
                                        static_cast<const uint8_t*>(at(v_codes, r0, pl.code_row)),
                                        static_cast<const uint16_t*>(at(v_scales, r0, srow)), at(Vhat, r0, row), n, D,
                                        is_wide(L), stream));
    return AQUAKV_OK;
  }
  if (has_v)
    HIP_TRY(aquakv::launch_predict(L->dtype, at(Vhat_prev, r0, (size_t)(L->d_in_v - D) * pl.eb), L->d_in_v - D,
                                   at(Khat, r0, row), D, L->w_v, L->b_v, Pbuf, n, D, stream));
  HIP_TRY(aquakv::launch_dequantize(L->dtype, quantizer_id(L), static_cast<const uint8_t*>(at(v_codes, r0, pl.code_row)),
                                    static_cast<const uint16_t*>(at(v_scales, r0, srow)), has_v ? Pbuf : nullptr, L->signs_v,
                                    L->codebook, at(Vhat, r0, row), n, L->kv_heads, is_wide(L), stream));
  return AQUAKV_OK;
}

}  // namespace

extern "C" {

int aquakv_version(void) { return AQUAKV_VERSION; }

const char* aquakv_status_string(int status) {
  switch (status) {
    case AQUAKV_OK: return "ok";
    case AQUAKV_EINVAL: return "invalid argument";
    case AQUAKV_ENULL: return "required pointer is NULL";
    case AQUAKV_EALIGN: return "pointer is not 16-byte aligned";
    case AQUAKV_EUNSUPPORTED: return "configuration not built";
    case AQUAKV_EWORKSPACE: return "workspace too small";
    case AQUAKV_EHIP: return "HIP error";
    default: return "unknown status";
  }
}

const char* aquakv_last_error(void) { return g_err; }

size_t aquakv_search_table_bytes(int32_t n_codewords) {
  return (n_codewords == 16 || n_codewords == 64 || n_codewords == 256) ? aquakv::kSearchTableBytes : 0;
}

int aquakv_build_search_table(const float* codebook, int32_t vq_dim, int32_t n_codewords, void* table, void* stream) {
  if (vq_dim != 2) return fail(vq_dim < 1 ? AQUAKV_EINVAL : AQUAKV_EUNSUPPORTED, "vq_dim=%d: only 2 is built", vq_dim);
  if (aquakv_search_table_bytes(n_codewords) == 0)
    return fail(AQUAKV_EINVAL, "n_codewords=%d: must be 16, 64 or 256", n_codewords);
  CHECK(check_ptr(codebook, "codebook", true));
  CHECK(check_ptr(table, "table", true));
  HIP_TRY(aquakv::launch_build_search_table(codebook, n_codewords, table, static_cast<hipStream_t>(stream)));
  return AQUAKV_OK;
}

size_t aquakv_workspace_bytes(const aquakv_layer* layer, int64_t tokens) {
  if (check_layer(layer) != AQUAKV_OK || tokens <= 0) return 0;
  const Plan pl = make_plan(layer, tokens);
  return pl.p_bytes + pl.khat_bytes;
}

int aquakv_fused_tile_heads(const aquakv_layer* layer, int64_t tokens) {
  if (check_layer(layer) != AQUAKV_OK || tokens <= 0) return 0;
  const Plan pl = make_plan(layer, tokens);
  if (!pl.fused_dec || layer->d_in_k == 0) return 0;
  return aquakv::two_heads_pays(pl.chunk, pl.D) ? 2 : 1;
}

int aquakv_predict(const aquakv_layer* L, int which, int64_t tokens, const void* x0, const void* x1, float* P,
                   void* stream) {
  CHECK(check_layer(L));
  if (which != AQUAKV_KEY && which != AQUAKV_VALUE) return fail(AQUAKV_EINVAL, "which=%d", which);
  if (tokens < 0) return fail(AQUAKV_EINVAL, "tokens=%lld", (long long)tokens);
  const int D = L->kv_heads * L->head_dim;
  const int d_in = which == AQUAKV_KEY ? L->d_in_k : L->d_in_v;
  if (d_in == 0) return fail(AQUAKV_EINVAL, "the layer has no %s predictor", which == AQUAKV_KEY ? "key" : "value");
  CHECK(check_ptr(x0, "x0", true));
  CHECK(check_ptr(x1, "x1", which == AQUAKV_VALUE));
  CHECK(check_ptr(P, "P", true));
  if (tokens == 0) return AQUAKV_OK;
  const int d0 = which == AQUAKV_KEY ? d_in : d_in - D;
  const int d1 = which == AQUAKV_KEY ? 0 : D;
  HIP_TRY(aquakv::launch_predict(L->dtype, x0, d0, which == AQUAKV_KEY ? nullptr : x1, d1,
                                 which == AQUAKV_KEY ? L->w_k : L->w_v, which == AQUAKV_KEY ? L->b_k : L->b_v, P,
                                 tokens, D, static_cast<hipStream_t>(stream)));
  return AQUAKV_OK;
}

int aquakv_quantize(const aquakv_layer* L, int which, int64_t tokens, const void* X, const float* P, uint8_t* codes,
                    uint16_t* scales, void* Xhat, void* stream) {
  CHECK(check_layer(L));
  if (which != AQUAKV_KEY && which != AQUAKV_VALUE) return fail(AQUAKV_EINVAL, "which=%d", which);
  if (tokens < 0) return fail(AQUAKV_EINVAL, "tokens=%lld", (long long)tokens);
  CHECK(check_ptr(X, "X", true));
  CHECK(check_ptr(P, "P", false));
  CHECK(check_ptr(codes, "codes", true));
  CHECK(check_scales(L, scales, "scales", true));
  CHECK(check_ptr(Xhat, "Xhat", false));
  HIP_TRY(aquakv::launch_quantize(L->dtype, quantizer_id(L), X, P, which == AQUAKV_KEY ? L->signs_k : L->signs_v,
                                  L->codebook, L->search_table, codes, scales, Xhat, tokens, L->kv_heads, is_wide(L),
                                  static_cast<hipStream_t>(stream)));
  return AQUAKV_OK;
}

int aquakv_dequantize(const aquakv_layer* L, int which, int64_t tokens, const uint8_t* codes, const uint16_t* scales,
                      const float* P, void* Xhat, void* stream) {
  CHECK(check_layer(L));
  if (which != AQUAKV_KEY && which != AQUAKV_VALUE) return fail(AQUAKV_EINVAL, "which=%d", which);
  if (tokens < 0) return fail(AQUAKV_EINVAL, "tokens=%lld", (long long)tokens);
  CHECK(check_ptr(codes, "codes", true));
  CHECK(check_scales(L, scales, "scales", true));
  CHECK(check_ptr(P, "P", false));
  CHECK(check_ptr(Xhat, "Xhat", true));
  HIP_TRY(aquakv::launch_dequantize(L->dtype, quantizer_id(L), codes, scales, P,
                                    which == AQUAKV_KEY ? L->signs_k : L->signs_v, L->codebook, Xhat, tokens,
                                    L->kv_heads, is_wide(L), static_cast<hipStream_t>(stream)));
  return AQUAKV_OK;
}

int aquakv_encode_layer(const aquakv_layer* L, int64_t tokens, const void* K, const void* V, const void* Khat_prev,
                        const void* Vhat_prev, uint8_t* k_codes, uint16_t* k_scales, uint8_t* v_codes,
                        uint16_t* v_scales, void* Khat, void* Vhat, void* workspace, size_t workspace_bytes,
                        void* stream_) {
  CHECK(check_layer(L));
  if (tokens < 0) return fail(AQUAKV_EINVAL, "tokens=%lld", (long long)tokens);
  const bool has_k = L->d_in_k != 0, has_v = L->d_in_v != 0;
  CHECK(check_ptr(K, "K", true));
  CHECK(check_ptr(V, "V", true));
  CHECK(check_ptr(Khat_prev, "Khat_prev", has_k));
  CHECK(check_ptr(Vhat_prev, "Vhat_prev", has_v));
  CHECK(check_ptr(k_codes, "k_codes", true));
  CHECK(check_scales(L, k_scales, "k_scales", true));
  CHECK(check_ptr(v_codes, "v_codes", true));
  CHECK(check_scales(L, v_scales, "v_scales", true));
  CHECK(check_ptr(Khat, "Khat", false));
  CHECK(check_ptr(Vhat, "Vhat", false));
  if (tokens == 0) return AQUAKV_OK;
  const Plan pl = make_plan(L, tokens);
  CHECK(check_ptr(workspace, "workspace", true));
  if (workspace_bytes < pl.p_bytes + pl.khat_bytes)
    return fail(AQUAKV_EWORKSPACE, "workspace %zu B < required %zu B", workspace_bytes, pl.p_bytes + pl.khat_bytes);

  const size_t row = (size_t)pl.D * pl.eb;
  {
    const size_t t = (size_t)tokens, crow = pl.code_row, srow = scale_row_bytes(L);
    const Range outs[] = {{Khat, t * row, "Khat"}, {Vhat, t * row, "Vhat"}, {k_codes, t * crow, "k_codes"},
                          {v_codes, t * crow, "v_codes"}, {k_scales, t * srow, "k_scales"}, {v_scales, t * srow, "v_scales"},
                          {workspace, pl.p_bytes + pl.khat_bytes, "workspace"}};
    const Range ins[] = {{K, t * row, "K"}, {V, t * row, "V"}, {Khat_prev, t * L->d_in_k * pl.eb, "Khat_prev"},
                         {Vhat_prev, has_v ? t * (L->d_in_v - pl.D) * pl.eb : 0, "Vhat_prev"}};
    const void* const inplace[] = {K, V, nullptr, nullptr, nullptr, nullptr, nullptr};
    CHECK(check_no_alias(outs, 7, ins, 4, inplace));
  }

  hipStream_t stream = static_cast<hipStream_t>(stream_);
  float* Pbuf = static_cast<float*>(workspace);
  void* khat_tmp = static_cast<unsigned char*>(workspace) + pl.p_bytes;

  for (int64_t r0 = 0; r0 < tokens; r0 += pl.chunk) {
    const int64_t n = tokens - r0 < pl.chunk ? tokens - r0 : pl.chunk;
    void* khat_dst = Khat != nullptr ? at(Khat, r0, row) : (has_v ? khat_tmp : nullptr);
    CHECK(encode_keys_chunk(L, pl, r0, n, K, Khat_prev, k_codes, k_scales, khat_dst, Pbuf, stream));
    CHECK(encode_values_chunk(L, pl, r0, n, V, Vhat_prev, khat_dst, v_codes, v_scales, Vhat, Pbuf, stream));
  }
  return AQUAKV_OK;
}

int aquakv_decode_layer(const aquakv_layer* L, int64_t tokens, const uint8_t* k_codes, const uint16_t* k_scales,
                        const uint8_t* v_codes, const uint16_t* v_scales, const void* Khat_prev, const void* Vhat_prev,
                        void* Khat, void* Vhat, void* workspace, size_t workspace_bytes, void* stream_) {
  CHECK(check_layer(L));
  if (tokens < 0) return fail(AQUAKV_EINVAL, "tokens=%lld", (long long)tokens);
  const bool want_v = Vhat != nullptr;
  const bool has_k = L->d_in_k != 0, has_v = L->d_in_v != 0 && want_v;
  CHECK(check_ptr(k_codes, "k_codes", true));
  CHECK(check_scales(L, k_scales, "k_scales", true));
  CHECK(check_ptr(v_codes, "v_codes", want_v));
  CHECK(check_scales(L, v_scales, "v_scales", want_v));
  CHECK(check_ptr(Khat_prev, "Khat_prev", has_k));
  CHECK(check_ptr(Vhat_prev, "Vhat_prev", has_v));
  CHECK(check_ptr(Khat, "Khat", true));
  CHECK(check_ptr(Vhat, "Vhat", false));
  if (tokens == 0) return AQUAKV_OK;
  const Plan pl = make_plan(L, tokens);
  CHECK(check_ptr(workspace, "workspace", true));
  if (workspace_bytes < pl.p_bytes + pl.khat_bytes)
    return fail(AQUAKV_EWORKSPACE, "workspace %zu B < required %zu B", workspace_bytes, pl.p_bytes + pl.khat_bytes);

  {
    const size_t t = (size_t)tokens, row = (size_t)pl.D * pl.eb, crow = pl.code_row, srow = scale_row_bytes(L);
    const Range outs[] = {{Khat, t * row, "Khat"}, {Vhat, t * row, "Vhat"}, {workspace, pl.p_bytes, "workspace"}};
    const Range ins[] = {{Khat_prev, t * L->d_in_k * pl.eb, "Khat_prev"},
                         {Vhat_prev, has_v ? t * (L->d_in_v - pl.D) * pl.eb : 0, "Vhat_prev"},
                         {k_codes, t * crow, "k_codes"}, {v_codes, want_v ? t * crow : 0, "v_codes"},
                         {k_scales, t * srow, "k_scales"}, {v_scales, want_v ? t * srow : 0, "v_scales"}};
    CHECK(check_no_alias(outs, 3, ins, 6));
  }
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  float* Pbuf = static_cast<float*>(workspace);

  for (int64_t r0 = 0; r0 < tokens; r0 += pl.chunk) {
    const int64_t n = tokens - r0 < pl.chunk ? tokens - r0 : pl.chunk;
    CHECK(decode_keys_chunk(L, pl, r0, n, k_codes, k_scales, Khat_prev, Khat, Pbuf, stream));
    if (want_v) CHECK(decode_values_chunk(L, pl, r0, n, v_codes, v_scales, Vhat_prev, Khat, Vhat, Pbuf, stream));
  }
  return AQUAKV_OK;
}

// ---- the two halves of Alg. "encode" / "decode" as calls of their own -------------------------------------------
// The key chain of a layer stack depends on keys only, the value chain on the previous values and this layer's keys,
// so a caller can run them on two streams (events between them) and overlap the kernels of neighbouring layers.
int aquakv_encode_keys(const aquakv_layer* L, int64_t tokens, const void* K, const void* Khat_prev, uint8_t* k_codes,
                       uint16_t* k_scales, void* Khat, void* workspace, size_t workspace_bytes, void* stream_) {
  CHECK(check_layer(L));
  if (tokens < 0) return fail(AQUAKV_EINVAL, "tokens=%lld", (long long)tokens);
  CHECK(check_ptr(K, "K", true));
  CHECK(check_ptr(Khat_prev, "Khat_prev", L->d_in_k != 0));
  CHECK(check_ptr(k_codes, "k_codes", true));
  CHECK(check_scales(L, k_scales, "k_scales", true));
  CHECK(check_ptr(Khat, "Khat", false));
  if (tokens == 0) return AQUAKV_OK;
  const Plan pl = make_plan(L, tokens);
  if (pl.p_bytes != 0) {
    CHECK(check_ptr(workspace, "workspace", true));
    if (workspace_bytes < pl.p_bytes) return fail(AQUAKV_EWORKSPACE, "workspace %zu B < required %zu B", workspace_bytes, pl.p_bytes);
  }
  const size_t row = (size_t)pl.D * pl.eb;
  {
    const size_t t = (size_t)tokens;
    const Range outs[] = {{Khat, t * row, "Khat"}, {k_codes, t * pl.code_row, "k_codes"},
                          {k_scales, t * scale_row_bytes(L), "k_scales"}, {workspace, pl.p_bytes, "workspace"}};
    const Range ins[] = {{K, t * row, "K"}, {Khat_prev, t * L->d_in_k * pl.eb, "Khat_prev"}};
    const void* const inplace[] = {K, nullptr, nullptr, nullptr};
    CHECK(check_no_alias(outs, 4, ins, 2, inplace));
  }
  for (int64_t r0 = 0; r0 < tokens; r0 += pl.chunk) {
    const int64_t n = tokens - r0 < pl.chunk ? tokens - r0 : pl.chunk;
    CHECK(encode_keys_chunk(L, pl, r0, n, K, Khat_prev, k_codes, k_scales, at(Khat, r0, row), static_cast<float*>(workspace),
                            static_cast<hipStream_t>(stream_)));
  }
  return AQUAKV_OK;
}

int aquakv_encode_values(const aquakv_layer* L, int64_t tokens, const void* V, const void* Vhat_prev, const void* Khat,
                         uint8_t* v_codes, uint16_t* v_scales, void* Vhat, void* workspace, size_t workspace_bytes,
                         void* stream_) {
  CHECK(check_layer(L));
  if (tokens < 0) return fail(AQUAKV_EINVAL, "tokens=%lld", (long long)tokens);
  const bool has_v = L->d_in_v != 0;
  CHECK(check_ptr(V, "V", true));
  CHECK(check_ptr(Vhat_prev, "Vhat_prev", has_v));
  CHECK(check_ptr(Khat, "Khat", has_v));
  CHECK(check_ptr(v_codes, "v_codes", true));
  CHECK(check_scales(L, v_scales, "v_scales", true));
  CHECK(check_ptr(Vhat, "Vhat", false));
  if (tokens == 0) return AQUAKV_OK;
  const Plan pl = make_plan(L, tokens);
  if (pl.p_bytes != 0) {
    CHECK(check_ptr(workspace, "workspace", true));
    if (workspace_bytes < pl.p_bytes) return fail(AQUAKV_EWORKSPACE, "workspace %zu B < required %zu B", workspace_bytes, pl.p_bytes);
  }
  const size_t row = (size_t)pl.D * pl.eb;
  {
    const size_t t = (size_t)tokens;
    const Range outs[] = {{Vhat, t * row, "Vhat"}, {v_codes, t * pl.code_row, "v_codes"},
                          {v_scales, t * scale_row_bytes(L), "v_scales"}, {workspace, pl.p_bytes, "workspace"}};
    const Range ins[] = {{V, t * row, "V"}, {Vhat_prev, has_v ? t * (L->d_in_v - pl.D) * pl.eb : 0, "Vhat_prev"},
                         {Khat, has_v ? t * row : 0, "Khat"}};
    const void* const inplace[] = {V, nullptr, nullptr, nullptr};
    CHECK(check_no_alias(outs, 4, ins, 3, inplace));
  }
  for (int64_t r0 = 0; r0 < tokens; r0 += pl.chunk) {
    const int64_t n = tokens - r0 < pl.chunk ? tokens - r0 : pl.chunk;
    CHECK(encode_values_chunk(L, pl, r0, n, V, Vhat_prev, at(Khat, r0, row), v_codes, v_scales, Vhat,
                              static_cast<float*>(workspace), static_cast<hipStream_t>(stream_)));
  }
  return AQUAKV_OK;
}

int aquakv_decode_values(const aquakv_layer* L, int64_t tokens, const uint8_t* v_codes, const uint16_t* v_scales,
                         const void* Vhat_prev, const void* Khat, void* Vhat, void* workspace, size_t workspace_bytes,
                         void* stream_) {
  CHECK(check_layer(L));
  if (tokens < 0) return fail(AQUAKV_EINVAL, "tokens=%lld", (long long)tokens);
  const bool has_v = L->d_in_v != 0;
  CHECK(check_ptr(v_codes, "v_codes", true));
  CHECK(check_scales(L, v_scales, "v_scales", true));
  CHECK(check_ptr(Vhat_prev, "Vhat_prev", has_v));
  CHECK(check_ptr(Khat, "Khat", has_v));
  CHECK(check_ptr(Vhat, "Vhat", true));
  if (tokens == 0) return AQUAKV_OK;
  const Plan pl = make_plan(L, tokens);
  if (pl.p_bytes != 0) {
    CHECK(check_ptr(workspace, "workspace", true));
    if (workspace_bytes < pl.p_bytes) return fail(AQUAKV_EWORKSPACE, "workspace %zu B < required %zu B", workspace_bytes, pl.p_bytes);
  }
  {
    const size_t t = (size_t)tokens, row = (size_t)pl.D * pl.eb;
    const Range outs[] = {{Vhat, t * row, "Vhat"}, {workspace, pl.p_bytes, "workspace"}};
    const Range ins[] = {{Vhat_prev, has_v ? t * (L->d_in_v - pl.D) * pl.eb : 0, "Vhat_prev"}, {Khat, has_v ? t * row : 0, "Khat"},
                         {v_codes, t * pl.code_row, "v_codes"}, {v_scales, t * scale_row_bytes(L), "v_scales"}};
    CHECK(check_no_alias(outs, 2, ins, 4));
  }
  for (int64_t r0 = 0; r0 < tokens; r0 += pl.chunk) {
    const int64_t n = tokens - r0 < pl.chunk ? tokens - r0 : pl.chunk;
    CHECK(decode_values_chunk(L, pl, r0, n, v_codes, v_scales, Vhat_prev, Khat, Vhat, static_cast<float*>(workspace),
                              static_cast<hipStream_t>(stream_)));
  }
  return AQUAKV_OK;
}

// ---- value side of attention: soft-max rows, decode of the values with the weighted sum over tokens ------------
namespace {
size_t weighted_part_bytes(int32_t batch, int32_t seq_len, int32_t q_heads) {
  const size_t chunks = ((size_t)seq_len + aquakv::kWeightedChunk - 1) / aquakv::kWeightedChunk;
  const size_t bytes = (size_t)batch * chunks * q_heads * 128 * sizeof(float);
  return (bytes + 255) & ~(size_t)255;
}
size_t weighted_stat_bytes(int32_t batch, int32_t seq_len, int32_t q_heads) {
  const size_t chunks = ((size_t)seq_len + aquakv::kWeightedChunk - 1) / aquakv::kWeightedChunk;
  const size_t bytes = (size_t)batch * chunks * q_heads * 2 * sizeof(float);
  return (bytes + 255) & ~(size_t)255;
}
bool weighted_fused(const aquakv_layer* L, const Plan& pl, int32_t seq_len) {
  return L->d_in_v != 0 && pl.fused_dec && seq_len % aquakv::kWeightedChunk == 0;
}
}  // namespace

int aquakv_softmax(int64_t rows, int64_t n, const float* scores, float* probs, void* stream) {
  if (rows < 0 || n < 0 || rows > 0x7fffffffLL) return fail(AQUAKV_EINVAL, "rows=%lld n=%lld", (long long)rows, (long long)n);
  CHECK(check_ptr(scores, "scores", true));
  CHECK(check_ptr(probs, "probs", true));
  HIP_TRY(aquakv::launch_softmax_rows(scores, probs, rows, n, static_cast<hipStream_t>(stream)));
  return AQUAKV_OK;
}

size_t aquakv_weighted_workspace_bytes(const aquakv_layer* L, int32_t batch, int32_t seq_len, int32_t q_heads) {
  if (check_layer(L) != AQUAKV_OK || batch < 1 || seq_len < 1 || q_heads < 1) return 0;
  const Plan pl = make_plan(L, (int64_t)batch * seq_len);
  return weighted_part_bytes(batch, seq_len, q_heads) + weighted_stat_bytes(batch, seq_len, q_heads) + pl.p_bytes;
}

namespace {
// shared body: softmax = false: `weights` are the weights; true: they are raw scores (soft-max taken per chunk and merged)
int decode_values_weighted(const aquakv_layer* L, int32_t batch, int32_t seq_len, int32_t q_heads, const uint8_t* v_codes,
                           const uint16_t* v_scales, const void* Vhat_prev, const void* Khat, const float* weights,
                           bool softmax, void* Vhat, float* out, float* row_stats, void* workspace, size_t workspace_bytes,
                           void* stream_) {
  CHECK(check_layer(L));
  if (batch < 0 || seq_len < 0) return fail(AQUAKV_EINVAL, "batch=%d seq_len=%d", batch, seq_len);
  if (q_heads < 1 || q_heads % L->kv_heads || q_heads / L->kv_heads > 8)
    return fail(AQUAKV_EINVAL, "q_heads=%d must be a multiple of kv_heads=%d, at most 8x", q_heads, L->kv_heads);
  const bool has_v = L->d_in_v != 0;
  CHECK(check_ptr(v_codes, "v_codes", true));
  CHECK(check_scales(L, v_scales, "v_scales", true));
  CHECK(check_ptr(Vhat_prev, "Vhat_prev", has_v));
  CHECK(check_ptr(Khat, "Khat", has_v));
  CHECK(check_ptr(weights, softmax ? "scores" : "weights", true));
  CHECK(check_ptr(Vhat, "Vhat", false));
  CHECK(check_ptr(out, "out", true));
  if (row_stats != nullptr && (reinterpret_cast<uintptr_t>(row_stats) & 3u))
    return fail(AQUAKV_EALIGN, "row_stats is not 4-byte aligned");
  const int64_t tokens = (int64_t)batch * seq_len;
  if (tokens == 0) return AQUAKV_OK;
  const Plan pl = make_plan(L, tokens);
  const bool fused = weighted_fused(L, pl, seq_len);
  if (!fused && Vhat == nullptr)
    return fail(AQUAKV_ENULL, "Vhat may be NULL only when the sums are taken inside the decode kernel (bf16, "
                              "a value predictor, seq_len a multiple of %d)",
                aquakv::kWeightedChunk);
  const size_t part_bytes = weighted_part_bytes(batch, seq_len, q_heads);
  const size_t stat_bytes = weighted_stat_bytes(batch, seq_len, q_heads);
  const size_t need = part_bytes + stat_bytes + (fused ? 0 : pl.p_bytes);
  CHECK(check_ptr(workspace, "workspace", true));
  if (workspace_bytes < need) return fail(AQUAKV_EWORKSPACE, "workspace %zu B < required %zu B", workspace_bytes, need);
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  unsigned char* wsb = static_cast<unsigned char*>(workspace);
  float* part = reinterpret_cast<float*>(wsb);
  float* pstats = softmax ? reinterpret_cast<float*>(wsb + part_bytes) : nullptr;
  float* Pbuf = reinterpret_cast<float*>(wsb + part_bytes + stat_bytes);
  if (fused) {
    const int D = pl.D;
    HIP_TRY(aquakv::launch_fused_weighted(quantizer_id(L), Vhat_prev, L->d_in_v - D, Khat, D, L->w_v, L->b_v, L->signs_v,
                                          L->codebook, v_codes, v_scales, Vhat, weights, part, pstats, seq_len, q_heads,
                                          tokens, D, is_wide(L), stream));
  } else {
    for (int64_t r0 = 0; r0 < tokens; r0 += pl.chunk) {
      const int64_t n = tokens - r0 < pl.chunk ? tokens - r0 : pl.chunk;
      CHECK(decode_values_chunk(L, pl, r0, n, v_codes, v_scales, Vhat_prev, Khat, Vhat, Pbuf, stream));
    }
    HIP_TRY(aquakv::launch_weighted_values(L->dtype, Vhat, weights, part, pstats, batch, seq_len, L->kv_heads, q_heads,
                                           stream));
  }
  HIP_TRY(aquakv::launch_combine_weighted(part, pstats, out, softmax ? row_stats : nullptr, batch, seq_len, q_heads, stream));
  return AQUAKV_OK;
}
}  // namespace

int aquakv_decode_values_weighted(const aquakv_layer* L, int32_t batch, int32_t seq_len, int32_t q_heads,
                                  const uint8_t* v_codes, const uint16_t* v_scales, const void* Vhat_prev,
                                  const void* Khat, const float* weights, void* Vhat, float* out, void* workspace,
                                  size_t workspace_bytes, void* stream) {
  return decode_values_weighted(L, batch, seq_len, q_heads, v_codes, v_scales, Vhat_prev, Khat, weights, false, Vhat, out,
                                nullptr, workspace, workspace_bytes, stream);
}

int aquakv_decode_values_attend(const aquakv_layer* L, int32_t batch, int32_t seq_len, int32_t q_heads,
                                const uint8_t* v_codes, const uint16_t* v_scales, const void* Vhat_prev, const void* Khat,
                                const float* scores, void* Vhat, float* out, float* row_stats, void* workspace,
                                size_t workspace_bytes, void* stream) {
  return decode_values_weighted(L, batch, seq_len, q_heads, v_codes, v_scales, Vhat_prev, Khat, scores, true, Vhat, out,
                                row_stats, workspace, workspace_bytes, stream);
}

int aquakv_attend_raw(int32_t dtype, int32_t batch, int32_t tokens, int32_t kv_heads, int32_t q_heads, const void* K,
                      const void* V, const void* q, const float* rope_cos, const float* rope_sin, float score_scale,
                      float* out, float* row_stats, int32_t accumulate, void* stream) {
  if (dtype != AQUAKV_BF16 && dtype != AQUAKV_FP32) return fail(AQUAKV_EINVAL, "dtype=%d", dtype);
  if (batch < 0 || tokens < 0) return fail(AQUAKV_EINVAL, "batch=%d tokens=%d", batch, tokens);
  if (tokens > aquakv::kAttendRawMaxTokens)
    return fail(AQUAKV_EUNSUPPORTED, "tokens=%d: at most %d uncompressed tokens per call", tokens, aquakv::kAttendRawMaxTokens);
  if (kv_heads < 1 || q_heads < 1 || q_heads % kv_heads)
    return fail(AQUAKV_EINVAL, "q_heads=%d must be a multiple of kv_heads=%d", q_heads, kv_heads);
  CHECK(check_ptr(K, "K", tokens != 0));
  CHECK(check_ptr(V, "V", tokens != 0));
  CHECK(check_ptr(q, "q", true));
  CHECK(check_ptr(out, "out", true));
  CHECK(check_ptr(row_stats, "row_stats", true));
  if ((rope_cos == nullptr) != (rope_sin == nullptr)) return fail(AQUAKV_ENULL, "rope_cos and rope_sin go together");
  CHECK(check_ptr(rope_cos, "rope_cos", false));
  CHECK(check_ptr(rope_sin, "rope_sin", false));
  if (batch == 0) return AQUAKV_OK;
  if (tokens == 0) {
    if (!accumulate) return fail(AQUAKV_EINVAL, "tokens=0 leaves nothing to write without a result to merge into");
    return AQUAKV_OK;
  }
  HIP_TRY(aquakv::launch_attend_raw(dtype, K, V, q, rope_cos, rope_sin, score_scale, out, row_stats, batch, tokens, kv_heads,
                                    q_heads, accumulate != 0, static_cast<hipStream_t>(stream)));
  return AQUAKV_OK;
}

// ---- calibration: ridge least-squares fit of one predictor (Alg. "Calibration") --------------------------------
size_t aquakv_fit_workspace_bytes(int32_t d_in, int32_t d_out) {
  if (d_in < 64 || d_in > 8192 || d_in % 64 || d_out < 64 || d_out > 8192 || d_out % 64) return 0;
  return aquakv::fit_workspace_bytes(d_in, d_out);
}

int aquakv_fit_predictor(int32_t dtype, int64_t tokens, const void* x0, int32_t d0, const void* x1, int32_t d1,
                         const void* Y, int32_t d_out, double rate, void* W, double* W64, float* bias, void* workspace,
                         size_t workspace_bytes, void* stream) {
  if (dtype != AQUAKV_BF16 && dtype != AQUAKV_FP32) return fail(AQUAKV_EINVAL, "dtype=%d", dtype);
  if (tokens < 1) return fail(AQUAKV_EINVAL, "tokens=%lld: at least one row is needed", (long long)tokens);
  if (d0 < 64 || d0 % 64 || d1 < 0 || d1 % 64) return fail(AQUAKV_EINVAL, "d0=%d d1=%d must be multiples of 64, d0 >= 64", d0, d1);
  if (d_out < 64 || d_out % 64) return fail(AQUAKV_EINVAL, "d_out=%d must be a positive multiple of 64", d_out);
  if ((int64_t)d0 + d1 > 8192 || d_out > 8192) return fail(AQUAKV_EUNSUPPORTED, "at most 8192 inputs and outputs");
  if (!(rate >= 0.0) || rate > 1e6) return fail(AQUAKV_EINVAL, "rate=%g", rate);
  CHECK(check_ptr(x0, "x0", true));
  CHECK(check_ptr(x1, "x1", d1 != 0));
  CHECK(check_ptr(Y, "Y", true));
  CHECK(check_ptr(W, "W", true));
  CHECK(check_ptr(W64, "W64", false));
  CHECK(check_ptr(bias, "bias", false));
  CHECK(check_ptr(workspace, "workspace", true));
  const size_t need = aquakv::fit_workspace_bytes(d0 + d1, d_out);
  if (workspace_bytes < need) return fail(AQUAKV_EWORKSPACE, "workspace %zu B < required %zu B", workspace_bytes, need);
  HIP_TRY(aquakv::launch_fit_predictor(dtype, tokens, x0, d0, d1 != 0 ? x1 : nullptr, d1, Y, d_out, rate, W, W64, bias, workspace,
                                       static_cast<hipStream_t>(stream)));
  return AQUAKV_OK;
}

size_t aquakv_scores_workspace_bytes(const aquakv_layer* L, int32_t batch, int32_t q_heads) {
  if (check_layer(L) != AQUAKV_OK || batch < 1 || q_heads < 1) return 0;
  if (L->dtype != AQUAKV_BF16 || is_wide(L) || !aquakv::folded_scores_supported(L->kv_heads, L->d_in_k, q_heads)) return 0;
  return aquakv::folded_scores_workspace_bytes(batch, q_heads);
}

}  // extern "C"

namespace {
// The folded form keeps per-call operands (the folded queries) in device memory.  Callers that cannot allocate
// take them from this array instead of a workspace of their own: aquakv_decode_attn_scores_folded_static.
// Host code never uses the array's name as an address: the device address is asked for once per device
// (hipGetSymbolAddress, with that device current) and kept.
constexpr int kStaticFoldBatches = 64;                                    // batch x passes of one call
constexpr size_t kStaticFoldBytes = (size_t)kStaticFoldBatches * aquakv::kFoldedBytesPerBatch;   // about 9 MiB
__device__ __align__(256) unsigned char scratch[kStaticFoldBytes];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// device address of `scratch` on the current device (looked up on the first call per device)
int static_scratch(void** out) {
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(AQUAKV_EUNSUPPORTED, "device ordinal %d: at most %d devices", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (ptr == nullptr) return fail(AQUAKV_EHIP, "hipGetSymbolAddress returned a null address");
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return AQUAKV_OK;
}

enum ScoresForm { kFormDefinition = 0, kFormFolded = 1 };

// shared body of the scoring entry points; rope_cos / rope_sin both NULL: no rotary embedding
int decode_attn_scores(const aquakv_layer* L, int32_t batch, int32_t seq_len, int32_t q_heads, const uint8_t* k_codes,
                       const uint16_t* k_scales, const void* Khat_prev, const void* q, const float* rope_cos,
                       const float* rope_sin, float score_scale, float* scores, void* Khat_out, void* workspace,
                       size_t workspace_bytes, void* stream_, int form) {
  CHECK(check_layer(L));
  if (batch < 0 || seq_len < 0) return fail(AQUAKV_EINVAL, "batch=%d seq_len=%d", batch, seq_len);
  if (q_heads < 1 || q_heads % L->kv_heads || q_heads / L->kv_heads > 8)
    return fail(AQUAKV_EINVAL, "q_heads=%d must be a multiple of kv_heads=%d, at most 8x", q_heads, L->kv_heads);
  const bool has_k = L->d_in_k != 0;
  CHECK(check_ptr(k_codes, "k_codes", true));
  CHECK(check_scales(L, k_scales, "k_scales", true));
  CHECK(check_ptr(Khat_prev, "Khat_prev", has_k));
  CHECK(check_ptr(q, "q", true));
  CHECK(check_ptr(scores, "scores", true));
  CHECK(check_ptr(Khat_out, "Khat_out", false));
  const int64_t tokens = (int64_t)batch * seq_len;
  const Plan pl = make_plan(L, tokens > 0 ? tokens : 1);
  if (form == kFormFolded) {
    if (!(has_k && pl.fused && !is_wide(L) && aquakv::folded_scores_supported(L->kv_heads, L->d_in_k, q_heads)))
      return fail(AQUAKV_EUNSUPPORTED, "the folded form is built for bf16 layers with 8 kv heads, a key predictor with 1024 "
                                       "inputs, rotation groups of one head and at most 64 query heads");
    if (tokens == 0) return AQUAKV_OK;
    // predictor folded into the query: Khat_prev and the codes are read once, nothing is recomputed
    CHECK(check_ptr(workspace, "workspace", true));
    const size_t need = aquakv::folded_scores_workspace_bytes(batch, q_heads);
    if (workspace_bytes < need) return fail(AQUAKV_EWORKSPACE, "workspace %zu B < required %zu B", workspace_bytes, need);
    // the round-to-nearest backbone has neither rotation nor grid: whatever the layer holds there is not passed on
    HIP_TRY(aquakv::launch_folded_scores(quantizer_id(L), Khat_prev, L->w_k, L->b_k, is_rtn(L) ? nullptr : L->signs_k,
                                         is_rtn(L) ? nullptr : L->codebook, k_codes, k_scales, q, score_scale, scores,
                                         workspace, batch, seq_len, q_heads, static_cast<hipStream_t>(stream_)));
    return AQUAKV_OK;
  }
  if (tokens == 0) return AQUAKV_OK;
  if (has_k && pl.fused_dec) {
    // one fused launch over all rows: prediction, inverse quantizer and dot products
    HIP_TRY(aquakv::launch_fused_scores(quantizer_id(L), Khat_prev, L->d_in_k, L->w_k, L->b_k, L->signs_k, L->codebook,
                                        k_codes, k_scales, q, score_scale, scores, Khat_out, seq_len, q_heads, tokens,
                                        pl.D, rope_cos, rope_sin, is_wide(L), static_cast<hipStream_t>(stream_)));
    return AQUAKV_OK;
  }
  if (has_k) {
    CHECK(check_ptr(workspace, "workspace", true));
    if (workspace_bytes < pl.p_bytes)
      return fail(AQUAKV_EWORKSPACE, "workspace %zu B < required %zu B", workspace_bytes, pl.p_bytes);
  }
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  float* Pbuf = static_cast<float*>(workspace);
  const size_t row = (size_t)pl.D * pl.eb;
  const size_t srow = scale_row_bytes(L);
  for (int64_t r0 = 0; r0 < tokens; r0 += pl.chunk) {
    const int64_t n = tokens - r0 < pl.chunk ? tokens - r0 : pl.chunk;
    if (has_k)
      HIP_TRY(aquakv::launch_predict(L->dtype, at(Khat_prev, r0, (size_t)L->d_in_k * pl.eb), L->d_in_k, nullptr, 0,
                                     L->w_k, L->b_k, Pbuf, n, pl.D, stream));
    HIP_TRY(aquakv::launch_attn_scores(L->dtype, quantizer_id(L), static_cast<const uint8_t*>(at(k_codes, r0, pl.code_row)),
                                       static_cast<const uint16_t*>(at(k_scales, r0, srow)), has_k ? Pbuf : nullptr,
                                       L->signs_k, L->codebook, q, score_scale, scores, at(Khat_out, r0, row), r0, n,
                                       seq_len, L->kv_heads, q_heads, rope_cos, rope_sin, is_wide(L), stream));
  }
  return AQUAKV_OK;
}
}  // namespace

extern "C" {

int aquakv_decode_attn_scores(const aquakv_layer* L, int32_t batch, int32_t seq_len, int32_t q_heads,
                              const uint8_t* k_codes, const uint16_t* k_scales, const void* Khat_prev, const void* q,
                              float score_scale, float* scores, void* Khat_out, void* workspace,
                              size_t workspace_bytes, void* stream_) {
  return decode_attn_scores(L, batch, seq_len, q_heads, k_codes, k_scales, Khat_prev, q, nullptr, nullptr, score_scale,
                            scores, Khat_out, workspace, workspace_bytes, stream_, kFormDefinition);
}

int aquakv_decode_attn_scores_folded(const aquakv_layer* L, int32_t batch, int32_t seq_len, int32_t q_heads,
                                     const uint8_t* k_codes, const uint16_t* k_scales, const void* Khat_prev,
                                     const void* q, float score_scale, float* scores, void* workspace,
                                     size_t workspace_bytes, void* stream_) {
  return decode_attn_scores(L, batch, seq_len, q_heads, k_codes, k_scales, Khat_prev, q, nullptr, nullptr, score_scale,
                            scores, nullptr, workspace, workspace_bytes, stream_, kFormFolded);
}

int aquakv_decode_attn_scores_folded_static(const aquakv_layer* L, int32_t batch, int32_t seq_len, int32_t q_heads,
                                            const uint8_t* k_codes, const uint16_t* k_scales, const void* Khat_prev,
                                            const void* q, float score_scale, float* scores, void* stream_) {
  CHECK(check_layer(L));
  if (batch < 0 || q_heads < 1) return fail(AQUAKV_EINVAL, "batch=%d q_heads=%d", batch, q_heads);
  const size_t need = aquakv::folded_scores_workspace_bytes(batch, q_heads);
  if (need > kStaticFoldBytes)
    return fail(AQUAKV_EUNSUPPORTED, "batch=%d with %d query heads needs %zu B of folded queries; the built-in buffer holds "
                                     "%zu B (batch x passes <= %d, one pass per 32 query heads): use "
                                     "aquakv_decode_attn_scores_folded with a workspace",
                batch, q_heads, need, kStaticFoldBytes, kStaticFoldBatches);
  void* ptr = nullptr;
  CHECK(static_scratch(&ptr));
  return decode_attn_scores(L, batch, seq_len, q_heads, k_codes, k_scales, Khat_prev, q, nullptr, nullptr, score_scale,
                            scores, nullptr, ptr, kStaticFoldBytes, stream_, kFormFolded);
}

int aquakv_decode_attn_scores_rope(const aquakv_layer* L, int32_t batch, int32_t seq_len, int32_t q_heads,
                                   const uint8_t* k_codes, const uint16_t* k_scales, const void* Khat_prev,
                                   const void* q, const float* rope_cos, const float* rope_sin, float score_scale,
                                   float* scores, void* Khat_out, void* workspace, size_t workspace_bytes,
                                   void* stream_) {
  CHECK(check_ptr(rope_cos, "rope_cos", true));
  CHECK(check_ptr(rope_sin, "rope_sin", true));
  return decode_attn_scores(L, batch, seq_len, q_heads, k_codes, k_scales, Khat_prev, q, rope_cos, rope_sin, score_scale,
                            scores, Khat_out, workspace, workspace_bytes, stream_, kFormDefinition);
}

}  // extern "C"
