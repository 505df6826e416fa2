// Fused predictor + inverse quantizer (Alg. "decode" of the AQUA-KV paper: predictor of Sect. 3.2, backbone of
// Sect. 2) on tiles of 256 token rows x 256 outputs = two kv heads: the shape for long token ranges.
//
// Same arithmetic as fused_kernels.hip (same matrix instruction and K order per output, same group bodies), hence the
// same bits; what differs is the tile.  A workgroup of 8 wavefronts multiplies 256 x 256 (main loop in
// gemm_two_heads.h: a third less L2 -> LDS traffic and 0.75 instead of 1.25 operand reads per matrix instruction),
// wave w owning the 64 token rows 64 (w / 2) ... of head w % 2 of the pair.  A wave's accumulators are two blocks of
// 32 rows; the epilogue parks one block at a time in the wave's own 32 LDS rows and decodes it in two passes of 16
// groups (one per quad of lanes), so the LDS footprint is that of the one-head kernel.
//
// Half as many, twice as large workgroups: worth it when the token range still gives every CU the same number of
// rounds (two_heads_pays).
#include "fused_epilogue.h"
#include "gemm_two_heads.h"
#include "kernels.h"

namespace aquakv {
namespace {

constexpr int kPark2Bytes = kWaves2 * 32 * kLdP * 4;                      // one 32-row block per wave: 135168
constexpr int kEpilogue2Bytes = (int)sizeof(Lds) + kPark2Bytes;
constexpr int kFused2LdsBytes = kEpilogue2Bytes > kMainLoop2LdsBytes ? kEpilogue2Bytes : kMainLoop2LdsBytes;
static_assert(kFused2LdsBytes <= 160 * 1024, "LDS of one CU");

enum Mode2 : int { kEncode2 = 0, kDecode2 = 1, kScores2 = 2 };

// WIDE (decode; 8 heads): rotation groups of 1024 = the whole token.  A wave still owns one head of its 64
// tokens, so the inverse rotation's stages across the heads are taken on the grid points of all 8 heads, which the lane
// fetches itself (fused_epilogue.h); the round-to-nearest backbone has no rotation and only reads its step and zero
// point per token.
template <int NCW, int MODE, bool WIDE = false>
__global__ __launch_bounds__(kWaves2 * 64) void fused_two_heads_kernel(
    const bf16_t* __restrict__ x0, int d0, const bf16_t* __restrict__ x1, int d1, const bf16_t* __restrict__ W,
    const float* __restrict__ bias, const int8_t* __restrict__ signs, const float* __restrict__ codebook,
    const uint32_t* __restrict__ table, const bf16_t* X, uint8_t* codes, uint16_t* scales, bf16_t* Xhat,
    const bf16_t* __restrict__ qv, float score_scale, float* __restrict__ scores, int seq_len, int q_heads, int64_t T,
    int D, const float* __restrict__ rope_cos, const float* __restrict__ rope_sin) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[kFused2LdsBytes];
  Lds& cl = *reinterpret_cast<Lds*>(smem);
  constexpr int kGridPoints = is_rtn(NCW) ? 0 : NCW;
  static_assert(kGridPoints <= kWaves2 * 64, "one grid point per thread");
  float cb_a = 0.f, cb_b = 0.f;                      // kept in registers while the main loop owns the LDS
  if ((int)threadIdx.x < kGridPoints) { cb_a = codebook[2 * threadIdx.x]; cb_b = codebook[2 * threadIdx.x + 1]; }
  const bool use_table = MODE == kEncode2 && !is_rtn(NCW) && table != nullptr;
  QueryStage queries = {};                           // scores: the queries of the tile's two kv heads, via LDS

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int H = D / kGroup, H2 = D / BN2;
  const int logical = remap_block(blockIdx.x, gridDim.x);
  const int tile_m = logical / H2, pair = logical % H2;
  const int64_t m0 = (int64_t)tile_m * BM2;
  const int head = 2 * pair + (wave & 1);            // this wave's kv head
  const int nw = head * kGroup;                      // its first output column
  const int64_t mw = m0 + (wave >> 1) * 64;          // its first token row
  const int q = lane & 3;                            // position in the quad that owns a group

  if constexpr (MODE == kScores2) queries.request(qv, m0, BM2, T, seq_len, q_heads, 2 * pair * (q_heads / H), 2 * (q_heads / H));
  constexpr bool kEnc = MODE == kEncode2;
  static_assert(!WIDE || MODE == kDecode2, "groups across the heads: only the decode variant pays on this tile");
  constexpr bool kWideGrid = WIDE && !is_rtn(NCW);
  // decode: codes and scale; encode: the 32 values of the row to quantize
  struct In { CodeWords w; u32x4 x[kEnc ? 4 : 1]; };
  constexpr int kPasses = 4;                         // 2 blocks x 2 passes of 16 groups
  In in[kEnc ? 2 : kPasses];                         // encode: this pass's and the next one's
  const auto fetch = [&](int pi, In& in) {
    int64_t row = mw + pi * 16 + (lane >> 2);
    row = row < T ? row : T - 1;
    if constexpr (kEnc) {
      const u32x4* src = reinterpret_cast<const u32x4*>(X + row * D + nw + q * kValsPerLane);
#pragma unroll
      for (int k = 0; k < 4; ++k) in.x[k] = src[k];
      return;
    }
    const int64_t gid = row * H + head;
    in.w = request_words<NCW, WIDE>(codes, scales, gid, q);
  };
  const auto fetch_wide = [&](int pi, WideCodes<NCW>& wc) {
    int64_t row = mw + pi * 16 + (lane >> 2);
    row = row < T ? row : T - 1;
    request_wide_codes<NCW>(codes, row, q, wc);
  };
  WideCodes<NCW> wide_codes;                         // of the pass at hand; the next pass's are fetched while it runs

  f32x16 acc[2][4];
  gemm_mainloop_two_heads(smem, x0, d0, x1, d1, W, T, m0, pair * BN2, acc, [&] {
    if constexpr (kEnc) {
      fetch(0, in[0]);
    } else {
#pragma unroll
      for (int pi = 0; pi < kPasses; ++pi) fetch(pi, in[pi]);
      if constexpr (kWideGrid) fetch_wide(0, wide_codes);
    }
  });

  // the LDS is free again: the grid (and the encoder's cell table, requested now and stored once the first block is
  // parked), then block after block of the tile (+ bias) parked row-major in fp32
  TableRegs<kWaves2 * 64> table_regs;
  if (use_table) table_regs.request(table);
  if ((int)threadIdx.x < kGridPoints)
    cl.cb[threadIdx.x] = make_float4(cb_a, cb_b, -0.5f * (cb_a * cb_a + cb_b * cb_b), 0.f);
  float* const q_lds = reinterpret_cast<float*>(cl.table);      // (no cell table in this mode)
  if constexpr (MODE == kScores2) {
    static_assert(MODE != kScores2 || 16 * kQueryLdsStride * 4 <= (int)sizeof(cl.table), "queries of two kv heads fit");
    queries.store(q_lds, 2 * (q_heads / H));
  }
  float* const wl = reinterpret_cast<float*>(smem + sizeof(Lds)) + wave * 32 * kLdP;
  float sf[32] = {};
  if constexpr (!is_rtn(NCW)) load_signs(signs, head, q, sf);
  float bv[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) bv[j] = bias != nullptr ? bias[nw + j * 32 + (lane & 31)] : 0.f;

#pragma unroll
  for (int blk = 0; blk < 2; ++blk) {
    park_block(wl, acc[blk], bv, lane);
    // The parked rows are the wave's own: block 1 only needs the wave's writes to have landed.  Block 0 also waits
    // for the grid, which other waves stage.
    if (blk == 0) {
      if (use_table) table_regs.store(cl.table);
      __syncthreads();
    } else {
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      __builtin_amdgcn_wave_barrier();
    }
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
      const int pi = 2 * blk + pass;
      const In ip = in[kEnc ? (pi & 1) : pi];
      if constexpr (kEnc) {
        if (pi + 1 < kPasses) fetch(pi + 1, in[(pi + 1) & 1]);      // the next pass's rows, while this one is worked on
      }
      const int lrow = pass * 16 + (lane >> 2);
      const int64_t row = mw + blk * 32 + lrow;
      const bool active = row < T;
      const int64_t rowc = active ? row : T - 1;
      const int64_t off = rowc * D + nw + q * kValsPerLane;
      const int64_t gid = rowc * H + head;
      float p[32], v[32];
      read_parked(wl + lrow * kLdP, q, p);
      if constexpr (kEnc) {
#pragma unroll
        for (int k = 0; k < 4; ++k) unpack_bf16x8(ip.x[k], &v[8 * k]);
        quantize_group<NCW>(v, p, sf, q, cl.cb, use_table ? cl.table : nullptr, active, gid, codes, scales, Xhat != nullptr);
      } else if constexpr (kWideGrid) {
        const WideCodes<NCW> wc = wide_codes;
        if (pi + 1 < kPasses) fetch_wide(pi + 1, wide_codes);
        dequantize_across_heads<NCW>(wc, ip.w.scale, head, q, p, sf, cl.cb, v);
      } else {
        dequantize_words<NCW>(ip.w, p, sf, q, cl.cb, v);
      }
      if (Xhat != nullptr && active) Storage<bf16_t>::store32(Xhat + off, v);
      if constexpr (MODE == kScores2)
        score_row(v, q, head, H, q_heads, seq_len, rowc, active, qv, score_scale, scores, rope_cos, rope_sin,
                  queries.staged ? q_lds + (wave & 1) * (q_heads / H) * kQueryLdsStride : nullptr);
      __builtin_amdgcn_sched_barrier(0);
    }
    // every lane's reads of this block have returned before the next block overwrites the rows
    if (blk == 0) {
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      __builtin_amdgcn_wave_barrier();
    }
  }
}

template <int MODE>
hipError_t launch2(int n_codewords, const void* x0, int d0, const void* x1, int d1, const void* W, const float* bias,
                   const int8_t* signs, const float* codebook, const void* table, const void* X, uint8_t* codes,
                   uint16_t* scales, void* Xhat, const void* q, float score_scale, float* scores, int seq_len, int q_heads, int64_t T, int D,
                   const float* rope_cos, const float* rope_sin, bool wide, hipStream_t stream) {
  if (T == 0) return hipSuccess;
  if (D % BN2 != 0 || (wide && (MODE != kDecode2 || D != 8 * kGroup))) return hipErrorInvalidValue;
  const unsigned blocks = (unsigned)(((T + BM2 - 1) / BM2) * (D / BN2));
#define AQUAKV_FUSED2_W(N, WIDE)                                                                                      \
  fused_two_heads_kernel<N, MODE, WIDE><<<blocks, kWaves2 * 64, 0, stream>>>(                                         \
      static_cast<const bf16_t*>(x0), d0, static_cast<const bf16_t*>(x1), d1, static_cast<const bf16_t*>(W), bias,    \
      signs, codebook, static_cast<const uint32_t*>(table), static_cast<const bf16_t*>(X), codes, scales,              \
      static_cast<bf16_t*>(Xhat), static_cast<const bf16_t*>(q), score_scale, scores, seq_len, q_heads, T, D, rope_cos, \
      rope_sin)
#define AQUAKV_FUSED2(N)                                           \
  do {                                                             \
    if constexpr (MODE == kDecode2) {                              \
      if (wide) { AQUAKV_FUSED2_W(N, true); break; }               \
    }                                                              \
    AQUAKV_FUSED2_W(N, false);                                     \
  } while (0)
  if (n_codewords == kRtn2) AQUAKV_FUSED2(kRtn2);
  else if (n_codewords == kRtn4) AQUAKV_FUSED2(kRtn4);
  else if (n_codewords == 16) AQUAKV_FUSED2(16);
  else if (n_codewords == 64) AQUAKV_FUSED2(64);
  else AQUAKV_FUSED2(256);
#undef AQUAKV_FUSED2
#undef AQUAKV_FUSED2_W
  return hipGetLastError();
}

}  // namespace

// A CU holds one workgroup of either kernel (LDS), so a launch takes ceil(tiles / CUs) rounds.  The 256 x 256 tile
// does twice the work per round at a better rate (measured 9 - 13 % on the main loop), the 256 x 128 tile wastes less
// of the last round: take the large tile when its rounds cost at most as much as the small tile's.
bool two_heads_pays(int64_t T, int D) {
  constexpr int64_t kCUs = 256;                      // MI355X
  if (D % BN2 != 0) return false;
  const int64_t big = ((T + BM2 - 1) / BM2) * (D / BN2);
  const int64_t rounds_big = (big + kCUs - 1) / kCUs, rounds_small = (2 * big + kCUs - 1) / kCUs;
  return 2 * rounds_big <= rounds_small;
}

hipError_t launch_fused_decode_two_heads(int n_codewords, const void* x0, int d0, const void* x1, int d1, const void* W,
                                         const float* bias, const int8_t* signs, const float* codebook,
                                         const uint8_t* codes, const uint16_t* scales, void* Xhat, int64_t T, int D,
                                         bool wide, hipStream_t stream) {
  return launch2<kDecode2>(n_codewords, x0, d0, x1, d1, W, bias, signs, codebook, nullptr, nullptr,
                           const_cast<uint8_t*>(codes), const_cast<uint16_t*>(scales), Xhat, nullptr, 0.f, nullptr, 1, 1, T,
                           D, nullptr, nullptr, wide, stream);
}

hipError_t launch_fused_encode_two_heads(int n_codewords, const void* x0, int d0, const void* x1, int d1, const void* W,
                                         const float* bias, const int8_t* signs, const float* codebook, const void* table,
                                         const void* X, uint8_t* codes, uint16_t* scales, void* Xhat, int64_t T, int D,
                                         hipStream_t stream) {
  return launch2<kEncode2>(n_codewords, x0, d0, x1, d1, W, bias, signs, codebook, table, X, codes, scales, Xhat, nullptr,
                           0.f, nullptr, 1, 1, T, D, nullptr, nullptr, false, stream);
}

hipError_t launch_fused_scores_two_heads(int n_codewords, const void* x0, int d0, const void* W, const float* bias,
                                         const int8_t* signs, const float* codebook, const uint8_t* codes,
                                         const uint16_t* scales, const void* q, float score_scale, float* scores,
                                         void* Khat_out, int seq_len, int q_heads, int64_t T, int D,
                                         const float* rope_cos, const float* rope_sin, hipStream_t stream) {
  return launch2<kScores2>(n_codewords, x0, d0, nullptr, 0, W, bias, signs, codebook, nullptr, nullptr,
                           const_cast<uint8_t*>(codes), const_cast<uint16_t*>(scales), Khat_out, q, score_scale, scores,
                           seq_len, q_heads, T, D, rope_cos, rope_sin, false, stream);
}

}  // namespace aquakv
