// Fused predictor kernels (bf16): the prediction never leaves the chip.
//
// Alg. "encode" / "decode" of the AQUA-KV paper apply the linear predictor of Sect. 3.2 and
// then the backbone quantizer of Sect. 2 (or its inverse) to the same rows.  One workgroup
// (8 wavefronts) computes a 256-row x 128-column tile of the prediction on the matrix cores -- 128 columns
// are exactly one kv head = one rotation group per row -- parks it in LDS in fp32, and runs
// the quantizer (encode), its inverse (decode), its inverse plus the grouped-query q.k
// dot products (scores), or its inverse plus the weighted sum over the tile's tokens that the
// value side of attention needs (weighted), on those 256 groups as the epilogue.  Against separate kernels this
// saves writing and re-reading 4 bytes per value of fp32 predictions and a launch.
//
// Arithmetic is the same as in the stand-alone kernels (same main loop, same group bodies,
// prediction carried in fp32), so fused and unfused paths give identical bits.
#include "fused_epilogue.h"
#include "gemm_core.h"
#include "kernels.h"

namespace aquakv {
namespace {

static_assert(BN == kGroup, "a tile column block is one rotation group");
constexpr int kPredBytes = BM * kLdP * 4;           // the parked tile (layout: fused_epilogue.h): 135168
// LDS use over time: the main loop's ring of k-tiles (3 x 48 KiB), then the grid and the cell table (at the start
// of the array, so that a grid point's slot is its LDS address) followed by the parked prediction tile, all written
// once the main loop is done.
constexpr int kEpilogueLdsBytes = kPredBytes + (int)sizeof(Lds);
constexpr int kFusedLdsBytes = kEpilogueLdsBytes > kMainLoopLdsBytes ? kEpilogueLdsBytes : kMainLoopLdsBytes;
static_assert(kFusedLdsBytes <= 160 * 1024, "LDS of one CU");

enum Mode : int { kEncode = 0, kDecode = 1, kScores = 2, kWeighted = 3 };

// kWeighted: a wave keeps the bf16 values it decodes (32 token rows x 128) in the part of its parked rows it has
// already consumed, one row every kVRowBytes (264 B: rows 8 apart then sit 16 banks apart, which makes the
// token-strided 2-byte reads of the matrix-core operand conflict free), followed by its share of the sums
// (16 head slots x 128 fp32) and, in the soft-max form, three rows of 16 head-slot statistics.
constexpr int kVRowBytes = kGroup * 2 + 8;
constexpr int kVBufBytes = 32 * kVRowBytes;          // 8448 = exactly 16 parked rows
static_assert(kVBufBytes == 16 * kLdP * 4, "the decoded rows of both passes fill the first pass's parked rows");
constexpr int kStatBytes = kVBufBytes + 16 * kGroup * 4;    // wave's maxima [16], weight sums [16], tile maxima [16] (wave 0)
static_assert(kStatBytes + 3 * 16 * 4 <= 32 * kLdP * 4, "sums and statistics fit behind the decoded rows");
typedef unsigned int u32x2_alias __attribute__((ext_vector_type(2), may_alias));
typedef unsigned short u16_alias __attribute__((may_alias));
typedef float f32_alias __attribute__((may_alias));

// WIDE (decode, scores, weighted; 8 heads): rotation groups of 1024 = the whole token.  The tile is still one head of
// 256 tokens, so the inverse rotation's stages across the heads are taken on the grid points of all 8 heads, which
// the lane fetches itself, added in the tree the stand-alone kernels use (Rot<true>::iwht), before its own 128-point
// stages; the round-to-nearest backbone has no rotation and only reads its step and zero point per token.
template <int NCW, int MODE, int WAVES, bool WIDE = false>
__global__ __launch_bounds__(WAVES * 64) void fused_kernel(
    const bf16_t* __restrict__ x0, int d0, const bf16_t* __restrict__ x1, int d1, const bf16_t* __restrict__ W,
    const float* __restrict__ bias, const int8_t* __restrict__ signs, const float* __restrict__ codebook,
    const uint32_t* __restrict__ table, const bf16_t* X, uint8_t* codes, uint16_t* scales, bf16_t* Xhat,
    const bf16_t* __restrict__ qv, float score_scale, float* __restrict__ scores, int seq_len, int q_heads, int64_t T,
    int D, const float* __restrict__ rope_cos, const float* __restrict__ rope_sin, const float* __restrict__ weights,
    float* __restrict__ part) {
  static_assert(!WIDE || MODE != kEncode, "the quantizer needs the whole group: groups across the heads are not fused");
  __shared__ __attribute__((aligned(16))) unsigned char smem[kFusedLdsBytes];
  Lds& cl = *reinterpret_cast<Lds*>(smem);
  unsigned char* const park = smem + sizeof(Lds);          // the parked tile, each wave its own rows
  const bool use_table = MODE == kEncode && table != nullptr;
  // grid and cell table: requested now, kept in registers while the main loop owns the LDS
  static_assert(NCW <= WAVES * 64, "one grid point per thread");
  constexpr int kGridPoints = is_rtn(NCW) ? 0 : NCW;
  float cb_a = 0.f, cb_b = 0.f;
  TableRegs<WAVES * 64> table_regs;
  if (threadIdx.x < kGridPoints) { cb_a = codebook[2 * threadIdx.x]; cb_b = codebook[2 * threadIdx.x + 1]; }
  if (use_table) table_regs.request(table);
  const auto stage_tables = [&] {
    if (threadIdx.x < kGridPoints) cl.cb[threadIdx.x] = make_float4(cb_a, cb_b, -0.5f * (cb_a * cb_a + cb_b * cb_b), 0.f);
    if (use_table) table_regs.store(cl.table);
  };

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int H = D / BN;
  const int logical = remap_block(blockIdx.x, gridDim.x);
  const int tile_m = logical / H, head = logical % H;
  const int64_t m0 = (int64_t)tile_m * BM;
  const int n0 = head * BN;

  constexpr int MI = BM / WAVES / 32;              // 32-row blocks per wave
  constexpr int kRowsPerWave = MI * 32;
  const int q = lane & 3;                          // position in the quad that owns a group
  QueryStage queries = {};                         // scores: the queries of the tile's kv head, via LDS (no cell table in that mode)
  if constexpr (MODE == kScores) queries.request(qv, m0, BM, T, seq_len, q_heads, head * (q_heads / H), q_heads / H);

  // What the epilogue reads from global memory (rows to quantize, or codes and scales) is
  // requested from inside the main loop, when its own last operand loads are out, so the
  // latency is covered by the remaining MFMA work.
  struct In { u32x4 x[4]; CodeWords w; };
  constexpr int kPasses = kRowsPerWave / 16;          // passes of 16 groups per wave, one group per quad
  In in[kPasses];
  const auto fetch = [&](int pass, In& in) {
    int64_t row = m0 + wave * kRowsPerWave + pass * 16 + (lane >> 2);
    row = row < T ? row : T - 1;
    if constexpr (MODE == kEncode) {
      const u32x4* src = reinterpret_cast<const u32x4*>(X + row * D + n0 + q * kValsPerLane);
#pragma unroll
      for (int k = 0; k < 4; ++k) in.x[k] = src[k];
    } else {
      const int64_t gid = row * H + head;
      in.w = request_words<NCW, WIDE>(codes, scales, gid, q);
    }
  };
  // WIDE, grids: the code bytes of this lane's 16 sub-vector slots in each of the 8 heads of its token
  constexpr bool kWideGrid = WIDE && !is_rtn(NCW);
  const auto fetch_wide = [&](int pass, WideCodes<NCW>& wc) {
    int64_t row = m0 + wave * kRowsPerWave + pass * 16 + (lane >> 2);
    row = row < T ? row : T - 1;
    request_wide_codes<NCW>(codes, row, q, wc);
  };
  WideCodes<NCW> wide_codes;                             // of the pass at hand; the next pass's are fetched while it runs

  // kWeighted: the attention weights of query head slot lane % 16 (of this kv head) for 8 of the wave's 32 token rows,
  // in the layout of the A operand of the 16x16x32 matrix instruction; slots beyond the group's heads stay zero.
  // The launcher guarantees seq_len % BM == 0, so a tile lies inside one sequence and has no rows beyond T.
  u32x4 wreg[2] = {};
  f32x16 acc[MI][4];
  gemm_mainloop<WAVES>(smem, x0, d0, x1, d1, W, T, m0, n0, acc, [&] {
#pragma unroll
    for (int pass = 0; pass < kPasses; ++pass) fetch(pass, in[pass]);
    if constexpr (kWideGrid) fetch_wide(0, wide_codes);
    if constexpr (MODE == kWeighted) {
      static_assert(MODE != kWeighted || kRowsPerWave == 32, "one 32-token contraction per wave");
      const int rep = q_heads / H, slot = lane & 15;
      if (slot < rep) {
        const int64_t r0 = m0 + wave * kRowsPerWave + 8 * (lane >> 4);
        const int64_t b = r0 / seq_len, t = r0 % seq_len;
        const u32x4* src = reinterpret_cast<const u32x4*>(weights + (b * q_heads + head * rep + slot) * seq_len + t);
        wreg[0] = src[0]; wreg[1] = src[1];
      }
    }
  });

  // the LDS is free again: grid and table, then the tile (+ bias) parked row-major in fp32, each wave its own rows
  stage_tables();
  float* const q_lds = reinterpret_cast<float*>(cl.table);
  if constexpr (MODE == kScores) queries.store(q_lds, q_heads / H);
  float* wl = reinterpret_cast<float*>(park) + wave * kRowsPerWave * kLdP;
  {
    float bv[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) bv[j] = bias != nullptr ? bias[n0 + j * 32 + (lane & 31)] : 0.f;
#pragma unroll
    for (int i = 0; i < MI; ++i) park_block(wl + i * 32 * kLdP, acc[i], bv, lane);
  }
  __syncthreads();

  // Epilogue: passes of 16 groups per wave, one group per quad.
  float sf[32] = {};
  if constexpr (!is_rtn(NCW)) load_signs(signs, head, q, sf);
  // one pass: 16 groups of this wave (rows pass*16 .. +15), inputs already in `in`
  const auto do_pass = [&](int pass, const In& in) {
    const int lrow = pass * 16 + (lane >> 2);
    const int64_t row = m0 + wave * kRowsPerWave + lrow;
    const bool active = row < T;
    const int64_t rowc = active ? row : T - 1;
    const int64_t gid = rowc * H + head;
    const int64_t off = rowc * D + n0 + q * kValsPerLane;
    float p[32], v[32];
    read_parked(wl + lrow * kLdP, q, p);
    if constexpr (MODE == kEncode) {
#pragma unroll
      for (int k = 0; k < 4; ++k) unpack_bf16x8(in.x[k], &v[8 * k]);
      quantize_group<NCW>(v, p, sf, q, cl.cb, use_table ? cl.table : nullptr, active, gid, codes, scales,
                          Xhat != nullptr);
      if (Xhat != nullptr && active) Storage<bf16_t>::store32(Xhat + off, v);
    } else {
      if constexpr (!WIDE || is_rtn(NCW)) {
        dequantize_words<NCW>(in.w, p, sf, q, cl.cb, v);
      } else {
        const WideCodes<NCW> wc = wide_codes;
        if (pass + 1 < kPasses) fetch_wide(pass + 1, wide_codes);
        dequantize_across_heads<NCW>(wc, in.w.scale, head, q, p, sf, cl.cb, v);
      }
      if (Xhat != nullptr && active) Storage<bf16_t>::store32(Xhat + off, v);
      if constexpr (MODE == kWeighted) {
        // every parked row of this pass has been read by now (no load may sink below this point): the decoded
        // rows, rounded as they are stored, go where the first pass's rows were
        asm volatile("" ::: "memory");
        unsigned char* dst = reinterpret_cast<unsigned char*>(wl) + lrow * kVRowBytes + q * (kValsPerLane * 2);
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          u32x2_alias w2;
          w2.x = Storage<bf16_t>::pack2(v[4 * k], v[4 * k + 1]);
          w2.y = Storage<bf16_t>::pack2(v[4 * k + 2], v[4 * k + 3]);
          *reinterpret_cast<u32x2_alias*>(dst + 8 * k) = w2;
        }
      }
      if constexpr (MODE == kScores)
        score_row(v, q, head, H, q_heads, seq_len, rowc, active, qv, score_scale, scores, rope_cos, rope_sin,
                  queries.staged ? q_lds : nullptr);
    }
  };
#pragma unroll
  for (int pass = 0; pass < kPasses; ++pass) {
    do_pass(pass, in[pass]);
    __builtin_amdgcn_sched_barrier(0);
  }

  if constexpr (MODE == kWeighted) {
    // sums[slot][dim] = sum over the wave's 32 tokens of weight[slot][token] * Vhat[token][dim] on the matrix cores:
    // 16 head slots x 16 dims x 32 tokens per instruction.  The weights go in as a bf16 pair hi + lo (hi = rounded
    // weight, lo = rounded remainder), which carries 16 of their mantissa bits; the values are bf16 as stored.
    typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4v;
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_wave_barrier();
    const int rep = q_heads / H;
    // Soft-max form (pstats given): `weights` holds raw scores.  The tile's maximum per head slot is taken over the
    // 8 scores of a lane, the 4 lane groups of the slot and the 8 waves, the weights become exp(score - maximum),
    // and maximum and weight sum go out with the sums so that the tiles of a sequence can be merged afterwards.
    float* const pstats = scores;
    unsigned char* const wregion = reinterpret_cast<unsigned char*>(wl);
    float wf[8] = {__uint_as_float(wreg[0].x), __uint_as_float(wreg[0].y), __uint_as_float(wreg[0].z), __uint_as_float(wreg[0].w),
                   __uint_as_float(wreg[1].x), __uint_as_float(wreg[1].y), __uint_as_float(wreg[1].z), __uint_as_float(wreg[1].w)};
    if (pstats != nullptr) {
      float mx = fmaxf(fmaxf(fmaxf(wf[0], wf[1]), fmaxf(wf[2], wf[3])), fmaxf(fmaxf(wf[4], wf[5]), fmaxf(wf[6], wf[7])));
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      if (lane < 16) reinterpret_cast<f32_alias*>(wregion + kStatBytes)[lane] = mx;
      __syncthreads();
      float mt = -INFINITY;
#pragma unroll
      for (int w = 0; w < WAVES; ++w)
        mt = fmaxf(mt, reinterpret_cast<const f32_alias*>(park + (size_t)w * kRowsPerWave * kLdP * 4 + kStatBytes)[lane & 15]);
      if (wave == 0 && lane < 16) reinterpret_cast<f32_alias*>(wregion + kStatBytes + 128)[lane] = mt;
#pragma unroll
      for (int j = 0; j < 8; ++j) wf[j] = expf(wf[j] - mt);
    }
    u32x4 whi, wlo;
    {
      uint32_t hi[4], lo[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float a = wf[2 * j], b = wf[2 * j + 1];
        hi[j] = Storage<bf16_t>::pack2(a, b);
        lo[j] = Storage<bf16_t>::pack2(a - __uint_as_float(hi[j] << 16), b - __uint_as_float(hi[j] & 0xffff0000u));
      }
      whi.x = hi[0]; whi.y = hi[1]; whi.z = hi[2]; whi.w = hi[3];
      wlo.x = lo[0]; wlo.y = lo[1]; wlo.z = lo[2]; wlo.w = lo[3];
    }
    const bf16x8 a_hi = __builtin_bit_cast(bf16x8, whi), a_lo = __builtin_bit_cast(bf16x8, wlo);
    const int n = lane & 15, kg = lane >> 4;
    const unsigned char* vb = reinterpret_cast<const unsigned char*>(wl) + kg * 8 * kVRowBytes + n * 2;
    f32_alias* red = reinterpret_cast<f32_alias*>(reinterpret_cast<unsigned char*>(wl) + kVBufBytes);
#pragma unroll
    for (int nb = 0; nb < kGroup / 16; ++nb) {
      u32x4 bw;
      uint32_t bq[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t e0 = *reinterpret_cast<const u16_alias*>(vb + (2 * j) * kVRowBytes + nb * 32);
        const uint32_t e1 = *reinterpret_cast<const u16_alias*>(vb + (2 * j + 1) * kVRowBytes + nb * 32);
        bq[j] = e0 | (e1 << 16);
      }
      bw.x = bq[0]; bw.y = bq[1]; bw.z = bq[2]; bw.w = bq[3];
      const bf16x8 bfrag = __builtin_bit_cast(bf16x8, bw);
      f32x4v c = {0.f, 0.f, 0.f, 0.f};
      c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a_lo, bfrag, c, 0, 0, 0);
      c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a_hi, bfrag, c, 0, 0, 0);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        red[(4 * kg + r) * kGroup + nb * 16 + n] = c[r];     // row 4 kg + r of the product; rows beyond rep are unused
      }
    }
    if (pstats != nullptr) {
      // sum of the wave's weights per head slot: one more block against a column of ones
      u32x4 one;
      one.x = one.y = one.z = one.w = 0x3F803F80u;
      const bf16x8 ones = __builtin_bit_cast(bf16x8, one);
      f32x4v c = {0.f, 0.f, 0.f, 0.f};
      c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a_lo, ones, c, 0, 0, 0);
      c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a_hi, ones, c, 0, 0, 0);
      if (n == 0) {
#pragma unroll
        for (int r = 0; r < 4; ++r) reinterpret_cast<f32_alias*>(wregion + kStatBytes + 64)[4 * kg + r] = c[r];
      }
    }
    __syncthreads();
    // the tile's sums: the 8 waves' shares added in wave order
    for (int idx = threadIdx.x; idx < rep * kGroup; idx += WAVES * 64) {
      float sum = 0.f;
#pragma unroll
      for (int w = 0; w < WAVES; ++w)
        sum += *reinterpret_cast<const f32_alias*>(park + (size_t)w * kRowsPerWave * kLdP * 4 + kVBufBytes + idx * 4);
      part[((int64_t)tile_m * q_heads + head * rep + idx / kGroup) * kGroup + idx % kGroup] = sum;
    }
    if (pstats != nullptr && (int)threadIdx.x < rep) {
      float l = 0.f;
#pragma unroll
      for (int w = 0; w < WAVES; ++w)
        l += reinterpret_cast<const f32_alias*>(park + (size_t)w * kRowsPerWave * kLdP * 4 + kStatBytes + 64)[threadIdx.x];
      float* dst = pstats + ((int64_t)tile_m * q_heads + head * rep + threadIdx.x) * 2;
      dst[0] = reinterpret_cast<const f32_alias*>(park + kStatBytes + 128)[threadIdx.x];
      dst[1] = l;
    }
  }
}

// n_codewords: the quantizer id (grid size, or kRtn2 / kRtn4)
template <int MODE>
hipError_t launch(int n_codewords, const void* x0, int d0, const void* x1, int d1, const void* W, const float* bias,
                  const int8_t* signs, const float* codebook, const void* table, const void* X, uint8_t* codes,
                  uint16_t* scales, void* Xhat, const void* q, float score_scale, float* scores, int seq_len,
                  int q_heads, int64_t T, int D, const float* rope_cos, const float* rope_sin, const float* weights,
                  float* part, bool wide, hipStream_t stream) {
  if (T == 0) return hipSuccess;
  if (wide && (MODE == kEncode || D != 8 * BN)) return hipErrorInvalidValue;
  const unsigned blocks = (unsigned)(((T + BM - 1) / BM) * (D / BN));
  // 8 wavefronts per tile (two per SIMD): the main loop is bound by L2 -> LDS traffic either
  // way, and the second wave fills the issue slots the first leaves in the VALU-heavy epilogue
  // (measured: encode 10 % faster than with 4 wavefronts, decode unchanged).
#ifndef AQUAKV_FUSED_WAVES
#define AQUAKV_FUSED_WAVES 8
#endif
  constexpr int kWaves = AQUAKV_FUSED_WAVES;
#define AQUAKV_FUSED_W(N, WIDE)                                                                                  \
  fused_kernel<N, MODE, kWaves, WIDE><<<blocks, kWaves * 64, 0, stream>>>(                                       \
      static_cast<const bf16_t*>(x0), d0, static_cast<const bf16_t*>(x1), d1, static_cast<const bf16_t*>(W), bias, \
      signs, codebook, static_cast<const uint32_t*>(table), static_cast<const bf16_t*>(X), codes, scales,         \
      static_cast<bf16_t*>(Xhat), static_cast<const bf16_t*>(q), score_scale, scores, seq_len, q_heads, T, D, rope_cos,  \
      rope_sin, weights, part)
#define AQUAKV_FUSED(N)                                            \
  do {                                                             \
    if constexpr (MODE != kEncode) {                               \
      if (wide) { AQUAKV_FUSED_W(N, true); break; }                \
    }                                                              \
    AQUAKV_FUSED_W(N, false);                                      \
  } while (0)
  if (n_codewords == kRtn2) AQUAKV_FUSED(kRtn2);
  else if (n_codewords == kRtn4) AQUAKV_FUSED(kRtn4);
  else if (n_codewords == 16) AQUAKV_FUSED(16);
  else if (n_codewords == 64) AQUAKV_FUSED(64);
  else AQUAKV_FUSED(256);
#undef AQUAKV_FUSED
#undef AQUAKV_FUSED_W
  return hipGetLastError();
}

}  // namespace

hipError_t launch_fused_encode(int n_codewords, const void* x0, int d0, const void* x1, int d1, const void* W,
                               const float* bias, const int8_t* signs, const float* codebook, const void* table,
                               const void* X, uint8_t* codes, uint16_t* scales, void* Xhat, int64_t T, int D,
                               hipStream_t stream) {
  if (two_heads_pays(T, D))
    return launch_fused_encode_two_heads(n_codewords, x0, d0, x1, d1, W, bias, signs, codebook, table, X, codes, scales,
                                         Xhat, T, D, stream);
  return launch<kEncode>(n_codewords, x0, d0, x1, d1, W, bias, signs, codebook, table, X, codes, scales, Xhat, nullptr,
                         0.f, nullptr, 1, 1, T, D, nullptr, nullptr, nullptr, nullptr, false, stream);
}

hipError_t launch_fused_decode(int n_codewords, const void* x0, int d0, const void* x1, int d1, const void* W,
                               const float* bias, const int8_t* signs, const float* codebook, const uint8_t* codes,
                               const uint16_t* scales, void* Xhat, int64_t T, int D, bool wide, hipStream_t stream) {
  if (two_heads_pays(T, D))
    return launch_fused_decode_two_heads(n_codewords, x0, d0, x1, d1, W, bias, signs, codebook, codes, scales, Xhat, T, D,
                                         wide, stream);
  return launch<kDecode>(n_codewords, x0, d0, x1, d1, W, bias, signs, codebook, nullptr, nullptr,
                         const_cast<uint8_t*>(codes), const_cast<uint16_t*>(scales), Xhat, nullptr, 0.f, nullptr, 1, 1,
                         T, D, nullptr, nullptr, nullptr, nullptr, wide, stream);
}

hipError_t launch_fused_scores(int n_codewords, const void* x0, int d0, const void* W, const float* bias,
                               const int8_t* signs, const float* codebook, const uint8_t* codes,
                               const uint16_t* scales, const void* q, float score_scale, float* scores, void* Khat_out,
                               int seq_len, int q_heads, int64_t T, int D, const float* rope_cos, const float* rope_sin,
                               bool wide, hipStream_t stream) {
  // (groups across the heads: the scoring variant of the large tile spills and is slower than this one, 120 against 109 us)
  if (!wide && two_heads_pays(T, D))
    return launch_fused_scores_two_heads(n_codewords, x0, d0, W, bias, signs, codebook, codes, scales, q, score_scale,
                                         scores, Khat_out, seq_len, q_heads, T, D, rope_cos, rope_sin, stream);
  return launch<kScores>(n_codewords, x0, d0, nullptr, 0, W, bias, signs, codebook, nullptr, nullptr,
                         const_cast<uint8_t*>(codes), const_cast<uint16_t*>(scales), Khat_out, q, score_scale, scores,
                         seq_len, q_heads, T, D, rope_cos, rope_sin, nullptr, nullptr, wide, stream);
}

hipError_t launch_fused_weighted(int n_codewords, const void* x0, int d0, const void* x1, int d1, const void* W,
                                 const float* bias, const int8_t* signs, const float* codebook, const uint8_t* codes,
                                 const uint16_t* scales, void* Xhat, const float* weights, float* part, float* pstats,
                                 int seq_len, int q_heads, int64_t T, int D, bool wide, hipStream_t stream) {
  // pstats travels in the kernel's `scores` argument, which this mode does not use otherwise
  return launch<kWeighted>(n_codewords, x0, d0, x1, d1, W, bias, signs, codebook, nullptr, nullptr,
                           const_cast<uint8_t*>(codes), const_cast<uint16_t*>(scales), Xhat, nullptr, 0.f, pstats,
                           seq_len, q_heads, T, D, nullptr, nullptr, weights, part, wide, stream);
}

}  // namespace aquakv
