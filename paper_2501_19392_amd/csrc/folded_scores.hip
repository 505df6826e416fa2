// q.k scoring straight from the compressed cache with the key predictor folded into the query.
//
// Alg. "decode" of the AQUA-KV paper reconstructs a key as  Khat = Khat_prev W^T + b + Q^-1(codes)
// (Sect. 3.2 predictor, Sect. 2 backbone quantizer).  A score is linear in the key, so
//
//   q . Khat[t] = Khat_prev[t] . (W_h^T q)  +  q . b_h  +  sigma[t] * (R q) . C[codes[t]]
//
// with W_h / b_h the 128 predictor rows / bias entries of the query's kv head, R q = H (s * q) / sqrt(g)
// the rotated query (q . s*(H z)/sqrt(g) = (H (s*q))/sqrt(g) . z, H symmetric) and C[codes] the 64 grid
// points of the group.  Per token that is a 1024-long dot product per query head (instead of the
// 1024 x 1024 predictor product) and 64 table look-ups per kv head (instead of an inverse transform),
// so the call is bound by reading Khat_prev and the codes once: 2 KiB + 272 B per token.
//
// Two kernels.  `fold_query_kernel` (one small launch per call) computes, per batch entry and query
// head, u = W_h^T q in fp32 and splits it into bf16 high and low parts (the pair carries 16 mantissa
// bits, so the matrix cores can take it without a visible rounding), the rotated query and q . b.
// `folded_scores_kernel` streams tiles of 32 tokens: the 8 wavefronts of a workgroup each own 128 of
// the 1024 input channels and keep their slice of u in registers as MFMA operands for the whole
// kernel; a token tile goes from global memory straight into LDS (double buffered), every wave
// multiplies its slice (32 query heads x 32 tokens x 128 channels, high and low part into one
// accumulator).  The code term is a matrix product too: wave h multiplies the rotated queries of kv
// head h by the group's 64 grid points (looked up in LDS, fp16 operands: a correction term) and scales
// the result by the group's sigma.  The 8 partial tiles are added in a fixed order through LDS.
// Nothing but the scores is written.
//
// A pass handles up to 4 query heads per kv head (32 rows = one MFMA block).  Models with more (8 query heads
// per kv head) take two passes over the cache, pass p scoring query heads 4 p ... 4 p + 3 of every kv head.
#include "codec_core.h"
#include "gemm_core.h"
#include "kernels.h"

namespace aquakv {
namespace {

constexpr int kFoldK = 1024;                    // predictor input channels (8 waves x 128)
constexpr int kFoldQ = 32;                      // query heads per call (one MFMA block of rows)
constexpr int kTokTile = 32;                    // tokens per tile (one MFMA block of columns)
constexpr int kUFragBytes = 1024;               // one MFMA operand of u: 64 lanes x 8 bf16
constexpr int kUBytesPerBatch = 8 * 2 * 8 * kUFragBytes;      // [wave][high, low][k step] = 128 KiB

// workspace layout per batch entry: u operands, rotated queries [32][128] fp32, q . b [32] fp32
constexpr size_t kFoldBytesPerBatch = (size_t)kUBytesPerBatch + kFoldQ * 128 * 4 + kFoldQ * 4;
static_assert(kFoldBytesPerBatch == kFoldedBytesPerBatch, "the size the C-ABI layer plans with");

// ------------------------------------------------------------------ query folding
// grid = batch * kv_heads * 8, 256 threads: block (b, h, cc) owns input channels 128 cc ... + 127 for the
// query heads of kv head h.  Thread (cg, dp) multiplies 8 consecutive channels by 8 of the 128 predictor
// rows (one 128-bit load per row, all in flight at once); the 16 row groups are added in a fixed order
// through LDS.  Blocks with cc == 0 also write q . b and the rotated queries.
constexpr int kFoldChunks = 8;
__global__ __launch_bounds__(256) void fold_query_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ W,
                                                         const float* __restrict__ bias,
                                                         const int8_t* __restrict__ signs, unsigned char* ws,
                                                         int q_heads, int kv_heads, int r0, int rep) {
  // q_heads: query heads of the model; this pass takes query heads r0 ... r0 + rep - 1 (rep <= 4) of every kv head
  // and numbers them h * rep + r ("row" below)
  __shared__ float qs[4][128];
  __shared__ float part[16][4][128 + 4];
  const int cc = blockIdx.x % kFoldChunks;
  const int bh = blockIdx.x / kFoldChunks;
  const int b = bh / kv_heads, h = bh % kv_heads;
  const int rep_model = q_heads / kv_heads;
  const int rows = kv_heads * rep;               // rows of this pass that exist
  const int tid = threadIdx.x;
  const int cg = tid & 15, dp = tid >> 4;
  // predictor rows 8 dp ... + 7 of this head, channels 128 cc + 8 cg ... + 7
  u32x4 wraw[8];
  const bf16_t* Wc = W + ((size_t)h * 128 + dp * 8) * kFoldK + cc * 128 + cg * 8;
#pragma unroll
  for (int d = 0; d < 8; ++d) wraw[d] = *reinterpret_cast<const u32x4*>(Wc + (size_t)d * kFoldK);
  for (int e = tid; e < rep * 128; e += 256)
    qs[e >> 7][e & 127] = static_cast<float>(q[((size_t)b * q_heads + h * rep_model + r0 + (e >> 7)) * 128 + (e & 127)]);
  __syncthreads();

  unsigned char* wsb = ws + (size_t)b * kFoldBytesPerBatch;
  bf16_t* U = reinterpret_cast<bf16_t*>(wsb);
  float* qrot = reinterpret_cast<float*>(wsb + kUBytesPerBatch);
  float* cdot = qrot + kFoldQ * 128;

  // partial u[r][i] = sum over this thread's 8 rows d (ascending) of q[r][d] * W[h * 128 + d][i], fp32
  float acc[4][8];
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int k = 0; k < 8; ++k) acc[r][k] = 0.f;
#pragma unroll
  for (int d = 0; d < 8; ++d) {
    float w[8];
    unpack_bf16x8(wraw[d], w);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      if (r < rep) {
        const float qv = qs[r][dp * 8 + d];
#pragma unroll
        for (int k = 0; k < 8; ++k) acc[r][k] = __fmaf_rn(qv, w[k], acc[r][k]);
      }
    }
  }
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int k = 0; k < 8; ++k) part[dp][r][cg * 8 + k] = acc[r][k];
  __syncthreads();
  {
    // thread (channel, half) finishes query heads r = half, half + 2: row groups added in ascending order
    const int col = tid & 127, half = tid >> 7;
    // operand layout: [wave = i / 128][high, low][k step = (i % 128) / 16][lane = head + 32 * ((i % 16) / 8)][i % 8]
    const int ks = col >> 4, khalf = (col & 15) >> 3, e = col & 7;
    const size_t frag = ((size_t)(cc * 2 + 0) * 8 + ks) * (kUFragBytes / 2);
    const size_t lo_off = 8 * (kUFragBytes / 2);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      if (r < rep && (r & 1) == half) {
        float uv = 0.f;
#pragma unroll
        for (int g = 0; g < 16; ++g) uv += part[g][r][col];
        const bf16_t hi = static_cast<bf16_t>(uv);
        const bf16_t lo = static_cast<bf16_t>(uv - static_cast<float>(hi));
        const size_t pos = (size_t)(h * rep + r + 32 * khalf) * 8 + e;
        U[frag + pos] = hi;
        U[frag + lo_off + pos] = lo;
      }
    }
    // rows of query heads that do not exist multiply as zero: kv head h clears rows q_heads + h, + 8, ...
    if (half == 0) {
      for (int qh = rows + h; qh < kFoldQ; qh += kv_heads) {
        const size_t pos = (size_t)(qh + 32 * khalf) * 8 + e;
        U[frag + pos] = static_cast<bf16_t>(0.f);
        U[frag + lo_off + pos] = static_cast<bf16_t>(0.f);
      }
    }
  }
  if (cc != 0) return;
  // q . b
  if (tid < rep) {
    float c = 0.f;
    if (bias != nullptr) {
#pragma unroll 16
      for (int d = 0; d < 128; ++d) c = __fmaf_rn(qs[tid][d], bias[h * 128 + d], c);
    }
    cdot[h * rep + tid] = c;
  }
  // rotated query: one quad of lanes per query head (second wave, so that it overlaps the q . b loop)
  if (tid >= 64 && tid < 64 + 4 * rep) {
    const int r = (tid - 64) >> 2, qd = tid & 3;
    float v[32];
    if (signs != nullptr) {
      float sf[32];
      load_signs(signs, h, qd, sf);
#pragma unroll
      for (int k = 0; k < 32; ++k) v[k] = qs[r][32 * qd + k] * sf[k];
      wht128(v, qd);
      const float norm = quad_sign(qd) * kRsqrtG;
#pragma unroll
      for (int k = 0; k < 32; ++k) v[k] *= norm;
    } else {                                   // backbone without a rotation: the code term multiplies q itself
#pragma unroll
      for (int k = 0; k < 32; ++k) v[k] = qs[r][32 * qd + k];
    }
#pragma unroll
    for (int k = 0; k < 32; ++k) qrot[(h * rep + r) * 128 + 32 * qd + k] = v[k];
  }
}

// code m (0..15) of the 16 codes held in the first c/2 dwords of `raw`
template <int NCW> __device__ __forceinline__ int code_of(const u32x4& raw, int m) {
  constexpr int c = CodeBits<NCW>::c;
  const uint32_t d[4] = {raw.x, raw.y, raw.z, raw.w};
  const int bit = c * m, w = bit >> 5, sh = bit & 31;
  uint32_t x = d[w] >> sh;
  if (sh + c > 32) x |= d[w + 1] << (32 - sh);
  return (int)(x & ((1u << c) - 1u));
}

// ------------------------------------------------------------------ streaming kernel
// LDS: per wave a ring of 2 slots x 8 KiB (its 128 channels of a 32-token tile: 2 sub-tiles of
// [32 rows][128 B], swizzled like the predictor main loop's tiles), the exchange area for the partial
// tiles (each wave finishes 2 of the 16 accumulator registers and receives those of the 7 others),
// and the grid.
constexpr int kSlotBytes = 2 * 4096;
constexpr int kRingBytes = 8 * 2 * kSlotBytes;                   // 128 KiB
constexpr int kRedBytes = 16 * 7 * 64 * 4;                       // 28 KiB
constexpr int kFoldLdsBytes = kRingBytes + kRedBytes + 256 * 4;
static_assert(kFoldLdsBytes <= 160 * 1024, "LDS of one CU");

template <int NCW>
__global__ __launch_bounds__(512) void folded_scores_kernel(const bf16_t* __restrict__ Khat_prev,
                                                            const uint8_t* __restrict__ codes,
                                                            const uint16_t* __restrict__ scales,
                                                            const float* __restrict__ codebook,
                                                            const unsigned char* __restrict__ ws, float score_scale,
                                                            float* __restrict__ scores, int seq_len, int q_heads,
                                                            int tiles_per_seq, int blocks_per_seq, int r0, int rep) {
  // q_heads: query heads of the model (row stride of `scores`); this pass scores query heads r0 ... r0 + rep - 1
  // (rep <= 4) of every kv head, numbered h * rep + r as in fold_query_kernel
  constexpr int c = CodeBits<NCW>::c;
  constexpr int H = 8;
  __shared__ __attribute__((aligned(16))) unsigned char smem[kFoldLdsBytes];
  float* red = reinterpret_cast<float*>(smem + kRingBytes);                        // [register][source][lane]
  uint32_t* cb_s = reinterpret_cast<uint32_t*>(smem + kRingBytes + kRedBytes);     // grid point -> (a, b) as two fp16
  typedef __attribute__((address_space(3))) unsigned char* lptr_t;
  typedef const __attribute__((address_space(1))) char* gptr_t;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int b = blockIdx.x / blocks_per_seq;
  // The workgroups of a sequence walk its tiles interleaved: workgroup j takes tiles j, j + blocks_per_seq, ...
  // so that the workgroups running at the same time read neighbouring tiles (measured 1 - 2 % over giving each
  // workgroup a contiguous range).
  const int tile0 = blockIdx.x % blocks_per_seq;
  const int tstep = blocks_per_seq;
  const int ntiles = (tiles_per_seq - tile0 + blocks_per_seq - 1) / blocks_per_seq;
  const int rows = H * rep;
  const int rep_model = q_heads / H;
  const unsigned char* wsb = ws + (size_t)b * kFoldBytesPerBatch;
  const float* qrot = reinterpret_cast<const float*>(wsb + kUBytesPerBatch);
  const float* cdot = qrot + kFoldQ * 128;
  const int ftok = lane & 31, fk = lane >> 5;               // MFMA operand lane: row / column, half of the 16 k

  // Operands kept in registers for the whole kernel, rows = query heads:
  //  u[high, low][k step]: this wave's 128 channels of W^T q;
  //  r[k step]: the rotated queries of the query heads of kv head `wave` (other rows zero) in fp16, with the
  //  128 rotated coordinates ordered so that the lanes with fk = 0 hold coordinates 0..63 and fk = 1 hold 64..127.
  // The code term is a correction to the predicted key, so fp16 (11 significant bits, against the 8 the
  // stored keys themselves have) is ample for it; the predictor term keeps 16 bits through the high / low split.
  bf16x8 u[2][8];
  f16x8 r[8];
#pragma unroll
  for (int hl = 0; hl < 2; ++hl)
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
      u[hl][ks] = *reinterpret_cast<const bf16x8*>(wsb + ((size_t)(wave * 2 + hl) * 8 + ks) * kUFragBytes + lane * 16);
  {
    const bool mine = ftok < rows && ftok / rep == wave;
    const float* src = qrot + (mine ? ftok : 0) * 128 + 64 * fk;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const f32x4 a0 = reinterpret_cast<const f32x4*>(src + 8 * ks)[0];
      const f32x4 a1 = reinterpret_cast<const f32x4*>(src + 8 * ks)[1];
      const float v[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) r[ks][e] = static_cast<_Float16>(mine ? v[e] : 0.f);
    }
  }
  if (tid < (1 << c)) {
    _Float16 a, bb;
    if constexpr (is_rtn(NCW)) {               // c bits = the codes of two consecutive values, as numbers
      a = static_cast<_Float16>((float)(tid & ((1 << (c / 2)) - 1)));
      bb = static_cast<_Float16>((float)(tid >> (c / 2)));
    } else {
      a = static_cast<_Float16>(codebook[2 * tid]);
      bb = static_cast<_Float16>(codebook[2 * tid + 1]);
    }
    cb_s[tid] = (uint32_t)__builtin_bit_cast(uint16_t, a) | ((uint32_t)__builtin_bit_cast(uint16_t, bb) << 16);
  }

  // A wave loads what it multiplies: global -> LDS directly, 8 instructions of 1 KiB per tile.  Instruction i
  // fills rows 8 (i % 4) ... + 7 of sub-tile i / 4 (channels 128 wave + 64 (i / 4) ... + 63); lane l -> row
  // l / 8, 16-byte slot l % 8, which holds chunk slot ^ ((row >> 1) & 7) of the row (the swizzle of lds_off).
  const int64_t seq_row0 = (int64_t)b * seq_len;            // first token row of this sequence
  const lptr_t lds3 = (lptr_t)smem;
  // per-lane byte offsets of the 4 row groups (row, chunk) relative to the tile's first row and the sub-tile
  auto lane_offset = [&](int g, int last) {
    const int drow = g * 8 + (lane >> 3);
    const int row = drow < last ? drow : last;
    return (uint32_t)(row * (kFoldK * 2) + (((lane & 7) ^ ((drow >> 1) & 7)) << 4));
  };
  uint32_t voff[4];
#pragma unroll
  for (int g = 0; g < 4; ++g) voff[g] = lane_offset(g, kTokTile - 1);
  auto request_tile = [&](int tile, int slot) {
    const int t0 = tile * kTokTile;
    const int last = seq_len - 1 - t0;                      // tile-local index of the last valid token (>= 0)
    const char* base = reinterpret_cast<const char*>(Khat_prev) + (seq_row0 + t0) * (kFoldK * 2) + wave * 256;
    const uint64_t ub = reinterpret_cast<uint64_t>(base);
    // (readfirstlane returns a signed int: widen through uint32_t, or the low half would be sign-extended)
    const uint32_t ub_lo = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)ub);
    const uint32_t ub_hi = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(ub >> 32));
    const gptr_t sbase = (gptr_t)(((uint64_t)ub_hi << 32) | ub_lo);
    const bool ragged = last < kTokTile - 1;                // only the last tile of a sequence
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const uint32_t off = ragged ? lane_offset(i & 3, last) : voff[i & 3];
      __builtin_amdgcn_global_load_lds(sbase + (i >> 2) * 128 + off, lds3 + ((wave * 2 + slot) * kSlotBytes + i * 1024), 16,
                                       0, 0);
    }
  };
  // The compiler does not track direct-to-LDS loads; loads complete in issue order, so "at most the 8 newest
  // outstanding" means every tile but the last requested one has landed.
  auto barrier = [&] {
    __builtin_amdgcn_s_waitcnt(0x0070 | 15 | (3 << 14));    // lgkmcnt(0): own LDS traffic done
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };

  // codes and scale of the group (token lane % 32 of a tile, kv head = wave): the half of the 64 codes that
  // belongs to rotated coordinates 64 fk ... + 63
  struct Packed { u32x4 r0, r1; uint32_t scale, scale2; };   // scale: fp16 bits; round-to-nearest: (step, zero) of both groups
  auto fetch_codes = [&](int tile, Packed& p) {
    const int t = tile * kTokTile + ftok;
    const int64_t gid = (seq_row0 + (t < seq_len ? t : seq_len - 1)) * H + wave;
    const uint8_t* src = codes + gid * (8 * c) + fk * (4 * c);
    p.r0 = u32x4{0, 0, 0, 0};
    p.r1 = u32x4{0, 0, 0, 0};
    if constexpr (c == 4) {
      const u32x4 v = *reinterpret_cast<const u32x4*>(src);
      p.r0.x = v.x; p.r0.y = v.y; p.r1.x = v.z; p.r1.y = v.w;
    } else if constexpr (c == 6) {
      const u32x2* s2 = reinterpret_cast<const u32x2*>(src);
      const u32x2 a = s2[0], bb = s2[1], cc = s2[2];
      p.r0.x = a.x; p.r0.y = a.y; p.r0.z = bb.x; p.r1.x = bb.y; p.r1.y = cc.x; p.r1.z = cc.y;
    } else {
      p.r0 = reinterpret_cast<const u32x4*>(src)[0];
      p.r1 = reinterpret_cast<const u32x4*>(src)[1];
    }
    if constexpr (is_rtn(NCW)) {
      const u32x2 m = reinterpret_cast<const u32x2*>(scales)[gid];      // (step, zero) of the head's two groups of 64
      p.scale = m.x; p.scale2 = m.y;
    } else {
      p.scale = scales[gid]; p.scale2 = 0;
    }
  };

  // pipeline: tiles it + 1 (requested one iteration ago) and, from the middle of iteration it on, it + 2 are in
  // flight while tile it is multiplied; codes are fetched two tiles ahead
  // the two query heads this lane finishes per tile (see the end of the loop) and their q . b
  const int qh0 = 8 * (wave >> 1) + 4 * fk + 2 * (wave & 1);
  const float cd0 = qh0 < rows ? cdot[qh0] : 0.f;
  const float cd1 = qh0 + 1 < rows ? cdot[qh0 + 1] : 0.f;
  // the model's query head behind a row of this pass
  const auto model_head = [&](int row) { return (row / rep) * rep_model + r0 + row % rep; };
  float* const out0 = scores + ((size_t)b * q_heads + model_head(qh0)) * seq_len;
  float* const out1 = scores + ((size_t)b * q_heads + model_head(qh0 + 1)) * seq_len;
  Packed c0, c1;
  fetch_codes(tile0, c0);
  c1 = c0;
  if (ntiles > 1) fetch_codes(tile0 + tstep, c1);
  request_tile(tile0, 0);
  if (ntiles > 1) request_tile(tile0 + tstep, 1);
  barrier();                                                // the grid is in LDS
  for (int it = 0; it < ntiles; ++it) {
    const int slot = it & 1;
    const int t0 = (tile0 + it * tstep) * kTokTile;
    const unsigned char* tile_lds = smem + (wave * 2 + slot) * kSlotBytes;
    if (it + 1 < ntiles) __builtin_amdgcn_s_waitcnt(0x0f70 | 8);          // vmcnt(8): all but the newest tile request
    else __builtin_amdgcn_s_waitcnt(0x0f70);                              // vmcnt(0)
    asm volatile("" ::: "memory");

    // predictor term: this wave's 128 channels, [32 query heads] x [32 tokens]; the operand of the next step is
    // requested before the MFMAs of the current one (sched_barrier keeps the order and with it the register count)
    f32x16 acc;
#pragma unroll
    for (int k = 0; k < 16; ++k) acc[k] = 0.f;
    auto tok_frag = [&](int ks) {
      return *reinterpret_cast<const bf16x8*>(tile_lds + (ks >> 2) * 4096 + lds_off(ftok, 2 * (ks & 3) + fk));
    };
    {
      bf16x8 tok = tok_frag(0);
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const bf16x8 cur_tok = tok;
        if (ks + 1 < 8) tok = tok_frag(ks + 1);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(u[0][ks], cur_tok, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(u[1][ks], cur_tok, acc, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    // this wave's reads of the slot have returned: refill it with tile it + 2 at once (its codes first, so that
    // the count of outstanding loads at the top of the loop still separates the tiles); the code term below
    // does not touch the slot
    Packed cn = c1;
    if (it + 2 < ntiles) fetch_codes(tile0 + (it + 2) * tstep, cn);
    __builtin_amdgcn_s_waitcnt(0x0070 | 15 | (3 << 14));    // lgkmcnt(0)
    asm volatile("" ::: "memory");
    if (it + 2 < ntiles) request_tile(tile0 + (it + 2) * tstep, slot);
    asm volatile("" ::: "memory");
    // Round-to-nearest backbone: the lane's 64 values are one group with its own step and zero point, the other half
    // of the token's head (lane ^ 32) another.  Both go into one accumulator, so the operand carries
    // (code - zero) * step / max(step of the two groups) in fp16 and the result is scaled by that maximum.
    f16x8 rtn_mul, rtn_add;
    float rtn_scale = 0.f;
    if constexpr (is_rtn(NCW)) {
      const float s_a = half_bits_to_float((uint16_t)(c0.scale & 0xffffu)), s_b = half_bits_to_float((uint16_t)(c0.scale2 & 0xffffu));
      rtn_scale = fmaxf(s_a, s_b);
      const uint32_t mine = fk ? c0.scale2 : c0.scale;
      const float ratio = rtn_scale > 0.f ? __fdiv_rn(fk ? s_b : s_a, rtn_scale) : 0.f;
      const _Float16 rh = static_cast<_Float16>(ratio);
      const _Float16 ah = static_cast<_Float16>(-(float)(mine >> 16) * static_cast<float>(rh));
#pragma unroll
      for (int e = 0; e < 8; ++e) { rtn_mul[e] = rh; rtn_add[e] = ah; }
    }
    // code term on the matrix cores: [query heads of this kv head] x [32 tokens] x [128 rotated coordinates]
    f32x16 acc_c;
#pragma unroll
    for (int k = 0; k < 16; ++k) acc_c[k] = 0.f;
    {
      // the 4 grid points of step ks for this lane: codes 4 ks ... + 3 of its 32
      auto lookup = [&](int ks) {
        const u32x4& raw = ks < 4 ? c0.r0 : c0.r1;
        return u32x4{cb_s[code_of<NCW>(raw, 4 * (ks & 3))], cb_s[code_of<NCW>(raw, 4 * (ks & 3) + 1)],
                     cb_s[code_of<NCW>(raw, 4 * (ks & 3) + 2)], cb_s[code_of<NCW>(raw, 4 * (ks & 3) + 3)]};
      };
      u32x4 pts = lookup(0);
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        f16x8 cf = __builtin_bit_cast(f16x8, pts);
        if constexpr (is_rtn(NCW)) cf = cf * rtn_mul + rtn_add;          // (code - zero) * step / max step
        if (ks + 1 < 8) pts = lookup(ks + 1);
        acc_c = __builtin_amdgcn_mfma_f32_32x32x16_f16(r[ks], cf, acc_c, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    // the lane's column is one token: the code term is scaled by that group's sigma
    const float s16 = is_rtn(NCW) ? rtn_scale : half_bits_to_float((uint16_t)c0.scale);
    c0 = c1;
    c1 = cn;

    // every wave hands the registers it does not finish itself to their owners (register k belongs to wave k / 2)
#pragma unroll
    for (int k = 0; k < 16; ++k) acc[k] = __fmaf_rn(acc_c[k], s16, acc[k]);
#pragma unroll
    for (int owner = 0; owner < 8; ++owner) {
      if (owner != wave) {
        f32x2 pr;
        pr.x = acc[2 * owner]; pr.y = acc[2 * owner + 1];
        reinterpret_cast<f32x2*>(red)[(owner * 7 + (wave < owner ? wave : wave - 1)) * 64 + lane] = pr;
      }
    }
    barrier();                                              // all partial tiles are in LDS

    // This wave finishes registers 2 wave and 2 wave + 1: register k of this lane is query head
    // 8 (k / 4) + 4 fk + k % 4 and token ftok.  Own partial first, then the 7 others in wave order.
    float dot0 = acc[0], dot1 = acc[1];
#pragma unroll
    for (int w = 1; w < 8; ++w) {
      dot0 = wave == w ? acc[2 * w] : dot0;
      dot1 = wave == w ? acc[2 * w + 1] : dot1;
    }
    const f32x2* rsrc = reinterpret_cast<const f32x2*>(red) + (wave * 7) * 64 + lane;
#pragma unroll
    for (int j = 0; j < 7; ++j) {
      const f32x2 pr = rsrc[j * 64];
      dot0 += pr.x;
      dot1 += pr.y;
    }
    if (t0 + ftok < seq_len) {
      if (qh0 < rows) out0[t0 + ftok] = (dot0 + cd0) * score_scale;
      if (qh0 + 1 < rows) out1[t0 + ftok] = (dot1 + cd1) * score_scale;
    }
    barrier();                                              // partials consumed: the exchange area may be rewritten
  }
}

}  // namespace

namespace {
constexpr int kRepPerPass = kFoldQ / 8;          // query heads per kv head in one pass
inline int passes_for(int q_heads) { return (q_heads / 8 + kRepPerPass - 1) / kRepPerPass; }
}  // namespace

size_t folded_scores_workspace_bytes(int batch, int q_heads) {
  return (size_t)passes_for(q_heads) * batch * kFoldBytesPerBatch;
}

bool folded_scores_supported(int kv_heads, int d_in_k, int q_heads) {
  return kv_heads == 8 && d_in_k == kFoldK && q_heads <= 2 * kFoldQ && q_heads % kv_heads == 0;
}

hipError_t launch_folded_scores(int n_codewords, const void* Khat_prev, const void* W, const float* bias,
                                const int8_t* signs, const float* codebook, const uint8_t* codes,
                                const uint16_t* scales, const void* q, float score_scale, float* scores, void* workspace,
                                int batch, int seq_len, int q_heads, hipStream_t stream) {
  if (batch == 0 || seq_len == 0) return hipSuccess;
  const int tiles_per_seq = (seq_len + kTokTile - 1) / kTokTile;
  // enough workgroups to fill the 256 CUs several times over; up to 32 tiles each, over which the query operands
  // loaded at kernel start are reused
  int tiles_per_block = (int)(((int64_t)tiles_per_seq * batch) / 1024);
  tiles_per_block = tiles_per_block < 1 ? 1 : tiles_per_block > 32 ? 32 : tiles_per_block;
  const int blocks_per_seq = (tiles_per_seq + tiles_per_block - 1) / tiles_per_block;
  const unsigned blocks = (unsigned)(blocks_per_seq * batch);
  const int rep_model = q_heads / 8;
#define AQUAKV_FOLDED(N)                                                                                       \
  folded_scores_kernel<N><<<blocks, 512, 0, stream>>>(static_cast<const bf16_t*>(Khat_prev), codes, scales,      \
                                                      codebook, ws, score_scale, scores, seq_len, q_heads,      \
                                                      tiles_per_seq, blocks_per_seq, r0, rep)
  for (int pass = 0; pass < passes_for(q_heads); ++pass) {
    unsigned char* ws = static_cast<unsigned char*>(workspace) + (size_t)pass * batch * kFoldBytesPerBatch;
    const int r0 = pass * kRepPerPass;
    const int rep = rep_model - r0 < kRepPerPass ? rep_model - r0 : kRepPerPass;
    fold_query_kernel<<<batch * 8 * kFoldChunks, 256, 0, stream>>>(static_cast<const bf16_t*>(q),
                                                                    static_cast<const bf16_t*>(W), bias, signs, ws,
                                                                    q_heads, 8, r0, rep);
    if (n_codewords == kRtn2) AQUAKV_FOLDED(kRtn2);
    else if (n_codewords == kRtn4) AQUAKV_FOLDED(kRtn4);
    else if (n_codewords == 16) AQUAKV_FOLDED(16);
    else if (n_codewords == 64) AQUAKV_FOLDED(64);
    else AQUAKV_FOLDED(256);
  }
#undef AQUAKV_FOLDED
  return hipGetLastError();
}

}  // namespace aquakv
