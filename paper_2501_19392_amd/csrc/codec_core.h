// Building blocks of the backbone quantizer (Sect. 2 "Vector Quantization" of the AQUA-KV
// paper) for one rotation group held by a quad of lanes x 32 values: nearest-grid-point
// search (full, or through the cell table), code packing, and the quantize / dequantize
// bodies shared by the streaming kernels and by the epilogues of the fused predictor kernels.
//
// Nearest grid point.  The definition is a search over all n grid points.  The kernels reach
// the same answer with a 64 x 64 table of square cells over [-4, 4]^2 (border cells are
// unbounded outwards): each cell lists, in ascending order, every grid point that can be
// nearest to some point of the (slightly enlarged) cell -- at most 4 (3 for n = 16), else the
// cell is marked and the lane falls back to the full search.  Only the listed points are
// scored, with the same fp32 expression and the same lowest-index tie rule as the full
// search, so both give identical codes.
//
// Inside the kernels a grid point is named by its "slot" (Slot<NCW>): for n = 16 the byte offset 16 j of its
// entry in the LDS copy of the grid, which still fits a byte of a table entry and is the address the look-up
// needs; for the larger grids the index j itself.
#pragma once
#include "device_utils.h"

namespace aquakv {

constexpr int kCells = 64;                   // table is kCells x kCells
// The cells tile [-R, R]^2 (border cells reach out to infinity).  R = 4 for the grids of 16 and 64 points.  For the
// 256-point grid R = 3.25: where the cell edges fall relative to the grid decides how many cells see more candidates than an
// entry holds, and with R = 4 twelve such cells sit where a Gaussian puts 0.9 % of its mass (so nearly every wave of 1024
// sub-vectors meets one), with R = 3.25 they hold less than 1e-5 of it.
__host__ __device__ constexpr float cell_half_range(int n) { return n == 256 ? 3.25f : 4.0f; }
__host__ __device__ constexpr float cell_scale(int n) { return kCells / (2.0f * cell_half_range(n)); }   // cells per unit
// Table layout (32-bit words): kCells * kCells cell entries, then kOvfLists overflow lists of two words each.
// A cell entry lists up to 4 candidate slots, one per byte from the lowest, ascending, the last one repeated.  A cell
// with more candidates than the kernels score per cell (3 for the 16-point grid, else 4) is CROWDED: its entry is
// crowded_entry(n, L) = 0xFF in the top byte, the largest slot (top = (n - 1) << shift) in the two middle bytes and L
// in the lowest, so that every byte the quantizer may score before it looks at the flag is a slot the grid array can
// be read at (the 16-point grid never scores the top byte, the others hold 256 entries).  L = list << shift names the
// overflow list with the cell's (up to 8) candidates, again one per byte, ascending, last repeated; L = top means no
// list (more than 8 candidates, or no list left): the full search.  An entry is crowded iff it compares >=
// crowded_threshold(n), which no ordinary entry does except, with 256 points, those that list point 255: such cells
// get an overflow list as well, and the ones that list nothing else share list 0.
constexpr int kCellWords = kCells * kCells;
constexpr int kOvfLists = 128;
constexpr int kOvfCand = 8;                  // candidates per overflow list
constexpr int kTableWords = kCellWords + 2 * kOvfLists;
__host__ __device__ constexpr int slot_shift(int n) { return n == 16 ? 4 : 0; }
__host__ __device__ constexpr uint32_t slot_top(int n) { return (uint32_t)(n - 1) << slot_shift(n); }
__host__ __device__ constexpr uint32_t crowded_threshold(int n) {
  return n == 256 ? 0xFF000000u : ((slot_top(n) + 1u) << 24);
}
__host__ __device__ constexpr uint32_t crowded_entry(int n, uint32_t L) {
  return 0xFF000000u | (slot_top(n) << 16) | (slot_top(n) << 8) | L;
}
// lists a grid of n points can name: L = list << shift must stay below top
__host__ __device__ constexpr int ovf_capacity(int n) { return n == 16 ? 15 : (n - 1 < kOvfLists ? n - 1 : kOvfLists); }

// Quantizer ids, the NCW template argument everywhere: 16 / 64 / 256 = a grid of that many points in R^2;
// kRtn2 / kRtn4 = the uniform round-to-nearest backbone with 2 / 4 bits per value (see rtn_quantize_group).
constexpr int kRtn2 = 2, kRtn4 = 4;
__host__ __device__ constexpr bool is_rtn(int id) { return id < 16; }

// c = code bits per pair of values (a lane holds 16 pairs = 4c code bytes, whatever the quantizer)
template <int NCW> struct CodeBits;
template <> struct CodeBits<kRtn2> { static constexpr int c = 4; };
template <> struct CodeBits<kRtn4> { static constexpr int c = 8; };
template <> struct CodeBits<16> { static constexpr int c = 4; };
template <> struct CodeBits<64> { static constexpr int c = 6; };
template <> struct CodeBits<256> { static constexpr int c = 8; };

// Grid in LDS as (a, b, -(a^2+b^2)/2, unused): argmin ||y - C||^2 = argmax y.C - |C|^2/2.
template <int NCW>
__device__ __forceinline__ void load_codebook(const float* __restrict__ codebook, float4* cb) {
  if constexpr (is_rtn(NCW)) return;          // no grid
  for (int j = threadIdx.x; j < NCW; j += blockDim.x) {
    const float a = codebook[2 * j], b = codebook[2 * j + 1];
    cb[j] = make_float4(a, b, -0.5f * (a * a + b * b), 0.f);
  }
}

__device__ __forceinline__ float score(float y0, float y1, const float4 c) {
  return __fmaf_rn(y0, c.x, __fmaf_rn(y1, c.y, c.z));
}

template <int NCW> struct Slot {
  static constexpr int kShift = slot_shift(NCW);            // slot = j << kShift
};
// the LDS entry of a grid point from its slot (SHIFT = 4: the slot is the byte offset itself)
template <int SHIFT> __device__ __forceinline__ float4 grid_entry(const float4* cb, int slot) {
  return *reinterpret_cast<const float4*>(reinterpret_cast<const char*>(cb) + ((uint32_t)slot << (4 - SHIFT)));
}

// Table search: score the (up to 4, ascending, last one repeated) candidates of the cell; returns the winner's slot.
// Sets `crowded` if the cell lists too many points; the caller then redoes those of the lane's
// sub-vectors from the cell's overflow list, or with the full search (rare; keeps the hot path small).
template <int NCW>
__device__ __forceinline__ int search_cell(float y0, float y1, const float4* cb, const uint32_t* table,
                                           bool& crowded) {
  constexpr int SH = Slot<NCW>::kShift;
  const float fx = __builtin_amdgcn_fmed3f(__fmaf_rn(y0, cell_scale(NCW), 0.5f * kCells), 0.0f, kCells - 0.5f);
  const float fy = __builtin_amdgcn_fmed3f(__fmaf_rn(y1, cell_scale(NCW), 0.5f * kCells), 0.0f, kCells - 0.5f);
  const uint32_t e = table[(int)fy * kCells + (int)fx];
  crowded = e >= crowded_threshold(NCW);
  int slot = e & 0xff;
  float best = score(y0, y1, grid_entry<SH>(cb, slot));
  constexpr int kCand = NCW == 16 ? 3 : 4;       // the builder marks cells of a 16-point grid with more than 3
#pragma unroll
  for (int k = 1; k < kCand; ++k) {
    const int j = (e >> (8 * k)) & 0xff;
    const float s = score(y0, y1, grid_entry<SH>(cb, j));
    const bool better = s > best;                // duplicates of the last candidate never win
    best = better ? s : best;
    slot = better ? j : slot;
  }
  return slot;
}

// Full search (the definition: all n points, lowest index wins ties) for the sub-vectors of this lane whose bit is
// set in `mask`; writes their slots (grid points in the outer, rolled loop and 8 sub-vectors at a time, so that code
// and live registers stay small).
template <int NCW>
__device__ __forceinline__ void search_full_masked(const float (&v)[32], float inv, const float4* cb, uint32_t mask,
                                                   int (&idx)[16]) {
#pragma unroll 1
  for (int half = 0; half < 2; ++half) {
    float y[16], best[8];
    int bi[8];
    const float4 c0 = cb[0];
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      // select this half's values without dynamic register indexing
      y[2 * m] = (half ? v[16 + 2 * m] : v[2 * m]) * inv;
      y[2 * m + 1] = (half ? v[16 + 2 * m + 1] : v[2 * m + 1]) * inv;
      best[m] = score(y[2 * m], y[2 * m + 1], c0);
      bi[m] = 0;
    }
#pragma unroll 1
    for (int j = 1; j < NCW; ++j) {
      const float4 cj = cb[j];
#pragma unroll
      for (int m = 0; m < 8; ++m) {
        const float s = score(y[2 * m], y[2 * m + 1], cj);
        const bool better = s > best[m];
        best[m] = better ? s : best[m];
        bi[m] = better ? (j << Slot<NCW>::kShift) : bi[m];
      }
    }
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      const bool take = (mask >> (8 * half + m)) & 1;
      if (half) idx[8 + m] = take ? bi[m] : idx[8 + m];
      else idx[m] = take ? bi[m] : idx[m];
    }
  }
}

// The sub-vectors of this lane whose bit is set in `mask` sit in crowded cells: those whose cell has an overflow list
// are decided among the list's candidates (ascending, strict comparison: the lowest index wins ties, as in the full
// search); those without get their bit in the returned mask and are left to search_full_masked.
template <int NCW>
__device__ __forceinline__ uint32_t search_overflow_masked(const float (&v)[32], float inv, const float4* cb,
                                                           const uint32_t* table, uint32_t mask, int (&idx)[16]) {
  constexpr int SH = Slot<NCW>::kShift;
  uint32_t full = 0;
#pragma unroll 1
  for (int half = 0; half < 2; ++half) {
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      const bool mine = (mask >> (8 * half + m)) & 1;
      if (__builtin_amdgcn_ballot_w64(mine) != 0) {                  // somebody in the wave
        const float y0 = (half ? v[16 + 2 * m] : v[2 * m]) * inv, y1 = (half ? v[16 + 2 * m + 1] : v[2 * m + 1]) * inv;
        const float fx = __builtin_amdgcn_fmed3f(__fmaf_rn(y0, cell_scale(NCW), 0.5f * kCells), 0.0f, kCells - 0.5f);
        const float fy = __builtin_amdgcn_fmed3f(__fmaf_rn(y1, cell_scale(NCW), 0.5f * kCells), 0.0f, kCells - 0.5f);
        const uint32_t low = table[(int)fy * kCells + (int)fx] & 0xffu;
        const bool listed = mine && low != slot_top(NCW);
        full |= (mine && !listed) ? 1u << (8 * half + m) : 0u;
        const uint32_t* list = table + kCellWords + 2 * (listed ? (int)(low >> SH) : 0);
        // two rounds of four candidates: the four grid points of a round are fetched together (a loop over single
        // candidates would wait for LDS eight times in a row); rolled, because this path is rare and its size is not
        int slot = (int)(list[0] & 0xff);
        float best = score(y0, y1, grid_entry<SH>(cb, slot));
#pragma unroll 1
        for (int rnd = 0; rnd < 2; ++rnd) {
          const uint32_t w = list[rnd];
          float4 c[4];
#pragma unroll
          for (int k = 0; k < 4; ++k) c[k] = grid_entry<SH>(cb, (int)((w >> (8 * k)) & 0xff));
#pragma unroll
          for (int k = 0; k < 4; ++k) {                     // (the first candidate again in round 0: a tie, no change)
            const float sc = score(y0, y1, c[k]);
            const bool better = sc > best;
            best = better ? sc : best;
            slot = better ? (int)((w >> (8 * k)) & 0xff) : slot;
          }
          // a list ends in repeats of its last candidate: no second round if no lane of the wave has more than four
          if (__builtin_amdgcn_ballot_w64(listed && list[1] != (w >> 24) * 0x01010101u) == 0) break;
        }
        if (half) idx[8 + m] = listed ? slot : idx[8 + m];
        else idx[m] = listed ? slot : idx[m];
      }
    }
  }
  return full;
}

// 16 codes of c bits per lane = 4c contiguous bytes of the group's little-endian bit string.  `slot`: the 16 slots.
template <int NCW>
__device__ __forceinline__ void store_codes(uint8_t* __restrict__ codes, int64_t gid, int q, const int (&slot)[16]) {
  constexpr int c = CodeBits<NCW>::c;
  constexpr int SH = Slot<NCW>::kShift;
  uint32_t* dst = reinterpret_cast<uint32_t*>(codes + gid * (kGroup / 2 * c / 8) + q * (2 * c));
  if constexpr (c == 4) {
    uint32_t d[2] = {0, 0};
#pragma unroll
    for (int m = 0; m < 16; ++m) {
      const int pos = 4 * (m & 7);                   // the index j = slot >> SH goes to bit `pos`
      d[m >> 3] |= pos >= SH ? (uint32_t)slot[m] << (pos - SH) : (uint32_t)slot[m] >> (SH - pos);
    }
    u32x2 v; v.x = d[0]; v.y = d[1];
    *reinterpret_cast<u32x2*>(dst) = v;
  } else if constexpr (c == 6) {
    static_assert(c != 6 || SH == 0, "slots of the larger grids are indices");
    uint32_t d[3] = {0, 0, 0};
#pragma unroll
    for (int m = 0; m < 16; ++m) {
      const int bit = 6 * m, w = bit >> 5, sh = bit & 31;
      d[w] |= (uint32_t)slot[m] << sh;
      if (sh > 26) d[w + 1] |= (uint32_t)slot[m] >> (32 - sh);
    }
    dst[0] = d[0]; dst[1] = d[1]; dst[2] = d[2];
  } else {
    static_assert(c != 8 || SH == 0, "slots of the larger grids are indices");
    u32x4 v;
    uint32_t d[4];
#pragma unroll
    for (int w = 0; w < 4; ++w)
      d[w] = (uint32_t)slot[4 * w] | ((uint32_t)slot[4 * w + 1] << 8) | ((uint32_t)slot[4 * w + 2] << 16) |
             ((uint32_t)slot[4 * w + 3] << 24);
    v.x = d[0]; v.y = d[1]; v.z = d[2]; v.w = d[3];
    *reinterpret_cast<u32x4*>(dst) = v;
  }
}

// the 4c code bytes of a lane, as loaded into (the first c/2 dwords of) a register quad -> 16 indices
template <int NCW>
__device__ __forceinline__ void unpack_codes(const u32x4 raw, int (&idx)[16]) {
  constexpr int c = CodeBits<NCW>::c;
  const uint32_t d[4] = {raw.x, raw.y, raw.z, raw.w};
  if constexpr (c == 4) {
#pragma unroll
    for (int m = 0; m < 16; ++m) idx[m] = (d[m >> 3] >> (4 * (m & 7))) & 15;
  } else if constexpr (c == 6) {
#pragma unroll
    for (int m = 0; m < 16; ++m) {
      const int bit = 6 * m, w = bit >> 5, sh = bit & 31;
      uint32_t x = d[w] >> sh;
      if (sh > 26) x |= d[w + 1] << (32 - sh);
      idx[m] = x & 63;
    }
  } else {
#pragma unroll
    for (int m = 0; m < 16; ++m) idx[m] = (d[m >> 2] >> (8 * (m & 3))) & 255;
  }
}

__device__ __forceinline__ float half_bits_to_float(uint16_t h) {
  return static_cast<float>(__builtin_bit_cast(_Float16, h));
}

// slots (SHIFT = Slot<NCW>::kShift) or indices (SHIFT = 0) of the lane's 16 grid points -> the points times `scale`
// (recon_scale(sigma16, lane): the input of the inverse transform)
template <int SHIFT = 0>
__device__ __forceinline__ void gather_zhat(const int (&slot)[16], float scale, const float4* cb, float (&z)[32]) {
#pragma unroll
  for (int m = 0; m < 16; ++m) {
    const float4 cw = grid_entry<SHIFT>(cb, slot[m]);
    z[2 * m] = cw.x * scale;
    z[2 * m + 1] = cw.y * scale;
  }
}

struct Lds {
  float4 cb[256];
  uint32_t table[kTableWords];
};

template <int NCW>
__device__ __forceinline__ void stage_lds(Lds& lds, const float* __restrict__ codebook,
                                          const uint32_t* __restrict__ table) {
  load_codebook<NCW>(codebook, lds.cb);
  if (table != nullptr) {
    const u32x4* src = reinterpret_cast<const u32x4*>(table);
    u32x4* dst = reinterpret_cast<u32x4*>(lds.table);
    for (int i = threadIdx.x; i < kTableWords / 4; i += blockDim.x) dst[i] = src[i];
  }
  __syncthreads();
}


// The table on its way from memory to LDS through registers (kernels that request it while their LDS is still in
// other use): 16-byte chunk t + i * THREADS for thread t.
template <int THREADS> struct TableRegs {
  static constexpr int kChunks = kTableWords / 4;
  static constexpr int kPerThread = (kChunks + THREADS - 1) / THREADS;
  u32x4 r[kPerThread];
  __device__ __forceinline__ void request(const uint32_t* __restrict__ table) {
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
      const int ch = (int)threadIdx.x + i * THREADS;
      if ((i + 1) * THREADS <= kChunks || ch < kChunks) r[i] = reinterpret_cast<const u32x4*>(table)[ch];
    }
  }
  __device__ __forceinline__ void store(uint32_t* lds_table) const {
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
      const int ch = (int)threadIdx.x + i * THREADS;
      if ((i + 1) * THREADS <= kChunks || ch < kChunks) reinterpret_cast<u32x4*>(lds_table)[ch] = r[i];
    }
  }
};

// ------------------------------------------------------------------ uniform round-to-nearest backbone
// Sect. 4.1 "Backbone quantization" of the paper: b-bit round-to-nearest with per-group normalisation, groups of
// 64 consecutive channels of a token = the 2 x 32 values of a lane pair (quad lanes 0,1 and 2,3).  Per group:
// lo = min(0, min r), hi = max(0, max r), step = (hi - lo) / (2^b - 1) stored as fp16, zero = round(-lo / step),
// code = clamp(round(r / step) + zero, 0, 2^b - 1) with the stored step, rounding half to even.  Stored per
// group: (fp16 step, 16-bit zero point), i.e. `scales` holds two uint16 per group, [T, H, 2 groups, 2].
// Codes: b bits per value in channel order, little-endian: the lane's 32 values are 4b contiguous bytes.
template <int BITS>
__device__ __forceinline__ void rtn_store_codes(uint8_t* __restrict__ codes, int64_t gid, int q, const uint32_t (&code)[32]) {
  uint32_t* dst = reinterpret_cast<uint32_t*>(codes + gid * (kGroup * BITS / 8) + q * (4 * BITS));
  constexpr int kPerWord = 32 / BITS;
  uint32_t d[BITS] = {};
#pragma unroll
  for (int r = 0; r < 32; ++r) d[r / kPerWord] |= code[r] << (BITS * (r % kPerWord));
  if constexpr (BITS == 2) {
    u32x2 v; v.x = d[0]; v.y = d[1];
    *reinterpret_cast<u32x2*>(dst) = v;
  } else {
    u32x4 v; v.x = d[0]; v.y = d[1]; v.z = d[2]; v.w = d[3];
    *reinterpret_cast<u32x4*>(dst) = v;
  }
}

// the lane's code bytes (first BITS dwords of `raw`) and its group's (step, zero) word -> p + (code - zero) * step
template <int BITS>
__device__ __forceinline__ void rtn_reconstruct(const u32x4 raw, uint32_t meta, const float (&p)[32], float (&v)[32]) {
  const uint32_t d[4] = {raw.x, raw.y, raw.z, raw.w};
  constexpr int kPerWord = 32 / BITS;
  const float s16 = half_bits_to_float((uint16_t)(meta & 0xffffu));
  const int zero = (int)(meta >> 16);
#pragma unroll
  for (int r = 0; r < 32; ++r) {
    const int code = (int)((d[r / kPerWord] >> (BITS * (r % kPerWord))) & ((1u << BITS) - 1u));
    v[r] = __fmaf_rn((float)(code - zero), s16, p[r]);     // the product is exact: small integer x fp16
  }
}

// the (step, zero) word of the lane's group: two groups of 64 per head, or (WIDE, 8 heads) one group per token
template <bool WIDE = false>
__device__ __forceinline__ uint32_t rtn_load_meta(const uint16_t* __restrict__ scales, int64_t gid, int q) {
  return reinterpret_cast<const uint32_t*>(scales)[WIDE ? gid >> 3 : gid * 2 + (q >> 1)];
}

// Q(x - p) for the 32 values this lane holds of head group gid; same contract as quantize_group below
// (`l`: lane % 4, or with WIDE lane % 32: the group is then the whole token of 8 heads, one (step, zero) per token).
template <int BITS, bool WIDE = false>
__device__ __forceinline__ void rtn_quantize_group(float (&v)[32], const float (&p)[32], int l, bool active, int64_t gid,
                                                   uint8_t* __restrict__ codes, uint16_t* __restrict__ scales,
                                                   bool want_hat) {
  const int q = l & 3;
  constexpr float kTop = (float)((1 << BITS) - 1);
  float lo = 0.f, hi = 0.f;
#pragma unroll
  for (int r = 0; r < 32; ++r) {
    v[r] -= p[r];
    lo = fminf(lo, v[r]);
    hi = fmaxf(hi, v[r]);
  }
  lo = fminf(lo, quad_xor<1>(lo));
  hi = fmaxf(hi, quad_xor<1>(hi));
  if constexpr (WIDE) {
    lo = fminf(lo, quad_xor<2>(lo));    hi = fmaxf(hi, quad_xor<2>(hi));
    lo = fminf(lo, swizzle_xor<4>(lo)); hi = fmaxf(hi, swizzle_xor<4>(hi));
    lo = fminf(lo, row_xor8(lo));       hi = fmaxf(hi, row_xor8(hi));
    lo = fminf(lo, swizzle_xor<16>(lo)); hi = fmaxf(hi, swizzle_xor<16>(hi));
  }
  const float step = fminf(__fdiv_rn(hi - lo, kTop), 65504.0f);
  const _Float16 s16h = static_cast<_Float16>(step);      // round to nearest even
  const float s16 = static_cast<float>(s16h);
  const bool ok = s16 > 0.f;
  const float inv = ok ? __fdiv_rn(1.0f, s16) : 0.f;
  const float zf = ok ? __builtin_amdgcn_fmed3f(__builtin_rintf(__fdiv_rn(-lo, s16)), 0.f, kTop) : 0.f;
  uint32_t code[32];
#pragma unroll
  for (int r = 0; r < 32; ++r)
    code[r] = (uint32_t)__builtin_amdgcn_fmed3f(__builtin_rintf(v[r] * inv) + zf, 0.f, kTop);
  if (active) {
    rtn_store_codes<BITS>(codes, gid, q, code);
    const uint32_t word = (uint32_t)__builtin_bit_cast(uint16_t, s16h) | ((uint32_t)zf << 16);
    if constexpr (WIDE) {
      if (l == 0) reinterpret_cast<uint32_t*>(scales)[gid >> 3] = word;
    } else {
      if ((q & 1) == 0) reinterpret_cast<uint32_t*>(scales)[gid * 2 + (q >> 1)] = word;
    }
  }
  if (want_hat) {
#pragma unroll
    for (int r = 0; r < 32; ++r) v[r] = __fmaf_rn((float)code[r] - zf, s16, p[r]);
  }
}

// ------------------------------------------------------------------ group bodies
// Q(x - p) for the 32 coordinates this lane holds of head group `gid` (= token * H + head).  On entry
// v = x; on exit v holds the (unrounded) reconstruction p + Q^-1(codes) if `want_hat`.  Codes and the
// scale are stored when `active` (inactive lanes only keep the cross-lane exchanges in step).
// `l` is the lane's index inside its rotation group: lane % 4 for groups of 128 (WIDE = false, one
// scale per head group), lane % 32 for groups of 1024 = the whole token (WIDE = true, kv_heads = 8, one
// scale per token at scales[gid / 8]).  The code bytes have the same layout in both cases.
template <int NCW, bool WIDE = false>
__device__ __forceinline__ void quantize_group(float (&v)[32], const float (&p)[32], const float (&sf)[32], int l,
                                               const float4* cb, const uint32_t* table, bool active, int64_t gid,
                                               uint8_t* __restrict__ codes, uint16_t* __restrict__ scales,
                                               bool want_hat) {
  if constexpr (is_rtn(NCW)) {
    rtn_quantize_group<NCW, WIDE>(v, p, l, active, gid, codes, scales, want_hat);
    return;
  }
#pragma unroll
  for (int r = 0; r < 32; ++r) v[r] = (v[r] - p[r]) * sf[r];                              // s * (x - p), exact product
  const int q = l & 3;
  Rot<WIDE>::wht(v, l);                                   // w = +-H u (unnormalised, lane sign pending)

  float ss = 0.f;
#pragma unroll
  for (int r = 0; r < 32; ++r) ss = __fmaf_rn(v[r], v[r], ss);
  ss = Rot<WIDE>::sum(ss);
  // z = w / sqrt(g)  =>  rms(z) = sqrt(sum w^2) / g
  float sigma = __fsqrt_rn(ss) * Rot<WIDE>::kInvG;
  sigma = fminf(sigma, 65504.0f);
  const _Float16 s16h = static_cast<_Float16>(sigma);     // round to nearest even
  const float s16 = static_cast<float>(s16h);
  const float inv = s16 > 0.f ? Rot<WIDE>::sign(l) * __fdiv_rn(Rot<WIDE>::kNorm, s16) : 0.f;   // also undoes the lane sign

  int idx[16];                                            // slots (Slot<NCW>)
  if (table != nullptr) {
    uint32_t crowded_mask = 0;
#pragma unroll
    for (int m = 0; m < 16; ++m) {
      bool crowded;
      idx[m] = search_cell<NCW>(v[2 * m] * inv, v[2 * m + 1] * inv, cb, table, crowded);
      crowded_mask |= crowded ? 1u << m : 0u;
    }
    if (__builtin_expect(__builtin_amdgcn_ballot_w64(crowded_mask != 0) != 0, 0)) {
      const uint32_t full_mask = search_overflow_masked<NCW>(v, inv, cb, table, crowded_mask, idx);
      if (__builtin_amdgcn_ballot_w64(full_mask != 0) != 0) search_full_masked<NCW>(v, inv, cb, full_mask, idx);
    }
  } else {
#pragma unroll
    for (int m = 0; m < 16; ++m) idx[m] = 0;
    search_full_masked<NCW>(v, inv, cb, 0xffffu, idx);      // the definition: scan all n points
  }
  if (active) {
    store_codes<NCW>(codes, gid, q, idx);
    if (l == 0) scales[WIDE ? gid >> 3 : gid] = __builtin_bit_cast(uint16_t, s16h);
  }
  if (want_hat) {
    gather_zhat<Slot<NCW>::kShift>(idx, recon_scale<WIDE>(s16, l), cb, v);
    reconstruct<WIDE>(v, l, sf, p);
  }
}

// the lane's share of a group's codes (and of its scales) as the kernels hold them between request and use
struct CodeWords { u32x4 code; uint32_t scale; };   // scale: fp16 bits (grids) or (step, zero point) (round-to-nearest)

// requests the code bytes of quad position q of group gid (4 c bytes: the lane's 16 sub-vectors)
template <int NCW>
__device__ __forceinline__ u32x4 request_codes(const uint8_t* __restrict__ codes, int64_t gid, int q) {
  constexpr int c = CodeBits<NCW>::c;
  const uint32_t* src = reinterpret_cast<const uint32_t*>(codes + gid * (kGroup / 2 * c / 8) + q * (2 * c));
  u32x4 out = {0, 0, 0, 0};
  if constexpr (c == 4) {
    const u32x2 v2 = *reinterpret_cast<const u32x2*>(src);
    out.x = v2.x; out.y = v2.y;
  } else if constexpr (c == 6) {
    out.x = src[0]; out.y = src[1]; out.z = src[2];
  } else {
    out = *reinterpret_cast<const u32x4*>(src);
  }
  return out;
}

// the words of quad position l % 4 of head group gid (WIDE: one scale word per token, at gid / 8)
template <int NCW, bool WIDE = false>
__device__ __forceinline__ CodeWords request_words(const uint8_t* __restrict__ codes, const uint16_t* __restrict__ scales,
                                                   int64_t gid, int q) {
  CodeWords w;
  w.code = request_codes<NCW>(codes, gid, q);
  if constexpr (is_rtn(NCW)) w.scale = rtn_load_meta<WIDE>(scales, gid, q);
  else w.scale = scales[WIDE ? gid >> 3 : gid];
  return w;
}

// Q^-1(codes) + p from the words requested earlier (unrounded, in v); l: lane % 4, or with WIDE lane % 32
template <int NCW, bool WIDE = false>
__device__ __forceinline__ void dequantize_words(const CodeWords& w, const float (&p)[32], const float (&sf)[32], int l,
                                                 const float4* cb, float (&v)[32]) {
  if constexpr (is_rtn(NCW)) {
    rtn_reconstruct<NCW>(w.code, w.scale, p, v);
  } else {
    int idx[16];
    unpack_codes<NCW>(w.code, idx);
    gather_zhat(idx, recon_scale<WIDE>(half_bits_to_float((uint16_t)w.scale), l), cb, v);
    reconstruct<WIDE>(v, l, sf, p);
  }
}

}  // namespace aquakv
