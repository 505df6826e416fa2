// Device-side helpers shared by the gfx950 streaming kernels: storage-type
// loads/stores, the 128-point Walsh-Hadamard butterfly over a quad of lanes,
// and the reconstruction tail used by quantize / dequantize / scores.
//
// Work decomposition of the streaming kernels: one rotation group (128 values
// of one token and kv head) is held by a QUAD of lanes, 32 consecutive values
// per lane (lane q owns coordinates 32q .. 32q+31).  Five of the seven
// butterfly stages then run inside a lane and only two cross lanes, both as
// DPP quad permutes that fold into the add.  Every global access is a 128-bit
// load/store and the packed codes of a lane are contiguous bytes.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace aquakv {

constexpr int kGroup = 128;          // head_dim = rotation group
constexpr int kLanesPerGroup = 4;
constexpr int kValsPerLane = 32;
constexpr float kRsqrtG = 0.088388347648318440550f;   // 1/sqrt(128)

typedef __bf16 bf16_t;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// ---------------------------------------------------------------- 32-value row access
template <typename T> struct Storage;

template <> struct Storage<float> {
  static __device__ __forceinline__ void load32(const float* p, float (&v)[32]) {
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const f32x4 a = reinterpret_cast<const f32x4*>(p)[c];
      v[4 * c] = a.x; v[4 * c + 1] = a.y; v[4 * c + 2] = a.z; v[4 * c + 3] = a.w;
    }
  }
  static __device__ __forceinline__ void store32(float* p, const float (&v)[32]) {
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      f32x4 a;
      a.x = v[4 * c]; a.y = v[4 * c + 1]; a.z = v[4 * c + 2]; a.w = v[4 * c + 3];
      reinterpret_cast<f32x4*>(p)[c] = a;
    }
  }
  static __device__ __forceinline__ float round(float x) { return x; }
};

template <> struct Storage<bf16_t> {
  static __device__ __forceinline__ void load32(const bf16_t* p, float (&v)[32]) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const u32x4 r = reinterpret_cast<const u32x4*>(p)[c];
      const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        v[8 * c + 2 * i] = __uint_as_float(w[i] << 16);
        v[8 * c + 2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
      }
    }
  }
  static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    f32x2_t f;
    f.x = lo; f.y = hi;
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));   // one packed RNE convert
  }
  static __device__ __forceinline__ void store32(bf16_t* p, const float (&v)[32]) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      u32x4 r;
      r.x = pack2(v[8 * c], v[8 * c + 1]); r.y = pack2(v[8 * c + 2], v[8 * c + 3]);
      r.z = pack2(v[8 * c + 4], v[8 * c + 5]); r.w = pack2(v[8 * c + 6], v[8 * c + 7]);
      reinterpret_cast<u32x4*>(p)[c] = r;
    }
  }
  static __device__ __forceinline__ float round(float x) {
    return static_cast<float>(static_cast<bf16_t>(x));
  }
};

// 8 bf16 in a 16-byte register quad -> fp32
__device__ __forceinline__ void unpack_bf16x8(const u32x4 r, float* v) {
  const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    v[2 * i] = __uint_as_float(w[i] << 16);
    v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
  }
}

__device__ __forceinline__ void load32_f32(const float* p, float (&v)[32]) { Storage<float>::load32(p, v); }

// ---------------------------------------------------------------- cross-lane moves inside a quad
// Value of `x` held by lane (lane ^ MASK), MASK in {1, 2}: DPP quad_perm.
template <int MASK> __device__ __forceinline__ float quad_xor(float x) {
  static_assert(MASK == 1 || MASK == 2, "mask");
  const int xi = __float_as_int(x);
  constexpr int ctrl = MASK == 1 ? 0xB1 /* [1,0,3,2] */ : 0x4E /* [2,3,0,1] */;
  return __int_as_float(__builtin_amdgcn_mov_dpp(xi, ctrl, 0xF, 0xF, true));   // folds into the consuming add
}

// Sum over the 4 lanes of a group; every lane gets the total (fixed order).
__device__ __forceinline__ float quad_sum(float x) {
  x = x + quad_xor<1>(x);
  x = x + quad_xor<2>(x);
  return x;
}

// ---------------------------------------------------------------- 128-point WHT
// v[r] is coordinate 32*q + r of the group (q = lane % 4).  Unnormalised Sylvester-order
// transform: coordinate bits 0..4 are butterflied in registers, bits 5..6 across the quad.
//
// A cross-lane butterfly wants partner + v on the lane holding the 0-bit and partner - v on
// the other.  Both lanes instead run the same multiply-add v + s * partner with a per-lane
// s = +1 / -1 (one DPP instruction per value, exact), which leaves the upper lane with the
// NEGATED result.  The sign is the same for all 32 values of a lane, passes through the
// following (linear) stage unchanged, and is handed back to the caller, who folds it into a
// multiplication it performs anyway:  true transform = quad_sign(q) * (what wht128 leaves in v).
//
// The compiler does not fold the lane permute into a multiply-add, so the stage is written as
// v_fmac_f32 with a DPP quad permute on its first source (dst += permuted(dst) * s).  A DPP
// read of a register written by the VALU instruction just before it needs two idle issue
// slots; the compiler cannot see into the block, so each block of 16 starts with them.
#define AQUAKV_FMAC_DPP(i, perm) "v_fmac_f32_dpp %" #i ", %" #i ", %16 quad_perm:" perm " row_mask:0xf bank_mask:0xf\n\t"
#define AQUAKV_FMAC_DPP16(perm)                                                                               \
  "s_nop 1\n\t" AQUAKV_FMAC_DPP(0, perm) AQUAKV_FMAC_DPP(1, perm) AQUAKV_FMAC_DPP(2, perm) AQUAKV_FMAC_DPP(3, perm)  \
  AQUAKV_FMAC_DPP(4, perm) AQUAKV_FMAC_DPP(5, perm) AQUAKV_FMAC_DPP(6, perm) AQUAKV_FMAC_DPP(7, perm)               \
  AQUAKV_FMAC_DPP(8, perm) AQUAKV_FMAC_DPP(9, perm) AQUAKV_FMAC_DPP(10, perm) AQUAKV_FMAC_DPP(11, perm)             \
  AQUAKV_FMAC_DPP(12, perm) AQUAKV_FMAC_DPP(13, perm) AQUAKV_FMAC_DPP(14, perm) AQUAKV_FMAC_DPP(15, perm)
template <int MASK> __device__ __forceinline__ void wht_quad_stage(float (&v)[32], float s) {
  static_assert(MASK == 1 || MASK == 2, "mask");
#pragma unroll
  for (int b = 0; b < 32; b += 16) {
    if constexpr (MASK == 1)
      asm(AQUAKV_FMAC_DPP16("[1,0,3,2]")
          : "+v"(v[b]), "+v"(v[b + 1]), "+v"(v[b + 2]), "+v"(v[b + 3]), "+v"(v[b + 4]), "+v"(v[b + 5]), "+v"(v[b + 6]),
            "+v"(v[b + 7]), "+v"(v[b + 8]), "+v"(v[b + 9]), "+v"(v[b + 10]), "+v"(v[b + 11]), "+v"(v[b + 12]),
            "+v"(v[b + 13]), "+v"(v[b + 14]), "+v"(v[b + 15])
          : "v"(s));
    else
      asm(AQUAKV_FMAC_DPP16("[2,3,0,1]")
          : "+v"(v[b]), "+v"(v[b + 1]), "+v"(v[b + 2]), "+v"(v[b + 3]), "+v"(v[b + 4]), "+v"(v[b + 5]), "+v"(v[b + 6]),
            "+v"(v[b + 7]), "+v"(v[b + 8]), "+v"(v[b + 9]), "+v"(v[b + 10]), "+v"(v[b + 11]), "+v"(v[b + 12]),
            "+v"(v[b + 13]), "+v"(v[b + 14]), "+v"(v[b + 15])
          : "v"(s));
  }
}

__device__ __forceinline__ float quad_sign(int q) { return (q == 1 || q == 2) ? -1.0f : 1.0f; }

// INV: the inverse-side convention.  The caller has multiplied the lane's INPUT by the parity sign of its lane bits
// (Rot::sign; free when the input is built with a per-lane scale anyway); with s = -1 on the lower and +1 on the upper
// lane of a cross-lane stage, v + s * partner is then the true butterfly on both lanes, (-a) + s (-b) being -(a + s b)
// exactly, and nothing is left pending on the output.
template <bool INV = false> __device__ __forceinline__ void wht128(float (&v)[32], int q) {
  constexpr float up = INV ? 1.0f : -1.0f;               // s on the lane that holds the 1-bit
#pragma unroll
  for (int h = 1; h < 32; h <<= 1) {
#pragma unroll
    for (int r = 0; r < 32; ++r) {
      if ((r & h) == 0) {
        const float a = v[r], b = v[r + h];
        v[r] = a + b;
        v[r + h] = a - b;
      }
    }
  }
  wht_quad_stage<1>(v, (q & 1) ? up : -up);
  wht_quad_stage<2>(v, (q & 2) ? up : -up);
}

// ---------------------------------------------------------------- 1024-point WHT (rotation group = whole token)
// A token's 1024 values (8 heads x 128) sit in 32 consecutive lanes, lane j holding coordinates 32 j ... 32 j + 31,
// i.e. 8 quads that each hold one head.  H_1024 = H_8 (x) H_128: after wht128 inside every quad, three more
// butterfly stages pair lanes j and j ^ 4, j ^ 8, j ^ 16.  Same multiply-add form and pending lane sign as the
// quad stages; lane ^ 8 is a DPP row rotation by 8, lane ^ 4 and lane ^ 16 go through ds_swizzle.
template <int XOR_MASK> __device__ __forceinline__ float swizzle_xor(float x) {
  static_assert(XOR_MASK == 4 || XOR_MASK == 16, "mask");
  // bit-mask mode: lane' = ((lane & 0x1f) | 0) ^ XOR_MASK within each group of 32 lanes
  return __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(x), (XOR_MASK << 10) | 0x1f));
}
__device__ __forceinline__ float row_xor8(float x) {     // value of lane ^ 8 (rotation by 8 within a row of 16)
  return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(x), 0x128 /* row_ror:8 */, 0xF, 0xF, true));
}
template <bool INV = false> __device__ __forceinline__ void wht1024_tail(float (&v)[32], int lane32) {
  constexpr float up = INV ? 1.0f : -1.0f;               // as in wht128
  const float s4 = (lane32 & 4) ? up : -up, s8 = (lane32 & 8) ? up : -up, s16 = (lane32 & 16) ? up : -up;
#pragma unroll
  for (int r = 0; r < 32; ++r) v[r] = __fmaf_rn(swizzle_xor<4>(v[r]), s4, v[r]);
#pragma unroll
  for (int r = 0; r < 32; ++r) v[r] = __fmaf_rn(row_xor8(v[r]), s8, v[r]);
#pragma unroll
  for (int r = 0; r < 32; ++r) v[r] = __fmaf_rn(swizzle_xor<16>(v[r]), s16, v[r]);
}
// sum over the 32 lanes of a token; every lane gets the total (fixed order)
__device__ __forceinline__ float token_sum(float x) {
  x = quad_sum(x);
  x = x + swizzle_xor<4>(x);
  x = x + row_xor8(x);
  x = x + swizzle_xor<16>(x);
  return x;
}

// Rotation group layouts.  WIDE = false: one group = one head = a quad of lanes (g = 128).  WIDE = true: one group =
// the whole token vector of 8 heads = 32 lanes (g = 1024).  `l` is the lane's index inside its token (0..31).
template <bool WIDE> struct Rot {
  static constexpr float kNorm = WIDE ? 0.03125f : kRsqrtG;            // 1 / sqrt(g)
  static constexpr float kInvG = WIDE ? 1.0f / 1024 : 1.0f / kGroup;
  static __device__ __forceinline__ void wht(float (&v)[32], int l) {
    wht128(v, l & 3);
    if constexpr (WIDE) wht1024_tail(v, l);
  }
  // The same transform (H_8 (x) H_128 is symmetric) with the stages across the heads first, used for the inverse:
  // a kernel that holds one head of a token per quad and fetches the other heads' grid points itself can then
  // reproduce it bit for bit by adding the 8 heads in the same tree, ((0 1)(2 3))((4 5)(6 7)), before its own wht128.
  // Inverse-side convention (see wht128): input pre-multiplied by sign(l), true output.
  static __device__ __forceinline__ void iwht(float (&v)[32], int l) {
    if constexpr (WIDE) wht1024_tail<true>(v, l);
    wht128<true>(v, l & 3);
  }
  // sign pending on the lane's values after wht(): -1 for every cross-lane stage in which the lane was the upper one
  static __device__ __forceinline__ float sign(int l) {
    const int bits = WIDE ? (l & 31) : (l & 3);
    return (__builtin_popcount(bits) & 1) ? -1.0f : 1.0f;
  }
  static __device__ __forceinline__ float sum(float x) { return WIDE ? token_sum(x) : quad_sum(x); }
};

// the 32 RHT signs this lane needs as +-1.0f: multiplying by them is exact, so s * x costs one multiplication and
// s * w + p one fused multiply-add that rounds exactly like the addition p +- w
__device__ __forceinline__ void load_signs(const int8_t* signs, int head, int q, float (&sf)[32]) {
  const u32x4* src = reinterpret_cast<const u32x4*>(signs + head * kGroup + q * kValsPerLane);
#pragma unroll
  for (int c = 0; c < 2; ++c) {
    const u32x4 raw = src[c];
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int b = 0; b < 4; ++b)
        sf[16 * c + 4 * i + b] = __uint_as_float(0x3f800000u | (((w[i] >> (8 * b)) & 0x80u) << 24));
  }
}

// Reconstruction: Q^-1(codes) = s * H(sigma16 * C[codes]) / sqrt(g).  The transform is linear, so the factor
// 1 / sqrt(g) goes into the scale once per group, together with the lane's parity sign that the inverse-side
// convention of the cross-lane stages wants on its input: the grid points are multiplied by recon_scale(sigma16, l)
// when they are fetched, and after the inverse transform one fused multiply-add per value applies the RHT sign and
// adds the prediction.  Used unchanged by the quantize,
// dequantize, scoring and fused kernels so that all of them produce bit-identical keys / values.
template <bool WIDE = false> __device__ __forceinline__ float recon_scale(float s16, int l) {
  return s16 * (Rot<WIDE>::sign(l) * Rot<WIDE>::kNorm);
}
// z: grid points scaled by recon_scale (rotated domain) -> p + Q^-1(codes)
template <bool WIDE = false>
__device__ __forceinline__ void reconstruct(float (&z)[32], int l, const float (&sf)[32], const float (&p)[32]) {
  Rot<WIDE>::iwht(z, l);
#pragma unroll
  for (int r = 0; r < 32; ++r) z[r] = __fmaf_rn(z[r], sf[r], p[r]);
}

// Rotary embedding (RoFormer) of the 32 coordinates this lane holds of a 128-long head vector.  Coordinate d is
// paired with d + 64, which is the same register of lane q ^ 2; `cos_t` / `sin_t` point at the 64 angles of the
// token's position.  x'_d = x_d cos - x_{d+64} sin,  x'_{d+64} = x_{d+64} cos + x_d sin.
__device__ __forceinline__ void rope128(float (&v)[32], int q, const float* __restrict__ cos_t,
                                        const float* __restrict__ sin_t) {
  float c[32], s[32];
  load32_f32(cos_t + 32 * (q & 1), c);
  load32_f32(sin_t + 32 * (q & 1), s);
  const float sgn = (q & 2) ? 1.0f : -1.0f;
#pragma unroll
  for (int r = 0; r < 32; ++r) {
    const float partner = quad_xor<2>(v[r]);
    v[r] = __fmaf_rn(v[r], c[r], sgn * (partner * s[r]));
  }
}

}  // namespace aquakv
