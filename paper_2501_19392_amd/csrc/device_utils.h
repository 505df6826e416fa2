// Device-side helpers shared by the gfx950 kernels: storage-type loads/stores,
// cross-lane moves, the 128-point Walsh-Hadamard butterfly over 16 lanes x 8
// values, and the reconstruction tail used by quantize / dequantize / scores.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace aquakv {

constexpr int kGroup = 128;          // head_dim = rotation group
constexpr int kLanesPerGroup = 16;   // one group = 16 lanes x 8 values
constexpr int kValsPerLane = 8;
constexpr float kRsqrtG = 0.088388347648318440550f;   // 1/sqrt(128)

typedef __bf16 bf16_t;

// ---------------------------------------------------------------- 8-value row access
template <typename T> struct Storage;

template <> struct Storage<float> {
  static __device__ __forceinline__ void load8(const float* p, float (&v)[8]) {
    const float4 a = reinterpret_cast<const float4*>(p)[0];
    const float4 b = reinterpret_cast<const float4*>(p)[1];
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
    v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
  static __device__ __forceinline__ void store8(float* p, const float (&v)[8]) {
    reinterpret_cast<float4*>(p)[0] = make_float4(v[0], v[1], v[2], v[3]);
    reinterpret_cast<float4*>(p)[1] = make_float4(v[4], v[5], v[6], v[7]);
  }
  static __device__ __forceinline__ float round(float x) { return x; }
};

template <> struct Storage<bf16_t> {
  static __device__ __forceinline__ void load8(const bf16_t* p, float (&v)[8]) {
    const uint4 r = *reinterpret_cast<const uint4*>(p);
    const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = __uint_as_float(w[i] << 16);
      v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
  static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    const bf16_t a = static_cast<bf16_t>(lo);   // round to nearest even
    const bf16_t b = static_cast<bf16_t>(hi);
    return static_cast<uint32_t>(__builtin_bit_cast(uint16_t, a)) |
           (static_cast<uint32_t>(__builtin_bit_cast(uint16_t, b)) << 16);
  }
  static __device__ __forceinline__ void store8(bf16_t* p, const float (&v)[8]) {
    uint4 r;
    r.x = pack2(v[0], v[1]); r.y = pack2(v[2], v[3]);
    r.z = pack2(v[4], v[5]); r.w = pack2(v[6], v[7]);
    *reinterpret_cast<uint4*>(p) = r;
  }
  static __device__ __forceinline__ float round(float x) {
    return static_cast<float>(static_cast<bf16_t>(x));
  }
};

// ---------------------------------------------------------------- cross-lane moves
// Value of `x` held by lane (lane ^ MASK), MASK in {1, 2, 4, 8}: stays inside a
// row of 16 lanes, done with DPP (no LDS traffic).
template <int MASK> __device__ __forceinline__ float lane_xor(float x) {
  const int xi = __float_as_int(x);
  int r;
  if constexpr (MASK == 1) {
    r = __builtin_amdgcn_update_dpp(xi, xi, 0xB1, 0xF, 0xF, false);        // quad_perm [1,0,3,2]
  } else if constexpr (MASK == 2) {
    r = __builtin_amdgcn_update_dpp(xi, xi, 0x4E, 0xF, 0xF, false);        // quad_perm [2,3,0,1]
  } else if constexpr (MASK == 4) {
    r = __builtin_amdgcn_update_dpp(xi, xi, 0x104, 0xF, 0x5, false);       // row_shl:4 -> banks 0,2
    r = __builtin_amdgcn_update_dpp(r, xi, 0x114, 0xF, 0xA, false);        // row_shr:4 -> banks 1,3
  } else {
    static_assert(MASK == 8, "mask");
    r = __builtin_amdgcn_update_dpp(xi, xi, 0x128, 0xF, 0xF, false);       // row_ror:8
  }
  return __int_as_float(r);
}
template <int MASK> __device__ __forceinline__ uint32_t lane_xor_u32(uint32_t x) {
  return __float_as_uint(lane_xor<MASK>(__uint_as_float(x)));
}

// Sum over the 16 lanes of a group; every lane gets the total (fixed order).
__device__ __forceinline__ float group_sum16(float x) {
  x = x + lane_xor<1>(x);
  x = x + lane_xor<2>(x);
  x = x + lane_xor<4>(x);
  x = x + lane_xor<8>(x);
  return x;
}

// ---------------------------------------------------------------- 128-point WHT
// v[i] is coordinate 8*sub + i of the group (sub = lane % 16).  Unnormalised
// Sylvester-order transform: index bits 0..2 are butterflied in registers, bits
// 3..6 across lanes.  The lane holding the 0-bit keeps a+b, the other a-b.
template <int MASK> __device__ __forceinline__ void wht_lane_stage(float (&v)[8], uint32_t upper_signbit) {
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const float partner = lane_xor<MASK>(v[i]);
    const float self = __uint_as_float(__float_as_uint(v[i]) ^ upper_signbit);   // -v on the upper lane
    v[i] = partner + self;
  }
}

__device__ __forceinline__ void wht128(float (&v)[8], int sub) {
#pragma unroll
  for (int h = 1; h < 8; h <<= 1) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if ((i & h) == 0) {
        const float a = v[i], b = v[i + h];
        v[i] = a + b;
        v[i + h] = a - b;
      }
    }
  }
  wht_lane_stage<1>(v, (uint32_t)(sub & 1) << 31);
  wht_lane_stage<2>(v, (uint32_t)(sub & 2) << 30);
  wht_lane_stage<4>(v, (uint32_t)(sub & 4) << 29);
  wht_lane_stage<8>(v, (uint32_t)(sub & 8) << 28);
}

// sign bits of the 8 RHT signs this lane needs (+1 -> 0, -1 -> 0x80000000)
__device__ __forceinline__ void load_sign_bits(const int8_t* signs, int head, int sub, uint32_t (&sb)[8]) {
  const uint2 raw = *reinterpret_cast<const uint2*>(signs + head * kGroup + sub * kValsPerLane);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    sb[i] = ((raw.x >> (8 * i)) & 0x80u) << 24;
    sb[4 + i] = ((raw.y >> (8 * i)) & 0x80u) << 24;
  }
}

// Reconstruction tail: zhat (rotated, already scaled by sigma16) -> s*H(zhat)/sqrt(g) + p.
// Used unchanged by the quantize, dequantize and scoring kernels so that all
// three produce bit-identical keys/values.
__device__ __forceinline__ void reconstruct(float (&z)[8], int sub, const uint32_t (&sb)[8], const float (&p)[8]) {
  wht128(z, sub);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const float x = __uint_as_float(__float_as_uint(z[i] * kRsqrtG) ^ sb[i]);
    z[i] = x + p[i];
  }
}

}  // namespace aquakv
