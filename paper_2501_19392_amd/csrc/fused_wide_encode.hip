// Fused predictor + quantizer for rotation groups of 1024 = the whole token vector of 8 kv heads (the grouping of
// the paper's experiments, Sect. 4.1 "Backbone quantization"; Alg. "encode").
//
// The group scale and the three butterfly stages across the heads need all 8 heads of a token before a single code
// can be chosen, so a workgroup owns 64 token rows x all 1024 outputs (main loop in gemm_token_slab.h, wave h = head
// h).  The epilogue takes the tile in two halves of 32 tokens: the half's predictions (+ bias) are parked in LDS as
// fp32 [32][1024], and the quantizer of the stand-alone kernels (quantize_group<.., WIDE>: 32 consecutive lanes per
// token, lane l = head l / 4, quad position l % 4, 32 values per lane) runs on 16 tokens per pass.  The second half's
// accumulators stay in registers meanwhile.  The prediction never reaches memory; same main-loop bits and the same
// quantizer code as the split path, so both give identical codes and reconstructions.
#include "codec_core.h"
#include "gemm_token_slab.h"
#include "kernels.h"

namespace aquakv {
namespace {

constexpr int kHalfRows = 32;
constexpr int kParkBytes = kHalfRows * kSlabCols * 4;                  // 128 KiB
constexpr int kWideEpilogueBytes = (int)sizeof(Lds) + kParkBytes;      // grid + table, then the parked half
constexpr int kWideLdsBytes = kWideEpilogueBytes > kSlabLdsBytes ? kWideEpilogueBytes : kSlabLdsBytes;
static_assert(kWideLdsBytes <= 160 * 1024, "LDS of one CU");

// Float index of column `col` of parked row `row`.  A lane of the quantizer reads 8 consecutive 16-byte slots (32 of
// its token's values), lane l slots 8 l ... 8 l + 7; the 16 lanes served together would fall on two bank groups, so the
// slot is XOR-ed with (slot / 16) % 8 = (l / 2) % 8: 16 lanes x 1 slot then cover all 64 banks once.  The parking
// writes come in the matrix layout, two rows 4 apart per instruction: bit 3 of the slot is flipped on those rows
// (row / 4 odd), which sends the two rows to different bank halves and leaves the reads (one row per 16 lanes) as
// they are.
__device__ __forceinline__ int park_index(int row, int col) {
  const int slot = col >> 2;
  const int s = slot ^ ((slot >> 4) & 7) ^ (((row >> 2) & 1) << 3);
  return row * kSlabCols + ((s << 2) | (col & 3));
}

// W [1024, K] -> k-tile after k-tile of 32 k, each the 64 KiB LDS image of its tile (gemm_token_slab.h): 16-byte chunk
// ch of row r of k-tile kt goes to byte kt * 64 KiB + slab_lds_off(r, ch).  One thread per chunk.
__global__ __launch_bounds__(256) void retile_w_kernel(const bf16_t* __restrict__ W, bf16_t* __restrict__ Wt, int K) {
  const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;          // (kt, r, slot) with slot fastest
  const int slot = (int)(id & 3), r = (int)((id >> 2) & (kSlabCols - 1));
  const int64_t kt = id >> 12;
  if (kt >= K / kSlabBK) return;
  const int ch = slot ^ ((r >> 2) & 3);
  const u32x4 v = *reinterpret_cast<const u32x4*>(W + (int64_t)r * K + kt * kSlabBK + ch * 8);
  *reinterpret_cast<u32x4*>(reinterpret_cast<unsigned char*>(Wt) + kt * kSlabBTileBytes + r * kSlabRowBytes + slot * 16) = v;
}

template <int NCW>
__global__ __launch_bounds__(kSlabWaves * 64) void fused_wide_encode_kernel(
    const bf16_t* __restrict__ x0, int d0, const bf16_t* __restrict__ x1, int d1, const bf16_t* __restrict__ Wt,
    const float* __restrict__ bias, const int8_t* __restrict__ signs, const float* __restrict__ codebook,
    const uint32_t* __restrict__ table, const bf16_t* X, uint8_t* codes, uint16_t* scales, bf16_t* Xhat, int64_t T) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[kWideLdsBytes];
  Lds& cl = *reinterpret_cast<Lds*>(smem);
  float* const park = reinterpret_cast<float*>(smem + sizeof(Lds));
  constexpr int kThreadsW = kSlabWaves * 64;
  constexpr int H = kSlabCols / kGroup;                                // 8
  const bool use_table = !is_rtn(NCW) && table != nullptr;     // (a round-to-nearest layer's grid pointers are never read)
  // grid and cell table: requested now, kept in registers while the main loop owns the LDS
  constexpr int kGridPoints = is_rtn(NCW) ? 0 : NCW;
  static_assert(kGridPoints <= kThreadsW, "one grid point per thread");
  float cb_a = 0.f, cb_b = 0.f;
  TableRegs<kThreadsW> table_regs;
  if ((int)threadIdx.x < kGridPoints) { cb_a = codebook[2 * threadIdx.x]; cb_b = codebook[2 * threadIdx.x + 1]; }
  if (use_table) table_regs.request(table);

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int64_t m0 = (int64_t)blockIdx.x * kSlabRows;
  // the quantizer's view: 16 tokens per pass, 32 consecutive lanes per token
  const int l = threadIdx.x & 31;                    // lane inside its token: head l / 4, quad position l % 4
  const int tslot = threadIdx.x >> 5;                // token of the pass, 0..15
  const int head = l >> 2, q = l & 3;

  struct In { u32x4 x[4]; };
  const auto fetch = [&](int half, int pass, In& in) {
    int64_t row = m0 + half * kHalfRows + pass * 16 + tslot;
    row = row < T ? row : T - 1;
    const u32x4* src = reinterpret_cast<const u32x4*>(X + row * kSlabCols + l * kValsPerLane);
#pragma unroll
    for (int k = 0; k < 4; ++k) in.x[k] = src[k];
  };
  In in_next;

  f32x16 acc[2][4];
  gemm_mainloop_token_slab(smem, x0, d0, x1, d1, Wt, T, m0, acc, [&] { fetch(0, 0, in_next); });

  float sf[32] = {};
  if constexpr (!is_rtn(NCW)) load_signs(signs, head, q, sf);

#pragma unroll
  for (int half = 0; half < 2; ++half) {
    if (half == 1) __syncthreads();                  // every wave is done reading the first half's rows
    {
      const int frow = lane & 31, fk = lane >> 5;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int col = wave * kGroup + j * 32 + frow;
        const float bv = bias != nullptr ? bias[col] : 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int prow = (r >> 2) * 8 + fk * 4 + (r & 3);
          park[park_index(prow, col)] = acc[half][j][r] + bv;
        }
      }
    }
    if (half == 0) {                                 // the ring is free: grid and table
      if ((int)threadIdx.x < kGridPoints)
        cl.cb[threadIdx.x] = make_float4(cb_a, cb_b, -0.5f * (cb_a * cb_a + cb_b * cb_b), 0.f);
      if (use_table) table_regs.store(cl.table);
    }
    __syncthreads();                                 // a token's 32 lanes read columns parked by all 8 waves

#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
      const In in = in_next;
      if (pass == 0) fetch(half, 1, in_next);        // the next pass's rows, while this one is worked on
      else if (half == 0) fetch(1, 0, in_next);
      const int prow = pass * 16 + tslot;
      const int64_t row = m0 + half * kHalfRows + prow;
      const bool active = row < T;
      const int64_t rowc = active ? row : T - 1;
      const int64_t gid = rowc * H + head;
      const int64_t off = rowc * kSlabCols + l * kValsPerLane;
      float p[32], v[32];
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const f32x4 a = *reinterpret_cast<const f32x4*>(park + park_index(prow, l * kValsPerLane + 4 * k));
        p[4 * k] = a.x; p[4 * k + 1] = a.y; p[4 * k + 2] = a.z; p[4 * k + 3] = a.w;
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) unpack_bf16x8(in.x[k], &v[8 * k]);
      quantize_group<NCW, true>(v, p, sf, l, cl.cb, use_table ? cl.table : nullptr, active, gid, codes, scales,
                                Xhat != nullptr);
      if (Xhat != nullptr && active) Storage<bf16_t>::store32(Xhat + off, v);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
}

}  // namespace

hipError_t launch_fused_encode_wide(int n_codewords, const void* x0, int d0, const void* x1, int d1, const void* W,
                                    void* w_retiled, const float* bias, const int8_t* signs, const float* codebook,
                                    const void* table, const void* X, uint8_t* codes, uint16_t* scales, void* Xhat,
                                    int64_t T, int D, hipStream_t stream) {
  if (T == 0) return hipSuccess;
  if (D != kSlabCols || w_retiled == nullptr) return hipErrorInvalidValue;
  const int K = d0 + d1;
  retile_w_kernel<<<(unsigned)((int64_t)kSlabCols * K / 8 / 256), 256, 0, stream>>>(static_cast<const bf16_t*>(W),
                                                                                   static_cast<bf16_t*>(w_retiled), K);
  const unsigned blocks = (unsigned)((T + kSlabRows - 1) / kSlabRows);
#define AQUAKV_WIDE(N)                                                                                               \
  fused_wide_encode_kernel<N><<<blocks, kSlabWaves * 64, 0, stream>>>(                                               \
      static_cast<const bf16_t*>(x0), d0, static_cast<const bf16_t*>(x1), d1, static_cast<const bf16_t*>(w_retiled), \
      bias, signs, codebook, static_cast<const uint32_t*>(table), static_cast<const bf16_t*>(X), codes, scales,      \
      static_cast<bf16_t*>(Xhat), T)
  if (n_codewords == kRtn2) AQUAKV_WIDE(kRtn2);
  else if (n_codewords == kRtn4) AQUAKV_WIDE(kRtn4);
  else if (n_codewords == 16) AQUAKV_WIDE(16);
  else if (n_codewords == 64) AQUAKV_WIDE(64);
  else AQUAKV_WIDE(256);
#undef AQUAKV_WIDE
  return hipGetLastError();
}

}  // namespace aquakv
