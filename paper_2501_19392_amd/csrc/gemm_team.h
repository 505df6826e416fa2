// bf16 MFMA main loop of the linear predictors (Sect. 3.2 of the AQUA-KV paper) for a team of four
// wavefronts, one per SIMD, software-pipelined by hand: fragment reads, direct-to-LDS loads and the
// hand-over of a k-tile are spread between the matrix instructions so that a single wavefront keeps
// its SIMD's matrix core fed.  Used by the stand-alone predictor kernel (predict_gemm.hip).
//
// Same tile (256 token rows x 128 outputs = one kv head), same k-tiles, same three-stage LDS ring,
// same direct-to-LDS loads and the same MFMA instruction per 16 k as gemm_core.h, with two
// differences:
//  * The operands are swapped: A = 32 rows of W, B = 32 token rows, so a lane's accumulator registers
//    hold 16 outputs of ONE token (lane % 32), rows 8 * blk + 4 * (lane / 32) + r of the A block in
//    register 4 * blk + r.  The rows of W are handed to the A blocks in a permuted order (w_row), chosen
//    so that lane half hf = lane / 32 ends up with the 64 CONSECUTIVE outputs n = 64 hf + 16 j + 4 blk + r
//    of its token (j: A block): a lane stores 256 contiguous bytes of fp32, 16 bytes at a time.
//    Every output still accumulates K ascending in one accumulator, 16 k per instruction, the same
//    products in the same groups as gemm_core.h: the same bits.
//  * A k-tile is published through LDS words instead of s_barrier: every wave writes its own count of
//    finished tiles, asks for the other three counts, and looks at them one step of matrix work later,
//    so the latency of the hand-over hides behind MFMAs (a barrier stalls the wave until the slowest
//    one arrives).  Waits are bounded: a wave that waited far longer than any k-tile can take goes on
//    (the results are then wrong, but the grid always drains).
#pragma once
#include "gemm_core.h"

namespace aquakv {

constexpr int kTeamWaves = 4;
constexpr int kTeamThreads = kTeamWaves * 64;
constexpr uint32_t kSpinLimit = 1u << 22;          // polls of about 100 cycles each: seconds, never reached in practice

// Row of the 128-row W tile that sits in row q = 32 j + rho of the LDS tile (A block j, row rho = 8 blk + 4 h + r
// of the block): n = 64 h + 16 j + 4 blk + r.
__host__ __device__ constexpr int w_row(int q) {
  return 64 * ((q >> 2) & 1) + 16 * (q >> 5) + 4 * ((q >> 3) & 3) + (q & 3);
}

// Synchronisation words of a team (zeroed by the kernel before first use).
struct alignas(16) TeamFlags {
  uint32_t arrive[4];         // per wave: k-tiles published (soft barrier of the main loop)
};

// The synchronisation words are read and written with explicit LDS instructions.  Through ordinary loads and
// stores the compiler would order them after every outstanding direct-to-LDS load (it cannot tell the words
// from the ring) and wait for all of them, which would undo the prefetch distance of the ring.
__device__ __forceinline__ uint32_t lds_address(const volatile void* p) {
  return (uint32_t)(size_t)(const __attribute__((address_space(3))) void*)p;
}
// request the four words at `words` (16-byte aligned); the value is valid after flags_arrived()
__device__ __forceinline__ u32x4 flags_request(uint32_t words) {
  u32x4 v;
  asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(words) : "memory");
  return v;
}
__device__ __forceinline__ void flags_arrived(u32x4& v) { asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(v) : : "memory"); }
// wrap-safe: all four counts have reached `want`
__device__ __forceinline__ bool flags_reached(const u32x4& v, uint32_t want) {
  const int d0 = (int)(v.x - want), d1 = (int)(v.y - want), d2 = (int)(v.z - want), d3 = (int)(v.w - want);
  return __builtin_amdgcn_readfirstlane(min(min(d0, d1), min(d2, d3))) >= 0;
}

// Poll until all four words at `words` (LDS byte address, 16-byte aligned) are >= `want`.
__device__ __forceinline__ void team_wait(uint32_t words, uint32_t want) {
  for (uint32_t spin = 0; spin < kSpinLimit; ++spin) {
    u32x4 v = flags_request(words);
    flags_arrived(v);
    if (flags_reached(v, want)) return;
    __builtin_amdgcn_s_sleep(1);
  }
}

// One lane of the wave stores `value` at LDS byte address `word`.
__device__ __forceinline__ void team_post(uint32_t word, uint32_t value) {
  if ((threadIdx.x & 63) == 0) asm volatile("ds_write_b32 %0, %1" : : "v"(word), "v"(value) : "memory");
}

// acc[j][i]: outputs n = 64 (lane / 32) + 16 j + 4 blk + r (register 4 blk + r) of token 64 wave + 32 i + lane % 32.
// `arrive_words`: this team's four words in LDS; `epoch`: this wave's running count of published k-tiles (same in all
// four waves of the team).  Requirements as gemm_mainloop: K = d0 + d1 a multiple of 128, d0 of 64.
// `before_drain()` is called once, when the last operand loads are out.
template <typename BeforeDrain>
__device__ __forceinline__ void gemm_team_mainloop(unsigned char* lds_base, const uint32_t* arrive_words, uint32_t& epoch,
                                                   const bf16_t* __restrict__ x0, int d0, const bf16_t* __restrict__ x1,
                                                   int d1, const bf16_t* __restrict__ W, int64_t T, int64_t m0, int n0,
                                                   f32x16 (&acc)[4][2], BeforeDrain&& before_drain) {
  constexpr int MI = 2;                            // 32-token blocks per wave
  constexpr int kAChunks = BM * 8 / kTeamThreads;  // load instructions per thread and k-tile for x (8)
  constexpr int kBChunks = BN * 8 / kTeamThreads;  // for W (4)
  constexpr int kPieces = kAChunks + kBChunks;     // 12
  constexpr int kPieceBytes = kTeamThreads * 16;   // LDS filled by one load instruction of the team
  constexpr int kFragPieces = MI + 4;              // token blocks [0..MI), W blocks [0..4)
  constexpr int kMma = MI * 4;                     // MFMAs per step of 16 k
  typedef __attribute__((address_space(3))) unsigned char* lptr_t;
  typedef const __attribute__((address_space(1))) char* gptr_t;
  const int tid = threadIdx.x & (kTeamThreads - 1);
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int K = d0 + d1;
  const int nk = K / BK;
  const uint32_t arrive = lds_address(arrive_words);      // LDS byte address of the team's four words

  struct Frag { bf16x8 v[kFragPieces]; };

  // Addresses of the direct-to-LDS loads: a scalar base per k-tile and piece plus one per-lane byte offset per
  // operand (the accumulators take 128 registers; nothing per piece is kept).
  // Piece pc of x covers tile rows r0 + 32 pc, piece pc of W the LDS rows r0 + 32 pc, which hold W rows
  // w_row(r0) + 16 pc.  Rows beyond the last valid token row (ragged last tile only) are clamped to it.
  const int ch16 = ((tid & 7) ^ ((tid >> 4) & 7)) * 16;
  const int r0 = tid >> 3;                                                  // 0..31
  const int last = (int)((T - 1 - m0) < (BM - 1) ? (T - 1 - m0) : (BM - 1));
  const uint32_t offW = (uint32_t)w_row(r0) * (uint32_t)(K * 2) + ch16;
  const char* const wbase = reinterpret_cast<const char*>(W) + (int64_t)n0 * K * 2;
  const auto uniform_ptr = [](const char* p) {
    const uint64_t u = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)u);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(u >> 32));
    return (gptr_t)(((uint64_t)hi << 32) | lo);
  };
  const lptr_t lds3 = (lptr_t)lds_base;
  auto load_piece = [&](int kt, int stage_off, int pc) {
    const int k0 = kt * BK;
    const lptr_t dst = lds3 + (stage_off + pc * kPieceBytes + wave * 1024);
    if (pc < kAChunks) {
      const bool second = k0 >= d0;
      const int ld2 = __builtin_amdgcn_readfirstlane((second ? d1 : d0) * 2);
      const gptr_t base = uniform_ptr(reinterpret_cast<const char*>(second ? x1 : x0) +
                                      (m0 * ld2 + (int64_t)(second ? k0 - d0 : k0) * 2));
      const int row = r0 + 32 * pc;
      const uint32_t off = (uint32_t)__umul24(row < last ? row : last, ld2) + ch16;
      __builtin_amdgcn_global_load_lds(base + off, dst, 16, 0, 0);
    } else {
      const gptr_t base = uniform_ptr(wbase + ((int64_t)k0 * 2 + (int64_t)(pc - kAChunks) * 16 * K * 2));
      __builtin_amdgcn_global_load_lds(base + offW, dst, 16, 0, 0);
    }
  };
  const int frow = lane & 31;
  const int fk = lane >> 5;
  auto frag_piece = [&](int stage_off, int ks, Frag& f, int pc) {
    const int off = pc < MI ? lds_off(wave * (MI * 32) + pc * 32 + frow, ks * 2 + fk)
                            : kATileBytes + lds_off((pc - MI) * 32 + frow, ks * 2 + fk);
    f.v[pc] = *reinterpret_cast<const bf16x8*>(lds_base + stage_off + off);
  };

#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.f;

  auto mma8 = [&](const Frag& f, auto&& extra) {
#pragma unroll
    for (int m = 0; m < kMma; ++m) {
      const int i = m >> 2, j = m & 3;
      // A = 32 rows of W (outputs), B = 32 token rows: the accumulator's columns are tokens
      acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.v[MI + j], f.v[i], acc[j][i], 0, 0, 0);
      extra(m);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  auto spread = [&](int m, int n, auto&& item) {
    if (2 * m < n) item(2 * m);
    if (2 * m + 1 < n) item(2 * m + 1);
  };
  // Publishing a k-tile to the team is split in two so that its latency hides behind matrix work.  post(): this
  // wave's loads of the tile have landed and its reads of the stage that is about to be refilled have returned;
  // it writes its count and requests the four counts.  check(), one step of MFMAs later: the counts have come
  // back; if one of the other three waves is not there yet, poll until it is.
  u32x4 seen;
  auto post = [&](bool more_in_flight) {
    if (more_in_flight) __builtin_amdgcn_s_waitcnt(0x0070 | (kPieces & 15) | ((kPieces >> 4) << 14));
    else __builtin_amdgcn_s_waitcnt(0x0070);
    asm volatile("" ::: "memory");
    ++epoch;
    team_post(arrive + 4 * wave, epoch);
    seen = flags_request(arrive);
    __builtin_amdgcn_sched_barrier(0);
  };
  auto check = [&] {
    flags_arrived(seen);
    if (!flags_reached(seen, epoch)) team_wait(arrive, epoch);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
  };

  Frag f[4];
#pragma unroll
  for (int pc = 0; pc < kPieces; ++pc) load_piece(0, 0, pc);
#pragma unroll
  for (int pc = 0; pc < kPieces; ++pc) load_piece(1, kStageBytes, pc);
  post(true);
  check();

  // Iteration t: tile t is in the stage at s0, tile t+2 goes to the stage at s2 (that of tile t-1).  On entry
  // (t > 0) tile t has been posted by this wave but not yet checked, and f[2], f[3] hold steps 2 and 3 of tile t-1:
  //   MFMAs (t-1, 2)                                   the counts of the other waves come back meanwhile
  //   check
  //   MFMAs (t-1, 3)  + fragment reads (t, 0), (t, 1) + 4 of the 12 loads of tile t+2
  //   MFMAs (t,   0)  + fragment reads (t, 2)         + the other 8 loads
  //   MFMAs (t,   1)  + fragment reads (t, 3)
  //   post tile t+1
  // At most two memory instructions follow an MFMA, and every fragment is requested at least five MFMAs before
  // its first use.
  auto iteration = [&](int t, int s0, int s2, bool first, bool do_load, bool last) {
    if (!first) {
      mma8(f[2], [&](int) {});
      check();
      mma8(f[3], [&](int m) {
        spread(m, 2 * kFragPieces + 4, [&](int e) {
          if (e < kFragPieces) frag_piece(s0, 0, f[0], e);
          else if (e < 2 * kFragPieces) frag_piece(s0, 1, f[1], e - kFragPieces);
          else if (do_load) load_piece(t + 2, s2, e - 2 * kFragPieces);
        });
      });
    } else {
#pragma unroll
      for (int pc = 0; pc < kFragPieces; ++pc) { frag_piece(s0, 0, f[0], pc); frag_piece(s0, 1, f[1], pc); }
      if (do_load) {
#pragma unroll
        for (int pc = 0; pc < 4; ++pc) load_piece(t + 2, s2, pc);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    mma8(f[0], [&](int m) {
      spread(m, kFragPieces + 8, [&](int e) {
        if (e < kFragPieces) frag_piece(s0, 2, f[2], e);
        else if (do_load) load_piece(t + 2, s2, 4 + e - kFragPieces);
      });
    });
    mma8(f[1], [&](int m) { spread(m, kFragPieces, [&](int e) { frag_piece(s0, 3, f[3], e); }); });
    if (!last) post(do_load);
  };
  const auto next_stage = [](int s) { return s + kStageBytes == kMainLoopLdsBytes ? 0 : s + kStageBytes; };

  int s0 = 0, s2 = 2 * kStageBytes;
  iteration(0, s0, s2, true, nk > 2, false);
  s0 = next_stage(s0); s2 = next_stage(s2);
  int t = 1;
  for (; t + 2 < nk; ++t) {
    iteration(t, s0, s2, false, true, false);
    s0 = next_stage(s0); s2 = next_stage(s2);
  }
  before_drain();
  __builtin_amdgcn_sched_barrier(0);
  for (; t < nk; ++t) {
    iteration(t, s0, s2, false, false, t + 1 == nk);
    s0 = next_stage(s0); s2 = next_stage(s2);
  }
  mma8(f[2], [&](int) {});
  mma8(f[3], [&](int) {});
}

}  // namespace aquakv
