// Batched projection with fused softmax statistics for many rows, bf16 (arXiv
// 2407.21082, Sections 3.2 and 3.4.1: every head on every token of a calibration
// batch, Section 3.4.1 "Calibration of Confidence Thresholds"; the same kernel
// serves the large row counts of the dynamic-exit cascade, Section 3.4.2).
//
// This is the compute-bound shape (512 rows x 50304 logits x d = 2048: about 500
// flop per byte of weights), so the kernel is organised around matrix-core
// throughput:
//
//  * v_mfma_f32_32x32x16_bf16: one wave per SIMD issues these back to back at the
//    full rate of the matrix core (the 16x16x32 form needs two waves per SIMD for
//    that, which would halve the accumulator tile a wave can hold);
//  * one workgroup of 4 waves per CU.  The workgroup owns a contiguous slice of
//    the vocabulary, walked in passes of at most 7 tiles of 32 rows, and a group
//    of 4*NB blocks of 32 tokens; a wave owns NB token blocks and all tiles of
//    the pass: up to 7*2 accumulator tiles = 224 registers;
//  * the weights stay in the layout the decode kernel uses (fragments of 16 rows
//    x 32 k).  They travel global -> LDS by DMA loads, once per workgroup, four
//    k-steps ahead, and the LDS read applies the lane permutation that turns two
//    16-row fragments into the two 32-row x 16-k operands of a k-step, so no
//    second copy of the weights is needed.  A weight operand is re-read for the
//    next k-step right after its last matrix instruction of this one, which
//    spreads the LDS reads of the four waves evenly over the step;
//  * the activations (L2 resident, private to a wave) are written by the
//    LayerNorm kernel directly in 32x16 operand order and loaded straight into
//    registers three k-steps ahead, into the registers just freed;
//  * every wave issues the same, compile-time number of loads per k-step in
//    program order, so "what the next step needs has landed" is a wait on a
//    count, followed by the one barrier per k-step that publishes the weights;
//  * at the end of a pass the accumulator tiles are folded into per-lane running
//    statistics (one exponential per logit); logits are never stored.
//
// Measured on this shape the loop is bound by the rate the matrix cores sustain
// on real (toggling) data, not by memory: removing all loads from the loop does
// not shorten it, and the vendor GEMM library reaches the same rate without the
// statistics.
#include "eh_internal.hpp"
#include "eh_kernels.hpp"

#include <type_traits>

namespace eh {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kG32Waves = 4;
constexpr int kG32Threads = kG32Waves * kWave;
constexpr int kMaxMT = 7;     // 32-row tiles per pass
constexpr int kSlots = 8;     // LDS ring: k-steps of weight fragments (a slot is rewritten 7 steps after its last read)
constexpr int kSlotBytes = 2 * kMaxMT * 1024;
#ifndef EH_G32_DEPTH
#define EH_G32_DEPTH 3
#endif
constexpr int kDepth = EH_G32_DEPTH;  // activation register sets = k-steps a load may take (<= 6: ring of 8)
// the weight ring, then 16 bytes per thread: the two largest logits of its (at most 2) token blocks
// between passes (registers are too scarce to keep them live across the k loop)
__host__ __device__ constexpr size_t g32_ring_bytes() { return (size_t)kSlots * kSlotBytes; }
__host__ __device__ constexpr size_t g32_lds_bytes() { return g32_ring_bytes() + kG32Threads * 16; }

#define EH_LDS __attribute__((address_space(3)))
#define EH_GLOBAL __attribute__((address_space(1)))
typedef EH_LDS frag_t lds_frag_t;

// A 16-byte global load the compiler does not track: the kernel keeps its own
// count of loads in flight (see pass32), so the register must not be read
// before the matching wait.  The build checks the generated code for that.
// Address = wave-uniform base (scalar registers) + per-lane byte offset + IMM.
template <int IMM>
__device__ __forceinline__ void load_untracked(frag_t& dst, const EH_GLOBAL char* base, uint32_t lane_off) {
  asm volatile("global_load_dwordx4 %0, %1, %2 offset:%3" : "=v"(dst) : "v"(lane_off), "s"(base), "n"(IMM) : "memory");
}

// Makes the compiler keep a wave-uniform pointer in scalar registers.
__device__ __forceinline__ const EH_GLOBAL char* uniform_ptr(const void* p) {
  const uint64_t v = (uint64_t)p;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return (const EH_GLOBAL char*)(((uint64_t)hi << 32) | lo);
}

__device__ __forceinline__ f32x16 mma32(const frag_t& a, const frag_t& b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                 __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// The 16 logits a lane holds of one 32-row tile (accumulator register j = 4g+i: vocabulary row
// rowbase + 8g + i, increasing in j), all inside the vocabulary, pushed at once.  A single wave
// per SIMD cannot hide the latency of a dependent chain, so the work is laid out as wide,
// independent instruction groups: one maximum over the 16 (the running statistics are rescaled
// at most once, in a branch that is rarely taken after the first tiles), then 16 independent
// exponentials, then short sums.
__device__ __forceinline__ float max3(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

template <bool ARGMAX_ONLY>
__device__ __forceinline__ void stats_push16(Stats& s, const f32x16& z, int rowbase) {
  // eight three-way maxima (a NaN operand is ignored, as by fmaxf)
  const float zmax = max3(max3(max3(z[0], z[1], z[2]), max3(z[3], z[4], z[5]), z[15]),
                          max3(z[6], z[7], z[8]), max3(max3(z[9], z[10], z[11]), max3(z[12], z[13], z[14]), z[15]));
  if (zmax > s.zb) {
    int j = 15;
#pragma unroll
    for (int i = 14; i >= 0; --i) j = (z[i] == zmax) ? i : j;  // lowest index attaining the maximum
    if (!ARGMAX_ONLY) {
      const float mn = zmax * kLog2e;
      const float dm = s.m - mn;
      const float sc = fast_exp2(dm);
      s.U = sc * (s.U + dm * s.S);
      s.S = sc * s.S;
      s.m = mn;
    }
    s.zb = zmax;
    s.ib = rowbase + (j >> 2) * 8 + (j & 3);
  }
  if (!ARGMAX_ONLY) {
    float t[16], e[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) t[i] = z[i] * kLog2e - s.m;
#pragma unroll
    for (int i = 0; i < 16; ++i) e[i] = fast_exp2(t[i]);
    float S4[4], U4[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      S4[g] = (e[g] + e[g + 4]) + (e[g + 8] + e[g + 12]);
      U4[g] = t[g] * e[g];
      U4[g] += t[g + 4] * e[g + 4];
      U4[g] += t[g + 8] * e[g + 8];
      U4[g] += t[g + 12] * e[g + 12];
    }
    s.S += (S4[0] + S4[1]) + (S4[2] + S4[3]);
    s.U += (U4[0] + U4[1]) + (U4[2] + U4[3]);
  }
}

// The same for the training objectives: the head's and the model's 16 logits of one tile
// (same rows, same tokens), all inside the vocabulary.
__device__ __forceinline__ void kl_push16(KlStats& s, const f32x16& zs, const f32x16& zt, int rowbase) {
  const float a = max3(max3(max3(zs[0], zs[1], zs[2]), max3(zs[3], zs[4], zs[5]), zs[15]),
                       max3(zs[6], zs[7], zs[8]), max3(max3(zs[9], zs[10], zs[11]), max3(zs[12], zs[13], zs[14]), zs[15]));
  const float b = max3(max3(max3(zt[0], zt[1], zt[2]), max3(zt[3], zt[4], zt[5]), zt[15]),
                       max3(zt[6], zt[7], zt[8]), max3(max3(zt[9], zt[10], zt[11]), max3(zt[12], zt[13], zt[14]), zt[15]));
  const float na = a * kLog2e, nb = b * kLog2e;
  if (na > s.ms) {
    const float sc = fast_exp2(s.ms - na);
    s.Ss *= sc;
    s.C *= sc;
    s.ms = na;
  }
  if (nb > s.mt) {
    s.St *= fast_exp2(s.mt - nb);
    s.mt = nb;
  }
  float e[16], f[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) e[i] = fast_exp2(zs[i] * kLog2e - s.ms);
#pragma unroll
  for (int i = 0; i < 16; ++i) f[i] = fast_exp2(zt[i] * kLog2e - s.mt);
  float S4[4], T4[4], C4[4];
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    S4[g] = (e[g] + e[g + 4]) + (e[g + 8] + e[g + 12]);
    T4[g] = (f[g] + f[g + 4]) + (f[g + 8] + f[g + 12]);
    C4[g] = e[g] * (zs[g] - zt[g]);
    C4[g] += e[g + 4] * (zs[g + 4] - zt[g + 4]);
    C4[g] += e[g + 8] * (zs[g + 8] - zt[g + 8]);
    C4[g] += e[g + 12] * (zs[g + 12] - zt[g + 12]);
  }
  s.Ss += (S4[0] + S4[1]) + (S4[2] + S4[3]);
  s.St += (T4[0] + T4[1]) + (T4[2] + T4[3]);
  s.C += (C4[0] + C4[1]) + (C4[2] + C4[3]);
  // the label's logit: accumulator j = 4g+i holds row rowbase + 8g + i
  const int off = s.lab - rowbase;
  if (off >= 0 && off < 32 && (off & 4) == 0) {
    const int j = (off >> 3) * 4 + (off & 3);
#pragma unroll
    for (int i = 0; i < 16; ++i)
      if (i == j) s.zl = zs[i];
  }
}

// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>), in order
template <int N, typename F, int I = 0>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<N, F, I + 1>(static_cast<F&&>(f));
  }
}

// DMA loads a wave issues per k-step: the 2*MT fragments of a step are dealt
// round-robin to the four waves; a wave with fewer real fragments repeats its
// last one (same bytes to the same place) so that all waves count alike.
__host__ __device__ constexpr int dma_per_wave(int mt) { return (2 * mt + kG32Waves - 1) / kG32Waves; }

// One pass: MT tiles of 32 vocabulary rows starting at 16-row tile T16 (the workgroup's tiles end
// at t16_end, its rows at row_hi; a missing last half tile is masked), all of k, this
// wave's NB blocks of 32 tokens.
//
// k-step s (32 values of k) uses, per tile m, the operands a[m][0], a[m][1] (the
// two 16-k halves, 32 rows each) and, per token block n, b[s % D][n][0..1], with
// D = kDepth register sets.  Step s:
//   wait until my loads up to B(s) and my share of DMA(s+1) have landed;
//   tile 0's 2*NB matrix instructions; barrier (now every wave's share of DMA(s+1)
//   is in LDS); then for each tile m: [its matrix instructions,] a[m] <- LDS slot of
//   step s+1, and one piece of DMA(s+D+1); after the last tile's use of b[n] that
//   register set is reloaded with B(s+D).  The ring slot DMA(s+D+1) goes to (8
//   slots) was last read at least two steps ago and those reads have fed matrix
//   instructions since, so nobody is reading it.
// Loads return in order and every wave issues them in the order
//   DMA(0) | DMA(1) B(0) | DMA(2) B(1) | ... | DMA(s+D) B(s+D-1) | ...
// (inside a step the pieces of its DMA and its B loads interleave, which does not
// change the counts), so at the wait that opens step s the loads that may still be in
// flight are exactly the last D-1 groups, DMA(s+2) B(s+1) ... DMA(s+D) B(s+D-1): a
// wait on a compile-time count.
// TOP2: also track the two largest logits of every token (z1 >= z2, with multiplicity) for the
// "difference of the two largest probabilities" confidence metric (Section 3.4.1).
//
// DUAL (the training objectives of Section 3.3, which need the logits of an exit head and of
// the model's own head for the same token and vocabulary entry at once): the MT tiles are
// MT/2 vocabulary tiles of the head's weights followed by the same MT/2 tiles of the model's
// weights (wdelta bytes further), the NB token blocks are NB/2 blocks of the head's
// activations followed by the same NB/2 blocks of the model's (yq2), and a tile only meets
// the blocks of its own side: accumulator [m][j] and [m + MT/2][j] then hold the two logits
// of the same (vocabulary row, token) in the same register of the same lane.
struct NothingBetween {
  __device__ __forceinline__ void operator()() const {}
};
// `between` runs when the k loop is over and nobody reads the ring any more, before the
// statistics of the pass are worked out: the place to ask for the next pass's first weights, so
// that the memory system has something to do while this wave computes.
template <int MT, int NB, bool ARGMAX_ONLY, bool TOP2, bool DUAL = false, typename ST = Stats, typename BT = NothingBetween>
__device__ __forceinline__ void pass32(const frag_t* __restrict__ Wf, const frag_t* __restrict__ yq,
                                       int T16, int t16_end, int KS, int row_hi, int lane, int wave,
                                       EH_LDS char* lds, ST (&st)[DUAL ? NB / 2 : NB], long long wdelta = 0,
                                       const frag_t* __restrict__ yq2 = nullptr, BT between = BT()) {
  static_assert(!DUAL || (MT % 2 == 0 && NB % 2 == 0), "two equal sides");
  constexpr int NA = DUAL ? NB / 2 : NB;  // accumulator tiles per weight tile
  constexpr int MH = MT / 2, NH = NB / 2;
  constexpr int kDma = dma_per_wave(MT);
  constexpr int kGroup = kDma + 2 * NB;            // loads a wave issues per k-step
  constexpr int kInFlight = (kDepth - 1) * kGroup;  // younger than what SYNC needs
  static_assert(kInFlight < 64, "vmcnt field");
  constexpr int NF = 2 * MT;  // 16-row fragments per k-step

  f32x16 acc[MT][NA];
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int n = 0; n < NA; ++n)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[m][n][i] = 0.f;

  const int lastk = KS - 1;
  const uint32_t lane16 = (uint32_t)lane << 4;  // byte offset of a lane inside a fragment
  // DMA sources of this wave: fragment f = wave + 4*i of the step (or a repeat);
  // wave-uniform byte offsets of (tile, k = 0) from the start of the weights
  const EH_GLOBAL char* wbase = uniform_ptr(Wf);
  long long wsrc[kDma];
  int wdst[kDma];
#pragma unroll
  for (int i = 0; i < kDma; ++i) {
    int f = wave + kG32Waves * i;
    if (f >= NF) f = (wave < NF) ? wave + kG32Waves * ((NF - 1 - wave) / kG32Waves) : NF - 1;
    // a missing odd half tile repeats the last one (masked later)
    const bool side2 = DUAL && f >= 2 * MH;
    const int t16 = min(T16 + (side2 ? f - 2 * MH : f), t16_end - 1);
    wsrc[i] = (((long long)t16 * KS) << 10) + (side2 ? wdelta : 0);
    wdst[i] = f * 1024;
  }
  // weight fragments of k-step ks into their ring slot: this wave's i-th fragment, or all of them
  auto dma_part = [&](auto ic, int ks) {
    constexpr int i = decltype(ic)::value;
    const int k = min(ks, lastk);
    EH_LDS char* slot = lds + (ks & (kSlots - 1)) * kSlotBytes;
    __builtin_amdgcn_global_load_lds((const EH_GLOBAL void*)(wbase + wsrc[i] + ((long long)k << 10) + lane16),
                                     (EH_LDS void*)(slot + wdst[i]), 16, 0, 0);
  };
  auto dma = [&](int ks) { static_for<kDma>([&](auto ic) { dma_part(ic, ks); }); };
  // the same with the step's scalars (k offset in bytes, ring slot offset) worked out beforehand
  auto dma_part_pre = [&](auto ic, long long k10, int slotoff) {
    constexpr int i = decltype(ic)::value;
    __builtin_amdgcn_global_load_lds((const EH_GLOBAL void*)(wbase + wsrc[i] + k10 + lane16),
                                     (EH_LDS void*)(lds + slotoff + wdst[i]), 16, 0, 0);
  };
  // activations: block n, k-step ks, half h -> fragment (n, 2*ks + h) of 2*KS per block
  const EH_GLOBAL char* ybase = uniform_ptr(yq);
  const EH_GLOBAL char* ybase2 = uniform_ptr(DUAL ? yq2 : yq);
  auto b_ptr = [&](int n, int ks) {
    const bool side2 = DUAL && n >= NH;
    return (side2 ? ybase2 : ybase) + (((long long)(side2 ? n - NH : n) * 2 * KS + 2 * min(ks, lastk)) << 10);
  };
  auto load_b = [&](frag_t (&dst)[2], int n, int ks) {
    const EH_GLOBAL char* p = b_ptr(n, ks);
    load_untracked<0>(dst[0], p, lane16);
    load_untracked<1024>(dst[1], p, lane16);
  };
  auto load_b_half = [&](frag_t& dst, int n, int ks, auto hc) {
    load_untracked<decltype(hc)::value * 1024>(dst, b_ptr(n, ks), lane16);
  };
  auto load_b_half_pre = [&](frag_t& dst, int n, long long b10, auto hc) {
    const bool side2 = DUAL && n >= NH;
    const EH_GLOBAL char* p = (side2 ? ybase2 : ybase) + (((long long)(side2 ? n - NH : n) * 2 * KS) << 10) + b10;
    load_untracked<decltype(hc)::value * 1024>(dst, p, lane16);
  };
  // LDS read with the 16x32 -> 32x16 lane permutation: lane l takes row l%32 and
  // k group 2h + l/32, i.e. lane (2h + l/32)*16 + l%16 of fragment (l%32)/16.
  // These reads are not tracked by the compiler either (it would wait for all of
  // them at once): LDS reads return in order, tile m's two reads are followed by
  // those of the other MT-1 tiles before tile m is used again, so the wait before
  // a tile's matrix instructions is lgkmcnt(2*(MT-1)).  Nothing else in the loop
  // may use that counter (no scalar loads); the build checks the generated code.
  const uint32_t laneoff = (uint32_t)(uintptr_t)lds + ((lane & 31) >> 4) * 1024 + (((lane >> 5) * 16 + (lane & 15)) << 4);
  auto fetch_a_half = [&](frag_t& ah, auto mc, auto hc, int ks) {
    constexpr int m = decltype(mc)::value;
    constexpr int h = decltype(hc)::value;
    const uint32_t p = laneoff + (ks & (kSlots - 1)) * kSlotBytes;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(ah) : "v"(p), "n"(m * 2048 + h * 512) : "memory");
  };
  auto fetch_a = [&](frag_t (&a)[2], auto mc, int ks) {
    fetch_a_half(a[0], mc, std::integral_constant<int, 0>{}, ks);
    fetch_a_half(a[1], mc, std::integral_constant<int, 1>{}, ks);
  };
  constexpr int kLdsInFlight = 2 * (MT - 1);

  frag_t a[MT][2];
  frag_t b[kDepth][NB][2];
  // One k-step on register set b.  The step opens with the wait that proves this wave's
  // loads up to B(ks) and its share of DMA(ks+1) have landed; tile 0 then runs at once
  // (its weights are in registers already), and the barrier that publishes DMA(ks+1)
  // to the other waves comes behind tile 0's matrix instructions, as do, spread over the
  // tiles, the LDS reads for step ks+1 and the pieces of DMA(ks+D+1): a single wave issues
  // about one instruction per four cycles, so everything that is not a matrix instruction
  // has to sit between matrix instructions or the matrix core idles while it is issued.
  // Scalars of a step's loads are worked out a few tiles ahead, where the wave has issue slots
  // to spare (a wave issues one instruction per four clocks: anything left for the slot it is
  // needed in delays the next matrix instruction): at tile kPre the byte offset of the
  // activations of step ks+D, and k offset and ring slot of the weights of the NEXT step's DMA.
  constexpr bool kAhead = MT >= 4;
  constexpr int kPre = MT - 3;
  long long nx_k10 = (long long)min(kDepth + 1, lastk) << 10;  // for step 0: DMA(D+1)
  int nx_slot = ((kDepth + 1) & (kSlots - 1)) * kSlotBytes;
  long long nx_b10 = 0;
  auto step = [&](frag_t (&b)[NB][2], int ks) {
    asm volatile("s_waitcnt vmcnt(%0) ; step-sync" ::"n"(kInFlight) : "memory");
#pragma unroll
    for (int n = 0; n < NB; ++n) {
      asm volatile("" : "+v"(b[n][0]));
      asm volatile("" : "+v"(b[n][1]));
    }
    static_for<MT>([&](auto mc) {
      constexpr int m = decltype(mc)::value;
      asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(a[m][0]), "+v"(a[m][1]) : "n"(kLdsInFlight));
      // a wave issues one instruction per four cycles, and up to seven fit behind a matrix
      // instruction: each k half is re-read right behind the matrix instructions that used it,
      // instead of everything queueing up behind the tile's last one
      static_for<2>([&](auto hc) {
        constexpr int h = decltype(hc)::value;
#pragma unroll
        for (int n = 0; n < NB; ++n) {
          if (!DUAL || ((n < NH) == (m < MH))) {
            const int j = DUAL ? (n < NH ? n : n - NH) : n;
            acc[m][j] = mma32(a[m][h], b[n][h], acc[m][j]);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (m == 0 && h == 1) asm volatile("s_barrier" ::: "memory");
        if constexpr (m != 0) fetch_a_half(a[m][h], mc, hc, ks + 1);
        if constexpr (m == MT - 1) {  // the last use of this k half of the activations: reload it for step ks+D
#pragma unroll
          for (int n = 0; n < NB; ++n) {
            if constexpr (kAhead) load_b_half_pre(b[n][h], n, nx_b10, hc);
            else load_b_half(b[n][h], n, ks + kDepth, hc);
          }
        }
        if constexpr (h == 0) {
          // DMA piece i travels with tile min(i, MT-1), behind its first matrix instructions
          // (the slot it fills was last read several steps ago: no need to be past the barrier)
          static_for<kDma>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            if constexpr ((i < MT - 1 ? i : MT - 1) == m) {
              if constexpr (kAhead) dma_part_pre(ic, nx_k10, nx_slot);
              else dma_part(ic, ks + kDepth + 1);
            }
          });
          if constexpr (kAhead && m == kPre) {
            nx_b10 = (long long)(2 * min(ks + kDepth, lastk)) << 10;
            asm volatile("" : "+s"(nx_b10));
          }
          __builtin_amdgcn_sched_barrier(0);
        } else if constexpr (kAhead && m == kPre) {
          // this step's DMA pieces (tiles 0 .. kDma-1 <= kPre, first slot) are out: the next step's
          nx_k10 = (long long)min(ks + kDepth + 2, lastk) << 10;
          nx_slot = ((ks + kDepth + 2) & (kSlots - 1)) * kSlotBytes;
          asm volatile("" : "+s"(nx_k10), "+s"(nx_slot));
        }
      });
      if constexpr (m == 0) fetch_a(a[m], mc, ks + 1);  // slot ks+1 is complete only behind the barrier
      __builtin_amdgcn_sched_barrier(0);
    });
  };

  // nobody may still be reading the ring (previous pass) when it is refilled
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
  // Prologue.  Issue order: DMA(0) | DMA(1) B(0) | DMA(2) B(1) | ... | DMA(D) B(D-1)
  dma(0);
#pragma unroll
  for (int j = 0; j < kDepth; ++j) {
    dma(j + 1);
#pragma unroll
    for (int n = 0; n < NB; ++n) load_b(b[j][n], n, j);
  }
  // DMA(0) landed everywhere (younger: D whole groups), then a <- slot 0
  asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(kDepth * kGroup) : "memory");
  static_for<MT>([&](auto mc) { fetch_a(a[decltype(mc)::value], mc, 0); });
  // From here the wait that opens step s sees, younger than B(s) and DMA(s+1), exactly
  // the D-1 groups DMA(s+2) B(s+1) ... DMA(s+D) B(s+D-1).
  int ks = 0;
  for (; ks + kDepth <= KS; ks += kDepth) {
#pragma unroll
    for (int j = 0; j < kDepth; ++j) step(b[j], ks + j);
  }
  // the last KS % D steps, nested so that step j+1 is only reachable through step j
  auto tail = [&](auto self, auto jc) {
    constexpr int j = decltype(jc)::value;
    if constexpr (j < kDepth - 1) {
      if (ks + j < KS) {
        step(b[j], ks + j);
        self(self, std::integral_constant<int, j + 1>{});
      }
    }
  };
  tail(tail, std::integral_constant<int, 0>{});
  // The loads issued past the end (clamped) still write their registers: wait for
  // them, and keep every destination register reserved until here, or the
  // compiler would hand it out again while a load is still on its way to it.
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
#pragma unroll
  for (int n = 0; n < NB; ++n)
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int j = 0; j < kDepth; ++j) asm volatile("" ::"v"(b[j][n][h]));
#pragma unroll
  for (int m = 0; m < MT; ++m) asm volatile("" ::"v"(a[m][0]), "v"(a[m][1]));
  between();

  // accumulator register 4g+i of lane l: vocabulary row 32*tile + 8g + 4*(l/32) + i, token l%32
  const int half = lane >> 5;
  if constexpr (DUAL) {
#pragma unroll
    for (int m = 0; m < MH; ++m) {
      if (T16 * 16 + (m + 1) * 32 <= row_hi) {  // wave-uniform: only the workgroup's last tile can be ragged
#pragma unroll
        for (int n = 0; n < NA; ++n) kl_push16(st[n], acc[m][n], acc[m + MH][n], T16 * 16 + m * 32 + half * 4);
        __builtin_amdgcn_sched_barrier(0);
        continue;
      }
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int row0 = T16 * 16 + m * 32 + g * 8 + half * 4;
#pragma unroll
        for (int n = 0; n < NA; ++n) {
          const f32x4 zs = {acc[m][n][4 * g], acc[m][n][4 * g + 1], acc[m][n][4 * g + 2], acc[m][n][4 * g + 3]};
          const f32x4 zt = {acc[m + MH][n][4 * g], acc[m + MH][n][4 * g + 1], acc[m + MH][n][4 * g + 2],
                            acc[m + MH][n][4 * g + 3]};
          kl_push4(st[n], zs, zt, row0, row_hi);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    return;
  } else {
  float z1[NB], z2[NB];
  EH_LDS float* top2 = (EH_LDS float*)(lds + g32_ring_bytes()) + threadIdx.x * 4;
  if constexpr (TOP2) {
#pragma unroll
    for (int n = 0; n < NB; ++n) { z1[n] = top2[2 * n]; z2[n] = top2[2 * n + 1]; }
  }
#pragma unroll
  for (int m = 0; m < MT; ++m) {
    // wave-uniform: only the vocabulary's last tile can be ragged
    if (T16 * 16 + (m + 1) * 32 <= row_hi) {
#pragma unroll
      for (int n = 0; n < NB; ++n) {
        stats_push16<ARGMAX_ONLY>(st[n], acc[m][n], T16 * 16 + m * 32 + half * 4);
        if constexpr (TOP2) {
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const float zi = acc[m][n][i];
            z2[n] = fmaxf(z2[n], fminf(zi, z1[n]));
            z1[n] = fmaxf(z1[n], zi);
          }
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      continue;
    }
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int row0 = T16 * 16 + m * 32 + g * 8 + half * 4;
#pragma unroll
      for (int n = 0; n < NB; ++n) {
        const f32x4 z = {acc[m][n][4 * g], acc[m][n][4 * g + 1], acc[m][n][4 * g + 2], acc[m][n][4 * g + 3]};
        stats_push4<ARGMAX_ONLY>(st[n], z, row0, row_hi);
        if constexpr (TOP2) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float zi = (row0 + i < row_hi) ? z[i] : -INFINITY;
            z2[n] = fmaxf(z2[n], fminf(zi, z1[n]));
            z1[n] = fmaxf(z1[n], zi);
          }
        }
      }
      // keep the instruction scheduler from pulling all accumulators into
      // vector registers at once (it would spill inside the k loop's tail)
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  if constexpr (TOP2) {
#pragma unroll
    for (int n = 0; n < NB; ++n) { top2[2 * n] = z1[n]; top2[2 * n + 1] = z2[n]; }
  }
  }
}

// This workgroup's slice of the vocabulary in 16-row tiles, [t0, t1).  gran = 2 hands out whole
// 32-row tiles (no matrix instruction is spent on a half tile: the compute-bound shapes);
// gran = 1 hands out 16-row tiles, which halves the imbalance between workgroups (the
// bandwidth-bound shapes, where a workgroup's time is its bytes).
__device__ __forceinline__ void vocab_slice(int VT16, int gran, int& t0, int& t1) {
  const int units = (VT16 + gran - 1) / gran;
  t0 = gran * (int)((long long)units * blockIdx.x / gridDim.x);
  t1 = min(VT16, gran * (int)((long long)units * (blockIdx.x + 1) / gridDim.x));
}

// grid.x = workgroups over the vocabulary, grid.y = groups of 4*NB blocks of 32 tokens,
// grid.z = heads (Wf_tab, if given, holds the weights of head blockIdx.z; activations and
// outputs of consecutive heads lie y_stride fragments / part_stride records apart): the heads
// of one launch are independent, so a workgroup of the next head starts wherever one of this
// head has finished and the imbalance between workgroups does not idle the chip per head.
template <int NB, bool ARGMAX_ONLY, bool TOP2>
__global__ __launch_bounds__(kG32Threads, 1) void gemm32_stats_kernel(
    const frag_t* __restrict__ Wf, const frag_t* const* __restrict__ Wf_tab, const frag_t* __restrict__ yq,
    long long y_stride, int VT16, int KS, int V, int gran, const int* __restrict__ n_rows_dev, int n_rows,
    int R_pad, Stats* __restrict__ partials, float* __restrict__ second, long long part_stride) {
  if (Wf_tab) Wf = Wf_tab[blockIdx.z];
  yq += (long long)blockIdx.z * y_stride;
  partials += (long long)blockIdx.z * part_stride;
  if (TOP2) second += (long long)blockIdx.z * part_stride;
  extern __shared__ __attribute__((aligned(16))) char g32_smem[];
  EH_LDS char* lds = (EH_LDS char*)g32_smem;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  int n_live = n_rows;
  if (n_rows_dev) n_live = min(max(*n_rows_dev, 0), n_rows);
  const int live_blocks = (n_live + 31) >> 5;
  // the whole workgroup leaves if its token group is empty (the waves share
  // barriers, so a single wave must not leave on its own; waves beyond the live
  // rows compute on zero or stale activation fragments and write nothing)
  if (live_blocks - (int)(blockIdx.y * kG32Waves * NB) <= 0) return;
  const int nb_first = (blockIdx.y * kG32Waves + wave) * NB;  // my first token block
  const int nb_live = min(NB, live_blocks - nb_first);
  int T0, T1;
  vocab_slice(VT16, gran, T0, T1);
  const int row_hi = min(V, T1 * 16);
  Stats st[NB];
#pragma unroll
  for (int n = 0; n < NB; ++n) stats_init(st[n]);
  EH_LDS float* top2 = (EH_LDS float*)(lds + g32_ring_bytes()) + threadIdx.x * 4;
  if constexpr (TOP2) {
#pragma unroll
    for (int i = 0; i < 4; ++i) top2[i] = -INFINITY;
  }
  const frag_t* ybase = yq + (long long)nb_first * 2 * KS * kWave;
  for (int t = T0; t < T1;) {
    const int left = (T1 - t + 1) >> 1;  // 32-row tiles, the last one possibly half
    // split what is left into passes of at most kMaxMT tiles of about equal size
    const int passes = (left + kMaxMT - 1) / kMaxMT;
    const int mt = (left + passes - 1) / passes;
    switch (mt) {
      case 7: pass32<7, NB, ARGMAX_ONLY, TOP2>(Wf, ybase, t, T1, KS, row_hi, lane, wave, lds, st); break;
      case 6: pass32<6, NB, ARGMAX_ONLY, TOP2>(Wf, ybase, t, T1, KS, row_hi, lane, wave, lds, st); break;
      case 5: pass32<5, NB, ARGMAX_ONLY, TOP2>(Wf, ybase, t, T1, KS, row_hi, lane, wave, lds, st); break;
      case 4: pass32<4, NB, ARGMAX_ONLY, TOP2>(Wf, ybase, t, T1, KS, row_hi, lane, wave, lds, st); break;
      case 3: pass32<3, NB, ARGMAX_ONLY, TOP2>(Wf, ybase, t, T1, KS, row_hi, lane, wave, lds, st); break;
      case 2: pass32<2, NB, ARGMAX_ONLY, TOP2>(Wf, ybase, t, T1, KS, row_hi, lane, wave, lds, st); break;
      default: pass32<1, NB, ARGMAX_ONLY, TOP2>(Wf, ybase, t, T1, KS, row_hi, lane, wave, lds, st); break;
    }
    t += 2 * mt;
  }
  // lanes l and l+32 hold the same token: fold the two row groups
#pragma unroll
  for (int n = 0; n < NB; ++n) {
    st[n] = stats_merge(st[n], stats_shfl_xor(st[n], 32));
    if constexpr (TOP2) {
      const float a1 = top2[2 * n], a2 = top2[2 * n + 1];
      const float o1 = __shfl_xor(a1, 32), o2 = __shfl_xor(a2, 32);
      const float u2 = fmaxf(fminf(a1, o1), fmaxf(a2, o2));  // second largest of the union
      if (lane < 32 && n < nb_live) second[(long long)blockIdx.x * R_pad + (nb_first + n) * 32 + lane] = u2;
    }
    if (lane < 32 && n < nb_live)
      partials[(long long)blockIdx.x * R_pad + (nb_first + n) * 32 + lane] = st[n];
  }
}

// The two projections of the training objectives (Section 3.3) fused: grid.x = workgroups over
// the vocabulary, grid.y = groups of 4*NBH blocks of 32 tokens; a wave owns NBH token blocks,
// for which it holds the head's and the model's activations, and walks its slice of the
// vocabulary in passes of at most 3 tiles of 32 rows of both weight matrices.
template <int NBH>
__global__ __launch_bounds__(kG32Threads, 1) void gemm32_kl_kernel(
    const frag_t* __restrict__ Wf, long long wdelta, const frag_t* __restrict__ yq, const frag_t* __restrict__ yq2,
    int VT16, int KS, int V, int n_rows, int R_pad, const int* __restrict__ labels, KlStats* __restrict__ partials) {
  extern __shared__ __attribute__((aligned(16))) char g32_smem[];
  EH_LDS char* lds = (EH_LDS char*)g32_smem;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int live_blocks = (n_rows + 31) >> 5;
  if (live_blocks - (int)(blockIdx.y * kG32Waves * NBH) <= 0) return;
  const int nb_first = (blockIdx.y * kG32Waves + wave) * NBH;
  const int nb_live = min(NBH, live_blocks - nb_first);
  int T0, T1;
  vocab_slice(VT16, 2, T0, T1);
  const int row_hi = min(V, T1 * 16);
  KlStats st[NBH];
#pragma unroll
  for (int n = 0; n < NBH; ++n) {
    const int token = (nb_first + n) * 32 + (lane & 31);
    kl_init(st[n], (labels && token < n_rows) ? labels[token] : -1);
  }
  const frag_t* y1 = yq + (long long)nb_first * 2 * KS * kWave;
  const frag_t* y2 = yq2 + (long long)nb_first * 2 * KS * kWave;
  constexpr int kMaxMH = 3;
  for (int t = T0; t < T1;) {
    const int left = (T1 - t + 1) >> 1;
    const int passes = (left + kMaxMH - 1) / kMaxMH;
    const int mh = (left + passes - 1) / passes;
    switch (mh) {
      case 3:
        pass32<6, 2 * NBH, false, false, true, KlStats>(Wf, y1, t, T1, KS, row_hi, lane, wave, lds, st, wdelta, y2);
        break;
      case 2:
        pass32<4, 2 * NBH, false, false, true, KlStats>(Wf, y1, t, T1, KS, row_hi, lane, wave, lds, st, wdelta, y2);
        break;
      default:
        pass32<2, 2 * NBH, false, false, true, KlStats>(Wf, y1, t, T1, KS, row_hi, lane, wave, lds, st, wdelta, y2);
        break;
    }
    t += 2 * mh;
  }
#pragma unroll
  for (int n = 0; n < NBH; ++n) {
    st[n] = kl_merge(st[n], kl_shfl_xor(st[n], 32));  // lanes l and l+32 hold the same token
    if (lane < 32 && n < nb_live) partials[(long long)blockIdx.x * R_pad + (nb_first + n) * 32 + lane] = st[n];
  }
}

// ---------------------------------------------------------------------------------------------
// Persistent kernel for 17 .. 256 rows (arXiv 2407.21082: the dynamic-exit cascade of Section
// 3.4.2 on a batch of decode rows, and the verification pass of Section 4.3.1).  At these row
// counts a head is a pure weight stream (at most 256 flop per byte), so what matters is that
// the stream never stops: one launch runs every head, and nothing in it waits for a decision.
//
//  * Workgroups 0 .. n_stream-1 stream: each owns a slice of the vocabulary of every head and
//    runs pass32 on it, head after head.  Before head l it only checks that the activations of
//    head l are there (a counter that is long complete by then) and reads how many columns they
//    have; behind it, it leaves its partial statistics and bumps a counter.
//  * The last workgroups serve: wave by wave they own rows.  For head l they wait for all
//    streaming workgroups' partial statistics, merge those of their rows, apply the exit test
//    (strict H < tau, the last head always answers), publish which rows go on, and then write
//    the LayerNorm of the survivors for head l+2, compacted (column = rank among the rows
//    alive after head l).  Head l+1 is already being streamed at that time on the rows that
//    were alive after head l-1: a row that leaves at head l wastes a column there, nothing else.
//  * Hand-overs use no fence (a device-scope fence writes back and invalidates the whole L2 of
//    a die: 50 us per head when every wave issues a few).  Every head has its own activation
//    buffer, written once per launch with device-coherent stores before the counter that
//    announces it is bumped, so no cache can hold an older copy of a line when it is first
//    read; partial statistics (two buffers, reused) are written with device-coherent stores and
//    read with device-coherent loads; counters and masks are device-scope atomics.  A writer
//    waits for its stores to be acknowledged before it bumps the counter.
//  * Every wait is bounded (spin_limit polls); a time-out sets the context's status word and an
//    abort word that ends every other wait.
//
// All workgroups must be resident at once (grid = compute units, one workgroup each).
// ---------------------------------------------------------------------------------------------
#ifdef EH_DIAGNOSTICS
// Diagnostics build: workgroup `who`'s first lane stamps the 100 MHz wall clock into the words
// behind the control block (slot 2*i, 2*i+1 = low, high).
#define EH_ROWS_STAMP(i) do { if (threadIdx.x == 0 && (blockIdx.x == 0 || (int)blockIdx.x == p.n_stream)) { \
    const unsigned long long t_ = wall_clock64(); int* d_ = p.ctl + rows_ctl_ints(p.l1 - p.l0) + (blockIdx.x == 0 ? 0 : 64) + 2 * (i); \
    d_[0] = (int)(unsigned)t_; d_[1] = (int)(unsigned)(t_ >> 32); } } while (0)
#else
#define EH_ROWS_STAMP(i) ((void)0)
#endif
// All stores of this wave have been acknowledged (vector stores count in vmcnt).
#define EH_STORES_DONE() asm volatile("s_waitcnt vmcnt(0)" ::: "memory")
// Nothing below may be moved above a wait that has just returned.
#define EH_AFTER_WAIT() asm volatile("" ::: "memory")
constexpr int kRowsServiceWgs = 12;  // 3144 16-row tiles over 244 streaming workgroups: 13 at most each, as over 256
constexpr int kRowsWords = kRowsMax / 32;

// control block (ints): [0] abort; then per head (relative index j = l - l0, with two spare):
// ready[j] (LayerNorm contributions for head j), done[j] (streaming workgroups finished),
// decided[j] (service waves that published head j's decisions), alive[j][8] (rows entering head j);
// then 256 words for the merged targets of a verification
constexpr int kSpread = 16;  // words a counter is spread over: 250 adds to one word take 6 us to drain
__host__ __device__ inline int rows_ctl_ints(int n_heads) { return 16 + (n_heads + 2) * (3 * kSpread + 2 * kRowsWords) + kRowsMax; }
struct RowsCtl {
  int* base;
  int nh2;  // n_heads + 2
  __device__ __forceinline__ int* abort_word() const { return base; }
  // counters are kSpread words each: a contributor adds to word (its index % kSpread), a waiter sums them
  __device__ __forceinline__ int* ready(int j) const { return base + 16 + j * kSpread; }
  __device__ __forceinline__ int* done(int j) const { return base + 16 + (nh2 + j) * kSpread; }
  __device__ __forceinline__ int* decided(int j) const { return base + 16 + (2 * nh2 + j) * kSpread; }
  // rows entering head j: 8 64-bit words {rows decided by head j-1 : those of them that stay}
  __device__ __forceinline__ int* alive64(int j) const { return base + 16 + 3 * nh2 * kSpread + j * 2 * kRowsWords; }
  // verification: the merged argmax of every position
  __device__ __forceinline__ int* target(int pos) const { return base + 16 + nh2 * (3 * kSpread + 2 * kRowsWords) + pos; }
};

__device__ __forceinline__ int ctl_load(const int* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void ctl_add(int* counter, int who, int v) {
  (void)__hip_atomic_fetch_add(counter + (who & (kSpread - 1)), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// A whole wave waits until the counter (the sum of its kSpread words) under `mask` reaches
// `target`, and returns the sum; -1 if the launch was aborted or the wait timed out (which aborts
// the launch).
// `naps`: sleeps of 64 x 8 clocks between two looks.  A wave with time to spare (the service
// waves while a head streams) looks less often: every look is a trip to memory that competes with
// the weight stream.
__device__ __forceinline__ int rows_wait(const RowsParams& p, const RowsCtl& c, const int* counter, int target, int lane,
                                         int mask = 0x7fffffff, int naps = 1) {
  for (int spins = 0;; ++spins) {
    int v = lane < kSpread ? ctl_load(counter + lane) : 0;
#pragma unroll
    for (int x = kSpread / 2; x > 0; x >>= 1) v += __shfl_xor(v, x);
    v = __builtin_amdgcn_readfirstlane(v);
    if ((v & mask) >= target) return v;
    if (__builtin_amdgcn_readfirstlane(ctl_load(c.abort_word())) != 0) return -1;
    if (spins >= p.spin_limit) {
      if (lane == 0) {
        atomicExch(p.status, 1);
        __hip_atomic_store(c.abort_word(), 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      return -1;
    }
    for (int k = 0; k < naps; ++k) __builtin_amdgcn_s_sleep(8);
  }
}

// Device-coherent accesses (no cache of another die keeps serving an older copy): 16-byte and
// 4-byte stores, and loads that are only ISSUED here -- the caller waits (s_waitcnt vmcnt(0))
// before it looks at the registers; the build checks that in the generated code.
__device__ __forceinline__ void store_coherent(frag_t* dst, const frag_t& v) {
  asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(dst), "v"(v) : "memory");
}
__device__ __forceinline__ void store_coherent(int* dst, int v) {
  asm volatile("global_store_dword %0, %1, off sc1" ::"v"(dst), "v"(v) : "memory");
}
__device__ __forceinline__ void issue_load_coherent(frag_t& dst, const frag_t* src) {
  asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(dst) : "v"(src) : "memory");
}
__device__ __forceinline__ void issue_load_coherent(int& dst, const int* src) {
  asm volatile("global_load_dword %0, %1, off sc1" : "=v"(dst) : "v"(src) : "memory");
}
#define EH_LOADS_DONE() asm volatile("s_waitcnt vmcnt(0)" ::: "memory")
// A partial statistics record travels as (m, S, U, zb) in one array and ib in another.
__device__ __forceinline__ frag_t stats_head(const Stats& s) {
  return mk_frag(__float_as_uint(s.m), __float_as_uint(s.S), __float_as_uint(s.U), __float_as_uint(s.zb));
}
__device__ __forceinline__ Stats stats_from(const frag_t& h, int ib) {
  Stats s;
  s.m = __uint_as_float(h.x); s.S = __uint_as_float(h.y); s.U = __uint_as_float(h.z); s.zb = __uint_as_float(h.w);
  s.ib = ib;
  return s;
}
// 16-byte chunk c of the row at column p of an activation buffer in 32-row operand order
__device__ __forceinline__ void put_chunk32_coherent(frag_t* __restrict__ yf, int KS, int p, int c, const frag_t& v) {
  frag_t* dst = yf + (int64_t)(p >> 5) * KS * kWave * 2;
  store_coherent(dst + (c >> 1) * kWave + (c & 1) * 32 + (p & 31), v);
}

struct RowMask {
  unsigned w[kRowsWords];
  __device__ __forceinline__ void set_all(int n) {
#pragma unroll
    for (int i = 0; i < kRowsWords; ++i) {
      const int left = n - 32 * i;
      w[i] = left >= 32 ? 0xffffffffu : (left > 0 ? ((1u << left) - 1u) : 0u);
    }
  }
  __device__ __forceinline__ void load(const int* src) {
#pragma unroll
    for (int i = 0; i < kRowsWords; ++i) w[i] = (unsigned)ctl_load(src + i);
  }
  __device__ __forceinline__ bool test(int r) const {
    unsigned v = 0;
#pragma unroll
    for (int i = 0; i < kRowsWords; ++i) v = (i == (r >> 5)) ? w[i] : v;
    return (v >> (r & 31)) & 1u;
  }
  __device__ __forceinline__ int count() const {
    int n = 0;
#pragma unroll
    for (int i = 0; i < kRowsWords; ++i) n += __popc(w[i]);
    return n;
  }
  // number of set bits below r
  __device__ __forceinline__ int rank(int r) const {
    int n = 0;
#pragma unroll
    for (int i = 0; i < kRowsWords; ++i) {
      if (i < (r >> 5)) n += __popc(w[i]);
      else if (i == (r >> 5)) n += __popc(w[i] & ((1u << (r & 31)) - 1u));
    }
    return n;
  }
};

// A pass for a wave that owns no live token block: it still has to bring its share of the
// weights into the ring and keep every barrier of pass32<MT, ...> (one when the pass opens, one
// behind the prologue, one per k-step), but issues nothing else.  Its loads are the DMA pieces
// only, in pass32's order: at the wait that opens step ks the pieces of steps ks+2 .. ks+D may
// still be in flight.
template <int MT, typename BT = NothingBetween>
__device__ __forceinline__ void pass32_idle(const frag_t* __restrict__ Wf, int T16, int t16_end, int KS, int lane,
                                            int wave, EH_LDS char* lds, BT between = BT()) {
  constexpr int kDma = dma_per_wave(MT);
  constexpr int NF = 2 * MT;
  const int lastk = KS - 1;
  const uint32_t lane16 = (uint32_t)lane << 4;
  const EH_GLOBAL char* wbase = uniform_ptr(Wf);
  long long wsrc[kDma];
  int wdst[kDma];
#pragma unroll
  for (int i = 0; i < kDma; ++i) {
    int f = wave + kG32Waves * i;
    if (f >= NF) f = (wave < NF) ? wave + kG32Waves * ((NF - 1 - wave) / kG32Waves) : NF - 1;
    const int t16 = min(T16 + f, t16_end - 1);
    wsrc[i] = ((long long)t16 * KS) << 10;
    wdst[i] = f * 1024;
  }
  auto dma = [&](int ks) {
    const int k = min(ks, lastk);
    EH_LDS char* slot = lds + (ks & (kSlots - 1)) * kSlotBytes;
#pragma unroll
    for (int i = 0; i < kDma; ++i)
      __builtin_amdgcn_global_load_lds((const EH_GLOBAL void*)(wbase + wsrc[i] + ((long long)k << 10) + lane16),
                                       (EH_LDS void*)(slot + wdst[i]), 16, 0, 0);
  };
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
  dma(0);
#pragma unroll
  for (int j = 0; j < kDepth; ++j) dma(j + 1);
  asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(kDepth * kDma) : "memory");
  for (int ks = 0; ks < KS; ++ks) {
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"((kDepth - 1) * kDma) : "memory");
    dma(ks + kDepth + 1);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  between();
}

// The weights of the first kDepth + 1 k-steps of a pass, asked for ahead of time by this wave's DMA
// share (the pass will fetch them again: what this buys is that they then come from the L2 and
// not from HBM, and that the memory system has work while the waves compute).  They land in ring
// slots, which nobody uses for them; the one slot that another wave of the workgroup may still
// be reading when this is called right behind a k loop -- the operands of that loop's last step,
// slot (KS - 1) mod 8 -- is left alone.  Waited for by the vmcnt(0) that opens the next pass at
// the latest.
template <int MT>
__device__ __forceinline__ void ring_prefetch(const frag_t* __restrict__ Wf, int T16, int t16_end, int KS, int lane,
                                              int wave, EH_LDS char* lds) {
  constexpr int kDma = dma_per_wave(MT);
  constexpr int NF = 2 * MT;
  constexpr int kAhead = kDepth + 1;  // k-steps asked for (seven were slower than four)
  static_assert(kAhead <= kSlots, "one slot per k-step");
  const int lastk = KS - 1;
  const int busy = lastk & (kSlots - 1);
  const uint32_t lane16 = (uint32_t)lane << 4;
  const EH_GLOBAL char* wbase = uniform_ptr(Wf);
#pragma unroll
  for (int ks = 0; ks < kAhead; ++ks) {
    if (ks == busy) continue;  // uniform
    const int k = min(ks, lastk);
#pragma unroll
    for (int i = 0; i < kDma; ++i) {
      int f = wave + kG32Waves * i;
      if (f >= NF) f = (wave < NF) ? wave + kG32Waves * ((NF - 1 - wave) / kG32Waves) : NF - 1;
      const int t16 = min(T16 + f, t16_end - 1);
      __builtin_amdgcn_global_load_lds((const EH_GLOBAL void*)(wbase + ((((long long)t16 * KS) + k) << 10) + lane16),
                                       (EH_LDS void*)(lds + ks * kSlotBytes + f * 1024), 16, 0, 0);
    }
  }
}

// LayerNorm of one row by one wave into column `pos` of an activation buffer (32-row operand order).
__device__ __forceinline__ void rows_layernorm(const RowsParams& p, int l, int r, frag_t* __restrict__ yl, int pos, int lane) {
  const char* row = (const char*)p.h + ((long long)l * p.layer_stride + (long long)r * p.row_stride) * DtBf16::ESZ;
  auto put = [&](int c, const frag_t& v) { put_chunk32_coherent(yl, p.KS, pos, c, v); };
  if (p.KS * 4 <= kLnCache * kWave)  // the row fits the wave's registers: one trip to memory, not three
    group_layernorm_cached<DtBf16, 1>(row, p.d, p.KS * 4, p.gamma[l], p.beta[l], p.eps, lane, (double*)nullptr, put);
  else
    group_layernorm<DtBf16, 1>(row, p.d, p.KS * 4, p.gamma[l], p.beta[l], p.eps, lane, (double*)nullptr, put);
}

// Merge of the streaming workgroups' partial statistics of one column (one wave), in
// finalize_kernel's order.  All records are requested before any is looked at: a device-coherent
// load is a trip to memory, and one after the other they took 40 us per row.
__device__ __forceinline__ Stats rows_merge(const frag_t* __restrict__ part4, const int* __restrict__ parti, int n_parts,
                                            int R_pad, int col, int lane) {
  constexpr int kPer = (1024 + kWave - 1) / kWave;  // records per lane at most (n_parts <= 1024)
  Stats s;
  stats_init(s);
  for (int g0 = 0; g0 < n_parts; g0 += 4 * kWave) {
    frag_t h[4];
    int ib[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int g = min(g0 + lane + i * kWave, n_parts - 1);
      issue_load_coherent(h[i], part4 + (long long)g * R_pad + col);
      issue_load_coherent(ib[i], parti + (long long)g * R_pad + col);
    }
    EH_LOADS_DONE();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      asm volatile("" : "+v"(h[i]), "+v"(ib[i]));
      if (g0 + lane + i * kWave < n_parts) s = stats_merge(s, stats_from(h[i], ib[i]));
    }
  }
  (void)kPer;
#pragma unroll
  for (int x = 32; x > 0; x >>= 1) s = stats_merge(s, stats_shfl_xor(s, x));
  return s;
}

// The same for two columns at once (one wait for the records of both).
__device__ __forceinline__ void rows_merge2(const frag_t* __restrict__ part4, const int* __restrict__ parti, int n_parts,
                                            int R_pad, int col0, int col1, int lane, Stats& s0, Stats& s1) {
  stats_init(s0);
  stats_init(s1);
  for (int g0 = 0; g0 < n_parts; g0 += 4 * kWave) {
    frag_t h[2][4];
    int ib[2][4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int g = min(g0 + lane + i * kWave, n_parts - 1);
      issue_load_coherent(h[0][i], part4 + (long long)g * R_pad + col0);
      issue_load_coherent(ib[0][i], parti + (long long)g * R_pad + col0);
      issue_load_coherent(h[1][i], part4 + (long long)g * R_pad + col1);
      issue_load_coherent(ib[1][i], parti + (long long)g * R_pad + col1);
    }
    EH_LOADS_DONE();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      asm volatile("" : "+v"(h[0][i]), "+v"(ib[0][i]), "+v"(h[1][i]), "+v"(ib[1][i]));
      if (g0 + lane + i * kWave < n_parts) {
        s0 = stats_merge(s0, stats_from(h[0][i], ib[0][i]));
        s1 = stats_merge(s1, stats_from(h[1][i], ib[1][i]));
      }
    }
  }
#pragma unroll
  for (int x = 32; x > 0; x >>= 1) {
    s0 = stats_merge(s0, stats_shfl_xor(s0, x));
    s1 = stats_merge(s1, stats_shfl_xor(s1, x));
  }
}

// Returns false if the launch was aborted (or every row has left).
template <bool ARGMAX_ONLY>
__device__ __forceinline__ bool rows_stream(const RowsParams& p, const RowsCtl& c, EH_LDS char* lds, int lane, int wave,
                                            double* red, int* flag) {
  const int g = blockIdx.x, tid = threadIdx.x;
  const int nh = p.l1 - p.l0;
  const int nsw = ((int)gridDim.x - p.n_stream) * kG32Waves;  // service waves
  // my slice of the vocabulary, in 16-row tiles (bytes balanced: the stream paces these shapes)
  const int T0 = (int)((long long)p.VT16 * g / p.n_stream);
  const int T1 = (int)((long long)p.VT16 * (g + 1) / p.n_stream);
  const int row_hi = min(p.V, T1 * 16);
  const int mt_first = T0 < T1 ? (((T1 - T0 + 1) >> 1) + (((T1 - T0 + 1) >> 1) + kMaxMT - 1) / kMaxMT - 1) / ((((T1 - T0 + 1) >> 1) + kMaxMT - 1) / kMaxMT) : 0;
  // tiles per pass of a head's first pass; its first weights are brought towards the L2 while
  // something else is going on (here: the LayerNorm of the first head)
  auto warm = [&](const frag_t* Wn) {
    switch (mt_first) {
      case 7: ring_prefetch<7>(Wn, T0, T1, p.KS, lane, wave, lds); break;
      case 6: ring_prefetch<6>(Wn, T0, T1, p.KS, lane, wave, lds); break;
      case 5: ring_prefetch<5>(Wn, T0, T1, p.KS, lane, wave, lds); break;
      case 4: ring_prefetch<4>(Wn, T0, T1, p.KS, lane, wave, lds); break;
      case 3: ring_prefetch<3>(Wn, T0, T1, p.KS, lane, wave, lds); break;
      case 2: ring_prefetch<2>(Wn, T0, T1, p.KS, lane, wave, lds); break;
      case 1: ring_prefetch<1>(Wn, T0, T1, p.KS, lane, wave, lds); break;
      default: break;
    }
  };
  EH_ROWS_STAMP(0);
  warm(p.Wf[p.l0]);
  // LayerNorm of the first head's rows, spread over the streaming workgroups (four waves per row)
  for (int r = g; r < p.n_rows; r += p.n_stream) {
    const char* row = (const char*)p.h + ((long long)p.l0 * p.layer_stride + (long long)r * p.row_stride) * DtBf16::ESZ;
    auto put = [&](int ch, const frag_t& v) { put_chunk32_coherent(p.y, p.KS, r, ch, v); };
    if (p.KS * 4 <= kLnCache * kWave)
      group_layernorm_cached<DtBf16, kLnWaves>(row, p.d, p.KS * 4, p.gamma[p.l0], p.beta[p.l0], p.eps, tid, red, put);
    else
      group_layernorm<DtBf16, kLnWaves>(row, p.d, p.KS * 4, p.gamma[p.l0], p.beta[p.l0], p.eps, tid, red, put);
    __syncthreads();
  }
  EH_STORES_DONE();
  __syncthreads();
  if (tid == 0) ctl_add(c.ready(0), g, 1);
  EH_ROWS_STAMP(1);
  // the first head's activations are complete when every streaming workgroup has written its rows
  if (wave == 0) {
    const int v = rows_wait(p, c, c.ready(0), p.n_stream, lane);
    if (lane == 0) *flag = v;
  }
  __syncthreads();
  int word = *flag;
  __syncthreads();
  if (word < 0) return false;
  EH_AFTER_WAIT();
  int ncols = p.n_rows;
  EH_ROWS_STAMP(2);
  for (int j = 0; j < nh; ++j) {
    const int l = p.l0 + j;
    if (ncols == 0) return false;  // every row has left: the same for all workgroups
    // token blocks of 32 columns, dealt to the four waves as evenly as they go (at most 2 each)
    const int nblocks = (ncols + 31) >> 5;
    const int nb_live = nblocks / kG32Waves + (wave < nblocks % kG32Waves ? 1 : 0);
    const int nb_first = wave * (nblocks / kG32Waves) + min(wave, nblocks % kG32Waves);
    Stats st[2];
    stats_init(st[0]);
    stats_init(st[1]);
    const frag_t* Wf = p.Wf[l];
    const frag_t* ybase = p.y + (long long)j * p.y_stride + (long long)nb_first * 2 * p.KS * kWave;
    for (int t = T0; t < T1;) {
      const int left = (T1 - t + 1) >> 1;
      const int passes = (left + kMaxMT - 1) / kMaxMT;
      const int mt = (left + passes - 1) / passes;
      // behind the head's last k loop, while its statistics are worked out and handed on: the
      // start of the next head's weights is asked for (towards the L2; the next pass fetches it
      // again from there), so that this workgroup's share of the memory system does not idle
      const bool hand_on = t + 2 * mt >= T1 && j + 1 < nh;
      auto btw = [&]() {
        if (hand_on) warm(p.Wf[l + 1]);
      };
#define EH_ROWS_PASS(MT_)                                                                                     \
  if (nb_live <= 0) pass32_idle<MT_>(Wf, t, T1, p.KS, lane, wave, lds, btw);                                     \
  else if (nb_live == 1) pass32<MT_, 1, ARGMAX_ONLY, false, false, Stats>(Wf, ybase, t, T1, p.KS, row_hi, lane, wave, lds, \
                                                        reinterpret_cast<Stats(&)[1]>(st[0]), 0, nullptr, btw);  \
  else pass32<MT_, 2, ARGMAX_ONLY, false, false, Stats>(Wf, ybase, t, T1, p.KS, row_hi, lane, wave, lds, st, 0, nullptr, btw)
      switch (mt) {
        case 7: EH_ROWS_PASS(7); break;
        case 6: EH_ROWS_PASS(6); break;
        case 5: EH_ROWS_PASS(5); break;
        case 4: EH_ROWS_PASS(4); break;
        case 3: EH_ROWS_PASS(3); break;
        case 2: EH_ROWS_PASS(2); break;
        default: EH_ROWS_PASS(1); break;
      }
#undef EH_ROWS_PASS
      t += 2 * mt;
    }
    if (j < 8) EH_ROWS_STAMP(3 + 2 * j);
    const long long part_at = (long long)(j & 1) * p.n_stream * p.R_pad + (long long)g * p.R_pad;
#pragma unroll
    for (int n = 0; n < 2; ++n) {
      st[n] = stats_merge(st[n], stats_shfl_xor(st[n], 32));  // lanes l and l+32 hold the same token
      if (lane < 32 && n < nb_live) {
        store_coherent(p.part4 + part_at + (nb_first + n) * 32 + lane, stats_head(st[n]));
        store_coherent(p.parti + part_at + (nb_first + n) * 32 + lane, st[n].ib);
      }
    }
    if (j + 1 < nh) {
      // while those stores travel: look whether the next head's activations are there (they have
      // been for a while, as a rule).  Heads from the third on carry their column count in the
      // upper bits of the counter.
      if (wave == 0) {
        const int v = rows_wait(p, c, c.ready(j + 1), nsw, lane, 0xff);
        if (lane == 0) *flag = v;
      }
    }
    EH_STORES_DONE();
    __syncthreads();
    if (tid == 0) ctl_add(c.done(j), g, 1);
    if (j < 8) EH_ROWS_STAMP(4 + 2 * j);
    if (j + 1 < nh) {
      word = *flag;
      __syncthreads();  // the flag is rewritten at the end of the next head
      if (word < 0) return false;
      EH_AFTER_WAIT();
      ncols = j + 1 >= 2 ? (word >> 8) : p.n_rows;
    }
  }
  return true;
}

// LayerNorm of one row by one wave from operands fetched earlier (raw: the row's 16-byte chunks
// lane + 64*i; gam / bet: gamma and beta of the same chunks), in group_layernorm_cached's order.
constexpr int kSvcChunks = kLnCache;  // chunks of a row per lane: d <= 8 * 64 * 8
struct SvcRow {
  frag_t raw[kSvcChunks];
};
__device__ __forceinline__ void svc_load_row(const RowsParams& p, int l, int r, int lane, SvcRow& out) {
  const char* row = (const char*)p.h + ((long long)l * p.layer_stride + (long long)r * p.row_stride) * DtBf16::ESZ;
  const int live_chunks = p.d / DtBf16::EPL;
#pragma unroll
  for (int i = 0; i < kSvcChunks; ++i) {
    const int c = lane + i * kWave;
    out.raw[i] = mk_frag(0, 0, 0, 0);
    if (c < live_chunks) out.raw[i] = *(const frag_t*)(row + (long long)c * 16);
  }
}
// The row's normalised chunks replace the raw ones in `row` (chunk lane + 64*i; zero beyond d).
__device__ __forceinline__ void svc_layernorm(const RowsParams& p, int l, SvcRow& row, int lane) {
  const int live_chunks = p.d / DtBf16::EPL, n_chunks = p.KS * 4;
  const float* __restrict__ gamma = p.gamma[l];
  const float* __restrict__ beta = p.beta[l];
  double s = 0.0;
#pragma unroll
  for (int i = 0; i < kSvcChunks; ++i) {
    if (lane + i * kWave < live_chunks) {
      float x[8];
      decode_elems<DtBf16>(row.raw[i], x);
#pragma unroll
      for (int e = 0; e < 8; ++e) s += (double)x[e];
    }
  }
  const double mu = wave_sum(s) / (double)p.d;
  double v = 0.0;
#pragma unroll
  for (int i = 0; i < kSvcChunks; ++i) {
    if (lane + i * kWave < live_chunks) {
      float x[8];
      decode_elems<DtBf16>(row.raw[i], x);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const double cdev = (double)x[e] - mu;
        v += cdev * cdev;
      }
    }
  }
  const double rstd = 1.0 / sqrt(wave_sum(v) / (double)p.d + (double)p.eps);
#pragma unroll
  for (int i = 0; i < kSvcChunks; ++i) {
    const int c = lane + i * kWave;
    if (c < n_chunks) {
      frag_t o = mk_frag(0, 0, 0, 0);
      if (c < live_chunks) {
        float x[8];
        decode_elems<DtBf16>(row.raw[i], x);
        // gamma and beta start on 256-byte boundaries (allocations of the context)
        const f32x4 g0 = *(const f32x4*)(gamma + c * 8), g1 = *(const f32x4*)(gamma + c * 8 + 4);
        const f32x4 b0 = *(const f32x4*)(beta + c * 8), b1 = *(const f32x4*)(beta + c * 8 + 4);
        double y[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          y[e] = (double)g0[e] * (((double)x[e] - mu) * rstd) + (double)b0[e];
          y[e + 4] = (double)g1[e] * (((double)x[e + 4] - mu) * rstd) + (double)b1[e];
        }
        o = pack_elems<DtBf16>(y);
      }
      row.raw[i] = o;
    }
  }
}
// Writes a row normalised by svc_layernorm to column `pos` of an activation buffer.
__device__ __forceinline__ void svc_store(const RowsParams& p, const SvcRow& row, frag_t* __restrict__ yl, int pos, int lane) {
  const int n_chunks = p.KS * 4;
#pragma unroll
  for (int i = 0; i < kSvcChunks; ++i) {
    const int c = lane + i * kWave;
    if (c < n_chunks) put_chunk32_coherent(yl, p.KS, pos, c, row.raw[i]);
  }
}

// Service waves of a cascade (mode 0).  sw = index of this wave among the nsw service waves; it
// owns the rows r = sw, sw + nsw, ...  A head's turn is a chain of trips to memory (partial
// statistics in, decisions out, everybody's decisions in, activations out), and the streaming
// workgroups wait if it takes longer than a head's stream, so: the LayerNorm of head l+2 is computed for the wave's (first two) live rows
// BEFORE the wait for head l's statistics -- it does not depend on them, only whether and where it is
// stored does -- all
// partial records of (up to two) rows are requested at once, and a row's decision travels as one
// 64-bit word {decided | stays} so that no second counter is needed.
__device__ __forceinline__ void rows_serve_cascade(const RowsParams& p, const RowsCtl& c, int lane, int sw, int nsw) {
  const int nh = p.l1 - p.l0;
  const bool fits = p.KS * 4 <= kSvcChunks * kWave;  // a row fits one wave's registers
  // the second head's activations for every row (identity columns); the first head's are
  // written by the streaming workgroups
  if (nh > 1) {
    for (int r = sw; r < p.n_rows; r += nsw) rows_layernorm(p, p.l0 + 1, r, p.y + p.y_stride, r, lane);
    EH_STORES_DONE();
    if (lane == 0) ctl_add(c.ready(1), sw, 1);
  }
  RowMask cols, alive;  // columns of head j (rows alive after head j-2), rows entering head j
  cols.set_all(p.n_rows);
  alive.set_all(p.n_rows);
  const int r0 = sw, r1 = sw + nsw;  // the two rows of the fast path
  for (int j = 0; j < nh; ++j) {
    const int l = p.l0 + j;
    const bool last = l == p.n_heads - 1;
    const bool more = !last && j + 2 < nh;  // head j+2 exists: its LayerNorm is this turn's job
    const bool a0 = r0 < p.n_rows && alive.test(r0), a1 = r1 < p.n_rows && alive.test(r1);
    SvcRow row0, row1;
    if (j == 2) EH_ROWS_STAMP(6);
    if (more && fits) {
      if (a0) svc_load_row(p, l + 2, r0, lane, row0);
      if (a1) svc_load_row(p, l + 2, r1, lane, row1);
      if (a0) svc_layernorm(p, l + 2, row0, lane);
      if (a1) svc_layernorm(p, l + 2, row1, lane);
    }
    if (j == 2) EH_ROWS_STAMP(0);
    if (rows_wait(p, c, c.done(j), p.n_stream, lane, 0x7fffffff, 8) < 0) return;
    EH_AFTER_WAIT();
    if (j == 2) EH_ROWS_STAMP(1);
    const long long part_at = (long long)(j & 1) * p.n_stream * p.R_pad;
    const float tau = p.tau[l];
    RowMask stay, mine;  // rows of mine that go on / that were decided this turn
    stay.set_all(0);
    mine.set_all(0);
    int evals = 0;
    Stats s01[2];
    const bool both = a0 && a1;  // the first two rows together: one trip to memory for both
    if (both)
      rows_merge2(p.part4 + part_at, p.parti + part_at, p.n_stream, p.R_pad, cols.rank(r0), cols.rank(r1), lane, s01[0], s01[1]);
    for (int r = sw, k = 0; r < p.n_rows; r += nsw, ++k) {
      if (!alive.test(r)) continue;
      Stats s;
      if (both && k < 2) s = s01[k];
      else s = rows_merge(p.part4 + part_at, p.parti + part_at, p.n_stream, p.R_pad, cols.rank(r), lane);
      float H, lse;
      stats_finalize(s, H, lse);
      ++evals;
      const bool leaves = last || (H < tau);  // NaN never passes the test
      if (lane == 0) {
        if (p.H_out) p.H_out[(long long)l * p.n_rows + r] = H;
        if (leaves) {
          p.exit_layer[r] = l;
          p.token[r] = stats_token(s);
        }
      }
#pragma unroll
      for (int i = 0; i < kRowsWords; ++i) {
        if (i == (r >> 5)) {
          mine.w[i] |= 1u << (r & 31);
          if (!leaves) stay.w[i] |= 1u << (r & 31);
        }
      }
    }
    if (lane == 0 && evals && p.n_evals) atomicAdd(p.n_evals, (unsigned long long)evals);
    if (j == 2) EH_ROWS_STAMP(2);
    if (last || j + 1 == nh) return;
    // publish: one 64-bit word per 32 rows, {decided rows : rows that stay}, so a reader that sees
    // a row decided sees whether it stays
    unsigned long long* words = (unsigned long long*)c.alive64(j + 1);
    if (lane == 0) {
#pragma unroll
      for (int i = 0; i < kRowsWords; ++i)
        if (mine.w[i])
          (void)__hip_atomic_fetch_or(words + i, ((unsigned long long)mine.w[i] << 32) | stay.w[i], __ATOMIC_RELAXED,
                                      __HIP_MEMORY_SCOPE_AGENT);
    }
    // wait until every row that entered this head has been decided
    RowMask next;
    for (int spins = 0;; ++spins) {
      unsigned long long v = 0;
      if (lane < kRowsWords) v = __hip_atomic_load(words + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      bool okw = true;
#pragma unroll
      for (int i = 0; i < kRowsWords; ++i) {
        const unsigned long long vi = __shfl(v, i);
        next.w[i] = (unsigned)vi;
        okw = okw && ((unsigned)(vi >> 32) == alive.w[i]);
      }
      if (okw) break;
      if (__builtin_amdgcn_readfirstlane(ctl_load(c.abort_word())) != 0) return;
      if (spins >= p.spin_limit) {
        if (lane == 0) {
          atomicExch(p.status, 1);
          __hip_atomic_store(c.abort_word(), 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        return;
      }
      __builtin_amdgcn_s_sleep(4);
    }
    EH_AFTER_WAIT();
    if (j == 2) EH_ROWS_STAMP(3);
    if (j + 2 < nh) {
      frag_t* yl = p.y + (long long)(j + 2) * p.y_stride;
      int written = 0;
      for (int r = sw; r < p.n_rows; r += nsw) {
        if (!next.test(r)) continue;
        if (fits && r == r0) svc_store(p, row0, yl, next.rank(r), lane);
        else if (fits && r == r1) svc_store(p, row1, yl, next.rank(r), lane);
        else rows_layernorm(p, l + 2, r, yl, next.rank(r), lane);
        ++written;
      }
      if (j == 2) EH_ROWS_STAMP(4);
      EH_STORES_DONE();
      if (j == 2) EH_ROWS_STAMP(5);
      // low byte: service waves done; above it: the columns written (their sum is the head's column count)
      if (lane == 0) ctl_add(c.ready(j + 2), sw, 1 + (written << 8));
    }
    if (next.count() == 0) return;  // the same masks in every service wave
    cols = alive;
    alive = next;
  }
}

// Tail of a verification (mode 1; every workgroup streams, none only serves): when all partial
// argmax records are there, workgroup g merges those of the positions g, g + grid, ... (one
// record per thread), and when all positions are merged workgroup b < B walks draft row b's prefix.
__device__ __forceinline__ void rows_verify_tail(const RowsParams& p, const RowsCtl& c, int lane, int wave, int* flag,
                                                 float* red_z, int* red_i) {
  const int g = blockIdx.x, tid = threadIdx.x;
  if (wave == 0) {
    const int v = rows_wait(p, c, c.done(0), p.n_stream, lane);
    if (lane == 0) *flag = v >= 0 ? 1 : 0;
  }
  __syncthreads();
  int ok = *flag;
  __syncthreads();
  if (!ok) return;
  EH_AFTER_WAIT();
  EH_ROWS_STAMP(20);
  for (int pos = g; pos < p.n_rows; pos += p.n_stream) {
    float zb = -INFINITY;
    int ib = 0x7fffffff;
    for (int q0 = 0; q0 < p.n_stream; q0 += 4 * kG32Threads) {  // all records requested before any is used
      frag_t h[4];
      int ri[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int q = min(q0 + tid + i * kG32Threads, p.n_stream - 1);
        issue_load_coherent(h[i], p.part4 + (long long)q * p.R_pad + pos);
        issue_load_coherent(ri[i], p.parti + (long long)q * p.R_pad + pos);
      }
      EH_LOADS_DONE();
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        asm volatile("" : "+v"(h[i]), "+v"(ri[i]));
        const float rz = __uint_as_float(h[i].w);
        if (q0 + tid + i * kG32Threads < p.n_stream && (rz > zb || (rz == zb && ri[i] < ib))) { zb = rz; ib = ri[i]; }
      }
    }
#pragma unroll
    for (int x = 32; x > 0; x >>= 1) {
      const float oz = __shfl_xor(zb, x);
      const int oi = __shfl_xor(ib, x);
      if (oz > zb || (oz == zb && oi < ib)) { zb = oz; ib = oi; }
    }
    if (lane == 0) { red_z[wave] = zb; red_i[wave] = ib; }
    __syncthreads();
    if (tid == 0) {
#pragma unroll
      for (int w2 = 1; w2 < kG32Waves; ++w2)
        if (red_z[w2] > zb || (red_z[w2] == zb && red_i[w2] < ib)) { zb = red_z[w2]; ib = red_i[w2]; }
      const int t = argmax_or_none(ib);
      __hip_atomic_store(c.target(pos), t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (p.target) p.target[pos] = t;
      EH_STORES_DONE();
      ctl_add(c.decided(0), pos, 1);
    }
    __syncthreads();
  }
  EH_ROWS_STAMP(21);
  if (g < p.B && wave == 0) {
    // the first wave walks draft row g's prefix: all targets are fetched at once (one device-scope
    // round trip per 64 positions, not one per position), the first mismatch is a ballot away
    if (rows_wait(p, c, c.decided(0), p.n_rows, lane) < 0) return;
    EH_AFTER_WAIT();
    int len = p.k;
    if (p.draft_len) len = min(max(p.draft_len[g], 0), p.k);
    for (int j0 = 0; j0 <= p.k; j0 += kWave) {
      const int j = j0 + lane;
      int t = 0, d = -1;
      if (j <= p.k) t = ctl_load(c.target(g * (p.k + 1) + j));
      if (j < len) d = p.draft[(long long)g * p.k + j];
      const bool stop = j <= p.k && !(j < len && d == t);  // position j is not an accepted draft token
      const unsigned long long m = __ballot(stop);
      if (m) {  // the prefix ends in this group of positions (position k always stops)
        const int first = __builtin_ctzll(m);
        const int tok = __shfl(t, first);
        if (lane == 0) {
          p.accepted[g] = j0 + first;
          p.next_token[g] = tok;
        }
        EH_ROWS_STAMP(22);
        break;
      }
    }
  }
}

template <bool ARGMAX_ONLY>
__global__ __launch_bounds__(kG32Threads, 1) void gemm32_stats_kernel_rows(const RowsParams p) {
  extern __shared__ __attribute__((aligned(16))) char g32_smem[];
  __shared__ double red[2 * kLnWaves];
  __shared__ int flag;
  __shared__ float red_z[kG32Waves];
  __shared__ int red_i[kG32Waves];
  EH_LDS char* lds = (EH_LDS char*)g32_smem;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  if (p.live && *(volatile const int*)p.live == 0) return;  // the same word for every workgroup: all or none
  if (p.mode == 1) {
    // A verification has no preset launch in front of it.  Its results start as "not done" (the
    // thread that writes them here is the one that writes the real ones later), and the last
    // workgroup clears the control block of the verification after this one: nobody uses that
    // block now (the launch before this one did, and it is over).  Both happen before the
    // status test, so that a launch that does nothing still leaves a clean block behind.
    if ((int)blockIdx.x < p.B && threadIdx.x == 0) {
      p.accepted[blockIdx.x] = -1;
      p.next_token[blockIdx.x] = -1;
    }
    if (blockIdx.x == gridDim.x - 1)
      for (int i = threadIdx.x; i < p.n_ctl_next; i += kG32Threads) p.ctl_next[i] = 0;
  }
  // a launch that gave up has not been acknowledged yet (eh_check clears the flag): do nothing
  if (*(volatile int*)p.status != 0) return;
  RowsCtl c{p.ctl, p.l1 - p.l0 + 2};
  if ((int)blockIdx.x < p.n_stream) {
    const bool ok = rows_stream<ARGMAX_ONLY>(p, c, lds, lane, wave, red, &flag);
    if (ok && p.mode == 1) rows_verify_tail(p, c, lane, wave, &flag, red_z, red_i);
    return;
  }
  const int sg = (int)blockIdx.x - p.n_stream, nsg = (int)gridDim.x - p.n_stream;
  if (p.mode == 0) rows_serve_cascade(p, c, lane, sg * kG32Waves + wave, nsg * kG32Waves);
}

// Presets of a cascade launch: the control block to zero, the outputs to "not decided".
__global__ void rows_preset_kernel(int* __restrict__ ctl, int n_ctl, int* __restrict__ exit_layer, int* __restrict__ token,
                                   int n_rows, float* __restrict__ H_out, int n_H, const int* __restrict__ live) {
  if (live && *live == 0) return;
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_ctl) ctl[i] = 0;
  if (i < n_rows) { exit_layer[i] = -1; token[i] = -1; }
  if (H_out && i < n_H) H_out[i] = NAN;
}

template <int NBH>
void launch_kl(dim3 g, hipStream_t s, const frag_t* Wf, long long wdelta, const frag_t* yq, const frag_t* yq2,
               int VT16, int KS, int V, int n_rows, int R_pad, const int* labels, KlStats* partials) {
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void*)gemm32_kl_kernel<NBH>, hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)g32_lds_bytes());
    attr_set = true;
  }
  hipLaunchKernelGGL((gemm32_kl_kernel<NBH>), g, dim3(kG32Threads), g32_lds_bytes(), s, Wf, wdelta, yq, yq2, VT16,
                     KS, V, n_rows, R_pad, labels, partials);
}

template <int NB, bool AO, bool TOP2>
void launch32(dim3 g, hipStream_t s, const frag_t* Wf, const frag_t* const* Wf_tab, const frag_t* yq,
              long long y_stride, int VT16, int KS, int V, int gran, const int* n_rows_dev, int n_rows, int R_pad,
              Stats* partials, float* second, long long part_stride) {
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void*)gemm32_stats_kernel<NB, AO, TOP2>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)g32_lds_bytes());
    attr_set = true;
  }
  hipLaunchKernelGGL((gemm32_stats_kernel<NB, AO, TOP2>), g, dim3(kG32Threads), g32_lds_bytes(), s, Wf, Wf_tab, yq,
                     y_stride, VT16, KS, V, gran, n_rows_dev, n_rows, R_pad, partials, second, part_stride);
}

}  // namespace

// n_heads > 1: heads head .. head+n_heads-1 in one launch (grid.z), their activations y_stride
// fragments and their partials (and second largest logits) part_stride records apart.
hipError_t gemm32_launch_heads(const eh_ctx* c, int head, int n_heads, const int* n_rows_dev, int n_rows,
                               bool argmax_only, const frag_t* yf, long long y_stride, Stats* partials,
                               float* second, long long part_stride, int* n_parts, hipStream_t s) {
  const int R_pad = (n_rows + 31) & ~31;
  const int blocks = R_pad / 32;
  const int nb = blocks <= kG32Waves ? 1 : 2;
  const int groups = (blocks + kG32Waves * nb - 1) / (kG32Waves * nb);
  const int cus = c->num_cu > 0 ? c->num_cu : 256;
  const int VT32 = (c->VT + 1) / 2;
  const int gx = std::max(1, std::min(VT32, cus / groups));
  dim3 g(gx, groups, n_heads);
  *n_parts = gx;
  // one token group of at most 5 blocks streams the weights once and is paced by that stream:
  // balance the bytes (16-row tiles); otherwise balance the matrix instructions (32-row tiles)
  const int gran = (groups == 1 && blocks <= 5) ? 1 : 2;
  const frag_t* Wf = c->Wf[head];
  const frag_t* const* tab = n_heads > 1 ? (const frag_t* const*)(c->d_Wf + head) : nullptr;
#define EH_L32(NB_, AO_, T2_)                                                                              \
  launch32<NB_, AO_, T2_>(g, s, Wf, tab, yf, y_stride, c->VT, c->KS, c->V, gran, n_rows_dev, n_rows, R_pad, \
                          partials, second, part_stride)
  if (second) {  // entropy statistics plus the second largest logit
    if (argmax_only) return hipErrorInvalidValue;
    if (nb == 1) EH_L32(1, false, true);
    else EH_L32(2, false, true);
  } else if (nb == 1) {
    if (argmax_only) EH_L32(1, true, false);
    else EH_L32(1, false, false);
  } else {
    if (argmax_only) EH_L32(2, true, false);
    else EH_L32(2, false, false);
  }
#undef EH_L32
  return hipGetLastError();
}

hipError_t gemm32_launch(const eh_ctx* c, int head, const int* n_rows_dev, int n_rows, bool argmax_only,
                         const frag_t* yf, Stats* partials, float* second, int* n_parts, hipStream_t s) {
  return gemm32_launch_heads(c, head, 1, n_rows_dev, n_rows, argmax_only, yf, 0, partials, second, 0, n_parts, s);
}

hipError_t rows_prepare(eh_ctx* c) {
  c->rows_grid = 0;
  if (c->dtype != EH_BF16 || !c->bias.empty()) return hipSuccess;
  hipDeviceProp_t prop;
  hipError_t e = hipGetDeviceProperties(&prop, c->device);
  if (e != hipSuccess) return e;
  const int cus = prop.multiProcessorCount;
  if (cus < 4 * kRowsServiceWgs) return hipSuccess;  // too small a device to set workgroups aside
  const void* fns[2] = {(const void*)gemm32_stats_kernel_rows<false>, (const void*)gemm32_stats_kernel_rows<true>};
  for (const void* fn : fns) {
    e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)g32_lds_bytes());
    if (e != hipSuccess) { (void)hipGetLastError(); return hipSuccess; }
    int per_cu = 0;
    e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, kG32Threads, g32_lds_bytes());
    if (e != hipSuccess || per_cu < 1) { (void)hipGetLastError(); return hipSuccess; }
  }
  // the kernel's workgroups wait for each other: all of them must be resident at once
  c->rows_grid = cus;
  return hipSuccess;
}

hipError_t rows_launch(const eh_ctx* c, const RowsParams& p, hipStream_t s) {
  // every pointer the kernel dereferences unconditionally, and the sizes its indexing assumes
  if (!p.status || !p.ctl || !p.y || !p.part4 || !p.parti || !p.Wf || !p.gamma || !p.beta || !p.tau || !p.h) return hipErrorInvalidValue;
  if (c->rows_grid <= kRowsServiceWgs || p.n_stream != (p.mode == 0 ? c->rows_grid - rows_service_workgroups(p.n_rows) : c->rows_grid)) return hipErrorInvalidValue;
  if (p.n_rows < 1 || p.n_rows > kRowsMax || p.R_pad < p.n_rows || p.R_pad % 32 != 0) return hipErrorInvalidValue;
  if (p.l0 < 0 || p.l1 <= p.l0 || p.l1 > p.n_heads || rows_ctl_ints(p.l1 - p.l0) + 128 > c->rows_ctl_ints) return hipErrorInvalidValue;
  if ((long long)(p.R_pad / 16 + 32) * p.KS * kWave > p.y_stride) return hipErrorInvalidValue;  // one buffer per head
  if (p.mode == 0 ? (!p.exit_layer || !p.token) : (!p.accepted || !p.next_token || (p.k > 0 && !p.draft) || p.B * (p.k + 1) != p.n_rows))
    return hipErrorInvalidValue;
  if (p.mode == 1) {
    if (!p.ctl_next || p.n_ctl_next < rows_ctl_ints(1) || p.B > c->rows_grid) return hipErrorInvalidValue;
  } else {
    const int n_ctl = rows_ctl_ints(p.l1 - p.l0);
    const int n_H = p.H_out ? p.n_heads * p.n_rows : 0;
    const int n = std::max(std::max(n_ctl, n_H), p.n_rows);
    hipLaunchKernelGGL(rows_preset_kernel, dim3((n + 255) / 256), dim3(256), 0, s, p.ctl, n_ctl, p.exit_layer, p.token,
                       p.n_rows, p.H_out, n_H, p.live);
  }
  if (p.argmax_only)
    hipLaunchKernelGGL((gemm32_stats_kernel_rows<true>), dim3(c->rows_grid), dim3(kG32Threads), g32_lds_bytes(), s, p);
  else
    hipLaunchKernelGGL((gemm32_stats_kernel_rows<false>), dim3(c->rows_grid), dim3(kG32Threads), g32_lds_bytes(), s, p);
  return hipGetLastError();
}

int rows_control_ints(int n_heads) { return rows_ctl_ints(n_heads) + 128; }  // + 128 words of time stamps (diagnostics build)
int rows_service_workgroups(int) { return kRowsServiceWgs; }

hipError_t gemm32_kl_launch(const eh_ctx* c, int head, int model_head, int n_rows, const frag_t* yf_head,
                            const frag_t* yf_model, const int* labels, KlStats* partials, int* n_parts,
                            hipStream_t s) {
  const int R_pad = (n_rows + 31) & ~31;
  const int blocks = R_pad / 32;
  const int nbh = blocks <= kG32Waves ? 1 : 2;
  const int groups = (blocks + kG32Waves * nbh - 1) / (kG32Waves * nbh);
  const int cus = c->num_cu > 0 ? c->num_cu : 256;
  const int VT32 = (c->VT + 1) / 2;
  const int gx = std::max(1, std::min(VT32, cus / groups));
  dim3 g(gx, groups);
  *n_parts = gx;
  const long long wdelta = (const char*)c->Wf[model_head] - (const char*)c->Wf[head];
  if (nbh == 1)
    launch_kl<1>(g, s, c->Wf[head], wdelta, yf_head, yf_model, c->VT, c->KS, c->V, n_rows, R_pad, labels, partials);
  else
    launch_kl<2>(g, s, c->Wf[head], wdelta, yf_head, yf_model, c->VT, c->KS, c->V, n_rows, R_pad, labels, partials);
  return hipGetLastError();
}

}  // namespace eh
