// Batched projection with fused softmax statistics for many rows (arXiv
// 2407.21082, Sections 3.2 and 3.4.1: every head on every token of a calibration
// batch, Section 3.4.1 "Calibration of Confidence Thresholds").
//
// This is the compute-bound shape (512 rows x 50304 logits x d = 2048: about 500
// flop per byte of weights), so the kernel is organised around matrix-core
// throughput:
//
//  * one workgroup of 4 waves per CU, one wave per SIMD with the whole register
//    file to itself (up to 224 accumulator registers);
//  * a workgroup owns a contiguous slice of 12-13 vocabulary tiles (16 rows each)
//    and walks it in two passes of 6-7 tiles; every weight byte is read from HBM
//    exactly once per head;
//  * a wave owns NB token blocks (16 tokens each; 8 blocks = 128 tokens at 512
//    rows) and all tiles of the pass: per k-step MT weight fragments and NB
//    activation fragments, already in matrix-core operand order, feed MT*NB
//    independent MFMAs, i.e. about 30 multiply-adds per operand byte;
//  * weight fragments travel global -> LDS with DMA loads a few k-steps ahead,
//    once per workgroup, and LDS -> registers one k-step ahead; activation
//    fragments (L2 resident, private to a wave) go straight to registers two
//    k-steps ahead; one barrier per k-step is the only synchronisation;
//  * at the end of a pass the MT*NB accumulator tiles are folded into per-lane
//    running statistics (one exponential per logit); logits are never stored.
#include "eh_internal.hpp"
#include "eh_kernels.hpp"

namespace eh {

namespace {

constexpr int kGemmWaves = 4;
constexpr int kGemmThreads = kGemmWaves * kWave;
constexpr int kMaxMT = 7;

#define EH_LDS __attribute__((address_space(3)))
#define EH_GLOBAL __attribute__((address_space(1)))
typedef EH_LDS frag_t lds_frag_t;

constexpr int kSlots = 4;      // LDS ring: k-steps of weight fragments resident
constexpr int kAFrags = 8;     // weight fragments per slot (kMaxMT rounded up)
__host__ __device__ constexpr size_t gemm_lds_bytes() { return (size_t)kSlots * kAFrags * 1024; }

// A 16-byte global load the compiler does not track: the kernel keeps its own
// count of loads in flight (see gemm_pass), so the register must not be read
// before the matching wait.
__device__ __forceinline__ void load_untracked(frag_t& dst, const EH_GLOBAL frag_t* src) {
  asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(dst) : "v"(src) : "memory");
}

// One pass: MT vocabulary tiles starting at t0, all of k, this wave's NB token
// blocks.
//  * Weight fragments (from HBM, shared by the four waves) travel global -> LDS by
//    DMA loads into a ring of kSlots k-steps, each wave fetching two of the (at
//    most 8) fragments of a step, and LDS -> registers one k-step ahead.
//  * Activation fragments (L2 resident, private to the wave) are loaded straight
//    into registers: two sets, and a fragment is refilled for the step after next
//    right after its burst of MT MFMAs.
//  * Every wave issues exactly 2 DMA loads and NB register loads per k-step, all
//    in program order, so "everything needed for the next step has landed" is a
//    wait on a compile-time count, followed by the one barrier per k-step that
//    makes the shared weight fragments visible.
template <typename DT, int MT, int NB, bool ARGMAX_ONLY>
__device__ __forceinline__ void gemm_pass(const frag_t* __restrict__ Wf, const frag_t* __restrict__ yf,
                                          int t0, int KS, int V, int lane, int wave, EH_LDS char* lds,
                                          Stats (&st)[NB]) {
  f32x4 acc[MT][NB];
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int b = 0; b < NB; ++b) acc[m][b] = f32x4{0.f, 0.f, 0.f, 0.f};
  constexpr int kSlotBytes = kAFrags * 1024;
  // At the sync before step s+1 the loads that may still be in flight are, in
  // issue order: DMA(s+3) [right after the sync before step s], B(s+2) [step s]
  constexpr int kInFlight = 2 + NB;
  static_assert(kInFlight < 64, "vmcnt field");
  const int m1 = min(wave, MT - 1), m2 = (wave + 4 < MT) ? wave + 4 : m1;
  const EH_GLOBAL frag_t* wa1 = (const EH_GLOBAL frag_t*)Wf + ((long long)(t0 + m1) * KS) * kWave + lane;
  const EH_GLOBAL frag_t* wa2 = (const EH_GLOBAL frag_t*)Wf + ((long long)(t0 + m2) * KS) * kWave + lane;
  const EH_GLOBAL frag_t* yb = (const EH_GLOBAL frag_t*)yf + lane;
  const int lastk = KS - 1;
  auto dma = [&](int ks) {  // weight fragments of k-step ks into their ring slot
    const int k = min(ks, lastk);
    EH_LDS char* slot = lds + (ks & (kSlots - 1)) * kSlotBytes;
    __builtin_amdgcn_global_load_lds((const EH_GLOBAL void*)(wa1 + (long long)k * kWave), (EH_LDS void*)(slot + m1 * 1024), 16, 0, 0);
    __builtin_amdgcn_global_load_lds((const EH_GLOBAL void*)(wa2 + (long long)k * kWave), (EH_LDS void*)(slot + m2 * 1024), 16, 0, 0);
  };
  auto load_b = [&](frag_t& dst, int n, int ks) {
    load_untracked(dst, yb + ((long long)n * KS + min(ks, lastk)) * kWave);
  };
  auto fetch_a = [&](frag_t (&a)[MT], int ks) {  // LDS -> registers
    const lds_frag_t* slot = (const lds_frag_t*)(lds + (ks & (kSlots - 1)) * kSlotBytes) + lane;
#pragma unroll
    for (int m = 0; m < MT; ++m) a[m] = slot[m * kWave];
  };
  // one k-step: MFMAs on (a, b), each activation fragment refilled for step ks+2
  auto step = [&](const frag_t (&a)[MT], frag_t (&b)[NB], int ks) {
#pragma unroll
    for (int n = 0; n < NB; ++n) {
#pragma unroll
      for (int m = 0; m < MT; ++m) acc[m][n] = DT::mma(a[m], b[n], acc[m][n]);
      load_b(b[n], n, ks + 2);
    }
  };
  // The sync before step s: "DMA(s) and B(s) have landed" (a wait on the number
  // of younger loads), every wave has finished reading the ring slot of step s-1
  // (lgkmcnt), barrier.  The register set passes through it so that no MFMA that
  // uses it can be moved above the wait.  Right after it the slot of step s-1 is
  // free for everybody and is refilled with step s+3.
#define EH_SYNC(bset, s_)                                                                          \
  do {                                                                                             \
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0) ; step-sync\n\ts_barrier" ::"n"(kInFlight) : "memory");       \
    _Pragma("unroll") for (int n_ = 0; n_ < NB; ++n_) asm volatile("" : "+v"(bset[n_]));           \
    dma((s_) + 3);                                                                                 \
  } while (0)

  // nobody may still be reading the ring (previous pass) when it is refilled
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
  frag_t a0[MT], a1[MT], b0[NB], b1[NB];
  dma(0);
  dma(1);
#pragma unroll
  for (int n = 0; n < NB; ++n) load_b(b0[n], n, 0);
  dma(2);
#pragma unroll
  for (int n = 0; n < NB; ++n) load_b(b1[n], n, 1);
  EH_SYNC(b0, 0);  // landed: DMA(0), DMA(1), b0; in flight may stay DMA(2), b1
  fetch_a(a0, 0);
  int ks = 0;
  for (; ks + 1 < KS; ks += 2) {
    step(a0, b0, ks);      // b0 <- B(ks+2)
    EH_SYNC(b1, ks + 1);   // landed: DMA(ks+1), b1 = B(ks+1); then DMA(ks+4) is issued
    fetch_a(a1, ks + 1);
    step(a1, b1, ks + 1);  // b1 <- B(ks+3)
    EH_SYNC(b0, ks + 2);   // landed: DMA(ks+2), b0 = B(ks+2); then DMA(ks+5)
    fetch_a(a0, ks + 2);
  }
  if (ks < KS) step(a0, b0, ks);  // odd number of k-steps
#undef EH_SYNC
  // The loads issued past the end (clamped) still write their registers: wait for
  // them, and keep every destination register reserved until here, or the
  // compiler would hand it out again while a load is still on its way to it.
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
  for (int n = 0; n < NB; ++n) asm volatile("" ::"v"(b0[n]), "v"(b1[n]));
  const int q = lane >> 4;
#pragma unroll
  for (int m = 0; m < MT; ++m) {
    const int row0 = (t0 + m) * 16 + q * 4;
#pragma unroll
    for (int n = 0; n < NB; ++n) stats_push4<ARGMAX_ONLY>(st[n], acc[m][n], row0, V);
  }
}

// grid.x = workgroups over the vocabulary, grid.y = groups of kGemmWaves*NB token blocks
template <typename DT, int NB, bool ARGMAX_ONLY>
__global__ __launch_bounds__(kGemmThreads, 1) void gemm_stats_kernel(
    const frag_t* __restrict__ Wf, const frag_t* __restrict__ yf, int VT, int KS, int V,
    const int* __restrict__ n_rows_dev, int n_rows, int R_pad, Stats* __restrict__ partials) {
  extern __shared__ __attribute__((aligned(16))) char gemm_smem[];
  EH_LDS char* lds = (EH_LDS char*)gemm_smem;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  int n_live = n_rows;
  if (n_rows_dev) n_live = min(max(*n_rows_dev, 0), n_rows);
  const int nb_first = (blockIdx.y * kGemmWaves + wave) * NB;  // my first token block
  const int nb_live = min(NB, ((n_live + 15) >> 4) - nb_first);
  // the whole workgroup leaves if its first wave has nothing to do (the waves
  // share barriers, so a single wave must not leave on its own; waves beyond the
  // live rows compute on zero-filled or stale activation fragments and their
  // results are not written)
  if (((n_live + 15) >> 4) - (int)(blockIdx.y * kGemmWaves * NB) <= 0) return;
  const int T0 = (int)((long long)VT * blockIdx.x / gridDim.x);
  const int T1 = (int)((long long)VT * (blockIdx.x + 1) / gridDim.x);
  Stats st[NB];
#pragma unroll
  for (int b = 0; b < NB; ++b) stats_init(st[b]);
  const frag_t* ybase = yf + (long long)nb_first * KS * kWave;
  for (int t = T0; t < T1;) {
    const int left = T1 - t;
    // split what is left into passes of at most kMaxMT tiles of about equal size
    const int passes = (left + kMaxMT - 1) / kMaxMT;
    const int mt = (left + passes - 1) / passes;
    switch (mt) {
      case 7: gemm_pass<DT, 7, NB, ARGMAX_ONLY>(Wf, ybase, t, KS, V, lane, wave, lds, st); break;
      case 6: gemm_pass<DT, 6, NB, ARGMAX_ONLY>(Wf, ybase, t, KS, V, lane, wave, lds, st); break;
      case 5: gemm_pass<DT, 5, NB, ARGMAX_ONLY>(Wf, ybase, t, KS, V, lane, wave, lds, st); break;
      case 4: gemm_pass<DT, 4, NB, ARGMAX_ONLY>(Wf, ybase, t, KS, V, lane, wave, lds, st); break;
      case 3: gemm_pass<DT, 3, NB, ARGMAX_ONLY>(Wf, ybase, t, KS, V, lane, wave, lds, st); break;
      case 2: gemm_pass<DT, 2, NB, ARGMAX_ONLY>(Wf, ybase, t, KS, V, lane, wave, lds, st); break;
      default: gemm_pass<DT, 1, NB, ARGMAX_ONLY>(Wf, ybase, t, KS, V, lane, wave, lds, st); break;
    }
    t += mt;
  }
  // lanes n, n+16, n+32, n+48 hold the same token: fold the four row groups
#pragma unroll
  for (int b = 0; b < NB; ++b) {
    st[b] = stats_merge(st[b], stats_shfl_xor(st[b], 16));
    st[b] = stats_merge(st[b], stats_shfl_xor(st[b], 32));
    if (lane < 16 && b < nb_live && nb_live > 0)
      partials[(long long)blockIdx.x * R_pad + (nb_first + b) * 16 + lane] = st[b];
  }
}

template <typename DT, bool AO>
void launch_nb(int nb, dim3 g, hipStream_t s, const frag_t* Wf, const frag_t* yf, int VT, int KS, int V,
               const int* n_rows_dev, int n_rows, int R_pad, Stats* partials) {
#define EH_G(NB)                                                                                     \
  do {                                                                                               \
    static bool attr_set = false;                                                                    \
    if (!attr_set) {                                                                                 \
      (void)hipFuncSetAttribute((const void*)gemm_stats_kernel<DT, NB, AO>,                          \
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)gemm_lds_bytes()); \
      attr_set = true;                                                                               \
    }                                                                                                \
    hipLaunchKernelGGL((gemm_stats_kernel<DT, NB, AO>), g, dim3(kGemmThreads), gemm_lds_bytes(), s, \
                       Wf, yf, VT, KS, V, n_rows_dev, n_rows, R_pad, partials);                      \
  } while (0)
  switch (nb) {
    case 1: EH_G(1); break;
    case 2: EH_G(2); break;
    case 3: EH_G(3); break;
    case 4: EH_G(4); break;
    case 6: EH_G(6); break;
    default: EH_G(8); break;
  }
#undef EH_G
}

}  // namespace

// Token blocks per wave for a given number of 16-row blocks.
static int pick_nb(int blocks) {
  const int per_wave = (blocks + kGemmWaves - 1) / kGemmWaves;
  if (per_wave <= 4) return per_wave;
  if (per_wave <= 6) return 6;
  return 8;
}

hipError_t gemm_launch(const eh_ctx* c, int head, const int* n_rows_dev, int n_rows, bool argmax_only,
                       const frag_t* yf, Stats* partials, int* n_parts, hipStream_t s) {
  const int R_pad = (n_rows + 15) & ~15;
  const int blocks = R_pad / 16;
  const int nb = pick_nb(blocks);
  const int groups = (blocks + kGemmWaves * nb - 1) / (kGemmWaves * nb);
  const int gx = std::min(c->num_cu > 0 ? c->num_cu : 256, c->VT);
  dim3 g(gx, groups);
  *n_parts = gx;
  const frag_t* Wf = c->Wf[head];
  if (c->dtype != EH_F32) return hipErrorInvalidValue;  // bf16 has its own kernel (32x32x16 instructions)
  if (argmax_only) launch_nb<DtF32, true>(nb, g, s, Wf, yf, c->VT, c->KS, c->V, n_rows_dev, n_rows, R_pad, partials);
  else launch_nb<DtF32, false>(nb, g, s, Wf, yf, c->VT, c->KS, c->V, n_rows_dev, n_rows, R_pad, partials);
  return hipGetLastError();
}

}  // namespace eh
