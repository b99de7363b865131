// Threshold calibration on the device (arXiv 2407.21082, Section 3.4.1,
// "Calibration of Confidence Thresholds"), entropy as the confidence metric.
//
// For one head and a level epsilon the threshold is the largest entropy v among
// the M calibration tokens such that, of the C(v) tokens with entropy <= v (all
// tokens at least as confident), the R(v) whose prediction equals the model's
// (eq. (2)) make up a proportion R(v)/C(v) >= epsilon.  Tokens of equal entropy are
// taken as a whole (v runs over the distinct entropies), NaN entropies are no
// candidates and are counted nowhere, and "no v qualifies" gives tau = -inf.
//
// R/C is not monotone in v, so there is nothing to bisect; but only the largest
// qualifying v is wanted, and whole ranges of v can be ruled out from counts alone.
// The entropies become order-preserving 32-bit keys, and the key range that the data
// occupies is cut three times: into up to 8192 bins, each of those into up to 2048,
// each of those into up to 256 single keys.  A bin whose tokens number cnt, cor of
// them correct, on top of C0 tokens and R0 correct ones below it, holds
//   - a top candidate (its largest key) with exactly C = C0 + cnt, R = R0 + cor, and
//   - inner candidates whose proportion is at most (R0 + cor) / (C0 + cor)
//     (R0 / (C0 + 1) if cor = 0): the correct tokens first, no wrong one.
// Walking down from the largest keys, a level keeps, for each epsilon, the bins whose
// bound reaches epsilon until the first bin whose top candidate qualifies, that one
// included; everything below it is smaller than a key that qualifies and everything
// else above it cannot qualify.  The next level counts only the tokens of kept bins.
// At the last level the bins are single keys and the first one that qualifies is the
// answer.  All quotients are the correctly rounded double divisions of the section's
// proportion; rounding is monotone, so the bound survives it.
//
// Passes over the tokens: one that reads entropy, prediction and reference (12 bytes),
// packs the correctness bits and finds the key range, two that read the entropies again
// (4 bytes each; the second sets the tokens of kept bins aside), and one over the tokens set
// aside.  The tables are small: 128 kept bins of the first level and 1024 of the second,
// over all epsilon together.  Data that keeps more (a
// proportion that hovers at epsilon over a wide range of thresholds) sets a flag that
// the host reads back, and the call is then served by the full sort below it: rocPRIM's
// radix sort of (key, correctness) pairs, a running sum, and a search of every position.
#include <cstdlib>
#include <cstring>

#include <rocprim/device/device_radix_sort.hpp>
#include <rocprim/device/device_scan.hpp>
#include <rocprim/functional.hpp>

#include "eh_internal.hpp"
#include "eh_kernels.hpp"

namespace eh {

namespace {

constexpr int kMaxEps = 64;
struct EpsList {
  double v[kMaxEps];
  int n;
};

// Order-preserving map of a float to an unsigned key, inverted so that ascending
// keys are descending entropies; NaN -> 0 (sorts first; no finite or infinite
// value maps to 0).
__device__ __forceinline__ uint32_t entropy_key(float h) {
  if (h != h) return 0u;
  if (h == 0.f) h = 0.f;  // -0 and +0 are one value
  const uint32_t u = __float_as_uint(h);
  const uint32_t asc = u ^ ((u >> 31) ? 0xFFFFFFFFu : 0x80000000u);
  return ~asc;
}
__device__ __forceinline__ float key_entropy(uint32_t key) {
  const uint32_t asc = ~key;
  return __uint_as_float(asc ^ ((asc >> 31) ? 0x80000000u : 0xFFFFFFFFu));
}

__global__ __launch_bounds__(256) void calib_keys_kernel(const float* __restrict__ H,
                                                         const int* __restrict__ pred,
                                                         const int* __restrict__ ref, int64_t M,
                                                         uint32_t* __restrict__ keys,
                                                         uint32_t* __restrict__ vals) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= M) return;
  keys[i] = entropy_key(H[i]);
  vals[i] = pred[i] == ref[i] ? 1u : 0u;
}

__global__ void calib_init_kernel(unsigned* __restrict__ best, int n, unsigned M) {
  if ((int)threadIdx.x < n) best[threadIdx.x] = M;
}

// keys ascending, prefix = inclusive running count of correct tokens in that order.
// Workgroups of 1024 positions.  Only a position before the best one found so far can
// improve it, and positions are visited roughly in ascending order: the workgroup reads
// the current bests once (possibly stale, which only costs a redundant atomic) and skips
// every level that is already settled before its first position.
__global__ __launch_bounds__(1024) void calib_search_kernel(const uint32_t* __restrict__ keys,
                                                            const uint32_t* __restrict__ prefix, int64_t M,
                                                            EpsList eps, unsigned* __restrict__ best) {
  __shared__ unsigned cur[kMaxEps];
  __shared__ unsigned wg_min[kMaxEps];
  if ((int)threadIdx.x < eps.n) {
    cur[threadIdx.x] = __builtin_nontemporal_load(&best[threadIdx.x]);
    wg_min[threadIdx.x] = 0xFFFFFFFFu;
  }
  __syncthreads();
  const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const unsigned wg_first = (unsigned)((int64_t)blockIdx.x * blockDim.x);
  const int lane = threadIdx.x & 63;
  bool cand = false;
  // proportion of correct predictions among the tokens at least as confident as this one:
  // the section's quotient as a correctly rounded double (IEEE division), compared with the
  // levels as it stands, so that exactly p of q tokens meet a level written as the decimal p/q
  double prop = 0.0;
  if (j < M) {
    const uint32_t k = keys[j];
    cand = k != 0u && (j == 0 || keys[j - 1] != k);
    if (cand) {
      const uint32_t total = prefix[M - 1];
      prop = (double)(total - (j ? prefix[j - 1] : 0u)) / (double)(M - j);
    }
  }
  bool any = false;
  for (int e = 0; e < eps.n; ++e) {
    if (cur[e] <= wg_first) continue;  // uniform over the workgroup
    any = true;
    // lanes hold ascending positions: the first lane that qualifies is the wave's minimum
    const unsigned long long q = __ballot(cand && prop >= eps.v[e]);
    if (lane == 0 && q) atomicMin(&wg_min[e], (unsigned)(j + __builtin_ctzll(q)));
  }
  if (!any) return;  // uniform
  __syncthreads();
  if ((int)threadIdx.x < eps.n && wg_min[threadIdx.x] != 0xFFFFFFFFu) atomicMin(&best[threadIdx.x], wg_min[threadIdx.x]);
}

__global__ void calib_read_kernel(const uint32_t* __restrict__ keys, const unsigned* __restrict__ best, int n,
                                  unsigned M, float* __restrict__ tau, long long* __restrict__ n_exit) {
  const int e = threadIdx.x;
  if (e >= n) return;
  const unsigned b = best[e];
  tau[e] = b < M ? key_entropy(keys[b]) : -INFINITY;
  if (n_exit) n_exit[e] = b < M ? (long long)(M - b) : 0;
}


// ---------------------------------------------------------------------------------
// The refinement: three levels of counts instead of a sort.

constexpr int kBins1 = 8192;       // bins of level 1
constexpr int kBins2 = 2048;       // bins of one kept level-1 bin
constexpr int kBins3 = 256;        // single keys of one kept level-2 bin
constexpr int kCap1 = 128;         // kept bins of level 1, all epsilon together
constexpr int kCap2 = 1024;        // kept bins of level 2
constexpr int kChunk = 2048;       // tokens four waves take at a time: 4 x 8 x 64 (a workgroup of 1024: four times that)
constexpr int kStageWave = 1024;    // tokens of kept bins a wave holds back before it appends them
constexpr int kSegment = 32768;    // tokens behind one row of level-1 partial counts (16-bit counters)
constexpr int64_t kRefineMax = (int64_t)1 << 27;  // larger sets go to the sort (4096 partial rows)

// ascending key of a non-NaN entropy (the key of the sort above, not inverted)
__device__ __forceinline__ uint32_t ascending_key(float h) {
  if (h == 0.f) h = 0.f;
  const uint32_t u = __float_as_uint(h);
  return u ^ ((u >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}
__device__ __forceinline__ float ascending_entropy(uint32_t asc) {
  return __uint_as_float(asc ^ ((asc >> 31) ? 0x80000000u : 0xFFFFFFFFu));
}

// Device memory of one call.  Counts are pairs in one 64-bit word: tokens in the low half,
// correct tokens in the high half.
struct CalibWork {
  uint64_t* bits;     // [ceil(M / 64)] correctness of token i in bit i % 64 of word i / 64
  uint32_t* part1;    // [ceil(M / kSegment)][kBins1] level-1 counts of a segment, 16 + 16 bits
  uint32_t* kept;     // [M] tokens of kept level-1 bins: correct << 31 | row << 20 | key bits below s
  // preset to 0
  uint32_t* key_max;  // [1] largest key (with key_min: the range the data occupies)
  int* n_kept;        // [3] kept bins of level 1, of level 2; tokens in `kept`
  uint64_t* h1;       // [kBins1]
  uint64_t* sel1;     // [kBins1] which epsilon keep the bin
  uint64_t* h2;       // [kCap1][kBins2]
  uint64_t* sel2;     // [kCap1][kBins2]
  uint64_t* h3;       // [kCap2][kBins3]
  // preset to -1
  uint32_t* key_min;  // [1]
  int* overflow;      // [1] -1, or 0 once a table has proved too small
  int* slot1;         // [kBins1] row of a kept bin in h2
  int* slot2;         // [kCap1][kBins2] row of a kept bin in h3
};

// How the occupied key range [lo, hi] is cut: level 1 takes the bits above s, level 2 the
// next b2, level 3 the last b3.
struct Cut {
  uint32_t base;
  int s, b2, b3;
  bool empty;
};
__device__ __forceinline__ Cut cut_of(const CalibWork& w) {
  Cut c;
  const uint32_t lo = *w.key_min, hi = *w.key_max;
  c.empty = lo > hi;
  c.base = lo;
  const uint32_t span = c.empty ? 0u : hi - lo;
  c.s = 0;
  while ((span >> c.s) >= (uint32_t)kBins1) ++c.s;  // at most 19
  c.b2 = c.s < 11 ? c.s : 11;
  c.b3 = c.s - c.b2;                                // at most 8
  return c;
}

struct Pair {
  uint32_t c, r;
};
__device__ __forceinline__ Pair operator+(Pair a, Pair b) { return Pair{a.c + b.c, a.r + b.r}; }
__device__ __forceinline__ Pair pair_of(uint64_t v) { return Pair{(uint32_t)v, (uint32_t)(v >> 32)}; }

// Exclusive prefix of one Pair per thread over the 256 threads of a workgroup; *total_c
// receives the sum of the first members.
__device__ __forceinline__ Pair block_exclusive(Pair v, Pair* sh /* [4] */, int* total_c = nullptr) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  Pair inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t c = __shfl_up(inc.c, o), r = __shfl_up(inc.r, o);
    if (lane >= o) inc = inc + Pair{c, r};
  }
  __syncthreads();  // sh may still be read from the call before
  if (lane == 63) sh[wave] = inc;
  __syncthreads();
  Pair off{0, 0};
  for (int k = 0; k < wave; ++k) off = off + sh[k];
  if (total_c) *total_c = (int)(sh[0].c + sh[1].c + sh[2].c + sh[3].c);
  return Pair{off.c + inc.c - v.c, off.r + inc.r - v.r};
}
__device__ __forceinline__ int block_max(int v, int* sh /* [4] */) {
#pragma unroll
  for (int o = 32; o; o >>= 1) {
    const int u = __shfl_xor(v, o);
    v = u > v ? u : v;
  }
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  int m = sh[0];
  for (int k = 1; k < 4; ++k) m = sh[k] > m ? sh[k] : m;
  return m;
}

struct NodeShared {
  Pair scan[4];
  int red[4];
  Pair at_top;  // counts up to and including the bin that node_scan names
};

// One node: nb <= 256 * PER bins of counts in ascending key order, on top of `below`.
// Thread t looks at bins [PER * t, PER * (t + 1)).  Gives back the bins' exclusive prefixes
// (below included).  With JUDGE also the mask of the bins that may hold a qualifying
// candidate and, as the return value, the highest bin whose top candidate qualifies (-1:
// none); without it the return value is -1.
template <int PER, bool JUDGE>
__device__ __forceinline__ int node_scan(const uint64_t* __restrict__ t, int nb, Pair below, double eps,
                                         Pair (&pre)[PER], unsigned& may, NodeShared& sh) {
  const int b0 = threadIdx.x * PER;
  Pair v[PER];
  Pair sum{0, 0};
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    v[j] = b0 + j < nb ? pair_of(t[b0 + j]) : Pair{0, 0};
    sum = sum + v[j];
  }
  Pair run = block_exclusive(sum, sh.scan) + below;
  may = 0;
  int top = -1;
  Pair top_incl{0, 0};
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    pre[j] = run;
    const Pair incl = run + v[j];
    if (JUDGE && v[j].c) {
      const double bound = v[j].r ? (double)incl.r / (double)(run.c + v[j].r) : (double)run.r / (double)(run.c + 1u);
      if (bound >= eps) may |= 1u << j;
      if ((double)incl.r / (double)incl.c >= eps) {
        top = b0 + j;
        top_incl = incl;
      }
    }
    run = incl;
  }
  if (!JUDGE) return -1;
  const int best = block_max(top, sh.red);
  if (best >= 0 && best == top) sh.at_top = top_incl;
  __syncthreads();
  return best;
}

// Pass 0: correctness bits and the key range.  One workgroup of 1024 per segment of kSegment
// tokens, a wave 8 x 64 consecutive tokens at a time.
__global__ __launch_bounds__(1024) void calib_pack_kernel(const float* __restrict__ H, const int* __restrict__ pred,
                                                          const int* __restrict__ ref, int64_t M, CalibWork w) {
  __shared__ uint32_t sh_lo[16], sh_hi[16];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t n_groups = (M + 63) >> 6;
  uint32_t lo = 0xFFFFFFFFu, hi = 0u;
  constexpr int U = 8;
  for (int k = 0; k < kSegment / (16 * U * 64); ++k) {
    const int64_t g0 = ((int64_t)blockIdx.x * (kSegment / (16 * U * 64)) + k) * (16 * U) + wave * U;
    float h[U];
    int a[U], b[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t i = ((g0 + u) << 6) + lane;
      const bool in = i < M;
      h[u] = in ? H[i] : NAN;
      a[u] = in ? __builtin_nontemporal_load(pred + i) : 0;
      b[u] = in ? __builtin_nontemporal_load(ref + i) : 1;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const unsigned long long ok = __ballot(a[u] == b[u]);
      if (g0 + u < n_groups && lane == 0) w.bits[g0 + u] = ok;
      if (h[u] == h[u]) {
        const uint32_t key = ascending_key(h[u]);
        lo = key < lo ? key : lo;
        hi = key > hi ? key : hi;
      }
    }
  }
#pragma unroll
  for (int o = 32; o; o >>= 1) {
    const uint32_t l2 = __shfl_xor(lo, o), h2 = __shfl_xor(hi, o);
    lo = l2 < lo ? l2 : lo;
    hi = h2 > hi ? h2 : hi;
  }
  if (lane == 0) {
    sh_lo[wave] = lo;
    sh_hi[wave] = hi;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int k = 1; k < 16; ++k) {
      lo = sh_lo[k] < lo ? sh_lo[k] : lo;
      hi = sh_hi[k] > hi ? sh_hi[k] : hi;
    }
    if (lo <= hi) {
      atomicMin(w.key_min, lo);
      atomicMax(w.key_max, hi);
    }
  }
}

// The tokens a lane holds of one trip: 8, from 8 consecutive groups of 64 (a workgroup of 1024
// takes 8192 consecutive tokens per trip).
struct Trip {
  float h[8];
  unsigned long long ok[8];
};
__device__ __forceinline__ Trip load_trip(const float* __restrict__ H, int64_t M, const CalibWork& w, int64_t trip) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t n_groups = (M + 63) >> 6;
  Trip t;
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    const int64_t g = trip * (blockDim.x / 64 * 8) + wave * 8 + u;
    const int64_t i = (g << 6) + lane;
    t.h[u] = i < M ? H[i] : NAN;
    t.ok[u] = g < n_groups ? w.bits[g] : 0ull;
  }
  return t;
}
// f(u, valid, key offset from the range's base, correct) for the lane's 8 tokens; `valid` is
// false for a NaN entropy or a token past the end.
template <class F>
__device__ __forceinline__ void for_trip(const Trip& t, uint32_t base, F&& f) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int u = 0; u < 8; ++u) f(u, t.h[u] == t.h[u], ascending_key(t.h[u]) - base, (unsigned)((t.ok[u] >> lane) & 1ull));
}

// Pass 1: one workgroup (of 1024) per segment of kSegment tokens counts into 16 + 16 bit bins
// of its own in LDS (no bin can hold more than the segment) and writes them out.
__global__ __launch_bounds__(1024) void calib_count1_kernel(const float* __restrict__ H, int64_t M, CalibWork w) {
  __shared__ uint32_t bins[kBins1];
  for (int b = threadIdx.x; b < kBins1; b += 1024) bins[b] = 0;
  __syncthreads();
  const Cut c = cut_of(w);
  if (!c.empty)
    for (int k = 0; k < kSegment / (4 * kChunk); ++k)
      for_trip(load_trip(H, M, w, (int64_t)blockIdx.x * (kSegment / (4 * kChunk)) + k), c.base,
               [&](int, bool valid, uint32_t off, unsigned ok) {
                 if (valid) atomicAdd(&bins[off >> c.s & (kBins1 - 1)], 1u + (ok << 16));
               });
  __syncthreads();
  uint32_t* out = w.part1 + (size_t)blockIdx.x * kBins1;
  for (int b = threadIdx.x; b < kBins1; b += 1024) out[b] = bins[b];
}
// grid (kBins1 / 256, 16): each thread adds up one bin over a sixteenth of the segments.
__global__ __launch_bounds__(256) void calib_sum1_kernel(CalibWork w, int n_parts) {
  const int b = blockIdx.x * 256 + threadIdx.x;
  const int per = (n_parts + gridDim.y - 1) / gridDim.y;
  const int p0 = blockIdx.y * per, p1 = p0 + per < n_parts ? p0 + per : n_parts;
  uint32_t cnt = 0, cor = 0;
#pragma unroll 8
  for (int p = p0; p < p1; ++p) {
    const uint32_t v = w.part1[(size_t)p * kBins1 + b];
    cnt += v & 0xFFFFu;
    cor += v >> 16;
  }
  if (cnt) atomicAdd((unsigned long long*)&w.h1[b], (unsigned long long)cnt | ((unsigned long long)cor << 32));
}

// A workgroup barrier that orders LDS traffic only: counts sent to memory by atomics that
// return nothing are not waited for.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// table[idx] += (1, ok) for the lanes that are `on`; lanes of a wave that name the same word
// (tokens of one entropy value sit together in the data as often as not) add once for all.
__device__ __forceinline__ void add_counted(uint64_t* __restrict__ table, uint32_t idx, bool on, unsigned ok) {
  unsigned long long pending = __ballot(on);
  const unsigned long long right = __ballot(on && ok);
  const int lane = threadIdx.x & 63;
  while (pending) {  // uniform over the wave
    const int leader = __builtin_ctzll(pending);
    const uint32_t word = __shfl(idx, leader);
    const unsigned long long same = __ballot(on && idx == word);
    if (lane == leader)
      atomicAdd((unsigned long long*)&table[word],
                (unsigned long long)__popcll(same) | ((unsigned long long)__popcll(same & right) << 32));
    pending &= ~same;
  }
}

// Keeps a bin of a level for epsilon `e`; the first to keep it gives it a row in the next table.
__device__ __forceinline__ void keep_bin(uint64_t* sel, int* slot, int* n_kept, int cap, int* overflow, int e) {
  const uint64_t old = atomicOr((unsigned long long*)sel, 1ull << e);
  if (old == 0) {
    const int row = atomicAdd(n_kept, 1);
    if (row < cap)
      *slot = row;
    else
      *overflow = 0;
  }
}

// What the levels hand on, per epsilon: the kept bins in the order in which the next level
// walks them, with the counts below each, so that no later kernel has to scan a table again.
constexpr int kList2 = 256;  // kept level-2 bins of one epsilon
struct EpsWalk {
  int n1;                  // kept level-1 bins, ascending
  int bin1[kCap1];
  Pair below1[kCap1];
  int n2;                  // kept level-2 bins, descending: the order of the final walk
  uint32_t at2[kList2];    // index into sel2 / slot2: row of the level-1 bin * kBins2 + bin
  uint32_t hi2[kList2];    // the key bits above level 3: level-1 bin << b2 | bin
  Pair below2[kList2];
};

// Level 1, one workgroup per epsilon.
__global__ __launch_bounds__(256) void calib_keep1_kernel(CalibWork w, EpsList eps, EpsWalk* __restrict__ walks) {
  __shared__ NodeShared sh;
  __shared__ int bin[kCap1];
  constexpr int PER = kBins1 / 256;
  const int e = blockIdx.x;
  EpsWalk& walk = walks[e];
  Pair pre[PER];
  unsigned may;
  const int top = node_scan<PER, true>(w.h1, kBins1, Pair{0, 0}, eps.v[e], pre, may, sh);
  const int b0 = threadIdx.x * PER;
  unsigned mine = 0;
#pragma unroll
  for (int j = 0; j < PER; ++j) mine |= (unsigned)((may >> j & 1u) && b0 + j >= top) << j;
  int total;
  int k = (int)block_exclusive(Pair{(uint32_t)__popc(mine), 0u}, sh.scan, &total).c;
#pragma unroll
  for (int j = 0; j < PER; ++j)
    if ((mine >> j & 1u) && k < kCap1) {
      bin[k] = b0 + j;
      walk.bin1[k] = b0 + j;
      walk.below1[k] = pre[j];
      ++k;
    }
  if (threadIdx.x == 0) {
    walk.n1 = total < kCap1 ? total : kCap1;
    if (total > kCap1) *w.overflow = 0;
  }
  __syncthreads();
  // one bin per thread: the atomics of a workgroup are in flight together
  if ((int)threadIdx.x < total && threadIdx.x < kCap1) {
    const int b = bin[threadIdx.x];
    keep_bin(&w.sel1[b], &w.slot1[b], &w.n_kept[0], kCap1, w.overflow, e);
  }
}

// Pass 2: tokens of kept level-1 bins are counted by their next b2 bits and set aside for
// pass 3.  One workgroup of 1024 per segment, as in pass 1.
__global__ __launch_bounds__(1024) void calib_count2_kernel(const float* __restrict__ H, int64_t M, CalibWork w) {
  __shared__ __align__(16) signed char slot[kBins1];  // rows are below kCap1 = 128
  __shared__ uint32_t stage[16][kStageWave];  // a region per wave: no barrier while the tokens stream
  __shared__ int n_wave[16], at;
  // everything the kernel needs before the tokens is asked for at once: the latency is paid once
  const int ov = *w.overflow;
  const Cut c = cut_of(w);
  {
    constexpr int N = kBins1 / 4 / 1024;
    int4 v[N];
#pragma unroll
    for (int k = 0; k < N; ++k) v[k] = ((const int4*)w.slot1)[k * 1024 + threadIdx.x];
#pragma unroll
    for (int k = 0; k < N; ++k) {
      char4 c4;
      c4.x = (signed char)v[k].x, c4.y = (signed char)v[k].y, c4.z = (signed char)v[k].z, c4.w = (signed char)v[k].w;
      ((char4*)slot)[k * 1024 + threadIdx.x] = c4;
    }
  }
  __syncthreads();
  if (ov == 0 || c.empty) return;
  const uint32_t ms = (1u << c.s) - 1u;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t* mine = stage[wave];
  int n = 0;  // uniform over the wave
  constexpr int kTrips = kSegment / (4 * kChunk);
  for (int k = 0; k < kTrips; ++k) {
    const Trip t = load_trip(H, M, w, (int64_t)blockIdx.x * kTrips + k);
    int rows[8];  // all eight table look-ups of a trip in flight together
    for_trip(t, c.base, [&](int u, bool valid, uint32_t off, unsigned) {
      rows[u] = valid ? slot[off >> c.s & (kBins1 - 1)] : -1;
    });
    for_trip(t, c.base, [&](int u, bool, uint32_t off, unsigned ok) {
      const int row = rows[u];
      const unsigned long long on = __ballot(row >= 0);
      if (!on) return;  // uniform over the wave
      const uint32_t within = off & ms;
      add_counted(w.h2, (uint32_t)row * kBins2 + (within >> c.b3), row >= 0, ok);
      if (n + 64 > kStageWave) {  // a wave whose tokens are mostly kept: it appends what it holds by itself
        int first = 0;
        if (lane == 0) first = atomicAdd(&w.n_kept[2], n);
        first = __shfl(first, 0);
        for (int i = lane; i < n; i += 64) w.kept[first + i] = mine[i];
        n = 0;
      }
      if (row >= 0) mine[n + __popcll(on & ((1ull << lane) - 1ull))] = (ok << 31) | ((uint32_t)row << 20) | within;
      n += __popcll(on);
    });
  }
  // the workgroup appends what its waves still hold with one reservation
  if (lane == 0) n_wave[wave] = n;
  lds_barrier();
  if (threadIdx.x == 0) {
    int total = 0;
    for (int k = 0; k < 16; ++k) total += n_wave[k];
    at = total ? atomicAdd(&w.n_kept[2], total) : 0;
  }
  lds_barrier();
  int first = at;
  for (int k = 0; k < wave; ++k) first += n_wave[k];
  for (int i = lane; i < n; i += 64) w.kept[first + i] = mine[i];
}

// One node for one wave: nb <= 64 * PER bins, lane l looks at bins [PER * l, PER * (l + 1)).
// As node_scan with JUDGE; the counts up to and including the bin returned come back in at_top.
template <int PER>
__device__ __forceinline__ int wave_node_scan(const uint64_t* __restrict__ t, int nb, Pair below, double eps,
                                              Pair (&pre)[PER], unsigned& may, Pair& at_top) {
  const int lane = threadIdx.x & 63;
  const int b0 = lane * PER;
  Pair v[PER];
  Pair sum{0, 0};
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    v[j] = b0 + j < nb ? pair_of(t[b0 + j]) : Pair{0, 0};
    sum = sum + v[j];
  }
  Pair inc = sum;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t c = __shfl_up(inc.c, o), r = __shfl_up(inc.r, o);
    if (lane >= o) inc = inc + Pair{c, r};
  }
  Pair run{below.c + inc.c - sum.c, below.r + inc.r - sum.r};
  may = 0;
  int top = -1;
  Pair top_incl{0, 0};
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    pre[j] = run;
    const Pair incl = run + v[j];
    if (v[j].c) {
      const double bound = v[j].r ? (double)incl.r / (double)(run.c + v[j].r) : (double)run.r / (double)(run.c + 1u);
      if (bound >= eps) may |= 1u << j;
      if ((double)incl.r / (double)incl.c >= eps) {
        top = b0 + j;
        top_incl = incl;
      }
    }
    run = incl;
  }
  int best = top;
#pragma unroll
  for (int o = 32; o; o >>= 1) {
    const int u = __shfl_xor(best, o);
    best = u > best ? u : best;
  }
  const int owner = best >= 0 ? best / PER : 0;
  at_top = Pair{(uint32_t)__shfl((int)top_incl.c, owner), (uint32_t)__shfl((int)top_incl.r, owner)};
  return best;
}

// Level 2, one workgroup per epsilon: down the kept level-1 bins, four at a time (a wave
// each), until a top candidate qualifies.
__global__ __launch_bounds__(256) void calib_keep2_kernel(CalibWork w, EpsList eps, EpsWalk* __restrict__ walks) {
  __shared__ int top_w[4], cnt_w[4];
  __shared__ uint32_t at2[kList2];
  constexpr int PER = kBins2 / 64;
  const int ov = *w.overflow;
  const Cut c = cut_of(w);
  const int e = blockIdx.x;
  EpsWalk& walk = walks[e];
  const int n1 = walk.n1;
  if (ov == 0) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int n2 = 0;  // uniform over the workgroup
  for (int r = 0; 4 * r < n1; ++r) {
    const int i = n1 - 1 - (4 * r + wave);  // uniform over the wave
    int top = -1, cnt = 0, before = 0, row = 0, bin1 = 0;
    unsigned keep = 0;
    Pair pre[PER];
    if (i >= 0) {
      bin1 = walk.bin1[i];
      row = w.slot1[bin1];
      unsigned may;
      Pair at_top;
      top = wave_node_scan<PER>(w.h2 + (size_t)row * kBins2, 1 << c.b2, walk.below1[i], eps.v[e], pre, may, at_top);
#pragma unroll
      for (int j = 0; j < PER; ++j) keep |= (unsigned)((may >> j & 1u) && lane * PER + j >= top) << j;
      int inc = __popc(keep);
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int u = __shfl_up(inc, o);
        if (lane >= o) inc += u;
      }
      before = inc - __popc(keep);
      cnt = __shfl(inc, 63);
    }
    if (lane == 0) {
      top_w[wave] = top;
      cnt_w[wave] = cnt;
    }
    __syncthreads();
    int stop = 4, first = n2, all = 0;
    for (int k = 3; k >= 0; --k)
      if (top_w[k] >= 0) stop = k;
    for (int k = 0; k < 4 && k <= stop; ++k) {
      if (k < wave) first += cnt_w[k];
      all += cnt_w[k];
    }
    if (i >= 0 && wave <= stop) {  // the bins of this node, from the top
      int at = first + cnt - 1 - before;
#pragma unroll
      for (int j = 0; j < PER; ++j)
        if (keep >> j & 1u) {
          if (at < kList2) {
            at2[at] = (uint32_t)row * kBins2 + lane * PER + j;
            walk.at2[at] = (uint32_t)row * kBins2 + lane * PER + j;
            walk.hi2[at] = ((uint32_t)bin1 << c.b2) | (uint32_t)(lane * PER + j);
            walk.below2[at] = pre[j];
          }
          --at;
        }
    }
    n2 += all;
    __syncthreads();  // top_w and cnt_w are rewritten in the next round
    if (stop < 4) break;  // uniform: every smaller key is below one that qualifies
  }
  if (threadIdx.x == 0) {
    walk.n2 = n2 < kList2 ? n2 : kList2;
    if (n2 > kList2) *w.overflow = 0;
  }
  for (int k = threadIdx.x; k < n2 && k < kList2; k += 256)
    keep_bin(&w.sel2[at2[k]], &w.slot2[at2[k]], &w.n_kept[1], kCap2, w.overflow, e);
}

// Pass 3: the tokens set aside whose level-2 bin is kept are counted by their last b3 bits,
// that is, by key.
__global__ __launch_bounds__(256) void calib_count3_kernel(CalibWork w) {
  if (*w.overflow == 0) return;
  const Cut c = cut_of(w);
  const int n = w.n_kept[2];
  const uint32_t m3 = (1u << c.b3) - 1u;
  for (int i0 = blockIdx.x * 256; i0 < n; i0 += gridDim.x * 256) {  // uniform over the workgroup
    const int i = i0 + threadIdx.x;
    const uint32_t v = i < n ? w.kept[i] : 0u;
    const uint32_t within = v & 0xFFFFFu, row1 = (v >> 20) & 127u;
    const int row = i < n ? w.slot2[(size_t)row1 * kBins2 + (within >> c.b3)] : -1;
    add_counted(w.h3, (uint32_t)row * kBins3 + (within & m3), row >= 0, v >> 31);
  }
}

// Level 3, one workgroup per epsilon: the first single key, from the top, that qualifies.
// Four kept level-2 bins at a time, a wave each.
__global__ __launch_bounds__(256) void calib_pick_kernel(CalibWork w, EpsList eps, const EpsWalk* __restrict__ walks,
                                                         float* __restrict__ tau, long long* __restrict__ n_exit) {
  __shared__ int top_w[4];
  __shared__ uint32_t cnt_w[4];
  constexpr int PER = kBins3 / 64;
  const int ov = *w.overflow;
  const Cut c = cut_of(w);
  const int e = blockIdx.x;
  const EpsWalk& walk = walks[e];
  const int n2 = walk.n2;
  if (ov == 0) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int r = 0; 4 * r < n2; ++r) {
    const int q = 4 * r + wave;  // uniform over the wave
    int top = -1;
    Pair at_top{0, 0};
    if (q < n2) {
      const int row = w.slot2[walk.at2[q]];
      Pair pre[PER];
      unsigned may;
      top = wave_node_scan<PER>(w.h3 + (size_t)row * kBins3, 1 << c.b3, walk.below2[q], eps.v[e], pre, may, at_top);
    }
    if (lane == 0) {
      top_w[wave] = top;
      cnt_w[wave] = at_top.c;
    }
    __syncthreads();
    for (int k = 0; k < 4; ++k)
      if (top_w[k] >= 0) {  // uniform
        if (threadIdx.x == 0) {
          tau[e] = ascending_entropy(c.base + ((walk.hi2[4 * r + k] << c.b3) | (uint32_t)top_w[k]));
          if (n_exit) n_exit[e] = (long long)cnt_w[k];
        }
        return;
      }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    tau[e] = -INFINITY;
    if (n_exit) n_exit[e] = 0;
  }
}

// Presets the tables: n0 words of 0 from p0, n1 words of -1 from p1.
__global__ __launch_bounds__(256) void calib_preset_kernel(int* __restrict__ p0, int64_t n0, int* __restrict__ p1,
                                                           int64_t n1) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n0)
    p0[i] = 0;
  else if (i - n0 < n1)
    p1[i - n0] = -1;
}

}  // namespace

namespace {

// Grows the call scratch; an earlier call may still be using the old buffer on some stream.
hipError_t calib_reserve(CalibScratch& sc, size_t need) {
  if (sc.bytes >= need) return hipSuccess;
  hipError_t e = hipDeviceSynchronize();
  if (e != hipSuccess) return e;
  if (sc.buf) (void)hipFree(sc.buf);
  sc.buf = nullptr;
  sc.bytes = 0;
  e = hipMalloc(&sc.buf, need);
  if (e != hipSuccess) return e;
  sc.bytes = need;
  return hipSuccess;
}

// The full sort: always enough, about 60 bytes of traffic per token.
hipError_t calibrate_sort(CalibScratch& sc, const float* H, const int* pred, const int* ref, int64_t M,
                          const EpsList& el, float* tau_out, long long* n_exit_out, hipStream_t s) {
  const int n_eps = el.n;
  size_t tmp_sort = 0, tmp_scan = 0;
  hipError_t e = rocprim::radix_sort_pairs(nullptr, tmp_sort, (uint32_t*)nullptr, (uint32_t*)nullptr,
                                           (uint32_t*)nullptr, (uint32_t*)nullptr, (size_t)M, 0u, 32u, s);
  if (e == hipSuccess)
    e = rocprim::inclusive_scan(nullptr, tmp_scan, (uint32_t*)nullptr, (uint32_t*)nullptr, (size_t)M,
                                rocprim::plus<uint32_t>(), s);
  if (e != hipSuccess) return e;
  const size_t tmp_bytes = ((tmp_sort > tmp_scan ? tmp_sort : tmp_scan) + 255) & ~(size_t)255;
  // one buffer: keys_in, vals_in, keys_out, vals_out, prefix (M words each), bests, primitive scratch
  const size_t words = 5 * (size_t)M + kMaxEps;
  e = calib_reserve(sc, words * sizeof(uint32_t) + 256 + tmp_bytes);
  if (e != hipSuccess) return e;
  uint32_t* buf = (uint32_t*)sc.buf;
  uint32_t *k0 = buf, *v0 = buf + M, *k1 = buf + 2 * M, *v1 = buf + 3 * M, *pf = buf + 4 * M;
  unsigned* best = buf + 5 * M;
  void* tmp = (char*)sc.buf + ((words * sizeof(uint32_t) + 255) & ~(size_t)255);
  const unsigned grid = (unsigned)((M + 255) / 256);
  hipLaunchKernelGGL(calib_keys_kernel, dim3(grid), dim3(256), 0, s, H, pred, ref, M, k0, v0);
  size_t ts = tmp_bytes;
  e = rocprim::radix_sort_pairs(tmp, ts, k0, k1, v0, v1, (size_t)M, 0u, 32u, s);
  ts = tmp_bytes;
  if (e == hipSuccess) e = rocprim::inclusive_scan(tmp, ts, v1, pf, (size_t)M, rocprim::plus<uint32_t>(), s);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(calib_init_kernel, dim3(1), dim3(kMaxEps), 0, s, best, n_eps, (unsigned)M);
  hipLaunchKernelGGL(calib_search_kernel, dim3((unsigned)((M + 1023) / 1024)), dim3(1024), 0, s, k1, pf, M, el,
                     best);
  hipLaunchKernelGGL(calib_read_kernel, dim3(1), dim3(kMaxEps), 0, s, k1, best, n_eps, (unsigned)M, tau_out,
                     n_exit_out);
  return hipGetLastError();
}

// The refinement.  *enough comes back false if a table was too small for the data (the
// outputs are then not written).  Waits for the stream: the flag is read on the host.
hipError_t calibrate_refine(CalibScratch& sc, const float* H, const int* pred, const int* ref, int64_t M,
                            const EpsList& el, float* tau_out, long long* n_exit_out, hipStream_t s, bool* enough) {
  hipError_t e;
  if (!sc.host_flag) {
    e = hipHostMalloc((void**)&sc.host_flag, sizeof(int), hipHostMallocDefault);
    if (e != hipSuccess) return e;
  }
  const size_t n_groups = (size_t)((M + 63) >> 6);
  const size_t n_segments = (size_t)((M + kSegment - 1) / kSegment);
  const size_t kept_cap = (size_t)M;
  const size_t zero_words = 4 + 2 * ((size_t)kBins1 + kBins1 + 2 * (size_t)kCap1 * kBins2 + (size_t)kCap2 * kBins3);
  const size_t ones_words = 4 + (size_t)kBins1 + (size_t)kCap1 * kBins2;
  e = calib_reserve(sc, (2 * n_groups + n_segments * kBins1 + kept_cap + 8 + zero_words + ones_words) * 4 + kMaxEps * sizeof(EpsWalk) + 256);
  if (e != hipSuccess) return e;
  CalibWork w;
  uint32_t* p = (uint32_t*)sc.buf;
  w.bits = (uint64_t*)p;
  p += (2 * n_groups + 3) & ~(size_t)3;
  w.part1 = p;
  p += n_segments * kBins1;
  w.kept = p;
  p += (kept_cap + 3) & ~(size_t)3;
  uint32_t* zero0 = p;
  w.key_max = p;
  w.n_kept = (int*)(p + 1);
  p += 4;
  w.h1 = (uint64_t*)p;
  p += 2 * kBins1;
  w.sel1 = (uint64_t*)p;
  p += 2 * kBins1;
  w.h2 = (uint64_t*)p;
  p += 2 * (size_t)kCap1 * kBins2;
  w.sel2 = (uint64_t*)p;
  p += 2 * (size_t)kCap1 * kBins2;
  w.h3 = (uint64_t*)p;
  p += 2 * (size_t)kCap2 * kBins3;
  uint32_t* ones0 = p;
  w.key_min = p;
  w.overflow = (int*)(p + 1);
  p += 4;  // slot1 is read 16 bytes at a time
  w.slot1 = (int*)p;
  p += kBins1;
  w.slot2 = (int*)p;
  p += (size_t)kCap1 * kBins2;
  EpsWalk* walks = (EpsWalk*)p;
  hipLaunchKernelGGL(calib_preset_kernel, dim3((unsigned)((zero_words + ones_words + 255) / 256)), dim3(256), 0, s,
                     (int*)zero0, (int64_t)zero_words, (int*)ones0, (int64_t)ones_words);
  hipLaunchKernelGGL(calib_pack_kernel, dim3((unsigned)n_segments), dim3(1024), 0, s, H, pred, ref, M, w);
  hipLaunchKernelGGL(calib_count1_kernel, dim3((unsigned)n_segments), dim3(1024), 0, s, H, M, w);
  hipLaunchKernelGGL(calib_sum1_kernel, dim3(kBins1 / 256, 16), dim3(256), 0, s, w, (int)n_segments);
  hipLaunchKernelGGL(calib_keep1_kernel, dim3(el.n), dim3(256), 0, s, w, el, walks);
  hipLaunchKernelGGL(calib_count2_kernel, dim3((unsigned)n_segments), dim3(1024), 0, s, H, M, w);
  hipLaunchKernelGGL(calib_keep2_kernel, dim3(el.n), dim3(256), 0, s, w, el, walks);
  hipLaunchKernelGGL(calib_count3_kernel, dim3(256), dim3(256), 0, s, w);
  hipLaunchKernelGGL(calib_pick_kernel, dim3(el.n), dim3(256), 0, s, w, el, walks, tau_out, n_exit_out);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  e = hipMemcpyAsync(sc.host_flag, w.overflow, sizeof(int), hipMemcpyDeviceToHost, s);
  if (e != hipSuccess) return e;
  e = hipStreamSynchronize(s);
  if (e != hipSuccess) return e;
  *enough = *sc.host_flag != 0;
  return hipSuccess;
}

}  // namespace

hipError_t calibrate_run(CalibScratch& sc, const float* H, const int* pred, const int* ref, int64_t M,
                         const double* eps, int n_eps, float* tau_out, long long* n_exit_out, hipStream_t s) {
  EpsList el;
  el.n = n_eps;
  for (int i = 0; i < n_eps; ++i) el.v[i] = eps[i];
  const char* force = getenv("EH_CALIBRATE_SORT");
  bool enough = false;
  if (!(force && force[0] == '1') && M <= kRefineMax) {
    const hipError_t e = calibrate_refine(sc, H, pred, ref, M, el, tau_out, n_exit_out, s, &enough);
    if (e != hipSuccess) return e;
  }
  if (enough) return hipSuccess;
  ++sc.n_sorted;
  return calibrate_sort(sc, H, pred, ref, M, el, tau_out, n_exit_out, s);
}

}  // namespace eh
