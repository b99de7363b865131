// Threshold calibration on the device (arXiv 2407.21082, Section 3.4.1,
// "Calibration of Confidence Thresholds"), entropy as the confidence metric.
//
// For one head: the M calibration tokens are sorted by ascending confidence
// (descending entropy) together with their correctness bits (eq. (2): the
// head's prediction equals the model's), the correct ones are counted by a
// running sum, and for every requested level epsilon the first position in that
// order is found whose suffix -- all tokens at least as confident -- holds a
// proportion of correct predictions of at least epsilon; tau is the entropy at
// that position.  Ties are taken as a whole (only the first position of a run
// of equal entropies is a candidate), NaN entropies are no candidates and are in
// no suffix, and "no position qualifies" gives tau = -inf.
//
// The sort and the running sum are rocPRIM's device-wide primitives (a plain
// radix sort of 32-bit keys with 32-bit values, an inclusive scan); the key
// transform, the candidate search for all epsilon at once and the read-out are
// kernels of this file.  The whole thing is bound by memory traffic: about 60
// bytes per token over all passes.
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

}  // namespace

hipError_t calibrate_run(CalibScratch& sc, const float* H, const int* pred, const int* ref, int64_t M,
                         const double* eps, int n_eps, float* tau_out, long long* n_exit_out, hipStream_t s) {
  EpsList el;
  el.n = n_eps;
  for (int i = 0; i < n_eps; ++i) el.v[i] = eps[i];
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
  const size_t need = words * sizeof(uint32_t) + 256 + tmp_bytes;
  if (sc.bytes < need) {
    // grow only; an earlier call may still be using the old buffer on some stream
    e = hipDeviceSynchronize();
    if (e != hipSuccess) return e;
    if (sc.buf) (void)hipFree(sc.buf);
    sc.buf = nullptr;
    sc.bytes = 0;
    e = hipMalloc(&sc.buf, need);
    if (e != hipSuccess) return e;
    sc.bytes = need;
  }
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

}  // namespace eh
