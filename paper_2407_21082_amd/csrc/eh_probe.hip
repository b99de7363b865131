// Measurement kernels of libeh (see include/eh_probe.h): a plain read of the
// context's weight buffers and a registers-only matrix-core instruction stream.
// They give the practical ceilings beside the published peaks; nothing of the
// method (arXiv 2407.21082) is computed here.
#include "eh_probe.h"

#include <hip/hip_runtime.h>

#include <string>

#include "eh_internal.hpp"

using namespace eh;

namespace {

#define EH_LDS __attribute__((address_space(3)))
#define EH_GLOBAL __attribute__((address_space(1)))
typedef EH_GLOBAL const frag_t gfrag_t;

constexpr int kReadWaves = 8;   // register variant: waves per workgroup
constexpr int kRing = 4;        // fragments per register buffer (two buffers per wave)
constexpr int kLdsWaves = 4;    // LDS variant: waves per workgroup
constexpr int kLdsSlots = 16;   // 1 KiB slots per wave
constexpr int kLdsBatch = 4;    // loads issued between two waits

__device__ __forceinline__ gfrag_t* table_entry(const frag_t* const* table, int l) {
  typedef const frag_t* entry_t;
  typedef __attribute__((address_space(4))) const entry_t centry_t;
  return (gfrag_t*)((centry_t*)table)[l];
}

// Fragments [f0, f1) of every head in turn through two alternating register buffers, so that
// 4 to 8 KiB per wave are always in flight, across head boundaries too.
__global__ __launch_bounds__(kReadWaves * kWave, 1) void probe_read_reg_kernel(const frag_t* const* __restrict__ Wf,
                                                                               int l0, int l1, long long frags,
                                                                               uint32_t* __restrict__ sink) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const long long lo = frags * blockIdx.x / gridDim.x, hi = frags * (blockIdx.x + 1) / gridDim.x;
  const long long f0 = lo + (hi - lo) * wave / kReadWaves, f1 = lo + (hi - lo) * (wave + 1) / kReadWaves;
  const int n = (int)(f1 - f0);
  const int last = n > 0 ? n - 1 : 0;
  const int G = (n + kRing - 1) / kRing, G2 = (G + 1) & ~1;
  uint32_t acc = 0;
  frag_t bufA[kRing], bufB[kRing];
  auto load = [&](gfrag_t* head, int idx) { return __builtin_nontemporal_load(head + (f0 + min(idx, last)) * kWave + lane); };
  auto fold = [&](const frag_t (&b)[kRing]) {
#pragma unroll
    for (int j = 0; j < kRing; ++j) acc ^= b[j].x ^ b[j].y ^ b[j].z ^ b[j].w;
  };
  {
    gfrag_t* h0 = table_entry(Wf, l0);
#pragma unroll
    for (int j = 0; j < kRing; ++j) bufA[j] = load(h0, j);
#pragma unroll
    for (int j = 0; j < kRing; ++j) bufB[j] = load(h0, kRing + j);
  }
  for (int l = l0; l < l1; ++l) {
    gfrag_t* cur = table_entry(Wf, l);
    gfrag_t* nxt = l + 1 < l1 ? table_entry(Wf, l + 1) : cur;
    for (int g = 0; g < G2; g += 2) {
      fold(bufA);
      {
        const bool same = g + 2 < G2;
        gfrag_t* src = same ? cur : nxt;
        const int base = (same ? g + 2 : 0) * kRing;
#pragma unroll
        for (int j = 0; j < kRing; ++j) bufA[j] = load(src, base + j);
      }
      fold(bufB);
      {
        const bool same = g + 3 < G2;
        gfrag_t* src = same ? cur : nxt;
        const int base = (same ? g + 3 : 1) * kRing;
#pragma unroll
        for (int j = 0; j < kRing; ++j) bufB[j] = load(src, base + j);
      }
    }
  }
  fold(bufA);
  fold(bufB);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) acc ^= __shfl_xor(acc, o);
  if (lane == 0) atomicXor(&sink[blockIdx.x], acc);
}

// The same span per wave, 16 bytes per lane straight into a ring of LDS slots (the load path of
// the batched kernel); kLdsSlots - kLdsBatch KiB per wave stay in flight.
__global__ __launch_bounds__(kLdsWaves * kWave, 1) void probe_read_lds_kernel(const frag_t* const* __restrict__ Wf,
                                                                              int l0, int l1, long long frags,
                                                                              uint32_t* __restrict__ sink) {
  __shared__ __attribute__((aligned(16))) char ring[kLdsWaves * kLdsSlots * 1024];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const long long lo = frags * blockIdx.x / gridDim.x, hi = frags * (blockIdx.x + 1) / gridDim.x;
  const long long f0 = lo + (hi - lo) * wave / kLdsWaves, f1 = lo + (hi - lo) * (wave + 1) / kLdsWaves;
  const int n = (int)(f1 - f0);
  const int last = n > 0 ? n - 1 : 0;
  EH_LDS char* mine = (EH_LDS char*)ring + wave * kLdsSlots * 1024;
  int slot = 0;
  for (int l = l0; l < l1; ++l) {
    const EH_GLOBAL char* src = (const EH_GLOBAL char*)table_entry(Wf, l) + ((f0 * kWave + lane) << 4);
    for (int i = 0; i < n; i += kLdsBatch) {
#pragma unroll
      for (int j = 0; j < kLdsBatch; ++j) {
        const long long f = min(i + j, last);
        __builtin_amdgcn_global_load_lds((const EH_GLOBAL void*)(src + (f << 10)), (EH_LDS void*)(mine + slot * 1024), 16,
                                         0, 0);
        slot = (slot + 1) & (kLdsSlots - 1);
      }
      // at most kLdsSlots - kLdsBatch loads may still be on their way: the slots the next batch
      // overwrites have landed
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kLdsSlots - kLdsBatch) : "memory");
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  const uint32_t v = *(EH_LDS uint32_t*)(mine + lane * 4);
  uint32_t acc = v;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) acc ^= __shfl_xor(acc, o);
  if (lane == 0) atomicXor(&sink[blockIdx.x], acc);
}

typedef __attribute__((ext_vector_type(8))) __bf16 pbf16x8;
typedef __attribute__((ext_vector_type(16))) float pf32x16;

__device__ __forceinline__ pbf16x8 probe_operand(unsigned s, bool zero) {
  pbf16x8 v;
  for (int i = 0; i < 8; ++i) {
    unsigned h = (threadIdx.x * 2654435761u + i * 40503u + s * 97u + blockIdx.x * 7919u);
    h ^= h >> 13;
    h *= 0x5bd1e995u;
    h ^= h >> 15;
    v[i] = zero ? (__bf16)0.0f : (__bf16)(((int)(h & 0xffff) - 32768) * (1.0f / 32768.f));
  }
  return v;
}

// 7 x 2 accumulator tiles of 32 x 32, two k halves: the register tile of the batched kernel
__global__ __launch_bounds__(256, 1) void probe_mfma_kernel(float* __restrict__ out, int iters, int zero) {
  constexpr int MT = 7, NB = 2;
  pbf16x8 a[MT][2], b[NB][2];
  for (int m = 0; m < MT; ++m)
    for (int h = 0; h < 2; ++h) a[m][h] = probe_operand(1 + m * 2 + h, zero);
  for (int n = 0; n < NB; ++n)
    for (int h = 0; h < 2; ++h) b[n][h] = probe_operand(101 + n * 2 + h, zero);
  pf32x16 acc[MT][NB];
  for (int m = 0; m < MT; ++m)
    for (int n = 0; n < NB; ++n)
      for (int j = 0; j < 16; ++j) acc[m][n][j] = 0;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
      for (int n = 0; n < NB; ++n)
#pragma unroll
        for (int h = 0; h < 2; ++h)
          acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[m][h], b[n][h], acc[m][n], 0, 0, 0);
    asm volatile("" : "+v"(a[0][0]), "+v"(b[0][0]));  // nothing may be hoisted out of the loop
  }
  float s = 0;
  for (int m = 0; m < MT; ++m)
    for (int n = 0; n < NB; ++n)
      for (int j = 0; j < 16; ++j) s += acc[m][n][j];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

eh_status probe_fail(eh_ctx* ctx, eh_status st, const char* msg) {
  ctx->err = msg;
  return st;
}

}  // namespace

extern "C" {

eh_status eh_probe_read_weights(eh_ctx* ctx, int32_t how, int32_t per_head, int32_t head0, int32_t n_heads_read,
                                uint32_t* sink, int64_t* bytes_out, void* stream) {
  if (!ctx) return EH_ERR_NULL;
  if (!sink) return probe_fail(ctx, EH_ERR_NULL, "sink is NULL");
  if (how != EH_PROBE_READ_REGISTERS && how != EH_PROBE_READ_LDS) return probe_fail(ctx, EH_ERR_RANGE, "unknown read variant");
  if (head0 < 0 || n_heads_read < 1 || head0 + n_heads_read > ctx->n_heads) return probe_fail(ctx, EH_ERR_RANGE, "heads out of range");
  const int grid = ctx->num_cu > 0 && ctx->num_cu <= 1024 ? ctx->num_cu : 256;
  const long long frags = (long long)ctx->VT * ctx->KS;
  if (frags < (long long)grid * kReadWaves * 2 * kRing) return probe_fail(ctx, EH_ERR_SHAPE, "weights too small for the read probe");
  if (bytes_out) *bytes_out = frags * 1024 * n_heads_read;
  int prev = -1;
  (void)hipGetDevice(&prev);
  if (prev != ctx->device) (void)hipSetDevice(ctx->device);
  hipStream_t s = (hipStream_t)stream;
  const int l1 = head0 + n_heads_read;
  for (int l = head0; l < l1; l += per_head ? 1 : n_heads_read) {
    const int le = per_head ? l + 1 : l1;
    if (how == EH_PROBE_READ_REGISTERS)
      hipLaunchKernelGGL(probe_read_reg_kernel, dim3(grid), dim3(kReadWaves * kWave), 0, s,
                         (const frag_t* const*)ctx->d_Wf, l, le, frags, sink);
    else
      hipLaunchKernelGGL(probe_read_lds_kernel, dim3(grid), dim3(kLdsWaves * kWave), 0, s,
                         (const frag_t* const*)ctx->d_Wf, l, le, frags, sink);
  }
  const hipError_t e = hipGetLastError();
  if (prev >= 0 && prev != ctx->device) (void)hipSetDevice(prev);
  if (e != hipSuccess) {
    ctx->err = std::string("read probe launch: ") + hipGetErrorString(e);
    return EH_ERR_HIP;
  }
  return EH_OK;
}

eh_status eh_probe_mfma(eh_ctx* ctx, int32_t iters, int32_t random_operands, float* sink, double* flops_out,
                        void* stream) {
  if (!ctx) return EH_ERR_NULL;
  if (!sink) return probe_fail(ctx, EH_ERR_NULL, "sink is NULL");
  if (iters < 1 || iters > (1 << 20)) return probe_fail(ctx, EH_ERR_RANGE, "iters outside [1, 2^20]");
  const int grid = ctx->num_cu > 0 && ctx->num_cu <= 1024 ? ctx->num_cu : 256;
  if (flops_out) *flops_out = 2.0 * 32 * 32 * 16 * 28 * (double)iters * grid * 4;
  int prev = -1;
  (void)hipGetDevice(&prev);
  if (prev != ctx->device) (void)hipSetDevice(ctx->device);
  hipLaunchKernelGGL(probe_mfma_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, sink, iters, random_operands ? 0 : 1);
  const hipError_t e = hipGetLastError();
  if (prev >= 0 && prev != ctx->device) (void)hipSetDevice(prev);
  if (e != hipSuccess) {
    ctx->err = std::string("mfma probe launch: ") + hipGetErrorString(e);
    return EH_ERR_HIP;
  }
  return EH_OK;
}

eh_status eh_probe_calibrate_sorted(eh_ctx* ctx, int64_t* calls_out) {
  if (!ctx || !calls_out) return EH_ERR_NULL;
  *calls_out = (int64_t)ctx->calib.n_sorted;
  return EH_OK;
}

}  // extern "C"
