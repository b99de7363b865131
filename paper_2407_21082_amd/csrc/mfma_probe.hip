// Matrix-core rate probe for gfx950: what v_mfma_f32_32x32x16_bf16 and
// v_mfma_f32_16x16x32_bf16 sustain on this chip with registers as the only
// operands (no memory traffic in the timed part), one workgroup of 4 waves per CU.
// It gives the practical ceiling against which the batched projection kernel's
// MFMA fraction is to be read: the published peak (2.5 PFLOP/s dense bf16) is
// reached only on operands that do not toggle; on random operands the chip
// sustains markedly less.
//
//   mfma_probe            prints one line per case
#include <hip/hip_runtime.h>

#include <cstdio>

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ __forceinline__ bf16x8 operand(unsigned s, bool zero) {
  bf16x8 v;
  for (int i = 0; i < 8; ++i) {
    unsigned h = (threadIdx.x * 2654435761u + i * 40503u + s * 97u + blockIdx.x * 7919u);
    h ^= h >> 13;
    h *= 0x5bd1e995u;
    h ^= h >> 15;
    v[i] = zero ? (__bf16)0.0f : (__bf16)(((int)(h & 0xffff) - 32768) * (1.0f / 32768.f));
  }
  return v;
}

// MT x NB accumulator tiles of 32x32, two k halves: the register tile of the batched kernel
template <int MT, int NB>
__global__ __launch_bounds__(256, 1) void probe32(float* out, int iters, int zero) {
  bf16x8 a[MT][2], b[NB][2];
  for (int m = 0; m < MT; ++m)
    for (int h = 0; h < 2; ++h) a[m][h] = operand(1 + m * 2 + h, zero);
  for (int n = 0; n < NB; ++n)
    for (int h = 0; h < 2; ++h) b[n][h] = operand(101 + n * 2 + h, zero);
  f32x16 acc[MT][NB];
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

// NACC independent 16x16 accumulator tiles
template <int NACC>
__global__ __launch_bounds__(256, 1) void probe16(float* out, int iters, int zero) {
  const bf16x8 a = operand(1, zero), b = operand(2, zero);
  f32x4 acc[NACC];
  for (int i = 0; i < NACC; ++i) acc[i] = f32x4{0, 0, 0, 0};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < NACC; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[i], 0, 0, 0);
  }
  float s = 0;
  for (int i = 0; i < NACC; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

template <typename F>
static int timeit(const char* name, F launch, double flops) {
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return 1;
  launch();
  if (hipDeviceSynchronize() != hipSuccess) return 1;
  float best = 1e30f;
  for (int rep = 0; rep < 3; ++rep) {
    (void)hipEventRecord(e0);
    launch();
    (void)hipEventRecord(e1);
    if (hipEventSynchronize(e1) != hipSuccess) return 1;
    float ms = 0;
    (void)hipEventElapsedTime(&ms, e0, e1);
    best = ms < best ? ms : best;
  }
  printf("%-58s %8.3f ms  %7.1f TFLOP/s\n", name, best, flops / best * 1e-9);
  fflush(stdout);
  return 0;
}

int main() {
  int dev = 0, cus = 256;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) {
    fprintf(stderr, "mfma_probe: no HIP device\n");
    return 2;
  }
  cus = prop.multiProcessorCount;
  float* out = nullptr;
  if (hipMalloc(&out, (size_t)cus * 2 * 256 * 4) != hipSuccess) return 2;
  printf("%s, %d CUs, one workgroup of 4 waves per CU unless stated\n", prop.gcnArchName, cus);
  int rc = 0;
#define P32(MT, NB, Z, IT)                                                                         \
  rc |= timeit("32x32x16 " #MT "x" #NB " tiles, " #IT " iterations, operands " Z,                   \
               [&] { hipLaunchKernelGGL((probe32<MT, NB>), dim3(cus), dim3(256), 0, 0, out, IT, Z[0] == 'z'); }, \
               2.0 * 32 * 32 * 16 * MT * NB * 2 * (double)IT * cus * 4)
  P32(7, 2, "zero", 4000);
  P32(7, 2, "random", 4000);
  P32(7, 2, "random", 130);  // about one pass of the batched kernel
  P32(7, 1, "random", 8000);
  P32(2, 2, "random", 14000);
#define P16(NACC, WGS, Z, IT)                                                                      \
  rc |= timeit("16x16x32 " #NACC " tiles, " #WGS " workgroups per CU, operands " Z,                 \
               [&] { hipLaunchKernelGGL((probe16<NACC>), dim3(cus * WGS), dim3(256), 0, 0, out, IT, Z[0] == 'z'); }, \
               2.0 * 16 * 16 * 32 * NACC * (double)IT * cus * WGS * 4)
  P16(56, 1, "zero", 5000);
  P16(56, 1, "random", 5000);
  P16(16, 2, "random", 20000);
  hipError_t e = hipDeviceSynchronize();
  (void)hipFree(out);
  return (rc || e != hipSuccess) ? 1 : 0;
}
