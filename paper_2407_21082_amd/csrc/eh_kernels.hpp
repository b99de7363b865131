// General-purpose kernels of libeh: weight re-tiling, LayerNorm + packing,
// the streaming projection with fused softmax statistics, the cross-workgroup
// merge, the exit decision with compaction and the DSSD prefix compare.
// (arXiv 2407.21082: Section 3.2 heads, 3.4.1 entropy/argmax, 3.4.2 exit rule,
// 4.3.1 verification.)
#pragma once
#include "eh_device.hpp"

namespace eh {

// ---------------------------------------------------------------------------
// Row-major W [V, d] -> fragment-major copy (done once, at context creation).
// One thread per 16-byte chunk of the destination.
// ---------------------------------------------------------------------------
template <typename DT>
__global__ __launch_bounds__(256) void repack_w_kernel(const void* __restrict__ W, int V, int d,
                                                       int VT, int KS, frag_t* __restrict__ Wf) {
  const int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t total = (int64_t)VT * KS * kWave;
  if (o >= total) return;
  const int lane = (int)(o % kWave);
  const int64_t f = o / kWave;
  const int ks = (int)(f % KS);
  const int vt = (int)(f / KS);
  const int r = lane & 15, q = lane >> 4;
  const int row = vt * 16 + r;
  const int k0 = ks * DT::KPF + q * DT::EPL;
  frag_t v = mk_frag(0, 0, 0, 0);
  if (row < V && k0 < d) {
    const char* src = (const char*)W + ((int64_t)row * d + k0) * DT::ESZ;
    v = *(const frag_t*)src;  // d % EPL == 0 and a 16-byte aligned base are checked by the host
  }
  Wf[o] = v;
}

// ---------------------------------------------------------------------------
// LayerNorm of each live row, written as y fragments.  One wave per output
// position p (gathered through row_idx).  Mean and variance are two-pass and
// the whole normalisation runs in fp64: it costs nothing at these sizes and it
// makes the bf16 rounding of y independent of the reduction order.
// Positions >= live rows (up to R_pad) are zero-filled.
// ---------------------------------------------------------------------------
template <typename DT>
__device__ __forceinline__ void load_elems(const void* row, int k0, float (&x)[DT::EPL]);

// 16 bytes of a row -> its EPL elements as float
template <typename DT>
__device__ __forceinline__ void decode_elems(const frag_t& v, float (&x)[DT::EPL]);
template <>
__device__ __forceinline__ void decode_elems<DtBf16>(const frag_t& v, float (&x)[8]) {
  x[0] = bf16_bits_to_f32(v.x & 0xffffu); x[1] = bf16_bits_to_f32(v.x >> 16);
  x[2] = bf16_bits_to_f32(v.y & 0xffffu); x[3] = bf16_bits_to_f32(v.y >> 16);
  x[4] = bf16_bits_to_f32(v.z & 0xffffu); x[5] = bf16_bits_to_f32(v.z >> 16);
  x[6] = bf16_bits_to_f32(v.w & 0xffffu); x[7] = bf16_bits_to_f32(v.w >> 16);
}
template <>
__device__ __forceinline__ void decode_elems<DtF32>(const frag_t& v, float (&x)[4]) {
  x[0] = __uint_as_float(v.x); x[1] = __uint_as_float(v.y);
  x[2] = __uint_as_float(v.z); x[3] = __uint_as_float(v.w);
}
template <>
__device__ __forceinline__ void load_elems<DtBf16>(const void* row, int k0, float (&x)[8]) {
  decode_elems<DtBf16>(*(const frag_t*)((const char*)row + (int64_t)k0 * 2), x);
}
template <>
__device__ __forceinline__ void load_elems<DtF32>(const void* row, int k0, float (&x)[4]) {
  decode_elems<DtF32>(*(const frag_t*)((const char*)row + (int64_t)k0 * 4), x);
}

template <typename DT>
__device__ __forceinline__ frag_t pack_elems(const double (&y)[DT::EPL]);
template <>
__device__ __forceinline__ frag_t pack_elems<DtBf16>(const double (&y)[8]) {
  uint32_t b[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) b[i] = f64_to_bf16_bits(y[i]);
  return mk_frag(b[0] | (b[1] << 16), b[2] | (b[3] << 16), b[4] | (b[5] << 16), b[6] | (b[7] << 16));
}
template <>
__device__ __forceinline__ frag_t pack_elems<DtF32>(const double (&y)[4]) {
  return mk_frag(__float_as_uint((float)y[0]), __float_as_uint((float)y[1]),
                    __float_as_uint((float)y[2]), __float_as_uint((float)y[3]));
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// Rows are normalised by a workgroup of NW waves (kLnWaves in the kernels below; the decode
// kernel has its own single-wave LayerNorm).  Sum over the workgroup: per wave, then over
// the waves' totals in wave order through LDS (`red`, NW doubles, one array per call site
// so that no barrier is needed between consecutive sums).
constexpr int kLnWaves = 4;
constexpr int kLnThreads = kLnWaves * kWave;
template <int NW>
__device__ __forceinline__ double group_sum(double v, double* red, int tid) {
  v = wave_sum(v);
  if (NW == 1) return v;
  if ((tid & (kWave - 1)) == 0) red[tid >> 6] = v;
  __syncthreads();
  double t = red[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) t += red[w];
  return t;
}

// LayerNorm of one row by NW waves (tid = thread in the group); out(c, chunk) receives the
// packed chunk c (EPL consecutive outputs starting at k = c*EPL) for every c < n_chunks.
// red: 2*NW doubles of LDS.
template <typename DT, int NW, typename OutFn>
__device__ __forceinline__ void group_layernorm(const void* row, int d, int n_chunks,
                                                const float* __restrict__ gamma,
                                                const float* __restrict__ beta, float eps, int tid,
                                                double* red, OutFn out) {
  constexpr int NT = NW * kWave;
  const int live_chunks = d / DT::EPL;
  double s = 0.0;
  for (int c = tid; c < live_chunks; c += NT) {
    float x[DT::EPL];
    load_elems<DT>(row, c * DT::EPL, x);
#pragma unroll
    for (int i = 0; i < DT::EPL; ++i) s += (double)x[i];
  }
  const double mu = group_sum<NW>(s, red, tid) / (double)d;
  double v = 0.0;
  for (int c = tid; c < live_chunks; c += NT) {
    float x[DT::EPL];
    load_elems<DT>(row, c * DT::EPL, x);
#pragma unroll
    for (int i = 0; i < DT::EPL; ++i) {
      const double cdev = (double)x[i] - mu;
      v += cdev * cdev;
    }
  }
  const double var = group_sum<NW>(v, red + NW, tid) / (double)d;
  const double rstd = 1.0 / sqrt(var + (double)eps);
  for (int c = tid; c < n_chunks; c += NT) {
    frag_t o = mk_frag(0, 0, 0, 0);
    if (c < live_chunks) {
      float x[DT::EPL];
      load_elems<DT>(row, c * DT::EPL, x);
      double y[DT::EPL];
#pragma unroll
      for (int i = 0; i < DT::EPL; ++i) {
        const int k = c * DT::EPL + i;
        y[i] = (double)gamma[k] * (((double)x[i] - mu) * rstd) + (double)beta[k];
      }
      o = pack_elems<DT>(y);
    }
    out(c, o);
  }
}

// Same arithmetic, in the same order, for rows of at most kLnCache*64 chunks: the row is read
// from memory once and kept in registers for the three sweeps (mean, variance, output).
constexpr int kLnCache = 8;
template <typename DT, int NW, typename OutFn>
__device__ __forceinline__ void group_layernorm_cached(const void* row, int d, int n_chunks,
                                                       const float* __restrict__ gamma,
                                                       const float* __restrict__ beta, float eps, int tid,
                                                       double* red, OutFn out) {
  constexpr int NT = NW * kWave;
  constexpr int NJ = kLnCache / NW;
  static_assert(NJ * NW == kLnCache, "cache split");
  const int live_chunks = d / DT::EPL;
  frag_t raw[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int c = tid + j * NT;
    raw[j] = mk_frag(0, 0, 0, 0);
    if (c < live_chunks) raw[j] = *(const frag_t*)((const char*)row + (int64_t)c * 16);
  }
  double s = 0.0;
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    if (tid + j * NT < live_chunks) {
      float x[DT::EPL];
      decode_elems<DT>(raw[j], x);
#pragma unroll
      for (int i = 0; i < DT::EPL; ++i) s += (double)x[i];
    }
  }
  const double mu = group_sum<NW>(s, red, tid) / (double)d;
  double v = 0.0;
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    if (tid + j * NT < live_chunks) {
      float x[DT::EPL];
      decode_elems<DT>(raw[j], x);
#pragma unroll
      for (int i = 0; i < DT::EPL; ++i) {
        const double cdev = (double)x[i] - mu;
        v += cdev * cdev;
      }
    }
  }
  const double var = group_sum<NW>(v, red + NW, tid) / (double)d;
  const double rstd = 1.0 / sqrt(var + (double)eps);
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int c = tid + j * NT;
    if (c < n_chunks) {
      frag_t o = mk_frag(0, 0, 0, 0);
      if (c < live_chunks) {
        float x[DT::EPL];
        decode_elems<DT>(raw[j], x);
        double y[DT::EPL];
#pragma unroll
        for (int i = 0; i < DT::EPL; ++i) {
          const int k = c * DT::EPL + i;
          y[i] = (double)gamma[k] * (((double)x[i] - mu) * rstd) + (double)beta[k];
        }
        o = pack_elems<DT>(y);
      }
      out(c, o);
    }
  }
}

// One workgroup of kLnWaves waves per row.
// RB = rows per activation block: 16 (fragments of 16 rows x KPF k, the operand
// order of the 16x16 matrix instructions) or 32 (bf16 only: fragments of 32 rows
// x 16 k for v_mfma_f32_32x32x16_bf16; lane l of fragment (block, k16) holds row
// l%32, k = 16*k16 + 8*(l/32) .. +8).  R_pad is a multiple of RB; rows between
// the live rows and R_pad are zero-filled.
// Writes 16-byte chunk c of the row at position p of the activation workspace.
template <int RB>
__device__ __forceinline__ void put_chunk(frag_t* __restrict__ yf, int KS, int p, int c, const frag_t& v) {
  const int nb = p / RB, n = p % RB;
  // a block holds KS*4 chunks of 16 bytes per row either way
  frag_t* dst = yf + (int64_t)nb * KS * kWave * (RB / 16);
  if (RB == 16) dst[(c >> 2) * kWave + (c & 3) * 16 + n] = v;
  else dst[(c >> 1) * kWave + (c & 1) * 32 + n] = v;
}

// LayerNorm of the row at `row` into position p (the whole workgroup of kLnWaves waves; every
// thread of it must call; red: 2*kLnWaves doubles of LDS).
template <typename DT, int RB>
__device__ __forceinline__ void ln_write_row(const void* __restrict__ row, int d, int KS,
                                             const float* __restrict__ gamma,
                                             const float* __restrict__ beta, float eps,
                                             frag_t* __restrict__ yf, int p, int tid, double* red) {
  static_assert(RB == 16 || (RB == 32 && DT::EPL == 8), "row block");
  const int n_chunks = KS * 4;
  auto put = [&](int c, const frag_t& v) { put_chunk<RB>(yf, KS, p, c, v); };
  if (n_chunks <= kLnCache * kWave)
    group_layernorm_cached<DT, kLnWaves>(row, d, n_chunks, gamma, beta, eps, tid, red, put);
  else
    group_layernorm<DT, kLnWaves>(row, d, n_chunks, gamma, beta, eps, tid, red, put);
}

template <typename DT, int RB>
__device__ __forceinline__ void ln_pack_row(const void* __restrict__ h, int64_t row_stride,
                                            const int* __restrict__ row_idx, int n_live, int R_pad, int d,
                                            int KS, const float* __restrict__ gamma,
                                            const float* __restrict__ beta, float eps,
                                            frag_t* __restrict__ yf, int p, int tid, double* red) {
  if (p >= R_pad) return;
  if (p >= n_live) {
    for (int c = tid; c < KS * 4; c += kLnThreads) put_chunk<RB>(yf, KS, p, c, mk_frag(0, 0, 0, 0));
    return;
  }
  const int64_t r = row_idx ? row_idx[p] : p;
  ln_write_row<DT, RB>((const char*)h + r * row_stride * DT::ESZ, d, KS, gamma, beta, eps, yf, p, tid, red);
}

template <typename DT, int RB>
__global__ __launch_bounds__(kLnThreads) void ln_pack_kernel(const void* __restrict__ h, int64_t row_stride,
                                                     const int* __restrict__ row_idx,
                                                     const int* __restrict__ n_rows_dev, int n_rows,
                                                     int R_pad, int d, int KS,
                                                     const float* __restrict__ gamma,
                                                     const float* __restrict__ beta, float eps,
                                                     frag_t* __restrict__ yf) {
  int n_live = n_rows;
  if (n_rows_dev) n_live = min(max(*n_rows_dev, 0), n_rows);
  __shared__ double red[2 * kLnWaves];
  ln_pack_row<DT, RB>(h, row_stride, row_idx, n_live, R_pad, d, KS, gamma, beta, eps, yf, blockIdx.x,
                      threadIdx.x, red);
}

// The same for several heads at once: blockIdx.y = head (relative to the first),
// whose hidden states start layer_stride elements after the previous head's and
// whose output goes y_stride fragments after it.
template <typename DT, int RB>
__global__ __launch_bounds__(kLnThreads) void ln_pack_heads_kernel(const void* __restrict__ h_layers,
                                                           int64_t layer_stride, int64_t row_stride,
                                                           int n_rows, int R_pad, int d, int KS,
                                                           const float* const* __restrict__ gamma_tab,
                                                           const float* const* __restrict__ beta_tab,
                                                           float eps, frag_t* __restrict__ yf,
                                                           int64_t y_stride) {
  const int l = blockIdx.y;
  const void* h = (const char*)h_layers + (int64_t)l * layer_stride * DT::ESZ;
  __shared__ double red[2 * kLnWaves];
  ln_pack_row<DT, RB>(h, row_stride, nullptr, n_rows, R_pad, d, KS, gamma_tab[l], beta_tab[l], eps,
                      yf + (int64_t)l * y_stride, blockIdx.x, threadIdx.x, red);
}

// ---------------------------------------------------------------------------
// Streaming projection with fused softmax statistics (general row counts).
// Each wave owns whole vocabulary tiles (16 rows, all of k) and NB token
// blocks; both operands come straight from global memory in fragment order.
// The logits live only in the accumulators.  Per workgroup one Stats record
// per token is written to `partials[blockIdx.x][R_pad]`.
// ---------------------------------------------------------------------------
template <typename DT, int NB, bool ARGMAX_ONLY>
__global__ __launch_bounds__(256) void stream_kernel(const frag_t* __restrict__ Wf,
                                                     const frag_t* __restrict__ yf,
                                                     const float* __restrict__ bias, int VT, int KS,
                                                     int V, int nb0, const int* __restrict__ n_rows_dev,
                                                     int n_rows, int R_pad, Stats* __restrict__ partials) {
  __shared__ Stats red[4][NB][16];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int q = lane >> 4, n = lane & 15;
  int n_live = n_rows;
  if (n_rows_dev) n_live = min(max(*n_rows_dev, 0), n_rows);
  const int nb_live = min(NB, (n_live - nb0 * 16 + 15) >> 4);
  if (nb_live <= 0) return;  // uniform over the grid

  Stats st[NB];
#pragma unroll
  for (int b = 0; b < NB; ++b) stats_init(st[b]);

  const int gw = blockIdx.x * 4 + wave, tw = gridDim.x * 4;
  const frag_t* yp = yf + (int64_t)nb0 * KS * kWave + lane;
  for (int vt = gw; vt < VT; vt += tw) {
    f32x4 acc[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) acc[b] = f32x4{0.f, 0.f, 0.f, 0.f};
    const frag_t* wp = Wf + (int64_t)vt * KS * kWave + lane;
    constexpr int U = (NB <= 1) ? 8 : (NB <= 2) ? 4 : 2;
    int ks = 0;
    for (; ks + U <= KS; ks += U) {
      frag_t a[U];
#pragma unroll
      for (int u = 0; u < U; ++u) a[u] = __builtin_nontemporal_load(wp + (int64_t)(ks + u) * kWave);
#pragma unroll
      for (int u = 0; u < U; ++u) {
#pragma unroll
        for (int b = 0; b < NB; ++b) {
          if (b < nb_live) {
            const frag_t y = yp[((int64_t)b * KS + ks + u) * kWave];
            acc[b] = DT::mma(a[u], y, acc[b]);
          }
        }
      }
    }
    for (; ks < KS; ++ks) {
      const frag_t a = __builtin_nontemporal_load(wp + (int64_t)ks * kWave);
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        if (b < nb_live) {
          const frag_t y = yp[((int64_t)b * KS + ks) * kWave];
          acc[b] = DT::mma(a, y, acc[b]);
        }
      }
    }
    const int row0 = vt * 16 + q * 4;
    f32x4 bz = f32x4{0.f, 0.f, 0.f, 0.f};
    if (bias) bz = *(const f32x4*)(bias + row0);  // bias is padded to VT*16 entries
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      if (b < nb_live) stats_push4<ARGMAX_ONLY>(st[b], acc[b] + bz, row0, V);
    }
  }

  // lanes n, n+16, n+32, n+48 hold the same token: fold the four row groups
#pragma unroll
  for (int b = 0; b < NB; ++b) {
    st[b] = stats_merge(st[b], stats_shfl_xor(st[b], 16));
    st[b] = stats_merge(st[b], stats_shfl_xor(st[b], 32));
    if (q == 0) red[wave][b][n] = st[b];
  }
  __syncthreads();
  for (int i = threadIdx.x; i < NB * 16; i += blockDim.x) {
    const int b = i >> 4, t = i & 15;
    if (b < nb_live) {
      Stats s = red[0][b][t];
      s = stats_merge(s, red[1][b][t]);
      s = stats_merge(s, red[2][b][t]);
      s = stats_merge(s, red[3][b][t]);
      partials[(int64_t)blockIdx.x * R_pad + (nb0 + b) * 16 + t] = s;
    }
  }
}

// ---------------------------------------------------------------------------
// Merge the per-workgroup partials of each live row and finalise:
// H = ln2 (log2 S - U/S), lse = ln2 (m + log2 S), argmax = ib.
// One wave per row (the cascade step kernel merges the same way with its first wave).
// ---------------------------------------------------------------------------
__device__ __forceinline__ void stats_finalize(const Stats& s, float& H, float& lse) {
  const double S = (double)s.S, U = (double)s.U;
  const double l2 = log2(S);
  H = (float)(kLn2d * (l2 - U / S));
  lse = (float)(kLn2d * ((double)s.m + l2));
}

// blockIdx.y = head (relative): partials advance by part_stride records per head,
// outputs by out_stride elements (both 0 for a single head).
static __global__ __launch_bounds__(64) void finalize_kernel(const Stats* __restrict__ partials, int n_parts,
                                                      int R_pad, const int* __restrict__ n_rows_dev,
                                                      int n_rows, float* __restrict__ H,
                                                      float* __restrict__ lse, int* __restrict__ argmax,
                                                      int64_t part_stride, int64_t out_stride) {
  const int p = blockIdx.x, lane = threadIdx.x;
  int n_live = n_rows;
  if (n_rows_dev) n_live = min(max(*n_rows_dev, 0), n_rows);
  if (p >= n_live) return;
  partials += (int64_t)blockIdx.y * part_stride;
  const int64_t o = (int64_t)blockIdx.y * out_stride + p;
  Stats s;
  stats_init(s);
  for (int g = lane; g < n_parts; g += kWave) s = stats_merge(s, partials[(int64_t)g * R_pad + p]);
#pragma unroll
  for (int x = 32; x > 0; x >>= 1) s = stats_merge(s, stats_shfl_xor(s, x));
  if (lane == 0) {
    float h, l;
    stats_finalize(s, h, l);
    if (H) H[o] = h;
    if (lse) lse[o] = l;
    if (argmax) argmax[o] = stats_token(s);
  }
}

// Final merge with the other two confidence metrics of Section 3.4.1: besides the
// statistics, the second largest logit z2 (with multiplicity) is merged over the
// workgroups' slices -- second of a union = max(min(z1a, z1b), max(z2a, z2b)) -- and
//   max_prob = p(argmax) = 1 / S        (S sums 2^(t - m) with m the largest t: its own term is 1)
//   margin   = p1 - p2 = (1 - e^(z2 - z1)) / S.
static __global__ __launch_bounds__(64) void finalize_metrics_kernel(
    const Stats* __restrict__ partials, const float* __restrict__ second, int n_parts, int R_pad, int n_rows,
    float* __restrict__ H, float* __restrict__ lse, int* __restrict__ argmax, float* __restrict__ max_prob,
    float* __restrict__ margin, int64_t part_stride, int64_t out_stride) {
  const int p = blockIdx.x, lane = threadIdx.x;
  if (p >= n_rows) return;
  partials += (int64_t)blockIdx.y * part_stride;
  second += (int64_t)blockIdx.y * part_stride;
  const int64_t o = (int64_t)blockIdx.y * out_stride + p;
  Stats s;
  stats_init(s);
  float z2 = -INFINITY;
  for (int g = lane; g < n_parts; g += kWave) {
    const Stats q = partials[(int64_t)g * R_pad + p];
    z2 = fmaxf(fminf(s.zb, q.zb), fmaxf(z2, second[(int64_t)g * R_pad + p]));
    s = stats_merge(s, q);
  }
#pragma unroll
  for (int x = 32; x > 0; x >>= 1) {
    const Stats q = stats_shfl_xor(s, x);
    z2 = fmaxf(fminf(s.zb, q.zb), fmaxf(z2, __shfl_xor(z2, x)));
    s = stats_merge(s, q);
  }
  if (lane == 0) {
    float h, l;
    stats_finalize(s, h, l);
    if (H) H[o] = h;
    if (lse) lse[o] = l;
    if (argmax) argmax[o] = stats_token(s);
    const float p1 = 1.0f / s.S;  // NaN statistics give NaN metrics
    if (max_prob) max_prob[o] = p1;
    if (margin) margin[o] = p1 * (1.0f - fast_exp2((z2 - s.zb) * kLog2e));
  }
}

// ---------------------------------------------------------------------------
// Cascade step behind a head's projection (Sections 3.4.1, 3.4.2), one wave per
// position p of the head's active list: merge the partial statistics of the row,
// apply the exit rule, and for a row that goes on append it to the next head's
// active list and write its LayerNorm for the next head straight into the
// activation workspace at the position it got.  Positions are handed out by an
// atomic counter, so the next list is not in row order (nothing depends on the
// order: rows are independent and every output is indexed by the row).  Positions
// beyond the next head's live count keep whatever an earlier head left there; the
// projection never lets a token column influence another.
// ---------------------------------------------------------------------------
template <typename DT, int RB>
__global__ __launch_bounds__(kLnThreads) void cascade_post_kernel(
    const Stats* __restrict__ partials, int n_parts, int R_pad, const int* __restrict__ row_idx,
    const int* __restrict__ n_rows_dev, int n_rows, float tau, int is_last, int head,
    int* __restrict__ exit_layer,
    int* __restrict__ token, float* __restrict__ H_out, unsigned long long* __restrict__ n_evals,
    int* __restrict__ active_next, int* __restrict__ n_active_next, int* __restrict__ clear,
    const void* __restrict__ h_next, int64_t row_stride, int d, int KS,
    const float* __restrict__ gamma_next, const float* __restrict__ beta_next, float eps,
    frag_t* __restrict__ yf) {
  __shared__ double red[2 * kLnWaves];
  __shared__ int pos_s;
  const int p = blockIdx.x, tid = threadIdx.x, lane = tid & (kWave - 1);
  if (p == 0 && tid == 0 && clear) *clear = 0;  // the counter of the head after next
  int n_live = n_rows;
  if (n_rows_dev) n_live = min(max(*n_rows_dev, 0), n_rows);
  if (p >= n_live) return;
  const int r = row_idx ? row_idx[p] : p;
  if (tid < kWave) {  // the first wave merges and decides, exactly as finalize_kernel does
    Stats s;
    stats_init(s);
    for (int g = lane; g < n_parts; g += kWave) s = stats_merge(s, partials[(int64_t)g * R_pad + p]);
#pragma unroll
    for (int x = 32; x > 0; x >>= 1) s = stats_merge(s, stats_shfl_xor(s, x));
    if (lane == 0) {
      int pos = -1;
      float H, l;
      stats_finalize(s, H, l);
      if (H_out) H_out[r] = H;
      if (n_evals) atomicAdd(n_evals, 1ull);
      if (is_last || H < tau) {  // NaN never passes the test
        exit_layer[r] = head;
        token[r] = stats_token(s);
      } else {
        pos = atomicAdd(n_active_next, 1);
        active_next[pos] = r;
      }
      pos_s = pos;
    }
  }
  __syncthreads();
  const int pos = pos_s;
  if (pos < 0) return;
  ln_write_row<DT, RB>((const char*)h_next + (int64_t)r * row_stride * DT::ESZ, d, KS, gamma_next, beta_next,
                       eps, yf, pos, tid, red);
}

// ---------------------------------------------------------------------------
// Exit rule + stable compaction.  Single workgroup; positions are processed in
// chunks of blockDim.x with a block-wide exclusive scan of the "stays" flags.
// ---------------------------------------------------------------------------
static __global__ __launch_bounds__(256) void decide_kernel(const float* __restrict__ H,
                                                     const int* __restrict__ argmax,
                                                     const int* __restrict__ row_idx,
                                                     const int* __restrict__ n_rows_dev, int n_rows,
                                                     float tau, int is_last, int head,
                                                     int* __restrict__ exit_layer, int* __restrict__ token,
                                                     int* __restrict__ active_out,
                                                     int* __restrict__ n_active_out,
                                                     float* __restrict__ H_out,
                                                     unsigned long long* __restrict__ n_evals) {
  __shared__ int wave_tot[4];
  __shared__ int base_s;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int n_live = n_rows;
  if (n_rows_dev) n_live = min(max(*n_rows_dev, 0), n_rows);
  if (tid == 0) base_s = 0;
  __syncthreads();
  for (int start = 0; start < n_live; start += blockDim.x) {
    const int p = start + tid;
    const bool valid = p < n_live;
    int r = 0;
    bool stays = false;
    if (valid) {
      r = row_idx ? row_idx[p] : p;
      const float hp = H[p];
      const bool leaves = is_last || (hp < tau);
      stays = !leaves;
      if (leaves) {
        exit_layer[r] = head;
        token[r] = argmax[p];
      }
      if (H_out) H_out[r] = hp;
    }
    const unsigned long long bal = __ballot(stays);
    const int before = __popcll(bal & ((1ull << lane) - 1ull));
    if (lane == 0) wave_tot[wave] = __popcll(bal);
    __syncthreads();
    int off = base_s;
    for (int w = 0; w < wave; ++w) off += wave_tot[w];
    if (stays) active_out[off + before] = r;
    __syncthreads();
    if (tid == 0) base_s += wave_tot[0] + wave_tot[1] + wave_tot[2] + wave_tot[3];
    __syncthreads();
  }
  if (tid == 0) {
    if (n_active_out) *n_active_out = base_s;
    if (n_evals) *n_evals += (unsigned long long)n_live;
  }
}

// ---------------------------------------------------------------------------
// DSSD: length of the accepted prefix and the token that follows it.
// ---------------------------------------------------------------------------
static __global__ void verify_compare_kernel(const int* __restrict__ draft, const int* __restrict__ draft_len,
                                      const int* __restrict__ target, int B, int k,
                                      int* __restrict__ accepted, int* __restrict__ next_token) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  int len = k;
  if (draft_len) len = min(max(draft_len[b], 0), k);
  int n = 0;
  while (n < len && draft[(int64_t)b * k + n] == target[(int64_t)b * (k + 1) + n]) ++n;
  accepted[b] = n;
  next_token[b] = target[(int64_t)b * (k + 1) + n];
}

// The same behind the batched projection in one launch: workgroup b merges the partial
// argmax records of row b's k+1 positions (one wave per position, four at a time), then
// its first thread walks the prefix.  `target` (nullable) receives the merged argmaxes.
static __global__ __launch_bounds__(256) void verify_post_kernel(
    const Stats* __restrict__ partials, int n_parts, int R_pad, const int* __restrict__ draft,
    const int* __restrict__ draft_len, int k, int* __restrict__ target, int* __restrict__ accepted,
    int* __restrict__ next_token) {
  extern __shared__ int verify_tgt[];  // k + 1 entries
  const int b = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int j = wave; j <= k; j += 4) {
    const int p = b * (k + 1) + j;
    float zb = -INFINITY;
    int ib = 0x7fffffff;
    for (int g = lane; g < n_parts; g += kWave) {
      const Stats q = partials[(int64_t)g * R_pad + p];
      if (q.zb > zb || (q.zb == zb && q.ib < ib)) { zb = q.zb; ib = q.ib; }
    }
#pragma unroll
    for (int x = 32; x > 0; x >>= 1) {
      const float oz = __shfl_xor(zb, x);
      const int oi = __shfl_xor(ib, x);
      if (oz > zb || (oz == zb && oi < ib)) { zb = oz; ib = oi; }
    }
    if (lane == 0) {
      verify_tgt[j] = argmax_or_none(ib);
      if (target) target[p] = argmax_or_none(ib);
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int len = k;
    if (draft_len) len = min(max(draft_len[b], 0), k);
    int n = 0;
    while (n < len && draft[(int64_t)b * k + n] == verify_tgt[n]) ++n;
    accepted[b] = n;
    next_token[b] = verify_tgt[n];
  }
}

// ---------------------------------------------------------------------------
// DSSD drafting controller (Section 4.3.1, "Drafting phase"): one thread, run
// behind the cascade of a position.  state = {live, length, reason, fallback}:
// `live` is the device-side row count of the next position's cascade (0 once
// drafting has stopped, which turns the remaining launches into no-ops).
// ---------------------------------------------------------------------------
static __global__ void draft_init_kernel(int* __restrict__ state, int limit, int* __restrict__ exit_layers) {
  if (threadIdx.x == 0) {
    state[0] = limit > 0 ? 1 : 0;
    state[1] = 0;
    state[2] = limit > 0 ? -1 : 0;  // an empty buffer is full at once
    state[3] = -1;
  }
  for (int i = threadIdx.x; i < limit; i += blockDim.x) exit_layers[i] = -1;
}

static __global__ void draft_step_kernel(int* __restrict__ state, const int* __restrict__ exit_layer,
                                         const int* __restrict__ token, int last_head, int limit, int eos,
                                         int* __restrict__ draft, int* __restrict__ exit_layers) {
  if (state[0] == 0) return;
  const int e = *exit_layer, tk = *token;
  if (e < 0) {  // the cascade of this position gave up (reported by eh_check): stop, append nothing
    state[0] = 0;
    state[2] = 3;
    return;
  }
  if (e >= last_head) {  // no exit head was confident: the model's own prediction is the fallback
    state[0] = 0;
    state[2] = 2;
    state[3] = tk;
    return;
  }
  const int n = state[1];
  draft[n] = tk;
  exit_layers[n] = e;
  state[1] = n + 1;
  if (tk == eos) {
    state[0] = 0;
    state[2] = 1;
  } else if (n + 1 == limit) {
    state[0] = 0;
    state[2] = 0;
  }
}

static __global__ void draft_finish_kernel(const int* __restrict__ state, int* __restrict__ draft_len,
                                           int* __restrict__ stop_reason, int* __restrict__ fallback_token) {
  *draft_len = state[1];
  if (stop_reason) *stop_reason = state[2] < 0 ? 3 : state[2];  // still running: the positions ran out
  if (fallback_token) *fallback_token = state[3];
}

// ---------------------------------------------------------------------------
// Verification bookkeeping (Section 4.3.1, verification phase; the quantities
// reported in Section 4.3.2): adds one batch of rounds to the running counters
// {rounds, drafted, accepted, wasted, exit-layer sum}.  One workgroup; lengths
// are clamped to [0, k] and accepted counts to [0, length].
// ---------------------------------------------------------------------------
static __global__ void tally_kernel(const int* __restrict__ draft_len, const int* __restrict__ accepted, int B, int k,
                                    const int* __restrict__ exit_layers, unsigned long long* __restrict__ counters) {
  long long drafted = 0, acc = 0, layers = 0;
  for (int b = threadIdx.x; b < B; b += blockDim.x) {
    int n = draft_len ? draft_len[b] : k;
    n = n < 0 ? 0 : (n > k ? k : n);
    int a = accepted[b];
    a = a < 0 ? 0 : (a > n ? n : a);
    drafted += n;
    acc += a;
    if (exit_layers)
      for (int j = 0; j < n; ++j) layers += exit_layers[(int64_t)b * k + j];
  }
  for (int o = 32; o > 0; o >>= 1) {
    drafted += __shfl_xor(drafted, o);
    acc += __shfl_xor(acc, o);
    layers += __shfl_xor(layers, o);
  }
  if ((threadIdx.x & 63) == 0) {
    atomicAdd(&counters[1], (unsigned long long)drafted);
    atomicAdd(&counters[2], (unsigned long long)acc);
    atomicAdd(&counters[3], (unsigned long long)(drafted - acc));
    atomicAdd(&counters[4], (unsigned long long)layers);
  }
  if (threadIdx.x == 0) atomicAdd(&counters[0], (unsigned long long)B);
}

// ---------------------------------------------------------------------------
// Training objectives (Section 3.3): final merge of a token's partial statistics
// (one wave per token), then the means over the sequence (one workgroup, fixed
// summation order, fp64).
// ---------------------------------------------------------------------------
static __global__ __launch_bounds__(64) void kl_finalize_kernel(const KlStats* __restrict__ partials, int n_parts,
                                                         int R_pad, int n_rows, int V,
                                                         float* __restrict__ rows, float* __restrict__ kl_out,
                                                         float* __restrict__ ce_out) {
  const int p = blockIdx.x, lane = threadIdx.x;
  if (p >= n_rows) return;
  KlStats s;
  kl_init(s, -1);
  for (int g = lane; g < n_parts; g += kWave) {
    const KlStats q = partials[(int64_t)g * R_pad + p];
    const int lab = q.lab;
    s = kl_merge(s, q);
    s.lab = lab;
  }
#pragma unroll
  for (int x = 32; x > 0; x >>= 1) {
    const KlStats o = kl_shfl_xor(s, x);
    const int lab = max(s.lab, o.lab);  // lanes that merged nothing still hold -1
    s = kl_merge(s, o);
    s.lab = lab;
  }
  if (lane == 0) {
    const double Ss = (double)s.Ss, St = (double)s.St;
    const double lse_s = kLn2d * ((double)s.ms + log2(Ss));
    const double lse_t = kLn2d * ((double)s.mt + log2(St));
    const float kl = (float)((double)s.C / Ss - lse_s + lse_t);
    const float ce = (s.lab >= 0 && s.lab < V) ? (float)(lse_s - (double)s.zl) : NAN;
    rows[p] = kl;
    rows[R_pad + p] = ce;
    if (kl_out) kl_out[p] = kl;
    if (ce_out) ce_out[p] = ce;
  }
}

// loss[0] = L_CE, loss[1] = L_KL, loss[2] = alpha * L_CE + (1 - alpha) * L_KL
static __global__ __launch_bounds__(256) void kl_mean_kernel(const float* __restrict__ rows, int R_pad, int n_rows,
                                                      float alpha, float* __restrict__ loss) {
  __shared__ double skl[256], sce[256];
  double a = 0.0, b = 0.0;
  for (int r = threadIdx.x; r < n_rows; r += 256) {
    a += (double)rows[r];
    b += (double)rows[R_pad + r];
  }
  skl[threadIdx.x] = a;
  sce[threadIdx.x] = b;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) {
      skl[threadIdx.x] += skl[threadIdx.x + o];
      sce[threadIdx.x] += sce[threadIdx.x + o];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const double L_kl = skl[0] / n_rows, L_ce = sce[0] / n_rows;
    loss[0] = (float)L_ce;
    loss[1] = (float)L_kl;
    loss[2] = (float)((double)alpha * L_ce + (1.0 - (double)alpha) * L_kl);
  }
}

static __global__ void fill_f32_kernel(float* p, int64_t n, float v) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}
static __global__ void fill_i32_kernel(int* p, int64_t n, int v) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

}  // namespace eh
