// Device-side building blocks shared by the libeh kernels (gfx950 only).
//
// Data layout ("fragment-major"): both GEMM operands are kept in HBM in the
// order the 16x16 matrix-core instructions consume them, so that every wave
// load is one contiguous, fully coalesced 1 KiB read and no LDS transpose is
// needed.  A fragment is 64 lanes x 16 bytes:
//   lane = q*16 + r  (r = lane % 16, q = lane / 16)
//   W fragment (vt, ks):  lane holds W[vt*16 + r][ks*KPF + q*EPL .. +EPL)
//   y fragment (nb, ks):  lane holds y[nb*16 + r][ks*KPF + q*EPL .. +EPL)
// with EPL = elements per 16 bytes (8 bf16 / 4 f32) and KPF = 4*EPL the k
// extent of a fragment.  Fragments are stored [tile][ks][lane].  Rows beyond V
// (or beyond the live rows) and k beyond d are zero.
//
// One fragment pair feeds v_mfma_f32_16x16x32_bf16 (bf16) or four
// v_mfma_f32_16x16x4_f32 (f32); lane (q, r) of A meets lane (q, n) of B on the
// same k values, which is all the dot product needs.  The accumulator of a
// 16x16 product holds, in lane l and register i, output row 4*(l/16)+i (a
// vocabulary row) and column l%16 (a token): the softmax reduction over the
// vocabulary therefore runs down registers and over time inside a lane, and
// only the final merge crosses lanes.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace eh {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t frag_t __attribute__((ext_vector_type(4)));  // 16 bytes of one lane
__device__ __forceinline__ frag_t mk_frag(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  return frag_t{a, b, c, d};
}

constexpr int kWave = 64;
constexpr float kLog2e = 1.4426950408889634f;
constexpr double kLn2d = 0.69314718055994530942;
constexpr float kNegBig = -1.0e30f;  // finite stand-in for "no maximum yet" (keeps m - m' finite)

struct DtBf16 {
  static constexpr int EPL = 8;   // elements per lane per fragment
  static constexpr int KPF = 32;  // k extent of a fragment
  static constexpr int ESZ = 2;
  static __device__ __forceinline__ f32x4 mma(const frag_t& a, const frag_t& b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                   __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
};

struct DtF32 {
  static constexpr int EPL = 4;
  static constexpr int KPF = 16;
  static constexpr int ESZ = 4;
  static __device__ __forceinline__ f32x4 mma(const frag_t& a, const frag_t& b, f32x4 c) {
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.x), __uint_as_float(b.x), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.y), __uint_as_float(b.y), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.z), __uint_as_float(b.z), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.w), __uint_as_float(b.w), c, 0, 0, 0);
    return c;
  }
};

// fp32 -> bf16, round to nearest even (NaN stays NaN).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}
// fp64 -> bf16 with a single round to nearest even.  Going through fp32 with two
// roundings to nearest would be wrong whenever the fp32 value lands exactly on a bf16
// tie (once in about 2^16 values): the first step therefore rounds to odd (truncate
// toward zero, set the last bit if anything was lost), which leaves the second,
// nearest-even rounding to 8 bits exact because fp32 carries 16 bits more than bf16.
__device__ __forceinline__ uint32_t f64_to_bf16_bits(double y) {
  float f = (float)y;
  const double fd = (double)f;
  if (fd != y && fd == fd) {  // inexact, not NaN
    uint32_t u = __float_as_uint(f);
    if (fabs(fd) > fabs(y)) u -= 1u;  // one step toward zero (sign-magnitude encoding)
    u |= 1u;
    f = __uint_as_float(u);
  }
  return f32_to_bf16_bits(f);
}
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Running softmax statistics of a set of logits z_i, kept in the base-2 domain
// t_i = z_i * log2(e):  m = max t,  S = sum 2^(t-m),  U = sum (t-m) 2^(t-m),
// (zb, ib) = largest logit and the lowest index attaining it.
// Entropy (nats) = ln2 * (log2 S - U/S);  lse = ln2 * (m + log2 S).
struct Stats {
  float m, S, U, zb;
  int ib;
};

__device__ __forceinline__ void stats_init(Stats& s) {
  s.m = kNegBig; s.S = 0.f; s.U = 0.f; s.zb = -INFINITY; s.ib = 0x7fffffff;
}

// The index reported for a row: -1 if no logit ever compared greater than "nothing yet",
// i.e. every logit of the row is NaN (a hidden state with a NaN or Inf in it).
__device__ __forceinline__ int argmax_or_none(int ib) { return ib == 0x7fffffff ? -1 : ib; }
__device__ __forceinline__ int stats_token(const Stats& s) { return argmax_or_none(s.ib); }

// Associative merge: rescale both sides to the common maximum.
__device__ __forceinline__ Stats stats_merge(const Stats& a, const Stats& b) {
  Stats r;
  const bool bw = (b.zb > a.zb) || (b.zb == a.zb && b.ib < a.ib);
  r.zb = bw ? b.zb : a.zb;
  r.ib = bw ? b.ib : a.ib;
  const float m = fmaxf(a.m, b.m);
  const float da = a.m - m, db = b.m - m;
  const float ea = fast_exp2(da), eb = fast_exp2(db);
  r.S = ea * a.S + eb * b.S;
  r.U = ea * (a.U + da * a.S) + eb * (b.U + db * b.S);
  r.m = m;
  return r;
}

// Push four logits of consecutive vocabulary rows row0..row0+3 (rows >= V are
// padding and skipped).  Rows must arrive in increasing order within a lane so
// that "strictly greater" keeps the lowest index.
template <bool ARGMAX_ONLY>
__device__ __forceinline__ void stats_push4(Stats& s, f32x4 z, int row0, int V) {
  const int nvalid = V - row0;  // >= 4 everywhere but in the last tile
  float zc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) zc[i] = (i < nvalid) ? z[i] : -INFINITY;
  const float zmax = fmaxf(fmaxf(zc[0], zc[1]), fmaxf(zc[2], zc[3]));
  if (zmax > s.zb) {
    const int j = (zc[0] == zmax) ? 0 : (zc[1] == zmax) ? 1 : (zc[2] == zmax) ? 2 : 3;
    if (!ARGMAX_ONLY) {
      const float mn = zmax * kLog2e;
      const float dm = s.m - mn;
      const float sc = fast_exp2(dm);
      s.U = sc * (s.U + dm * s.S);
      s.S = sc * s.S;
      s.m = mn;
    }
    s.zb = zmax;
    s.ib = row0 + j;
  }
  if (!ARGMAX_ONLY) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (i < nvalid) {
        const float t = z[i] * kLog2e - s.m;  // <= 0 up to rounding for finite logits
        const float e = fast_exp2(t);
        s.S += e;
        s.U += t * e;
      }
    }
  }
}

__device__ __forceinline__ Stats stats_shfl_xor(const Stats& s, int mask) {
  Stats o;
  o.m = __shfl_xor(s.m, mask);
  o.S = __shfl_xor(s.S, mask);
  o.U = __shfl_xor(s.U, mask);
  o.zb = __shfl_xor(s.zb, mask);
  o.ib = __shfl_xor(s.ib, mask);
  return o;
}

// Running statistics for the training objectives (Section 3.3) of one token: the head's
// logits zs and the model's logits zt of the same vocabulary entries arrive together.
// Base-2 domain as above: ms = max zs*log2e, Ss = sum 2^(ts - ms), mt/St the same for the
// model, C = sum 2^(ts - ms) * (zs - zt) (natural units), zl = the head's logit of the label.
//   KL(head || model) = C / Ss - lse_s + lse_t,   CE = lse_s - zl,   lse = ln2 * (m + log2 S).
struct KlStats {
  float ms, Ss, C, mt, St, zl;
  int lab;
};

__device__ __forceinline__ void kl_init(KlStats& s, int label) {
  s.ms = kNegBig; s.Ss = 0.f; s.C = 0.f; s.mt = kNegBig; s.St = 0.f; s.zl = -INFINITY; s.lab = label;
}

__device__ __forceinline__ KlStats kl_merge(const KlStats& a, const KlStats& b) {
  KlStats r;
  r.ms = fmaxf(a.ms, b.ms);
  const float ea = fast_exp2(a.ms - r.ms), eb = fast_exp2(b.ms - r.ms);
  r.Ss = ea * a.Ss + eb * b.Ss;
  r.C = ea * a.C + eb * b.C;
  r.mt = fmaxf(a.mt, b.mt);
  r.St = fast_exp2(a.mt - r.mt) * a.St + fast_exp2(b.mt - r.mt) * b.St;
  r.zl = fmaxf(a.zl, b.zl);  // exactly one slice of the vocabulary holds the label
  r.lab = a.lab;
  return r;
}

// Four consecutive vocabulary rows row0..row0+3 of both heads (rows >= V are padding).
__device__ __forceinline__ void kl_push4(KlStats& s, f32x4 zs, f32x4 zt, int row0, int V) {
  const int nvalid = V - row0;
  float a = -INFINITY, b = -INFINITY;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (i < nvalid) {
      a = fmaxf(a, zs[i]);
      b = fmaxf(b, zt[i]);
    }
  }
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
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (i < nvalid) {
      const float e = fast_exp2(zs[i] * kLog2e - s.ms);
      s.Ss += e;
      s.C += e * (zs[i] - zt[i]);
      s.St += fast_exp2(zt[i] * kLog2e - s.mt);
      if (row0 + i == s.lab) s.zl = zs[i];
    }
  }
}

__device__ __forceinline__ KlStats kl_shfl_xor(const KlStats& s, int mask) {
  KlStats o;
  o.ms = __shfl_xor(s.ms, mask);
  o.Ss = __shfl_xor(s.Ss, mask);
  o.C = __shfl_xor(s.C, mask);
  o.mt = __shfl_xor(s.mt, mask);
  o.St = __shfl_xor(s.St, mask);
  o.zl = __shfl_xor(s.zl, mask);
  o.lab = __shfl_xor(s.lab, mask);
  return o;
}

}  // namespace eh
