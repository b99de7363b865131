// Persistent decode kernel: up to 16 rows through heads l0 .. l1-1 in ONE launch
// (arXiv 2407.21082, Section 3.4.2 exit rule in the entropy form of Section
// 4.3.1; per head the LayerNorm -> projection -> entropy/argmax of Sections 3.2
// and 3.4.1).
//
// Batch-1 decode is a pure weight stream (1 flop per byte), so the design goal
// is to keep HBM reads back to back from the first head to the exit head:
//
//  * one workgroup per CU, each owning a contiguous, tile-aligned slice of the
//    vocabulary of every head; inside it, 4 "streamer" waves split the slice's
//    fragments evenly and each reads its own contiguous span through a
//    register ring of P loads that runs on across head boundaries;
//  * the matrix cores do the k-reduction (one 16x16 tile of logits per 1 KiB
//    fragment pair); the streamers fold finished tiles into running softmax
//    statistics, tiles split between two waves are summed by the service wave;
//  * two more waves do everything that needs global round trips so that the
//    streamers never drain their rings: a LayerNorm wave prepares the next
//    head's rows in LDS (double buffered), and an exchange wave all-gathers
//    the workgroups' partial statistics through tagged records, merges them
//    and applies the threshold test (every workgroup reaches the same
//    decision from the same records; workgroup 0 writes the outputs);
//  * heads are speculated one ahead: streamers start head l+1 while the
//    decision for head l is still being formed and drop it if every row has
//    exited.  Nothing of a dropped head is ever published.
//
// Every wait on another workgroup is bounded (DecodeParams::spin_limit polls); a
// timeout sets the context's status word and makes every wave leave.  The kernel
// assumes that all its workgroups are resident at once (one per compute unit):
// the stream has to own the device while it runs.  Workgroup 0 presets the outputs
// of the live rows to -1 / NaN, so a launch that gives up leaves defined values.
#include "eh_internal.hpp"
#include "eh_kernels.hpp"

namespace eh {

namespace {

constexpr int kStreamers = 8;
constexpr int kThreads = (kStreamers + 2) * kWave;  // streamers + exchange wave + LayerNorm wave
constexpr int kRing = 4;              // fragments per ring buffer (two buffers per streamer wave)
constexpr int kMaxLag = 3;            // heads the streamers may be ahead of the oldest open exchange
constexpr int kSpinLimit = 1 << 22;   // polls of a flag of this workgroup (LDS) before giving up
constexpr int kMaxChunksPerLane = 4;  // LayerNorm keeps a row in registers: d <= 4*64*EPL

// LDS-only barrier: waits for this wave's LDS traffic, not for the global loads
// still in flight in the ring.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

#define EH_LDS __attribute__((address_space(3)))
#define EH_GLOBAL __attribute__((address_space(1)))
// Pointers read out of the per-head tables are generic to the compiler; casting
// them to the global address space keeps the weight stream on global_load (one
// counter, exact in-order waits) instead of flat_load.
typedef EH_GLOBAL const frag_t gfrag_t;
typedef EH_GLOBAL const f32x4 gf32x4_t;
typedef EH_GLOBAL const float gfloat_t;
// The per-head pointer tables are written once at context creation; reading them
// through the constant address space lets the streamers fetch a head's base with
// a scalar load instead of a vector load whose wait would drain the ring.
__device__ __forceinline__ gfrag_t* head_weights(const frag_t* const* table, int l) {
  typedef const frag_t* entry_t;
  typedef __attribute__((address_space(4))) const entry_t centry_t;
  return (gfrag_t*)((centry_t*)table)[l];
}
typedef EH_LDS frag_t lds_frag_t;
typedef EH_LDS f32x4 lds_f32x4_t;
typedef EH_LDS float lds_float_t;
typedef EH_LDS int lds_int_t;
typedef EH_LDS volatile int lds_vint_t;

// LDS layout (byte offsets from the dynamic LDS base); "par" is the head parity.
struct Smem {
  EH_LDS char* base;
  unsigned y_bytes;  // KS * 1 KiB
  __device__ __forceinline__ lds_frag_t* ybuf(int par) const { return (lds_frag_t*)(base + par * y_bytes); }
  __device__ __forceinline__ unsigned o1() const { return 2 * y_bytes; }
  // head pieces (the part of a wave's first tile that starts at k > 0): [par][kStreamers][64] f32x4
  __device__ __forceinline__ lds_f32x4_t* part(int par) const {
    return (lds_f32x4_t*)(base + o1() + par * (kStreamers * kWave * 16));
  }
  // per-token statistics of each streamer wave: [par][5][kStreamers][16] float (ib stored as bits)
  __device__ __forceinline__ lds_float_t* wst(int par) const {
    return (lds_float_t*)(base + o1() + 2 * (kStreamers * kWave * 16) + par * (5 * kStreamers * 16 * 4));
  }
  __device__ __forceinline__ unsigned o2() const {
    return o1() + 2 * (kStreamers * kWave * 16) + 2 * (5 * kStreamers * 16 * 4);
  }
  // head id + 1 of the head piece currently in part(par)[wave]
  __device__ __forceinline__ lds_vint_t* part_flag(int par) const { return (lds_vint_t*)(base + o2() + par * (kStreamers * 4)); }
  __device__ __forceinline__ unsigned o3() const { return o2() + 2 * (kStreamers * 4); }
  __device__ __forceinline__ lds_vint_t* abort_flag(int par) const { return (lds_vint_t*)(base + o3() + par * 4); }
  // rows entering head l, left by the exchange wave for the LayerNorm wave (by parity of l)
  __device__ __forceinline__ lds_vint_t* live_word(int par) const { return (lds_vint_t*)(base + o3() + 8 + par * 4); }
  // number of streamer waves that have finished the head of this parity
  __device__ __forceinline__ lds_vint_t* arrived(int par) const { return (lds_vint_t*)(base + o3() + 16 + par * 4); }
  // number of heads (absolute index + 1 of the last one) whose records this workgroup has sent
  __device__ __forceinline__ lds_vint_t* sent_word() const { return (lds_vint_t*)(base + o3() + 24); }
};

inline size_t smem_bytes(int KS) {
  return 2 * (size_t)KS * kWave * 16 + 2 * kStreamers * kWave * 16 + 2 * 5 * kStreamers * 16 * 4 + 2 * kStreamers * 4 + 32;
}

// Push with an explicit index tie-break (rows may arrive in any order).
__device__ __forceinline__ void stats_push4_any(Stats& s, f32x4 z, int row0, int V) {
  const int nvalid = V - row0;
  float zc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) zc[i] = (i < nvalid) ? z[i] : -INFINITY;
  const float zmax = fmaxf(fmaxf(zc[0], zc[1]), fmaxf(zc[2], zc[3]));
  const int j = (zc[0] == zmax) ? 0 : (zc[1] == zmax) ? 1 : (zc[2] == zmax) ? 2 : 3;
  if (zmax > s.zb || (zmax == s.zb && row0 + j < s.ib && nvalid > 0)) {
    if (zmax > s.zb) {
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
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (i < nvalid) {
      const float t = z[i] * kLog2e - s.m;
      const float e = fast_exp2(t);
      s.S += e;
      s.U += t * e;
    }
  }
}

// LayerNorm of one row held in registers (one global pass), fp64 arithmetic,
// written to LDS in fragment order as token column n.
template <typename DT>
__device__ __forceinline__ void ln_row_to_lds(const void* row, int d, int KS,
                                              const float* __restrict__ gamma,
                                              const float* __restrict__ beta, float eps, int lane, int n,
                                              lds_frag_t* ybuf) {
  const int live_chunks = d / DT::EPL;
  float x[kMaxChunksPerLane][DT::EPL];
#pragma unroll
  for (int i = 0; i < kMaxChunksPerLane; ++i) {
    const int c = lane + i * kWave;
    if (c < live_chunks) load_elems<DT>(row, c * DT::EPL, x[i]);
  }
  double s = 0.0;
#pragma unroll
  for (int i = 0; i < kMaxChunksPerLane; ++i) {
    if (lane + i * kWave < live_chunks) {
#pragma unroll
      for (int e = 0; e < DT::EPL; ++e) s += (double)x[i][e];
    }
  }
  const double mu = wave_sum(s) / (double)d;
  double v = 0.0;
#pragma unroll
  for (int i = 0; i < kMaxChunksPerLane; ++i) {
    if (lane + i * kWave < live_chunks) {
#pragma unroll
      for (int e = 0; e < DT::EPL; ++e) {
        const double c = (double)x[i][e] - mu;
        v += c * c;
      }
    }
  }
  const double rstd = 1.0 / sqrt(wave_sum(v) / (double)d + (double)eps);
#pragma unroll
  for (int i = 0; i < kMaxChunksPerLane; ++i) {
    const int c = lane + i * kWave;
    if (c < KS * 4) {
      frag_t o = mk_frag(0, 0, 0, 0);
      if (c < live_chunks) {
        double y[DT::EPL];
#pragma unroll
        for (int e = 0; e < DT::EPL; ++e) {
          const int k = c * DT::EPL + e;
          y[e] = (double)gamma[k] * (((double)x[i][e] - mu) * rstd) + (double)beta[k];
        }
        o = pack_elems<DT>(y);
      }
      ybuf[(c >> 2) * kWave + (c & 3) * 16 + n] = o;
    }
  }
}

// Diagnostics: workgroup 0 stamps the 100 MHz wall clock at the phases of head l.
// slots: 0 streamer0 starts head, 1 streamer0 reaches the head's barrier,
// 4 exchange wave passes the previous barrier, 5 records of head l-1 sent,
// 6 exchange and decision for head l-1 done, 7 LayerNorm(l+1) done (LayerNorm
// wave), 8 exchange wave passes barrier l.
#ifdef EH_DIAGNOSTICS
__device__ __forceinline__ void stamp(const DecodeParams& p, int l, int slot, int lane) {
  if (p.trace && lane == 0) {
    if (blockIdx.x == 0) p.trace[l * 16 + slot] = wall_clock64();
    // every workgroup's view of one head (the fourth of the launch): slots 0, 1, 5, 6
    if (l == p.l0 + 3 && (slot < 2 || slot == 5 || slot == 6))
      p.trace[p.n_heads_alloc * 16 + blockIdx.x * 4 + (slot < 2 ? slot : slot - 3)] = wall_clock64();
  }
}
#else
__device__ __forceinline__ void stamp(const DecodeParams&, int, int, int) {}
#endif

__device__ __forceinline__ unsigned long long poll_mask(const unsigned long long* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// The vocabulary slice of a workgroup.  Slices are cut at multiples of four rows
// (the rows one lane's accumulator registers hold), not at tile boundaries, so
// that every workgroup streams the same number of bytes to within 2 %: with
// whole tiles, 3144 tiles over 256 workgroups leave some with 13 tiles and some
// with 12, and everybody waits for the 13s.  A tile cut by a slice boundary is
// visited by both neighbours; each fetches only its own rows (the other lanes
// are pointed at one shared dummy address) and counts only its own rows.
struct Slice {
  int row_lo, row_hi;  // rows [row_lo, row_hi) are mine
  int T0, T1;          // tiles [T0, T1) contain them
};
__device__ __forceinline__ Slice my_slice(int V) {
  const int grid = gridDim.x, bid = blockIdx.x;
  const int U = (V + 3) >> 2;
  Slice s;
  s.row_lo = (int)((long long)U * bid / grid) * 4;
  s.row_hi = min((int)((long long)U * (bid + 1) / grid) * 4, V);
  s.T0 = s.row_lo >> 4;
  s.T1 = s.row_hi > s.row_lo ? (s.row_hi + 15) >> 4 : s.T0;
  return s;
}

// record of workgroup g, row n, head l in exchange round `round` (0 or 1)
__device__ __forceinline__ unsigned long long* record_ptr(const DecodeParams& p, int round, int l, int g, int n) {
  return p.records + ((((long long)round * p.n_heads_alloc + l) * gridDim.x + g) * 16 + n) * 5;
}
__device__ __forceinline__ void write_record(const DecodeParams& p, unsigned long long* r, const Stats& s) {
  const unsigned long long tag = (unsigned long long)p.epoch << 32;
  const unsigned w[5] = {__float_as_uint(s.m), __float_as_uint(s.S), __float_as_uint(s.U),
                         __float_as_uint(s.zb), (unsigned)s.ib};
#pragma unroll
  for (int i = 0; i < 5; ++i)
    __hip_atomic_store(r + i, tag | w[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ------------------------------------------------------------------ streamers
// The weight stream of one wave is cut into groups of kRing fragments.  Two
// register buffers of one group each alternate: while one is consumed the other
// (and the rest of this one) is in flight, so 8..15 KiB per wave are always on
// their way, across head boundaries too.  Per head the number of groups is
// rounded up to an even count so that the buffers keep their roles; a padding
// group consumes nothing and re-reads the span's last fragment (a cache hit).
template <typename DT>
__device__ __forceinline__ void streamer(const DecodeParams& p, const Smem& sm, int wave, int lane) {
  constexpr int P = kRing;
  const int KS = p.KS;
  const Slice sl = my_slice(p.V);
  const int T0 = sl.T0, T1 = sl.T1;
  const int nF = (T1 - T0) * KS;
  // The slice's fragments are split evenly over the streamer waves, so a tile
  // may be cut between two neighbouring waves (never more: every span is at least
  // a tile long).  Slices too small for that are split by whole tiles instead.
  const bool even = nF >= kStreamers * KS;
  const int F0 = even ? (int)((long long)nF * wave / kStreamers) : KS * ((T1 - T0) * wave / kStreamers);
  const int F1 = even ? (int)((long long)nF * (wave + 1) / kStreamers) : KS * ((T1 - T0) * (wave + 1) / kStreamers);
  const int n_w = F1 - F0;
  const int G = (n_w + P - 1) / P;
  const int G2 = (G + 1) & ~1;
  const long long fb = (long long)T0 * KS + F0;
  const int q = lane >> 4;
  const int last = n_w > 0 ? n_w - 1 : 0;
  // lanes whose row of the slice's first / last tile belongs to a neighbour
  const bool lo_foreign = (T0 * 16 + (lane & 15)) < sl.row_lo;
  const bool hi_foreign = ((T1 - 1) * 16 + (lane & 15)) >= sl.row_hi;

  // fragment idx of my span in the head whose weights start at `head`; foreign
  // rows are not fetched: their lanes all read the head's first 16 bytes instead
  auto load_slot = [&](gfrag_t* head, int idx) {
    const int f = F0 + idx;
    const bool foreign = (f < KS && lo_foreign) || (f >= nF - KS && hi_foreign);
    gfrag_t* a = foreign ? head : head + (fb + idx) * kWave + lane;
    return __builtin_nontemporal_load(a);
  };

  frag_t bufA[P], bufB[P];
  {
    gfrag_t* h0 = head_weights(p.Wf, p.l0);
#pragma unroll
    for (int j = 0; j < P; ++j) bufA[j] = load_slot(h0, min(j, last));
#pragma unroll
    for (int j = 0; j < P; ++j) bufB[j] = load_slot(h0, min(P + j, last));
  }
  lds_barrier();  // y of head l0 is in LDS

  for (int l = p.l0; l < p.l1; ++l) {
    const int par = l & 1;
    gfrag_t* wcur = head_weights(p.Wf, l);
    const bool has_next = l + 1 < p.l1;
    gfrag_t* wnxt = has_next ? head_weights(p.Wf, l + 1) : wcur;
    const lds_frag_t* yb = sm.ybuf(par) + lane;
    Stats st;
    stats_init(st);
    int t = T0 + F0 / KS, ks = F0 % KS;
    int piece_k0 = ks;
    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
    if (wave == 0) stamp(p, l, 0, lane);

    // A piece (a run of k-steps of one tile) is complete.  A whole tile is folded
    // into the running statistics.  A head piece (my first tile, begun by the
    // previous wave) is parked in LDS at once for that wave to pick up; a tail
    // piece (my last tile, finished by the next wave) stays in `tail` until the
    // end of the head.
    f32x4 tail = f32x4{0.f, 0.f, 0.f, 0.f};
    int tail_tile = -1;
    auto flush = [&](bool tile_end) {
      const int row0 = t * 16 + q * 4;
      if (piece_k0 == 0 && tile_end) {
        if (row0 >= sl.row_lo) stats_push4<false>(st, acc, row0, sl.row_hi);
      } else if (piece_k0 > 0) {
        sm.part(par)[wave * kWave + lane] = acc;
        if (lane == 0) sm.part_flag(par)[wave] = l + 1;  // after the data: LDS keeps a wave's order
      } else {
        tail = acc;
        tail_tile = t;
      }
      acc = f32x4{0.f, 0.f, 0.f, 0.f};
      piece_k0 = 0;
    };

    // consume group g held in buf
    auto consume = [&](const frag_t (&buf)[P], int g) {
      const int i0 = g * P;
      if (i0 + P <= n_w && ks + P <= KS) {
        // fast path: the whole group lies inside one tile
        frag_t y[P];
#pragma unroll
        for (int j = 0; j < P; ++j) y[j] = yb[(ks + j) * kWave];
#pragma unroll
        for (int j = 0; j < P; ++j) acc = DT::mma(buf[j], y[j], acc);
        ks += P;
        const bool tile_end = (ks == KS);
        if (tile_end || i0 + P == n_w) flush(tile_end);
        if (tile_end) { ks = 0; ++t; }
      } else {
#pragma unroll
        for (int j = 0; j < P; ++j) {
          if (i0 + j < n_w) {
            const frag_t y = yb[ks * kWave];
            acc = DT::mma(buf[j], y, acc);
            const bool tile_end = (ks == KS - 1);
            if (tile_end || i0 + j == n_w - 1) flush(tile_end);
            if (++ks == KS) { ks = 0; ++t; }
          }
        }
      }
    };

    // refill buf with group gg of this head, or of the next head once gg >= G2.
    // Unconditional on purpose: a load under a branch makes the compiler drain
    // the ring before every use.  With nothing left to fetch the slots re-read
    // this wave's last fragment.
    auto refill = [&](frag_t (&buf)[P], int gg) {
      const bool same = gg < G2;
      gfrag_t* src = same ? wcur : wnxt;
      const int base = (same ? gg : gg - G2) * P;
      const bool real = same || has_next;
#pragma unroll
      for (int j = 0; j < P; ++j) buf[j] = load_slot(src, real ? min(base + j, last) : last);
    };

    for (int g = 0; g < G2; g += 2) {
      if (*sm.abort_flag(par)) break;  // every row has exited: drop this (speculative) head
      consume(bufA, g);
      refill(bufA, g + 2);
      consume(bufB, g + 1);
      refill(bufB, g + 3);
    }
    const bool dropped = *sm.abort_flag(par) != 0;
    if (tail_tile >= 0 && !dropped) {
      // the rest of my last tile is the next wave's head piece, parked long ago
      bool there = false;
      for (int spins = 0; spins < kSpinLimit && !there; ++spins) {
        there = sm.part_flag(par)[wave + 1] == l + 1;
        if (!there) {
          if (*sm.abort_flag(par)) break;
          __builtin_amdgcn_s_sleep(2);
        }
      }
      if (there) {
        tail += sm.part(par)[(wave + 1) * kWave + lane];
        const int row0 = tail_tile * 16 + q * 4;
        if (row0 >= sl.row_lo) stats_push4<false>(st, tail, row0, sl.row_hi);
      } else if (!*sm.abort_flag(par)) {
        if (lane == 0) {  // cannot happen unless a wave is stuck: give up cleanly
          atomicExch(p.status, 1);
          *sm.abort_flag(par) = 1;
        }
      }
    }
    // one record per token: fold the four row groups, leave them for the exchange wave
    st = stats_merge(st, stats_shfl_xor(st, 16));
    st = stats_merge(st, stats_shfl_xor(st, 32));
    lds_float_t* ws = sm.wst(par);
    if (lane < 16) {
      ws[(0 * kStreamers + wave) * 16 + lane] = st.m;
      ws[(1 * kStreamers + wave) * 16 + lane] = st.S;
      ws[(2 * kStreamers + wave) * 16 + lane] = st.U;
      ws[(3 * kStreamers + wave) * 16 + lane] = st.zb;
      ws[(4 * kStreamers + wave) * 16 + lane] = __int_as_float(st.ib);
    }
    if (wave == 0) stamp(p, l, 1, lane);
    if (lane == 0) __hip_atomic_fetch_add((EH_LDS int*)sm.arrived(par), 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    lds_barrier();  // B_l
    if (*sm.abort_flag(par)) return;
  }
}

// ------------------------------------------------------------------ service wave
// Cross-workgroup exchange.  Statistics travel in records of five 64-bit words
// {tag, payload}, written with device-scope stores and read with device-scope
// loads until every word carries this launch's tag.  The all-gather runs in two
// rounds of radix 16 (workgroups of my group, then one member of every group):
// two memory hops, no tickets, no counters and no word that more than 16
// workgroups poll (a single hot word polled by all 256 slowed the whole weight
// stream down when it was tried).  All workgroups merge the same records in the
// same order, so they all reach the same (bitwise identical) statistics and the
// same exit decision on their own.  Records of a speculated head that is dropped
// are never written; a tag from an older launch never matches, so nothing has to
// be reset between launches.
struct Service {
  const DecodeParams& p;
  const Smem sm;
  int lane;
  unsigned live;  // rows that enter the oldest head not yet decided

  __device__ __forceinline__ void fail_all(int par) {
    if (lane == 0) {
      atomicExch(p.status, 1);
      *sm.abort_flag(par) = 1;
    }
  }

  // Sends this workgroup's round-0 records of head l (parity par): the streamer
  // waves have left one record per token each in LDS; merged in wave order.
  __device__ __forceinline__ void announce(int l) {
    const lds_float_t* ws = sm.wst(l & 1);
    if (lane < 16 && ((live >> lane) & 1u)) {
      Stats s;
      stats_init(s);
#pragma unroll
      for (int w = 0; w < kStreamers; ++w) {
        Stats o;
        o.m = ws[(0 * kStreamers + w) * 16 + lane];
        o.S = ws[(1 * kStreamers + w) * 16 + lane];
        o.U = ws[(2 * kStreamers + w) * 16 + lane];
        o.zb = ws[(3 * kStreamers + w) * 16 + lane];
        o.ib = __float_as_int(ws[(4 * kStreamers + w) * 16 + lane]);
        s = stats_merge(s, o);
      }
      write_record(p, record_ptr(p, 0, l, blockIdx.x, lane), s);
    }
  }

  // A record as loaded: five {tag, payload} words.
  struct Raw {
    unsigned long long w[5];
  };
  __device__ __forceinline__ Raw load_record(const unsigned long long* r) const {
    Raw x;
#pragma unroll
    for (int i = 0; i < 5; ++i) x.w[i] = __hip_atomic_load(r + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return x;
  }
  // True if every word carries this launch's tag; then `o` is the record.
  __device__ __forceinline__ bool decode_record(const Raw& x, Stats& o) const {
    bool ok = true;
#pragma unroll
    for (int i = 0; i < 5; ++i) ok = ok && ((unsigned)(x.w[i] >> 32) == p.epoch);
    o.m = __uint_as_float((unsigned)x.w[0]);
    o.S = __uint_as_float((unsigned)x.w[1]);
    o.U = __uint_as_float((unsigned)x.w[2]);
    o.zb = __uint_as_float((unsigned)x.w[3]);
    o.ib = (int)(unsigned)x.w[4];
    return ok;
  }

  // Lane i < count holds (in `x`) the record of the i-th source of a round.  If
  // every record is there they are merged in lane order (fixed tree), so every
  // reader of the same records gets bitwise the same result, and true is
  // returned; otherwise false (nothing is kept: the caller tries again later).
  __device__ __forceinline__ bool merge_round(const Raw& x, int count, Stats& out) const {
    Stats s;
    stats_init(s);
    bool have = true;
    if (lane < count) have = decode_record(x, s);
    if (!__all(have)) return false;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) s = stats_merge(s, stats_shfl_xor(s, o));
    // the merge is not bitwise symmetric in its operands (fused multiply-adds), so
    // lanes may differ in the last bit: everybody takes lane 0's result, which is
    // computed from the same operands in the same order in every workgroup
    out.m = __shfl(s.m, 0); out.S = __shfl(s.S, 0); out.U = __shfl(s.U, 0);
    out.zb = __shfl(s.zb, 0); out.ib = __shfl(s.ib, 0);
    return true;
  }

  // A two-round all-gather with radix kRadix, then finalise and
  // decide.  Round 0: the statistics of the workgroups of my group -> my round-1
  // record (identical for all members of a group).  Round 1: one member of every
  // group -> the statistics of the whole vocabulary.  A record is polled by at
  // most kRadix workgroups, and a workgroup polls at most 2*kRadix records per
  // row, so the waiting costs little bandwidth and has no hot spot.
  //
  // Several heads are in flight at once: `c` is the oldest head not yet decided,
  // `sent` the number of heads announced so far.  Round 0 runs for every announced
  // head (its result does not depend on earlier decisions; rows that turn out to
  // have exited only cost a wasted record), round 1 and the decision run for head
  // c only, in order.  done0 holds, for the heads c .. c+3 (slot = head & 3), the
  // rows whose round-1 record this workgroup has written; done1 the rows of head
  // c that are decided.  pass() makes one sweep and returns true if head c got
  // decided, with `live` then holding the rows that go on to head c+1.
  static constexpr int kRadix = 16;
  static constexpr int kWindow = 4;
  unsigned long long done0 = 0;
  unsigned done1 = 0, stay = 0;
  int c = 0, sent = 0;

  __device__ __forceinline__ bool pass() {
    const int grid = gridDim.x, me = blockIdx.x;
    const int member = me % kRadix;
    const int g0 = (me / kRadix) * kRadix;
    const int gsize = min(kRadix, grid - g0);
    const int ngroups = (grid + kRadix - 1) / kRadix;
    const bool writer = me == 0 && lane == 0;
    // One row per open head and round in a sweep (the lowest one that still needs
    // work), with all loads of the sweep issued before any is looked at, so that a
    // sweep costs one memory round trip however many heads are open.
    Raw x0[kWindow], x1;
    int row0[kWindow], row1 = -1;
#pragma unroll
    for (int k = 0; k < kWindow; ++k) {
      const int h = c + k;
      const int sh = (h & (kWindow - 1)) * 16;
      const unsigned todo = (h < sent) ? (live & ~(unsigned)((done0 >> sh) & 0xffffu)) : 0u;
      row0[k] = todo ? __ffs(todo) - 1 : -1;
      if (row0[k] >= 0 && lane < gsize) x0[k] = load_record(record_ptr(p, 0, h, g0 + lane, row0[k]));
    }
    const int sc = (c & (kWindow - 1)) * 16;
    if (c < sent) {
      const unsigned todo = (unsigned)((done0 >> sc) & 0xffffu) & live & ~done1;
      row1 = todo ? __ffs(todo) - 1 : -1;
      if (row1 >= 0 && lane < ngroups) {
        const int j = lane;
        const int src = j * kRadix + min(member, min(kRadix, grid - j * kRadix) - 1);
        x1 = load_record(record_ptr(p, 1, c, src, row1));
      }
    }
#pragma unroll
    for (int k = 0; k < kWindow; ++k) {
      if (row0[k] < 0) continue;
      const int h = c + k;
      Stats s;
      if (merge_round(x0[k], gsize, s)) {
        if (lane == 0) write_record(p, record_ptr(p, 1, h, me, row0[k]), s);
        done0 |= 1ull << ((h & (kWindow - 1)) * 16 + row0[k]);
      }
    }
    if (row1 >= 0) {
      const int n = row1;
      Stats s;
      if (merge_round(x1, ngroups, s)) {
        done1 |= 1u << n;
        float H, lse;
        stats_finalize(s, H, lse);
        if (p.decide) {
          const bool leaves = (c == p.n_heads - 1) || (H < p.tau[c]);
          if (!leaves) stay |= 1u << n;
          if (writer) {
            if (leaves) {
              p.exit_layer[n] = c;
              p.token[n] = stats_token(s);
            }
            if (p.H_out) p.H_out[(long long)c * p.n_rows + n] = H;
          }
        } else if (writer) {
          if (p.H) p.H[n] = H;
          if (p.lse) p.lse[n] = lse;
          if (p.argmax) p.argmax[n] = stats_token(s);
        }
      }
    }
    if (c >= sent || done1 != live) return false;
    if (writer && p.decide) {
      if (p.n_evals) atomicAdd(p.n_evals, (unsigned long long)__popc(live));
      if (p.H_out) {
        for (int n = 0; n < p.n_rows; ++n)
          if (!((live >> n) & 1u)) p.H_out[(long long)c * p.n_rows + n] = NAN;
        if (stay == 0u || c == p.l1 - 1) {
          const int total = (p.n_heads - (c + 1)) * p.n_rows;
          for (int i = 0; i < total; ++i) p.H_out[(long long)(c + 1) * p.n_rows + i] = NAN;
        }
      }
    }
    live = p.decide ? stay : 0u;
    done0 &= ~(0xffffull << sc);
    done1 = stay = 0u;
    ++c;
    return true;
  }

  template <typename DT>
  __device__ __forceinline__ void layernorm_rows(int l, unsigned rows, lds_frag_t* ybuf) {
    const int esz = DT::ESZ;
    for (int n = 0; n < 16; ++n) {
      if (!((rows >> n) & 1u)) continue;
      const long long r = p.row_idx ? p.row_idx[n] : n;
      const char* row = (const char*)p.h + ((long long)l * p.layer_stride + r * p.row_stride) * esz;
      ln_row_to_lds<DT>(row, p.d, p.KS, p.gamma[l], p.beta[l], p.eps, lane, n, ybuf);
    }
  }

  __device__ __forceinline__ unsigned initial_live() const {
    int n_live = p.n_rows;
    if (p.n_rows_dev) n_live = min(max(*p.n_rows_dev, 0), p.n_rows);
    return n_live >= 32 ? 0xffffffffu : ((1u << n_live) - 1u);
  }

  // Exchange wave.  In the window in which the streamers work on head l it sends
  // this workgroup's records of head l-1 and then keeps sweeping the open
  // exchanges until the streamers have finished head l.  Only when the oldest open
  // exchange falls more than kMaxLag heads behind does it hold the streamers back
  // (bounded wait), so one slow workgroup somewhere does not stall this one at
  // once.  The streamers are told as soon as every row has exited.
  __device__ __forceinline__ void run_exchange() {
    live = initial_live();
    if (lane == 0) *sm.live_word((p.l0 + 1) & 1) = (int)live;  // read by the LayerNorm wave in the first window
    c = sent = p.l0;
    lds_barrier();  // B_{-1}
    for (int l = p.l0; l < p.l1; ++l) {
      const int par = l & 1;
      stamp(p, l, 4, lane);
      if (lane == 0) *sm.arrived(par ^ 1) = 0;  // next window's count of finished streamers
      if (l > p.l0) {
        announce(l - 1);
        sent = l;
      }
      stamp(p, l, 5, lane);
      for (int spins = 0; c < sent; ++spins) {
        if (pass()) {
          spins = 0;
          if (live == 0u) {
            if (lane == 0) *sm.abort_flag(par) = 1;
            break;
          }
          continue;
        }
        // The streamers must not wait for this wave: between sweeps, watch (in LDS,
        // which costs nothing) for them to finish the head, and carry what is
        // still open over into the next window when they have.
        const bool may_defer = c >= l - kMaxLag;
        bool done = false;
        for (int k = 0; k < 24 && !done; ++k) {
          done = may_defer && *sm.arrived(par) >= kStreamers;
          if (!done) __builtin_amdgcn_s_sleep(2);
        }
        if (done) break;
        if (spins >= p.spin_limit) { fail_all(par); break; }
      }
      if (lane == 0) *sm.live_word(par) = (int)live;
      stamp(p, l, 6, lane);
      lds_barrier();  // B_l
      stamp(p, l, 8, lane);
      if (*sm.abort_flag(par)) return;
    }
    announce(p.l1 - 1);
    sent = p.l1;
    for (int spins = 0; c < sent && live != 0u; ++spins) {
      if (pass()) { spins = 0; continue; }
      if (spins >= p.spin_limit) {
        if (lane == 0) atomicExch(p.status, 1);
        return;
      }
      __builtin_amdgcn_s_sleep(4);
    }
  }

  // LayerNorm wave: one head ahead of the streamers (speculative: a row that turns
  // out to have exited only wastes its column).  The set of rows it normalises is
  // the one the exchange wave knew a window earlier, a superset of the live rows.
  template <typename DT>
  __device__ __forceinline__ void run_layernorm() {
    live = initial_live();
    layernorm_rows<DT>(p.l0, live, sm.ybuf(p.l0 & 1));
    lds_barrier();  // B_{-1}
    for (int l = p.l0; l < p.l1; ++l) {
      const int par = l & 1;
      live = (unsigned)*sm.live_word(par ^ 1);
      if (l + 1 < p.l1) layernorm_rows<DT>(l + 1, live, sm.ybuf(par ^ 1));
      stamp(p, l, 7, lane);
      lds_barrier();  // B_l
      if (*sm.abort_flag(par)) return;
    }
  }
};

template <typename DT>
__global__ __launch_bounds__(kThreads, 1) void decode_kernel(const DecodeParams p) {
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];
  Smem sm;
  sm.base = (EH_LDS char*)smem_raw;
  sm.y_bytes = (unsigned)p.KS * kWave * 16;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave-uniform, kept in an SGPR
  // no live row at all (the count lives on the device: e.g. a drafting loop that has stopped):
  // every workgroup reads the same word, so the whole grid leaves together
  if (p.n_rows_dev && *p.n_rows_dev <= 0) return;
  if (blockIdx.x == 0) {
    // Preset the outputs of the live rows (workgroup 0 is also the one that writes the results,
    // much later): whatever a launch that gives up has not finished reads -1 / NaN.
    int n_live = p.n_rows;
    if (p.n_rows_dev) n_live = min(*p.n_rows_dev, p.n_rows);
    const int t = threadIdx.x;
    if (p.decide) {
      if (t < n_live) { p.exit_layer[t] = -1; p.token[t] = -1; }
      if (p.H_out)
        for (int i = t; i < p.n_heads * p.n_rows; i += kThreads) p.H_out[i] = NAN;
    } else if (t < n_live) {
      if (p.H) p.H[t] = NAN;
      if (p.lse) p.lse[t] = NAN;
      if (p.argmax) p.argmax[t] = -1;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // landed before this workgroup's barrier below
  }
  // a launch that gave up has not been acknowledged yet (eh_check clears the flag): do nothing
  if (*(volatile int*)p.status != 0) return;
  // zero both activation buffers (columns of rows that are not live stay zero)
  {
    lds_frag_t* y = sm.ybuf(0);
    const int total = 2 * p.KS * kWave;
    for (int i = threadIdx.x; i < total; i += kThreads) y[i] = mk_frag(0, 0, 0, 0);
    if (threadIdx.x < 2) {
      *sm.abort_flag(threadIdx.x) = 0;
      *sm.arrived(threadIdx.x) = 0;
    }
    if (threadIdx.x == 2) *sm.sent_word() = 0;
    if (threadIdx.x < 2 * kStreamers) sm.part_flag(0)[threadIdx.x] = 0;
  }
  lds_barrier();
  if (wave < kStreamers) {
    streamer<DT>(p, sm, wave, lane);
  } else {
    Service sv{p, sm, lane, 0u};
    if (wave == kStreamers) sv.run_exchange();
    else sv.template run_layernorm<DT>();
  }
}

}  // namespace

hipError_t decode_prepare(eh_ctx* c) {
  c->decode_grid = 0;
  const int epl = c->dtype == EH_BF16 ? 8 : 4;
  if (c->d > kMaxChunksPerLane * kWave * epl) return hipSuccess;  // row does not fit the register LayerNorm
  if (!c->bias.empty()) return hipSuccess;  // heads with a bias vector take the general path
  const size_t smem = smem_bytes(c->KS);
  hipDeviceProp_t prop;
  hipError_t e = hipGetDeviceProperties(&prop, c->device);
  if (e != hipSuccess) return e;
  if (smem > (size_t)prop.sharedMemPerBlock && smem > (size_t)prop.maxSharedMemoryPerMultiProcessor) return hipSuccess;
  const void* fn = c->dtype == EH_BF16 ? (const void*)decode_kernel<DtBf16> : (const void*)decode_kernel<DtF32>;
  e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (e != hipSuccess) { (void)hipGetLastError(); return hipSuccess; }
  int per_cu = 0;
  e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, kThreads, smem);
  if (e != hipSuccess || per_cu < 1) { (void)hipGetLastError(); return hipSuccess; }
  // the kernel waits on other workgroups, so all of them must be resident at once
  c->num_cu = prop.multiProcessorCount;
  c->decode_grid = std::min(prop.multiProcessorCount, c->VT);
  c->decode_smem = smem;
  return hipSuccess;
}

hipError_t decode_launch(const eh_ctx* c, const DecodeParams& p, hipStream_t s) {
  if (c->dtype == EH_BF16)
    hipLaunchKernelGGL((decode_kernel<DtBf16>), dim3(c->decode_grid), dim3(kThreads), c->decode_smem, s, p);
  else
    hipLaunchKernelGGL((decode_kernel<DtF32>), dim3(c->decode_grid), dim3(kThreads), c->decode_smem, s, p);
  return hipGetLastError();
}

}  // namespace eh
