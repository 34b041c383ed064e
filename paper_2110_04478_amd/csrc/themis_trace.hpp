// Scalable queue simulation for traces: several collectives of different
// sizes sharing the per-dimension queues (one lane per scenario, state in a
// per-scenario region of the caller's HBM workspace).
//
// With thousands of chunks per scenario the state no longer fits LDS, and with
// one chunk size per collective Smallest-Chunk-First has far more than 16
// distinct resident sizes.  The structure is the same as in the LDS fast path,
// scaled up: every distinct resident size chunk_q * 2^-E(mask) over all
// (collective q, reduced-dims mask) pairs gets a rank (ascending size, equal
// sizes share a rank), every dimension owns one FIFO list per rank, and a
// two-level bitmap per dimension finds the lowest non-empty rank.  Each
// chunk-stage event then costs a bounded number of memory operations instead
// of a scan over all waiting chunks.
//
// Covered: power-of-two NPU counts under either queue policy, any NPU counts
// under first-in-first-out (stage times by the order's own divisions); up to
// kTraceMaxColl collectives, any release times (a release that falls on the
// very instant of a completion is left to the generic path, which orders the
// arrivals of both kinds by chunk id).  Everything else stays on the generic
// path.
#pragma once

#include "themis_fast.hpp"

namespace themis {

constexpr uint32_t kTraceMaxColl = 256;   // ranks <= 4096: 128 bitmap leaves, 4 summary words
constexpr uint32_t kTraceLeafWords = kTraceMaxColl * 16 / 32;
constexpr uint32_t kTraceSumWords = 4;
constexpr uint32_t kNoChunk = 0xffffu;
constexpr uint32_t kTraceCollBytes = 64;
// NPU counts that are not powers of two (division mode): a chunk's resident
// size depends on its whole order, so a collective has one size rank per
// (dimension, phase, order): 4 x 2 x 24 16-bit ranks.
constexpr uint32_t kTraceStates = 48;
constexpr uint32_t kTraceMaxRanks = kTraceMaxColl * 16;

// Byte offsets inside one scenario's region of the workspace.
struct TraceLayout {
  uint32_t G;   // chunk slots (max_chunks * max_coll)
  uint32_t Q;   // collectives the region is sized for
  uint32_t R;   // ranks per dimension: Q * 16 in halving mode, up to Q * 48 in division mode, 4096 at most
  uint32_t off_ht, off_bm, off_col, off_sq, off_sq2, off_rq, off_srd, off_mh;
  uint32_t bytes;  // multiple of 16; 0 if the batch cannot use this path
};

__host__ __device__ inline TraceLayout trace_layout(uint32_t max_chunks, uint32_t max_coll) {
  TraceLayout t;
  t.G = max_chunks * max_coll;
  t.Q = max_coll;
  t.R = max_coll * kTraceStates < kTraceMaxRanks ? max_coll * kTraceStates : kTraceMaxRanks;
  if (max_coll == 0u || max_coll > kTraceMaxColl) { t.bytes = 0; return t; }
  uint32_t o = t.G * 4u;                   // W: one dword per chunk
  t.off_ht = o;  o += 4u * t.R * 4u;       // head | tail << 16 per (dimension, rank)
  t.off_bm = o;  o += 4u * kTraceLeafWords * 4u;   // bitmap leaves (when they are not in LDS)
  // one 64-byte record per collective: the size rank of each of the 16 masks
  // (u16, one 32-byte row), the chunk bytes and the release time (f64 each)
  t.off_col = (o + 63u) & ~63u; o = t.off_col + t.Q * kTraceCollBytes;
  t.off_sq = o;  o += ((t.Q + 1u) & ~1u) * 2u;   // collectives sorted by chunk size
  t.off_sq2 = o; o += ((t.Q + 1u) & ~1u) * 2u;   // the merge sort's second buffer
  t.off_rq = o;  o += ((t.Q + 1u) & ~1u) * 2u;   // collectives sorted by release time
  // division mode: the ranks of every collective, and the heads of the merge that builds them
  t.off_srd = (o + 15u) & ~15u; o = t.off_srd + t.Q * 4u * kTraceStates * 2u;
  t.off_mh = (o + 15u) & ~15u;  o = t.off_mh + kTraceStates * 16u;
  t.bytes = (o + 63u) & ~63u;
  return t;
}

// One scenario's region with bounds-clamped accessors: an index that a logic
// error pushed out of range still stays inside the region.
struct TraceRegion {
  uint8_t* base;
  TraceLayout t;
  __device__ __forceinline__ uint32_t& W(uint32_t g) const {
    return ((uint32_t*)base)[min(g, t.G - 1u)];
  }
  __device__ __forceinline__ uint32_t& HT(uint32_t k, uint32_t r) const {
    return ((uint32_t*)(base + t.off_ht))[(k & 3u) * t.R + min(r, t.R - 1u)];
  }
  __device__ __forceinline__ uint32_t& BM(uint32_t k, uint32_t leaf) const {
    return ((uint32_t*)(base + t.off_bm))[(k & 3u) * kTraceLeafWords + (leaf & (kTraceLeafWords - 1u))];
  }
  __device__ __forceinline__ double& CH(uint32_t q) const {
    return *(double*)(base + t.off_col + min(q, t.Q - 1u) * kTraceCollBytes + 32u);
  }
  __device__ __forceinline__ uint16_t& SR(uint32_t q, uint32_t mask) const {
    return ((uint16_t*)(base + t.off_col + min(q, t.Q - 1u) * kTraceCollBytes))[mask & 15u];
  }
  // the 16 ranks of collective q as eight dwords (read as whole dwords what
  // SR() wrote as halves: the type says that it may alias them)
  typedef uint4 __attribute__((may_alias)) RankRow;
  __device__ __forceinline__ const RankRow* SRrow(uint32_t q) const {
    return (const RankRow*)(base + t.off_col + min(q, t.Q - 1u) * kTraceCollBytes);
  }
  __device__ __forceinline__ uint16_t& SQ(uint32_t j) const {
    return ((uint16_t*)(base + t.off_sq))[min(j, t.Q - 1u)];
  }
  // buffer 0 is SQ, buffer 1 the merge sort's spare, buffer 2 the release order
  __device__ __forceinline__ uint16_t& SQbuf(uint32_t which, uint32_t j) const {
    const uint32_t off = which == 0u ? t.off_sq : which == 1u ? t.off_sq2 : t.off_rq;
    return ((uint16_t*)(base + off))[min(j, t.Q - 1u)];
  }
  // division mode: rank of collective q's chunks waiting for dimension k in state st
  __device__ __forceinline__ uint16_t& SRD(uint32_t q, uint32_t k, uint32_t st) const {
    return ((uint16_t*)(base + t.off_srd))[(min(q, t.Q - 1u) * 4u + (k & 3u)) * kTraceStates +
                                           min(st, kTraceStates - 1u)];
  }
  // heads of the merge: value (f64), position (u32), what the list is (u32)
  __device__ __forceinline__ double& MHV(uint32_t l) const {
    return ((double*)(base + t.off_mh))[min(l, kTraceStates - 1u)];
  }
  __device__ __forceinline__ uint32_t& MHP(uint32_t l) const {
    return ((uint32_t*)(base + t.off_mh + kTraceStates * 8u))[min(l, kTraceStates - 1u)];
  }
  __device__ __forceinline__ uint32_t& MHL(uint32_t l) const {
    return ((uint32_t*)(base + t.off_mh + kTraceStates * 12u))[min(l, kTraceStates - 1u)];
  }
  __device__ __forceinline__ double& REL(uint32_t q) const {
    return *(double*)(base + t.off_col + min(q, t.Q - 1u) * kTraceCollBytes + 40u);
  }
};

// Chunk dword: bits 0-3 reduced-dims mask, bit 4 phase, bits 8-15 order code,
// bits 16-31 next chunk in its list (kNoChunk = last).
__device__ __forceinline__ uint32_t trace_word(uint32_t code, uint32_t state0) {
  return state0 | (code << 8) | (kNoChunk << 16);
}

// Collective indices in ascending (key, index) order into buffer `dst` (0 or
// 2; buffer 1 is the spare): a bottom-up merge sort (every step is a round
// trip to memory, so the number of steps matters: Q log Q instead of the
// Q^2 / 4 of an insertion sort).  Runs of `width` sorted indices are merged
// from one buffer into the other, the left run winning ties, so equal keys
// stay in index order.
template <typename KeyOf>
__device__ inline void trace_sort_collectives(const TraceRegion& rg, uint32_t Q, uint32_t dst,
                                              KeyOf key_of) {
  for (uint32_t a = 0; a < Q; ++a) rg.SQbuf(dst, a) = (uint16_t)a;
  uint32_t src = dst, other = 1u;
  for (uint32_t width = 1u; width < Q; width *= 2u) {
    for (uint32_t lo = 0u; lo < Q; lo += 2u * width) {
      const uint32_t mid = min(lo + width, Q), hi = min(lo + 2u * width, Q);
      uint32_t a = lo, b = mid;
      uint32_t ia = rg.SQbuf(src, a), ib = b < hi ? (uint32_t)rg.SQbuf(src, b) : 0u;
      double ka = key_of(ia), kb = b < hi ? key_of(ib) : inf64();
      for (uint32_t o = lo; o < hi; ++o) {
        const bool left = a < mid && (b >= hi || !(ka > kb));
        rg.SQbuf(other, o) = (uint16_t)(left ? ia : ib);
        if (left) {
          ++a;
          if (a < mid) { ia = rg.SQbuf(src, a); ka = key_of(ia); }
        } else {
          ++b;
          if (b < hi) { ib = rg.SQbuf(src, b); kb = key_of(ib); }
        }
      }
    }
    const uint32_t t = src; src = other; other = t;
  }
  if (src != dst)
    for (uint32_t a = 0; a < Q; ++a) rg.SQbuf(dst, a) = rg.SQbuf(src, a);
}

// Ranks of all resident sizes: a merge of the 2^D sorted lists
// { chunk_q * 2^-E(mask) : q in ascending chunk order }, one list per mask.
// Returns the number of distinct ranks.  lds: 48 dwords of this lane.
__device__ inline uint32_t trace_build_ranks(const TraceRegion& rg, uint32_t Q, uint32_t D,
                                             uint32_t epack, const LaneLds& lds) {
  trace_sort_collectives(rg, Q, 0u, [&](uint32_t q) { return (double)rg.CH(q); });
  // merge heads in LDS: value (dwords 2m, 2m+1) and position (dword 32 + m)
  const uint32_t nm = 1u << D;
  const double first = rg.CH(rg.SQ(0));
  for (uint32_t m = 0; m < 16u; ++m) {
    const double v = m < nm ? scale_down(first, esum(epack, m)) : inf64();
    *(uint32_t*)lds.dword(2u * m) = (uint32_t)__double2loint(v);
    *(uint32_t*)lds.dword(2u * m + 1u) = (uint32_t)__double2hiint(v);
    *(uint32_t*)lds.dword(32u + m) = 0u;
  }
  uint32_t rank = 0;
  double prev = -1.0;
  const uint32_t total = Q * nm;
  for (uint32_t out = 0; out < total; ++out) {
    uint32_t mb = 0;
    double vb = inf64();
    for (uint32_t m = 0; m < nm; ++m) {
      const double v = __hiloint2double((int)*(const uint32_t*)lds.dword(2u * m + 1u),
                                        (int)*(const uint32_t*)lds.dword(2u * m));
      if (v < vb) { vb = v; mb = m; }
    }
    if (out > 0u && vb > prev) ++rank;
    prev = vb;
    const uint32_t p = *(const uint32_t*)lds.dword(32u + mb);
    rg.SR(rg.SQ(p), mb) = (uint16_t)rank;
    const uint32_t pn = p + 1u;
    const double vn = pn < Q ? scale_down(rg.CH(rg.SQ(pn)), esum(epack, mb)) : inf64();
    *(uint32_t*)lds.dword(2u * mb) = (uint32_t)__double2loint(vn);
    *(uint32_t*)lds.dword(2u * mb + 1u) = (uint32_t)__double2hiint(vn);
    *(uint32_t*)lds.dword(32u + mb) = pn;
  }
  return rank + 1u;
}

// Division mode ----------------------------------------------------------
// Lexicographic rank (0..23) of an order code read as a permutation of all
// four dimensions (the unused fields take their own index).
__device__ __forceinline__ uint32_t trace_order_rank(uint32_t code, uint32_t D) {
  const uint32_t c8 = code | (0xe4u & ~((1u << (2u * D)) - 1u));
  const uint32_t o0 = c8 & 3u, o1 = (c8 >> 2) & 3u, o2 = (c8 >> 4) & 3u, o3 = (c8 >> 6) & 3u;
  const uint32_t r1 = o1 - (o1 > o0 ? 1u : 0u);
  return 6u * o0 + 2u * r1 + (o2 > o3 ? 1u : 0u);
}
// The state a chunk with stored order `code` is in while it waits in phase
// `phase` (its dimension follows from both): index into a collective's ranks.
__device__ __forceinline__ uint32_t trace_state(uint32_t code, uint32_t phase, uint32_t D) {
  return (phase & 1u) * 24u + trace_order_rank(code, D);
}

// Resident bytes of a chunk that waits for the dimension at `place` of its
// stored order, one division or multiplication at a time in the order the
// stages run (Sec. 2.1: a Reduce-Scatter stage leaves 1/P of the data, an
// All-Gather stage P times as much): the Smallest-Chunk-First key.
__device__ __forceinline__ double trace_resident_bytes(const Scenario& s, double chunk, uint32_t code,
                                                       uint32_t place, uint32_t phase, bool gather) {
  double x = chunk;
  const uint32_t D = (uint32_t)s.D;
  if (!gather) {
    const uint32_t divisions = phase ? D : place;
    for (uint32_t j = 0; j < divisions; ++j) {
      const uint32_t kj = (code >> (2u * j)) & 3u;
      x = x / (double)sel4((int)kj, s.P[0], s.P[1], s.P[2], s.P[3]);
    }
  }
  if (phase) {
    for (uint32_t j = D; j-- > place + 1u;) {
      const uint32_t kj = (code >> (2u * j)) & 3u;
      x = x * (double)sel4((int)kj, s.P[0], s.P[1], s.P[2], s.P[3]);
    }
  }
  return x;
}

// Lists per dimension that the ranks of division mode are merged from.
__device__ __forceinline__ uint32_t trace_division_lists(uint32_t D, bool one_phase) {
  return factorial_u32(D) * (one_phase ? 1u : 2u);
}

// Ranks of all resident sizes in division mode, per dimension: for every
// (phase, order) the sizes over the collectives in ascending chunk order are
// ascending (a rounded division or multiplication by a constant keeps the
// order), so the ranks of dimension k come from a merge of those lists, equal
// sizes sharing a rank.  Needs Q * trace_division_lists() <= R.
__device__ inline void trace_build_ranks_divided(const TraceRegion& rg, const Scenario& s, uint32_t Q,
                                                 bool gather, bool rs_only) {
  const uint32_t D = (uint32_t)s.D;
  trace_sort_collectives(rg, Q, 0u, [&](uint32_t q) { return (double)rg.CH(q); });
  const uint32_t F = factorial_u32(D);
  for (uint32_t k = 0; k < D; ++k) {
    uint32_t nl = 0;
    for (uint32_t idx = 0; idx < F; ++idx) {
      const uint32_t code = nth_permutation_code(D, idx);
      uint32_t place = 0;
      for (uint32_t j = 0; j < D; ++j) place = ((code >> (2u * j)) & 3u) == k ? j : place;
      for (uint32_t phase = gather ? 1u : 0u; phase < (rs_only ? 1u : 2u); ++phase) {
        rg.MHL(nl) = code | (phase << 8) | (place << 9);
        rg.MHP(nl) = 0u;
        rg.MHV(nl) = trace_resident_bytes(s, rg.CH(rg.SQ(0)), code, place, phase, gather);
        ++nl;
      }
    }
    uint32_t rank = 0;
    double prev = -1.0;
    const uint32_t total = Q * nl;
    for (uint32_t out = 0; out < total; ++out) {
      uint32_t lb = 0;
      double vb = inf64();
      for (uint32_t l = 0; l < nl; ++l) {
        const double v = rg.MHV(l);
        if (v < vb) { vb = v; lb = l; }
      }
      if (out > 0u && vb > prev) ++rank;
      prev = vb;
      const uint32_t what = rg.MHL(lb);
      const uint32_t code = what & 0xffu, phase = (what >> 8) & 1u, place = (what >> 9) & 3u;
      const uint32_t p = rg.MHP(lb);
      rg.SRD(rg.SQ(p), k, trace_state(code, phase, D)) = (uint16_t)rank;
      const uint32_t pn = p + 1u;
      rg.MHP(lb) = pn;
      rg.MHV(lb) = pn < Q ? trace_resident_bytes(s, rg.CH(rg.SQ(pn)), code, place, phase, gather)
                          : inf64();
    }
  }
}

// Per-lane LDS of the trace path: 48 dwords for trace_build_ranks, reused
// afterwards for the summary words (dwords 0-15) and, in the large variant,
// followed by the bitmap leaves of all four dimensions.  The large variant
// (132 KiB per wavefront, one wavefront per CU) is for batches of no more
// wavefronts than CUs, where nothing else could have used the LDS anyway.
// (the last four dwords: per dimension the lowest non-empty rank)
constexpr uint32_t kTraceLdsWords = 48 + 4;
constexpr uint32_t kTraceLdsWordsBitmaps = 16 + 4 * kTraceLeafWords + 4;

// Runs the simulation of one trace.  The region must hold CH[q] (resident
// bytes at mask 0 of a chunk of collective q), REL[q] (its release time; read
// only if has_release) and W[g] = trace_word(stored code, state0) for
// g = q*C + i; state0 / rs_only as in FastScenario.
// Returns false if time failed to advance somewhere (generic path decides).
// kReleases: the batch carries release times (has_release: this scenario has
// one that is not zero); without them the loop is compiled without the step
// that looks for the next release.  kFix: the batch carries fixed delays.
// kLdsBitmaps: the bitmap leaves live in LDS (kTraceLdsWordsBitmaps dwords per
// lane) instead of the region; the summary words always do.
// What the trace loop keeps per dimension, one register (pair) each.
struct TraceDims {
  double f0, f1, f2, f3;    // finish time of the running stage, a quiet NaN when idle
  double z0, z1, z2, z3;    // busy time
  uint32_t s0, s1, s2, s3;  // the running stage: chunk << 2 | dimension
  uint32_t n0, n1, n2, n3;  // what its completion will do (see simulate_trace_fast)
  uint32_t e0, e1, e2, e3;  // operations started (kept when queue orders are written)
};

// Dimension k of each lane starts a stage at `now` on x bytes: the lanes with
// k == j take their turn as the active ones, j = 0..3 (see start_stage_scaled):
//   t = [a_j +] x * c_j;  f_j = now + t;  z_j += t;  s_j = sv;  n_j = nx;
//   kQueue: pos = e_j, e_j += 1.
// Returns t; pos is left alone without kQueue.
#define THEMIS_TRACE_NEXT(J) "v_mov_b32_e32 %[n" #J "], %[nx]\n\t"
#define THEMIS_TRACE_COUNT(J) \
  "v_mov_b32_e32 %[pos], %[e" #J "]\n\t" "v_add_u32_e32 %[e" #J "], 1, %[e" #J "]\n\t"
#define THEMIS_TRACE_PLAIN(J)                                                             \
  THEMIS_LANES_OF(J) THEMIS_MUL(J) THEMIS_END(J) THEMIS_BUSY(J) THEMIS_SERVE(J) THEMIS_TRACE_NEXT(J) \
  THEMIS_ALL_LANES
#define THEMIS_TRACE_FULL(J)                                                           \
  THEMIS_LANES_OF(J) THEMIS_MUL(J) THEMIS_FIX(J) THEMIS_END(J) THEMIS_BUSY(J) THEMIS_SERVE(J) \
  THEMIS_TRACE_NEXT(J) THEMIS_TRACE_COUNT(J) THEMIS_ALL_LANES
#define THEMIS_N_OPERANDS [n0] "+v"(d.n0), [n1] "+v"(d.n1), [n2] "+v"(d.n2), [n3] "+v"(d.n3)
#define THEMIS_E_OPERANDS [e0] "+v"(d.e0), [e1] "+v"(d.e1), [e2] "+v"(d.e2), [e3] "+v"(d.e3)

// three: not zero, in every lane of the wavefront alike, when no lane has a
// fourth dimension: its turn is jumped over.
#define THEMIS_TRACE_TURNS(BODY)                                                       \
  "s_mov_b64 %[act], exec\n\t" BODY(0) BODY(1) BODY(2)                                 \
  "v_cmp_ne_u32_e32 vcc, 0, %[three]\n\t" "s_cbranch_vccnz .Lthree_dims_%=\n\t" BODY(3) ".Lthree_dims_%=:\n\t"
template <bool kFixAndQueue>
__device__ __forceinline__ double start_stage_trace(uint32_t k, uint32_t val, uint32_t nx,
                                                    double now, double x,
                                                    const double (&c)[kMaxDims],
                                                    const double (&a)[kMaxDims], TraceDims& d,
                                                    uint32_t& pos, uint32_t three) {
  uint64_t act;
  double t;
  if (kFixAndQueue) {
    asm volatile(THEMIS_TRACE_TURNS(THEMIS_TRACE_FULL)
        : [act] "=&s"(act), [t] "=&v"(t), [pos] "+v"(pos), THEMIS_F_OPERANDS, THEMIS_Z_OPERANDS,
          THEMIS_S_OPERANDS, THEMIS_N_OPERANDS, THEMIS_E_OPERANDS
        : [k] "v"(k), [val] "v"(val), [nx] "v"(nx), [now] "v"(now), [x] "v"(x), THEMIS_C_OPERANDS,
          THEMIS_A_OPERANDS, [three] "v"(three)
        : "vcc");
  } else {
    asm volatile(THEMIS_TRACE_TURNS(THEMIS_TRACE_PLAIN)
        : [act] "=&s"(act), [t] "=&v"(t), THEMIS_F_OPERANDS, THEMIS_Z_OPERANDS, THEMIS_S_OPERANDS,
          THEMIS_N_OPERANDS
        : [k] "v"(k), [val] "v"(val), [nx] "v"(nx), [now] "v"(now), [x] "v"(x), THEMIS_C_OPERANDS,
          [three] "v"(three)
        : "vcc");
  }
  return t;
}

// The stages that end now, as stages_ending(), with the fourth dimension's
// turn jumped over where no lane has one.
__device__ __forceinline__ uint32_t trace_stages_ending(double now, TraceDims& d, uint32_t& first,
                                                        uint32_t three) {
  uint64_t act;
  uint32_t done = 0u;
  first = ~0u;
  asm volatile("s_mov_b64 %[act], exec\n\t"
      THEMIS_ENDS_NOW(0, 1) THEMIS_ENDS_NOW(1, 2) THEMIS_ENDS_NOW(2, 4)
      "v_cmp_ne_u32_e32 vcc, 0, %[three]\n\t" "s_cbranch_vccnz .Lthree_dims_%=\n\t"
      THEMIS_ENDS_NOW(3, 8) ".Lthree_dims_%=:\n\t" THEMIS_PAD1
      : [act] "=&s"(act), [done] "+v"(done), [first] "+v"(first), THEMIS_F_OPERANDS
      : [now] "v"(now), [nan] "v"(nan64()), [s0] "v"(d.s0), [s1] "v"(d.s1), [s2] "v"(d.s2),
        [s3] "v"(d.s3), [three] "v"(three)
      : "vcc");
  return done;
}

// Bytes a stage moves when the NPU counts are not powers of two: the chunk's
// size divided step by step by the NPU counts of the dimensions before `pos` in
// its order, as the latency model of Sec. 4.5 walks it (a stand-alone
// All-Gather: grown step by step from the order's last dimension down to pos;
// its stored code is the reversed one).  The same operations in the same order
// as a scenario evaluated one division at a time, so the result is the same
// to the last bit.
__device__ __forceinline__ double trace_divided_bytes(const Scenario& s, double chunk, uint32_t code,
                                                      uint32_t pos, bool gather) {
  double x = chunk;
  if (gather) {
    for (uint32_t j = (uint32_t)s.D; j-- > pos;) {
      const uint32_t kj = (code >> (2u * j)) & 3u;
      x = x * (double)sel4((int)kj, s.P[0], s.P[1], s.P[2], s.P[3]);
    }
    return x;
  }
  for (uint32_t j = 0; j < pos; ++j) {
    const uint32_t kj = (code >> (2u * j)) & 3u;
    x = x / (double)sel4((int)kj, s.P[0], s.P[1], s.P[2], s.P[3]);
  }
  return x;
}

// divide: NPU counts that are not powers of two; CH[q] then holds the plain
// chunk bytes, every stage time comes from trace_divided_bytes() and the size
// ranks of Smallest-Chunk-First from trace_build_ranks_divided().
// kKnown: what the caller has seen to hold for every lane of the wavefront,
// so that the loop is compiled for it instead of testing per-lane flags
// (kTraceAnyLane: nothing; else All-Reduces (state0 = 0, rs_only = false) with
// scf and divide as the two bits say).
enum : int { kTraceAnyLane = -1, kTraceKnownScf = 1, kTraceKnownDivide = 2 };
template <bool kLdsBitmaps, bool kReleases, bool kFix, bool kQueue, int kKnown>
__device__ inline bool simulate_trace_fast(const Scenario& s, uint32_t Q, uint32_t epack,
                                           uint32_t state0_given, bool rs_only_given, bool scf_given,
                                           bool divide_given, bool has_release,
                                           const TraceRegion& rg, const LaneLds& lds,
                                           const SimOut& out, double& t_done,
                                           double (&busy)[kMaxDims],
                                           uint32_t (&executed_out)[kMaxDims]) {
  constexpr bool kAny = kKnown == kTraceAnyLane;
  const uint32_t state0 = kAny ? state0_given : 0u;
  const bool rs_only = kAny ? rs_only_given : false;
  const bool scf = kAny ? scf_given : (kKnown & kTraceKnownScf) != 0;
  const bool divide = kAny ? divide_given : (kKnown & kTraceKnownDivide) != 0;
  const uint32_t D = (uint32_t)s.D;
  const uint32_t C = s.C;
  const uint32_t G = Q * C;
  const uint32_t full = (1u << D) - 1u;
  const double kInf = inf64();
  // no lane of the wavefront has a fourth dimension: its turns are left out
  const uint32_t three = __builtin_amdgcn_ballot_w64(D > 3u) == 0ull ? 1u : 0u;
  // The list entry of (dimension, rank), clamped like TraceRegion::HT, from
  // local copies of the table's origin and size (read through the region, the
  // compiler fetches them from the kernel arguments again inside the loop, and
  // a lone wavefront waits for every such fetch).
  const uint32_t ranks = rg.t.R, last_rank = rg.t.R - 1u;
  uint32_t* const ht_origin = (uint32_t*)(rg.base + rg.t.off_ht);
  auto ht_index = [&](uint32_t k, uint32_t r) -> uint32_t {
    return __umul24(k & 3u, ranks) + min(r, last_rank);
  };
  auto HT = [&](uint32_t k, uint32_t r) -> uint32_t& { return ht_origin[ht_index(k, r)]; };

  if (scf) {
    if (divide) trace_build_ranks_divided(rg, s, Q, (state0 & 16u) != 0u, rs_only);
    else trace_build_ranks(rg, Q, D, epack, lds);
  }
  // non-empty bitmaps: one summary word per 32 leaves, one leaf bit per rank
  auto SUM = [&](uint32_t k, uint32_t sw) -> uint32_t& {
    return *(uint32_t*)lds.dword((k & 3u) * kTraceSumWords + (sw & (kTraceSumWords - 1u)));
  };
  auto BM = [&](uint32_t k, uint32_t leaf) -> uint32_t& {
    if (kLdsBitmaps)
      return *(uint32_t*)lds.dword(16u + (k & 3u) * kTraceLeafWords + (leaf & (kTraceLeafWords - 1u)));
    return rg.BM(k, leaf);
  };
  // the lowest non-empty rank of a dimension (kNoRank: nothing waits for it),
  // kept beside the bitmaps: a push lowers it, and when its list runs empty the
  // bitmaps say which rank is next
  constexpr uint32_t kNoRank = ~0u;
  auto LOW = [&](uint32_t k) -> uint32_t& {
    return *(uint32_t*)lds.dword((kLdsBitmaps ? 16u + 4u * kTraceLeafWords : 48u) + (k & 3u));
  };
  for (uint32_t k = 0; k < 4u; ++k) {
    for (uint32_t l = 0; l < kTraceLeafWords; ++l) BM(k, l) = 0u;
    for (uint32_t l = 0; l < kTraceSumWords; ++l) SUM(k, l) = 0u;
    LOW(k) = kNoRank;
  }

  // Per dimension (TraceDims): finish and busy time, the chunk it serves
  // (s: chunk << 2 | dimension) and what that chunk's completion will do,
  // worked out at dispatch so that the completion itself reads nothing but its
  // target list (n: the chunk's next word without its link in bits 0-15, the
  // next dimension in bits 16-18 (4 = finished) and the size rank there from
  // bit 19)
  static_assert(kQueue == kFix, "the two per-dimension extras come together");
  TraceDims d;
  d.f0 = d.f1 = d.f2 = d.f3 = nan64();
  d.z0 = d.z1 = d.z2 = d.z3 = 0.0;
  d.s0 = d.s1 = d.s2 = d.s3 = 0u;
  d.n0 = d.n1 = d.n2 = d.n3 = 0u;
  d.e0 = d.e1 = d.e2 = d.e3 = 0u;
  // tops: bit 4 * k + sw says that summary word sw of dimension k is not zero;
  // work: bit k says that dimension k has chunks waiting; idle: serves nothing
  uint32_t tops = 0u, work = 0u, idle = 15u;
  bool stalled = false;

  // g / C for g < 2^23 (chunk ids stay below 2^16) without a division or a
  // branch: the high half of g * ceil(2^32 / C), which fits 32 bits from C = 2
  // on; for C = 1 the multiplier is 0 and g itself is added
  const uint32_t c_inv = C == 1u ? 0u : (uint32_t)((0x100000000ull + C - 1u) / C);
  const uint32_t c_one = C == 1u ? ~0u : 0u;
  auto coll_of = [&](uint32_t g) -> uint32_t { return __umulhi(g, c_inv) + (g & c_one); };
  // rank of chunk g (word w) once it waits for dimension k with the given mask and phase
  auto rank_of = [&](uint32_t g, uint32_t w, uint32_t k, uint32_t mask, uint32_t phase) -> uint32_t {
    if (!scf) return 0u;
    if (divide) return (uint32_t)rg.SRD(coll_of(g), k, trace_state((w >> 8) & 0xffu, phase, D));
    return (uint32_t)rg.SR(coll_of(g), mask);
  };
  // Memory operations of one wavefront retire in order, so waiting for a load
  // also waits for every store issued before it: push and pop read first and
  // store last (word: the chunk's new word, stored here for that reason).
  // (a half of a chunk word, written in place: may alias the whole word)
  typedef uint16_t __attribute__((may_alias)) HalfOfWord;
  auto push = [&](uint32_t k, uint32_t r, uint32_t g, bool has_word, uint32_t word) {
    const uint32_t leaf = r >> 5, bit = 1u << (r & 31u);
    const uint32_t lw = BM(k, leaf);
    if (lw & bit) {
      const uint32_t ht = HT(k, r);
      const uint32_t tl = ht >> 16;
      if (has_word) rg.W(g) = word;
      ((HalfOfWord*)&rg.W(tl))[1] = (uint16_t)g;  // the old tail's next field
      HT(k, r) = (ht & 0xffffu) | (g << 16);
    } else {
      if (has_word) rg.W(g) = word;
      HT(k, r) = g | (g << 16);
      BM(k, leaf) = lw | bit;
      SUM(k, leaf >> 5) |= 1u << (leaf & 31u);
    }
    tops |= 1u << (4u * (k & 3u) + ((leaf >> 5) & 3u));
    work |= 1u << (k & 3u);
    LOW(k) = min(LOW(k), r);
  };
  // The stores of a push whose bitmap part the caller has done (had: the
  // rank's list had chunks already), given the list's entry as read before (ht, used when
  // had); returns the entry it stored
  auto push_link = [&](uint32_t k, uint32_t r, uint32_t g, uint32_t word, bool had, uint32_t ht) -> uint32_t {
    rg.W(g) = word;
    uint32_t entry = g | (g << 16);
    if (had) {
      ((HalfOfWord*)&rg.W(ht >> 16))[1] = (uint16_t)g;  // the old tail's next field
      entry = (ht & 0xffffu) | (g << 16);
    }
    HT(k, r) = entry;
    return entry;
  };
  // first chunk of the list of rank r, the lowest of dimension k, given the
  // list's entry ht; w receives its chunk word, size the resident bytes of a
  // chunk of that rank and row the size ranks of the chunk's collective.  Chunk
  // word and collective record are loaded together, and while they are on
  // their way the bitmaps are brought up to date: if the list runs empty its bit
  // goes and the dimension's next lowest rank is looked up (LDS round trips
  // that the wait on memory hides).
  // new_entry / at: the list's entry once its head is gone, for the caller to
  // store (at = all-ones: nothing to store, the list is empty now)
  auto pop = [&](uint32_t k, uint32_t r, uint32_t ht, uint32_t& w, double& size, uint4& row_lo,
                 uint4& row_hi, uint32_t& new_entry, uint32_t& at) -> uint32_t {
    const uint32_t h = ht & 0xffffu, tl = ht >> 16;
    w = rg.W(h);
    const uint32_t q = coll_of(h);
    // (the rank table is read whatever the policy: a load nobody uses costs
    // less here than a branch around it)
    const TraceRegion::RankRow* row = rg.SRrow(q);
    row_lo = row[0];
    if (!three) row_hi = row[1];  // (masks with the fourth dimension's bit)
    // the resident size from the chunk bytes of the collective, which sit in
    // the same 64 bytes as its rank row (the per-rank size table would be one
    // more line to fetch)
    size = rg.CH(q);
    if (h == tl) {
      const uint32_t leaf = r >> 5, sw = (leaf >> 5) & 3u;
      const uint32_t nlw = BM(k, leaf) & ~(1u << (r & 31u));
      BM(k, leaf) = nlw;
      uint32_t next = leaf * 32u + ((uint32_t)__builtin_ctz(nlw | 0x80000000u));
      if (!nlw) {
        const uint32_t rest = SUM(k, sw) & ~(1u << (leaf & 31u));
        SUM(k, sw) = rest;
        uint32_t sw2 = sw, sumw2 = rest;
        if (!rest) {
          tops &= ~(1u << (4u * k + sw));
          const uint32_t left = (tops >> (4u * k)) & 15u;
          if (left == 0u) work &= ~(1u << k);
          sw2 = (uint32_t)__builtin_ctz(left | 16u) & 3u;
          sumw2 = left ? SUM(k, sw2) : 0u;
        }
        next = kNoRank;
        if (sumw2) {
          const uint32_t leaf2 = sw2 * 32u + (uint32_t)__builtin_ctz(sumw2);
          next = leaf2 * 32u + ((uint32_t)__builtin_ctz(BM(k, leaf2) | 0x80000000u));
        }
      }
      LOW(k) = next;
    }
    if (!divide) size = scale_down(size, esum(epack, w & 15u));
    at = ~0u;
    new_entry = 0u;
    if (h != tl) {
      new_entry = (w >> 16) | (tl << 16);
      at = ht_index(k, r);
    }
    return h;
  };

  // a6: the chunks of a collective join the queues of their first dimensions
  // (initial mask) when it is released, collectives in (release time, index)
  // order, chunks in id order
  if (kReleases && has_release)
    trace_sort_collectives(rg, Q, 2u, [&](uint32_t q) { return (double)rg.REL(q); });
  uint32_t rel_next = 0;   // position in that order of the next collective to release
  double rel_time = 0.0;   // its release time, +inf when all are out
  double now = 0.0;
  auto release_due = [&]() {
    const uint32_t mask0 = state0 & 15u, phase0 = state0 >> 4;
    const uint32_t pos0 = 2u * ((uint32_t)__builtin_popcount(mask0) - phase0);
    while (rel_time <= now) {
      const uint32_t q = has_release ? (uint32_t)rg.SQbuf(2u, rel_next) : rel_next;
      for (uint32_t c = 0; c < C; ++c) {
        const uint32_t g = q * C + c;
        const uint32_t w0 = rg.W(g);
        const uint32_t k0 = (w0 >> (8u + pos0)) & 3u;
        push(k0, rank_of(g, w0, k0, mask0, phase0), g, false, 0u);
      }
      ++rel_next;
      rel_time = rel_next >= Q ? kInf : has_release ? (double)rg.REL(rg.SQbuf(2u, rel_next)) : 0.0;
    }
  };
  if (kReleases) {
    if (has_release) rel_time = Q ? (double)rg.REL(rg.SQbuf(2u, 0u)) : kInf;
    if (Q == 0u) rel_time = kInf;
    release_due();
  } else {
    const uint32_t mask0 = state0 & 15u, phase0 = state0 >> 4;
    const uint32_t pos0 = 2u * ((uint32_t)__builtin_popcount(mask0) - phase0);
    for (uint32_t g = 0; g < G; ++g) {
      const uint32_t w0 = rg.W(g);
      const uint32_t k0 = (w0 >> (8u + pos0)) & 3u;
      push(k0, rank_of(g, w0, k0, mask0, phase0), g, false, 0u);
    }
  }

  // One pass has three parts, and a wavefront waits for memory once in the
  // first and once in the last, whatever its lanes are doing:
  //   start   the stage picked by the previous pass starts (chunk word and
  //           collective record are read here, the list entry is at hand);
  //   advance once no idle dimension has chunks waiting, the clock moves to
  //           the earliest completion (or release) and the stages that end
  //           there are delivered, lowest chunk id first;
  //   pick    the next stage to start is chosen, and its list entry is read
  //           together with the entry of the list the (last) completed chunk
  //           joins.
  // A lane with two stages to start at one instant takes two passes, the other
  // lanes of the wavefront go on meanwhile.
  const uint64_t max_steps = (uint64_t)4u * D * G + Q + 16u;
  bool picked = false;
  uint32_t pk_k = 0u, pk_r = 0u, pk_ht = 0u;
  for (uint64_t step = 0; step <= max_steps; ++step) {
    // a7: an idle dimension with waiting chunks starts its first one
    if (picked) {
      const uint32_t k = pk_k;
      uint32_t w;
      double size;
      uint4 row_lo = {0u, 0u, 0u, 0u}, row_hi = {0u, 0u, 0u, 0u};
      uint32_t new_entry, entry_at;
      const uint32_t h = pop(k, pk_r, pk_ht, w, size, row_lo, row_hi, new_entry, entry_at);
      const uint32_t mask = w & 15u, phase = (w >> 4) & 1u;
      const uint32_t ek = (epack >> (8u * k)) & 0xffu;
      // the chunk's state after this stage: a Reduce-Scatter sets the
      // dimension's bit, an All-Gather clears it
      const uint32_t code = (w >> 8) & 0xffu;
      const uint32_t mask2 = mask ^ (1u << k);
      const bool finished = (phase != 0u && mask2 == 0u) || (rs_only && mask2 == full);
      const uint32_t phase2 = phase | ((mask2 == full) ? 1u : 0u);  // last RS: AG starts on the same dim
      // next stage: RS -> order[#reduced], AG -> order[#reduced - 1]
      const uint32_t p = (uint32_t)__builtin_popcount(mask2) - phase2;
      const uint32_t kn = finished ? 4u : (code >> ((2u * p) & 31u)) & 3u;
      const bool upper = (mask2 & 8u) != 0u;
      const uint32_t pair = sel4((int)(mask2 >> 1), upper ? row_hi.x : row_lo.x, upper ? row_hi.y : row_lo.y,
                                 upper ? row_hi.z : row_lo.z, upper ? row_hi.w : row_lo.w);
      uint32_t rk = scf ? (pair >> (16u * (mask2 & 1u))) & 0xffffu : 0u;
      // division mode: the rank row is per (dimension, phase, order), known only now
      if (divide && scf && !finished) rk = rg.SRD(coll_of(h), kn, trace_state(code, phase2, D));
      const uint32_t sv = (h << 2) | k;
      const uint32_t nx = mask2 | (phase2 << 4) | (code << 8) | (kn << 16) | (rk << 19);
      uint32_t pos = 0u;
      // bytes moved on k: the resident size before the chunk's Reduce-Scatter
      // on k, which an All-Gather on k finds 2^ek times smaller
      double bytes = scale_up(size, phase ? ek : 0u);
      if (divide) {
        // k's place in the chunk's order: the dimensions reduced before it
        const uint32_t place = ((uint32_t)__builtin_popcount(mask) - phase) & 3u;
        bytes = trace_divided_bytes(s, size, code, place, (state0 & 16u) != 0u);
      }
      const double t = start_stage_trace<kQueue>(k, sv, nx, now, bytes, s.coef, s.fix, d, pos, three);
      const double fin = now + t;
      // a stage that does not move the clock, or overflows it: generic path decides
      stalled |= !(fin > now && fin < kInf);
      idle &= ~(1u << k);
      if (kQueue && out.queue_order && pos < 2u * out.slots) put_entry(out, (int)k, pos, (h << 1) | phase);
      if (entry_at != ~0u) ht_origin[entry_at] = new_entry;
    }
    if (stalled) break;

    // a8: advance to the earliest completion, or to the next release if that
    // comes first
    bool moves = false, had = false;
    uint32_t kn = 0u, r = 0u, g = 0u, word = 0u;
    // the stages that end at the new instant, and the smallest
    // chunk << 2 | dimension among them
    uint32_t done = 0u, key = ~0u;
    if ((idle & work) == 0u) {
      const double next = min_f64(min_f64(d.f0, d.f1), min_f64(d.f2, d.f3));  // NaN: nothing runs
      if (!kReleases) {
        if (!(next < kInf)) break;
        now = next;
        done = trace_stages_ending(now, d, key, three);
      } else if (!(next < rel_time)) {
        if (!(rel_time < kInf)) break;  // nothing running, nothing left to release
        // chunks arriving at one instant from a release and from a completion
        // would have to be merged by id: the generic path does that
        if (rel_time == next) { stalled = true; break; }
        now = rel_time;
        release_due();
      } else {
        now = next;
        done = trace_stages_ending(now, d, key, three);
      }
      idle |= done;
    }
    // more than one stage ends at this very instant (rare): all but the last
    // are delivered here, lowest chunk id first, each with a wait of its own
    while ((done & (done - 1u)) != 0u) {
      const uint32_t k = key & 3u;
      const uint32_t nx = sel4((int)k, d.n0, d.n1, d.n2, d.n3);
      if (((nx >> 16) & 7u) < 4u)
        push((nx >> 16) & 7u, nx >> 19, key >> 2, true, (nx & 0xffffu) | (kNoChunk << 16));
      done &= ~(1u << k);
      key = min(min((done & 1u) ? d.s0 : ~0u, (done & 2u) ? d.s1 : ~0u),
                min((done & 4u) ? d.s2 : ~0u, (done & 8u) ? d.s3 : ~0u));
    }
    if (done != 0u) {
      const uint32_t k = key & 3u;
      const uint32_t nx = sel4((int)k, d.n0, d.n1, d.n2, d.n3);
      kn = (nx >> 16) & 7u;
      r = nx >> 19;
      g = key >> 2;
      word = (nx & 0xffffu) | (kNoChunk << 16);
      moves = kn < 4u;
    }
    // The bitmap part of the push and the pick, with the LDS reads issued
    // together: the leaf word and the summary word of the push's rank, and the
    // lowest rank of the dimension that starts a stage next.
    {
      const uint32_t leaf_r = r >> 5, bit_r = 1u << (r & 31u), sw_r = (leaf_r >> 5) & 3u;
      const uint32_t in_sum_r = 1u << (leaf_r & 31u);
      if (moves) {
        tops |= 1u << (4u * kn + sw_r);
        work |= 1u << kn;
      }
      const uint32_t need = idle & work;
      picked = need != 0u;
      pk_k = picked ? (uint32_t)__builtin_ctz(need) : 0u;
      const uint32_t lw_r = BM(kn, leaf_r);
      const uint32_t sum_r = SUM(kn, sw_r);
      pk_r = LOW(pk_k);
      had = moves && (lw_r & bit_r) != 0u;
      if (moves) {
        if (!had) {
          BM(kn, leaf_r) = lw_r | bit_r;
          SUM(kn, sw_r) = sum_r | in_sum_r;
        }
        // (the dimension's lowest rank was read before it is lowered here)
        atomicMin(&LOW(kn), r);
        if (kn == pk_k) pk_r = min(pk_r, r);
      }
    }
    const uint32_t ht_to = HT(kn, r);
    pk_ht = HT(pk_k, pk_r);
    if (moves) {
      const uint32_t entry = push_link(kn, r, g, word, had, ht_to);
      if (pk_k == kn && pk_r == r) pk_ht = entry;  // the very list just appended to
    }
  }

  t_done = now;
#pragma unroll
  for (uint32_t kk = 0; kk < 4u; ++kk) { busy[kk] = 0.0; executed_out[kk] = 0u; }
  busy[0] = d.z0; busy[1] = d.z1; busy[2] = d.z2; busy[3] = d.z3;
  executed_out[0] = d.e0; executed_out[1] = d.e1; executed_out[2] = d.e2; executed_out[3] = d.e3;
  return !stalled;
}

}  // namespace themis
