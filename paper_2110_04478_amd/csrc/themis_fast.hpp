// Fast path of the planner and of the queue simulation for scenarios whose
// NPU counts are all powers of two (every topology of the paper's Table 2):
// one lane per evaluation, scalar state in VGPRs, per-chunk state and the
// per-dimension queues in LDS.
//
// Why powers of two matter: dividing the resident size by P_k = 2^e_k is then
// an exact exponent decrement, so the size before any stage is
// chunk * 2^-E(mask), E(mask) = sum of e_k over the dimensions the chunk is
// currently reduced on.  That makes (a) every stage time a single multiply,
// bit-identical to the step-by-step divisions of the reference arithmetic,
// and (b) Smallest-Chunk-First an integer comparison of E(mask).
//
// Queue structure (paper Sec. 4.3): each dimension owns up to 16 FIFO lists,
// one per distinct resident size ("class" = rank of E(mask) among the 16
// masks; FIFO policy uses class 0 only).  Inside a list chunks are in
// (arrival time, chunk id) order because lists are appended in time order and
// simultaneous completions are appended in chunk-id order.  A 64-bit bitmap
// (16 bits per dimension) marks the non-empty lists, so "smallest chunk
// first" is a find-highest-bit and a list pop: O(1) per chunk-stage event
// instead of a scan over all chunks.
//
// LDS layout: every lane owns kLaneWords dwords, stored transposed
// (dword d of lane L at word d*64 + L) so that the 64 lanes of a wavefront
// always hit 64 different banks, whatever per-lane index they use.
#pragma once

#include "themis_device.hpp"

namespace themis {

constexpr int kFastCap = 64;           // chunks per evaluation the LDS layout holds
constexpr int kOffW = 0;               // u16 W[64] : code | mask<<8 | phase<<12
constexpr int kOffNext = 128;          // u8  NX[64]: next chunk in the same list
constexpr int kOffHead = 192;          // u8  H[4*16]: list heads
constexpr int kOffTail = 256;          // u8  T[4*16]: list tails
constexpr int kLaneBytes = 320;
constexpr int kLaneWords = kLaneBytes / 4;
constexpr int kFastLdsBytes = kLaneWords * 64 * 4;  // per wavefront

struct LaneLds {
  uint8_t* base;  // LDS block of the wavefront + 4*lane
  __device__ __forceinline__ uint32_t at(uint32_t byte) const {
    return ((byte >> 2) << 8) | (byte & 3u);
  }
  __device__ __forceinline__ uint32_t r8(uint32_t byte) const { return base[at(byte)]; }
  __device__ __forceinline__ void w8(uint32_t byte, uint32_t v) const { base[at(byte)] = (uint8_t)v; }
  __device__ __forceinline__ uint32_t r16(uint32_t byte) const {
    return *(const uint16_t*)(base + at(byte));
  }
  __device__ __forceinline__ void w16(uint32_t byte, uint32_t v) const {
    *(uint16_t*)(base + at(byte)) = (uint16_t)v;
  }
};

// Per-evaluation constants of the fast path.
struct FastScenario {
  uint32_t epack;   // e_k = log2 P_k in byte k (0 for unused dimensions)
  uint32_t etot;    // sum of e_k
  double chunk;     // bytes per chunk (normal binary64, exponent > etot)
};

__device__ __forceinline__ bool is_pow2(uint32_t p) { return (p & (p - 1u)) == 0u; }

// Can this scenario take the fast path?  Fills fs when it can.
__device__ __forceinline__ bool fast_eligible(const Scenario& s, double chunk, FastScenario& fs) {
  bool ok = s.valid && s.C <= (uint32_t)kFastCap;
  uint32_t ep = 0, et = 0;
#pragma unroll
  for (int k = 0; k < kMaxDims; ++k) {
    if (k < s.D) {
      ok = ok && is_pow2(s.P[k]);
      uint32_t e = 31u - (uint32_t)__clz((int)s.P[k]);
      ep |= e << (8 * k);
      et += e;
    }
  }
  // every halving must stay a normal number: biased exponent - etot >= 1
  uint32_t ex = (uint32_t)((__double_as_longlong(chunk) >> 52) & 0x7ff);
  ok = ok && ex < 0x7ffu && ex > et;
  fs.epack = ep;
  fs.etot = et;
  fs.chunk = chunk;
  return ok;
}

// x * 2^-e for a normal x whose exponent stays in range (checked above).
__device__ __forceinline__ double scale_down(double x, uint32_t e) {
  int hi = __double2hiint(x) - (int)(e << 20);
  return __hiloint2double(hi, __double2loint(x));
}

// Sum of e_k over the dimensions in mask.
__device__ __forceinline__ uint32_t esum(uint32_t epack, uint32_t mask) {
  uint32_t spread = (mask * 0x00204081u) & 0x01010101u;  // bit k -> byte k
  uint32_t sel = (spread * 0xffu) & epack;
  return __builtin_amdgcn_sad_u8(sel, 0u, 0u);            // add the four bytes
}

// ---------------------------------------------------------------------------
// Planner (Alg. 1) with static register indexing.  emit(c, code) receives
// every chunk's order code; load[] holds the Dim Load Tracker on return.
// ---------------------------------------------------------------------------
template <typename Emit>
__device__ __forceinline__ void plan_fast(const Scenario& s, const FastScenario& fs, bool themis,
                                          bool rel, double thr, double (&load)[kMaxDims],
                                          Emit emit) {
  const int D = s.D;
  uint32_t e[kMaxDims];
  double coef[kMaxDims];
#pragma unroll
  for (int k = 0; k < kMaxDims; ++k) {
    e[k] = (fs.epack >> (8 * k)) & 0xffu;
    coef[k] = (k < D) ? s.coef[k] : 0.0;   // unused dimensions: zero time, load stays +inf
    load[k] = (k < D) ? 0.0 : inf64();
  }
  const uint32_t field_mask = (1u << (2 * D)) - 1u;
  for (uint32_t c = 0; c < s.C; ++c) {
    // least / most loaded dimension, ties to the lower index
    double lo = load[0], hi = load[0], cmin = coef[0];
#pragma unroll
    for (int k = 1; k < kMaxDims; ++k) {
      bool used = k < D;
      bool less = used && load[k] < lo;
      lo = less ? load[k] : lo;
      cmin = less ? coef[k] : cmin;
      hi = (used && load[k] > hi) ? load[k] : hi;
    }
    double t = rel ? thr * (fs.chunk * cmin) : thr;
    bool sort = themis && !((hi - lo) < t);
    // after[a][b] (a < b): does a come after b in the chosen order?
    // stable ascending sort: only when a's load is strictly larger.
    bool after01 = sort && load[0] > load[1], after02 = sort && load[0] > load[2];
    bool after03 = sort && load[0] > load[3], after12 = sort && load[1] > load[2];
    bool after13 = sort && load[1] > load[3], after23 = sort && load[2] > load[3];
    // before[j][k]: j precedes k
    const bool b10 = after01, b20 = after02, b30 = after03;
    const bool b01 = !after01, b21 = after12, b31 = after13;
    const bool b02 = !after02, b12 = !after12, b32 = after23;
    const bool b03 = !after03, b13 = !after13, b23 = !after23;
    uint32_t r0 = (uint32_t)b10 + b20 + b30, r1 = (uint32_t)b01 + b21 + b31;
    uint32_t r2 = (uint32_t)b02 + b12 + b32, r3 = (uint32_t)b03 + b13 + b23;
    uint32_t code = ((1u << (2 * r1)) | (2u << (2 * r2)) | (3u << (2 * r3))) & field_mask;
    (void)r0;
    // resident size before the Reduce-Scatter on k: chunk / prod of P_j, j before k
    uint32_t E0 = (b10 ? e[1] : 0u) + (b20 ? e[2] : 0u) + (b30 ? e[3] : 0u);
    uint32_t E1 = (b01 ? e[0] : 0u) + (b21 ? e[2] : 0u) + (b31 ? e[3] : 0u);
    uint32_t E2 = (b02 ? e[0] : 0u) + (b12 ? e[1] : 0u) + (b32 ? e[3] : 0u);
    uint32_t E3 = (b03 ? e[0] : 0u) + (b13 ? e[1] : 0u) + (b23 ? e[2] : 0u);
    double t0 = scale_down(fs.chunk, E0) * coef[0];
    double t1 = scale_down(fs.chunk, E1) * coef[1];
    double t2 = scale_down(fs.chunk, E2) * coef[2];
    double t3 = scale_down(fs.chunk, E3) * coef[3];
    load[0] = load[0] + (t0 + t0);
    load[1] = load[1] + (t1 + t1);
    load[2] = load[2] + (t2 + t2);
    load[3] = load[3] + (t3 + t3);
    emit(c, code);
  }
}

// ---------------------------------------------------------------------------
// Queue simulation.
// ---------------------------------------------------------------------------
struct FastOut {
  uint8_t* queue_order;  // this evaluation's [4][2*slots] bytes, or null
  uint32_t slots;
  bool want_busy;
};

struct FastResult {
  double t_done;
  double busy[kMaxDims];
  uint32_t executed;  // per-dimension operation counts, one byte each
  bool ok;            // false: leave the answer to the generic path
};

// Class (rank of the resident size) of every mask, 4 bits each: the number of
// masks with a strictly smaller E, i.e. a strictly larger resident size.
__device__ __forceinline__ uint64_t build_rank_table(uint32_t epack, bool scf) {
  if (!scf) return 0ull;
  uint32_t E[16];
#pragma unroll
  for (uint32_t m = 0; m < 16; ++m) E[m] = esum(epack, m);
  uint64_t tab = 0;
#pragma unroll
  for (uint32_t m = 0; m < 16; ++m) {
    uint32_t r = 0;
#pragma unroll
    for (uint32_t o = 0; o < 16; ++o) r += (E[o] < E[m]) ? 1u : 0u;
    tab |= (uint64_t)r << (4 * m);
  }
  return tab;
}

// Chunk words W[c] must already be in LDS: code | 0<<8 (mask) | 0<<12 (phase).
template <bool kQueueOrder>
__device__ __forceinline__ FastResult simulate_fast(const Scenario& s, const FastScenario& fs,
                                                    bool scf, const LaneLds& lds,
                                                    const FastOut& out) {
  const int D = s.D;
  const uint32_t C = s.C;
  const uint32_t full = (1u << D) - 1u;
  const uint64_t ranktab = build_rank_table(fs.epack, scf);
  const double kInf = inf64();

  double f0 = kInf, f1 = kInf, f2 = kInf, f3 = kInf;  // finish time, +inf = idle
  double z0 = 0.0, z1 = 0.0, z2 = 0.0, z3 = 0.0;      // busy time
  uint32_t serving = 0;   // chunk id per dimension, one byte each
  uint32_t executed = 0;  // operations started per dimension, one byte each
  uint64_t nonempty = 0;  // bit 16*k + class
  FastResult res;
  res.ok = true;

  auto push = [&](uint32_t k, uint32_t cls, uint32_t c) {
    uint32_t q = 16u * k + cls;
    uint64_t bit = 1ull << q;
    if (nonempty & bit) {
      uint32_t t = lds.r8(kOffTail + q);
      lds.w8(kOffNext + t, c);
    } else {
      lds.w8(kOffHead + q, c);
      nonempty |= bit;
    }
    lds.w8(kOffTail + q, c);
  };

  // a6: every chunk waits at the dimension of its first stage, resident size
  // = chunk (mask 0, the lowest class), in chunk-id order
  for (uint32_t c = 0; c < C; ++c) push(lds.r16(kOffW + 2u * c) & 3u, 0u, c);

  double now = 0.0;
  const uint32_t max_steps = 2u * (uint32_t)D * C + 8u;
  for (uint32_t step = 0; step <= max_steps; ++step) {
    // a7: every idle dimension with waiting chunks starts its first one
    for (;;) {
      uint32_t need = 0;
      need |= (f0 == kInf && (nonempty & 0xffffull)) ? 1u : 0u;
      need |= (f1 == kInf && (nonempty & 0xffff0000ull)) ? 2u : 0u;
      need |= (f2 == kInf && (nonempty & 0xffff00000000ull)) ? 4u : 0u;
      need |= (f3 == kInf && (nonempty & 0xffff000000000000ull)) ? 8u : 0u;
      if (!need) break;
      uint32_t k = (uint32_t)__builtin_ctz(need);
      uint32_t field = (uint32_t)(nonempty >> (16u * k)) & 0xffffu;
      uint32_t cls = 31u - (uint32_t)__clz((int)field);  // smallest resident size
      uint32_t q = 16u * k + cls;
      uint32_t h = lds.r8(kOffHead + q);
      uint32_t tl = lds.r8(kOffTail + q);
      uint32_t w = lds.r16(kOffW + 2u * h);
      if (h == tl) nonempty &= ~(1ull << q);
      else lds.w8(kOffHead + q, lds.r8(kOffNext + h));
      uint32_t mask = (w >> 8) & 15u;
      uint32_t phase = (w >> 12) & 1u;
      // bytes moved on k = resident size before the chunk's Reduce-Scatter on
      // k; the All-Gather reuses it (mask still contains k then)
      uint32_t ek = (fs.epack >> (8u * k)) & 0xffu;
      uint32_t E = esum(fs.epack, mask) - (phase ? ek : 0u);
      double x = scale_down(fs.chunk, E);
      double t = x * sel4((int)k, s.coef[0], s.coef[1], s.coef[2], s.coef[3]);
      double f = now + t;
      if (!(f > now)) { res.ok = false; break; }  // time did not advance: generic path decides
      f0 = (k == 0u) ? f : f0; f1 = (k == 1u) ? f : f1;
      f2 = (k == 2u) ? f : f2; f3 = (k == 3u) ? f : f3;
      if (out.want_busy) {
        z0 = (k == 0u) ? z0 + t : z0; z1 = (k == 1u) ? z1 + t : z1;
        z2 = (k == 2u) ? z2 + t : z2; z3 = (k == 3u) ? z3 + t : z3;
      }
      uint32_t sh = 8u * k;
      serving = (serving & ~(0xffu << sh)) | (h << sh);
      if (kQueueOrder) {
        uint32_t pos = (executed >> sh) & 0xffu;
        if (pos < 2u * out.slots)  // always true for a consistent plan; keeps the store in bounds
          out.queue_order[(size_t)k * 2u * out.slots + pos] = (uint8_t)((h << 1) | phase);
      }
      executed += 1u << sh;
    }
    if (!res.ok) break;

    // a8: advance to the earliest completion
    double next = fmin(fmin(f0, f1), fmin(f2, f3));
    if (!(next < kInf)) break;  // nothing running: every chunk is done
    now = next;
    uint32_t done = (f0 == now ? 1u : 0u) | (f1 == now ? 2u : 0u) | (f2 == now ? 4u : 0u) |
                    (f3 == now ? 8u : 0u);
    f0 = (f0 == now) ? kInf : f0; f1 = (f1 == now) ? kInf : f1;
    f2 = (f2 == now) ? kInf : f2; f3 = (f3 == now) ? kInf : f3;
    // deliver all completions of this instant, lowest chunk id first, so that
    // equal arrival times are appended in chunk-id order
    do {
      uint32_t k = (uint32_t)__builtin_ctz(done);
      if (done & (done - 1u)) {
        uint32_t best = 0xffffu;
#pragma unroll
        for (uint32_t kk = 0; kk < (uint32_t)kMaxDims; ++kk) {
          uint32_t id = (serving >> (8u * kk)) & 0xffu;
          if ((done >> kk & 1u) && id < best) { best = id; k = kk; }
        }
      }
      done &= ~(1u << k);
      uint32_t c = (serving >> (8u * k)) & 0xffu;
      uint32_t w = lds.r16(kOffW + 2u * c);
      uint32_t code = w & 0xffu, mask = (w >> 8) & 15u, phase = (w >> 12) & 1u;
      uint32_t kn;
      bool finished = false;
      if (!phase) {
        mask |= 1u << k;
        if (mask == full) { phase = 1u; kn = k; }              // last RS: AG starts on the same dim
        else kn = (code >> (2u * __builtin_popcount(mask))) & 3u;
      } else {
        mask &= ~(1u << k);
        finished = mask == 0u;
        kn = finished ? 0u : (code >> (2u * (__builtin_popcount(mask) - 1u))) & 3u;
      }
      if (!finished) {
        lds.w16(kOffW + 2u * c, code | (mask << 8) | (phase << 12));
        uint32_t cls = (uint32_t)(ranktab >> (4u * mask)) & 15u;
        push(kn, cls, c);
      }
    } while (done);
  }

  res.t_done = now;
  res.busy[0] = z0; res.busy[1] = z1; res.busy[2] = z2; res.busy[3] = z3;
  res.executed = executed;
  return res;
}

}  // namespace themis
