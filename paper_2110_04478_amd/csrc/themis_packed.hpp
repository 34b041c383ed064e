// Event loop of the power-of-two fast path on 16-bit chunk records, for
// evaluations with hundreds of chunks: the LDS block of a lane is what limits
// how many wavefronts a CU holds, and with one or two of them per CU the loop
// is bound by latency, not by instruction issue, so a record half as large
// (twice the wavefronts) is worth some more arithmetic per event.
//
// A chunk's record holds only what cannot be derived:
//   bits 0-8    next chunk in its list (its own id: it is the last one)
//   bit  9      phase (0 Reduce-Scatter, 1 All-Gather)
//   bits 10-14  order: o0 | o1 << 2 | (o2 > o3) << 4, the order code with the
//               unused fields filled by their own index (a permutation of 0..3
//               is fixed by its first two entries and the order of the rest)
// The reduced-dims mask of the 32-bit layouts is implied: a chunk waiting for
// dimension k is reduced on the dimensions before k in its order (and on k, in
// the All-Gather phase).  The queue structure is the one of simulate_fast
// (paper Sec. 4.3: per dimension one FIFO list per resident-size class); a
// list's tail entry carries the upper bits of the tail chunk's record, so that
// appending behind it is one 16-bit store and not a read-modify-write.
//
// Lane block: u16 record[kChunks], u16 head[64], u16 tail[64], transposed like
// every other layout (dword d of lane L at word d*64 + L).
#pragma once

#include "themis_fast.hpp"

namespace themis {

template <uint32_t kChunks>
struct LayoutPacked {
  static constexpr bool kPacked = true;
  static constexpr uint32_t kCap = kChunks;
  static_assert(kChunks <= 512 && kChunks % 2 == 0, "9-bit chunk ids, two records per dword");
  static constexpr uint32_t kHeadBase = kChunks / 2;
  static constexpr uint32_t kTailBase = kHeadBase + 32;
  static constexpr uint32_t kLaneWords = kTailBase + 32;
  static constexpr uint32_t kWavesPerSimd = (160u * 1024u / (kLaneWords * 256u) + 3u) / 4u;
  static constexpr uint32_t kIdMask = 0x1ffu;
  using Ids = Pack4<uint64_t, 16>;
  using Classes = Classes16;
  static __device__ __forceinline__ uint16_t* half(const LaneLds& l, uint32_t base, uint32_t i) {
    return (uint16_t*)(l.base + ((base + (i >> 1)) << 8) + 2u * (i & 1u));
  }
  static __device__ __forceinline__ uint16_t* record(const LaneLds& l, uint32_t c) { return half(l, 0u, c); }
  static __device__ __forceinline__ uint16_t* head(const LaneLds& l, uint32_t q) { return half(l, kHeadBase, q); }
  static __device__ __forceinline__ uint16_t* tail(const LaneLds& l, uint32_t q) { return half(l, kTailBase, q); }
  // order field of an order code whose unused fields are zero (D dimensions)
  static __device__ __forceinline__ uint32_t order_field(uint32_t code, uint32_t D) {
    const uint32_t c8 = code | (0xe4u & ~((1u << (2u * D)) - 1u));
    return (c8 & 15u) | ((((c8 >> 4) & 3u) > (c8 >> 6)) ? 16u : 0u);
  }
  // state0: initial mask | phase << 4 as in FastScenario (the mask is implied)
  static __device__ __forceinline__ void init_chunk(const LaneLds& l, uint32_t c, uint32_t code,
                                                    uint32_t state0, uint32_t D) {
    *record(l, c) = (uint16_t)(c | ((state0 >> 4) << 9) | (order_field(code, D) << 10));
  }
};

// The four dimensions of an order field, first to last.
struct PackedOrder {
  uint32_t o0, o1, o2, o3, first_two;  // first_two: bits of o0 and o1
  __device__ __forceinline__ explicit PackedOrder(uint32_t field) {
    o0 = field & 3u;
    o1 = (field >> 2) & 3u;
    first_two = (1u << o0) | (1u << o1);
    const uint32_t rest = 15u ^ first_two;  // two bits
    const uint32_t lo = (uint32_t)__builtin_ctz(rest), hi = 31u - (uint32_t)__builtin_clz(rest);
    const bool swap = (field & 16u) != 0u;
    o2 = swap ? hi : lo;
    o3 = swap ? lo : hi;
  }
  __device__ __forceinline__ uint32_t at(uint32_t pos) const { return sel4((int)pos, o0, o1, o2, o3); }
};

// Same contract as simulate_fast (records initialised with L::init_chunk(),
// result.ok false leaves the evaluation to the generic path); power-of-two
// model only.
template <typename L, int kQueueOrder, bool kBusy, bool kFix>
__device__ __forceinline__ FastResult simulate_packed(const Scenario& s, const Pow2Model& model,
                                                      const LaneLds& lds, const FastOut& out) {
  static_assert(kQueueOrder == kNoQueueOrder || kQueueOrder == kBytes || kQueueOrder == kShorts,
                "entries are stored one by one");
  const uint32_t D = (uint32_t)s.D;
  const uint32_t C = s.C;
  const uint32_t full = (1u << D) - 1u;
  const double kInf = inf64();
  const uint32_t epack = model.fs.epack;
  const uint64_t ranktab = model.ranktab;
  const bool rs_only = model.rs_only();

  // per dimension (DimState::s0..s3), the stage it serves and what its
  // completion does:
  //   bits 0-5 list to join, 6-11 upper record bits then, 12 chunk is done,
  //   13-14 the dimension, 15-23 the chunk
  DimState d;
  d.f0 = d.f1 = d.f2 = d.f3 = nan64();
  d.z0 = d.z1 = d.z2 = d.z3 = 0.0;
  d.s0 = d.s1 = d.s2 = d.s3 = 0u;
  typename L::Ids executed;  // operations started per dimension (kept when queue orders are written)
  uint32_t started = 0;      // operations started in all
  Classes16 classes(lds);
  uint32_t work = 0;      // bit k: some list of dimension k holds chunks
  uint32_t idle = full;   // bit k: dimension k serves nothing
  const uint32_t row_len = 2u * out.slots;

  // chunk c (upper record bits `up`: phase | order << 1) becomes the last of list q
  auto push = [&](uint32_t q, uint32_t c, uint32_t up) {
    const bool had = classes.mark(q);
    uint16_t* tp = L::tail(lds, q);
    const uint32_t t = *tp;
    const uint32_t rec = c | (up << 9);
    *L::record(lds, c) = (uint16_t)rec;  // own id: end of list
    // an empty list takes c as its head, otherwise the old tail's record points to c
    uint16_t* dst = had ? L::record(lds, t & L::kIdMask) : L::head(lds, q);
    *dst = (uint16_t)(had ? ((t & ~L::kIdMask) | c) : c);
    *tp = (uint16_t)rec;
    work |= 1u << (q >> 4);
  };

  // a6: every chunk waits at the dimension of its first stage, in chunk-id order
  {
    const uint32_t mask0 = model.state0() & 15u, phase0 = (model.state0() >> 4) & 1u;
    const uint32_t pos0 = (uint32_t)__builtin_popcount(mask0) - phase0;
    const uint32_t cls0 = (uint32_t)(ranktab >> (4u * mask0)) & 15u;
    for (uint32_t c = 0; c < C; ++c) {
      const uint32_t up = (uint32_t)*L::record(lds, c) >> 9;
      push(16u * PackedOrder(up >> 1).at(pos0) + cls0, c, up);
    }
  }

  double now = 0.0;
  const uint32_t max_steps = 4u * D * C + 16u;
  for (uint32_t step = 0; step <= max_steps; ++step) {
    // a7: an idle dimension with waiting chunks starts its first one (one stage
    // per pass, as in simulate_fast: here it pays for every output set)
    if (const uint32_t need = idle & work) {
      const uint32_t k = (uint32_t)__builtin_ctz(need);
      uint32_t field;
      const uint32_t cls = classes.lowest(k, field);  // smallest resident size
      const uint32_t q = 16u * k + cls;
      uint16_t* hp = L::head(lds, q);
      const uint32_t h = *hp;
      const uint32_t w = *L::record(lds, h);
      const uint32_t nx = w & L::kIdMask;
      *hp = (uint16_t)nx;  // harmless when the list is now empty
      const bool emptied = nx == h;
      const bool no_work = classes.popped(k, cls, q, field, emptied);
      work &= ~((no_work ? 1u : 0u) << k);
      const uint32_t kbit = 1u << k;
      idle &= ~kbit;

      const uint32_t phase = (w >> 9) & 1u;
      const bool ag = phase != 0u;
      const PackedOrder ord(w >> 10);
      // where k stands in the chunk's order, and the dimensions before it
      const bool p0 = k == ord.o0, p1 = k == ord.o1, p2 = k == ord.o2;
      const uint32_t before = p0 ? 0u : p1 ? (1u << ord.o0) : p2 ? ord.first_two
                                                                 : (ord.first_two | (1u << ord.o2));
      // what the completion of this stage will do: a Reduce-Scatter adds k to
      // the reduced dimensions and goes on to the next one of the order, the
      // last one turns into the All-Gather on the same dimension; an
      // All-Gather takes k off and goes back to the previous one
      {
        const uint32_t with_k = before | kbit;
        const bool last_rs = !ag && with_k == full;
        const bool finished = ag ? p0 : (last_rs && rs_only);
        const uint32_t mask = ag ? before : with_k;
        const uint32_t prev = p1 ? ord.o0 : p2 ? ord.o1 : ord.o2;
        const uint32_t succ = p0 ? ord.o1 : p1 ? ord.o2 : ord.o3;
        const uint32_t kn = last_rs ? k : ag ? prev : succ;
        const uint32_t up = (w >> 9) | (last_rs ? 1u : 0u);
        const uint32_t qn = 16u * kn + ((uint32_t)(ranktab >> (4u * mask)) & 15u);
        const uint32_t v = qn | (up << 6) | (finished ? 0x1000u : 0u) | (k << 13) | (h << 15);
        // bytes moved on k = resident size before the chunk's Reduce-Scatter on
        // k; the All-Gather on k reuses that time
        start_stage_scaled<kBusy, kFix>(k, v, now, scale_down(model.fs.base, esum(epack, before)),
                                        s.coef, s.fix, d);
      }
      if (kQueueOrder != kNoQueueOrder) {
        const uint32_t at = executed.get(k);
        const uint32_t entry = (h << 1) | phase;
        // at < row_len always holds for a consistent plan; it keeps the store in bounds
        if (kQueueOrder == kBytes) {
          if (at < row_len) out.queue_order[k * row_len + at] = (uint8_t)entry;
        } else {
          if (at < row_len) ((uint16_t*)out.queue_order)[k * row_len + at] = (uint16_t)entry;
        }
      }
      if (kQueueOrder != kNoQueueOrder) executed.inc(k);
      ++started;
    }
    if ((idle & work) != 0u) continue;  // all stages of an instant start before the clock moves

    // a8: advance to the earliest completion
    const double next = min_f64(min_f64(d.f0, d.f1), min_f64(d.f2, d.f3));
    if (!(next < kInf)) break;  // NaN: nothing running, every chunk is done (+inf: overflow)
    now = next;
    // deliver all completions of this instant, lowest chunk id first, so that
    // equal arrival times are appended in chunk-id order
    uint32_t g;
    uint32_t done = stages_ending(now, d, g);
    idle |= done;
    for (;;) {
      if ((g & 0x1000u) == 0u) push(g & 63u, g >> 15, (g >> 6) & 63u);
      done &= ~(1u << ((g >> 13) & 3u));
      if (done == 0u) break;
      // one more stage ends at this very instant (rare): the smallest one left
      g = min(min((done & 1u) ? d.s0 : ~0u, (done & 2u) ? d.s1 : ~0u),
              min((done & 4u) ? d.s2 : ~0u, (done & 8u) ? d.s3 : ~0u));
    }
  }

  FastResult res;
  // as in simulate_fast: every stage ran and completed, and none was too short
  // to move the clock
  const double t_min = model.t_min(D);
  const uint32_t stages = model.one_phase() ? D : 2u * D;
  res.ok = started == stages * C && idle == full && (now + 0.25 * t_min > now);
  res.t_done = now;
  res.busy[0] = d.z0; res.busy[1] = d.z1; res.busy[2] = d.z2; res.busy[3] = d.z3;
#pragma unroll
  for (uint32_t k = 0; k < (uint32_t)kMaxDims; ++k) res.executed[k] = executed.get(k);
  return res;
}

}  // namespace themis
