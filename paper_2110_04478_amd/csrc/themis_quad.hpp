// Event loop with four lanes per evaluation: lane j of a quad owns dimension j
// of the network (its FIFO lists per size class, the stage it serves, its
// finish and busy time), the four share one LDS block, and the clock of the
// evaluation is the minimum of the quad's finish times (paper Sec. 4.3 for the
// queues, Sec. 4.6.2 for the simulation that keeps every NPU's view the same).
//
// The mapping with one lane per evaluation keeps a whole evaluation's records
// in that lane's LDS block; at 512 chunks that is 80 KiB per wavefront and two
// wavefronts per CU, each alone on its SIMD and waiting out every dependent
// instruction and every LDS read.  Here a wavefront holds 16 evaluations in
// 20 KiB, eight wavefronts fit a CU, and a lane never has to pick one of four
// dimensions' registers: the arithmetic of a stage start and of a completion is
// plain code on the lane's own registers.  What it costs: a pass of the loop
// still handles one completion instant per evaluation, so four times as many
// wavefront-passes are needed for the same batch.
//
// Per evaluation (quad g of the wavefront), half-word i at byte 32 * i + 2 * g
// of the block (one shift and add; two quads share a dword, which the LDS
// serves like any other access to one bank):
//   i = c          record of chunk c, as in LayoutPacked: bits 0-8 next chunk of
//                  its list (its own id: last), bit 9 phase, bits 10-14 order
//   i = 512 + q    head of list q = 16 * dimension + class
//   i = 576 + q    record of the list's last chunk, 0xffff while it is empty
// The lists of dimension j are popped by lane j only; a completion appends to a
// list of another dimension (or its own), so appends are made one at a time
// per quad, in chunk-id order when several stages end at one instant, and the
// owner learns of them through a quad-wide OR of (dimension, class) bits.
#pragma once

#include "themis_packed.hpp"

namespace themis {

struct LayoutQuad {
  static constexpr uint32_t kCap = 512;
  static constexpr uint32_t kQuads = (uint32_t)kBlock / 4u;
  static constexpr uint32_t kHeadBase = kCap;
  static constexpr uint32_t kTailBase = kCap + 64u;
  static constexpr uint32_t kHalves = kCap + 128u;
  static constexpr uint32_t kBlockWords = kHalves / 2u * kQuads;  // 20 KiB per wavefront
  static constexpr uint32_t kWavesPerSimd = 2;
  static constexpr uint32_t kIdMask = 0x1ffu;
  static constexpr uint32_t kEmpty = 0xffffu;  // (a record's bit 15 is never set)
  static __device__ __forceinline__ uint16_t* half(uint8_t* base, uint32_t i) {
    return (uint16_t*)(base + (i << 5));
  }
  static __device__ __forceinline__ uint16_t* record(uint8_t* b, uint32_t c) { return half(b, c & kIdMask); }
  static __device__ __forceinline__ uint16_t* head(uint8_t* b, uint32_t q) { return half(b, kHeadBase + (q & 63u)); }
  static __device__ __forceinline__ uint16_t* tail(uint8_t* b, uint32_t q) { return half(b, kTailBase + (q & 63u)); }
  static __device__ __forceinline__ void init_chunk(uint8_t* b, uint32_t c, uint32_t code,
                                                    uint32_t state0, uint32_t D) {
    *record(b, c) = (uint16_t)(c | ((state0 >> 4) << 9) | (LayoutPacked<512>::order_field(code, D) << 10));
  }
};

// Values of the quad's other lanes: quad_perm [1,0,3,2] and [2,3,0,1].
__device__ __forceinline__ uint32_t quad_swap1(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0xb1, 0xf, 0xf, true);
}
__device__ __forceinline__ uint32_t quad_swap2(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x4e, 0xf, 0xf, true);
}
__device__ __forceinline__ uint32_t quad_min_u32(uint32_t v) {
  v = min(v, quad_swap1(v));
  return min(v, quad_swap2(v));
}
__device__ __forceinline__ uint32_t quad_or(uint32_t v) {
  v |= quad_swap1(v);
  return v | quad_swap2(v);
}
__device__ __forceinline__ uint32_t quad_sum(uint32_t v) {
  v += quad_swap1(v);
  return v + quad_swap2(v);
}
// Minimum of the quad's doubles, quiet NaNs skipped (NaN if all four are).
__device__ __forceinline__ double quad_min_f64(double v) {
  double o = __hiloint2double((int)quad_swap1((uint32_t)__double2hiint(v)),
                              (int)quad_swap1((uint32_t)__double2loint(v)));
  v = min_f64(v, o);
  o = __hiloint2double((int)quad_swap2((uint32_t)__double2hiint(v)),
                       (int)quad_swap2((uint32_t)__double2loint(v)));
  return min_f64(v, o);
}

struct QuadResult {
  double t_done;
  bool ok;  // false: leave the evaluation to the follow-up passes
};

// All four lanes of a quad call this with the same scenario and model; base is
// the quad's first byte in the wavefront's block (block + 2 * quad), whose
// records were written with LayoutQuad::init_chunk().  Power-of-two model only,
// times only.  Every lane of the wavefront has to be here (the quads exchange
// values with lane-crossing moves and leave the loop together).
template <bool kFix>
__device__ __forceinline__ QuadResult simulate_quad(const Scenario& s, const Pow2Model& model,
                                                    uint8_t* base, bool take_part) {
  using L = LayoutQuad;
  const uint32_t k = threadIdx.x & 3u;  // the lane's dimension
  const uint32_t D = (uint32_t)s.D;
  const uint32_t C = take_part ? s.C : 0u;
  const uint32_t full = (1u << D) - 1u;
  const uint32_t kbit = 1u << k;
  const double kInf = inf64();
  const uint32_t epack = model.fs.epack;
  const uint64_t ranktab = model.ranktab;
  const bool rs_only = model.rs_only();
  const double coef = sel4((int)k, s.coef[0], s.coef[1], s.coef[2], s.coef[3]);
  const double fix = kFix ? sel4((int)k, s.fix[0], s.fix[1], s.fix[2], s.fix[3]) : 0.0;

  double f = nan64();    // finish time of the stage the dimension serves, NaN when idle
  uint32_t sv = 0u;      // that stage: bits 0-5 list to join, 6-11 upper record bits then,
                         // 12 chunk is done, 15-23 the chunk
  uint32_t cm = 0u;      // bit c: list 16 * k + c holds chunks
  uint32_t started = 0u;

  for (uint32_t c = 0; c < 16u; ++c) *L::tail(base, 16u * k + c) = (uint16_t)L::kEmpty;

  // chunk c (upper record bits `up`: phase | order << 1) becomes the last of list q
  auto push = [&](uint32_t q, uint32_t c, uint32_t up) {
    uint16_t* tp = L::tail(base, q);
    const uint32_t t = *tp;
    const bool had = t != L::kEmpty;
    const uint32_t rec = c | (up << 9);
    *L::record(base, c) = (uint16_t)rec;  // own id: end of list
    uint16_t* dst = had ? L::record(base, t & L::kIdMask) : L::head(base, q);
    *dst = (uint16_t)(had ? ((t & ~L::kIdMask) | c) : c);
    *tp = (uint16_t)rec;
  };

  // a6: every chunk waits at the dimension of its first stage, in chunk-id
  // order; each lane takes the chunks that start on its own dimension
  {
    const uint32_t mask0 = model.state0() & 15u, phase0 = (model.state0() >> 4) & 1u;
    const uint32_t pos0 = (uint32_t)__builtin_popcount(mask0) - phase0;
    const uint32_t cls0 = (uint32_t)(ranktab >> (4u * mask0)) & 15u;
    for (uint32_t c = 0; c < C; ++c) {
      const uint32_t up = (uint32_t)*L::record(base, c) >> 9;
      if (PackedOrder(up >> 1).at(pos0) == k) {
        push(16u * k + cls0, c, up);
        cm |= 1u << cls0;
      }
    }
  }
  // the other lanes' records are written: their links must not be read before
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();

  double now = 0.0;
  bool went_on = true;  // every stage moved the clock
  const uint32_t max_steps = 2u * (uint32_t)kMaxDims * L::kCap + 16u;
  for (uint32_t step = 0; step <= max_steps; ++step) {
    // a7: an idle dimension with waiting chunks starts the first chunk of its
    // lowest class (smallest resident size); all dimensions at once
    if (!(f == f) && cm != 0u) {
      const uint32_t cls = (uint32_t)__builtin_ctz(cm);
      const uint32_t q = 16u * k + cls;
      uint16_t* hp = L::head(base, q);
      const uint32_t h = *hp;
      const uint32_t w = *L::record(base, h);
      const uint32_t nx = w & L::kIdMask;
      if (nx == h) {
        cm &= ~(1u << cls);
        *L::tail(base, q) = (uint16_t)L::kEmpty;
      } else {
        *hp = (uint16_t)nx;
      }
      const bool ag = ((w >> 9) & 1u) != 0u;
      const PackedOrder ord(w >> 10);
      // where k stands in the chunk's order, and the dimensions before it
      const bool p0 = k == ord.o0, p1 = k == ord.o1, p2 = k == ord.o2;
      const uint32_t before = p0 ? 0u : p1 ? (1u << ord.o0) : p2 ? ord.first_two
                                                                 : (ord.first_two | (1u << ord.o2));
      // what the completion of this stage will do (as in simulate_packed)
      const uint32_t with_k = before | kbit;
      const bool last_rs = !ag && with_k == full;
      const bool finished = ag ? p0 : (last_rs && rs_only);
      const uint32_t mask = ag ? before : with_k;
      const uint32_t prev = p1 ? ord.o0 : p2 ? ord.o1 : ord.o2;
      const uint32_t succ = p0 ? ord.o1 : p1 ? ord.o2 : ord.o3;
      const uint32_t kn = last_rs ? k : ag ? prev : succ;
      const uint32_t up = (w >> 9) | (last_rs ? 1u : 0u);
      const uint32_t qn = 16u * kn + ((uint32_t)(ranktab >> (4u * mask)) & 15u);
      sv = qn | ((up & 63u) << 6) | (finished ? 0x1000u : 0u) | (h << 15);
      // bytes moved on k = resident size before the chunk's Reduce-Scatter on k
      double t = scale_down(model.fs.base, esum(epack, before)) * coef;
      if (kFix) t = fix + t;
      f = now + t;
      went_on = went_on && f > now;
      ++started;
    }
    // (appends below read what the pops above have stored)
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    // a8: the clock moves to the earliest completion of the evaluation
    const double next = quad_min_f64(f);
    const bool running = next < kInf;   // NaN: nothing runs; +inf: overflow
    if (__builtin_amdgcn_ballot_w64(running) == 0ull) break;
    if (running) now = next;
    // the stages that end now hand their chunks on, one at a time per quad, the
    // lowest chunk id first, so that equal arrival times are appended in
    // chunk-id order
    bool pending = running && f == next;
    if (pending) f = nan64();
    uint32_t told_lo = 0u, told_hi = 0u;  // bit 16 * (dimension & 1) + class, dimensions 0-1 | 2-3
    do {
      // (every lane takes part in the exchange: no lane-crossing move may sit
      // behind a condition that differs inside a quad)
      const uint32_t key = pending ? sv : ~0u;
      const uint32_t first = quad_min_u32(key);
      const bool mine = pending && key == first;
      if (mine) {
        if ((sv & 0x1000u) == 0u) {
          const uint32_t qn = sv & 63u;
          push(qn, sv >> 15, (sv >> 6) & 63u);
          const uint32_t bit = 1u << (qn & 31u);
          told_lo |= qn < 32u ? bit : 0u;
          told_hi |= qn < 32u ? 0u : bit;
        }
        pending = false;
      }
      // the next append of the quad must find this one's stores
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
    } while (__builtin_amdgcn_ballot_w64(pending) != 0ull);
    told_lo = quad_or(told_lo);
    told_hi = quad_or(told_hi);
    cm |= ((k & 2u ? told_hi : told_lo) >> (16u * (k & 1u))) & 0xffffu;
  }

  QuadResult res;
  const double t_min = model.t_min(D);
  const uint32_t stages = model.one_phase() ? D : 2u * D;
  const bool settled = !(f == f) && cm == 0u && went_on;
  const uint32_t started_all = quad_sum(started);
  const uint32_t settled_all = quad_min_u32(settled ? 1u : 0u);
  res.ok = started_all == stages * s.C && settled_all == 1u && (now + 0.25 * t_min > now);
  res.t_done = now;
  return res;
}

}  // namespace themis
