// LDS path of the queue simulation for NPU counts that are not powers of two.
//
// Dividing the resident size by an arbitrary P_k rounds, so the size of a
// chunk is no longer a function of the set of dimensions it is reduced on: it
// depends on the order of the divisions, i.e. on the chunk's own dimension
// order, and an All-Gather's multiplications do not undo them bit for bit.
// What still holds: a chunk's sizes and stage times are fixed by its order
// code alone.  So the sizes and times are tabulated once per scenario, per
// distinct order code ("slot", at most kSlots of them) and stage, with exactly
// the divisions and multiplications of the step-by-step arithmetic, and the
// event loop of themis_fast.hpp runs unchanged on top of the tables:
//   time[slot][pos]    stage time of the Reduce-Scatter (and of the All-Gather,
//                      which reuses it) on the pos-th dimension of the order
//   class[slot][stage] Smallest-Chunk-First class of the resident size before
//                      that stage: its rank among the sizes that can wait for
//                      the same dimension (two per slot, so at most 16)
// The slot of a chunk rides in the three spare bits of its state byte.
//
// Covered: single All-Reduce / Reduce-Scatter collectives of at most 64 chunks
// with at most kSlots distinct order codes.  Everything else stays with the
// generic path.
#pragma once

#include "themis_fast.hpp"

namespace themis {

struct LayoutTable : LayoutByte<64> {
  static constexpr uint32_t kSlots = 8;
  static constexpr uint32_t kTimeBase = LayoutByte<64>::kLaneWords;      // kSlots x 4 doubles
  static constexpr uint32_t kClassBase = kTimeBase + kSlots * 4u * 2u;   // kSlots x 8 bytes
  static constexpr uint32_t kLaneWords = kClassBase + kSlots * 8u / 4u;  // 160 dwords
  static constexpr uint32_t kWavesPerSimd = 1;
};

__device__ __forceinline__ double lds_double(const LaneLds& lds, uint32_t dword) {
  return __hiloint2double((int)*(const uint32_t*)lds.dword(dword + 1u),
                          (int)*(const uint32_t*)lds.dword(dword));
}
__device__ __forceinline__ void lds_put_double(const LaneLds& lds, uint32_t dword, double v) {
  *(uint32_t*)lds.dword(dword) = (uint32_t)__double2loint(v);
  *(uint32_t*)lds.dword(dword + 1u) = (uint32_t)__double2hiint(v);
}

// The model that simulate_fast() runs on (same members as Pow2Model).
struct TableModel {
  LaneLds lds;
  uint32_t D;
  bool rs;      // stand-alone Reduce-Scatter
  bool scf;
  double tmin;  // smallest tabulated stage time
  __device__ __forceinline__ uint32_t state0() const { return 0u; }
  __device__ __forceinline__ bool rs_only() const { return rs; }
  __device__ __forceinline__ bool one_phase() const { return rs; }
  __device__ __forceinline__ uint32_t keep(uint32_t w) const { return w & 0xe0u; }
  __device__ __forceinline__ double stage_time(uint32_t, uint32_t, uint32_t w) const {
    // RS: the next dimension of the order; AG: the last one still reduced
    const uint32_t pos = (uint32_t)__builtin_popcount(w & 15u) - ((w >> 4) & 1u);
    return lds_double(lds, LayoutTable::kTimeBase + 2u * (((w >> 5) & 7u) * 4u + (pos & 3u)));
  }
  __device__ __forceinline__ uint32_t size_class(uint32_t w, uint32_t mask, uint32_t phase) const {
    if (!scf) return 0u;
    // stage the chunk waits for: RS stage #reduced, AG stage 2D - #reduced
    const uint32_t r = (uint32_t)__builtin_popcount(mask);
    const uint32_t stage = (phase ? 2u * D - r : r) & 7u;
    const uint32_t idx = ((w >> 5) & 7u) * 8u + stage;
    return lds.dword(LayoutTable::kClassBase + (idx >> 2))[idx & 3u];
  }
  __device__ __forceinline__ double t_min(uint32_t) const { return tmin; }
};

// Assigns slots to the chunks' order codes and fills the chunk words and the
// tables.  code_at(c) yields chunk c's order code (already checked to be a
// permutation).  Returns false when the scenario has more than kSlots distinct
// codes.  Uses the time table's space as scratch while it ranks the sizes.
template <typename CodeAt>
__device__ inline bool table_setup(const Scenario& s, double chunk, bool scf, const LaneLds& lds,
                                   CodeAt code_at, TableModel& model) {
  const uint32_t D = (uint32_t)s.D;
  const bool rs = s.ctype == THEMIS_COLL_REDUCE_SCATTER;
  uint64_t codes = 0;  // one byte per slot
  uint32_t n = 0;
  bool fits = true;
  for (uint32_t c = 0; c < s.C; ++c) {
    const uint32_t code = code_at(c);
    uint32_t slot = n;
#pragma unroll
    for (uint32_t j = 0; j < LayoutTable::kSlots; ++j)
      if (j < n && ((uint32_t)(codes >> (8u * j)) & 0xffu) == code) slot = j;
    if (slot == n) {
      if (n == LayoutTable::kSlots) { fits = false; slot = 0; }
      else { codes |= (uint64_t)code << (8u * n); ++n; }
    }
    LayoutTable::init_chunk(lds, c, code, slot << 5);
  }
  if (!fits) return false;

  // Smallest-Chunk-First classes, one dimension at a time: the sizes before
  // the Reduce-Scatter and before the All-Gather on that dimension of every
  // slot (scratch: doubles 2*slot and 2*slot+1 of the time table), then each
  // one's rank among them
  if (scf) {
    for (uint32_t k = 0; k < D; ++k) {
      for (uint32_t sl = 0; sl < n; ++sl) {
        const uint32_t code = (uint32_t)(codes >> (8u * sl)) & 0xffu;
        double x = chunk, before_rs = 0.0, before_ag = 0.0;
        uint32_t pos_k = 0;
        for (uint32_t j = 0; j < D; ++j) {  // Reduce-Scatter stages shrink the resident size
          const uint32_t kj = (code >> (2u * j)) & 3u;
          if (kj == k) { before_rs = x; pos_k = j; }
          x = x / (double)sel4((int)kj, s.P[0], s.P[1], s.P[2], s.P[3]);
        }
        for (uint32_t j = D; j-- > 0u;) {   // All-Gather stages grow it back, last dimension first
          const uint32_t kj = (code >> (2u * j)) & 3u;
          if (kj == k) before_ag = x;
          x = x * (double)sel4((int)kj, s.P[0], s.P[1], s.P[2], s.P[3]);
        }
        (void)pos_k;
        lds_put_double(lds, LayoutTable::kTimeBase + 4u * sl, before_rs);
        lds_put_double(lds, LayoutTable::kTimeBase + 4u * sl + 2u, before_ag);
      }
      const uint32_t entries = 2u * n;  // entry 2*slot: RS, 2*slot+1: AG
      for (uint32_t e = 0; e < entries; ++e) {
        if (rs && (e & 1u)) continue;   // a stand-alone Reduce-Scatter has no All-Gather stages
        const double v = lds_double(lds, LayoutTable::kTimeBase + 2u * e);
        uint32_t smaller = 0;
        for (uint32_t o = 0; o < entries; ++o) {
          if (rs && (o & 1u)) continue;
          smaller += lds_double(lds, LayoutTable::kTimeBase + 2u * o) < v ? 1u : 0u;
        }
        const uint32_t sl = e >> 1;
        const uint32_t code = (uint32_t)(codes >> (8u * sl)) & 0xffu;
        uint32_t pos = 0;
        for (uint32_t j = 0; j < D; ++j)
          if (((code >> (2u * j)) & 3u) == k) pos = j;
        const uint32_t stage = (e & 1u) ? 2u * D - 1u - pos : pos;
        const uint32_t idx = sl * 8u + stage;
        lds.dword(LayoutTable::kClassBase + (idx >> 2))[idx & 3u] = (uint8_t)smaller;
      }
    }
  }

  // stage times: x * coef on the pos-th dimension of the order, x divided step by step
  double tmin = inf64();
  for (uint32_t sl = 0; sl < n; ++sl) {
    const uint32_t code = (uint32_t)(codes >> (8u * sl)) & 0xffu;
    double x = chunk;
    for (uint32_t j = 0; j < D; ++j) {
      const uint32_t kj = (code >> (2u * j)) & 3u;
      const double t = x * sel4((int)kj, s.coef[0], s.coef[1], s.coef[2], s.coef[3]);
      lds_put_double(lds, LayoutTable::kTimeBase + 2u * (sl * 4u + j), t);
      tmin = min_f64(tmin, t);
      x = x / (double)sel4((int)kj, s.P[0], s.P[1], s.P[2], s.P[3]);
    }
  }
  model.lds = lds;
  model.D = D;
  model.rs = rs;
  model.scf = scf;
  model.tmin = tmin;
  return true;
}

}  // namespace themis
