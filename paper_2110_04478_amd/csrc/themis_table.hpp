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
// Covered: single collectives (All-Reduce, Reduce-Scatter, All-Gather) of at
// most 64 chunks with at most kSlots distinct order codes (LayoutTable: every
// network of up to three dimensions).  With more distinct codes (four
// dimensions: up to 24) the sizes that can wait for one dimension no longer
// fit 16 classes; the wide variant (LayoutTableWideT, Classes64, DivModelT)
// gives every dimension 64 classes (one bitmap register pair each), keeps the
// slot in its own byte of the chunk word, pays for the larger list tables by
// redoing a stage time's divisions at each dispatch instead of tabulating
// them, and also comes with 128 chunk words.  Everything else stays with the
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
  bool gather;  // stand-alone All-Gather (chunk words hold the order code reversed)
  bool scf;
  double tmin;  // smallest tabulated stage time
  __device__ __forceinline__ uint32_t state0() const { return gather ? (((1u << D) - 1u) | 16u) : 0u; }
  __device__ __forceinline__ bool rs_only() const { return rs; }
  __device__ __forceinline__ bool one_phase() const { return rs || gather; }
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
  const bool gather = s.ctype == THEMIS_COLL_ALL_GATHER;
  const uint32_t state0 = gather ? (((1u << D) - 1u) | 16u) : 0u;
  uint64_t codes = 0;  // one byte per slot
  uint32_t n = 0;
  bool fits = true;
  for (uint32_t c = 0; c < s.C; ++c) {
    // a stand-alone All-Gather walks its code from the last field to the first
    const uint32_t code = gather ? reverse_code(code_at(c), (int)D) : code_at(c);
    uint32_t slot = n;
#pragma unroll
    for (uint32_t j = 0; j < LayoutTable::kSlots; ++j)
      if (j < n && ((uint32_t)(codes >> (8u * j)) & 0xffu) == code) slot = j;
    if (slot == n) {
      if (n == LayoutTable::kSlots) { fits = false; slot = 0; }
      else { codes |= (uint64_t)code << (8u * n); ++n; }
    }
    LayoutTable::init_chunk(lds, c, code, state0 | (slot << 5));
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
        for (uint32_t j = 0; j < D && !gather; ++j) {  // Reduce-Scatter stages shrink the resident size
          const uint32_t kj = (code >> (2u * j)) & 3u;
          if (kj == k) before_rs = x;
          x = x / (double)sel4((int)kj, s.P[0], s.P[1], s.P[2], s.P[3]);
        }
        for (uint32_t j = D; j-- > 0u;) {   // All-Gather stages grow it (back), last field first
          const uint32_t kj = (code >> (2u * j)) & 3u;
          if (kj == k) before_ag = x;
          x = x * (double)sel4((int)kj, s.P[0], s.P[1], s.P[2], s.P[3]);
        }
        lds_put_double(lds, LayoutTable::kTimeBase + 4u * sl, before_rs);
        lds_put_double(lds, LayoutTable::kTimeBase + 4u * sl + 2u, before_ag);
      }
      const uint32_t entries = 2u * n;  // entry 2*slot: RS, 2*slot+1: AG
      // a stand-alone Reduce-Scatter has only the even entries, an All-Gather only the odd ones
      const uint32_t first = gather ? 1u : 0u, step = (rs || gather) ? 2u : 1u;
      for (uint32_t e = first; e < entries; e += step) {
        const double v = lds_double(lds, LayoutTable::kTimeBase + 2u * e);
        uint32_t smaller = 0;
        for (uint32_t o = first; o < entries; o += step)
          smaller += lds_double(lds, LayoutTable::kTimeBase + 2u * o) < v ? 1u : 0u;
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
    if (gather) {
      // stages run from the code's last field to its first; each moves the grown size
      for (uint32_t j = D; j-- > 0u;) {
        const uint32_t kj = (code >> (2u * j)) & 3u;
        x = x * (double)sel4((int)kj, s.P[0], s.P[1], s.P[2], s.P[3]);
        const double t = x * sel4((int)kj, s.coef[0], s.coef[1], s.coef[2], s.coef[3]);
        lds_put_double(lds, LayoutTable::kTimeBase + 2u * (sl * 4u + j), t);
        tmin = min_f64(tmin, t);
      }
      continue;
    }
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
  model.gather = gather;
  model.scf = scf;
  model.tmin = tmin;
  return true;
}

// ---------------------------------------------------------------------------
// Wide variant: up to 24 distinct order codes, 64 size classes per dimension.
// ---------------------------------------------------------------------------
// Per-lane LDS (240 dwords, 60 KiB per wavefront, 2 wavefronts per CU):
//   dwords 0..63     chunk c: byte 0 mask | phase << 4, byte 1 next chunk,
//                    byte 2 order code, byte 3 slot
//   dwords 64..127   u8 head[256]: first chunk of list q = 64*dim + class
//   dwords 128..191  u8 tail[256]
//   dwords 192..239  class[slot][stage] bytes, 24 slots x 8 stages
// Before the event loop starts, the head and tail tables double as scratch
// for the setup (slot codes, then the sizes being ranked).
struct Classes64 {
  static constexpr uint32_t kPerDim = 64;
  // one 64-bit word per dimension, in registers: a four-way select by the
  // dimension costs less than the LDS round trips of a bitmap kept there
  uint64_t n0 = 0, n1 = 0, n2 = 0, n3 = 0;
  __device__ __forceinline__ explicit Classes64(const LaneLds&) {}
  __device__ __forceinline__ uint64_t of(uint32_t k) const { return sel4((int)k, n0, n1, n2, n3); }
  __device__ __forceinline__ void put(uint32_t k, uint64_t v) {
    n0 = k == 0u ? v : n0; n1 = k == 1u ? v : n1; n2 = k == 2u ? v : n2; n3 = k == 3u ? v : n3;
  }
  __device__ __forceinline__ bool mark(uint32_t q) {
    const uint32_t k = q >> 6;
    const uint64_t v = of(k), bit = 1ull << (q & 63u);
    put(k, v | bit);
    return (v & bit) != 0ull;
  }
  __device__ __forceinline__ uint32_t lowest(uint32_t k, uint32_t& field) const {
    field = 0u;
    return (uint32_t)__builtin_ctzll(of(k) | (1ull << 63));
  }
  __device__ __forceinline__ bool popped(uint32_t k, uint32_t cls, uint32_t, uint32_t, bool emptied) {
    const uint64_t v = of(k) ^ ((uint64_t)(emptied ? 1u : 0u) << cls);  // the bit was set
    put(k, v);
    return v == 0ull;
  }
};

template <uint32_t kChunks>
struct LayoutTableWideT {
  static constexpr bool kPacked = false;
  static constexpr uint32_t kCap = kChunks;
  static_assert(kChunks == 64 || kChunks == 128, "8-bit links; ids as in LayoutByte");
  static constexpr uint32_t kSlots = 24;
  // kChunks chunk dwords, then u8 head[256], u8 tail[256], u8 class[kSlots][8]
  static constexpr uint32_t kHeadBase = kChunks, kTailBase = kChunks + 64, kClassBase = kChunks + 128;
  static constexpr uint32_t kLaneWords = kClassBase + kSlots * 8u / 4u;  // 240 / 304
  static constexpr uint32_t kWavesPerSimd = 1;
  static constexpr uint32_t kEnd = 0xffu;
  using Link = uint8_t;
  using Classes = Classes64;
  using Ids = typename std::conditional<(kChunks <= 64), Pack4<uint32_t, 8>, Pack4<uint64_t, 16>>::type;
  static __device__ __forceinline__ void init_chunk(const LaneLds& l, uint32_t c, uint32_t code,
                                                    uint32_t slot, uint32_t state0) {
    *(uint32_t*)l.dword(c) = (slot << 24) | (code << 16) | (kEnd << 8) | state0;
  }
  static __device__ __forceinline__ uint32_t code(uint32_t w) { return (w >> 16) & 0xffu; }
  static __device__ __forceinline__ uint32_t next(uint32_t w) { return (w >> 8) & 0xffu; }
  static __device__ __forceinline__ void store_state(uint8_t* cp, uint32_t, uint32_t state) {
    *(uint16_t*)cp = (uint16_t)(state | (kEnd << 8));
  }
  static __device__ __forceinline__ Link* next_ptr(const LaneLds& l, uint32_t c) { return l.dword(c) + 1; }
  static __device__ __forceinline__ Link* head_ptr(const LaneLds& l, uint32_t q) {
    return l.base + ((kHeadBase + (q >> 2)) << 8) + (q & 3u);
  }
  static __device__ __forceinline__ Link* tail_ptr(const LaneLds& l, uint32_t q) {
    return l.base + ((kTailBase + (q >> 2)) << 8) + (q & 3u);
  }
};
using LayoutTableWide = LayoutTableWideT<64>;      // 240 dwords, two wavefronts per CU
using LayoutTableWide128 = LayoutTableWideT<128>;  // 304 dwords, two wavefronts per CU

// Model for the wide variant: classes from the table, stage times from the
// chunk size by the order's own divisions.
template <typename LT>
struct DivModelT {
  const Scenario& s;
  LaneLds lds;
  double chunk;
  double tmin;
  bool rs;
  bool gather;  // stand-alone All-Gather (chunk words hold the order code reversed)
  bool scf;
  __device__ __forceinline__ DivModelT(const Scenario& s_, const LaneLds& l, double chunk_, bool scf_)
      : s(s_), lds(l), chunk(chunk_), tmin(inf64()),
        rs(s_.ctype == THEMIS_COLL_REDUCE_SCATTER), gather(s_.ctype == THEMIS_COLL_ALL_GATHER),
        scf(scf_) {}
  __device__ __forceinline__ uint32_t state0() const {
    return gather ? (((1u << s.D) - 1u) | 16u) : 0u;
  }
  __device__ __forceinline__ bool rs_only() const { return rs; }
  __device__ __forceinline__ bool one_phase() const { return rs || gather; }
  __device__ __forceinline__ uint32_t keep(uint32_t) const { return 0u; }  // the slot has its own byte
  // x * coef on the pos-th dimension of `code`, x divided step by step
  // (All-Gather: x grown step by step from the code's last field down to pos)
  __device__ __forceinline__ double time_at(uint32_t code, uint32_t pos) const {
    double x = chunk;
    if (gather) {
      for (uint32_t j = (uint32_t)s.D; j-- > pos;) {
        const uint32_t kj = (code >> (2u * j)) & 3u;
        x = x * (double)sel4((int)kj, s.P[0], s.P[1], s.P[2], s.P[3]);
      }
      const uint32_t k = (code >> (2u * pos)) & 3u;
      return x * sel4((int)k, s.coef[0], s.coef[1], s.coef[2], s.coef[3]);
    }
    for (uint32_t j = 0; j < pos; ++j) {
      const uint32_t kj = (code >> (2u * j)) & 3u;
      x = x / (double)sel4((int)kj, s.P[0], s.P[1], s.P[2], s.P[3]);
    }
    const uint32_t k = (code >> (2u * pos)) & 3u;
    return x * sel4((int)k, s.coef[0], s.coef[1], s.coef[2], s.coef[3]);
  }
  __device__ __forceinline__ double stage_time(uint32_t, uint32_t, uint32_t w) const {
    const uint32_t pos = ((uint32_t)__builtin_popcount(w & 15u) - ((w >> 4) & 1u)) & 3u;
    return time_at(LT::code(w), pos);
  }
  __device__ __forceinline__ uint32_t size_class(uint32_t w, uint32_t mask, uint32_t phase) const {
    if (!scf) return 0u;
    const uint32_t r = (uint32_t)__builtin_popcount(mask);
    const uint32_t stage = (phase ? 2u * (uint32_t)s.D - r : r) & 7u;
    const uint32_t slot = w >> 24;
    const uint32_t idx = (slot < LT::kSlots ? slot : 0u) * 8u + stage;
    return lds.dword(LT::kClassBase + (idx >> 2))[idx & 3u];
  }
  __device__ __forceinline__ double t_min(uint32_t) const { return tmin; }
};

// Setup of the wide variant; code_at as in table_setup().  Cannot fail: four
// dimensions have 24 orders.
template <typename LT, typename CodeAt>
__device__ inline void table_setup_wide(const Scenario& s, bool scf, const LaneLds& lds,
                                        CodeAt code_at, DivModelT<LT>& model) {
  const uint32_t D = (uint32_t)s.D;
  // scratch: slot codes as bytes from dword kHeadBase, sizes as doubles from dword kHeadBase + 8
  auto slot_code = [&](uint32_t sl) -> uint8_t& { return lds.dword(LT::kHeadBase + (sl >> 2))[sl & 3u]; };
  const uint32_t sizes = LT::kHeadBase + 8u;
  uint32_t n = 0;
  for (uint32_t c = 0; c < s.C; ++c) {
    const uint32_t code = model.gather ? reverse_code(code_at(c), (int)D) : code_at(c);
    uint32_t slot = n;
    for (uint32_t j = 0; j < n; ++j)
      if (slot_code(j) == code) slot = j;
    if (slot == n) {
      if (n < LT::kSlots) { slot_code(n) = (uint8_t)code; ++n; }
      else slot = 0;  // unreachable for checked codes
    }
    LT::init_chunk(lds, c, code, slot, model.state0());
  }
  double tmin = inf64();
  for (uint32_t sl = 0; sl < n; ++sl)
    for (uint32_t j = 0; j < D; ++j) tmin = min_f64(tmin, model.time_at(slot_code(sl), j));
  model.tmin = tmin;
  if (!scf) return;
  for (uint32_t k = 0; k < D; ++k) {
    for (uint32_t sl = 0; sl < n; ++sl) {
      const uint32_t code = slot_code(sl);
      double x = model.chunk, before_rs = 0.0, before_ag = 0.0;
      for (uint32_t j = 0; j < D && !model.gather; ++j) {
        const uint32_t kj = (code >> (2u * j)) & 3u;
        if (kj == k) before_rs = x;
        x = x / (double)sel4((int)kj, s.P[0], s.P[1], s.P[2], s.P[3]);
      }
      for (uint32_t j = D; j-- > 0u;) {
        const uint32_t kj = (code >> (2u * j)) & 3u;
        if (kj == k) before_ag = x;
        x = x * (double)sel4((int)kj, s.P[0], s.P[1], s.P[2], s.P[3]);
      }
      lds_put_double(lds, sizes + 4u * sl, before_rs);
      lds_put_double(lds, sizes + 4u * sl + 2u, before_ag);
    }
    const uint32_t entries = 2u * n;
    // a stand-alone Reduce-Scatter has only the even entries, an All-Gather only the odd ones
    const uint32_t first = model.gather ? 1u : 0u, step = model.one_phase() ? 2u : 1u;
    for (uint32_t e = first; e < entries; e += step) {
      const double v = lds_double(lds, sizes + 2u * e);
      uint32_t smaller = 0;
#pragma unroll 4
      for (uint32_t o = first; o < entries; o += step)
        smaller += lds_double(lds, sizes + 2u * o) < v ? 1u : 0u;
      const uint32_t sl = e >> 1;
      const uint32_t code = slot_code(sl);
      uint32_t pos = 0;
      for (uint32_t j = 0; j < D; ++j)
        if (((code >> (2u * j)) & 3u) == k) pos = j;
      const uint32_t stage = (e & 1u) ? 2u * D - 1u - pos : pos;
      const uint32_t idx = sl * 8u + stage;
      lds.dword(LT::kClassBase + (idx >> 2))[idx & 3u] = (uint8_t)smaller;
    }
  }
}

}  // namespace themis
