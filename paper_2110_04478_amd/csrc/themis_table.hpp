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
  static constexpr bool kScaledProduct = false;  // stage times come from stage_time()
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
  static constexpr bool kScaledProduct = false;  // stage times come from stage_time()
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

// ---------------------------------------------------------------------------
// More than 128 chunks with NPU counts that are not powers of two: 16-bit
// chunk records as in themis_packed.hpp, with the chunk's slot where that
// file keeps the order (a slot stands for one order code, kept in a small
// table), 64 classes per dimension as in the wide variant, and a stage time's
// divisions redone at each dispatch.
//   record: bits 0-8 next chunk of its list (its own id: the last one),
//           bit 9 phase, bits 10-14 slot
// Lane block: u16 record[kChunks], u16 head[256], u16 tail[256] (a tail entry
// carries the upper bits of the tail chunk's record), u8 class[kSlots][8],
// u8 code[kSlots].  One wavefront per CU.
// ---------------------------------------------------------------------------
template <uint32_t kChunks>
struct LayoutTablePacked {
  static constexpr uint32_t kCap = kChunks;
  static_assert(kChunks <= 512 && kChunks % 2 == 0, "9-bit chunk ids, two records per dword");
  static constexpr uint32_t kSlots = 24;
  static constexpr uint32_t kHeadBase = kChunks / 2, kTailBase = kHeadBase + 128;
  static constexpr uint32_t kClassBase = kTailBase + 128, kCodeBase = kClassBase + kSlots * 8u / 4u;
  static constexpr uint32_t kLaneWords = kCodeBase + kSlots / 4u;  // 438 / 566
  static constexpr uint32_t kIdMask = 0x1ffu;
  using Ids = Pack4<uint64_t, 16>;
  static __device__ __forceinline__ uint16_t* half(const LaneLds& l, uint32_t base, uint32_t i) {
    return (uint16_t*)(l.base + ((base + (i >> 1)) << 8) + 2u * (i & 1u));
  }
  static __device__ __forceinline__ uint16_t* record(const LaneLds& l, uint32_t c) { return half(l, 0u, c); }
  static __device__ __forceinline__ uint16_t* head(const LaneLds& l, uint32_t q) { return half(l, kHeadBase, q); }
  static __device__ __forceinline__ uint16_t* tail(const LaneLds& l, uint32_t q) { return half(l, kTailBase, q); }
  static __device__ __forceinline__ uint8_t* slot_code(const LaneLds& l, uint32_t sl) {
    const uint32_t i = sl < kSlots ? sl : 0u;
    return l.dword(kCodeBase + (i >> 2)) + (i & 3u);
  }
  static __device__ __forceinline__ uint8_t* size_class(const LaneLds& l, uint32_t sl, uint32_t stage) {
    const uint32_t i = (sl < kSlots ? sl : 0u) * 8u + (stage & 7u);
    return l.dword(kClassBase + (i >> 2)) + (i & 3u);
  }
};

// Slots, records and class table for simulate_table_packed(); code_at as in
// table_setup().  model: a DivModelT (its chunk-word members are not used).
template <typename L, typename Model, typename CodeAt>
__device__ inline void table_setup_packed(const Scenario& s, bool scf, const LaneLds& lds,
                                          CodeAt code_at, Model& model) {
  const uint32_t D = (uint32_t)s.D;
  const uint32_t phase0 = (model.state0() >> 4) & 1u;
  const uint32_t sizes = L::kHeadBase;  // scratch: two doubles per slot
  uint32_t n = 0;
  for (uint32_t c = 0; c < s.C; ++c) {
    const uint32_t code = model.gather ? reverse_code(code_at(c), (int)D) : code_at(c);
    uint32_t slot = n;
    for (uint32_t j = 0; j < n; ++j)
      if (*L::slot_code(lds, j) == code) slot = j;
    if (slot == n) {
      if (n < L::kSlots) { *L::slot_code(lds, n) = (uint8_t)code; ++n; }
      else slot = 0;  // unreachable for checked codes
    }
    *L::record(lds, c) = (uint16_t)(c | (phase0 << 9) | (slot << 10));
  }
  double tmin = inf64();
  for (uint32_t sl = 0; sl < n; ++sl)
    for (uint32_t j = 0; j < D; ++j) tmin = min_f64(tmin, model.time_at(*L::slot_code(lds, sl), j));
  model.tmin = tmin;
  if (!scf) return;
  for (uint32_t k = 0; k < D; ++k) {
    for (uint32_t sl = 0; sl < n; ++sl) {
      const uint32_t code = *L::slot_code(lds, sl);
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
      const uint32_t code = *L::slot_code(lds, sl);
      uint32_t pos = 0;
      for (uint32_t j = 0; j < D; ++j)
        if (((code >> (2u * j)) & 3u) == k) pos = j;
      *L::size_class(lds, sl, (e & 1u) ? 2u * D - 1u - pos : pos) = (uint8_t)smaller;
    }
  }
}

// The event loop of simulate_packed() on slots: same contract as
// simulate_fast (result.ok false leaves the evaluation to the generic path).
// A chunk in the Reduce-Scatter phase at position pos of its order waits for
// stage pos, in the All-Gather phase for stage 2 D - 1 - pos.
template <typename L, int kQueueOrder, bool kBusy, typename Model>
__device__ __forceinline__ FastResult simulate_table_packed(const Scenario& s, const Model& model,
                                                            const LaneLds& lds, const FastOut& out) {
  static_assert(kQueueOrder == kNoQueueOrder || kQueueOrder == kBytes || kQueueOrder == kShorts,
                "entries are stored one by one");
  const uint32_t D = (uint32_t)s.D;
  const uint32_t C = s.C;
  const uint32_t full = (1u << D) - 1u;
  const double kInf = inf64();
  const bool rs_only = model.rs_only();
  const bool scf = model.scf;

  double f0 = kInf, f1 = kInf, f2 = kInf, f3 = kInf;  // finish time, +inf = idle
  double z0 = 0.0, z1 = 0.0, z2 = 0.0, z3 = 0.0;      // busy time
  // per dimension, the stage it serves and what its completion does: bits 0-7
  // list to join, 8-13 upper record bits then, 14 chunk is done, 15-16 the
  // dimension, 17-25 the chunk
  uint32_t v0 = 0, v1 = 0, v2 = 0, v3 = 0;
  typename L::Ids executed;  // operations started per dimension (kept when queue orders are written)
  uint32_t started = 0;      // operations started in all
  Classes64 classes(lds);
  uint32_t work = 0;      // bit k: some list of dimension k holds chunks
  uint32_t idle = full;   // bit k: dimension k serves nothing
  const uint32_t row_len = 2u * out.slots;

  // chunk c (upper record bits `up`: phase | slot << 1) becomes the last of list q = 64 * dim + class
  auto push = [&](uint32_t q, uint32_t c, uint32_t up) {
    const bool had = classes.mark(q);
    uint16_t* tp = L::tail(lds, q);
    const uint32_t t = *tp;
    const uint32_t rec = c | (up << 9);
    *L::record(lds, c) = (uint16_t)rec;  // own id: end of list
    uint16_t* dst = had ? L::record(lds, t & L::kIdMask) : L::head(lds, q);
    *dst = (uint16_t)(had ? ((t & ~L::kIdMask) | c) : c);
    *tp = (uint16_t)rec;
    work |= 1u << (q >> 6);
  };
  auto class_of = [&](uint32_t slot, uint32_t stage) -> uint32_t {
    return scf ? (uint32_t)*L::size_class(lds, slot, stage) : 0u;
  };

  // a6: every chunk waits at the dimension of its first stage, in chunk-id order
  {
    const uint32_t phase0 = (model.state0() >> 4) & 1u;
    const uint32_t pos0 = phase0 ? D - 1u : 0u, stage0 = phase0 ? D : 0u;
    for (uint32_t c = 0; c < C; ++c) {
      const uint32_t up = (uint32_t)*L::record(lds, c) >> 9;
      const uint32_t code = *L::slot_code(lds, up >> 1);
      push(64u * ((code >> (2u * pos0)) & 3u) + class_of(up >> 1, stage0), c, up);
    }
  }

  double now = 0.0;
  const uint32_t max_steps = 4u * D * C + 16u;
  for (uint32_t step = 0; step <= max_steps; ++step) {
    // a7: an idle dimension with waiting chunks starts its first one
    if (const uint32_t need = idle & work) {
      const uint32_t k = (uint32_t)__builtin_ctz(need);
      uint32_t field;
      const uint32_t cls = classes.lowest(k, field);  // smallest resident size
      const uint32_t q = 64u * k + cls;
      uint16_t* hp = L::head(lds, q);
      const uint32_t h = *hp;
      const uint32_t w = *L::record(lds, h);
      const uint32_t nx = w & L::kIdMask;
      *hp = (uint16_t)nx;  // harmless when the list is now empty
      const bool no_work = classes.popped(k, cls, q, field, nx == h);
      work &= ~((no_work ? 1u : 0u) << k);
      idle &= ~(1u << k);

      const uint32_t phase = (w >> 9) & 1u;
      const bool ag = phase != 0u;
      const uint32_t slot = (w >> 10) & 31u;
      const uint32_t code = *L::slot_code(lds, slot);
      const uint32_t o0 = code & 3u, o1 = (code >> 2) & 3u, o2 = (code >> 4) & 3u, o3 = code >> 6;
      const bool p0 = k == o0, p1 = k == o1, p2 = k == o2;
      const uint32_t pos = p0 ? 0u : p1 ? 1u : p2 ? 2u : 3u;
      // the All-Gather on k reuses the time of the chunk's Reduce-Scatter on k
      double t = model.time_at(code, pos);
      t = sel4((int)k, s.fix[0], s.fix[1], s.fix[2], s.fix[3]) + t;
      const double f = now + t;
      const bool k0 = k == 0u, k1 = k == 1u, k2 = k == 2u, k3 = k == 3u;
      f0 = k0 ? f : f0; f1 = k1 ? f : f1; f2 = k2 ? f : f2; f3 = k3 ? f : f3;
      if (kBusy) {
        z0 = __builtin_fma(t, k0 ? 1.0 : 0.0, z0); z1 = __builtin_fma(t, k1 ? 1.0 : 0.0, z1);
        z2 = __builtin_fma(t, k2 ? 1.0 : 0.0, z2); z3 = __builtin_fma(t, k3 ? 1.0 : 0.0, z3);
      }
      // what the completion will do: a Reduce-Scatter goes on to the next
      // dimension of the order, the last one turns into the All-Gather on the
      // same dimension; an All-Gather goes back to the previous one
      {
        const bool last_rs = !ag && pos + 1u == D;
        const bool finished = ag ? p0 : (last_rs && rs_only);
        const uint32_t prev = p1 ? o0 : p2 ? o1 : o2;
        const uint32_t succ = p0 ? o1 : p1 ? o2 : o3;
        const uint32_t kn = last_rs ? k : ag ? prev : succ;
        const uint32_t stage = last_rs ? D : ag ? 2u * D - pos : pos + 1u;
        const uint32_t up = (w >> 9) | (last_rs ? 1u : 0u);
        const uint32_t qn = 64u * kn + class_of(slot, stage);
        const uint32_t v = qn | (up << 8) | (finished ? 0x4000u : 0u) | (k << 15) | (h << 17);
        v0 = k0 ? v : v0; v1 = k1 ? v : v1; v2 = k2 ? v : v2; v3 = k3 ? v : v3;
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
        executed.inc(k);
      }
      ++started;
    }
    if ((idle & work) != 0u) continue;  // all stages of an instant start before the clock moves

    // a8: advance to the earliest completion
    const double next = min_f64(min_f64(f0, f1), min_f64(f2, f3));
    if (!(next < kInf)) break;  // nothing running: every chunk is done
    now = next;
    const bool d0 = f0 == now, d1 = f1 == now, d2 = f2 == now, d3 = f3 == now;
    uint32_t done = (d0 ? 1u : 0u) | (d1 ? 2u : 0u) | (d2 ? 4u : 0u) | (d3 ? 8u : 0u);
    f0 = d0 ? kInf : f0; f1 = d1 ? kInf : f1; f2 = d2 ? kInf : f2; f3 = d3 ? kInf : f3;
    idle |= done;
    // deliver all completions of this instant, lowest chunk id first
    uint32_t g0 = d0 ? v0 : ~0u, g1 = d1 ? v1 : ~0u, g2 = d2 ? v2 : ~0u, g3 = d3 ? v3 : ~0u;
    for (;;) {
      const uint32_t g = min(min(g0, g1), min(g2, g3));
      if ((g & 0x4000u) == 0u) push(g & 255u, g >> 17, (g >> 8) & 63u);
      done &= ~(1u << ((g >> 15) & 3u));
      if (done == 0u) break;
      g0 = g0 == g ? ~0u : g0; g1 = g1 == g ? ~0u : g1;
      g2 = g2 == g ? ~0u : g2; g3 = g3 == g ? ~0u : g3;
    }
  }

  FastResult res;
  // as in simulate_fast: every stage ran and completed, and none was too short
  // to move the clock
  const double t_min = model.t_min(D);
  const uint32_t stages = model.one_phase() ? D : 2u * D;
  res.ok = started == stages * C && idle == full && (now + 0.25 * t_min > now);
  res.t_done = now;
  res.busy[0] = z0; res.busy[1] = z1; res.busy[2] = z2; res.busy[3] = z3;
#pragma unroll
  for (uint32_t k = 0; k < (uint32_t)kMaxDims; ++k) res.executed[k] = executed.get(k);
  return res;
}

}  // namespace themis
