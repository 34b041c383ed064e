// Event loop of the power-of-two fast path for up to 64 chunks on a per-lane
// LDS block small enough for twelve wavefronts per CU (three per SIMD).
//
// The loop of simulate_fast issues far fewer vector instructions than its
// SIMDs could take: with the two wavefronts per SIMD that its 80 dwords per
// lane allow, each wavefront spends a third of its time waiting for LDS reads
// and the other one cannot fill all of it.  A third wavefront per SIMD gains
// more than any instruction saved (wavefront counts that are not a multiple
// of four per CU gain nothing), so the block is cut to 48 dwords per lane:
//
//   16-bit record per chunk   bits 0-3   reduced-dims mask
//                             bits 4-9   first three fields of the order code
//                                        (the fourth is what is left: the XOR
//                                        of the three, for four dimensions)
//                             bits 10-15 next chunk of its list
//   8-bit tail per list       last chunk of list q = 16 * dimension + class
//
// The queue structure is the one of simulate_fast (paper Sec. 4.3: per
// dimension one FIFO list per resident-size class, appended in (arrival time,
// chunk id) order), but the lists are circular -- the tail's record points to
// the head -- so that one byte per list is enough.  The phase is not stored:
// a chunk waiting for dimension k is in its All-Gather phase exactly when k
// is among its reduced dimensions.
//
// Sub-dword elements normally cost address arithmetic (element -> dword and
// position inside it); here two (records) or four (tails) lanes share a dword
// instead: record c of lane L sits at byte c * 128 + (L & 31) * 4 + (L >> 5) * 2
// and tail q at q * 64 + (L & 15) * 4 + (L >> 4) behind the records, so every
// address is one shift-and-add.  Lanes that share a dword touch different
// bytes of it and hit the same bank with the same dword address, which the LDS
// serves without a conflict.
//
// What the completion of a stage will do (the list the chunk joins, its new
// record bits, whether it is finished) is worked out when the stage starts,
// from the record that has just been read, and kept in the dimension's
// register together with the chunk id; the completion itself then reads
// nothing but the tail of the list it appends to.
#pragma once

#include "themis_fast.hpp"

namespace themis {

struct LayoutRing {
  static constexpr bool kPacked = false;
  static constexpr bool kRing = true;
  static constexpr uint32_t kCap = 64;
  static constexpr uint32_t kRecBytes = kCap * 128u;   // 64 records x 64 lanes x 2 bytes
  static constexpr uint32_t kTailBytes = 64u * 64u;    // 64 lists x 64 lanes
  // The block itself needs 48 dwords per lane.  50 (12,800 bytes per
  // wavefront) is what measures best: twelve wavefronts per CU, three on every
  // SIMD.  With 48 or 49 a thirteenth wavefront fits, and kernels whose
  // registers allow a fourth wavefront on a SIMD then run 9 % slower (wavefront
  // counts per CU that are not a multiple of four never paid here); from 51 on
  // every kernel runs 7 % slower, as if only eleven were resident.
  static constexpr uint32_t kLaneWords = 50;
  static constexpr uint32_t kTableBytes = 24u * 8u * 2u;  // the wavefront's stage table (ring_loop)
  static_assert(kLaneWords * 256u >= kRecBytes + kTailBytes + kTableBytes, "block holds records, tails and table");
  static constexpr uint32_t kWavesPerSimd = 3;
  using Ids = Pack4<uint32_t, 8>;
  static __device__ __forceinline__ uint32_t lane_term_rec(uint32_t lane) {
    return (lane & 31u) * 4u + (lane >> 5) * 2u;
  }
  static __device__ __forceinline__ uint32_t lane_term_tail(uint32_t lane) {
    return kRecBytes + (lane & 15u) * 4u + (lane >> 4);
  }
  // l.base: block + lane_term_rec, l.aux: block + lane_term_tail
  static __device__ __forceinline__ uint16_t* rec(const LaneLds& l, uint32_t c) {
    return (uint16_t*)(l.base + (c << 7));
  }
  static __device__ __forceinline__ uint8_t* tail(const LaneLds& l, uint32_t q) {
    return l.aux + (q << 6);
  }
  // state0: initial mask | phase << 4 as in FastScenario (the phase is implied)
  static __device__ __forceinline__ void init_chunk(const LaneLds& l, uint32_t c, uint32_t code,
                                                    uint32_t state0) {
    *rec(l, c) = (uint16_t)((state0 & 15u) | ((code & 63u) << 4) | (c << 10));
  }
};

template <typename L, typename = void>
struct IsRing { static constexpr bool value = false; };
template <typename L>
struct IsRing<L, typename std::enable_if<L::kRing>::type> { static constexpr bool value = true; };

// Lowest set bit, all-ones for zero (the builtin is undefined there).
__device__ __forceinline__ uint32_t ffbl_or_ones(uint32_t v) {
  uint32_t r;
  asm("v_ffbl_b32 %0, %1" : "=v"(r) : "v"(v));
  return r;
}

// (a & mask) | (b & ~mask) in one instruction.
__device__ __forceinline__ uint32_t bfi(uint32_t mask, uint32_t a, uint32_t b) {
  uint32_t r;
  asm("v_bfi_b32 %0, %1, %2, %3" : "=v"(r) : "v"(mask), "v"(a), "v"(b));
  return r;
}

// All four fields of an order code from its first three: for four dimensions
// the fourth is the dimension left over, the XOR of the other three; for
// fewer the field is never looked at.
__device__ __forceinline__ uint32_t whole_code(uint32_t code6) {
  return code6 | (((code6 ^ (code6 >> 2) ^ (code6 >> 4)) & 3u) << 6);
}

// The ring loop's s0..s3 (DimState) hold the running stage as
//   bits 0-5   list the chunk joins when the stage completes
//   bit  6     the chunk is finished then
//   bits 7-16  low ten bits of its record then (mask, order fields)
//   bits 17-22 the chunk
// so the smallest value among the stages that end at an instant is the one of
// the lowest chunk id, and bits 7-22 are the record's bits and the chunk's link
// to itself as push() takes them.  With the wavefront's stage table (see
// ring_loop) the record's bits are a byte and the description is put together
// from whole bytes: bits 8-15 the record's low byte, bits 18-23 the chunk.
//
// The lanes of dimension J take their turn as the active ones (see
// start_stage_scaled): the stage time, the finish time, the busy time, the
// stage's description, and the dimension's sixteen bits taken out of the mask
// of idle dimensions.  At least five instructions follow the last v_cmpx
// inside every block, so no instruction that reads other lanes can come within
// the wait states an exec write by a vector instruction asks for.
// With kStaged the dimension also hands out the place of its next queue-order
// entry (w: byte offset inside the wavefront's staging block) and moves on by
// one entry, 64 bytes.
#define THEMIS_RING_BUSY_0(J)
#define THEMIS_RING_FIX_0(J)
#define THEMIS_RING_PLACE_0(J)
#define THEMIS_RING_BUSY_1(J) THEMIS_BUSY(J)
#define THEMIS_RING_FIX_1(J) THEMIS_FIX(J)
#define THEMIS_RING_PLACE_1(J) \
  "v_mov_b32_e32 %[at], %[w" #J "]\n\t" "v_add_u32_e32 %[w" #J "], 64, %[w" #J "]\n\t"
#define THEMIS_RING_START(J, IE, KEEP, BUSY, FIX, PLACE)                        \
  THEMIS_LANES_OF(J) THEMIS_MUL(J) THEMIS_RING_FIX_##FIX(J) THEMIS_END(J)      \
  THEMIS_RING_BUSY_##BUSY(J) THEMIS_SERVE(J) THEMIS_RING_PLACE_##PLACE(J)       \
  "v_and_b32_e32 %[" #IE "], %[" #KEEP "], %[" #IE "]\n\t" THEMIS_ALL_LANES
#define THEMIS_RING_STARTS(BUSY, FIX, PLACE)                                        \
  "s_mov_b64 %[act], exec\n\t"                                                      \
  THEMIS_RING_START(0, iel, upper, BUSY, FIX, PLACE) THEMIS_RING_START(1, iel, lower, BUSY, FIX, PLACE) \
  THEMIS_RING_START(2, ieh, upper, BUSY, FIX, PLACE) THEMIS_RING_START(3, ieh, lower, BUSY, FIX, PLACE)

// the two halves of a register, from scalar registers (a literal would make
// the instruction twice as long)
#define THEMIS_RING_HALVES [upper] "s"(0xffff0000u), [lower] "s"(0x0000ffffu)

// Place of the next queue-order entry of every dimension in the staging block.
struct RingPlaces { uint32_t w0, w1, w2, w3; };
#define THEMIS_W_OPERANDS [w0] "+v"(w.w0), [w1] "+v"(w.w1), [w2] "+v"(w.w2), [w3] "+v"(w.w3)

// Returns the place of this stage's queue-order entry (kStaged, else 0).
template <bool kBusy, bool kFix, bool kStaged>
__device__ __forceinline__ uint32_t ring_start_stage(uint32_t k, uint32_t val, double now, double x,
                                                     const double (&c)[kMaxDims],
                                                     const double (&a)[kMaxDims], DimState& d,
                                                     uint32_t& ie_lo, uint32_t& ie_hi, RingPlaces& w) {
  uint64_t act;
  double t;
  uint32_t at = 0u;
#define THEMIS_RING_OUT [act] "=&s"(act), [t] "=&v"(t), [iel] "+v"(ie_lo), [ieh] "+v"(ie_hi), \
                        THEMIS_F_OPERANDS, THEMIS_S_OPERANDS
#define THEMIS_RING_IN [k] "v"(k), [val] "v"(val), [now] "v"(now), [x] "v"(x), THEMIS_RING_HALVES, \
                       THEMIS_C_OPERANDS
  if (kStaged) {
    if (kBusy && kFix) {
      asm volatile(THEMIS_RING_STARTS(1, 1, 1)
          : THEMIS_RING_OUT, THEMIS_Z_OPERANDS, [at] "+v"(at), THEMIS_W_OPERANDS
          : THEMIS_RING_IN, THEMIS_A_OPERANDS : "vcc");
    } else if (kBusy) {
      asm volatile(THEMIS_RING_STARTS(1, 0, 1)
          : THEMIS_RING_OUT, THEMIS_Z_OPERANDS, [at] "+v"(at), THEMIS_W_OPERANDS
          : THEMIS_RING_IN : "vcc");
    } else if (kFix) {
      asm volatile(THEMIS_RING_STARTS(0, 1, 1)
          : THEMIS_RING_OUT, [at] "+v"(at), THEMIS_W_OPERANDS
          : THEMIS_RING_IN, THEMIS_A_OPERANDS : "vcc");
    } else {
      asm volatile(THEMIS_RING_STARTS(0, 0, 1)
          : THEMIS_RING_OUT, [at] "+v"(at), THEMIS_W_OPERANDS
          : THEMIS_RING_IN : "vcc");
    }
  } else if (kBusy && kFix) {
    asm volatile(THEMIS_RING_STARTS(1, 1, 0)
        : THEMIS_RING_OUT, THEMIS_Z_OPERANDS : THEMIS_RING_IN, THEMIS_A_OPERANDS : "vcc");
  } else if (kBusy) {
    asm volatile(THEMIS_RING_STARTS(1, 0, 0)
        : THEMIS_RING_OUT, THEMIS_Z_OPERANDS : THEMIS_RING_IN : "vcc");
  } else if (kFix) {
    asm volatile(THEMIS_RING_STARTS(0, 1, 0)
        : THEMIS_RING_OUT : THEMIS_RING_IN, THEMIS_A_OPERANDS : "vcc");
  } else {
    asm volatile(THEMIS_RING_STARTS(0, 0, 0) : THEMIS_RING_OUT : THEMIS_RING_IN : "vcc");
  }
#undef THEMIS_RING_OUT
#undef THEMIS_RING_IN
  return at;
}

// The clock has moved to `now`: every dimension whose stage ends now becomes
// idle (quiet NaN as its finish time, its sixteen bits back in the mask of
// idle dimensions).  Returns the bits of those dimensions plus sixteen times
// their number (32 and more: several at once) and, in `first`, the smallest
// stage description among them (all-ones if there is none).
#define THEMIS_RING_ENDS(J, BIT, IE, FIELD)                 \
  "v_cmpx_eq_f64_e32 vcc, %[now], %[f" #J "]\n\t"          \
  "v_mov_b64_e32 %[f" #J "], %[nan]\n\t"                   \
  "v_min_u32_e32 %[first], %[first], %[s" #J "]\n\t"       \
  "v_add_u32_e32 %[done], " #BIT ", %[done]\n\t"           \
  "v_or_b32_e32 %[" #IE "], %[" #FIELD "], %[" #IE "]\n\t" THEMIS_ALL_LANES
__device__ __forceinline__ uint32_t ring_stages_ending(double now, DimState& d, uint32_t& first,
                                                       uint32_t& ie_lo, uint32_t& ie_hi) {
  uint64_t act;
  uint32_t done = 0u;
  first = ~0u;
  asm volatile("s_mov_b64 %[act], exec\n\t"
      THEMIS_RING_ENDS(0, 17, iel, lower) THEMIS_RING_ENDS(1, 18, iel, upper)
      THEMIS_RING_ENDS(2, 20, ieh, lower) THEMIS_RING_ENDS(3, 24, ieh, upper)
      : [act] "=&s"(act), [done] "+v"(done), [first] "+v"(first), [iel] "+v"(ie_lo),
        [ieh] "+v"(ie_hi), THEMIS_F_OPERANDS
      : [now] "v"(now), [nan] "v"(nan64()), [s0] "v"(d.s0), [s1] "v"(d.s1), [s2] "v"(d.s2),
        [s3] "v"(d.s3), THEMIS_RING_HALVES
      : "vcc");
  return done;
}

constexpr uint32_t kRingFinished = 64u;

// Position of the next stage in a chunk's order once its reduced dimensions
// are mask2: the number of reduced dimensions, less one in the All-Gather
// phase (phase: the stage that ends is an All-Gather; mask2 == full: it is the
// last Reduce-Scatter, and the All-Gather starts on the same dimension).  The
// two cases exclude each other, so both go into one subtract-with-borrow.
__device__ __forceinline__ uint32_t ring_next_position(uint32_t mask2, uint32_t full, uint32_t phase) {
  uint32_t pos;
  asm("v_bcnt_u32_b32 %0, %1, 0\n\t"
      "v_cmp_eq_u32_e32 vcc, %1, %2\n\t"
      "v_subb_co_u32_e32 %0, vcc, %0, %3, vcc"
      : "=&v"(pos) : "v"(mask2), "v"(full), "v"(phase) : "vcc");
  return pos;
}

__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) {
  uint32_t r;
  asm("v_bitop3_b32 %0, %1, %2, %3 bitop3:0x96" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

// Lexicographic rank (0..23) of an order code whose D fields are a
// permutation of 0..D-1, read as a permutation of all four dimensions (the
// unused fields take their own index).
__device__ __forceinline__ uint32_t ring_order_rank(uint32_t code, uint32_t D) {
  const uint32_t c8 = code | (0xe4u & ~((1u << (2u * D)) - 1u));
  const uint32_t o0 = c8 & 3u, o1 = (c8 >> 2) & 3u, o2 = (c8 >> 4) & 3u, o3 = (c8 >> 6) & 3u;
  const uint32_t r1 = o1 - (o1 > o0 ? 1u : 0u);
  return 6u * o0 + 2u * r1 + (o2 > o3 ? 1u : 0u);
}

// The four-field order code of rank r (inverse of ring_order_rank).
__device__ __forceinline__ uint32_t ring_order_of_rank(uint32_t r) {
  uint32_t pool = 0x3210u, code = 0u, fact = 6u;
#pragma unroll
  for (uint32_t j = 0; j < 4u; ++j) {
    const uint32_t pick = r / fact;
    r -= pick * fact;
    code |= ((pool >> (4u * pick)) & 3u) << (2u * j);
    pool = (pool & ((1u << (4u * pick)) - 1u)) | ((pool >> (4u * (pick + 1u))) << (4u * pick));
    if (j < 2u) fact /= (3u - j);
  }
  return code;
}

// Entry (order of rank r, `behind` stages done) of the wavefront's stage table
// (see ring_loop): the chunk's states are walked from the initial one, with the
// transitions the loop without a table takes one at a time.
__device__ inline uint32_t ring_table_entry(uint32_t r, uint32_t behind, uint32_t state0,
                                            uint32_t full, uint32_t fin_mask, uint32_t epack,
                                            uint64_t ranktab) {
  const uint32_t code = ring_order_of_rank(r);
  uint32_t mask = state0 & 15u, phase = (state0 >> 4) & 1u;
  for (uint32_t i = 0; i <= behind; ++i) {
    const uint32_t pos = ((uint32_t)__builtin_popcount(mask) - phase) & 3u;
    const uint32_t k = (code >> (2u * pos)) & 3u;
    const uint32_t mask2 = (mask ^ (1u << k)) & 15u;
    const uint32_t phase2 = phase | (mask2 == full ? 1u : 0u);
    if (i == behind) {
      const uint32_t pos2 = ((uint32_t)__builtin_popcount(mask2) - phase2) & 3u;
      const uint32_t kn = (code >> (2u * pos2)) & 3u;
      const uint32_t cls2 = (uint32_t)(ranktab >> (4u * mask2)) & 15u;
      return (16u * kn + cls2) | (mask2 == fin_mask ? kRingFinished : 0u) | (phase << 9) |
             ((esum(epack, mask & mask2) & 63u) << 10);
    }
    mask = mask2;
    phase = phase2;
  }
  return 0u;
}

// Same contract as simulate_fast: records initialised with
// LayoutRing::init_chunk(), result.ok false leaves the evaluation to the
// generic path; power-of-two model only.  Queue orders leave as single
// entries: kBytes into the lane's own rows; kStagedBytes into the wavefront's
// staging block, entry j of dimension k of lane L at byte (k * 2 * slots + j) *
// 64 + L, so that the place of a dimension's next entry is one register that
// moves on by 64 (kept per dimension, advanced in the dimension's turn) and the
// entries the lanes store at about the same time share cache lines.  The
// stores go through a buffer descriptor of the block's size: whatever the
// records hold, nothing is written outside the block.  Nothing in the LDS
// block has to be cleared beforehand.
//
// The wavefront leaves the loop as a whole: a lane that is through (no list
// holds a chunk, no stage runs) finds nothing to start and nothing to complete
// in the passes its neighbours still need, so it needs no exit of its own and
// the loop carries no mask of lanes that have left.
//
// kTable: every lane of the wavefront evaluates the same network under the
// same policy (the usual parameter study: one topology, many bandwidths, sizes
// and thresholds), so what a stage does depends only on the chunk's order and
// on how many stages it has behind it.  The wavefront then shares one table in
// LDS, entry (order, stage):
//   bits 0-5   list the chunk joins when the stage completes
//   bit  6     the chunk is finished then
//   bit  9     the stage is an All-Gather
//   bits 10-15 sum of log2 P over the dimensions the chunk is reduced on,
//              the stage's own dimension left out (its resident-size exponent;
//              networks of more than 2^63 NPUs go without a table)
// and a chunk's record carries bits 0-2 the number of stages behind it and
// bits 3-7 its order as the lexicographic rank of the four-field code, in
// place of mask and order fields.  One table read replaces the arithmetic that
// derives all of that from mask and code at every stage start.
template <bool kTable, int kQueueOrder, bool kBusy, bool kFix>
__device__ __forceinline__ FastResult ring_loop(const Scenario& s, const Pow2Model& model,
                                                const LaneLds& lds, const FastOut& out,
                                                const uint8_t* table) {
  static_assert(kQueueOrder == kNoQueueOrder || kQueueOrder == kBytes || kQueueOrder == kStagedBytes,
                "entries are stored one by one");
  using L = LayoutRing;
  const uint32_t D = (uint32_t)s.D;
  const uint32_t C = s.C;
  const uint32_t full = (1u << D) - 1u;
  const double kInf = inf64();
  const uint32_t epack = model.fs.epack;
  const uint64_t ranktab = model.ranktab;
  // a chunk is finished when its mask comes back to zero (the last All-Gather
  // of an All-Reduce or an All-Gather; a Reduce-Scatter never leaves zero), a
  // stand-alone Reduce-Scatter when it is full
  const uint32_t fin_mask = model.rs_only() ? full : 0u;

  DimState d;
  d.f0 = d.f1 = d.f2 = d.f3 = nan64();
  d.z0 = d.z1 = d.z2 = d.z3 = 0.0;
  d.s0 = d.s1 = d.s2 = d.s3 = 0u;
  uint32_t ne_lo = 0u, ne_hi = 0u;    // bit q of the pair: list q holds chunks
  uint32_t ie_lo = ~0u, ie_hi = ~0u;  // the sixteen bits of every idle dimension
  typename L::Ids executed;           // operations started per dimension (kBytes)
  uint32_t started = 0;               // operations started in all (counted without queue orders)
  const uint32_t row_len = 2u * out.slots;
  constexpr bool kStaged = kQueueOrder == kStagedBytes;
  RingPlaces place;                   // kStaged: where each dimension's next entry goes
  place.w0 = out.lane_offset;
  place.w1 = out.lane_offset + 64u * row_len;
  place.w2 = out.lane_offset + 128u * row_len;
  place.w3 = out.lane_offset + 192u * row_len;
  __amdgpu_buffer_rsrc_t staging = __builtin_amdgcn_make_buffer_rsrc(
      kStaged ? out.queue_order : nullptr, 0, kStaged ? out.staging_bytes : 0u, 0x00020000);

  // chunk c = w >> 10, whose record is to carry w & 0x3ff (mask, order
  // fields), becomes the last of list q (only the low six bits of q count).
  // Branch-free: c takes over the old tail's link to the head, then the old
  // tail is made to point to c.  For an empty list c stands in as its own old
  // tail: the second store then writes c's record again, with c's own bits and
  // the link to itself.
  constexpr uint32_t kValShift = kTable ? 8u : 7u;  // a stage's description >> kValShift is push()'s w
  auto push = [&](uint32_t q, uint32_t w) {
    const uint64_t bit = 1ull << (q & 63u);
    const uint32_t b_lo = (uint32_t)bit, b_hi = (uint32_t)(bit >> 32);
    const bool had = ((ne_lo & b_lo) | (ne_hi & b_hi)) != 0u;
    uint8_t* tp = L::tail(lds, q & 63u);
    const uint32_t c = w >> 10;
    const uint32_t last = *tp & 63u;     // (an empty list's tail byte is whatever it last held)
    const uint32_t t = had ? last : c;
    uint16_t* rt_p = L::rec(lds, t);
    const uint32_t rt = *rt_p;
    *L::rec(lds, c) = (uint16_t)bfi(0x3ffu, w, rt);   // low ten bits of w, the old tail's link
    *rt_p = (uint16_t)bfi(0x3ffu, had ? rt : w, w);   // the old tail's own bits, link to c
    *tp = (uint8_t)c;
    ne_lo |= b_lo;
    ne_hi |= b_hi;
  };

  // a6: every chunk waits at the dimension of its first stage, in chunk-id
  // order, in the class of the initial mask
  {
    const uint32_t mask0 = model.state0() & 15u, phase0 = (model.state0() >> 4) & 1u;
    const uint32_t pos0 = 2u * ((uint32_t)__builtin_popcount(mask0) - phase0);
    const uint32_t cls0 = (uint32_t)(ranktab >> (4u * mask0)) & 15u;
    for (uint32_t c = 0; c < C; ++c) {
      const uint32_t low10 = (uint32_t)*L::rec(lds, c) & 0x3ffu;
      const uint32_t code = whole_code(low10 >> 4);
      // kTable: no stage behind it, the order by its rank
      push(16u * ((code >> pos0) & 3u) + cls0,
           (kTable ? ring_order_rank(code, D) << 3 : low10) | (c << 10));
    }
  }

  double now = 0.0;
  // One pass starts at most one stage and, once no idle dimension has chunks
  // waiting, advances the clock to the next completion (as in simulate_fast).
  // Every pass of a lane that is not through starts or completes a stage, so
  // 4 * D * C passes and a few always suffice; the bound is the same for all
  // lanes (it only has to end the loop whatever the records hold).
  constexpr uint32_t kMaxSteps = 4u * (uint32_t)kMaxDims * L::kCap + 16u;
  for (uint32_t step = 0; step < kMaxSteps; ++step) {
    // a7: the lowest idle dimension with chunks waiting starts the first chunk
    // of its lowest class -- the lowest set bit among the lists of idle dimensions
    const uint32_t q = min(ffbl_or_ones(ne_lo & ie_lo), ffbl_or_ones(ne_hi & ie_hi) | 32u);
    uint32_t pending = 0u;  // lists of idle dimensions that still hold chunks (q == 64: none do)
    if (q < 64u) {
      const uint32_t k = q >> 4;
      uint8_t* tp = L::tail(lds, q);
      const uint32_t t = *tp & 63u;
      uint16_t* rt_p = L::rec(lds, t);
      const uint32_t rt = *rt_p;
      const uint32_t h = rt >> 10;                    // the head follows the tail
      const uint32_t rh = *L::rec(lds, h);
      // the tail now points to the head's successor (h == t: the list is empty
      // and the record is written afresh when the chunk joins a list again)
      *rt_p = (uint16_t)bfi(0x3ffu, rt, rh);
      const uint64_t gone = (uint64_t)(((h ^ t) - 1u) >> 31) << q;  // the list's bit if h == t
      uint32_t entry, val;   // entry: chunk << 1 | All-Gather
      double bytes;
      if (kTable) {
        const uint32_t e = *(const uint16_t*)(table + 2u * (rh & 0xffu));
        // the head's id from the tail's link, above the entry's low ten bits
        const uint32_t he = bfi(0xfc00u, rt, e);
        entry = he >> 9;  // the phase is the bit below the id
        // byte 0: list and finished bit, byte 1: the record's low byte then (one
        // more stage behind it), byte 2: the chunk << 2 (and the phase below it)
        val = __builtin_amdgcn_perm(rh + 1u, he, 0x0c010400u);
        bytes = __hiloint2double(__double2hiint(model.fs.base) - (int)((e << 10) & 0x03f00000u),
                                 __double2loint(model.fs.base));
      } else {
        const uint32_t kbit = 1u << k;
        const uint32_t mask = rh & 15u;
        const uint32_t phase = (mask >> k) & 1u;  // waiting for k while reduced on k: All-Gather
        entry = (h + h) | phase;
        // what the completion of this stage will do: a Reduce-Scatter sets the
        // dimension's bit, an All-Gather clears it; the last Reduce-Scatter is
        // followed by the All-Gather on the same dimension
        const uint32_t mask2 = mask ^ kbit;
        // next stage: RS -> order[#reduced], AG -> order[#reduced - 1]
        const uint32_t pos = ring_next_position(mask2, full, phase);
        const uint32_t c6 = (rh >> 4) & 63u;
        const uint32_t code = (xor3(c6, c6 >> 2, c6 >> 4) << 6) | c6;   // bits 6-7: the fourth field
        const uint32_t kn = (code >> ((pos + pos) & 31u)) & 3u;         // (finished: not used)
        const uint32_t cls2 = (uint32_t)(ranktab >> (4u * mask2)) & 15u;
        const uint32_t q2 = (16u * kn + cls2) | (mask2 == fin_mask ? kRingFinished : 0u);
        // the chunk and its record's low bits then (the stage flips k's bit), above the list
        val = (bfi(0x3ffu, rh ^ kbit, rt) << 7) | q2;
        // (mask & mask2 is mask without k, whichever way the stage flips it)
        bytes = scale_down(model.fs.base, esum(epack, mask & mask2));
      }
      // bytes moved on k = resident size before the chunk's Reduce-Scatter on
      // k, i.e. with every reduced dimension but k itself taken off
      const uint32_t at = ring_start_stage<kBusy, kFix, kStaged>(k, val, now, bytes, s.coef, s.fix, d,
                                                                 ie_lo, ie_hi, place);
      if (kStaged) {
        __builtin_amdgcn_raw_buffer_store_b8((uint8_t)entry, staging, (int)at, 0, 0);
      } else if (kQueueOrder == kBytes) {
        const uint32_t pos_k = executed.get(k);
        // pos_k < row_len always holds for a consistent plan; it keeps the store in bounds
        if (pos_k < row_len) out.queue_order[k * row_len + pos_k] = (uint8_t)entry;
        executed.inc(k);
      } else {
        ++started;
      }
      // k is no longer among the idle dimensions, so whether its list has just
      // emptied does not matter here: the bit is taken out afterwards
      pending = (ne_lo & ie_lo) | (ne_hi & ie_hi);
      ne_lo ^= (uint32_t)gone;
      ne_hi ^= (uint32_t)(gone >> 32);
    }
    // all stages of an instant start before the clock moves; then the clock
    // advances to the earliest completion (NaN: nothing runs; +inf: overflow)
    // Both conditions as lane masks in scalar registers (of the lanes that are
    // here: a comparison writes zero for the others): the branch and the
    // wavefront's exit are then scalar work.
    const double next = min_f64(min_f64(d.f0, d.f1), min_f64(d.f2, d.f3));
    uint64_t more, running;
    asm volatile("v_cmp_ne_u32_e64 %0, 0, %1" : "=s"(more) : "v"(pending));
    asm volatile("v_cmp_lt_f64_e64 %0, %1, %2" : "=s"(running) : "v"(next), "s"(kInf));
    if (__builtin_amdgcn_inverse_ballot_w64(running & ~more)) {
      now = next;
      // a8: deliver all completions of this instant, lowest chunk id first, so
      // that equal arrival times are appended in chunk-id order
      uint32_t key;
      uint32_t done = ring_stages_ending(now, d, key, ie_lo, ie_hi);
      if ((key & kRingFinished) == 0u) push(key, key >> kValShift);
      // more stages end at this very instant (rare): the smallest one left, again and again
      while (done >= 32u) {
        done -= 16u;
        done &= ~((key == d.s0 ? 1u : 0u) | (key == d.s1 ? 2u : 0u) | (key == d.s2 ? 4u : 0u) |
                  (key == d.s3 ? 8u : 0u));
        key = min(min((done & 1u) ? d.s0 : ~0u, (done & 2u) ? d.s1 : ~0u),
                  min((done & 4u) ? d.s2 : ~0u, (done & 8u) ? d.s3 : ~0u));
        if ((key & kRingFinished) == 0u) push(key, key >> kValShift);
      }
    }
    // through: nothing waits, nothing runs -- for every lane of the wavefront
    if ((more | running) == 0ull) break;
  }

  FastResult res;
  // as in simulate_fast: every stage ran and completed, and none was too short
  // to move the clock
  const double t_min = model.t_min(D);
  const uint32_t stages = model.one_phase() ? D : 2u * D;
  if (kStaged) {
    // a dimension's place has moved on by 64 bytes per operation
    const uint32_t n0 = (place.w0 - out.lane_offset) >> 6;
    const uint32_t n1 = (place.w1 - out.lane_offset) >> 6, n2 = (place.w2 - out.lane_offset) >> 6;
    const uint32_t n3 = (place.w3 - out.lane_offset) >> 6;
    res.executed[0] = n0; res.executed[1] = n1 - row_len;
    res.executed[2] = n2 - 2u * row_len; res.executed[3] = n3 - 3u * row_len;
    started = n0 + n1 + n2 + n3 - 6u * row_len;
  } else if (kQueueOrder != kNoQueueOrder) {
    started = executed.sum();
  }
  res.ok = started == stages * C && (ie_lo & ie_hi) == ~0u && (ne_lo | ne_hi) == 0u &&
           (now + 0.25 * t_min > now);
  res.t_done = now;
  res.busy[0] = d.z0; res.busy[1] = d.z1; res.busy[2] = d.z2; res.busy[3] = d.z3;
  if (!kStaged) {
#pragma unroll
    for (uint32_t k = 0; k < (uint32_t)kMaxDims; ++k) res.executed[k] = executed.get(k);
  }
  return res;
}

constexpr uint32_t kRingTableEntries = 24u * 8u;

template <int kQueueOrder, bool kBusy, bool kFix>
__device__ __forceinline__ FastResult simulate_ring(const Scenario& s, const Pow2Model& model,
                                                    const LaneLds& lds, const FastOut& out) {
  using L = LayoutRing;
  // Do the lanes that are here (others may have left with an invalid scenario)
  // all evaluate the same network, collective type and queue policy?
  const uint32_t D = (uint32_t)s.D;
  const uint32_t full = (1u << D) - 1u;
  const uint32_t fin_mask = model.rs_only() ? full : 0u;
  const uint32_t sig[5] = {model.fs.epack, D | (model.state0() << 8) | (fin_mask << 16),
                           (uint32_t)model.ranktab, (uint32_t)(model.ranktab >> 32), 0u};
  bool same = true;
#pragma unroll
  for (int j = 0; j < 4; ++j) same = same && sig[j] == (uint32_t)__builtin_amdgcn_readfirstlane((int)sig[j]);
  const uint64_t here = __builtin_amdgcn_ballot_w64(true);
  // (the table's exponent field has six bits)
  if (__builtin_amdgcn_ballot_w64(!same || model.fs.etot > 63u) != 0ull)
    return ring_loop<false, kQueueOrder, kBusy, kFix>(s, model, lds, out, nullptr);
  // the table sits behind the records and tails of the wavefront's block; the
  // lanes that are here fill it together
  uint8_t* table = lds.aux - L::lane_term_tail(threadIdx.x) + L::kRecBytes + L::kTailBytes;
  const uint32_t lanes = (uint32_t)__builtin_popcountll(here);
  const uint32_t rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(here >> 32),
                                                  __builtin_amdgcn_mbcnt_lo((uint32_t)here, 0u));
  for (uint32_t i = rank; i < kRingTableEntries; i += lanes)
    ((uint16_t*)table)[i] = (uint16_t)ring_table_entry(i >> 3, i & 7u, model.state0(), full, fin_mask,
                                                       model.fs.epack, model.ranktab);
  // the stores of a wavefront reach the LDS in program order; the fence keeps
  // the compiler from moving the loop's reads above them
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  return ring_loop<true, kQueueOrder, kBusy, kFix>(s, model, lds, out, table);
}

}  // namespace themis
