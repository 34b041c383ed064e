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
// first" is a find-lowest-bit and a list pop: O(1) per chunk-stage event
// instead of a scan over all chunks.
//
// LDS layout: every lane owns kLaneWords dwords, stored transposed
// (dword d of lane L at word d*64 + L) so that the 64 lanes of a wavefront
// always hit 64 different banks, whatever per-lane index they use.
#pragma once

#include <type_traits>

#include "themis_device.hpp"

namespace themis {

struct LaneLds {
  uint8_t* base;  // LDS block of the wavefront + 4*lane
  uint8_t* aux;   // layouts with a second region (LayoutRing: the list tails)
  // byte address of dword d of this lane (transposed layout: 256 B apart)
  __device__ __forceinline__ uint8_t* dword(uint32_t d) const { return base + (d << 8); }
};

// Four small per-dimension counters packed in one register (pair).
template <typename Word, int kBits>
struct Pack4 {
  Word v = 0;
  static constexpr Word kMask = (Word(1) << kBits) - 1;
  static constexpr int kFieldBits = kBits;
  __device__ __forceinline__ uint32_t get(uint32_t k) const { return (uint32_t)((v >> (kBits * k)) & kMask); }
  __device__ __forceinline__ void inc(uint32_t k) { v += Word(1) << (kBits * k); }
  __device__ __forceinline__ uint32_t sum() const { return get(0) + get(1) + get(2) + get(3); }
};

// Which of a dimension's FIFO lists (one per size class) hold chunks: 16 classes
// per dimension, all four dimensions in one register pair.  List q = 16*k + class.
struct Classes16 {
  static constexpr uint32_t kPerDim = 16;
  uint64_t nonempty = 0;
  __device__ __forceinline__ explicit Classes16(const LaneLds&) {}
  // marks list q non-empty; returns whether it already was
  __device__ __forceinline__ bool mark(uint32_t q) {
    const uint64_t bit = 1ull << q;
    const bool had = (nonempty & bit) != 0ull;
    nonempty |= bit;
    return had;
  }
  // lowest non-empty class of dimension k (the caller knows there is one);
  // field: the lists of dimension k and above, for popped()
  __device__ __forceinline__ uint32_t lowest(uint32_t k, uint32_t& field) const {
    field = (uint32_t)(nonempty >> (16u * k));
    return (uint32_t)__builtin_ctz(field);
  }
  // list q = 16*k + cls lost its head chunk and is empty now if `emptied`;
  // returns whether no list of dimension k holds chunks any more
  __device__ __forceinline__ bool popped(uint32_t, uint32_t cls, uint32_t q, uint32_t field,
                                         bool emptied) {
    nonempty ^= (uint64_t)(emptied ? 1u : 0u) << q;  // the bit was set
    return ((field ^ ((emptied ? 1u : 0u) << cls)) & 0xffffu) == 0u;
  }
};

// Per-lane LDS layouts with 8-bit chunk ids (kChunks <= 128; 0xFF ends a list).
//
// Layout64 (80 dwords, 20 KiB per wavefront, 8 wavefronts per CU; the table
// layouts for other NPU counts build on it, power-of-two scenarios of up to 64
// chunks run on the ring layout of themis_ring.hpp instead):
//   dword c (0..63), one per chunk c AND per list q = 16*dim + class:
//     byte 0  chunk c: reduced-dims mask | phase << 4
//     byte 1  chunk c: next chunk in its list (0xFF = last)
//     byte 2  chunk c: order code
//     byte 3  list q: head chunk
//   dwords 64..79  u8 tail[64]: last chunk of list q
// LayoutByte<128> (144 dwords, 4 wavefronts per CU): the same with 128 chunk
// dwords, of which the first 64 carry the list heads.
// LayoutByte<16> (48 dwords, 12 KiB per wavefront, 13 wavefronts per CU; the
// kernel runs faster the more wavefronts share a SIMD): 16 chunk dwords with
// byte 3 unused, then u8 head[64] and u8 tail[64].
template <uint32_t kChunks>
struct LayoutByte {
  static constexpr bool kPacked = false;  // 32-bit chunk words, simulate_fast
  static constexpr uint32_t kCap = kChunks;
  static_assert(kChunks <= 128, "chunk ids and the list end mark share 8 bits");
  static constexpr bool kHeadInChunkWord = kChunks >= 64;
  static constexpr uint32_t kTailBase = kHeadInChunkWord ? kChunks : kChunks + 16;
  static constexpr uint32_t kLaneWords = kTailBase + 16;
  // wavefronts per SIMD that the LDS block allows (160 KiB per CU, 4 SIMDs,
  // rounded up): the kernels ask for a register budget that does not cap it lower
  static constexpr uint32_t kWavesPerSimd = (160u * 1024u / (kLaneWords * 256u) + 3u) / 4u;
  static constexpr uint32_t kEnd = 0xffu;
  using Link = uint8_t;               // width of a chunk id in LDS
  using Classes = Classes16;
  // per dimension: chunk id << 2 | dimension, and the operation count (up to 2 * kChunks)
  using Ids = typename std::conditional<(kChunks <= 64), Pack4<uint32_t, 8>, Pack4<uint64_t, 16>>::type;
  static __device__ __forceinline__ void init_chunk(const LaneLds& l, uint32_t c, uint32_t code,
                                                    uint32_t state0) {
    *(uint32_t*)l.dword(c) = (code << 16) | (kEnd << 8) | state0;
  }
  static __device__ __forceinline__ uint32_t code(uint32_t w) { return (w >> 16) & 0xffu; }
  static __device__ __forceinline__ uint32_t next(uint32_t w) { return (w >> 8) & 0xffu; }
  static __device__ __forceinline__ uint32_t code_of(const LaneLds& l, uint32_t c) {
    return l.dword(c)[2];
  }
  // new state of chunk c (whole dword w known), end of its list
  static __device__ __forceinline__ void store_state(uint8_t* cp, uint32_t, uint32_t state) {
    *(uint16_t*)cp = (uint16_t)(state | (kEnd << 8));
  }
  static __device__ __forceinline__ Link* next_ptr(const LaneLds& l, uint32_t c) { return l.dword(c) + 1; }
  static __device__ __forceinline__ Link* head_ptr(const LaneLds& l, uint32_t q) {
    if (kHeadInChunkWord) return l.dword(q) + 3;
    return l.base + ((kChunks + (q >> 2)) << 8) + (q & 3u);
  }
  static __device__ __forceinline__ Link* tail_ptr(const LaneLds& l, uint32_t q) {
    return l.base + ((kTailBase + (q >> 2)) << 8) + (q & 3u);
  }
};
using Layout64 = LayoutByte<64>;
using Layout16 = LayoutByte<16>;
using Layout128 = LayoutByte<128>;

// Per-evaluation constants of the fast path.
//
// Collective types share one machine.  A chunk's state is (mask of dimensions
// it is currently reduced on, phase); a Reduce-Scatter stage on k sets bit k,
// an All-Gather stage clears it, and the resident size is base * 2^-E(mask).
//   All-Reduce     : starts at (0, RS), base = chunk, ends when an AG stage
//                    empties the mask.
//   Reduce-Scatter : the same, but ends when the mask is full.
//   All-Gather     : starts at (full, AG) with base = chunk * 2^Etot, so the
//                    resident size starts at chunk and doubles back up; the
//                    AG half walks a code from its last field to its first,
//                    so the chunk words hold the order code reversed.
struct FastScenario {
  uint32_t epack;   // e_k = log2 P_k in byte k (0 for unused dimensions)
  uint32_t etot;    // sum of e_k
  double chunk;     // bytes per chunk (normal binary64, exponent > etot)
  double base;      // resident size at mask 0: chunk, or chunk * 2^etot for All-Gather
  uint32_t state0;  // initial mask | phase << 4
  bool rs_only;     // stand-alone Reduce-Scatter
  bool gather;      // stand-alone All-Gather
};

__device__ __forceinline__ bool is_pow2(uint32_t p) { return (p & (p - 1u)) == 0u; }

// x * 2^e for a normal x whose exponent stays in range.
__device__ __forceinline__ double scale_up(double x, uint32_t e) {
  int hi = __double2hiint(x) + (int)(e << 20);
  return __hiloint2double(hi, __double2loint(x));
}

// x * 2^-e for a normal x whose exponent stays in range (checked above).
__device__ __forceinline__ double scale_down(double x, uint32_t e) {
  int hi = __double2hiint(x) - (int)(e << 20);
  return __hiloint2double(hi, __double2loint(x));
}

// Sum of e_k over the dimensions in mask.
__device__ __forceinline__ uint32_t esum(uint32_t epack, uint32_t mask) {
  uint32_t spread = __umul24(mask, 0x00204081u) & 0x01010101u;  // bit k -> byte k (mask < 16)
  return __builtin_amdgcn_udot4(spread, epack, 0u, false);  // sum of byte products
}

// Can this scenario take the fast path?  Fills fs when it can.
__device__ __forceinline__ bool fast_eligible(const Scenario& s, double chunk, uint32_t cap,
                                              FastScenario& fs) {
  bool ok = s.valid && s.C <= cap;
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
  // every halving (doubling, for an All-Gather) must stay a normal number
  uint32_t ex = (uint32_t)((__double_as_longlong(chunk) >> 52) & 0x7ff);
  fs.gather = s.ctype == THEMIS_COLL_ALL_GATHER;
  fs.rs_only = s.ctype == THEMIS_COLL_REDUCE_SCATTER;
  ok = ok && ex < 0x7ffu && (fs.gather ? ex + et < 0x7ffu : ex > et);
  fs.epack = ep;
  fs.etot = et;
  fs.chunk = chunk;
  fs.base = fs.gather ? scale_up(chunk, ok ? et : 0u) : chunk;
  fs.state0 = fs.gather ? (((1u << s.D) - 1u) | 16u) : 0u;
  return ok;
}

// The order code as the chunk words hold it (see FastScenario).
__device__ __forceinline__ uint32_t stored_code(const Scenario& s, const FastScenario& fs,
                                                uint32_t code) {
  return fs.gather ? reverse_code(code, s.D) : code;
}

// Order code of the permutation of (0..D-1) with lexicographic index idx.
__device__ __forceinline__ uint32_t nth_permutation_code(uint32_t D, uint32_t idx) {
  uint32_t pool = 0x3210u;  // remaining dimensions, one nibble each, ascending
  uint32_t code = 0;
  uint32_t fact = D >= 4u ? 6u : D == 3u ? 2u : 1u;  // (D-1)!
  for (uint32_t j = 0; j < D; ++j) {
    const uint32_t pick = idx / fact;
    idx -= pick * fact;
    code |= ((pool >> (4u * pick)) & 3u) << (2u * j);
    pool = (pool & ((1u << (4u * pick)) - 1u)) | ((pool >> (4u * (pick + 1u))) << (4u * pick));
    const uint32_t left = D - 1u - j;
    if (left > 1u) fact /= left;
  }
  return code;
}

__device__ __forceinline__ uint32_t factorial_u32(uint32_t D) {
  return D >= 4u ? 24u : D == 3u ? 6u : D == 2u ? 2u : 1u;
}

// ---------------------------------------------------------------------------
// Planner (Alg. 1) with static register indexing.  emit(c, code) receives
// every chunk's order code; load[] holds the Dim Load Tracker on return.
// ---------------------------------------------------------------------------
// The ascending stable order of four loads is a function of the six
// comparisons load[a] > load[b] (a < b).  One table entry of eight dwords per
// outcome (bit 0: 0>1, 1: 0>2, 2: 0>3, 3: 1>2, 4: 1>3, 5: 2>3): dword k < 4
// holds the dimensions that come before dimension k, dimension j as a one in
// byte j (so that a byte-wise dot product with the packed exponents sums the
// exponents of those dimensions); dword 4 the order code of four dimensions.
constexpr uint32_t kPlanOrders = 64;
constexpr uint32_t kPlanOrderWords = 8;
__device__ __forceinline__ void plan_order_entry(uint32_t outcome, uint32_t* entry) {
  const bool after01 = (outcome & 1u) != 0u, after02 = (outcome & 2u) != 0u;
  const bool after03 = (outcome & 4u) != 0u, after12 = (outcome & 8u) != 0u;
  const bool after13 = (outcome & 16u) != 0u, after23 = (outcome & 32u) != 0u;
  // rank of a dimension: how many come before it
  const uint32_t r1 = (uint32_t)!after01 + after12 + after13;
  const uint32_t r2 = (uint32_t)!after02 + !after12 + after23;
  const uint32_t r3 = (uint32_t)!after03 + !after13 + !after23;
  entry[0] = (after01 ? 0x100u : 0u) | (after02 ? 0x10000u : 0u) | (after03 ? 0x1000000u : 0u);
  entry[1] = (after01 ? 0u : 1u) | (after12 ? 0x10000u : 0u) | (after13 ? 0x1000000u : 0u);
  entry[2] = (after02 ? 0u : 1u) | (after12 ? 0u : 0x100u) | (after23 ? 0x1000000u : 0u);
  entry[3] = (after03 ? 0u : 1u) | (after13 ? 0u : 0x100u) | (after23 ? 0u : 0x10000u);
  entry[4] = ((1u << (2u * r1)) | (2u << (2u * r2)) | (3u << (2u * r3))) & 0xffu;
  entry[5] = entry[6] = entry[7] = 0u;
}

// kTable: orders points to kPlanOrders entries of plan_order_entry() in LDS
// (16-byte aligned);
// the order and the sizes then come from one table read instead of the
// comparisons' arithmetic (the results are the same).
template <bool kTable = false, typename Emit>
__device__ __forceinline__ void plan_fast(const Scenario& s, const FastScenario& fs, bool themis,
                                          bool rel, double thr, double (&load)[kMaxDims],
                                          Emit emit, const uint32_t* orders = nullptr) {
  const int D = s.D;
  uint32_t e[kMaxDims];
  double coef[kMaxDims];
#pragma unroll
  for (int k = 0; k < kMaxDims; ++k) {
    e[k] = (fs.epack >> (8 * k)) & 0xffu;
    coef[k] = (k < D) ? s.coef[k] : 0.0;   // unused dimensions: zero time, load stays +inf
    load[k] = (k < D) ? tracker_start(s, k) : inf64();  // tracker starts at A_K
  }
  const uint32_t field_mask = (1u << (2 * D)) - 1u;
  for (uint32_t c = 0; c < s.C; ++c) {
    // least / most loaded dimension, ties to the lower index
    double lo = load[0], hi = load[0], cmin = coef[0];
    uint32_t emin = e[0];
#pragma unroll
    for (int k = 1; k < kMaxDims; ++k) {
      bool used = k < D;
      bool less = used && load[k] < lo;
      lo = less ? load[k] : lo;
      cmin = less ? coef[k] : cmin;
      emin = less ? e[k] : emin;
      hi = (used && load[k] > hi) ? load[k] : hi;
    }
    // a whole-chunk stage on the least-loaded dimension: an All-Gather moves
    // the grown size chunk * P
    const double whole = fs.gather ? scale_up(fs.chunk, emin) : fs.chunk;
    double t = rel ? thr * (whole * cmin) : thr;
    bool sort = themis && !((hi - lo) < t);
    // after[a][b] (a < b): does a come after b in the chosen order?
    // stable ascending sort: only when a's load is strictly larger.
    bool after01 = sort && load[0] > load[1], after02 = sort && load[0] > load[2];
    bool after03 = sort && load[0] > load[3], after12 = sort && load[1] > load[2];
    bool after13 = sort && load[1] > load[3], after23 = sort && load[2] > load[3];
    uint32_t code, E0, E1, E2, E3;
    if (kTable) {
      const uint32_t outcome = (after01 ? 1u : 0u) | (after02 ? 2u : 0u) | (after03 ? 4u : 0u) |
                               (after12 ? 8u : 0u) | (after13 ? 16u : 0u) | (after23 ? 32u : 0u);
      const uint32_t* entry = orders + kPlanOrderWords * outcome;
      const uint4 before = *(const uint4*)entry;
      code = entry[4] & field_mask;
      E0 = __builtin_amdgcn_udot4(before.x, fs.epack, 0u, false);
      E1 = __builtin_amdgcn_udot4(before.y, fs.epack, 0u, false);
      E2 = __builtin_amdgcn_udot4(before.z, fs.epack, 0u, false);
      E3 = __builtin_amdgcn_udot4(before.w, fs.epack, 0u, false);
    } else {
      // before[j][k]: j precedes k
      const bool b10 = after01, b20 = after02, b30 = after03;
      const bool b01 = !after01, b21 = after12, b31 = after13;
      const bool b02 = !after02, b12 = !after12, b32 = after23;
      const bool b03 = !after03, b13 = !after13, b23 = !after23;
      uint32_t r1 = (uint32_t)b01 + b21 + b31;
      uint32_t r2 = (uint32_t)b02 + b12 + b32, r3 = (uint32_t)b03 + b13 + b23;
      code = ((1u << (2 * r1)) | (2u << (2 * r2)) | (3u << (2 * r3))) & field_mask;
      // resident size before the Reduce-Scatter on k: chunk / prod of P_j, j before k
      E0 = (b10 ? e[1] : 0u) + (b20 ? e[2] : 0u) + (b30 ? e[3] : 0u);
      E1 = (b01 ? e[0] : 0u) + (b21 ? e[2] : 0u) + (b31 ? e[3] : 0u);
      E2 = (b02 ? e[0] : 0u) + (b12 ? e[1] : 0u) + (b32 ? e[3] : 0u);
      E3 = (b03 ? e[0] : 0u) + (b13 ? e[1] : 0u) + (b23 ? e[2] : 0u);
    }
    double t0, t1, t2, t3;
    if (fs.gather) {
      // the All-Gather visits the dimensions in the reverse order: the ones
      // after k in the ascending order are gathered before it, and its stage
      // moves the size grown by P_k as well:  E(after k) + e_k = etot - E(before k)
      code = reverse_code(code, D);
      t0 = scale_up(fs.chunk, fs.etot - E0) * coef[0];
      t1 = scale_up(fs.chunk, fs.etot - E1) * coef[1];
      t2 = scale_up(fs.chunk, fs.etot - E2) * coef[2];
      t3 = scale_up(fs.chunk, fs.etot - E3) * coef[3];
    } else {
      t0 = scale_down(fs.chunk, E0) * coef[0];
      t1 = scale_down(fs.chunk, E1) * coef[1];
      t2 = scale_down(fs.chunk, E2) * coef[2];
      t3 = scale_down(fs.chunk, E3) * coef[3];
    }
    if (s.ctype == THEMIS_COLL_ALL_REDUCE) {
      load[0] = load[0] + (t0 + t0);
      load[1] = load[1] + (t1 + t1);
      load[2] = load[2] + (t2 + t2);
      load[3] = load[3] + (t3 + t3);
    } else {
      load[0] = load[0] + t0;
      load[1] = load[1] + t1;
      load[2] = load[2] + t2;
      load[3] = load[3] + t3;
    }
    emit(c, code);
  }
}

// ---------------------------------------------------------------------------
// Queue simulation.
// ---------------------------------------------------------------------------
struct FastOut {
  // kStagedBytes: the lane's first byte inside its wavefront's staging block,
  // else this evaluation's [4][2*slots] entries; or null
  uint8_t* queue_order;
  uint32_t slots;
  uint32_t lane_offset = 0;  // kStagedBytes: added to every offset from queue_order
  uint32_t staging_bytes = 0;  // kStagedBytes: size of the staging block
};

struct FastResult {
  double t_done;
  double busy[kMaxDims];
  uint32_t executed[kMaxDims];  // operations each dimension ran
  bool ok;                      // false: leave the answer to the generic path
};

// Class (rank of the resident size) of every mask, 4 bits each: the number of
// masks with a strictly larger E, i.e. a strictly smaller resident size, so
// that the lowest non-empty class of a dimension holds its smallest chunks.
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
    for (uint32_t o = 0; o < 16; ++o) r += (E[o] > E[m]) ? 1u : 0u;
    tab |= (uint64_t)r << (4 * m);
  }
  return tab;
}

// Minimum of two doubles in one instruction (fmin() would first canonicalise
// both operands); of a quiet NaN and a number it returns the number.
__device__ __forceinline__ double min_f64(double a, double b) {
  double r;
  asm("v_min_f64 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}

// Dimension k (0..3, differing from lane to lane) starts a stage at `now`:
//   t = [fix_k +] x * coef_k   (start_stage_scaled)   or   t given (start_stage)
//   f_k = now + t   and, with kBusy,   z_k = z_k + t.
// Registers cannot be indexed by a lane's own k, and as selects this takes two
// per double and dimension (choosing coef_k, storing f_k, adding to z_k); here
// the lanes with k == j are made the active ones in turn, j = 0..3, and do
// their arithmetic on dimension j's registers directly.  The operations and
// their order are those of the plain code, so the results are bit-identical.
// The compiler does not look into these blocks: an instruction that reads
// other lanes (DPP, v_readlane, ...) must not follow the last v_cmpx within
// five wait states.  Every block therefore ends with at least five wait
// states of its own behind its last v_cmpx (the shorter variants are padded
// with a no-op), and is volatile so that it stays whole; build.py's
// exec_hazards() checks the compiled code on top of that.
#define THEMIS_LANES_OF(J) "v_cmpx_eq_u32_e32 vcc, " #J ", %[k]\n\t"
#define THEMIS_ALL_LANES "s_mov_b64 exec, %[act]\n\t"
#define THEMIS_FOUR(BODY) "s_mov_b64 %[act], exec\n\t" BODY(0) BODY(1) BODY(2) BODY(3)
#define THEMIS_MUL(J) "v_mul_f64 %[t], %[x], %[c" #J "]\n\t"
#define THEMIS_FIX(J) "v_add_f64 %[t], %[a" #J "], %[t]\n\t"
#define THEMIS_END(J) "v_add_f64 %[f" #J "], %[now], %[t]\n\t"
#define THEMIS_BUSY(J) "v_add_f64 %[z" #J "], %[z" #J "], %[t]\n\t"
#define THEMIS_SERVE(J) "v_mov_b32_e32 %[s" #J "], %[val]\n\t"

#define THEMIS_GIVEN(J) THEMIS_LANES_OF(J) THEMIS_END(J) THEMIS_SERVE(J) THEMIS_ALL_LANES
#define THEMIS_PAD1 "s_nop 0\n\t"
#define THEMIS_PAD2 "s_nop 1\n\t"
#define THEMIS_GIVEN_BUSY(J) \
  THEMIS_LANES_OF(J) THEMIS_END(J) THEMIS_BUSY(J) THEMIS_SERVE(J) THEMIS_ALL_LANES
#define THEMIS_SCALED(J) \
  THEMIS_LANES_OF(J) THEMIS_MUL(J) THEMIS_END(J) THEMIS_SERVE(J) THEMIS_ALL_LANES
#define THEMIS_SCALED_BUSY(J) \
  THEMIS_LANES_OF(J) THEMIS_MUL(J) THEMIS_END(J) THEMIS_BUSY(J) THEMIS_SERVE(J) THEMIS_ALL_LANES
#define THEMIS_SCALED_FIX(J) \
  THEMIS_LANES_OF(J) THEMIS_MUL(J) THEMIS_FIX(J) THEMIS_END(J) THEMIS_SERVE(J) THEMIS_ALL_LANES
#define THEMIS_SCALED_FIX_BUSY(J)                                                        \
  THEMIS_LANES_OF(J) THEMIS_MUL(J) THEMIS_FIX(J) THEMIS_END(J) THEMIS_BUSY(J) THEMIS_SERVE(J) \
  THEMIS_ALL_LANES

#define THEMIS_F_OPERANDS [f0] "+v"(d.f0), [f1] "+v"(d.f1), [f2] "+v"(d.f2), [f3] "+v"(d.f3)
#define THEMIS_Z_OPERANDS [z0] "+v"(d.z0), [z1] "+v"(d.z1), [z2] "+v"(d.z2), [z3] "+v"(d.z3)
#define THEMIS_S_OPERANDS [s0] "+v"(d.s0), [s1] "+v"(d.s1), [s2] "+v"(d.s2), [s3] "+v"(d.s3)
#define THEMIS_C_OPERANDS [c0] "v"(c[0]), [c1] "v"(c[1]), [c2] "v"(c[2]), [c3] "v"(c[3])
#define THEMIS_A_OPERANDS [a0] "v"(a[0]), [a1] "v"(a[1]), [a2] "v"(a[2]), [a3] "v"(a[3])

// What the event loop keeps per dimension, one register (pair) each.
struct DimState {
  double f0, f1, f2, f3;    // finish time of the running stage, a quiet NaN when idle
  double z0, z1, z2, z3;    // busy time
  uint32_t s0, s1, s2, s3;  // the running stage: chunk id << 2 | dimension
};

template <bool kBusy>
__device__ __forceinline__ void start_stage(uint32_t k, uint32_t val, double now, double t,
                                            DimState& d) {
  uint64_t act;  // the lanes that are here
  if (kBusy) {
    asm volatile(THEMIS_FOUR(THEMIS_GIVEN_BUSY) THEMIS_PAD1
        : [act] "=&s"(act), THEMIS_F_OPERANDS, THEMIS_S_OPERANDS, THEMIS_Z_OPERANDS
        : [k] "v"(k), [val] "v"(val), [now] "v"(now), [t] "v"(t) : "vcc");
  } else {
    asm volatile(THEMIS_FOUR(THEMIS_GIVEN) THEMIS_PAD2
        : [act] "=&s"(act), THEMIS_F_OPERANDS, THEMIS_S_OPERANDS
        : [k] "v"(k), [val] "v"(val), [now] "v"(now), [t] "v"(t) : "vcc");
  }
}

// c[]: per-byte latencies (coef), a[]: fixed delays per stage (used with kFix).
template <bool kBusy, bool kFix>
__device__ __forceinline__ void start_stage_scaled(uint32_t k, uint32_t val, double now, double x,
                                                   const double (&c)[kMaxDims],
                                                   const double (&a)[kMaxDims], DimState& d) {
  uint64_t act;
  double t;
  if (kBusy && kFix) {
    asm volatile(THEMIS_FOUR(THEMIS_SCALED_FIX_BUSY)
        : [act] "=&s"(act), [t] "=&v"(t), THEMIS_F_OPERANDS, THEMIS_S_OPERANDS, THEMIS_Z_OPERANDS
        : [k] "v"(k), [val] "v"(val), [now] "v"(now), [x] "v"(x), THEMIS_C_OPERANDS,
          THEMIS_A_OPERANDS : "vcc");
  } else if (kBusy) {
    asm volatile(THEMIS_FOUR(THEMIS_SCALED_BUSY)
        : [act] "=&s"(act), [t] "=&v"(t), THEMIS_F_OPERANDS, THEMIS_S_OPERANDS, THEMIS_Z_OPERANDS
        : [k] "v"(k), [val] "v"(val), [now] "v"(now), [x] "v"(x), THEMIS_C_OPERANDS : "vcc");
  } else if (kFix) {
    asm volatile(THEMIS_FOUR(THEMIS_SCALED_FIX)
        : [act] "=&s"(act), [t] "=&v"(t), THEMIS_F_OPERANDS, THEMIS_S_OPERANDS
        : [k] "v"(k), [val] "v"(val), [now] "v"(now), [x] "v"(x), THEMIS_C_OPERANDS,
          THEMIS_A_OPERANDS : "vcc");
  } else {
    asm volatile(THEMIS_FOUR(THEMIS_SCALED) THEMIS_PAD1
        : [act] "=&s"(act), [t] "=&v"(t), THEMIS_F_OPERANDS, THEMIS_S_OPERANDS
        : [k] "v"(k), [val] "v"(val), [now] "v"(now), [x] "v"(x), THEMIS_C_OPERANDS : "vcc");
  }
}

// The clock has moved to `now`: every dimension whose stage ends now becomes
// idle.  Returns the bits of those dimensions and, in `first`, the smallest
// chunk id << 2 | dimension among their stages (all-ones if there is none).
#define THEMIS_ENDS_NOW(J, BIT)                          \
  "v_cmpx_eq_f64_e32 vcc, %[now], %[f" #J "]\n\t"       \
  "v_mov_b64_e32 %[f" #J "], %[nan]\n\t"                \
  "v_min_u32_e32 %[first], %[first], %[s" #J "]\n\t"    \
  "v_or_b32_e32 %[done], " #BIT ", %[done]\n\t" THEMIS_ALL_LANES
template <typename Dims>
__device__ __forceinline__ uint32_t stages_ending(double now, Dims& d, uint32_t& first) {
  uint64_t act;
  uint32_t done = 0u;
  first = ~0u;
  asm volatile("s_mov_b64 %[act], exec\n\t"
      THEMIS_ENDS_NOW(0, 1) THEMIS_ENDS_NOW(1, 2) THEMIS_ENDS_NOW(2, 4) THEMIS_ENDS_NOW(3, 8) THEMIS_PAD1
      : [act] "=&s"(act), [done] "+v"(done), [first] "+v"(first), THEMIS_F_OPERANDS
      : [now] "v"(now), [nan] "v"(nan64()), [s0] "v"(d.s0), [s1] "v"(d.s1), [s2] "v"(d.s2),
        [s3] "v"(d.s3)
      : "vcc");
  return done;
}

// How the per-dimension queue orders leave the kernel.
// kBytes / kShorts store each 8- / 16-bit entry into the lane's own rows as
// it is produced.  kWords (8-bit entries) collects four entries per dimension
// in a register and stores them as one aligned dword (a quarter of the memory
// transactions); it needs rows that start on a 4-byte boundary (an even number
// of slots).  Either way every lane appends to its own four rows, so the
// stores of a wavefront never share a cache line.  kStagedBytes (8-bit
// entries, whole wavefronts) stores each entry into a staging order inside
// the wavefront's own block of the output, so that the entries the 64 lanes
// store at about the same time share cache lines; whoever asks for it puts
// the rows in place afterwards.  The order is the event loop's own: here dword
// w of lane L's rows (four entries) sits at byte (w * 64 + L) * 4, the ring
// loop keeps single bytes 64 apart (themis_ring.hpp).
enum QueueOrderMode { kNoQueueOrder = 0, kBytes = 1, kWords = 2, kShorts = 3, kStagedBytes = 4 };

// What the event loop needs to know about sizes and times, for scenarios with
// power-of-two NPU counts: the resident size is base * 2^-E(mask), so a stage
// time is one exponent adjustment and one multiply, and the size class of a
// mask comes from a 16 x 4-bit table in a register pair.
struct Pow2Model {
  const Scenario& s;
  const FastScenario& fs;
  uint64_t ranktab;
  __device__ __forceinline__ Pow2Model(const Scenario& s_, const FastScenario& fs_, bool scf)
      : s(s_), fs(fs_), ranktab(build_rank_table(fs_.epack, scf)) {}
  __device__ __forceinline__ uint32_t state0() const { return fs.state0; }
  __device__ __forceinline__ bool rs_only() const { return fs.rs_only; }
  __device__ __forceinline__ bool one_phase() const { return fs.rs_only || fs.gather; }
  // bits of the chunk's state byte that a state change must carry over
  __device__ __forceinline__ uint32_t keep(uint32_t) const { return 0u; }
  // time of the stage chunk word w is waiting for, on dimension k (kbit = 1 << k):
  // bytes moved on k = resident size before the chunk's Reduce-Scatter on k,
  // i.e. with every reduced dimension but k itself taken off; the All-Gather
  // reuses it (its mask still contains k)
  static constexpr bool kScaledProduct = true;  // stage time = stage_bytes() * coef[k]
  __device__ __forceinline__ double stage_bytes(uint32_t kbit, uint32_t w) const {
    return scale_down(fs.base, esum(fs.epack, w & 15u & ~kbit));
  }
  __device__ __forceinline__ double stage_time(uint32_t k, uint32_t kbit, uint32_t w) const {
    return stage_bytes(kbit, w) * sel4((int)k, s.coef[0], s.coef[1], s.coef[2], s.coef[3]);
  }
  // size class of a chunk (word w) once its state is (mask, phase)
  __device__ __forceinline__ uint32_t size_class(uint32_t, uint32_t mask, uint32_t) const {
    return (uint32_t)(ranktab >> (4u * mask)) & 15u;
  }
  // a lower bound of every stage time
  __device__ __forceinline__ double t_min(uint32_t D) const {
    double m = inf64();
#pragma unroll
    for (uint32_t k = 0; k < (uint32_t)kMaxDims; ++k) {
      const uint32_t ek = (fs.epack >> (8u * k)) & 0xffu;
      if (k < D) m = min_f64(m, scale_down(fs.base, fs.etot - ek) * s.coef[k]);
    }
    return m;
  }
};

// Chunk dwords must already be initialised with L::init_chunk().
// kFix: the batch carries fixed per-stage delays (a compile-time switch: even a
// wave-uniform run-time branch around the four-way selection cost 4 % on
// batches without delays).
// Model: Pow2Model or a type with the same members (sizes, times, classes).
template <typename L, int kQueueOrder, bool kBusy, bool kFix, typename Model>
__device__ __forceinline__ FastResult simulate_fast(const Scenario& s, const Model& model,
                                                    const LaneLds& lds, const FastOut& out) {
  using Link = typename L::Link;
  const uint32_t D = (uint32_t)s.D;
  const uint32_t C = s.C;
  const uint32_t full = (1u << D) - 1u;
  const double kInf = inf64();

  // an idle dimension's finish time is a quiet NaN: the minimum instruction
  // skips it, and no comparison with the clock holds
  DimState d;
  d.f0 = d.f1 = d.f2 = d.f3 = nan64();
  d.z0 = d.z1 = d.z2 = d.z3 = 0.0;
  d.s0 = d.s1 = d.s2 = d.s3 = 0u;
  typename L::Ids executed;  // operations started per dimension
  typename L::Classes classes(lds);  // which list q = kPerDim*dim + class holds chunks
  constexpr uint32_t kPerDim = L::Classes::kPerDim;
  uint32_t work = 0;      // bit k: some list of dimension k holds chunks
  uint32_t idle = full;   // bit k: dimension k serves nothing
  uint32_t a0 = 0, a1 = 0, a2 = 0, a3 = 0;  // kWords: last four queue entries per dimension
  const uint32_t row_len = 2u * out.slots;

  // append chunk c to list q (branch-free: an empty list takes c as its head,
  // otherwise the old tail's next field does)
  auto push = [&](uint32_t q, uint32_t c) {
    const bool had = classes.mark(q);
    Link* tp = L::tail_ptr(lds, q);
    uint32_t t = *tp;
    Link* dst = had ? L::next_ptr(lds, t) : L::head_ptr(lds, q);
    *dst = (Link)c;
    *tp = (Link)c;
    work |= 1u << (q / kPerDim);
  };

  // a6: every chunk waits at the dimension of its first stage, in chunk-id
  // order, in the class of the initial mask
  {
    const uint32_t mask0 = model.state0() & 15u, phase0 = (model.state0() >> 4) & 1u;
    const uint32_t pos0 = 2u * ((uint32_t)__builtin_popcount(mask0) - phase0);
    for (uint32_t c = 0; c < C; ++c) {
      const uint32_t w = *(const uint32_t*)lds.dword(c);
      push(kPerDim * ((L::code(w) >> pos0) & 3u) + model.size_class(w, mask0, phase0), c);
    }
  }

  double now = 0.0;
  // One pass starts at most one stage and, once no idle dimension has chunks
  // waiting, advances the clock to the next completion.  A lane that has to
  // start two stages at one instant takes two passes for it; the other lanes of
  // the wavefront go on with their own events meanwhile instead of waiting
  // through a second round of starts.
  const uint32_t max_steps = 4u * D * C + 16u;
  for (uint32_t step = 0; step <= max_steps; ++step) {
    // a7: an idle dimension with waiting chunks starts its first one
    if (const uint32_t need = idle & work) {
      const uint32_t k = (uint32_t)__builtin_ctz(need);
      // work bit k says that one of k's lists is non-empty
      uint32_t field;
      const uint32_t cls = classes.lowest(k, field);  // smallest resident size
      const uint32_t q = kPerDim * k + cls;
      Link* hp = L::head_ptr(lds, q);
      const uint32_t h = *hp;
      const uint32_t w = *(const uint32_t*)lds.dword(h);
      const uint32_t nx = L::next(w);
      *hp = (Link)nx;  // harmless when the list is now empty
      const bool emptied = nx == L::kEnd;
      const bool no_work = classes.popped(k, cls, q, field, emptied);
      work &= ~((no_work ? 1u : 0u) << k);
      const uint32_t kbit = 1u << k;
      idle &= ~kbit;

      const uint32_t phase = (w >> 4) & 1u;
      if constexpr (Model::kScaledProduct) {
        // t = bytes * coef_k, picked per lane inside
        start_stage_scaled<kBusy, kFix>(k, (h << 2) | k, now, model.stage_bytes(kbit, w), s.coef,
                                        s.fix, d);
      } else {
        double t = model.stage_time(k, kbit, w);
        if (kFix) t = sel4((int)k, s.fix[0], s.fix[1], s.fix[2], s.fix[3]) + t;
        start_stage<kBusy>(k, (h << 2) | k, now, t, d);
      }
      const bool k0 = k == 0u, k1 = k == 1u, k2 = k == 2u, k3 = k == 3u;
      if (kQueueOrder != kNoQueueOrder) {
        const uint32_t pos = executed.get(k);
        const uint32_t entry = (h << 1) | phase;
        // pos < row_len always holds for a consistent plan; it keeps the store in bounds
        if (kQueueOrder == kBytes) {
          if (pos < row_len) out.queue_order[k * row_len + pos] = (uint8_t)entry;
        } else if (kQueueOrder == kShorts) {
          if (pos < row_len) ((uint16_t*)out.queue_order)[k * row_len + pos] = (uint16_t)entry;
        } else if (kQueueOrder == kStagedBytes) {
          // byte pos & 3 of dword pos >> 2 of row k; consecutive dwords of a lane lie 256 bytes apart
          const uint32_t at = min(pos, row_len - 1u);  // pos < row_len for a consistent plan
          uint32_t word;  // k * dwords per row + at / 4 (a full-rate multiply-add)
          asm("v_mad_u32_u24 %0, %1, %2, %3" : "=v"(word) : "v"(k), "s"(out.slots >> 1), "v"(at >> 2));
          out.queue_order[((word << 8) | (at & 3u)) + out.lane_offset] = (uint8_t)entry;
        } else {
          // shift the entry in from the top: after four entries the register
          // holds them in memory (little-endian) order
          const uint32_t a = __builtin_amdgcn_alignbit(entry, sel4((int)k, a0, a1, a2, a3), 8u);
          a0 = k0 ? a : a0; a1 = k1 ? a : a1; a2 = k2 ? a : a2; a3 = k3 ? a : a3;
          if ((pos & 3u) == 3u && pos < row_len)
            ((uint32_t*)out.queue_order)[__umul24(k, out.slots >> 1) + (pos >> 2)] = a;
        }
      }
      executed.inc(k);
    }
    // all stages of an instant start before the clock moves
    if ((idle & work) != 0u) continue;

    // a8: advance to the earliest completion
    const double next = min_f64(min_f64(d.f0, d.f1), min_f64(d.f2, d.f3));
    if (!(next < kInf)) break;  // NaN: nothing running, every chunk is done (+inf: overflow)
    now = next;
    // deliver all completions of this instant, lowest chunk id first, so that
    // equal arrival times are appended in chunk-id order
    uint32_t key;
    uint32_t done = stages_ending(now, d, key);
    idle |= done;
    for (;;) {
      const uint32_t k = key & 3u;
      const uint32_t c = key >> 2;
      done &= ~(1u << k);
      uint8_t* cp = lds.dword(c);
      const uint32_t w = *(const uint32_t*)cp;
      const uint32_t code = L::code(w);
      uint32_t phase = (w >> 4) & 1u;
      // a Reduce-Scatter sets the dimension's bit, an All-Gather clears it
      const uint32_t mask = (w & 15u) ^ (1u << k);
      const bool finished = (phase != 0u && mask == 0u) || (model.rs_only() && mask == full);
      phase |= (mask == full) ? 1u : 0u;  // last Reduce-Scatter: All-Gather starts on the same dim
      if (!finished) {
        // next stage: RS -> order[#reduced], AG -> order[#reduced - 1]
        const uint32_t pos = (uint32_t)__builtin_popcount(mask) - phase;
        const uint32_t kn = (code >> (2u * pos)) & 3u;
        L::store_state(cp, w, mask | (phase << 4) | model.keep(w));
        push(kPerDim * kn + model.size_class(w, mask, phase), c);
      }
      if (done == 0u) break;
      // one more stage ends at this very instant (rare): the smallest one left
      key = min(min((done & 1u) ? d.s0 : ~0u, (done & 2u) ? d.s1 : ~0u),
                min((done & 4u) ? d.s2 : ~0u, (done & 8u) ? d.s3 : ~0u));
    }
  }

  if (kQueueOrder == kWords) {
    // entries that did not fill a whole dword yet, with unused-entry marks
    // (all-ones) behind them
    const uint32_t acc[kMaxDims] = {a0, a1, a2, a3};
#pragma unroll
    for (uint32_t k = 0; k < (uint32_t)kMaxDims; ++k) {
      const uint32_t n = executed.get(k);
      const uint32_t rem = n & 3u;
      if (rem != 0u && n < row_len)
        ((uint32_t*)out.queue_order)[__umul24(k, out.slots >> 1) + (n >> 2)] =
            (acc[k] >> (8u * (4u - rem))) | (0xffffffffu << (8u * rem));
    }
  }

  FastResult res;
  // The answer stands when every stage ran and completed and no stage was too
  // short to move the clock: each stage lasts at least t_min, the smallest
  // product over the dimensions, so `t_done + t_min / 4 > t_done` (t_min is
  // then at least two units in the last place of every earlier instant)
  // shows that each finish time was strictly after its start.  Anything else
  // (overflow to infinity, NaN, a vanishing stage) is left to the generic path.
  const double t_min = model.t_min(D);
  const uint32_t stages = model.one_phase() ? D : 2u * D;
  res.ok = executed.sum() == stages * C && idle == full && (now + 0.25 * t_min > now);
  res.t_done = now;
  res.busy[0] = d.z0; res.busy[1] = d.z1; res.busy[2] = d.z2; res.busy[3] = d.z3;
#pragma unroll
  for (uint32_t k = 0; k < (uint32_t)kMaxDims; ++k) res.executed[k] = executed.get(k);
  return res;
}

}  // namespace themis
