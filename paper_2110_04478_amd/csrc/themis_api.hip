// C ABI of the library (see include/themis.h) and the kernels behind it.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdlib>
#include <cstring>
#include <tuple>
#include <utility>

#include "themis.h"
#include "themis_device.hpp"
#include "themis_fast.hpp"
#include "themis_generic.hpp"
#include "themis_packed.hpp"
#include "themis_ring.hpp"
#include "themis_quad.hpp"
#include "themis_table.hpp"
#include "themis_trace.hpp"

// Scratch of themis_simulate_batch_noalloc: device memory the library itself
// brings along, one copy per GPU that loads the code object.  Host code never
// uses this name as an address; it asks the runtime for the array's device
// address once per device (scratch_of_current_device()).
static __device__ __align__(256) unsigned char scratch[THEMIS_STATIC_SCRATCH_BYTES];

namespace themis {

struct TraceView {
  bool on;
  uint32_t mc;     // collectives per scenario row (1 without a trace)
  uint32_t slots;  // chunk slots per scenario = max_chunks * mc
};

__host__ __device__ inline TraceView trace_view(const themis_batch_t& b) {
  TraceView t;
  t.on = b.n_coll != nullptr;
  t.mc = t.on ? b.max_coll : 1u;
  t.slots = b.max_chunks * t.mc;
  return t;
}

__device__ __forceinline__ double collective_size(const themis_batch_t& b, const TraceView& tv,
                                                  uint64_t i, uint32_t q) {
  return tv.on ? b.coll_size[(size_t)q * b.n + i] : b.size_bytes[i];
}

__device__ __forceinline__ double collective_release(const themis_batch_t& b, const TraceView& tv,
                                                     uint64_t i, uint32_t q) {
  return (tv.on && b.release_time) ? b.release_time[(size_t)q * b.n + i] : 0.0;
}

// Checks the collectives of scenario i (count, sizes, release times).
__device__ __forceinline__ bool collectives_ok(const themis_batch_t& b, const TraceView& tv,
                                               uint64_t i, uint32_t& Q) {
  Q = tv.on ? b.n_coll[i] : 1u;
  if (Q < 1u || Q > tv.mc) { Q = 0; return false; }
  bool ok = true;
  for (uint32_t q = 0; q < Q; ++q) {
    if (!finite_positive(collective_size(b, tv, i, q))) ok = false;
    double r = collective_release(b, tv, i, q);
    if (!(r >= 0.0 && r < inf64())) ok = false;
  }
  return ok;
}

__device__ __forceinline__ bool threshold_ok(double thr, bool rel) {
  return thr >= 0.0 && (!rel || thr < inf64());
}

// A completion time of this bit pattern (a NaN no computation produces) marks
// an evaluation that the LDS kernel leaves to the generic kernel launched
// right behind it.  Keeping the generic path out of the LDS kernels keeps its
// registers and scratch memory out of their budgets.
constexpr uint64_t kLeftToGeneric = 0x7ff8a5a55a5a0001ull;
__device__ __forceinline__ double left_to_generic() { return __longlong_as_double((long long)kLeftToGeneric); }
__device__ __forceinline__ bool is_left_to_generic(double t) {
  return (uint64_t)__double_as_longlong(t) == kLeftToGeneric;
}

// Every call that may hand evaluations over carries a number of its own (host
// counter, never 0); a kernel that marks one raises this word to its call's
// number, and the follow-up kernels of a call return at once while the word is
// below theirs -- then nothing of that call can be marked.  A larger number
// left by another call only costs the scan for marks.
__device__ unsigned long long g_marked_call = 0ull;
__device__ __forceinline__ void mark_left_to_generic(double* slot, unsigned long long call) {
  *slot = left_to_generic();
  atomicMax(&g_marked_call, call);
}
__device__ __forceinline__ bool nothing_marked(unsigned long long call) {
  return *(volatile unsigned long long*)&g_marked_call < call;
}

// ---------------------------------------------------------------------------
// themis_plan_batch: Alg. 1 per scenario (hot-path steps a1-a5).
// ---------------------------------------------------------------------------
// kPerCollective: one lane per (scenario, collective) instead of one per
// scenario -- the tracker starts afresh for every collective (Alg. 1 line 2),
// so the collectives of a trace are planned independently, and a batch of a
// few thousand traces has too few scenarios to fill the GPU.
template <bool kPerCollective>
__global__ void __launch_bounds__(kBlock)
plan_kernel(themis_batch_t b, uint8_t* __restrict__ orders, double* __restrict__ loads) {
  // the planner's order table, one entry per lane of the workgroup
  static_assert(kBlock == kPlanOrders, "one table entry per lane");
  __shared__ __attribute__((aligned(16))) uint32_t plan_orders[kPlanOrders * kPlanOrderWords];
  plan_order_entry(threadIdx.x, plan_orders + kPlanOrderWords * threadIdx.x);
  __syncthreads();
  const TraceView tv = trace_view(b);
  const uint64_t e = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
  const uint64_t i = kPerCollective ? e / tv.mc : e;
  if (i >= b.n) return;
  const uint32_t q_first = kPerCollective ? (uint32_t)(e - i * tv.mc) : 0u;
  const uint32_t q_end = kPerCollective ? q_first + 1u : tv.mc;
  Scenario s = load_scenario(b, i);
  const bool rel = b.threshold_mode == THEMIS_THR_REL;
  const double thr = b.threshold[i];
  const bool themis_on = b.inter_policy[i] != THEMIS_INTER_BASELINE;
  uint32_t Q;
  bool ok = collectives_ok(b, tv, i, Q) && s.valid && threshold_ok(thr, rel);

  uint8_t* row = orders + (size_t)i * tv.slots;
  double load[kMaxDims] = {0.0, 0.0, 0.0, 0.0};
  if (!ok) {
    for (uint32_t c = q_first * b.max_chunks; c < q_end * b.max_chunks; ++c) row[c] = 0xFFu;
  } else {
    // rows are written four codes at a time when they are 4-byte aligned
    const bool words = (b.max_chunks & 3u) == 0u;
    for (uint32_t q = q_first; q < q_end; ++q) {
      uint8_t* r = row + (size_t)q * b.max_chunks;
      uint32_t filled = 0;
      if (q < Q) {
        const double chunk = collective_size(b, tv, i, q) / (double)s.C;
        FastScenario fs;
        if (fast_eligible(s, chunk, THEMIS_MAX_CHUNKS, fs)) {
          uint32_t acc = 0;
          plan_fast<true>(s, fs, themis_on, rel, thr, load, [&](uint32_t c, uint32_t code) {
            if (words) {
              acc |= code << (8u * (c & 3u));
              if ((c & 3u) == 3u) { ((uint32_t*)r)[c >> 2] = acc; acc = 0; }
            } else {
              r[c] = (uint8_t)code;
            }
          }, plan_orders);
          if (words && (s.C & 3u)) {  // pad the last partial word with unused-slot marks
            acc |= 0xFFFFFFFFu << (8u * (s.C & 3u));
            ((uint32_t*)r)[s.C >> 2] = acc;
            filled = (s.C | 3u) + 1u;
          } else {
            filled = s.C;
          }
        } else {
#pragma unroll
          for (int k = 0; k < kMaxDims; ++k) load[k] = (k < s.D) ? tracker_start(s, k) : inf64();
          for (uint32_t c = 0; c < s.C; ++c)
            r[c] = (uint8_t)schedule_chunk(s, chunk, themis_on, rel, thr, load);
          filled = s.C;
        }
      }
      for (uint32_t c = filled; c < b.max_chunks; ++c) r[c] = 0xFFu;
    }
  }
  // the tracker of the scenario's last collective (an invalid scenario: NaN)
  if (loads && (!kPerCollective || q_first == (ok ? Q - 1u : 0u))) {
#pragma unroll
    for (int k = 0; k < kMaxDims; ++k)
      loads[(size_t)k * b.n + i] = ok ? ((k < s.D) ? load[k] : 0.0) : nan64();
  }
}

// ---------------------------------------------------------------------------
// themis_simulate_batch (hot-path steps a6-a9): LDS fast path, with the
// generic workspace path for the scenarios it does not cover.
// ---------------------------------------------------------------------------
// i: scenario; col: its column of the workspace arrays.
template <bool kEager>
__device__ __forceinline__ void simulate_generic_scenario(const themis_batch_t& b, const TraceView& tv,
                                                          const Scenario& s, uint32_t Q, uint64_t i,
                                                          uint64_t col, const uint8_t* row, bool scf,
                                                          const Workspace& w, const SimOut& out) {
  bool ok = true;
  bool has_release = false;
  // a6: every chunk waits at the dimension of its first stage
  for (uint32_t q = 0; q < Q; ++q) {
    double chunk = collective_size(b, tv, i, q) / (double)s.C;
    double rel = collective_release(b, tv, i, q);
    has_release |= rel > 0.0;
    for (uint32_t c = 0; c < s.C; ++c) {
      uint32_t code = row[(size_t)q * b.max_chunks + c];
      if (!order_code_ok(code, s.D)) ok = false;
      size_t at = (size_t)(q * s.C + c) * w.stride + col;
      w.meta[at] = code << 8;
      w.size[at] = chunk;
      w.arrival[at] = rel;
    }
  }
  if (!ok) { write_invalid(out); return; }
  simulate_generic<kEager>(
      s, Q, scf, w, col,
      [&](uint32_t q) { return collective_size(b, tv, i, q) / (double)s.C; },
      [&](uint32_t q) { return collective_release(b, tv, i, q); }, has_release, out);
}

// This lane's view of its wavefront's LDS block.
template <typename L>
__device__ __forceinline__ LaneLds lane_lds(uint32_t* lds_block) {
  LaneLds lds;
  if constexpr (IsRing<L>::value) {
    lds.base = (uint8_t*)lds_block + L::lane_term_rec(threadIdx.x);
    lds.aux = (uint8_t*)lds_block + L::lane_term_tail(threadIdx.x);
  } else {
    lds.base = (uint8_t*)lds_block + 4u * threadIdx.x;
    lds.aux = nullptr;
  }
  return lds;
}

// Chunk c's word / record in the lane's LDS block, whichever the layout keeps.
template <typename L>
__device__ __forceinline__ void init_chunk(const LaneLds& lds, uint32_t c, uint32_t code,
                                           uint32_t state0, uint32_t D) {
  if constexpr (L::kPacked) L::init_chunk(lds, c, code, state0, D);
  else L::init_chunk(lds, c, code, state0);
}

// The power-of-two event loop that goes with the layout.
template <typename L, int kQueueOrder, bool kBusy, bool kFix>
__device__ __forceinline__ FastResult simulate_pow2(const Scenario& s, const Pow2Model& model,
                                                    const LaneLds& lds, const FastOut& out) {
  if constexpr (IsRing<L>::value) {
    // entries leave one by one: collected dwords become single bytes
    constexpr int kMode = kQueueOrder == kWords ? (int)kBytes : kQueueOrder;
    return simulate_ring<kMode, kBusy, kFix>(s, model, lds, out);
  } else if constexpr (L::kPacked) {
    return simulate_packed<L, kQueueOrder, kBusy, kFix>(s, model, lds, out);
  } else {
    return simulate_fast<L, kQueueOrder, kBusy, kFix, Pow2Model>(s, model, lds, out);
  }
}

template <int kQueueOrder>
__device__ __forceinline__ void put_queue_entry(uint8_t* rows, uint32_t at, uint32_t v) {
  if (kQueueOrder == kShorts) ((uint16_t*)rows)[at] = (uint16_t)v;
  else rows[at] = (uint8_t)v;
}

template <typename L, int kQueueOrder, bool kBusy, bool kFix>
__global__ void __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(L::kWavesPerSimd)))
simulate_kernel(themis_batch_t b, const uint8_t* __restrict__ orders,
                double* __restrict__ t_done, void* __restrict__ queue_order, int entry_bytes,
                double* __restrict__ busy, unsigned long long hand_over) {
  __shared__ uint32_t lds_block[L::kLaneWords * kBlock];
  uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i >= b.n) return;
  const TraceView tv = trace_view(b);
  Scenario s = load_scenario(b, i);
  const bool scf = b.intra_policy[i] == THEMIS_INTRA_SCF;
  uint32_t Q;
  bool ok = collectives_ok(b, tv, i, Q) && s.valid;

  // Queue orders of a wavefront whose 64 scenarios all exist are staged
  // transposed inside the wavefront's own block of the output (kStagedBytes)
  // and put in place once the wavefront is through: a lane appends an entry to
  // one of its four rows at every event, and with the rows in place the
  // partly written lines of all resident wavefronts do not fit the L2, so they
  // go to memory several times over.
  // dwords per row that the last step holds in registers (a row has up to
  // kCap / 2).  Up to 64 chunks: with the four wavefronts per CU of the
  // 128-chunk layout the rows written in place do better (3.14 against 3.44 ms
  // for 262,144 scenarios of 126 chunks).
  constexpr uint32_t kStagedWords = L::kCap / 2u < 32u ? L::kCap / 2u : 32u;
  const uint32_t rows_bytes = (uint32_t)kMaxDims * 2u * tv.slots * (uint32_t)entry_bytes;
  const bool staged = kQueueOrder == kWords && queue_order != nullptr &&
                      (tv.slots >> 1) <= kStagedWords &&
                      (uint64_t)(blockIdx.x + 1u) * kBlock <= b.n;  // the same for all lanes
  enum { kRowsStaged = 1, kRowsAllOnes = 2, kRowsNotMine = 3 };
  uint32_t rows = kRowsNotMine;
  uint32_t executed[kMaxDims] = {0u, 0u, 0u, 0u};

  SimOut out;
  out.t_done = t_done + i;
  out.busy = busy ? busy + i : nullptr;
  out.busy_stride = b.n;
  out.entry_bytes = entry_bytes;
  out.slots = tv.slots;
  out.queue_order = (kQueueOrder != kNoQueueOrder && queue_order)
      ? (void*)((uint8_t*)queue_order + (size_t)i * rows_bytes) : nullptr;
  // an invalid scenario: NaN / all-ones (its rows at the end, if rows are staged in the block)
  auto invalid = [&]() {
    SimOut o = out;
    if (staged) o.queue_order = nullptr;
    write_invalid(o);
    rows = kRowsAllOnes;
  };

  do {
    if (!ok) { invalid(); break; }
    const uint8_t* row = orders + (size_t)i * tv.slots;
    FastScenario fs;
    bool fast = !tv.on &&
                fast_eligible(s, collective_size(b, tv, i, 0) / (double)s.C, L::kCap, fs);
    if (fast) {
      const LaneLds lds = lane_lds<L>(lds_block);
      // order codes -> chunk words (mask 0, Reduce-Scatter phase)
      bool codes_ok = true;
      if ((tv.slots & 3u) == 0u) {
        const uint32_t* row4 = (const uint32_t*)row;
        for (uint32_t c4 = 0; c4 < s.C; c4 += 4u) {
          uint32_t v = row4[c4 >> 2];
#pragma unroll
          for (uint32_t j = 0; j < 4u; ++j) {
            if (c4 + j < s.C) {
              uint32_t code = (v >> (8u * j)) & 0xffu;
              codes_ok = codes_ok && order_code_ok(code, s.D);
              init_chunk<L>(lds, c4 + j, stored_code(s, fs, code), fs.state0, (uint32_t)s.D);
            }
          }
        }
      } else {
        for (uint32_t c = 0; c < s.C; ++c) {
          uint32_t code = row[c];
          codes_ok = codes_ok && order_code_ok(code, s.D);
          init_chunk<L>(lds, c, stored_code(s, fs, code), fs.state0, (uint32_t)s.D);
        }
      }
      if (!codes_ok) { invalid(); break; }
      FastOut fo;
      fo.queue_order = (uint8_t*)out.queue_order;
      fo.slots = tv.slots;
      // staged: the same address for all lanes plus a 32-bit offset
      FastOut so;
      so.queue_order = (uint8_t*)queue_order + (size_t)blockIdx.x * kBlock * rows_bytes;
      so.slots = tv.slots;
      so.lane_offset = IsRing<L>::value ? threadIdx.x : 4u * threadIdx.x;
      so.staging_bytes = (uint32_t)kBlock * rows_bytes;
      FastResult r;
      if constexpr (kQueueOrder == kWords && !L::kPacked) {
        r = staged ? simulate_pow2<L, kStagedBytes, kBusy, kFix>(s, Pow2Model(s, fs, scf), lds, so)
                   : simulate_pow2<L, kWords, kBusy, kFix>(s, Pow2Model(s, fs, scf), lds, fo);
      } else {
        r = simulate_pow2<L, kQueueOrder, kBusy, kFix>(s, Pow2Model(s, fs, scf), lds, fo);
      }
      if (r.ok) {
        t_done[i] = r.t_done;
        if (busy) {
#pragma unroll
          for (int k = 0; k < kMaxDims; ++k) busy[(size_t)k * b.n + i] = r.busy[k];
        }
        if (staged) {
          rows = kRowsStaged;
#pragma unroll
          for (int k = 0; k < kMaxDims; ++k) executed[k] = r.executed[k];
        } else if (kQueueOrder != kNoQueueOrder && out.queue_order) {
          for (int k = 0; k < kMaxDims; ++k)
            for (uint32_t e = r.executed[k]; e < 2u * tv.slots; ++e)
              put_queue_entry<kQueueOrder>(fo.queue_order, (uint32_t)k * 2u * tv.slots + e, 0xFFFFu);
        }
        break;
      }
    }
    // hand_over != 0: follow-up kernels come (this call's number) and write
    // everything of this scenario, else nothing can take it
    if (!hand_over) { invalid(); break; }
    mark_left_to_generic(t_done + i, hand_over);
  } while (false);

  if constexpr (kQueueOrder == kWords) {
    if (staged) {
      // every lane fetches its own rows from the staging order (64 lanes read
      // 256 contiguous bytes per dword), waits until the whole wavefront has
      // all of them in registers, and writes them where they belong, with
      // all-ones from the first unused entry on
      const uint32_t wpr = tv.slots >> 1;  // dwords per row
      // the entries a lane fetches were stored by other lanes of its wavefront
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
      const uint32_t* from =
          (const uint32_t*)((uint8_t*)queue_order + (size_t)blockIdx.x * kBlock * rows_bytes) + threadIdx.x;
      uint32_t q[kMaxDims][kStagedWords];
      if constexpr (IsRing<L>::value) {
        // the ring loop stages single bytes, entry j of a row at byte 64 * j +
        // lane: the four lanes of a quad fetch the dwords of entries 4w .. 4w+3
        // (one each, the quad's four bytes of that entry) and exchange them, a
        // 4 x 4 byte transpose inside the quad
        const uint32_t sub = threadIdx.x & 3u;
        const uint32_t* from4 = (const uint32_t*)((uint8_t*)queue_order +
                                                  (size_t)blockIdx.x * kBlock * rows_bytes) +
                                sub * 16u + (threadIdx.x >> 2);
        // byte `sub` of the first operand's dword into byte 0, of the second's into byte 1
        const uint32_t pick = sub * 0x0101u + 0x0400u;
#pragma unroll
        for (uint32_t k = 0; k < (uint32_t)kMaxDims; ++k)
#pragma unroll
          for (uint32_t w = 0; w < kStagedWords; ++w)
            q[k][w] = w < wpr ? from4[(size_t)(k * wpr + w) * kBlock] : 0xffffffffu;
        // (the wait states a lane-crossing read asks for after a change of exec)
        asm volatile("s_waitcnt vmcnt(0)\n\ts_nop 4" ::: "memory");
#pragma unroll
        for (uint32_t k = 0; k < (uint32_t)kMaxDims; ++k)
#pragma unroll
          for (uint32_t w = 0; w < kStagedWords; ++w) {
            // lane a of the quad holds entry 4w + a: everybody takes byte `sub`
            // of all four.  One block per dword, three temporaries: left to the
            // compiler, the 128 dwords and its temporaries no longer fit the
            // registers of three wavefronts per SIMD.
            uint32_t t0, t1, t2;
            asm volatile(
                "v_mov_b32_dpp %[t0], %[q] quad_perm:[0,0,0,0] row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
                "v_mov_b32_dpp %[t1], %[q] quad_perm:[1,1,1,1] row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
                "v_mov_b32_dpp %[t2], %[q] quad_perm:[2,2,2,2] row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
                "v_perm_b32 %[t0], %[t1], %[t0], %[pick]\n\t"
                "v_mov_b32_dpp %[t1], %[q] quad_perm:[3,3,3,3] row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
                "v_perm_b32 %[t1], %[t1], %[t2], %[pick]\n\t"
                "v_perm_b32 %[q], %[t1], %[t0], %[join]"
                : [q] "+v"(q[k][w]), [t0] "=&v"(t0), [t1] "=&v"(t1), [t2] "=&v"(t2)
                : [pick] "v"(pick), [join] "s"(0x05040100u));
            if (rows != kRowsStaged) q[k][w] = 0xffffffffu;
          }
      } else {
#pragma unroll
        for (uint32_t k = 0; k < (uint32_t)kMaxDims; ++k)
#pragma unroll
          for (uint32_t w = 0; w < kStagedWords; ++w)
            q[k][w] = (w < wpr && rows == kRowsStaged) ? from[(size_t)(k * wpr + w) * kBlock] : 0xffffffffu;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      }
      if (rows != kRowsNotMine) {
        uint32_t* to = (uint32_t*)((uint8_t*)queue_order + (size_t)i * rows_bytes);
        // four dwords per store where the rows allow it: a quarter of the
        // memory transactions of this step
        const bool quads = (wpr & 3u) == 0u && ((uintptr_t)queue_order & 15u) == 0u;
        // rows without an unused entry (every dimension ran all 2 * slots
        // operations: an All-Reduce of `slots` chunks on four dimensions) need no marks
        bool full_rows = rows == kRowsStaged;
#pragma unroll
        for (uint32_t k = 0; k < (uint32_t)kMaxDims; ++k) full_rows = full_rows && executed[k] == 2u * tv.slots;
        const bool marks = __builtin_amdgcn_ballot_w64(!full_rows) != 0ull;  // the same for all lanes
#pragma unroll
        for (uint32_t k = 0; k < (uint32_t)kMaxDims; ++k)
#pragma unroll
          for (uint32_t w4 = 0; w4 < kStagedWords; w4 += 4u) {
            uint32_t v[4];
#pragma unroll
            for (uint32_t j = 0; j < 4u; ++j) {
              const uint32_t w = w4 + j;
              v[j] = w < kStagedWords ? q[k][w] : 0xffffffffu;
              if (marks) {
                // entries of this dword that are in use, 0..4; all-ones above them
                const int left = min(max((int)executed[k] - (int)(4u * w), 0), 4);
                v[j] |= (uint32_t)(0xffffffffull << (8 * left));
              }
            }
            if (quads) {
              if (w4 < wpr) *(uint4*)(to + k * wpr + w4) = make_uint4(v[0], v[1], v[2], v[3]);
            } else {
#pragma unroll
              for (uint32_t j = 0; j < 4u; ++j)
                if (w4 + j < wpr) to[k * wpr + w4 + j] = v[j];
            }
          }
      }
    }
  }
}

// Second kernel of themis_simulate_batch: the scenarios the LDS kernel marked.
// kLdsSlots > 0: the per-chunk arrays (20 bytes per chunk) live in LDS, laid
// out like the workspace with the 64 lanes as columns; for batches of at most
// kLdsSlots chunk slots per scenario, which then need no workspace at all.
// LDS a generic pass needs for kLdsSlots chunk slots per lane, in bytes.
constexpr size_t generic_lds_bytes(uint32_t lds_slots) {
  return lds_slots ? (size_t)((lds_slots * kBlock * 5u + 1u) / 2u) * sizeof(double) : 0u;
}

template <uint32_t kLdsSlots>
__device__ __forceinline__ void simulate_generic_pass(
    const themis_batch_t& b, const uint8_t* __restrict__ orders, double* __restrict__ t_done,
    void* __restrict__ queue_order, int entry_bytes, double* __restrict__ busy, Workspace w,
    void* lds_block) {
  if (kLdsSlots) w = carve_workspace(lds_block, kBlock, kLdsSlots);
  const TraceView tv = trace_view(b);
  // a few workgroups walk all groups of 64 scenarios: most groups have nothing marked
  const uint64_t groups = (b.n + kBlock - 1) / kBlock;
  for (uint64_t grp = blockIdx.x; grp < groups; grp += gridDim.x) {
    const uint64_t i = grp * kBlock + threadIdx.x;
    if (i >= b.n || !is_left_to_generic(t_done[i])) continue;
    const uint64_t col = kLdsSlots ? threadIdx.x : i;
    Scenario s = load_scenario(b, i);
    const bool scf = b.intra_policy[i] == THEMIS_INTRA_SCF;
    uint32_t Q;
    collectives_ok(b, tv, i, Q);  // marked scenarios passed this check already
    SimOut out;
    out.t_done = t_done + i;
    out.busy = busy ? busy + i : nullptr;
    out.busy_stride = b.n;
    out.entry_bytes = entry_bytes;
    out.slots = tv.slots;
    out.queue_order = queue_order
        ? (void*)((uint8_t*)queue_order + (size_t)i * kMaxDims * 2u * tv.slots * entry_bytes)
        : nullptr;
    // beyond the LDS variant's chunk count the arrays need the caller's workspace
    if (!kLdsSlots && !w.meta) { write_invalid(out); continue; }
    simulate_generic_scenario<(kLdsSlots > 0)>(b, tv, s, Q, i, col, orders + (size_t)i * tv.slots,
                                               scf, w, out);
  }
}

template <uint32_t kLdsSlots>
__global__ void __launch_bounds__(kBlock)
simulate_generic_kernel(themis_batch_t b, const uint8_t* __restrict__ orders,
                        double* __restrict__ t_done, void* __restrict__ queue_order,
                        int entry_bytes, double* __restrict__ busy, Workspace w,
                        unsigned long long call) {
  __shared__ double lds_block[kLdsSlots ? generic_lds_bytes(kLdsSlots) / sizeof(double) : 1u];
  if (nothing_marked(call)) return;
  simulate_generic_pass<kLdsSlots>(b, orders, t_done, queue_order, entry_bytes, busy, w, lds_block);
}

// Kernels between the two: marked scenarios whose NPU counts are not powers of
// two run the same LDS event loop on per-order-code tables (themis_table.hpp),
// first the variant for at most 8 distinct order codes, then (kWide) the one
// for any number of them; what they cannot take stays marked for the generic
// kernel.
// kVariant: 0 tables for at most 8 order codes (64 chunks), 1 any number of
// codes (64 chunks), 2 the same for up to 128 chunks, 3 and 4 16-bit chunk
// records for up to 256 and 512 chunks.
template <int kVariant>
struct TableVariant {
  using L = typename std::conditional<kVariant == 0, LayoutTable,
            typename std::conditional<kVariant == 1, LayoutTableWide,
            typename std::conditional<kVariant == 2, LayoutTableWide128,
            typename std::conditional<kVariant == 3, LayoutTablePacked<256>,
                                      LayoutTablePacked<512>>::type>::type>::type>::type;
};

template <int kQueueOrder, int kVariant>
__device__ __forceinline__ void simulate_table_pass(
    const themis_batch_t& b, const uint8_t* __restrict__ orders, double* __restrict__ t_done,
    void* __restrict__ queue_order, double* __restrict__ busy, void* lds_block) {
  using L = typename TableVariant<kVariant>::L;
  constexpr bool kWide = kVariant != 0;
  constexpr uint32_t kEntryBytes = kQueueOrder == kShorts ? 2u : 1u;
  const uint64_t groups = (b.n + kBlock - 1) / kBlock;
  for (uint64_t grp = blockIdx.x; grp < groups; grp += gridDim.x) {
    const uint64_t i = grp * kBlock + threadIdx.x;
    if (i >= b.n || !is_left_to_generic(t_done[i])) continue;
    Scenario s = load_scenario(b, i);
    const double S = b.size_bytes[i];
    if (!s.valid || s.C > L::kCap || !finite_positive(S)) continue;
    const uint8_t* row = orders + (size_t)i * b.max_chunks;
    bool codes_ok = true;
    for (uint32_t c = 0; c < s.C; ++c) codes_ok = codes_ok && order_code_ok(row[c], s.D);
    if (!codes_ok) continue;
    LaneLds lds;
    lds.base = (uint8_t*)lds_block + 4u * threadIdx.x;
    const bool scf = b.intra_policy[i] == THEMIS_INTRA_SCF;
    const double chunk = S / (double)s.C;
    auto code_at = [&](uint32_t c) { return (uint32_t)row[c]; };
    const uint32_t rows_bytes = (uint32_t)kMaxDims * 2u * b.max_chunks * kEntryBytes;
    FastOut fo;
    fo.queue_order = (kQueueOrder != kNoQueueOrder && queue_order)
        ? (uint8_t*)queue_order + (size_t)i * rows_bytes : nullptr;
    fo.slots = b.max_chunks;
    FastResult r;
    if constexpr (kVariant >= 3) {
      DivModelT<LayoutTableWide> model(s, lds, chunk, scf);
      table_setup_packed<L>(s, scf, lds, code_at, model);
      r = simulate_table_packed<L, kQueueOrder, true>(s, model, lds, fo);
    } else if constexpr (kWide) {
      DivModelT<L> model(s, lds, chunk, scf);
      table_setup_wide<L>(s, scf, lds, code_at, model);
      r = simulate_fast<L, kQueueOrder, true, true>(s, model, lds, fo);
    } else {
      TableModel model;
      if (!table_setup(s, chunk, scf, lds, code_at, model)) continue;
      r = simulate_fast<L, kQueueOrder, true, true>(s, model, lds, fo);
    }
    if (!r.ok) continue;
    t_done[i] = r.t_done;
    if (busy) {
#pragma unroll
      for (int k = 0; k < kMaxDims; ++k) busy[(size_t)k * b.n + i] = r.busy[k];
    }
    if (kQueueOrder != kNoQueueOrder && fo.queue_order) {
      for (int k = 0; k < kMaxDims; ++k)
        for (uint32_t e = r.executed[k]; e < 2u * b.max_chunks; ++e)
          put_queue_entry<kQueueOrder>(fo.queue_order, (uint32_t)k * 2u * b.max_chunks + e, 0xFFFFu);
    }
  }
}

constexpr size_t max_bytes(size_t a, size_t b) { return a > b ? a : b; }
template <int kVariant>
constexpr size_t table_lds_bytes() {
  if constexpr (kVariant < 0) return 0u;
  else return (size_t)TableVariant<kVariant>::L::kLaneWords * kBlock * sizeof(uint32_t);
}
constexpr uint32_t kNoGeneric = 0xffffffffu;

// Everything that follows the LDS kernel of themis_simulate_batch, in one
// launch: the table passes kTableA and kTableB (-1: none) and the generic pass
// (kGeneric: its chunk slots in LDS, 0: arrays in the workspace, kNoGeneric:
// none).  A workgroup walks the same groups of 64 scenarios in every pass, so
// what one pass leaves marked is seen by the next without any ordering between
// workgroups; the passes share one LDS block of the largest size among them.
template <int kQueueOrder, int kTableA, int kTableB, uint32_t kGeneric>
__global__ void __launch_bounds__(kBlock)
simulate_follow_up_kernel(themis_batch_t b, const uint8_t* __restrict__ orders,
                          double* __restrict__ t_done, void* __restrict__ queue_order,
                          int entry_bytes, double* __restrict__ busy, Workspace w,
                          unsigned long long call) {
  constexpr size_t kBytes_ = max_bytes(max_bytes(table_lds_bytes<kTableA>(), table_lds_bytes<kTableB>()),
                                       kGeneric == kNoGeneric ? 0u : generic_lds_bytes(kGeneric));
  __shared__ double lds_block[kBytes_ ? (kBytes_ + 7u) / 8u : 1u];
  if (nothing_marked(call)) return;
  if constexpr (kTableA >= 0)
    simulate_table_pass<kQueueOrder, kTableA>(b, orders, t_done, queue_order, busy, lds_block);
  if constexpr (kTableB >= 0) {
    __syncthreads();
    simulate_table_pass<kQueueOrder, kTableB>(b, orders, t_done, queue_order, busy, lds_block);
  }
  if constexpr (kGeneric != kNoGeneric) {
    __syncthreads();
    simulate_generic_pass<kGeneric>(b, orders, t_done, queue_order, entry_bytes, busy, w, lds_block);
  }
}

// ---------------------------------------------------------------------------
// themis_simulate_batch for traces (several collectives sharing the queues):
// the ranked-list path of themis_trace.hpp, else the generic path.
// ---------------------------------------------------------------------------
// kExtras: the batch carries release times or fixed delays (one switch for
// both keeps the number of variants down).
template <bool kLdsBitmaps, bool kExtras>
__global__ void __launch_bounds__(kBlock)
simulate_trace_kernel(themis_batch_t b, const uint8_t* __restrict__ orders,
                      double* __restrict__ t_done, void* __restrict__ queue_order,
                      int entry_bytes, double* __restrict__ busy, Workspace w, bool have_ws,
                      uint8_t* __restrict__ trace_area, TraceLayout tl) {
  __shared__ uint32_t lds_block[(kLdsBitmaps ? kTraceLdsWordsBitmaps : kTraceLdsWords) * kBlock];
  uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i >= b.n) return;
  const TraceView tv = trace_view(b);
  Scenario s = load_scenario(b, i);
  const bool scf = b.intra_policy[i] == THEMIS_INTRA_SCF;
  uint32_t Q;
  bool ok = collectives_ok(b, tv, i, Q) && s.valid;

  SimOut out;
  out.t_done = t_done + i;
  out.busy = busy ? busy + i : nullptr;
  out.busy_stride = b.n;
  out.entry_bytes = entry_bytes;
  out.slots = tv.slots;
  out.queue_order = queue_order
      ? (void*)((uint8_t*)queue_order + (size_t)i * kMaxDims * 2u * tv.slots * entry_bytes)
      : nullptr;
  if (!ok) { write_invalid(out); return; }

  const uint8_t* row = orders + (size_t)i * tv.slots;
  bool fast = trace_area != nullptr && tl.bytes != 0u && Q <= tl.Q;
  uint32_t epack = 0;
  FastScenario fs0;
  fs0.state0 = 0u; fs0.rs_only = false; fs0.gather = false;
  if (fast) {
    TraceRegion rg;
    rg.base = trace_area + (size_t)i * tl.bytes;
    rg.t = tl;
    // Every collective in the range where halvings are exact: sizes by
    // exponent arithmetic.  Otherwise (NPU counts that are not powers of two)
    // one division at a time, with size ranks per (dimension, phase, order)
    // under Smallest-Chunk-First as long as they fit the lists.
    bool has_release = false, divide = false;
    for (uint32_t q = 0; q < Q; ++q) {
      const double chunk = collective_size(b, tv, i, q) / (double)s.C;
      divide = divide || !fast_eligible(s, chunk, THEMIS_MAX_CHUNKS, fs0);
    }
    // (division mode ranks every (phase, order) of a dimension: more lists than the masks of halving mode)
    fast = fast && (!divide || !scf ||
                    Q * trace_division_lists((uint32_t)s.D, s.ctype != THEMIS_COLL_ALL_REDUCE) <= tl.R);
    for (uint32_t q = 0; q < Q; ++q) {
      const double chunk = collective_size(b, tv, i, q) / (double)s.C;
      fast_eligible(s, chunk, THEMIS_MAX_CHUNKS, fs0);   // (collective type, initial state; base and epack if exact)
      epack = fs0.epack;
      rg.CH(q) = divide ? chunk : fs0.base;  // resident size at mask 0
      if (kExtras) {
        const double release = collective_release(b, tv, i, q);
        rg.REL(q) = release;
        has_release = has_release || release > 0.0;
      }
    }
    bool codes_ok = true;
    if (fast) {
      for (uint32_t q = 0; q < Q; ++q)
        for (uint32_t c = 0; c < s.C; ++c) {
          const uint32_t code = row[(size_t)q * b.max_chunks + c];
          codes_ok = codes_ok && order_code_ok(code, s.D);
          rg.W(q * s.C + c) = trace_word(stored_code(s, fs0, code), fs0.state0);
        }
      if (!codes_ok) { write_invalid(out); return; }
      LaneLds lds;
      lds.base = (uint8_t*)lds_block + 4u * threadIdx.x;
      double T, z[kMaxDims];
      uint32_t ex[kMaxDims];
      // All-Reduces under one policy on one kind of NPU counts get a loop
      // compiled for exactly that when the whole wavefront is in the case
      const bool all_reduce = __builtin_amdgcn_ballot_w64(fs0.rs_only || fs0.state0 != 0u) == 0ull;
      const uint64_t lanes_scf = __builtin_amdgcn_ballot_w64(scf);
      const uint64_t lanes_divide = __builtin_amdgcn_ballot_w64(divide);
      const uint64_t lanes = __builtin_amdgcn_ballot_w64(true);
      int known = kTraceAnyLane;
      if (all_reduce && (lanes_scf == 0ull || lanes_scf == lanes) &&
          (lanes_divide == 0ull || lanes_divide == lanes))
        known = (lanes_scf ? kTraceKnownScf : 0) | (lanes_divide ? kTraceKnownDivide : 0);
      bool done;
#define THEMIS_TRACE_RUN(KNOWN)                                                                  \
  done = simulate_trace_fast<kLdsBitmaps, kExtras, kExtras, kExtras, KNOWN>(                     \
      s, Q, epack, fs0.state0, fs0.rs_only, scf, divide, has_release, rg, lds, out, T, z, ex)
      switch (known) {
        case 0: THEMIS_TRACE_RUN(0); break;
        case kTraceKnownScf: THEMIS_TRACE_RUN(kTraceKnownScf); break;
        case kTraceKnownDivide: THEMIS_TRACE_RUN(kTraceKnownDivide); break;
        case kTraceKnownScf | kTraceKnownDivide: THEMIS_TRACE_RUN(kTraceKnownScf | kTraceKnownDivide); break;
        default: THEMIS_TRACE_RUN(kTraceAnyLane); break;
      }
#undef THEMIS_TRACE_RUN
      if (done) {
        t_done[i] = T;
        if (busy) {
#pragma unroll
          for (int k = 0; k < kMaxDims; ++k) busy[(size_t)k * b.n + i] = z[k];
        }
        if (out.queue_order) {
          for (int k = 0; k < kMaxDims; ++k)
            for (uint32_t e = ex[k]; e < 2u * tv.slots; ++e) put_entry(out, k, e, 0xFFFFu);
        }
        return;
      }
    }
  }
  if (!have_ws) { write_invalid(out); return; }
  simulate_generic_scenario<false>(b, tv, s, Q, i, i, row, scf, w, out);
}

// ---------------------------------------------------------------------------
// themis_sweep (hot-path step a10): one lane per scenario x threshold x
// scheduler; the plan goes straight into LDS and only the time leaves.
// ---------------------------------------------------------------------------
template <bool kEager>
__device__ __forceinline__ void sweep_generic_evaluation(const Scenario& s, double chunk,
                                                         bool themis_on, bool rel, double th,
                                                         bool scf, uint64_t e, const Workspace& w,
                                                         const SimOut& out) {
  double load[kMaxDims];
#pragma unroll
  for (int k = 0; k < kMaxDims; ++k) load[k] = (k < s.D) ? tracker_start(s, k) : inf64();
  for (uint32_t c = 0; c < s.C; ++c) {
    uint32_t code = schedule_chunk(s, chunk, themis_on, rel, th, load);
    size_t at = (size_t)c * w.stride + e;
    w.meta[at] = code << 8;
    w.size[at] = chunk;
    w.arrival[at] = 0.0;
  }
  simulate_generic<kEager>(
      s, 1u, scf, w, e, [&](uint32_t) { return chunk; }, [&](uint32_t) { return 0.0; }, false,
      out);
}

// What one lane of a sweep evaluates.
struct SweepItem {
  uint64_t i;      // scenario
  double th;       // threshold
  bool themis_on;  // Themis or baseline order
  bool scf;        // Smallest-Chunk-First or FIFO
};

__device__ __forceinline__ SweepItem sweep_item(const themis_batch_t& b, uint64_t e, int n_thr,
                                                const double* thr, int thr_per_scenario,
                                                unsigned policy_mask, int n_pol) {
  SweepItem it;
  it.i = e / ((uint64_t)n_thr * n_pol);
  const uint32_t rem = (uint32_t)(e - it.i * (uint64_t)n_thr * n_pol);
  const int a = (int)(rem / (uint32_t)n_pol);
  const int col = (int)(rem - (uint32_t)a * (uint32_t)n_pol);
  // col-th set bit of the mask selects the scheduler
  int bit = 0;
  for (int seen = 0; bit < 3; ++bit)
    if (policy_mask & (1u << bit)) { if (seen == col) break; ++seen; }
  it.themis_on = bit != 0;
  it.scf = bit == 2;
  it.th = thr_per_scenario ? thr[(size_t)a * b.n + it.i] : thr[a];
  return it;
}

// The baseline order does not look at Alg. 1's threshold, so its column of a
// sweep needs one simulation per scenario, under the first threshold; the
// result is stored under every threshold.  A group of scenarios therefore has
// one workgroup per (threshold, scheduler) pair except the baseline's pairs
// beyond the first threshold: sweep_roles() of them.
__host__ __device__ __forceinline__ uint32_t sweep_roles(uint32_t n_thr, uint32_t n_pol,
                                                         unsigned policy_mask) {
  return n_thr * n_pol - ((policy_mask & THEMIS_SWEEP_BASELINE) ? n_thr - 1u : 0u);
}
// The pair a workgroup takes, as threshold * n_pol + column: the roles in turn,
// starting one further with every group (consecutive workgroups go to
// consecutive XCDs, and the number of roles is often a multiple of the eight
// XCDs: without the shift every XCD would see the same schedulers for every
// group, and they differ in cost).  Every workgroup of the grid has work, so
// the XCDs fill evenly -- workgroups are handed out in order, and a grid in
// which every eighth one returns at once keeps an eighth of the GPU idle.
__device__ __forceinline__ uint32_t sweep_block_role(uint32_t block, uint32_t n_thr, uint32_t n_pol,
                                                     unsigned policy_mask) {
  const uint32_t roles = sweep_roles(n_thr, n_pol, policy_mask);
  const uint32_t group = block / roles;
  const uint32_t r = (block - group * roles + group) % roles;
  if (!(policy_mask & THEMIS_SWEEP_BASELINE) || r < n_pol) return r;
  const uint32_t beyond = r - n_pol, others = n_pol - 1u;   // (others >= 1: r >= n_pol exists)
  return (1u + beyond / others) * n_pol + 1u + beyond % others;
}

// Stores the baseline's result under every threshold (NaN where that
// threshold itself is not valid).  e: the evaluation of the first threshold.
__device__ __forceinline__ void sweep_store_for_all_thresholds(
    const themis_batch_t& b, uint64_t i, uint64_t e, int n_thr, const double* thr,
    int thr_per_scenario, int n_pol, bool rel, double* t_done, double value,
    unsigned long long hand_over) {
  for (int a = 0; a < n_thr; ++a) {
    const double th = thr_per_scenario ? thr[(size_t)a * b.n + i] : thr[a];
    double* at = t_done + e + (uint64_t)a * (uint64_t)n_pol;
    if (!threshold_ok(th, rel)) *at = nan64();
    else if (hand_over) mark_left_to_generic(at, hand_over);
    else *at = value;
  }
}

// kBaseline: the sweep has a baseline column (compiled apart: what that
// column keeps alive across the event loop costs the other columns time).
template <typename L, bool kFix, bool kBaseline>
__global__ void __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(L::kWavesPerSimd)))
sweep_kernel(themis_batch_t b, int n_thr, const double* __restrict__ thr, int thr_per_scenario,
             unsigned policy_mask, int n_pol, double* __restrict__ t_done,
             unsigned long long hand_over) {
  __shared__ uint32_t lds_block[L::kLaneWords * kBlock];
  // A wavefront takes 64 consecutive scenarios under one threshold and one
  // scheduler: its lanes read consecutive inputs, and on a batch that keeps to
  // one network they all take the same path through the event loop.
  const uint32_t per = (uint32_t)n_thr * (uint32_t)n_pol;   // evaluations per scenario
  const uint32_t roles = sweep_roles((uint32_t)n_thr, (uint32_t)n_pol, policy_mask);
  const uint64_t i = (uint64_t)(blockIdx.x / roles) * kBlock + threadIdx.x;
  if (i >= b.n) return;
  const uint64_t e = i * per + sweep_block_role(blockIdx.x, (uint32_t)n_thr, (uint32_t)n_pol, policy_mask);
  const SweepItem it = sweep_item(b, e, n_thr, thr, thr_per_scenario, policy_mask, n_pol);
  const bool every_threshold = kBaseline && !it.themis_on;   // (the same for the whole wavefront)

  Scenario s = load_scenario(b, it.i);
  s.ctype = THEMIS_COLL_ALL_REDUCE;  // sweeps evaluate All-Reduce only
  const bool rel = b.threshold_mode == THEMIS_THR_REL;
  const double S = b.size_bytes[it.i];
  const bool input_ok = s.valid && finite_positive(S);
  if (every_threshold) {
    if (!input_ok) {
      for (int a = 0; a < n_thr; ++a) t_done[e + (uint64_t)a * (uint64_t)n_pol] = nan64();
      return;
    }
  } else if (!(input_ok && threshold_ok(it.th, rel))) {
    t_done[e] = nan64();
    return;
  }

  const double chunk = S / (double)s.C;
  FastScenario fs;
  if (fast_eligible(s, chunk, L::kCap, fs)) {
    const LaneLds lds = lane_lds<L>(lds_block);
    double load[kMaxDims];
    plan_fast(s, fs, it.themis_on, rel, it.th, load,
              [&](uint32_t c, uint32_t code) { init_chunk<L>(lds, c, code, 0u, (uint32_t)s.D); });
    FastOut fo;
    fo.queue_order = nullptr;
    fo.slots = b.max_chunks;
    // times only
    FastResult r =
        simulate_pow2<L, kNoQueueOrder, false, kFix>(s, Pow2Model(s, fs, it.scf), lds, fo);
    if (r.ok) {
      if (every_threshold)
        sweep_store_for_all_thresholds(b, it.i, e, n_thr, thr, thr_per_scenario, n_pol, rel, t_done,
                                       r.t_done, 0ull);
      else t_done[e] = r.t_done;
      return;
    }
  }
  if (every_threshold)
    sweep_store_for_all_thresholds(b, it.i, e, n_thr, thr, thr_per_scenario, n_pol, rel, t_done,
                                   nan64(), hand_over);
  else if (hand_over) mark_left_to_generic(t_done + e, hand_over);
  else t_done[e] = nan64();
}

// The same with four lanes per evaluation (themis_quad.hpp): a wavefront takes
// 16 consecutive scenarios under one threshold and one scheduler.
template <bool kFix, bool kBaseline>
__global__ void __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(LayoutQuad::kWavesPerSimd)))
sweep_quad_kernel(themis_batch_t b, int n_thr, const double* __restrict__ thr, int thr_per_scenario,
                  unsigned policy_mask, int n_pol, double* __restrict__ t_done,
                  unsigned long long hand_over) {
  using L = LayoutQuad;
  __shared__ uint32_t lds_block[L::kBlockWords];
  const uint32_t per = (uint32_t)n_thr * (uint32_t)n_pol;   // evaluations per scenario
  const uint32_t roles = sweep_roles((uint32_t)n_thr, (uint32_t)n_pol, policy_mask);
  const uint32_t quad = threadIdx.x >> 2;
  const uint64_t i = (uint64_t)(blockIdx.x / roles) * L::kQuads + quad;
  // a quad without a scenario stays: the wavefront leaves the event loop as a whole
  const bool exists = i < b.n;
  const uint64_t e = (exists ? i : 0u) * per +
                     sweep_block_role(blockIdx.x, (uint32_t)n_thr, (uint32_t)n_pol, policy_mask);
  const SweepItem it = sweep_item(b, e, n_thr, thr, thr_per_scenario, policy_mask, n_pol);
  const bool writer = exists && (threadIdx.x & 3u) == 0u;   // one lane of the quad stores the result
  const bool every_threshold = kBaseline && !it.themis_on;   // (the same for the whole wavefront)

  Scenario s = load_scenario(b, it.i);
  s.ctype = THEMIS_COLL_ALL_REDUCE;  // sweeps evaluate All-Reduce only
  const bool rel = b.threshold_mode == THEMIS_THR_REL;
  const double S = b.size_bytes[it.i];
  const bool ok = s.valid && finite_positive(S) && (every_threshold || threshold_ok(it.th, rel));
  const double chunk = S / (double)s.C;
  FastScenario fs;
  const bool eligible = fast_eligible(s, chunk, L::kCap, fs);
  // (a quad without a valid scenario only keeps the others company: no chunks, no events)
  const bool fast = exists && ok && eligible;
  uint8_t* base = (uint8_t*)lds_block + 2u * quad;
  if (fast) {
    // every lane of the quad plans (the same arithmetic, the same result) and
    // writes the records of the chunks whose id ends in its own two bits
    double load[kMaxDims];
    plan_fast(s, fs, it.themis_on, rel, it.th, load, [&](uint32_t c, uint32_t code) {
      if ((c & 3u) == (threadIdx.x & 3u)) L::init_chunk(base, c, code, 0u, (uint32_t)s.D);
    });
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
  const QuadResult r = simulate_quad<kFix>(s, Pow2Model(s, fs, it.scf), base, fast);
  if (!writer) return;
  if (every_threshold) {
    if (!ok) {
      for (int a = 0; a < n_thr; ++a) t_done[e + (uint64_t)a * (uint64_t)n_pol] = nan64();
    } else {
      const bool have = fast && r.ok;
      sweep_store_for_all_thresholds(b, it.i, e, n_thr, thr, thr_per_scenario, n_pol, rel, t_done,
                                     have ? r.t_done : nan64(), have ? 0ull : hand_over);
    }
    return;
  }
  if (!ok) t_done[e] = nan64();
  else if (fast && r.ok) t_done[e] = r.t_done;
  else if (hand_over) mark_left_to_generic(t_done + e, hand_over);
  else t_done[e] = nan64();
}

// The generic pass of themis_sweep: the evaluations still marked (kLdsSlots
// as in simulate_generic_pass).
template <uint32_t kLdsSlots>
__device__ __forceinline__ void sweep_generic_pass(
    const themis_batch_t& b, int n_thr, const double* __restrict__ thr, int thr_per_scenario,
    unsigned policy_mask, int n_pol, double* __restrict__ t_done, Workspace w, void* lds_block) {
  if (kLdsSlots) w = carve_workspace(lds_block, kBlock, kLdsSlots);
  const uint64_t total = b.n * (uint64_t)n_thr * (uint64_t)n_pol;
  const uint64_t groups = (total + kBlock - 1) / kBlock;
  for (uint64_t grp = blockIdx.x; grp < groups; grp += gridDim.x) {
    const uint64_t e = grp * kBlock + threadIdx.x;
    if (e >= total || !is_left_to_generic(t_done[e])) continue;
    const uint64_t col = kLdsSlots ? threadIdx.x : e;
    const SweepItem it = sweep_item(b, e, n_thr, thr, thr_per_scenario, policy_mask, n_pol);
    Scenario s = load_scenario(b, it.i);
    s.ctype = THEMIS_COLL_ALL_REDUCE;
    SimOut out;
    out.t_done = t_done + e;
    out.busy = nullptr;
    out.busy_stride = 0;
    out.queue_order = nullptr;
    out.entry_bytes = 1;
    out.slots = b.max_chunks;
    if (!kLdsSlots && !w.meta) { t_done[e] = nan64(); continue; }
    sweep_generic_evaluation<(kLdsSlots > 0)>(s, b.size_bytes[it.i] / (double)s.C, it.themis_on,
                                              b.threshold_mode == THEMIS_THR_REL, it.th, it.scf,
                                              col, w, out);
  }
}

template <uint32_t kLdsSlots>
__global__ void __launch_bounds__(kBlock)
sweep_generic_kernel(themis_batch_t b, int n_thr, const double* __restrict__ thr,
                     int thr_per_scenario, unsigned policy_mask, int n_pol,
                     double* __restrict__ t_done, Workspace w, unsigned long long call) {
  __shared__ double lds_block[kLdsSlots ? generic_lds_bytes(kLdsSlots) / sizeof(double) : 1u];
  if (nothing_marked(call)) return;
  sweep_generic_pass<kLdsSlots>(b, n_thr, thr, thr_per_scenario, policy_mask, n_pol, t_done, w,
                                lds_block);
}

// The same for themis_sweep: Alg. 1 with real divisions straight into the
// chunk words, then the table-driven event loop.
template <int kVariant>
__device__ __forceinline__ void sweep_table_pass(
    const themis_batch_t& b, int n_thr, const double* __restrict__ thr, int thr_per_scenario,
    unsigned policy_mask, int n_pol, double* __restrict__ t_done, void* lds_block) {
  using L = typename TableVariant<kVariant>::L;
  constexpr bool kWide = kVariant != 0;
  const uint64_t total = b.n * (uint64_t)n_thr * (uint64_t)n_pol;
  const uint64_t groups = (total + kBlock - 1) / kBlock;
  for (uint64_t grp = blockIdx.x; grp < groups; grp += gridDim.x) {
    const uint64_t e = grp * kBlock + threadIdx.x;
    if (e >= total || !is_left_to_generic(t_done[e])) continue;
    const SweepItem it = sweep_item(b, e, n_thr, thr, thr_per_scenario, policy_mask, n_pol);
    Scenario s = load_scenario(b, it.i);
    s.ctype = THEMIS_COLL_ALL_REDUCE;
    if (s.C > L::kCap) continue;
    const double chunk = b.size_bytes[it.i] / (double)s.C;
    const bool rel = b.threshold_mode == THEMIS_THR_REL;
    LaneLds lds;
    lds.base = (uint8_t*)lds_block + 4u * threadIdx.x;
    double load[kMaxDims];
#pragma unroll
    for (int k = 0; k < kMaxDims; ++k) load[k] = (k < s.D) ? tracker_start(s, k) : inf64();
    auto code_at = [&](uint32_t) { return schedule_chunk(s, chunk, it.themis_on, rel, it.th, load); };
    FastOut fo;
    fo.queue_order = nullptr;
    fo.slots = b.max_chunks;
    FastResult r;
    if constexpr (kVariant >= 3) {
      DivModelT<LayoutTableWide> model(s, lds, chunk, it.scf);
      table_setup_packed<L>(s, it.scf, lds, code_at, model);
      r = simulate_table_packed<L, kNoQueueOrder, false>(s, model, lds, fo);
    } else if constexpr (kWide) {
      DivModelT<L> model(s, lds, chunk, it.scf);
      table_setup_wide<L>(s, it.scf, lds, code_at, model);
      r = simulate_fast<L, kNoQueueOrder, false, true>(s, model, lds, fo);
    } else {
      TableModel model;
      if (!table_setup(s, chunk, it.scf, lds, code_at, model)) continue;
      r = simulate_fast<L, kNoQueueOrder, false, true>(s, model, lds, fo);
    }
    if (r.ok) t_done[e] = r.t_done;
  }
}

// Everything that follows the LDS kernel of themis_sweep, in one launch (see
// simulate_follow_up_kernel).
template <int kTableA, int kTableB, uint32_t kGeneric>
__global__ void __launch_bounds__(kBlock)
sweep_follow_up_kernel(themis_batch_t b, int n_thr, const double* __restrict__ thr,
                       int thr_per_scenario, unsigned policy_mask, int n_pol,
                       double* __restrict__ t_done, Workspace w, unsigned long long call) {
  constexpr size_t kBytes_ = max_bytes(max_bytes(table_lds_bytes<kTableA>(), table_lds_bytes<kTableB>()),
                                       kGeneric == kNoGeneric ? 0u : generic_lds_bytes(kGeneric));
  __shared__ double lds_block[kBytes_ ? (kBytes_ + 7u) / 8u : 1u];
  if (nothing_marked(call)) return;
  if constexpr (kTableA >= 0)
    sweep_table_pass<kTableA>(b, n_thr, thr, thr_per_scenario, policy_mask, n_pol, t_done, lds_block);
  if constexpr (kTableB >= 0) {
    __syncthreads();
    sweep_table_pass<kTableB>(b, n_thr, thr, thr_per_scenario, policy_mask, n_pol, t_done, lds_block);
  }
  if constexpr (kGeneric != kNoGeneric) {
    __syncthreads();
    sweep_generic_pass<kGeneric>(b, n_thr, thr, thr_per_scenario, policy_mask, n_pol, t_done, w,
                                 lds_block);
  }
}

// ---------------------------------------------------------------------------
// themis_sweep_best: per scenario and scheduler the best threshold of a sweep
// and the speed-up over the baseline (Sec. 5.3, Sec. 6.1).  One lane per
// (scenario, scheduler).
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
sweep_best_kernel(uint64_t n, uint32_t n_thr, uint32_t n_pol, const double* __restrict__ t_done,
                  int baseline_col, double* __restrict__ best_t, uint32_t* __restrict__ best_thr,
                  double* __restrict__ speedup) {
  const uint64_t e = (uint64_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= n * n_pol) return;
  const uint64_t i = e / n_pol;
  const uint32_t p = (uint32_t)(e - i * n_pol);
  const double* row = t_done + i * n_thr * n_pol;
  double best = nan64();
  uint32_t at = 0xffffffffu;
  for (uint32_t a = 0; a < n_thr; ++a) {
    const double t = row[(size_t)a * n_pol + p];
    // the first value that is not NaN, then every strictly smaller one
    if (t == t && (at == 0xffffffffu || t < best)) { best = t; at = a; }
  }
  best_t[e] = best;
  if (best_thr) best_thr[e] = at;
  if (speedup && baseline_col >= 0) speedup[e] = row[baseline_col] / best;
}

// ---------------------------------------------------------------------------
// themis_search_batch: every assignment of dimension orders to chunks.
// ---------------------------------------------------------------------------
// (D!)^C if it does not exceed bound, else 0.
__device__ __forceinline__ uint64_t assignment_count(uint32_t D, uint32_t C, uint64_t bound) {
  const uint64_t F = factorial_u32(D);
  uint64_t total = 1;
  for (uint32_t c = 0; c < C; ++c) {
    if (total > bound / F) return 0;
    total *= F;
  }
  return total;
}

// One lane per (scenario, assignment): times[i * max_assign + a].  Slots past
// a scenario's own count hold +inf; NaN marks a scenario that cannot be searched.
// kTable (L = LayoutTableWide): the follow-up kernel for the scenarios whose
// NPU counts are not powers of two, on per-order tables: the first kernel
// marks their slots (see g_marked_call), this one strides over all slots with
// a grid that just fills the device and returns at once if nothing is marked.
template <bool kTable, typename L, bool kFix>
__global__ void __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(L::kWavesPerSimd)))
search_eval_kernel(themis_batch_t b, uint64_t max_assign, double* __restrict__ times,
                   unsigned long long call) {
  __shared__ uint32_t lds_block[L::kLaneWords * kBlock];
  if (kTable && nothing_marked(call)) return;
  const uint64_t total = b.n * max_assign;
  for (uint64_t e = (uint64_t)blockIdx.x * kBlock + threadIdx.x; e < total;
       e += (uint64_t)gridDim.x * kBlock) {
  if (kTable && !is_left_to_generic(times[e])) continue;
  const uint64_t i = e / max_assign;
  const uint64_t a = e - i * max_assign;
  Scenario s = load_scenario(b, i);
  const bool scf = b.intra_policy[i] == THEMIS_INTRA_SCF;
  const double S = b.size_bytes[i];
  const double chunk = S / (double)s.C;
  FastScenario fs;
  const bool valid = s.valid && finite_positive(S) && s.C <= 64u;
  const bool pow2 = valid && fast_eligible(s, chunk, 64u, fs);   // (the same in both kernels)
  const uint64_t count = valid ? assignment_count((uint32_t)s.D, s.C, max_assign) : 0;
  if (count == 0) { times[e] = nan64(); continue; }
  if (a >= count) { times[e] = inf64(); continue; }
  if (!kTable && !pow2) { mark_left_to_generic(times + e, call); continue; }
  const uint32_t F = factorial_u32((uint32_t)s.D);
  // digit c of the assignment number, base D!
  auto code_at = [&](uint32_t c) {
    uint64_t rest = a;
    for (uint32_t j = 0; j < c; ++j) rest /= F;
    return nth_permutation_code((uint32_t)s.D, (uint32_t)(rest % F));
  };
  FastOut fo;
  fo.queue_order = nullptr;
  fo.slots = b.max_chunks;
  FastResult r;
  if constexpr (kTable) {
    LaneLds lds;
    lds.base = (uint8_t*)lds_block + 4u * threadIdx.x;
    DivModelT<L> model(s, lds, chunk, scf);
    table_setup_wide<L>(s, scf, lds, code_at, model);
    r = simulate_fast<L, kNoQueueOrder, false, true>(s, model, lds, fo);
  } else {
    const LaneLds lds = lane_lds<L>(lds_block);
    uint64_t rest = a;
    for (uint32_t c = 0; c < s.C; ++c) {
      const uint64_t q = rest / F;
      const uint32_t digit = (uint32_t)(rest - q * F);
      rest = q;
      L::init_chunk(lds, c, stored_code(s, fs, nth_permutation_code((uint32_t)s.D, digit)),
                    fs.state0);
    }
    r = simulate_pow2<L, kNoQueueOrder, false, kFix>(s, Pow2Model(s, fs, scf), lds, fo);
  }
  times[e] = r.ok ? r.t_done : nan64();
  }
}

// One wavefront per scenario: smallest time and the lowest assignment number
// that reaches it.
__global__ void __launch_bounds__(kBlock)
search_reduce_kernel(themis_batch_t b, uint64_t max_assign, const double* __restrict__ times,
                     double* __restrict__ best_t, uint8_t* __restrict__ best_orders) {
  const uint64_t i = blockIdx.x;
  const double* row = times + i * max_assign;
  double best = inf64();
  uint64_t arg = ~0ull;
  bool bad = false;
  for (uint64_t a = threadIdx.x; a < max_assign; a += kBlock) {
    const double t = row[a];
    bad |= !(t == t);
    if (t < best) { best = t; arg = a; }  // ascending a per lane: the first minimum stays
  }
  for (int off = 32; off > 0; off >>= 1) {
    const double ob = __shfl_down(best, off);
    const uint64_t oa = ((uint64_t)__shfl_down((uint32_t)(arg >> 32), off) << 32) |
                        __shfl_down((uint32_t)arg, off);
    const int obad = __shfl_down((int)bad, off);
    bad |= obad != 0;
    if (ob < best || (ob == best && oa < arg)) { best = ob; arg = oa; }
  }
  if (threadIdx.x != 0) return;
  const uint32_t D = b.ndims[i], C = b.chunks[i];
  const bool ok = !bad && arg != ~0ull && D >= 1u && D <= (uint32_t)kMaxDims && C <= b.max_chunks;
  best_t[i] = ok ? best : nan64();
  if (best_orders) {
    uint8_t* out = best_orders + i * b.max_chunks;
    const uint32_t F = factorial_u32(D);
    uint64_t rest = arg;
    for (uint32_t c = 0; c < b.max_chunks; ++c) {
      uint32_t code = 0xFFu;
      if (ok && c < C) {
        const uint64_t q = rest / F;
        code = nth_permutation_code(D, (uint32_t)(rest - q * F));
        rest = q;
      }
      out[c] = (uint8_t)code;
    }
  }
}

// ---------------------------------------------------------------------------
// themis_beam_search_batch: the chunks get their orders one after the other,
// and after every chunk the `width` best partial schedules are kept (Sec. 4.1,
// observation 2, names the space; Alg. 1 walks it keeping one).
// ---------------------------------------------------------------------------
constexpr uint32_t kBeamMaxWidth = 64;
constexpr uint32_t kBeamOrders = 24;  // D! <= 24 candidates per kept schedule

// One scenario's part of the workspace is found through these offsets.
struct BeamLayout {
  uint64_t n;
  uint32_t width, mc;
  size_t off_digits[2], off_rank[2], off_live, off_times, off_best, off_greedy_orders,
      off_greedy_t, bytes;
};
__host__ __device__ inline BeamLayout beam_layout(uint64_t n, uint32_t mc, uint32_t width) {
  BeamLayout l;
  l.n = n; l.width = width; l.mc = mc;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o = (o + bytes + 63u) & ~(size_t)63u; return at; };
  l.off_times = take((size_t)n * width * kBeamOrders * sizeof(double));
  l.off_best = take((size_t)n * sizeof(double));
  l.off_greedy_t = take((size_t)n * sizeof(double));
  l.off_live = take((size_t)n * sizeof(uint32_t));
  for (int h = 0; h < 2; ++h) {
    l.off_digits[h] = take((size_t)n * width * mc);
    l.off_rank[h] = take((size_t)n * width);
  }
  l.off_greedy_orders = take((size_t)n * mc);
  l.bytes = o;
  return l;
}

// Collective of the first m chunks of a C-chunk schedule: m chunks of size / m bytes.
__device__ __forceinline__ double beam_partial_size(double S, uint32_t C, uint32_t m) {
  return m == C ? S : (S / (double)C) * (double)m;
}

__global__ void __launch_bounds__(256)
beam_init_kernel(themis_batch_t b, BeamLayout l, uint8_t* __restrict__ ws) {
  const uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= b.n) return;
  const Scenario s = load_scenario(b, i);
  const bool ok = s.valid && finite_positive(b.size_bytes[i]) && s.C <= 64u;
  ((uint32_t*)(ws + l.off_live))[i] = ok ? 1u : 0u;   // the empty schedule
  (ws + l.off_rank[0])[i * l.width] = 0u;
}

// One lane per (scenario, kept schedule, order of chunk m - 1): its time into
// times[i][p * 24 + j], +inf where there is no such candidate, NaN where the
// simulation gave up.  kTable: the scenarios the power-of-two path does not
// take (other NPU counts), on per-order tables; each kernel leaves the other's
// scenarios alone.
template <bool kTable, bool kFix>
__global__ void __launch_bounds__(kBlock)
    __attribute__((amdgpu_waves_per_eu(kTable ? LayoutTableWide::kWavesPerSimd : LayoutRing::kWavesPerSimd)))
beam_eval_kernel(themis_batch_t b, BeamLayout l, uint8_t* __restrict__ ws, uint32_t m, int half) {
  using L = typename std::conditional<kTable, LayoutTableWide, LayoutRing>::type;
  __shared__ uint32_t lds_block[L::kLaneWords * kBlock];
  const uint64_t e = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
  const uint32_t per = l.width * kBeamOrders;
  if (e >= b.n * per) return;
  const uint64_t i = e / per;
  const uint32_t cand = (uint32_t)(e - i * per);
  const uint32_t p = cand / kBeamOrders, j = cand - p * kBeamOrders;
  double* times = (double*)(ws + l.off_times);
  Scenario s = load_scenario(b, i);
  const uint32_t live = ((const uint32_t*)(ws + l.off_live))[i];
  const uint32_t C = s.C;
  if (live == 0u || m > C) return;                       // nothing to do for this scenario
  const uint32_t F = factorial_u32((uint32_t)s.D);
  const double chunk = beam_partial_size(b.size_bytes[i], C, m) / (double)m;
  s.C = m;
  FastScenario fs;
  const bool pow2 = fast_eligible(s, chunk, LayoutRing::kCap, fs);
  if (pow2 == kTable) return;                            // the other kernel's scenario
  if (p >= live || j >= F) { times[e] = inf64(); return; }
  const bool scf = b.intra_policy[i] == THEMIS_INTRA_SCF;
  const uint8_t* digits = ws + l.off_digits[half] + (i * l.width + p) * l.mc;
  auto code_at = [&](uint32_t c) {
    return nth_permutation_code((uint32_t)s.D, c + 1u == m ? j : (uint32_t)digits[c]);
  };
  FastOut fo;
  fo.queue_order = nullptr;
  fo.slots = b.max_chunks;
  FastResult r;
  if constexpr (kTable) {
    LaneLds lds;
    lds.base = (uint8_t*)lds_block + 4u * threadIdx.x;
    DivModelT<L> model(s, lds, chunk, scf);
    table_setup_wide<L>(s, scf, lds, code_at, model);
    r = simulate_fast<L, kNoQueueOrder, false, true>(s, model, lds, fo);
  } else {
    const LaneLds lds = lane_lds<L>(lds_block);
    for (uint32_t c = 0; c < m; ++c) L::init_chunk(lds, c, stored_code(s, fs, code_at(c)), fs.state0);
    r = simulate_pow2<L, kNoQueueOrder, false, kFix>(s, Pow2Model(s, fs, scf), lds, fo);
  }
  times[e] = r.ok ? r.t_done : nan64();
}

// One wavefront per scenario keeps the `width` best candidates: smaller time
// first, equal times in ascending assignment number (the newest chunk's digit
// is the most significant, then the kept schedule's own number, known by its
// rank among the kept ones).
__global__ void __launch_bounds__(kBlock)
beam_select_kernel(themis_batch_t b, BeamLayout l, uint8_t* __restrict__ ws, uint32_t m, int half) {
  __shared__ uint32_t new_key[kBeamMaxWidth];
  const uint64_t i = blockIdx.x;
  uint32_t* live_p = (uint32_t*)(ws + l.off_live) + i;
  const uint32_t live = *live_p;
  const uint32_t D = b.ndims[i], C = b.chunks[i];
  if (live == 0u || m > C) return;
  const uint32_t F = factorial_u32(D);
  const double* times = (const double*)(ws + l.off_times) + i * l.width * kBeamOrders;
  const uint8_t* rank_in = ws + l.off_rank[half] + i * l.width;
  uint8_t* rank_out = ws + l.off_rank[half ^ 1] + i * l.width;
  const uint8_t* digits_in = ws + l.off_digits[half] + i * l.width * l.mc;
  uint8_t* digits_out = ws + l.off_digits[half ^ 1] + i * l.width * l.mc;
  const uint32_t nc = live * F;
  const uint32_t kept = nc < l.width ? nc : l.width;
  bool bad = false;
  for (uint32_t x = threadIdx.x; x < nc; x += kBlock) {
    const uint32_t px = x / F, jx = x - px * F;
    const double tx = times[px * kBeamOrders + jx];
    bad |= !(tx == tx);
    const uint32_t kx = jx * kBeamMaxWidth + rank_in[px];
    uint32_t before = 0;
    for (uint32_t y = 0; y < nc; ++y) {
      const uint32_t py = y / F, jy = y - py * F;
      const double ty = times[py * kBeamOrders + jy];
      const uint32_t ky = jy * kBeamMaxWidth + rank_in[py];
      before += (ty < tx || (ty == tx && ky < kx)) ? 1u : 0u;
    }
    if (before < kept) {
      uint8_t* row = digits_out + before * l.mc;
      for (uint32_t c = 0; c + 1u < m; ++c) row[c] = digits_in[px * l.mc + c];
      row[m - 1u] = (uint8_t)jx;
      new_key[before] = kx;
      if (before == 0u) ((double*)(ws + l.off_best))[i] = tx;
    }
  }
  const bool any_bad = __syncthreads_or(bad ? 1 : 0) != 0;
  if (threadIdx.x < kept) {
    uint32_t smaller = 0;
    for (uint32_t q = 0; q < kept; ++q) smaller += new_key[q] < new_key[threadIdx.x] ? 1u : 0u;
    rank_out[threadIdx.x] = (uint8_t)smaller;
  }
  // a simulation that gave up: the scenario has no answer
  if (threadIdx.x == 0) *live_p = any_bad ? 0u : kept;
}

// The better of the beam's best schedule and the greedy plan (the beam's on
// equal times); NaN / all-ones for scenarios without an answer.
__global__ void __launch_bounds__(256)
beam_finish_kernel(themis_batch_t b, BeamLayout l, const uint8_t* __restrict__ ws,
                   double* __restrict__ best_t, uint8_t* __restrict__ best_orders) {
  const uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= b.n) return;
  const uint32_t live = ((const uint32_t*)(ws + l.off_live))[i];
  const uint32_t D = b.ndims[i], C = b.chunks[i];
  const double tb = ((const double*)(ws + l.off_best))[i];
  const double tg = ((const double*)(ws + l.off_greedy_t))[i];
  const bool ok = live != 0u && tg == tg;
  const bool greedy = ok && tg < tb;
  best_t[i] = ok ? (greedy ? tg : tb) : nan64();
  if (!best_orders) return;
  // step m reads buffer (m - 1) & 1 and writes the other: a scenario's last step is m = C
  const uint8_t* digits = ws + l.off_digits[C & 1u] + i * l.width * l.mc;
  const uint8_t* plan = ws + l.off_greedy_orders + i * l.mc;
  for (uint32_t c = 0; c < b.max_chunks; ++c) {
    uint32_t code = 0xFFu;
    if (ok && c < C) code = greedy ? plan[c] : nth_permutation_code(D, digits[c]);
    best_orders[i * b.max_chunks + c] = (uint8_t)code;
  }
}

// ---------------------------------------------------------------------------
// themis_metrics_batch: average bandwidth utilisation (Sec. 3) and Ideal
// (Table 3) per scenario.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
metrics_kernel(themis_batch_t b, const double* __restrict__ t_done,
               const double* __restrict__ transfer, double* __restrict__ utilization,
               double* __restrict__ ideal) {
  uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= b.n) return;
  const int D = b.ndims[i];
  double u = nan64(), id = nan64();
  if (D >= 1 && D <= kMaxDims) {
    double num = 0.0, den = 0.0;
    for (int k = 0; k < D; ++k) {
      const double bw = b.bw[(size_t)k * b.n + i];
      num = num + transfer[(size_t)k * b.n + i] * bw;
      den = den + bw;
    }
    double total = 0.0;
    if (b.n_coll) {
      const uint32_t Q = b.n_coll[i] <= b.max_coll ? b.n_coll[i] : b.max_coll;
      for (uint32_t q = 0; q < Q; ++q) total = total + b.coll_size[(size_t)q * b.n + i];
    } else {
      total = b.size_bytes[i];
    }
    u = num / (t_done[i] * den);
    id = total / den;
  }
  if (utilization) utilization[i] = u;
  if (ideal) ideal[i] = id;
}

// ---------------------------------------------------------------------------
// themis_classify_batch: bandwidth provisioning class of each dimension pair
// (Sec. 6.3).  classes [6][n].
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
classify_kernel(themis_batch_t b, uint8_t* __restrict__ classes) {
  const uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= b.n) return;
  const int D = b.ndims[i];
  bool ok = D >= 1 && D <= kMaxDims;
  double P[kMaxDims], B[kMaxDims];
#pragma unroll
  for (int k = 0; k < kMaxDims; ++k) {
    const uint32_t p = b.npus[(size_t)k * b.n + i];
    P[k] = (double)p;
    B[k] = b.bw[(size_t)k * b.n + i];
    if (k < D && !(p >= 2u && finite_positive(B[k]))) ok = false;
  }
  int pair = 0;
#pragma unroll
  for (int K = 0; K < kMaxDims; ++K) {
    double shrink = 1.0;  // factor by which a chunk shrinks between dimK and dimL
#pragma unroll
    for (int L = K + 1; L < kMaxDims; ++L, ++pair) {
      shrink = shrink * P[L - 1];
      const double balanced = shrink * B[L];
      uint32_t c = B[K] < balanced ? THEMIS_BW_OVER_PROVISIONED
                 : B[K] > balanced ? THEMIS_BW_UNDER_PROVISIONED
                                   : THEMIS_BW_JUST_ENOUGH;
      if (!ok || L >= D) c = 0xFFu;
      classes[(size_t)pair * b.n + i] = (uint8_t)c;
    }
  }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
constexpr uint32_t kMaxSlots = 32767u;  // 16-bit queue entries, all-ones reserved

static int check_batch(const themis_batch_t* b, bool need_intra, bool need_inter) {
  if (!b) return THEMIS_ERR_INVALID_ARGUMENT;
  if (b->max_chunks < 1u || b->max_chunks > THEMIS_MAX_CHUNKS) return THEMIS_ERR_INVALID_ARGUMENT;
  if (b->threshold_mode != THEMIS_THR_ABS && b->threshold_mode != THEMIS_THR_REL)
    return THEMIS_ERR_INVALID_ARGUMENT;
  if (b->n == 0) return THEMIS_OK;
  if (!b->ndims || !b->npus || !b->bw || !b->chunks) return THEMIS_ERR_INVALID_ARGUMENT;
  if (need_inter && (!b->inter_policy || !b->threshold)) return THEMIS_ERR_INVALID_ARGUMENT;
  if (need_intra && !b->intra_policy) return THEMIS_ERR_INVALID_ARGUMENT;
  if (b->n_coll) {
    if (!b->coll_size || b->max_coll < 1u) return THEMIS_ERR_INVALID_ARGUMENT;
    if ((uint64_t)b->max_coll * b->max_chunks > kMaxSlots) return THEMIS_ERR_UNSUPPORTED;
  } else if (!b->size_bytes) {
    return THEMIS_ERR_INVALID_ARGUMENT;
  }
  if (b->n > (uint64_t)0x7fffffff * kBlock) return THEMIS_ERR_UNSUPPORTED;
  return THEMIS_OK;
}

// Compute units of the current device (0 if the query fails: callers then take
// the variant that suits large grids).
static unsigned compute_units() {
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
  return cus > 0 ? (unsigned)cus : 0u;
}

// Number of a call whose kernels may hand evaluations over (see g_marked_call).
static unsigned long long next_call_number() {
  static std::atomic<unsigned long long> counter{0};
  return ++counter;
}

// Launches through hipLaunchKernel and keeps the first error that a launch of
// this call returns: the process-wide "last error" may hold what an unrelated
// earlier call of the host program left there, and reading it would take that
// away from its owner.
struct Launcher {
  hipStream_t stream;
  hipError_t first = hipSuccess;
  explicit Launcher(void* s) : stream((hipStream_t)s) {}
  template <typename... P, typename... A>
  void operator()(void (*kernel)(P...), unsigned blocks, unsigned threads, A&&... a) {
    std::tuple<P...> params(std::forward<A>(a)...);  // converted to the kernel's own parameter types
    void* ptrs[sizeof...(P)];
    fill(ptrs, params, std::index_sequence_for<P...>{});
    const hipError_t e = hipLaunchKernel((const void*)kernel, dim3(blocks), dim3(threads), ptrs, 0, stream);
    if (first == hipSuccess) first = e;
  }
  int status() const { return first == hipSuccess ? THEMIS_OK : THEMIS_ERR_DEVICE; }

 private:
  template <typename T, size_t... I>
  static void fill(void** ptrs, T& params, std::index_sequence<I...>) {
    ((ptrs[I] = (void*)&std::get<I>(params)), ...);
  }
};

using SimKernel = void (*)(themis_batch_t, const uint8_t*, double*, void*, int, double*,
                           unsigned long long);

template <typename L, int kMode>
static SimKernel pick_flags(bool busy, bool fix) {
  return busy ? (fix ? simulate_kernel<L, kMode, true, true> : simulate_kernel<L, kMode, true, false>)
              : (fix ? simulate_kernel<L, kMode, false, true> : simulate_kernel<L, kMode, false, false>);
}

// Queue-entry store modes a layout is built with: four-at-a-time dword stores
// need 8-bit entries (at most 127 slots), 16-bit entries start at 128 slots.
template <typename L>
static SimKernel pick_mode(int mode, bool busy, bool fix) {
  constexpr bool words = L::kCap <= 128u, shorts = L::kCap >= 128u;
  switch (mode) {
    case kNoQueueOrder: return pick_flags<L, kNoQueueOrder>(busy, fix);
    case kBytes: return words ? pick_flags<L, words ? kBytes : kNoQueueOrder>(busy, fix) : nullptr;
    case kWords: return words ? pick_flags<L, words ? kWords : kBytes>(busy, fix) : nullptr;
    case kShorts: return shorts ? pick_flags<L, shorts ? kShorts : kBytes>(busy, fix) : nullptr;
  }
  return nullptr;
}

// Smallest LDS layout that holds max_chunks chunks per evaluation (the less
// LDS a wavefront takes, the more of them share a CU).
static uint32_t layout_capacity(uint32_t max_chunks) {
  return max_chunks > 256u ? 512u : max_chunks > 128u ? 256u : max_chunks > 64u ? 128u
       : max_chunks > 16u ? 64u : 16u;
}

static SimKernel pick_simulate_kernel(uint32_t cap, int mode, bool busy, bool fix) {
  if (cap == 16u) return pick_mode<Layout16>(mode, busy, fix);
  if (cap == 64u) return pick_mode<LayoutRing>(mode, busy, fix);
  if (cap == 128u) return pick_mode<Layout128>(mode, busy, fix);
  if (cap == 256u) return pick_mode<LayoutPacked<256>>(mode, busy, fix);
  return pick_mode<LayoutPacked<512>>(mode, busy, fix);
}

// The generic area comes first in the workspace, rounded up so that the trace
// regions behind it keep the workspace's alignment up to 64 bytes.
static size_t generic_area_bytes(uint64_t evals, uint64_t slots) {
  return (workspace_bytes(evals, slots) + 63u) & ~(size_t)63u;
}

static unsigned blocks_for(uint64_t items) { return (unsigned)((items + kBlock - 1) / kBlock); }

// Grid of a follow-up kernel (its workgroups stride over the groups of 64
// evaluations): enough to fill the device, no more.
static unsigned follow_up_blocks(uint64_t items) {
  const unsigned cus = compute_units();
  const unsigned cap = 8u * (cus ? cus : 256u);
  const unsigned all = blocks_for(items);
  return all < cap ? all : cap;
}

// Which mapping themis_sweep's LDS kernel uses for a layout capacity: four
// lanes per evaluation from kQuadFromCap chunks on, one lane below, unless
// themis_set_sweep_mapping() has fixed one of them.
constexpr uint32_t kQuadFromCap = 256;
static std::atomic<int> sweep_mapping{THEMIS_MAPPING_AUTO};
static bool sweep_mapping_is_quad(uint32_t cap) {
  const int forced = sweep_mapping.load(std::memory_order_relaxed);
  return forced != THEMIS_MAPPING_AUTO ? forced == THEMIS_MAPPING_QUAD : cap >= kQuadFromCap;
}

}  // namespace themis

using namespace themis;

extern "C" {

int themis_version(void) { return 103; }

const char* themis_status_string(int status) {
  switch (status) {
    case THEMIS_OK: return "success";
    case THEMIS_ERR_INVALID_ARGUMENT: return "invalid argument";
    case THEMIS_ERR_UNSUPPORTED: return "unsupported request";
    case THEMIS_ERR_DEVICE: return "HIP device error";
    case THEMIS_ERR_WORKSPACE: return "workspace missing, too small or misaligned, or the request exceeds the built-in scratch";
    default: return "unknown status";
  }
}

int themis_queue_entry_bytes(uint32_t max_chunks, uint32_t max_coll) {
  uint64_t slots = (uint64_t)max_chunks * (max_coll ? max_coll : 1u);
  return slots <= 127u ? 1 : 2;
}

size_t themis_workspace_bytes(uint64_t n, uint32_t max_chunks, uint32_t max_coll) {
  size_t generic = generic_area_bytes(n, (uint64_t)max_chunks * (max_coll ? max_coll : 1u));
  size_t trace = max_coll ? (size_t)n * trace_layout(max_chunks, max_coll).bytes : 0;
  return generic + trace;
}

int themis_plan_batch(const themis_batch_t* batch, uint8_t* orders, double* loads, void* stream) {
  int st = check_batch(batch, false, true);
  if (st != THEMIS_OK) return st;
  if (batch->n == 0) return THEMIS_OK;
  if (!orders) return THEMIS_ERR_INVALID_ARGUMENT;
  const TraceView tv = trace_view(*batch);
  if (batch->n * (uint64_t)tv.mc > (uint64_t)0x7fffffff * kBlock) return THEMIS_ERR_UNSUPPORTED;
  Launcher go(stream);
  if (tv.mc > 1u)
    go(plan_kernel<true>, blocks_for(batch->n * tv.mc), kBlock, *batch, orders, loads);
  else
    go(plan_kernel<false>, blocks_for(batch->n), kBlock, *batch, orders, loads);
  return go.status();
}

static int simulate_batch_impl(const themis_batch_t* batch, const uint8_t* orders, double* t_done,
                               void* queue_order, double* busy, void* workspace,
                               size_t workspace_bytes_given, void* stream) {
  int st = check_batch(batch, true, false);
  if (st != THEMIS_OK) return st;
  if (batch->n == 0) return THEMIS_OK;
  if (!orders || !t_done) return THEMIS_ERR_INVALID_ARGUMENT;
  if ((uintptr_t)workspace & 15u) return THEMIS_ERR_WORKSPACE;
  const TraceView tv = trace_view(*batch);
  const bool have_ws =
      workspace != nullptr && workspace_bytes_given >= workspace_bytes(batch->n, tv.slots);
  Workspace w = carve_workspace(workspace, batch->n, tv.slots);
  const int entry_bytes =
      themis_queue_entry_bytes(batch->max_chunks, tv.on ? batch->max_coll : 0u);
  const uint32_t cap = tv.on ? 512u : layout_capacity(batch->max_chunks);
  Launcher go(stream);
  // 8-bit entries are stored four at a time by the layouts with 8-bit chunk
  // ids when the rows (2*slots bytes each) start on 4-byte boundaries
  const bool words = entry_bytes == 1 && cap <= 128u && (tv.slots & 1u) == 0u &&
                     ((uintptr_t)queue_order & 3u) == 0u;
  const int mode = !queue_order ? kNoQueueOrder
                 : entry_bytes == 2 ? kShorts : (words ? kWords : kBytes);
  if (tv.on) {
    const TraceLayout tl = trace_layout(batch->max_chunks, batch->max_coll);
    const size_t generic = generic_area_bytes(batch->n, tv.slots);
    const bool have_trace = workspace != nullptr && tl.bytes != 0u &&
                            workspace_bytes_given >= generic + (size_t)batch->n * tl.bytes;
    uint8_t* trace_area = have_trace ? (uint8_t*)workspace + generic : nullptr;
    // few wavefronts (no more than CUs): the bitmap leaves move into the LDS nothing else would use
    const bool lds_bitmaps = blocks_for(batch->n) <= compute_units();
    const bool extras = batch->release_time != nullptr || batch->fixed_delay != nullptr ||
                        queue_order != nullptr;
    auto trace_kernel = lds_bitmaps ? (extras ? simulate_trace_kernel<true, true> : simulate_trace_kernel<true, false>)
                                    : (extras ? simulate_trace_kernel<false, true> : simulate_trace_kernel<false, false>);
    go(trace_kernel, blocks_for(batch->n), kBlock, *batch, orders, t_done, queue_order,
       entry_bytes, busy, w, have_ws, trace_area, tl);
    return go.status();
  }
  SimKernel kernel = pick_simulate_kernel(cap, mode, busy != nullptr,
                                          batch->fixed_delay != nullptr);
  if (!kernel) return THEMIS_ERR_DEVICE;
  // Scenarios outside the LDS path (marked in t_done) go through the table
  // passes and what those leave through the generic pass: its arrays in LDS up
  // to 64 chunks, in the workspace beyond.  One launch for all of it where that
  // costs nothing: beyond 64 chunks (the generic pass needs no LDS there), with
  // a workspace (the same), and on batches small enough for every wavefront to
  // be resident whatever the LDS block (there the launches are what counts).
  // A large batch of up to 64 chunks without a workspace keeps the generic pass
  // and its 80 KiB of LDS apart from the table passes.
  const unsigned long long call = next_call_number();
  go(kernel, blocks_for(batch->n), kBlock, *batch, orders, t_done, queue_order, entry_bytes, busy,
     call);
  const unsigned fb = follow_up_blocks(batch->n);
  const Workspace ws = have_ws ? w : Workspace{};
#define THEMIS_FOLLOW_UP(MODE, A, B, G) \
  go(simulate_follow_up_kernel<MODE, A, B, G>, fb, kBlock, *batch, orders, t_done, queue_order, \
     entry_bytes, busy, ws, call)
  // (8-bit entries up to 64 chunks, either up to 128, 16-bit entries beyond)
#define THEMIS_FOLLOW_UP_MODES(A, B, G)                                  \
  switch (mode) {                                                        \
    case kNoQueueOrder: THEMIS_FOLLOW_UP(kNoQueueOrder, A, B, G); break; \
    case kWords: THEMIS_FOLLOW_UP(kWords, A, B, G); break;               \
    default: THEMIS_FOLLOW_UP(kBytes, A, B, G); break;                   \
  }
  if (cap <= 64u) {
    const bool small = blocks_for(batch->n) <= 2u * compute_units();
    if (have_ws) {
      THEMIS_FOLLOW_UP_MODES(0, 1, 0u)
    } else if (small && cap <= 16u) {
      THEMIS_FOLLOW_UP_MODES(0, 1, 16u)
    } else if (small) {
      THEMIS_FOLLOW_UP_MODES(0, 1, 64u)
    } else {
      THEMIS_FOLLOW_UP_MODES(0, 1, kNoGeneric)
      auto generic = cap <= 16u ? simulate_generic_kernel<16> : simulate_generic_kernel<64>;
      go(generic, fb, kBlock, *batch, orders, t_done, queue_order, entry_bytes, busy, ws, call);
    }
  } else if (cap == 128u) {
    if (mode == kShorts) THEMIS_FOLLOW_UP(kShorts, 2, -1, 0u);
    else THEMIS_FOLLOW_UP_MODES(2, -1, 0u)
  } else if (cap == 256u) {
    if (mode == kNoQueueOrder) THEMIS_FOLLOW_UP(kNoQueueOrder, 3, -1, 0u);
    else THEMIS_FOLLOW_UP(kShorts, 3, -1, 0u);
  } else {
    if (mode == kNoQueueOrder) THEMIS_FOLLOW_UP(kNoQueueOrder, 4, -1, 0u);
    else THEMIS_FOLLOW_UP(kShorts, 4, -1, 0u);
  }
#undef THEMIS_FOLLOW_UP_MODES
#undef THEMIS_FOLLOW_UP
  return go.status();
}

int themis_simulate_batch(const themis_batch_t* batch, const uint8_t* orders, double* t_done,
                          void* queue_order, double* busy, void* workspace,
                          size_t workspace_bytes_given, void* stream) {
  return simulate_batch_impl(batch, orders, t_done, queue_order, busy, workspace,
                             workspace_bytes_given, stream);
}

// Device address of `scratch` on the current device, asked for once per device
// and kept: every GPU holds its own copy of the array at its own address.
static int scratch_of_current_device(void** out) {
  constexpr int kMaxDevices = 64;
  static std::atomic<void*> known[kMaxDevices];
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return THEMIS_ERR_DEVICE;
  void* p = known[dev].load(std::memory_order_acquire);
  if (!p) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return THEMIS_ERR_DEVICE;
    known[dev].store(p, std::memory_order_release);  // two first calls at once store the same address
  }
  *out = p;
  return THEMIS_OK;
}

int themis_simulate_batch_noalloc(const themis_batch_t* batch, const uint8_t* orders,
                                  double* t_done, void* queue_order, double* busy, void* stream) {
  int st = check_batch(batch, true, false);
  if (st != THEMIS_OK) return st;
  if (batch->n == 0) return THEMIS_OK;
  // what themis_simulate_batch would ask a caller for: traces keep their queues
  // there, single collectives only what the generic path needs beyond 64 chunks
  const bool trace = batch->n_coll != nullptr;
  const size_t need = (trace || batch->max_chunks > 64u)
      ? themis_workspace_bytes(batch->n, batch->max_chunks, trace ? batch->max_coll : 0u) : 0u;
  if (need > (size_t)THEMIS_STATIC_SCRATCH_BYTES) return THEMIS_ERR_WORKSPACE;
  void* ws = nullptr;
  st = scratch_of_current_device(&ws);
  if (st != THEMIS_OK) return st;
  // nothing in the scratch has to start at zero: the kernels initialise every
  // word they read (chunk state, list heads behind a set bitmap bit, bitmaps)
  return simulate_batch_impl(batch, orders, t_done, queue_order, busy, ws,
                             (size_t)THEMIS_STATIC_SCRATCH_BYTES, stream);
}

int themis_sweep(const themis_batch_t* batch, int n_thr, const double* thr, int thr_per_scenario,
                 unsigned policy_mask, double* t_done, void* workspace,
                 size_t workspace_bytes_given, void* stream) {
  int st = check_batch(batch, false, false);
  if (st != THEMIS_OK) return st;
  if (batch->n_coll) return THEMIS_ERR_UNSUPPORTED;  // sweeps are per single collective
  if (n_thr < 1 || !thr || (policy_mask & 7u) == 0u || (policy_mask & ~7u) != 0u)
    return THEMIS_ERR_INVALID_ARGUMENT;
  if (batch->n == 0) return THEMIS_OK;
  if (!t_done) return THEMIS_ERR_INVALID_ARGUMENT;
  if ((uintptr_t)workspace & 15u) return THEMIS_ERR_WORKSPACE;
  int n_pol = __builtin_popcount(policy_mask & 7u);
  uint64_t evals = batch->n * (uint64_t)n_thr * (uint64_t)n_pol;
  if (evals > (uint64_t)0x7fffffff * kBlock ||
      (uint64_t)blocks_for(batch->n) * (uint64_t)(n_thr * n_pol) > 0x7fffffffull)
    return THEMIS_ERR_UNSUPPORTED;
  const bool have_ws = workspace != nullptr &&
                       workspace_bytes_given >= workspace_bytes(evals, batch->max_chunks);
  Workspace w = carve_workspace(workspace, evals, batch->max_chunks);
  const uint32_t cap = layout_capacity(batch->max_chunks);
  const bool fix = batch->fixed_delay != nullptr;
  const bool base = (policy_mask & THEMIS_SWEEP_BASELINE) != 0u;
#define THEMIS_SWEEP_KERNEL(L)                                                          \
  (fix ? (base ? sweep_kernel<L, true, true> : sweep_kernel<L, true, false>)            \
       : (base ? sweep_kernel<L, false, true> : sweep_kernel<L, false, false>))
  auto kernel = cap == 16u ? THEMIS_SWEEP_KERNEL(Layout16)
              : cap == 64u ? THEMIS_SWEEP_KERNEL(LayoutRing)
              : cap == 128u ? THEMIS_SWEEP_KERNEL(Layout128)
              : cap == 256u ? THEMIS_SWEEP_KERNEL(LayoutPacked<256>)
                            : THEMIS_SWEEP_KERNEL(LayoutPacked<512>);
#undef THEMIS_SWEEP_KERNEL
  auto quad_kernel = fix ? (base ? sweep_quad_kernel<true, true> : sweep_quad_kernel<true, false>)
                         : (base ? sweep_quad_kernel<false, true> : sweep_quad_kernel<false, false>);
  const unsigned long long call = next_call_number();
  Launcher go(stream);
  // (one workgroup per group of scenarios and pair, the baseline once: see sweep_roles)
  const unsigned roles = sweep_roles((uint32_t)n_thr, (uint32_t)n_pol, policy_mask);
  if (sweep_mapping_is_quad(cap)) {
    const uint64_t groups = (batch->n + LayoutQuad::kQuads - 1u) / LayoutQuad::kQuads;
    if (groups * (uint64_t)(n_thr * n_pol) > 0x7fffffffull) return THEMIS_ERR_UNSUPPORTED;
    go(quad_kernel, (unsigned)groups * roles, kBlock,
       *batch, n_thr, thr, thr_per_scenario, policy_mask, n_pol, t_done, call);
  } else {
    go(kernel, blocks_for(batch->n) * roles, kBlock, *batch, n_thr, thr, thr_per_scenario,
       policy_mask, n_pol, t_done, call);
  }
  // the follow-up passes, in one launch where themis_simulate_batch does the same
  const unsigned fb = follow_up_blocks(evals);
  const Workspace ws = have_ws ? w : Workspace{};
#define THEMIS_FOLLOW_UP(A, B, G)                                                            \
  go(sweep_follow_up_kernel<A, B, G>, fb, kBlock, *batch, n_thr, thr, thr_per_scenario,      \
     policy_mask, n_pol, t_done, ws, call)
  if (cap <= 64u) {
    const bool small = blocks_for(evals) <= 2u * compute_units();
    if (have_ws) {
      THEMIS_FOLLOW_UP(0, 1, 0u);
    } else if (small && cap <= 16u) {
      THEMIS_FOLLOW_UP(0, 1, 16u);
    } else if (small) {
      THEMIS_FOLLOW_UP(0, 1, 64u);
    } else {
      THEMIS_FOLLOW_UP(0, 1, kNoGeneric);
      auto generic = cap <= 16u ? sweep_generic_kernel<16> : sweep_generic_kernel<64>;
      go(generic, fb, kBlock, *batch, n_thr, thr, thr_per_scenario, policy_mask, n_pol, t_done,
         ws, call);
    }
  } else if (cap == 128u) {
    THEMIS_FOLLOW_UP(2, -1, 0u);
  } else if (cap == 256u) {
    THEMIS_FOLLOW_UP(3, -1, 0u);
  } else {
    THEMIS_FOLLOW_UP(4, -1, 0u);
  }
#undef THEMIS_FOLLOW_UP
  return go.status();
}

int themis_set_sweep_mapping(int mapping) {
  if (mapping != THEMIS_MAPPING_AUTO && mapping != THEMIS_MAPPING_LANE &&
      mapping != THEMIS_MAPPING_QUAD)
    return THEMIS_ERR_INVALID_ARGUMENT;
  sweep_mapping.store(mapping, std::memory_order_relaxed);
  return THEMIS_OK;
}

size_t themis_search_workspace_bytes(uint64_t n, uint64_t max_assignments) {
  return (size_t)n * max_assignments * sizeof(double);
}

int themis_search_batch(const themis_batch_t* batch, uint64_t max_assignments, double* best_t,
                        uint8_t* best_orders, void* workspace, size_t workspace_bytes_given,
                        void* stream) {
  int st = check_batch(batch, true, false);
  if (st != THEMIS_OK) return st;
  if (batch->n_coll) return THEMIS_ERR_UNSUPPORTED;  // single collectives only
  if (max_assignments < 1u) return THEMIS_ERR_INVALID_ARGUMENT;
  if (batch->n == 0) return THEMIS_OK;
  if (!best_t) return THEMIS_ERR_INVALID_ARGUMENT;
  if (max_assignments > ((uint64_t)1 << 40) / batch->n) return THEMIS_ERR_UNSUPPORTED;
  const uint64_t evals = batch->n * max_assignments;
  if (evals > (uint64_t)0x7fffffff * kBlock || batch->n > 0x7fffffffull) return THEMIS_ERR_UNSUPPORTED;
  if (!workspace || ((uintptr_t)workspace & 7u) ||
      workspace_bytes_given < themis_search_workspace_bytes(batch->n, max_assignments))
    return THEMIS_ERR_WORKSPACE;
  double* times = (double*)workspace;
  const bool fix = batch->fixed_delay != nullptr;
  Launcher go(stream);
  auto eval = batch->max_chunks <= 16u
      ? (fix ? search_eval_kernel<false, Layout16, true> : search_eval_kernel<false, Layout16, false>)
      : (fix ? search_eval_kernel<false, LayoutRing, true> : search_eval_kernel<false, LayoutRing, false>);
  const unsigned long long call = next_call_number();
  go(eval, blocks_for(evals), kBlock, *batch, max_assignments, times, call);
  go(search_eval_kernel<true, LayoutTableWide, true>, follow_up_blocks(evals), kBlock, *batch,
     max_assignments, times, call);
  go(search_reduce_kernel, (unsigned)batch->n, kBlock, *batch, max_assignments, times, best_t,
     best_orders);
  return go.status();
}

size_t themis_beam_workspace_bytes(uint64_t n, uint32_t max_chunks, uint32_t width) {
  if (width < 1u || width > kBeamMaxWidth) return 0;
  return beam_layout(n, max_chunks, width).bytes;
}

int themis_beam_search_batch(const themis_batch_t* batch, uint32_t width, double* best_t,
                             uint8_t* best_orders, void* workspace, size_t workspace_bytes_given,
                             void* stream) {
  int st = check_batch(batch, false, true);
  if (st != THEMIS_OK) return st;
  if (batch->n_coll) return THEMIS_ERR_UNSUPPORTED;  // single collectives only
  if (width < 1u || width > kBeamMaxWidth) return THEMIS_ERR_INVALID_ARGUMENT;
  if (batch->max_chunks > 64u) return THEMIS_ERR_UNSUPPORTED;
  if (batch->n == 0) return THEMIS_OK;
  if (!best_t || !batch->intra_policy) return THEMIS_ERR_INVALID_ARGUMENT;
  const BeamLayout l = beam_layout(batch->n, batch->max_chunks, width);
  const uint64_t lanes = batch->n * (uint64_t)width * kBeamOrders;
  if (lanes > (uint64_t)0x7fffffff * kBlock || batch->n > 0x7fffffffull) return THEMIS_ERR_UNSUPPORTED;
  if (!workspace || ((uintptr_t)workspace & 63u) || workspace_bytes_given < l.bytes)
    return THEMIS_ERR_WORKSPACE;
  uint8_t* ws = (uint8_t*)workspace;
  // the greedy plan and its time (every scenario up to 64 chunks runs without a workspace)
  uint8_t* plan = ws + l.off_greedy_orders;
  double* plan_t = (double*)(ws + l.off_greedy_t);
  st = themis_plan_batch(batch, plan, nullptr, stream);
  if (st != THEMIS_OK) return st;
  st = simulate_batch_impl(batch, plan, plan_t, nullptr, nullptr, nullptr, 0, stream);
  if (st != THEMIS_OK) return st;
  const bool fix = batch->fixed_delay != nullptr;
  Launcher go(stream);
  const unsigned per_scenario = (unsigned)((batch->n + 255) / 256);
  go(beam_init_kernel, per_scenario, 256, *batch, l, ws);
  int half = 0;
  for (uint32_t m = 1; m <= batch->max_chunks; ++m) {
    go(fix ? beam_eval_kernel<false, true> : beam_eval_kernel<false, false>, blocks_for(lanes),
       kBlock, *batch, l, ws, m, half);
    go(beam_eval_kernel<true, true>, blocks_for(lanes), kBlock, *batch, l, ws, m, half);
    go(beam_select_kernel, (unsigned)batch->n, kBlock, *batch, l, ws, m, half);
    half ^= 1;
  }
  go(beam_finish_kernel, per_scenario, 256, *batch, l, (const uint8_t*)ws, best_t, best_orders);
  return go.status();
}

int themis_metrics_batch(const themis_batch_t* batch, const double* t_done, const double* transfer,
                         double* utilization, double* ideal, void* stream) {
  if (!batch) return THEMIS_ERR_INVALID_ARGUMENT;
  if (batch->n == 0) return THEMIS_OK;
  if (!batch->ndims || !batch->bw || !t_done || !transfer) return THEMIS_ERR_INVALID_ARGUMENT;
  if (batch->n_coll ? !batch->coll_size : !batch->size_bytes) return THEMIS_ERR_INVALID_ARGUMENT;
  if (batch->n > (uint64_t)0x7fffffff * 256u) return THEMIS_ERR_UNSUPPORTED;
  Launcher go(stream);
  go(metrics_kernel, (unsigned)((batch->n + 255) / 256), 256, *batch, t_done, transfer,
     utilization, ideal);
  return go.status();
}

int themis_classify_batch(const themis_batch_t* batch, uint8_t* classes, void* stream) {
  if (!batch) return THEMIS_ERR_INVALID_ARGUMENT;
  if (batch->n == 0) return THEMIS_OK;
  if (!batch->ndims || !batch->npus || !batch->bw || !classes) return THEMIS_ERR_INVALID_ARGUMENT;
  if (batch->n > (uint64_t)0x7fffffff * 256u) return THEMIS_ERR_UNSUPPORTED;
  Launcher go(stream);
  go(classify_kernel, (unsigned)((batch->n + 255) / 256), 256, *batch, classes);
  return go.status();
}

int themis_sweep_best(uint64_t n, int n_thr, int n_pol, const double* t_done, int baseline_col,
                      double* best_t, uint32_t* best_thr, double* speedup, void* stream) {
  if (n_thr < 1 || n_pol < 1 || n_pol > 3 || baseline_col >= n_pol) return THEMIS_ERR_INVALID_ARGUMENT;
  if (n == 0) return THEMIS_OK;
  if (!t_done || !best_t) return THEMIS_ERR_INVALID_ARGUMENT;
  if (n > (uint64_t)0x7fffffff * 64u) return THEMIS_ERR_UNSUPPORTED;
  const uint64_t items = n * (uint64_t)n_pol;
  Launcher go(stream);
  go(sweep_best_kernel, (unsigned)((items + 255) / 256), 256, n, (uint32_t)n_thr, (uint32_t)n_pol,
     t_done, baseline_col, best_t, best_thr, speedup);
  return go.status();
}

}  // extern "C"
