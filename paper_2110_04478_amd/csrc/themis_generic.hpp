// Generic (any NPU count, any chunk count, traces) planner and queue
// simulation: one lane per evaluation, per-chunk state in a caller-provided
// HBM workspace laid out [slot][evaluation] so that the 64 lanes of a
// wavefront, which walk the chunk slots in lock step, touch 64 consecutive
// elements.  It is exact for every valid input and serves as the fall-back of
// the register/LDS fast path, which only covers power-of-two NPU counts.
#pragma once

#include "themis_device.hpp"

namespace themis {

// Workspace view: three arrays of `slots` rows and `stride` columns.
struct Workspace {
  double* arrival;  // time the chunk joined the queue it waits in
  double* size;     // resident bytes before its next stage
  uint32_t* meta;   // stage (bits 0-3) | running (bit 4) | order code (bits 8-15)
  uint64_t stride;  // evaluations (columns)
};

__host__ __device__ inline size_t workspace_bytes(uint64_t evals, uint64_t slots) {
  return (size_t)evals * slots * (sizeof(double) * 2 + sizeof(uint32_t));
}

__host__ __device__ inline Workspace carve_workspace(void* base, uint64_t evals, uint64_t slots) {
  Workspace w;
  w.arrival = (double*)base;
  w.size = w.arrival + evals * slots;
  w.meta = (uint32_t*)(w.size + evals * slots);
  w.stride = evals;
  return w;
}

constexpr uint32_t kMetaRunning = 16u;

// Where a scenario's results go; any pointer may be null.
struct SimOut {
  double* t_done;        // one value
  double* busy;          // [4] with stride busy_stride
  uint64_t busy_stride;
  void* queue_order;     // this scenario's [4][2*slots] block
  int entry_bytes;       // 1 or 2
  uint32_t slots;
};

__device__ __forceinline__ void put_entry(const SimOut& o, int k, uint32_t pos, uint32_t v) {
  size_t at = (size_t)k * 2u * o.slots + pos;
  if (o.entry_bytes == 1) ((uint8_t*)o.queue_order)[at] = (uint8_t)v;
  else ((uint16_t*)o.queue_order)[at] = (uint16_t)v;
}

__device__ __forceinline__ void write_invalid(const SimOut& o) {
  if (o.t_done) *o.t_done = nan64();
  if (o.busy)
    for (int k = 0; k < kMaxDims; ++k) o.busy[(size_t)k * o.busy_stride] = nan64();
  if (o.queue_order)
    for (int k = 0; k < kMaxDims; ++k)
      for (uint32_t e = 0; e < 2u * o.slots; ++e) put_entry(o, k, e, 0xFFFFu);
}

// Queue simulation of one evaluation (column `col` of the workspace).
// Chunks g = 0..G-1 (G = Q*C) must already be initialised in the workspace:
// meta = code << 8 (stage 0), size = chunk bytes of its collective, arrival =
// release time.  chunk_of(q) returns collective q's chunk size, release_of(q)
// its release time; both are only consulted while replaying stage times.
// kEager: read a chunk's arrival time and size together with its meta word
// instead of only once it is known to be a candidate -- no branches and
// several chunks' loads in flight at once; for arrays in LDS, where the extra
// reads cost next to nothing.
template <bool kEager, typename ChunkOf, typename ReleaseOf>
__device__ void simulate_generic(const Scenario& s, uint32_t Q, bool scf, const Workspace& w,
                                 uint64_t col, ChunkOf chunk_of, ReleaseOf release_of,
                                 bool has_release, const SimOut& out) {
  const int D = s.D;
  const uint32_t C = s.C;
  const uint32_t G = Q * C;
  const bool all_reduce = s.ctype == THEMIS_COLL_ALL_REDUCE;
  const bool gather = s.ctype == THEMIS_COLL_ALL_GATHER;
  // an All-Reduce runs D Reduce-Scatter and D All-Gather stages (the latter in
  // reverse order), the stand-alone collectives only their own D
  const int last_stage = all_reduce ? 2 * D : D;

  int serving[kMaxDims] = {-1, -1, -1, -1};
  double finish[kMaxDims] = {0.0, 0.0, 0.0, 0.0};
  double busy[kMaxDims] = {0.0, 0.0, 0.0, 0.0};
  uint32_t executed[kMaxDims] = {0u, 0u, 0u, 0u};
  double now = 0.0, last_done = 0.0;

  // every pass either starts or completes at least one stage, or consumes a
  // release instant, so this bound is never reached by a valid scenario; it
  // only guarantees that the wave drains whatever the inputs are.
  const uint64_t max_pass = (uint64_t)2 * D * G + Q + 8u;
  for (uint64_t pass = 0; pass < max_pass; ++pass) {
    // (i) idle dimensions pick the first waiting chunk in policy order
    bool any_idle = false;
#pragma unroll
    for (int k = 0; k < kMaxDims; ++k) any_idle |= (k < D && serving[k] < 0);
    if (any_idle) {
      int best[kMaxDims] = {-1, -1, -1, -1};
      double bsize[kMaxDims] = {0.0, 0.0, 0.0, 0.0};
      double barr[kMaxDims] = {0.0, 0.0, 0.0, 0.0};
      uint32_t bmeta[kMaxDims] = {0u, 0u, 0u, 0u};
      if (kEager) {
        const uint32_t idle_dims = (serving[0] < 0 ? 1u : 0u) | (serving[1] < 0 ? 2u : 0u) |
                                   (serving[2] < 0 ? 4u : 0u) | (serving[3] < 0 ? 8u : 0u);
#pragma unroll 4
        for (uint32_t g = 0; g < G; ++g) {
          const size_t at = (size_t)g * w.stride + col;
          const uint32_t m = w.meta[at];
          const double arr = w.arrival[at];
          const double sz = scf ? w.size[at] : 0.0;
          const int stage = (int)(m & 15u);
          const uint32_t code = (m >> 8) & 0xFFu;
          const int pos = stage < D ? stage : 2 * D - 1 - stage;
          const int k = (int)((code >> ((2 * pos) & 31)) & 3u);
          // bitwise on purpose: selects, not branches
          const bool cand = (stage < last_stage) & ((m & kMetaRunning) == 0u) &
                            (((idle_dims >> k) & 1u) != 0u) & !(arr > now);
#pragma unroll
          for (int kk = 0; kk < kMaxDims; ++kk) {
            // ascending g with strict '<' keeps the lowest chunk id on ties
            const bool better = (best[kk] < 0) | (sz < bsize[kk]) |
                                ((sz == bsize[kk]) & (arr < barr[kk]));
            const bool upd = cand & (kk == k) & better;
            best[kk] = upd ? (int)g : best[kk];
            bsize[kk] = upd ? sz : bsize[kk];
            barr[kk] = upd ? arr : barr[kk];
            bmeta[kk] = upd ? m : bmeta[kk];
          }
        }
      } else {
        for (uint32_t g = 0; g < G; ++g) {
          size_t at = (size_t)g * w.stride + col;
          uint32_t m = w.meta[at];
          int stage = (int)(m & 15u);
          if (stage >= last_stage || (m & kMetaRunning)) continue;
          uint32_t code = (m >> 8) & 0xFFu;
          int pos = stage < D ? stage : 2 * D - 1 - stage;
          int k = (int)((code >> (2 * pos)) & 3u);
          if (sel4(k, serving[0], serving[1], serving[2], serving[3]) >= 0) continue;
          double arr = w.arrival[at];
          if (arr > now) continue;  // not released yet
          double sz = scf ? w.size[at] : 0.0;
#pragma unroll
          for (int kk = 0; kk < kMaxDims; ++kk) {
            if (kk == k) {
              bool first = best[kk] < 0;
              // ascending g with strict '<' keeps the lowest chunk id on ties
              bool better = (sz < bsize[kk]) || (sz == bsize[kk] && arr < barr[kk]);
              if (first || better) { best[kk] = (int)g; bsize[kk] = sz; barr[kk] = arr; bmeta[kk] = m; }
            }
          }
        }
      }
#pragma unroll
      for (int k = 0; k < kMaxDims; ++k) {
        if (k < D && serving[k] < 0 && best[k] >= 0) {
          uint32_t g = (uint32_t)best[k];
          size_t at = (size_t)g * w.stride + col;
          uint32_t m = bmeta[k];
          int stage = (int)(m & 15u);
          uint32_t code = (m >> 8) & 0xFFu;
          // stage time: x * coef[k] with x the resident size before the
          // chunk's Reduce-Scatter on k.  In the Reduce-Scatter phase that is
          // the current size; the All-Gather reuses the same product, so the
          // Reduce-Scatter size is replayed from the chunk size.
          double x;
          if (gather) {
            x = w.size[at] * (double)s.P[k];  // a stand-alone All-Gather moves the grown size
          } else if (stage < D) {
            x = w.size[at];
          } else {
            int pos = 2 * D - 1 - stage;
            x = chunk_of(g / C);
            for (int j = 0; j < pos; ++j) {
              int kj = (int)((code >> (2 * j)) & 3u);
              x = x / (double)sel4(kj, s.P[0], s.P[1], s.P[2], s.P[3]);
            }
          }
          double t = x * s.coef[k];
          if (s.has_fix) t = s.fix[k] + t;
          finish[k] = now + t;
          busy[k] = busy[k] + t;
          serving[k] = (int)g;
          w.meta[at] = m | kMetaRunning;
          if (out.queue_order)
            put_entry(out, k, executed[k], (g << 1) | ((gather || stage >= D) ? 1u : 0u));
          executed[k]++;
        }
      }
    }

    // (ii)+(iii) next instant: earliest completion or release
    double next = inf64();
#pragma unroll
    for (int k = 0; k < kMaxDims; ++k)
      if (k < D && serving[k] >= 0 && finish[k] < next) next = finish[k];
    if (has_release)
      for (uint32_t q = 0; q < Q; ++q) {
        double r = release_of(q);
        if (r > now && r < next) next = r;
      }
    if (!(next < inf64())) break;
    now = next;

    // (iv) deliver every completion that falls on this instant
#pragma unroll
    for (int k = 0; k < kMaxDims; ++k) {
      if (k < D && serving[k] >= 0 && finish[k] == now) {
        size_t at = (size_t)serving[k] * w.stride + col;
        uint32_t m = w.meta[at];
        int stage = (int)(m & 15u);
        double sz = w.size[at];
        double pk = (double)s.P[k];
        sz = (!gather && stage < D) ? sz / pk : sz * pk;
        w.size[at] = sz;
        w.arrival[at] = now;
        w.meta[at] = (m & ~(15u | kMetaRunning)) | (uint32_t)(stage + 1);
        serving[k] = -1;
        if (stage + 1 == last_stage) last_done = now;
      }
    }
  }

  // a stage time or clock value that overflowed leaves the model: reported
  // like an invalid scenario (these sums bound every one of them)
  bool finite = last_done < inf64();
#pragma unroll
  for (int k = 0; k < kMaxDims; ++k) finite = finite && busy[k] < inf64();
  if (!finite) { write_invalid(out); return; }

  if (out.t_done) *out.t_done = last_done;
  if (out.busy)
    for (int k = 0; k < kMaxDims; ++k) out.busy[(size_t)k * out.busy_stride] = busy[k];
  if (out.queue_order)
    for (int k = 0; k < kMaxDims; ++k)
      for (uint32_t e = (k < D ? executed[k] : 0u); e < 2u * out.slots; ++e)
        put_entry(out, k, e, 0xFFFFu);
}

}  // namespace themis
