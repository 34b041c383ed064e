// Device-side building blocks shared by the Themis kernels (gfx950 only).
//
// Mapping used throughout: one lane evaluates one scenario (or one
// scenario x threshold x scheduler combination in the sweep), because the
// planner (paper Alg. 1) and the queue simulation (paper Sec. 4.3, 4.6.2) are
// strictly sequential inside a scenario and independent across scenarios.
// Per-scenario inputs are structure-of-arrays, so a wavefront's 64 lanes read
// 64 consecutive values in one coalesced access.
//
// All floating point is binary64 and unfused: the translation unit is
// compiled with -ffp-contract=off, and every expression below is written in
// the exact operation order that the C ABI header documents.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "themis.h"

namespace themis {

constexpr int kMaxDims = THEMIS_MAX_DIMS;
constexpr int kBlock = 64;  // one wavefront per workgroup keeps divergence local

__device__ __forceinline__ double nan64() { return __longlong_as_double(0x7ff8000000000000ll); }
__device__ __forceinline__ double inf64() { return __longlong_as_double(0x7ff0000000000000ll); }

__device__ __forceinline__ bool finite_positive(double v) {
  return v > 0.0 && v < inf64();
}

// Select element k of four values held in registers (k differs per lane, so a
// private array would be spilled to scratch memory; compares + selects stay in
// VGPRs).
template <typename T>
__device__ __forceinline__ T sel4(int k, T a0, T a1, T a2, T a3) {
  T lo = (k & 1) ? a1 : a0;
  T hi = (k & 1) ? a3 : a2;
  return (k & 2) ? hi : lo;
}

// The network and collective of one scenario, in registers.
struct Scenario {
  int D;           // dimensions in use, 1..4
  uint32_t C;      // chunks per collective
  uint32_t P[kMaxDims];
  double coef[kMaxDims];  // seconds per resident byte: ((P-1)/P)/bw  (Sec. 4.5)
  double fix[kMaxDims];   // fixed delay per stage on the dimension (A_K of Sec. 4.5), 0 if none
  bool has_fix;           // the batch carries fixed delays
  int ctype;              // THEMIS_COLL_*
  bool valid;
};

// Loads scenario i of a batch and checks it (a1/a2 of the hot path).
__device__ __forceinline__ Scenario load_scenario(const themis_batch_t& b, uint64_t i) {
  Scenario s;
  s.D = b.ndims[i];
  s.C = b.chunks[i];
  s.valid = (s.D >= 1 && s.D <= kMaxDims) && (s.C >= 1u && s.C <= b.max_chunks);
  s.has_fix = b.fixed_delay != nullptr;
  s.ctype = b.collective_type ? (int)b.collective_type[i] : THEMIS_COLL_ALL_REDUCE;
  if (s.ctype > THEMIS_COLL_ALL_GATHER) { s.valid = false; s.ctype = THEMIS_COLL_ALL_REDUCE; }
#pragma unroll
  for (int k = 0; k < kMaxDims; ++k) {
    uint32_t p = b.npus[(size_t)k * b.n + i];
    double bw = b.bw[(size_t)k * b.n + i];
    bool used = k < s.D;
    double fx = (s.has_fix && used) ? b.fixed_delay[(size_t)k * b.n + i] : 0.0;
    if (used && !(p >= 2u && finite_positive(bw) && fx >= 0.0 && fx < inf64())) s.valid = false;
    if (!used || !s.valid) { p = 2u; bw = 1.0; fx = 0.0; }
    s.fix[k] = fx;
    s.P[k] = p;
    double pd = (double)p;
    s.coef[k] = ((double)(p - 1u) / pd) / bw;
  }
  return s;
}

// Decodes and checks an order code: fields 0..D-1 must be a permutation of
// 0..D-1 and the fields above must be zero.
__device__ __forceinline__ bool order_code_ok(uint32_t code, int D) {
  uint32_t seen = 0;
  bool ok = true;
#pragma unroll
  for (int j = 0; j < kMaxDims; ++j) {
    uint32_t k = (code >> (2 * j)) & 3u;
    if (j < D) {
      if ((int)k >= D || (seen & (1u << k))) ok = false;
      seen |= 1u << k;
    } else if (k != 0u) {
      ok = false;
    }
  }
  return ok;
}

// Order code with its D fields reversed.
__device__ __forceinline__ uint32_t reverse_code(uint32_t code, int D) {
  uint32_t r = 0;
#pragma unroll
  for (int j = 0; j < kMaxDims; ++j)
    if (j < D) r |= ((code >> (2 * j)) & 3u) << (2 * (D - 1 - j));
  return r;
}

// Tracker contents before the first chunk: the fixed delay A_K of the
// collective type (Sec. 4.5), i.e. one stage per dimension, two for All-Reduce.
__device__ __forceinline__ double tracker_start(const Scenario& s, int k) {
  return s.ctype == THEMIS_COLL_ALL_REDUCE ? s.fix[k] + s.fix[k] : s.fix[k];
}

// One step of Alg. 1's Scheduler.Schedule for the chunk that comes next, given
// the Dim Load Tracker contents load[0..3] (unused dimensions hold +inf on
// entry and are left untouched).  Returns the order code and adds the chunk's
// Reduce-Scatter + All-Gather time to the tracker.
//
//   thr_abs : threshold in seconds when rel == false
//   thr_rel : fraction of (chunk * coef[kmin]) when rel == true
__device__ __forceinline__ uint32_t schedule_chunk(const Scenario& s, double chunk,
                                                   bool themis, bool rel, double thr,
                                                   double (&load)[kMaxDims]) {
  const int D = s.D;
  // least and most loaded dimension; ties keep the lower index
  int kmin = 0;
  double lo = load[0], hi = load[0];
#pragma unroll
  for (int k = 1; k < kMaxDims; ++k) {
    if (k < D) {
      if (load[k] < lo) { lo = load[k]; kmin = k; }
      if (load[k] > hi) hi = load[k];
    }
  }
  const bool gather = s.ctype == THEMIS_COLL_ALL_GATHER;
  double t = thr;
  if (rel) {
    double cmin = sel4(kmin, s.coef[0], s.coef[1], s.coef[2], s.coef[3]);
    double whole = chunk;
    if (gather) whole = chunk * (double)sel4(kmin, s.P[0], s.P[1], s.P[2], s.P[3]);
    t = thr * (whole * cmin);
  }
  uint32_t code = 0xE4u;  // identity 0,1,2,3
  if (themis && !((hi - lo) < t)) {
    // rank of every dimension in the stable ascending order of the loads:
    // dimension a (a < b) goes after b only if its load is strictly larger.
    int rank[kMaxDims] = {0, 0, 0, 0};
#pragma unroll
    for (int a = 0; a < kMaxDims; ++a) {
#pragma unroll
      for (int bb = a + 1; bb < kMaxDims; ++bb) {
        bool after = load[a] > load[bb];
        rank[a] += after ? 1 : 0;
        rank[bb] += after ? 0 : 1;
      }
    }
    code = 0;
#pragma unroll
    for (int k = 0; k < kMaxDims; ++k) code |= (uint32_t)k << (2 * rank[k]);
  }
  code &= (1u << (2 * D)) - 1u;
  if (gather) code = reverse_code(code, D);  // descending loads, dimD..dim1 when tied

  // latency model + tracker update along the chosen order
  const bool twice = s.ctype == THEMIS_COLL_ALL_REDUCE;  // RS now and AG later on the same bytes
  double x = chunk;
#pragma unroll
  for (int j = 0; j < kMaxDims; ++j) {
    if (j < D) {
      int k = (code >> (2 * j)) & 3;
      double ck = sel4(k, s.coef[0], s.coef[1], s.coef[2], s.coef[3]);
      double pk = (double)sel4(k, s.P[0], s.P[1], s.P[2], s.P[3]);
      if (gather) x = x * pk;
      double tj = x * ck;
      double add = twice ? tj + tj : tj;
#pragma unroll
      for (int kk = 0; kk < kMaxDims; ++kk)
        if (kk == k) load[kk] = load[kk] + add;
      if (!gather) x = x / pk;
    }
  }
  return code;
}

}  // namespace themis
