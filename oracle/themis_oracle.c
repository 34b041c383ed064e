/*
 * themis_oracle.c -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, single-threaded CPU statement of what the batched Themis
 * evaluator computes (arXiv 2110.04478): the latency model, the greedy chunk
 * scheduler of Alg. 1 and the per-dimension queue simulation.  It exists so
 * that the GPU library can be checked against it; only the tests, the smoke
 * check and the benchmark's CPU-baseline leg may call it.  It shares no code,
 * header, table or helper with the GPU path.
 *
 * Everything is IEEE binary64, round to nearest, compiled with
 * -ffp-contract=off; no blocking, no reordering, no cleverness: each function
 * walks the paper's steps in the paper's order.
 *
 * Pinning (tests/test_oracle_pins.py): 1-D ring closed forms (All-Reduce
 * 2(P-1)/P*S/B, with fixed delays, stand-alone Reduce-Scatter / All-Gather),
 * the stage-time ratios and chunk orders of the paper's 4x4 worked example,
 * Alg. 1 replayed with exact rationals, load conservation, the
 * balanced-bandwidth reduction to the baseline order, an independent
 * exact-rational checker that rebuilds every start and end time from the
 * reported per-dimension orders and verifies work conservation and FIFO / SCF
 * conformance, brute force over all per-chunk orders for tiny C, hand values
 * for the derived metrics and the provisioning classes, hand values and the
 * library minimum / argmin for the best threshold of a sweep.  The batch drivers
 * (tests/test_oracle_batch_pins.py): hand-derived times for every column of a
 * sweep and for shared and per-scenario thresholds, each column rebuilt by the
 * schedule checker under its own policy, ragged traces with rows longer than
 * the chunk count replayed with rationals and checked operation by operation,
 * the 1-D sum of closed forms over a trace, hand values for the trace totals
 * of the metrics, per-scenario delays and collective types.  The beam search
 * (tests/test_oracle_beam_pins.py): equality with the exhaustive search when
 * nothing is dropped, a restatement of the procedure in Python whose scores the
 * rational checker confirms (ties by assignment number on dyadic networks,
 * delays as long as the stages for the size a partial schedule is scored at),
 * the bounds by the greedy plan and by the optimum, a width-1 step by hand.
 * The completion time
 * that the paper's timing figure would show for Themis on the worked example
 * is "parity unpinned": the figure is not available in text form.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define TO_MAX_DIMS 4

enum { TO_INTER_BASELINE = 0, TO_INTER_THEMIS = 1 };
enum { TO_INTRA_FIFO = 0, TO_INTRA_SCF = 1 };
enum { TO_THR_ABS = 0, TO_THR_REL = 1 };
/* CollectiveType of Alg. 1 */
enum { TO_ALL_REDUCE = 0, TO_REDUCE_SCATTER = 1, TO_ALL_GATHER = 2 };

/* ------------------------------------------------------------------------ */
/* Latency model (Sec. 4.5: latency of chunk i on dim K is n_K^i * B_K, with
 * n = (P-1)/P * resident size (footnote there) and B_K the per-byte latency,
 * i.e. the inverse of the dimension's bandwidth).                           */
/* ------------------------------------------------------------------------ */
void to_latency_coef(int ndims, const uint32_t *npus, const double *bw,
                     double *coef)
{
  for (int k = 0; k < ndims; ++k) {
    double p = (double)npus[k];
    coef[k] = ((double)(npus[k] - 1u) / p) / bw[k];
  }
}


static int finite_positive(double v) { return isfinite(v) && v > 0.0; }

/* Fixed per-stage delays (A_K = steps * step latency, Sec. 4.5) are optional;
 * when given they must be finite and not negative. */
int to_fixed_delay_valid(int ndims, const double *fixed_delay)
{
  if (!fixed_delay) return 1;
  for (int k = 0; k < ndims && k < TO_MAX_DIMS; ++k)
    if (!(isfinite(fixed_delay[k]) && fixed_delay[k] >= 0.0)) return 0;
  return 1;
}

/* A scenario is valid when the network and the collective make sense. */
int to_network_valid(int ndims, const uint32_t *npus, const double *bw)
{
  if (ndims < 1 || ndims > TO_MAX_DIMS) return 0;
  for (int k = 0; k < ndims; ++k) {
    if (npus[k] < 2u) return 0;
    if (!finite_positive(bw[k])) return 0;
  }
  return 1;
}

/* Decode an order code into dims[0..D-1]; returns 0 if it is not a
 * permutation of 0..D-1 with zero upper fields. */
int to_decode_order(int ndims, uint8_t code, int *dims)
{
  int seen = 0;
  for (int j = 0; j < TO_MAX_DIMS; ++j) {
    int k = (code >> (2 * j)) & 3;
    if (j < ndims) {
      if (k >= ndims || (seen & (1 << k))) return 0;
      seen |= 1 << k;
      dims[j] = k;
    } else if (k != 0) {
      return 0;
    }
  }
  return 1;
}

static uint8_t encode_order(int ndims, const int *dims)
{
  unsigned code = 0;
  for (int j = 0; j < ndims; ++j) code |= (unsigned)dims[j] << (2 * j);
  return (uint8_t)code;
}

/* ------------------------------------------------------------------------ */
/* Alg. 1.  Plans one collective of `size_bytes` split into C equal chunks.
 *   orders[C]        : order code of every chunk
 *   loads[4]         : final Dim Load Tracker contents
 *   stage_time[C][4] : (may be NULL) time of chunk i on dimension k
 * Returns 1 on success, 0 if the inputs are invalid (nothing written).       */
/* ------------------------------------------------------------------------ */
int to_plan(int ndims, const uint32_t *npus, const double *bw,
            const double *fixed_delay, int ctype, double size_bytes, uint32_t C,
            int inter_policy, int threshold_mode, double threshold,
            uint8_t *orders, double *loads, double *stage_time)
{
  if (!to_network_valid(ndims, npus, bw)) return 0;
  if (ctype < TO_ALL_REDUCE || ctype > TO_ALL_GATHER) return 0;
  if (!to_fixed_delay_valid(ndims, fixed_delay)) return 0;
  if (!finite_positive(size_bytes) || C < 1u) return 0;
  if (!(threshold >= 0.0)) return 0; /* also rejects NaN */
  if (threshold_mode == TO_THR_REL && !isfinite(threshold)) return 0;

  double coef[TO_MAX_DIMS];
  to_latency_coef(ndims, npus, bw, coef);

  /* Splitter: equal chunks (Alg. 1 line 3). */
  double chunk = size_bytes / (double)C;

  /* Dim Load Tracker reset to the fixed delay A_K of the collective type on
   * each dimension (Alg. 1 line 2, Sec. 4.5): an All-Reduce pays the per-stage
   * delay once for its Reduce-Scatter and once for its All-Gather. */
  double load[TO_MAX_DIMS] = {0.0, 0.0, 0.0, 0.0};
  if (fixed_delay)
    for (int k = 0; k < ndims; ++k)
      load[k] = (ctype == TO_ALL_REDUCE) ? fixed_delay[k] + fixed_delay[k]
                                         : fixed_delay[k];

  for (uint32_t i = 0; i < C; ++i) {
    /* Scheduler.Schedule: current loads, their min and max (line 18-19). */
    int kmin = 0;
    double lo = load[0], hi = load[0];
    for (int k = 1; k < ndims; ++k) {
      if (load[k] < lo) { lo = load[k]; kmin = k; }
      if (load[k] > hi) hi = load[k];
    }
    /* Threshold relative to "an RS/AG of a whole chunk on the least-loaded
     * dimension" (Sec. 5.3): an All-Gather stage that starts from `chunk`
     * bytes moves (P-1) * chunk of them. */
    double thr = threshold;
    if (threshold_mode == TO_THR_REL)
      thr = (ctype == TO_ALL_GATHER)
                ? threshold * ((chunk * (double)npus[kmin]) * coef[kmin])
                : threshold * (chunk * coef[kmin]);

    /* ascending order first (the Reduce-Scatter schedule, Alg. 1 line 23); an
     * All-Gather takes it in reverse (line 25: descending loads, and
     * dimD..dim1 as its baseline, Sec. 2.3) */
    int order[TO_MAX_DIMS];
    for (int k = 0; k < ndims; ++k) order[k] = k; /* baseline: dim1..dimD */
    if (inter_policy != TO_INTER_BASELINE && !((hi - lo) < thr)) {
      /* indices of the loads sorted ascending, stable: insertion sort that
       * moves an element only past strictly larger loads. */
      for (int a = 1; a < ndims; ++a) {
        int k = order[a];
        int b = a - 1;
        while (b >= 0 && load[order[b]] > load[k]) {
          order[b + 1] = order[b];
          --b;
        }
        order[b + 1] = k;
      }
    }

    if (ctype == TO_ALL_GATHER) {
      for (int a = 0, b = ndims - 1; a < b; ++a, --b) {
        int tmp = order[a]; order[a] = order[b]; order[b] = tmp;
      }
    }

    /* Latency Model + tracker update (lines 28-30).  The chunk shrinks by
     * P_k after its Reduce-Scatter on dimension k (Sec. 2.1); in an All-Reduce
     * its All-Gather on k later moves the same bytes, so the dimension is
     * charged twice.  A stand-alone All-Gather grows the chunk by P_k per
     * stage and moves (P_k-1)/P_k of the grown size. */
    double x = chunk;
    for (int j = 0; j < ndims; ++j) {
      int k = order[j];
      double t;
      if (ctype == TO_ALL_GATHER) {
        x = x * (double)npus[k];
        t = x * coef[k];
        load[k] = load[k] + t;
      } else {
        t = x * coef[k];
        load[k] = load[k] + ((ctype == TO_ALL_REDUCE) ? (t + t) : t);
        x = x / (double)npus[k];
      }
      if (stage_time) stage_time[(size_t)i * TO_MAX_DIMS + k] = t;
    }
    orders[i] = encode_order(ndims, order);
  }
  for (int k = 0; k < TO_MAX_DIMS; ++k) loads[k] = (k < ndims) ? load[k] : 0.0;
  return 1;
}

/* ------------------------------------------------------------------------ */
/* Queue simulation (Sec. 4.3 policies, Sec. 4.6.2 consistency simulation).
 *
 * n_coll collectives share the D servers.  Collective q has C chunks of
 * coll_size[q]/C bytes, all released at release[q] (NULL = 0); chunk i of
 * collective q has id g = q*C + i and order code orders[g].
 *
 *   t_done             : time the last stage of the last chunk ends
 *   coll_done[n_coll]  : (may be NULL) same per collective
 *   queue_order[4][2G] : (may be NULL) per dimension, the executed operations
 *                        (g << 1 | phase) in execution order
 *   busy[4]            : (may be NULL) total service time per dimension
 * fixed_delay[4] (may be NULL) is added to every stage's time on that
 * dimension (Sec. 4.5: A_K + N_K * B_K + idle_K).
 * Returns 1 on success, 0 on invalid input.                                  */
/* ------------------------------------------------------------------------ */
typedef struct {
  int stage;      /* 0..2D: next stage to run (2D = finished)              */
  int running;    /* currently being served                                */
  double size;    /* resident bytes before the next stage                  */
  double arrival; /* when it joined the queue it is waiting in             */
  int order[TO_MAX_DIMS];
  double t[TO_MAX_DIMS]; /* service time on dimension k (RS == AG)          */
} to_chunk;

static int stage_dim(const to_chunk *c, int ndims)
{
  return (c->stage < ndims) ? c->order[c->stage]
                            : c->order[2 * ndims - 1 - c->stage];
}

/* stages of one chunk: an All-Reduce runs D Reduce-Scatter and D All-Gather
 * stages, the stand-alone collectives only their own D (Sec. 2.3 footnote) */
static int stage_count(int ctype, int ndims)
{
  return (ctype == TO_ALL_REDUCE) ? 2 * ndims : ndims;
}

/* Does chunk a (id ga) go before chunk b (id gb) in one dimension's queue? */
static int goes_first(int intra_policy, const to_chunk *a, uint32_t ga,
                      const to_chunk *b, uint32_t gb)
{
  if (intra_policy == TO_INTRA_SCF) {
    if (a->size < b->size) return 1;
    if (a->size > b->size) return 0;
  }
  if (a->arrival < b->arrival) return 1;
  if (a->arrival > b->arrival) return 0;
  return ga < gb;
}

int to_simulate(int ndims, const uint32_t *npus, const double *bw,
                const double *fixed_delay, int ctype, uint32_t n_coll, const double *coll_size,
                const double *release, uint32_t C, int intra_policy,
                const uint8_t *orders, double *t_done, double *coll_done,
                uint32_t *queue_order, double *busy)
{
  if (!to_network_valid(ndims, npus, bw)) return 0;
  if (!to_fixed_delay_valid(ndims, fixed_delay)) return 0;
  if (n_coll < 1u || C < 1u) return 0;
  if (ctype < TO_ALL_REDUCE || ctype > TO_ALL_GATHER) return 0;
  const int last = stage_count(ctype, ndims);
  for (uint32_t q = 0; q < n_coll; ++q) {
    if (!finite_positive(coll_size[q])) return 0;
    if (release && !(isfinite(release[q]) && release[q] >= 0.0)) return 0;
  }
  uint32_t G = n_coll * C;

  double coef[TO_MAX_DIMS];
  to_latency_coef(ndims, npus, bw, coef);

  to_chunk *ch = (to_chunk *)calloc(G, sizeof(to_chunk));
  if (!ch) return 0;
  for (uint32_t q = 0; q < n_coll; ++q) {
    double chunk = coll_size[q] / (double)C;
    for (uint32_t i = 0; i < C; ++i) {
      uint32_t g = q * C + i;
      to_chunk *c = &ch[g];
      if (!to_decode_order(ndims, orders[g], c->order)) { free(ch); return 0; }
      c->stage = 0;
      c->running = 0;
      c->size = chunk;
      c->arrival = release ? release[q] : 0.0;
      /* stage times exactly as the planner's latency model computes them */
      double x = chunk;
      for (int j = 0; j < ndims; ++j) {
        int k = c->order[j];
        if (ctype == TO_ALL_GATHER) {
          x = x * (double)npus[k];
          c->t[k] = x * coef[k];
        } else {
          c->t[k] = x * coef[k];
          x = x / (double)npus[k];
        }
      }
    }
  }

  int serving[TO_MAX_DIMS];      /* chunk id being served, or -1 */
  double finish[TO_MAX_DIMS];
  uint32_t executed[TO_MAX_DIMS] = {0, 0, 0, 0};
  double busy_acc[TO_MAX_DIMS] = {0.0, 0.0, 0.0, 0.0};
  for (int k = 0; k < TO_MAX_DIMS; ++k) { serving[k] = -1; finish[k] = 0.0; }
  if (coll_done) for (uint32_t q = 0; q < n_coll; ++q) coll_done[q] = 0.0;

  double now = 0.0;
  double last_done = 0.0;
  for (;;) {
    /* (i) every idle dimension starts the best chunk waiting for it */
    for (int k = 0; k < ndims; ++k) {
      if (serving[k] >= 0) continue;
      int best = -1;
      for (uint32_t g = 0; g < G; ++g) {
        const to_chunk *c = &ch[g];
        if (c->stage >= last || c->running) continue;
        if (stage_dim(c, ndims) != k) continue;
        if (c->arrival > now) continue; /* not released yet */
        if (best < 0 || goes_first(intra_policy, c, g, &ch[best], (uint32_t)best))
          best = (int)g;
      }
      if (best < 0) continue;
      to_chunk *c = &ch[best];
      c->running = 1;
      serving[k] = best;
      /* stage time = fixed delay of one stage on k + bytes * per-byte latency */
      double service = fixed_delay ? fixed_delay[k] + c->t[k] : c->t[k];
      finish[k] = now + service;
      busy_acc[k] = busy_acc[k] + service;
      if (queue_order) {
        uint32_t phase = (ctype == TO_ALL_GATHER || c->stage >= ndims) ? 1u : 0u;
        queue_order[(size_t)k * 2u * G + executed[k]] = ((uint32_t)best << 1) | phase;
      }
      executed[k]++;
    }

    /* (ii)+(iii) next instant at which something happens */
    double next = INFINITY;
    for (int k = 0; k < ndims; ++k)
      if (serving[k] >= 0 && finish[k] < next) next = finish[k];
    for (uint32_t g = 0; g < G; ++g) {
      const to_chunk *c = &ch[g];
      if (c->stage < last && !c->running && c->arrival > now &&
          c->arrival < next)
        next = c->arrival;
    }
    if (next == INFINITY) break;
    now = next;

    /* (iv) deliver every completion that falls on this instant */
    for (int k = 0; k < ndims; ++k) {
      if (serving[k] < 0 || finish[k] != now) continue;
      uint32_t g = (uint32_t)serving[k];
      to_chunk *c = &ch[g];
      if (ctype != TO_ALL_GATHER && c->stage < ndims)
        c->size = c->size / (double)npus[k]; /* Reduce-Scatter stage */
      else
        c->size = c->size * (double)npus[k]; /* All-Gather stage */
      c->stage++;
      c->running = 0;
      c->arrival = now;
      serving[k] = -1;
      if (c->stage == last) {
        last_done = now;
        if (coll_done) coll_done[g / C] = now;
      }
    }
  }

  free(ch);
  /* A stage time or a clock value that overflowed binary64 leaves the model:
   * such a scenario is reported like an invalid one.  Every clock value is at
   * most the completion time and every stage time at most its dimension's
   * busy time, so these sums being finite covers all of them. */
  if (!isfinite(last_done)) return 0;
  for (int k = 0; k < ndims; ++k)
    if (!isfinite(busy_acc[k])) return 0;
  *t_done = last_done;
  if (busy) for (int k = 0; k < TO_MAX_DIMS; ++k) busy[k] = busy_acc[k];
  return 1;
}

/* ------------------------------------------------------------------------ */
/* Batch drivers over structure-of-arrays inputs (host pointers): scenario i
 * of n, per-dimension fields laid out [4][n].  Only scenarios in
 * [begin, end) are processed so that a caller may fan ranges out to threads. */
/* ------------------------------------------------------------------------ */
static void gather_network(uint64_t n, uint64_t i, const uint32_t *npus,
                           const double *bw, uint32_t *p, double *b)
{
  for (int k = 0; k < TO_MAX_DIMS; ++k) {
    p[k] = npus[(size_t)k * n + i];
    b[k] = bw[(size_t)k * n + i];
  }
}

/* fixed_delay is [4][n] or NULL; returns a pointer to f[4] or NULL */
static const double *gather_fixed(uint64_t n, uint64_t i,
                                  const double *fixed_delay, double *f)
{
  if (!fixed_delay) return NULL;
  for (int k = 0; k < TO_MAX_DIMS; ++k) f[k] = fixed_delay[(size_t)k * n + i];
  return f;
}

/* orders: [n][slots] with slots = max_chunks * max(1,max_coll); loads [4][n]
 * (may be NULL).  n_coll/coll_size NULL = one collective of size_bytes[i]. */
void to_plan_batch(uint64_t n, uint64_t begin, uint64_t end,
                   uint32_t max_chunks, int threshold_mode,
                   const uint8_t *ndims, const uint32_t *npus,
                   const double *bw, const double *size_bytes,
                   const uint32_t *chunks, const uint8_t *inter_policy,
                   const double *threshold, const double *fixed_delay,
                   const uint8_t *collective_type, uint32_t max_coll,
                   const uint32_t *n_coll, const double *coll_size,
                   uint8_t *orders, double *loads)
{
  uint32_t mc = (n_coll && max_coll > 0u) ? max_coll : 1u;
  size_t slots = (size_t)max_chunks * mc;
  for (uint64_t i = begin; i < end; ++i) {
    uint32_t p[TO_MAX_DIMS];
    double b[TO_MAX_DIMS], ld[TO_MAX_DIMS] = {0, 0, 0, 0}, fx[TO_MAX_DIMS];
    gather_network(n, i, npus, bw, p, b);
    const double *fixed = gather_fixed(n, i, fixed_delay, fx);
    uint8_t *row = orders + (size_t)i * slots;
    memset(row, 0xFF, slots);
    uint32_t C = chunks[i];
    uint32_t Q = n_coll ? n_coll[i] : 1u;
    int ok = (C >= 1u && C <= max_chunks && Q >= 1u && Q <= mc);
    for (uint32_t q = 0; ok && q < Q; ++q) {
      double S = n_coll ? coll_size[(size_t)q * n + i] : size_bytes[i];
      ok = to_plan((int)ndims[i], p, b, fixed,
                   collective_type ? (int)collective_type[i] : TO_ALL_REDUCE,
                   S, C, (int)inter_policy[i], threshold_mode, threshold[i],
                   row + (size_t)q * max_chunks, ld, NULL);
    }
    if (!ok) {
      memset(row, 0xFF, slots);
      for (int k = 0; k < TO_MAX_DIMS; ++k) ld[k] = NAN;
    }
    if (loads)
      for (int k = 0; k < TO_MAX_DIMS; ++k) loads[(size_t)k * n + i] = ld[k];
  }
}

/* queue_order: NULL or [n][4][2*slots] uint16 (unused entries 0xFFFF);
 * busy: NULL or [4][n]; t_done [n]. */
void to_simulate_batch(uint64_t n, uint64_t begin, uint64_t end,
                       uint32_t max_chunks, const uint8_t *ndims,
                       const uint32_t *npus, const double *bw,
                       const double *size_bytes, const uint32_t *chunks,
                       const uint8_t *intra_policy, const double *fixed_delay,
                       const uint8_t *collective_type, uint32_t max_coll,
                       const uint32_t *n_coll,
                       const double *coll_size, const double *release_time,
                       const uint8_t *orders,
                       double *t_done, uint16_t *queue_order, double *busy)
{
  uint32_t mc = (n_coll && max_coll > 0u) ? max_coll : 1u;
  size_t slots = (size_t)max_chunks * mc;
  uint32_t *qo = queue_order
      ? (uint32_t *)malloc(sizeof(uint32_t) * TO_MAX_DIMS * 2u * slots) : NULL;
  double *cs = (double *)malloc(sizeof(double) * mc);
  double *rl = (double *)malloc(sizeof(double) * mc);
  uint8_t *od = (uint8_t *)malloc(slots);
  for (uint64_t i = begin; i < end; ++i) {
    uint32_t p[TO_MAX_DIMS];
    double b[TO_MAX_DIMS], bz[TO_MAX_DIMS] = {0, 0, 0, 0}, fx[TO_MAX_DIMS];
    gather_network(n, i, npus, bw, p, b);
    const double *fixed = gather_fixed(n, i, fixed_delay, fx);
    uint32_t C = chunks[i];
    uint32_t Q = n_coll ? n_coll[i] : 1u;
    int D = (int)ndims[i];
    int ok = (C >= 1u && C <= max_chunks && Q >= 1u && Q <= mc);
    double T = NAN;
    if (ok) {
      for (uint32_t q = 0; q < Q; ++q) {
        cs[q] = n_coll ? coll_size[(size_t)q * n + i] : size_bytes[i];
        rl[q] = (n_coll && release_time) ? release_time[(size_t)q * n + i] : 0.0;
        /* compact the [max_coll][max_chunks] rows into q*C + i numbering */
        memcpy(od + (size_t)q * C,
               orders + (size_t)i * slots + (size_t)q * max_chunks, C);
      }
      ok = to_simulate(D, p, b, fixed,
                       collective_type ? (int)collective_type[i] : TO_ALL_REDUCE,
                       Q, cs, rl, C, (int)intra_policy[i], od, &T, NULL, qo, bz);
    }
    if (!ok) {
      T = NAN;
      for (int k = 0; k < TO_MAX_DIMS; ++k) bz[k] = NAN;
    }
    t_done[i] = T;
    if (busy)
      for (int k = 0; k < TO_MAX_DIMS; ++k) busy[(size_t)k * n + i] = bz[k];
    if (queue_order) {
      uint16_t *row = queue_order + (size_t)i * TO_MAX_DIMS * 2u * slots;
      memset(row, 0xFF, sizeof(uint16_t) * TO_MAX_DIMS * 2u * slots);
      if (ok) {
        uint32_t G = Q * C;
        /* an All-Reduce runs two operations per chunk and dimension, the
         * stand-alone collectives one */
        uint32_t per_dim = (collective_type && collective_type[i] != TO_ALL_REDUCE) ? G : 2u * G;
        for (int k = 0; k < D; ++k)
          for (uint32_t e = 0; e < per_dim; ++e)
            row[(size_t)k * 2u * slots + e] = (uint16_t)qo[(size_t)k * 2u * G + e];
      }
    }
  }
  free(qo); free(cs); free(rl); free(od);
}

/* Fused plan + simulate for scenario x threshold x scheduler.
 * policy_mask bits: 1 baseline+FIFO, 2 Themis+FIFO, 4 Themis+SCF, evaluated
 * in ascending bit order.  thr: [n_thr] shared, or [n_thr][n] when
 * thr_per_scenario.  t_done: [n][n_thr][n_pol]. */
void to_sweep(uint64_t n, uint64_t begin, uint64_t end, uint32_t max_chunks,
              int threshold_mode, const uint8_t *ndims, const uint32_t *npus,
              const double *bw, const double *size_bytes,
              const uint32_t *chunks, const double *fixed_delay, int n_thr,
              const double *thr, int thr_per_scenario, unsigned policy_mask,
              double *t_done)
{
  int n_pol = 0;
  for (int bit = 0; bit < 3; ++bit) if (policy_mask & (1u << bit)) ++n_pol;
  uint8_t *od = (uint8_t *)malloc(max_chunks);
  for (uint64_t i = begin; i < end; ++i) {
    uint32_t p[TO_MAX_DIMS];
    double b[TO_MAX_DIMS], ld[TO_MAX_DIMS], fx[TO_MAX_DIMS];
    gather_network(n, i, npus, bw, p, b);
    const double *fixed = gather_fixed(n, i, fixed_delay, fx);
    uint32_t C = chunks[i];
    for (int a = 0; a < n_thr; ++a) {
      double th = thr_per_scenario ? thr[(size_t)a * n + i] : thr[a];
      int col = 0;
      for (int bit = 0; bit < 3; ++bit) {
        if (!(policy_mask & (1u << bit))) continue;
        int inter = (bit == 0) ? TO_INTER_BASELINE : TO_INTER_THEMIS;
        int intra = (bit == 2) ? TO_INTRA_SCF : TO_INTRA_FIFO;
        double T = NAN;
        int ok = (C >= 1u && C <= max_chunks);
        if (ok)
          ok = to_plan((int)ndims[i], p, b, fixed, TO_ALL_REDUCE, size_bytes[i],
                       C, inter, threshold_mode, th, od, ld, NULL);
        if (ok) {
          double S = size_bytes[i];
          ok = to_simulate((int)ndims[i], p, b, fixed, TO_ALL_REDUCE, 1u, &S, NULL,
                           C, intra, od, &T, NULL, NULL, NULL);
        }
        if (!ok) T = NAN;
        t_done[((size_t)i * n_thr + a) * n_pol + col] = T;
        ++col;
      }
    }
  }
  free(od);
}

/* ------------------------------------------------------------------------ */
/* Derived quantities of the paper's evaluation.
 *   utilization : average bandwidth utilisation (Sec. 3): the utilisation of
 *                 every dimension, N_K / (T * BW_K) with N_K = transfer_K *
 *                 BW_K the bytes it moved, weighted by its bandwidth:
 *                 sum_K transfer_K * BW_K / (T * sum_K BW_K)
 *   ideal       : Table 3 "Ideal": collective size / total bandwidth
 * transfer[4] are the seconds each dimension spent moving bytes (the
 * bandwidth part of its load).                                              */
/* ------------------------------------------------------------------------ */
void to_metrics(int ndims, const double *bw, double total_bytes, double t_done,
                const double *transfer, double *utilization, double *ideal)
{
  double num = 0.0, den = 0.0;
  for (int k = 0; k < ndims; ++k) {
    num = num + transfer[k] * bw[k];
    den = den + bw[k];
  }
  *utilization = num / (t_done * den);
  *ideal = total_bytes / den;
}

/* t_done [n], transfer [4][n] -> utilization [n], ideal [n] */
void to_metrics_batch(uint64_t n, uint64_t begin, uint64_t end,
                      const uint8_t *ndims, const double *bw,
                      const double *size_bytes, uint32_t max_coll,
                      const uint32_t *n_coll, const double *coll_size,
                      const double *t_done, const double *transfer,
                      double *utilization, double *ideal)
{
  (void)max_coll;
  for (uint64_t i = begin; i < end; ++i) {
    double b[TO_MAX_DIMS], tr[TO_MAX_DIMS];
    for (int k = 0; k < TO_MAX_DIMS; ++k) {
      b[k] = bw[(size_t)k * n + i];
      tr[k] = transfer[(size_t)k * n + i];
    }
    double total = 0.0;
    if (n_coll) for (uint32_t q = 0; q < n_coll[i]; ++q) total = total + coll_size[(size_t)q * n + i];
    else total = size_bytes[i];
    int D = (int)ndims[i];
    if (D < 1 || D > TO_MAX_DIMS) { utilization[i] = NAN; ideal[i] = NAN; continue; }
    to_metrics(D, b, total, t_done[i], tr, &utilization[i], &ideal[i]);
  }
}

/* ------------------------------------------------------------------------ */
/* Exhaustive search (Sec. 4.1, observation 2): every chunk may take any of
 * the D! dimension orders, so a collective has (D!)^C schedules once the
 * All-Gather order of an All-Reduce is tied to the reverse of its
 * Reduce-Scatter order.  For tiny C all of them are simulated; the best
 * completion time and the first assignment that reaches it are returned.
 *
 * Assignment number a gives chunk c the permutation with lexicographic index
 * (a / (D!)^c) mod D! of (0, 1, .., D-1).
 * Returns 1 on success; 0 if the inputs are invalid or (D!)^C > max_assign. */
/* ------------------------------------------------------------------------ */
static void nth_permutation(int ndims, uint32_t idx, int *dims)
{
  int pool[TO_MAX_DIMS] = {0, 1, 2, 3};
  uint32_t fact = 1;
  for (int j = 2; j < ndims; ++j) fact *= (uint32_t)j; /* (D-1)! */
  for (int j = 0; j < ndims; ++j) {
    uint32_t pick = idx / fact;
    idx %= fact;
    dims[j] = pool[pick];
    for (int m = (int)pick; m < ndims - 1 - j; ++m) pool[m] = pool[m + 1];
    if (ndims - 1 - j > 0) fact /= (uint32_t)(ndims - 1 - j);
  }
}

int to_search(int ndims, const uint32_t *npus, const double *bw,
              const double *fixed_delay, int ctype, double size_bytes,
              uint32_t C, int intra_policy, uint64_t max_assign, double *best_t,
              uint8_t *best_orders, uint64_t *n_assign)
{
  if (!to_network_valid(ndims, npus, bw) || C < 1u) return 0;
  uint64_t F = 1;
  for (int j = 2; j <= ndims; ++j) F *= (uint64_t)j;
  uint64_t total = 1;
  for (uint32_t c = 0; c < C; ++c) {
    if (total > max_assign / F) return 0; /* too many schedules */
    total *= F;
  }
  uint8_t *od = (uint8_t *)malloc(C);
  double best = INFINITY;
  int any = 0;
  for (uint64_t a = 0; a < total; ++a) {
    uint64_t rest = a;
    for (uint32_t c = 0; c < C; ++c) {
      int dims[TO_MAX_DIMS];
      nth_permutation(ndims, (uint32_t)(rest % F), dims);
      rest /= F;
      od[c] = encode_order(ndims, dims);
    }
    double T;
    if (!to_simulate(ndims, npus, bw, fixed_delay, ctype, 1u, &size_bytes, NULL,
                     C, intra_policy, od, &T, NULL, NULL, NULL)) {
      free(od);
      return 0;
    }
    if (!any || T < best) { /* strict: the first best assignment wins */
      best = T;
      any = 1;
      memcpy(best_orders, od, C);
    }
  }
  free(od);
  *best_t = best;
  if (n_assign) *n_assign = total;
  return 1;
}

/* best_t [n], best_orders [n][max_chunks] (0xFF padded / on failure) */
void to_search_batch(uint64_t n, uint64_t begin, uint64_t end,
                     uint32_t max_chunks, const uint8_t *ndims,
                     const uint32_t *npus, const double *bw,
                     const double *size_bytes, const uint32_t *chunks,
                     const uint8_t *intra_policy, const double *fixed_delay,
                     const uint8_t *collective_type, uint64_t max_assign,
                     double *best_t, uint8_t *best_orders)
{
  for (uint64_t i = begin; i < end; ++i) {
    uint32_t p[TO_MAX_DIMS];
    double b[TO_MAX_DIMS], fx[TO_MAX_DIMS];
    gather_network(n, i, npus, bw, p, b);
    const double *fixed = gather_fixed(n, i, fixed_delay, fx);
    uint8_t *row = best_orders + (size_t)i * max_chunks;
    memset(row, 0xFF, max_chunks);
    uint32_t C = chunks[i];
    double T = NAN;
    int ok = (C >= 1u && C <= max_chunks);
    if (ok)
      ok = to_search((int)ndims[i], p, b, fixed,
                     collective_type ? (int)collective_type[i] : TO_ALL_REDUCE,
                     size_bytes[i], C, (int)intra_policy[i], max_assign, &T, row,
                     NULL);
    if (!ok) { T = NAN; memset(row, 0xFF, max_chunks); }
    best_t[i] = T;
  }
}

/* ------------------------------------------------------------------------ */
/* Beam search over per-chunk orders (Sec. 4.1, observation 2 names the space
 * of per-chunk schedules; Sec. 4.2 settles for a greedy walk through it).
 * The chunks are given their orders one after the other, chunk 0 first.  A
 * partial schedule of m chunks is scored by the completion time of a
 * collective of just those m chunks -- of size_bytes if m == C, else of
 * (size_bytes / C) * m bytes -- simulated under intra_policy.  Every kept
 * partial schedule is extended by each of the D! orders for the next chunk,
 * and the `width` best extensions are kept: smaller time first, equal times in
 * ascending assignment number (chunk c's order has the lexicographic index
 * digit_c among the permutations of (0..D-1); the number of a partial
 * schedule is sum_c digit_c * (D!)^c, so the newest chunk's digit is the most
 * significant).  With width >= (D!)^C nothing is ever dropped and the result
 * is that of to_search.  The result of the search is the better of the best
 * full schedule of the beam and the schedule Alg. 1 gives under inter_policy /
 * threshold (the beam's on equal times), so it is never worse than the greedy
 * scheduler.
 * Returns 1 on success, 0 on invalid inputs or width outside 1..TO_MAX_BEAM. */
/* ------------------------------------------------------------------------ */
#define TO_MAX_BEAM 64

typedef struct {
  double t;
  uint32_t parent; /* position in the previous beam */
  uint32_t digit;  /* order of the newest chunk */
  uint32_t rank;   /* position of the parent's number among the previous beam's numbers */
} to_candidate;

/* a before b: smaller time, then smaller assignment number */
static int candidate_before(const to_candidate *a, const to_candidate *b)
{
  if (a->t != b->t) return a->t < b->t;
  if (a->digit != b->digit) return a->digit < b->digit;
  return a->rank < b->rank;
}

int to_beam_search(int ndims, const uint32_t *npus, const double *bw,
                   const double *fixed_delay, int ctype, double size_bytes,
                   uint32_t C, int inter_policy, int intra_policy,
                   int threshold_mode, double threshold, uint32_t width,
                   double *best_t, uint8_t *best_orders)
{
  if (!to_network_valid(ndims, npus, bw) || C < 1u) return 0;
  if (width < 1u || width > TO_MAX_BEAM) return 0;
  uint32_t F = 1;
  for (int j = 2; j <= ndims; ++j) F *= (uint32_t)j;

  /* beam[r]: digits of the r-th best partial schedule; numrank[r]: how many
   * of the beam's schedules have a smaller assignment number */
  uint8_t *beam = (uint8_t *)calloc((size_t)width * C, 1);
  uint8_t *next = (uint8_t *)calloc((size_t)width * C, 1);
  uint8_t *od = (uint8_t *)malloc(C);
  to_candidate *cand = (to_candidate *)malloc(sizeof(to_candidate) * width * F);
  uint32_t numrank[TO_MAX_BEAM], newrank[TO_MAX_BEAM];
  double beam_t[TO_MAX_BEAM];
  uint32_t live = 1; /* the empty schedule */
  numrank[0] = 0;
  int ok = 1;
  for (uint32_t m = 1; ok && m <= C; ++m) {
    double size_m = (m == C) ? size_bytes : (size_bytes / (double)C) * (double)m;
    uint32_t nc = 0;
    for (uint32_t p = 0; ok && p < live; ++p) {
      for (uint32_t c = 0; c + 1 < m; ++c) {
        int dims[TO_MAX_DIMS];
        nth_permutation(ndims, beam[(size_t)p * C + c], dims);
        od[c] = encode_order(ndims, dims);
      }
      for (uint32_t j = 0; ok && j < F; ++j) {
        int dims[TO_MAX_DIMS];
        nth_permutation(ndims, j, dims);
        od[m - 1] = encode_order(ndims, dims);
        double T;
        ok = to_simulate(ndims, npus, bw, fixed_delay, ctype, 1u, &size_m, NULL, m,
                         intra_policy, od, &T, NULL, NULL, NULL);
        cand[nc].t = T;
        cand[nc].parent = p;
        cand[nc].digit = j;
        cand[nc].rank = numrank[p];
        ++nc;
      }
    }
    if (!ok) break;
    /* the `width` best, by selection: candidate x is taken at position
     * (number of candidates before it) if that is below width */
    uint32_t kept = nc < width ? nc : width;
    for (uint32_t x = 0; x < nc; ++x) {
      uint32_t before = 0;
      for (uint32_t y = 0; y < nc; ++y) before += (uint32_t)candidate_before(&cand[y], &cand[x]);
      if (before >= kept) continue;
      uint8_t *row = next + (size_t)before * C;
      memcpy(row, beam + (size_t)cand[x].parent * C, C);
      row[m - 1] = (uint8_t)cand[x].digit;
      beam_t[before] = cand[x].t;
      /* its number among the kept ones: newest digit first, then the parent's */
      newrank[before] = cand[x].digit * TO_MAX_BEAM + cand[x].rank;
    }
    for (uint32_t r = 0; r < kept; ++r) {
      uint32_t smaller = 0;
      for (uint32_t q = 0; q < kept; ++q) smaller += (uint32_t)(newrank[q] < newrank[r]);
      numrank[r] = smaller;
    }
    uint8_t *sw = beam; beam = next; next = sw;
    live = kept;
  }
  if (ok) {
    for (uint32_t c = 0; c < C; ++c) {
      int dims[TO_MAX_DIMS];
      nth_permutation(ndims, beam[c], dims);
      best_orders[c] = encode_order(ndims, dims);
    }
    *best_t = beam_t[0];
    /* the greedy scheduler's plan, if it is strictly better */
    double ld[TO_MAX_DIMS] = {0, 0, 0, 0}, Tg;
    ok = to_plan(ndims, npus, bw, fixed_delay, ctype, size_bytes, C, inter_policy,
                 threshold_mode, threshold, od, ld, NULL) &&
         to_simulate(ndims, npus, bw, fixed_delay, ctype, 1u, &size_bytes, NULL, C,
                     intra_policy, od, &Tg, NULL, NULL, NULL);
    if (ok && Tg < *best_t) {
      *best_t = Tg;
      memcpy(best_orders, od, C);
    }
  }
  free(beam); free(next); free(od); free(cand);
  return ok;
}

/* best_t [n], best_orders [n][max_chunks] (0xFF padded / on failure) */
void to_beam_search_batch(uint64_t n, uint64_t begin, uint64_t end,
                          uint32_t max_chunks, int threshold_mode,
                          const uint8_t *ndims, const uint32_t *npus,
                          const double *bw, const double *size_bytes,
                          const uint32_t *chunks, const uint8_t *inter_policy,
                          const uint8_t *intra_policy, const double *threshold,
                          const double *fixed_delay, const uint8_t *collective_type,
                          uint32_t width, double *best_t, uint8_t *best_orders)
{
  for (uint64_t i = begin; i < end; ++i) {
    uint32_t p[TO_MAX_DIMS];
    double b[TO_MAX_DIMS], fx[TO_MAX_DIMS];
    gather_network(n, i, npus, bw, p, b);
    const double *fixed = gather_fixed(n, i, fixed_delay, fx);
    uint8_t *row = best_orders + (size_t)i * max_chunks;
    memset(row, 0xFF, max_chunks);
    uint32_t C = chunks[i];
    double T = NAN;
    int ok = (C >= 1u && C <= max_chunks);
    if (ok)
      ok = to_beam_search((int)ndims[i], p, b, fixed,
                          collective_type ? (int)collective_type[i] : TO_ALL_REDUCE,
                          size_bytes[i], C, (int)inter_policy[i], (int)intra_policy[i],
                          threshold_mode, threshold[i], width, &T, row);
    if (!ok) { T = NAN; memset(row, 0xFF, max_chunks); }
    best_t[i] = T;
  }
}

/* ------------------------------------------------------------------------ */
/* Bandwidth provisioning of a dimension pair (Sec. 6.3, with the balance
 * condition of Sec. 3.3): for K < L the baseline schedule keeps both
 * dimensions equally busy when BW(dimK) = P_K * P_{K+1} * .. * P_{L-1} * BW(dimL).
 *   0  just enough      BW(dimK) == that product
 *   1  over-provisioned BW(dimK) <  it (dimL has bandwidth the baseline wastes)
 *   2  under-provisioned BW(dimK) > it
 * The product is accumulated left to right in double precision. */
/* ------------------------------------------------------------------------ */
int to_provision_class(int K, int L, const uint32_t *npus, const double *bw)
{
  double shrink = 1.0;
  for (int j = K; j < L; ++j) shrink = shrink * (double)npus[j];
  double balanced = shrink * bw[L];
  if (bw[K] < balanced) return 1;
  if (bw[K] > balanced) return 2;
  return 0;
}

/* classes [6][n], pairs in the order (1,2) (1,3) (1,4) (2,3) (2,4) (3,4) of
 * the paper's 1-based dimension names; 0xFF for pairs outside the network or
 * an invalid network. */
void to_classify_batch(uint64_t n, uint64_t begin, uint64_t end,
                       const uint8_t *ndims, const uint32_t *npus,
                       const double *bw, uint8_t *classes)
{
  for (uint64_t i = begin; i < end; ++i) {
    uint32_t P[TO_MAX_DIMS];
    double B[TO_MAX_DIMS];
    gather_network(n, i, npus, bw, P, B);
    int D = (int)ndims[i];
    int ok = to_network_valid(D, P, B);
    int pair = 0;
    for (int K = 0; K < TO_MAX_DIMS; ++K)
      for (int L = K + 1; L < TO_MAX_DIMS; ++L, ++pair)
        classes[(size_t)pair * n + i] =
            (ok && L < D) ? (uint8_t)to_provision_class(K, L, P, B) : 0xFF;
  }
}

/* ------------------------------------------------------------------------ */
/* Best threshold of a sweep (Sec. 5.3 fixes one Threshold for all
 * experiments; a parameter study asks which one is best per scenario) and the
 * speed-up over the baseline schedule (Sec. 6.1).
 * t_done [n][n_thr][n_pol]; per scenario i and scheduler column p:
 *   best_t   = the smallest t_done[i][a][p] over a that is not NaN (NaN if
 *              there is none), best_thr = the lowest a that reaches it
 *              (0xFFFFFFFF if there is none),
 *   speedup  = t_done[i][0][baseline_col] / best_t   (baseline_col >= 0).  */
/* ------------------------------------------------------------------------ */
void to_sweep_best(uint64_t n, uint32_t n_thr, uint32_t n_pol,
                   const double *t_done, int baseline_col, double *best_t,
                   uint32_t *best_thr, double *speedup)
{
  for (uint64_t i = 0; i < n; ++i) {
    for (uint32_t p = 0; p < n_pol; ++p) {
      double best = NAN;
      uint32_t at = 0xFFFFFFFFu;
      for (uint32_t a = 0; a < n_thr; ++a) {
        double t = t_done[((size_t)i * n_thr + a) * n_pol + p];
        if (isnan(t)) continue;
        if (at == 0xFFFFFFFFu || t < best) { best = t; at = a; }
      }
      best_t[(size_t)i * n_pol + p] = best;
      if (best_thr) best_thr[(size_t)i * n_pol + p] = at;
      if (speedup && baseline_col >= 0)
        speedup[(size_t)i * n_pol + p] =
            t_done[(size_t)i * n_thr * n_pol + (uint32_t)baseline_col] / best;
    }
  }
}
