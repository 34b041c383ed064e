/*
 * themis.h -- C ABI of the MI355X (gfx950) batched evaluator for the Themis
 * collective chunk scheduler (arXiv 2110.04478).
 *
 * The library evaluates, for very large batches of independent scenarios,
 *   (1) the bandwidth-aware greedy chunk scheduler (paper Alg. 1,
 *       Sec. 4.2) that gives every chunk of a hierarchical All-Reduce its own
 *       order of network dimensions, and
 *   (2) the deterministic per-dimension queue simulation (paper Sec. 4.3
 *       intra-dimension policy, Sec. 4.6.2 consistency simulation) that turns
 *       such a plan into per-dimension execution orders and a completion time.
 * Nothing is communicated between devices: the collective is modelled, as in
 * the paper's own evaluation.
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  - Every pointer inside themis_batch_t and every array argument is a DEVICE
 *    pointer (HBM of the current HIP device), caller-owned.  The library never
 *    allocates or frees memory.  Outputs are fully overwritten.
 *  - State the library keeps, and why concurrent calls (other threads, other
 *    streams) and replays of a captured HIP graph are safe with it:
 *      a process-wide host counter that gives every simulate / sweep call a
 *      number, and one 64-bit word per GPU that a kernel raises (atomic
 *      maximum) to its call's number when it leaves an evaluation to the
 *      call's follow-up kernels.  A follow-up kernel skips its scan for such
 *      evaluations only while the word is below its own call's number; a
 *      larger number left by another call, or by the original run of a
 *      replayed graph, only costs that scan, and a smaller one can never hide
 *      a mark of this call.  Results never depend on either.
 *      themis_simulate_batch_noalloc additionally uses a scratch array that
 *      the library holds on every GPU (see there).
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls only enqueue kernels on that stream and return; they do not
 *    synchronise.
 *  - Arrays are structure-of-arrays: a per-dimension field is laid out
 *    [THEMIS_MAX_DIMS][n] (dimension-major), so a wavefront reads 64
 *    consecutive scenarios' values in one coalesced access.
 *  - Return value: THEMIS_OK (0) or a negative themis_status_t.  Argument
 *    errors that the host can see (NULL pointers, n == 0 is allowed and is a
 *    no-op, max_chunks out of range, ...) are reported without launching
 *    anything.  Errors inside one scenario (ndims outside 1..4, P < 2, a
 *    bandwidth / size / threshold that is not positive and finite, chunks
 *    outside 1..max_chunks) do not fail the batch: that scenario's times are
 *    written as NaN and its order codes / queue entries as all-ones bytes.
 *  - All times are seconds in IEEE binary64, sizes are bytes, bandwidths
 *    bytes/second (uni-directional, per NPU, per dimension).  Arithmetic is
 *    unfused (no FMA contraction) and in the operation order documented at
 *    each entry point, so results are reproducible bit for bit.
 *
 * Model (paper Sec. 2.1, 2.3, 4.5; A_K = 0, bandwidth term only)
 * -------------------------------------------------------------
 *   chunk      = size_bytes / chunks
 *   coef[k]    = ((P_k - 1) / P_k) / bw_k          seconds per resident byte
 *   A Reduce-Scatter stage on dimension k entered with x resident bytes costs
 *   x * coef[k] and leaves x / P_k.  The All-Gather stage of the same chunk on
 *   the same dimension moves the same bytes and costs the same time, and
 *   multiplies the resident size by P_k.  A chunk runs D Reduce-Scatter stages
 *   in its own dimension order, then D All-Gather stages in the reverse order.
 */
#ifndef THEMIS_H
#define THEMIS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define THEMIS_MAX_DIMS 4
/* Largest ChunksPerCollective accepted (the paper sweeps 4..512, Sec. 6.1). */
#define THEMIS_MAX_CHUNKS 512

typedef enum themis_status {
  THEMIS_OK = 0,
  THEMIS_ERR_INVALID_ARGUMENT = -1, /* NULL pointer, bad size or enum      */
  THEMIS_ERR_UNSUPPORTED = -2,      /* a valid request this build lacks    */
  THEMIS_ERR_DEVICE = -3,           /* a HIP call failed (launch, device)  */
  THEMIS_ERR_WORKSPACE = -4         /* workspace missing, small, misaligned */
} themis_status_t;

/* Inter-dimension scheduler of a scenario (paper Table 3). */
enum { THEMIS_INTER_BASELINE = 0, THEMIS_INTER_THEMIS = 1 };
/* Intra-dimension queue policy (paper Sec. 4.3): first-in-first-out, or
 * Smallest-Chunk-First on the resident size before the stage. */
enum { THEMIS_INTRA_FIFO = 0, THEMIS_INTRA_SCF = 1 };
/* Meaning of threshold[] in line 19 of Alg. 1:
 *   ABS: seconds.
 *   REL: fraction f; Threshold = f * (time of a Reduce-Scatter of one whole
 *        chunk on the currently least-loaded dimension).  The paper's default
 *        (Sec. 5.3) is f = 1/16. */
enum { THEMIS_THR_ABS = 0, THEMIS_THR_REL = 1 };

/* CollectiveType of Alg. 1. */
enum { THEMIS_COLL_ALL_REDUCE = 0, THEMIS_COLL_REDUCE_SCATTER = 1, THEMIS_COLL_ALL_GATHER = 2 };

/* Bits of themis_sweep's policy_mask, evaluated in ascending bit order. */
enum {
  THEMIS_SWEEP_BASELINE = 1u,    /* baseline order + FIFO   */
  THEMIS_SWEEP_THEMIS_FIFO = 2u, /* Alg. 1 + FIFO           */
  THEMIS_SWEEP_THEMIS_SCF = 4u   /* Alg. 1 + SCF            */
};

/*
 * One batch of n independent scenarios (inputs of Alg. 1 plus the network:
 * P_1 x ... x P_D with one bandwidth per dimension, Sec. 2.3).
 * All pointers are device pointers; the struct itself lives on the host.
 */
typedef struct themis_batch {
  uint64_t n;              /* number of scenarios                              */
  uint32_t max_chunks;     /* row stride of `orders`; 1..THEMIS_MAX_CHUNKS;
                              every chunks[i] must be <= max_chunks           */
  uint32_t threshold_mode; /* THEMIS_THR_ABS or THEMIS_THR_REL (whole batch)   */
  const uint8_t *ndims;    /* [n]    D, 1..THEMIS_MAX_DIMS                     */
  const uint32_t *npus;    /* [4][n] P_k >= 2; rows k >= D are ignored         */
  const double *bw;        /* [4][n] bytes/s, > 0 and finite                   */
  const double *size_bytes;/* [n]    CollectiveSize S, > 0 and finite          */
  const uint32_t *chunks;  /* [n]    ChunksPerCollective C                     */
  const uint8_t *inter_policy; /* [n] THEMIS_INTER_*                           */
  const uint8_t *intra_policy; /* [n] THEMIS_INTRA_* (used by simulate only)   */
  const double *threshold; /* [n]    >= 0 (may be +inf in ABS mode)            */
  /* Optional trace extension (several collectives sharing the per-dimension
   * queues; NULL / 0 = one collective of size_bytes released at t = 0).
   * When n_coll is non-NULL, scenario i issues n_coll[i] collectives; number q
   * has coll_size[q*n + i] bytes, is planned on its own (the load tracker is
   * reset per collective, Alg. 1 line 2) and releases all its chunks at
   * release_time[q*n + i] seconds (NULL = all zero). */
  uint32_t max_coll;          /* leading extent of coll_size / release_time    */
  const uint32_t *n_coll;     /* [n]            1..max_coll                    */
  const double *coll_size;    /* [max_coll][n]                                 */
  const double *release_time; /* [max_coll][n]  >= 0, or NULL                  */
  /* Optional fixed delay A_K (Sec. 4.5: number of steps of the dimension's
   * basic algorithm x step latency), in seconds per Reduce-Scatter or
   * All-Gather stage on dimension k; NULL = 0.  The load tracker of Alg. 1
   * then starts at fixed_delay[k] + fixed_delay[k] (one All-Reduce = one
   * stage of each kind per dimension), and every stage on k takes
   * fixed_delay[k] + bytes * per-byte latency in the simulation. */
  const double *fixed_delay;  /* [4][n] >= 0 and finite, or NULL               */
  /* Optional CollectiveType of Alg. 1 per scenario; NULL = All-Reduce.
   * A stand-alone Reduce-Scatter runs only the D Reduce-Scatter stages
   * (tracker += t, started at fixed_delay[k]); a stand-alone All-Gather of
   * size_bytes per NPU runs D stages, each of which multiplies the resident
   * size by P_k and takes (size * P_k) * coef[k]; its order is the reverse of
   * the ascending sort (descending loads, ties to the higher dimension, so
   * equal loads give dimD..dim1, its baseline order), its relative Threshold
   * is threshold * ((chunk * P_kmin) * coef[kmin]), and its queue entries
   * carry phase 1.  Each dimension then executes `chunks` operations, not
   * 2 * chunks.  themis_sweep evaluates All-Reduce only. */
  const uint8_t *collective_type; /* [n] THEMIS_COLL_*, or NULL               */
} themis_batch_t;

/* Library version as major*10000 + minor*100 + patch. */
int themis_version(void);

/* Static English description of a status code (never NULL). */
const char *themis_status_string(int status);

/*
 * Order code of one chunk: byte o0 | o1<<2 | o2<<4 | o3<<6, the 0-based
 * dimensions in the order its Reduce-Scatter stages visit them (fields at
 * positions >= D are zero).  The All-Gather order is the reverse (Alg. 1
 * line 8).  0xFF marks an invalid scenario or an unused chunk slot.
 *
 * Queue-order entry: (chunk_id << 1) | phase, phase 0 = Reduce-Scatter,
 * 1 = All-Gather, listed per dimension in the order the dimension executed
 * them (Sec. 4.6.2).  chunk_id is q*chunks + i in trace mode.  The entry is
 * one byte when slots <= 127 and two bytes (little endian uint16) otherwise,
 * where slots = max_chunks * max(1, max_coll); themis_queue_entry_bytes()
 * returns that width.  Unused entries are all-ones.
 */
int themis_queue_entry_bytes(uint32_t max_chunks, uint32_t max_coll);

/*
 * Bytes of scratch that themis_simulate_batch / themis_sweep may need:
 *   - single collectives with power-of-two NPU counts and sizes whose
 *     halvings stay in the normal binary64 range run entirely in registers
 *     and LDS and need no workspace;
 *   - single collectives with NPU counts that are not powers of two run in
 *     LDS as well, on per-order tables, at every chunk count, and need no
 *     workspace either;
 *   - what no LDS path takes (e.g. stage times too short to move the clock,
 *     times that leave the binary64 range on the way) goes to a slower generic
 *     path, whose per-chunk state sits in LDS up to 64 chunks and in the
 *     workspace beyond;
 *   - traces (n_coll != NULL) keep their per-scenario queues in the workspace
 *     (up to 256 collectives on the fast path, whatever the NPU counts; with
 *     NPU counts that are not powers of two under Smallest-Chunk-First up to
 *     4096 / (D! * 2) collectives -- 341 on three dimensions, 85 on four --,
 *     D! for a stand-alone Reduce-Scatter or All-Gather; beyond that the
 *     generic path, same results, far slower).
 * For themis_sweep pass n * n_thr * n_pol as n and max_coll = 0.
 * Passing a smaller or NULL workspace is allowed: every scenario that would
 * have needed it then comes back as NaN / all-ones, like an invalid one (the
 * call cannot report this through its return value, because it does not wait
 * for the device).  The workspace must be 16-byte aligned, must stay untouched
 * until the stream has drained, and two calls in flight at once need a
 * workspace each.
 */
size_t themis_workspace_bytes(uint64_t n, uint32_t max_chunks, uint32_t max_coll);

/*
 * themis_plan_batch -- Alg. 1 (Schedule_Collective + Scheduler.Schedule) for
 * every scenario.
 *
 * Per scenario, with load[k] = 0 (A_K = 0, Sec. 4.5) and for chunk i = 0..C-1:
 *   kmin = lowest index of the smallest load; lo = load[kmin]; hi = max load
 *   Threshold = threshold (ABS) or threshold * (chunk * coef[kmin]) (REL)
 *   order = 0,1,..,D-1 if inter_policy is BASELINE or (hi - lo) < Threshold,
 *           else the dimensions sorted by load ascending, ties keeping the
 *           lower index first (so equal loads give the baseline order)
 *   x = chunk; for j = 0..D-1, k = order[j]:
 *       t = x * coef[k]; load[k] = load[k] + (t + t); x = x / P_k
 * (the tracker accumulates the Reduce-Scatter and the All-Gather time of the
 * chunk on every dimension: the total communication time of the caption of
 * the paper's scheduling figure).
 *
 *   orders : [n][max_chunks] uint8 order codes (slots >= chunks[i] = 0xFF).
 *            In trace mode: [n][max_coll][max_chunks].
 *   loads  : [4][n] final tracker contents in seconds (rows >= D are 0), or
 *            NULL.  In trace mode: the loads of the last collective.
 */
int themis_plan_batch(const themis_batch_t *batch, uint8_t *orders,
                      double *loads, void *stream);

/*
 * themis_simulate_batch -- deterministic execution of a plan (Sec. 4.3, 4.6.2).
 *
 * Every dimension is one non-preemptive, work-conserving server.  All chunks
 * of a collective wait at the dimension of their first stage from the
 * collective's release time.  Whenever a dimension is idle and chunks wait for
 * it, it starts the one with the smallest key
 *   FIFO: (arrival time at this dimension, chunk_id)
 *   SCF : (resident size before the stage, arrival time, chunk_id)
 * for the stage's time (see Model above); all completions that fall on the
 * same instant are delivered before any dimension picks its next chunk.
 *
 *   orders      : [n][max_chunks] (trace: [n][max_coll][max_chunks]) order
 *                 codes, e.g. themis_plan_batch's output; any permutation
 *                 code is accepted, a malformed one invalidates the scenario.
 *   t_done      : [n] completion time of the last stage.
 *   queue_order : NULL, or [n][4][2*slots] entries (see above).  The array
 *                 also serves as staging while the call runs (rows are put in
 *                 place at the end), so it holds the result only once the
 *                 call's work on the stream is complete, like every output,
 *                 and it must not overlap any other argument.
 *   busy        : NULL, or [4][n] seconds each dimension spent serving.
 *   workspace, workspace_bytes : see themis_workspace_bytes().
 * A scenario whose stage times or clock overflow binary64 (bandwidths or
 * sizes hundreds of orders of magnitude apart) comes back like an invalid one.
 */
int themis_simulate_batch(const themis_batch_t *batch, const uint8_t *orders,
                          double *t_done, void *queue_order, double *busy,
                          void *workspace, size_t workspace_bytes,
                          void *stream);

/*
 * themis_simulate_batch_noalloc -- themis_simulate_batch for callers that
 * cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results and kernels; the scratch that themis_simulate_batch takes
 * from the caller's workspace sits in a device array of
 * THEMIS_STATIC_SCRATCH_BYTES that the library itself holds on every GPU it is
 * loaded on, for the life of the process.  The call allocates and frees
 * nothing.
 *   - A batch that would need more (themis_workspace_bytes(n, max_chunks,
 *     max_coll) for traces, and for single collectives of more than 64 chunk
 *     slots; nothing otherwise) is refused with THEMIS_ERR_WORKSPACE before
 *     anything is launched.
 *   - All calls on one GPU share that GPU's array: two such calls must not be
 *     in flight at once on one GPU (different streams or threads), or they race.
 *     Contents left by an earlier call are never read.
 *   - The first call on a device asks the runtime for the array's address
 *     (no stream work); make one call per device before capturing a graph.
 */
#define THEMIS_STATIC_SCRATCH_BYTES (32u << 20)
int themis_simulate_batch_noalloc(const themis_batch_t *batch, const uint8_t *orders,
                                  double *t_done, void *queue_order, double *busy,
                                  void *stream);

/*
 * themis_sweep -- fused plan + simulate for every scenario x threshold x
 * scheduler of policy_mask (the parameter studies of Sec. 6.1), keeping only
 * completion times.  inter_policy / intra_policy / threshold of the batch are
 * ignored.
 *
 *   thr        : n_thr thresholds (meaning per batch->threshold_mode); shared
 *                by all scenarios ([n_thr], thr_per_scenario = 0) or one set
 *                per scenario ([n_thr][n], thr_per_scenario != 0).
 *   t_done     : [n][n_thr][n_pol], n_pol = popcount(policy_mask), schedulers
 *                in ascending bit order.  THEMIS_SWEEP_BASELINE ignores the
 *                threshold: it is simulated once per scenario and its value
 *                repeats along n_thr (NaN under a threshold that is itself
 *                not valid, as in the other columns).
 */
int themis_sweep(const themis_batch_t *batch, int n_thr, const double *thr,
                 int thr_per_scenario, unsigned policy_mask, double *t_done,
                 void *workspace, size_t workspace_bytes, void *stream);

/*
 * themis_set_sweep_mapping -- how themis_sweep's LDS kernel spreads the
 * evaluations over the lanes of a wavefront.  The simulation of Sec. 4.6.2 /
 * Sec. 4.3 is the same either way and so are the results; the mappings differ
 * in speed only.
 *   THEMIS_MAPPING_AUTO : the faster one for the batch's chunk capacity (the
 *                         library's choice, the default)
 *   THEMIS_MAPPING_LANE : one lane per evaluation
 *   THEMIS_MAPPING_QUAD : four lanes per evaluation, one per dimension
 * Process-wide, takes effect with the next call of themis_sweep; meant for
 * measurements and tests.  Returns THEMIS_ERR_INVALID_ARGUMENT for any other
 * value.
 */
#define THEMIS_MAPPING_AUTO 0
#define THEMIS_MAPPING_LANE 1
#define THEMIS_MAPPING_QUAD 2
int themis_set_sweep_mapping(int mapping);

/*
 * themis_sweep_best -- what a parameter study reports per scenario and
 * scheduler: the threshold that gives the smallest completion time (Sec. 5.3
 * fixes one Threshold for all experiments; this finds the best one per
 * scenario) and the speed-up over the baseline schedule (Sec. 6.1).
 *
 *   t_done       : [n][n_thr][n_pol] device doubles as written by themis_sweep.
 *   baseline_col : column p of the baseline scheduler (0 when policy_mask
 *                  contained THEMIS_SWEEP_BASELINE), or -1 for no speed-up.
 *   best_t       : [n][n_pol] min over a of t_done[i][a][p]; NaN entries are
 *                  skipped, NaN if all n_thr entries are.
 *   best_thr     : [n][n_pol] lowest a that reaches it, 0xFFFFFFFF if none.
 *                  May be NULL.
 *   speedup      : [n][n_pol] t_done[i][0][baseline_col] / best_t[i][p] (the
 *                  baseline ignores the threshold, so a = 0 stands for all).
 *                  May be NULL; not written when baseline_col < 0.
 */
int themis_sweep_best(uint64_t n, int n_thr, int n_pol, const double *t_done,
                      int baseline_col, double *best_t, uint32_t *best_thr,
                      double *speedup, void *stream);

/*
 * themis_metrics_batch -- the derived quantities of the paper's evaluation.
 *
 *   utilization[i] = sum_k transfer[k][i] * bw[k][i] / (t_done[i] * sum_k bw[k][i])
 *       the average bandwidth utilisation of Sec. 3: each dimension's
 *       utilisation (bytes it moved / (T * its bandwidth)) weighted by its
 *       bandwidth.  transfer is the time each dimension spent moving bytes:
 *       themis_plan_batch's loads or themis_simulate_batch's busy (minus the
 *       fixed delays, if any were given).
 *   ideal[i]       = total collective bytes / sum_k bw[k][i]   (Table 3 "Ideal")
 * Sums run over k = 0..D-1 in ascending order.  Either output may be NULL.
 * Invalid scenarios (ndims outside 1..4) give NaN.
 */
int themis_metrics_batch(const themis_batch_t *batch, const double *t_done,
                         const double *transfer, double *utilization,
                         double *ideal, void *stream);

/*
 * themis_search_batch -- exhaustive search over per-chunk dimension orders
 * for tiny chunk counts (Sec. 4.1, observation 2: a collective of C chunks has
 * (D!)^C schedules once an All-Reduce's All-Gather order is tied to the
 * reverse of its Reduce-Scatter order), to measure how far the greedy
 * scheduler is from the best schedule.
 *
 * Assignment number a (0 <= a < (D!)^C) gives chunk c the permutation of
 * (0, 1, .., D-1) with lexicographic index (a / (D!)^c) mod D!.  Every
 * assignment is simulated with the scenario's intra_policy (and fixed_delay /
 * collective_type, if given); inter_policy and threshold are ignored.
 *
 *   max_assignments : upper bound on (D!)^C over the batch; a scenario with
 *                     more schedules than this comes back as NaN / all-ones.
 *   best_t      : [n] smallest completion time.
 *   best_orders : [n][max_chunks] order codes of the first assignment (lowest
 *                 a) that reaches it; slots >= chunks[i] are 0xFF.  May be NULL.
 *   workspace   : themis_search_workspace_bytes(n, max_assignments) bytes
 *                 (one time per scenario and assignment), required.
 * Covers single collectives (n_coll == NULL) of at most 64 chunks, any NPU
 * counts (power-of-two counts on the fast path, others on per-order tables);
 * other scenarios come back as NaN / all-ones.
 */
size_t themis_search_workspace_bytes(uint64_t n, uint64_t max_assignments);
int themis_search_batch(const themis_batch_t *batch, uint64_t max_assignments,
                        double *best_t, uint8_t *best_orders, void *workspace,
                        size_t workspace_bytes, void *stream);

/*
 * themis_beam_search_batch -- beam search over per-chunk dimension orders for
 * up to 64 chunks (Sec. 4.1, observation 2 names the space of per-chunk
 * schedules; Alg. 1 walks it greedily, keeping one schedule; Sec. 4.2's note
 * leaves better searches open).  The chunks are given their orders one after
 * the other, chunk 0 first.  A partial schedule of m chunks is scored by the
 * completion time of a collective of just those m chunks -- of size_bytes if
 * m == chunks, else of (size_bytes / chunks) * m bytes -- under the scenario's
 * intra_policy (and fixed_delay / collective_type, if given).  Every kept
 * partial schedule is extended by each of the D! orders for the next chunk and
 * the `width` best extensions are kept: smaller time first, equal times in
 * ascending assignment number (numbering of themis_search_batch: the newest
 * chunk's digit is the most significant).  With width >= (D!)^chunks nothing
 * is dropped and the result is that of themis_search_batch.  The answer is the
 * better of the beam's best full schedule and the plan of themis_plan_batch
 * under the scenario's inter_policy / threshold (the beam's on equal times), so
 * it is never worse than the greedy scheduler.
 *
 *   width       : 1..64 schedules kept per step.
 *   best_t      : [n] completion time of the schedule found.
 *   best_orders : [n][max_chunks] its order codes; slots >= chunks[i] are
 *                 0xFF.  May be NULL.
 *   workspace   : themis_beam_workspace_bytes(n, max_chunks, width) bytes,
 *                 64-byte aligned, required (the kept schedules, one time per
 *                 scenario and candidate, the greedy plan).
 * Covers single collectives (n_coll == NULL) with max_chunks <= 64, any NPU
 * counts (power-of-two counts on the fast path, others on per-order tables).
 * Invalid scenarios, and scenarios one of whose partial schedules neither
 * path can simulate, come back as NaN / all-ones.  Launches 3 kernels per
 * chunk slot; the work is n * width * D! simulations per step.
 */
size_t themis_beam_workspace_bytes(uint64_t n, uint32_t max_chunks, uint32_t width);
int themis_beam_search_batch(const themis_batch_t *batch, uint32_t width, double *best_t,
                             uint8_t *best_orders, void *workspace, size_t workspace_bytes,
                             void *stream);

/*
 * themis_classify_batch -- bandwidth provisioning class of every dimension
 * pair of each scenario's network (Sec. 6.3, balance condition of Sec. 3.3).
 * For K < L the baseline keeps dimK and dimL equally busy when
 * BW(dimK) = P_K * P_{K+1} * .. * P_{L-1} * BW(dimL) (product accumulated left
 * to right in double precision); dimL is over-provisioned when BW(dimK) is
 * below that (the case Themis recovers) and under-provisioned when above (the
 * design points the paper advises against).
 *
 *   classes : [6][n] device bytes, THEMIS_BW_* per pair, pairs in the order
 *             (1,2) (1,3) (1,4) (2,3) (2,4) (3,4) of the paper's 1-based
 *             dimension names; 0xFF for pairs outside the network and for
 *             scenarios whose ndims / npus / bw are invalid.
 * Only ndims, npus and bw of the batch are read.
 */
enum {
  THEMIS_BW_JUST_ENOUGH = 0,
  THEMIS_BW_OVER_PROVISIONED = 1,
  THEMIS_BW_UNDER_PROVISIONED = 2
};
int themis_classify_batch(const themis_batch_t *batch, uint8_t *classes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* THEMIS_H */
