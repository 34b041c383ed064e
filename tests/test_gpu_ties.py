"""GPU parity on networks where many stages end at the very same binary64
instant (the method's determinism edge case: Sec. 4.6.2 asks every NPU to
derive the same per-dimension orders, so simultaneous completions must be
delivered in one fixed order -- all of an instant before any dispatch, in
chunk-id order).

workloads.dyadic_ties() draws power-of-two NPU counts, per-byte latencies that
are powers of two along the just-enough bandwidth ladder of Sec. 3.3 / 6.3 and
chunks of 2^m bytes: every stage time is a power of two and every clock value
an exact sum, so completions on different dimensions coincide again and again.
Each test says which branch of the kernels it is there for; all compare order
codes, queue orders, completion and busy times element by element with the
oracle, through the C ABI.
"""
import itertools

import numpy as np
import pytest

from test_gpu_parity import (assert_close, check_batch, gpu, w, widen_queue,  # noqa: F401
                             _with_collective_types)

pytestmark = pytest.mark.gpu


def simultaneous_completions(b, i, orders, queue_order):
    """How many instants of scenario i (an All-Reduce without delays) see two or
    more dimensions complete a stage, counted by replaying the reported
    per-dimension orders in floating point."""
    D, C = int(b.ndims[i]), int(b.chunks[i])
    P = [int(b.npus[k, i]) for k in range(D)]
    coef = [((P[k] - 1) / P[k]) / b.bw[k, i] for k in range(D)]
    chunk = b.size_bytes[i] / C
    t = {}
    for c in range(C):
        dims = [(int(orders[i, c]) >> (2 * j)) & 3 for j in range(D)]
        x = chunk
        for k in dims:
            t[(c, k)] = x * coef[k]
            x = x / P[k]
    stage_dims = {c: None for c in range(C)}
    for c in range(C):
        dims = [(int(orders[i, c]) >> (2 * j)) & 3 for j in range(D)]
        stage_dims[c] = dims + dims[::-1]
    done_stage = [0] * C
    ready = [0.0] * C
    free_at = [0.0] * D
    ptr = [0] * D
    ends = []
    progressed = True
    while progressed:
        progressed = False
        for k in range(D):
            while ptr[k] < 2 * C:
                c = int(queue_order[i, k, ptr[k]]) >> 1
                if stage_dims[c][done_stage[c]] != k:
                    break
                end = max(free_at[k], ready[c]) + t[(c, k)]
                free_at[k] = ready[c] = end
                done_stage[c] += 1
                ptr[k] += 1
                ends.append((end, k))
                progressed = True
    assert len(ends) == 2 * D * C
    per_instant = {}
    for end, k in ends:
        per_instant.setdefault(end, set()).add(k)
    return sum(1 for dims in per_instant.values() if len(dims) > 1)


def _dyadic_delays(b, seed):
    """Fixed delays per stage that are multiples of 2^-14 s: sums stay exact."""
    rng = np.random.default_rng(seed)
    b.fixed_delay = np.ascontiguousarray(rng.integers(0, 9, (4, b.n)) * 2.0 ** -14)
    return b


def _arbitrary_orders(b, seed):
    rng = np.random.default_rng(seed)
    orders = np.full((b.n, b.slots), 0xFF, np.uint8)
    for i in range(b.n):
        D = int(b.ndims[i])
        perms = np.argsort(rng.random((int(b.chunks[i]), D)), axis=1)
        orders[i, :perms.shape[0]] = (perms << (2 * np.arange(D))).sum(axis=1)
    return orders


def _check_given_orders(gpu, oracle, b, orders):
    import torch
    o_t, o_qo, o_busy = oracle.simulate_batch(b, orders, threads=8)
    d = gpu.to_device(b)
    t, qo, busy = gpu.themis_simulate_batch(d, torch.from_numpy(orders).cuda())
    torch.cuda.synchronize()
    assert np.isfinite(o_t).all()
    assert_close("t_done", t.cpu().numpy(), o_t)
    assert np.array_equal(widen_queue(qo), o_qo)
    assert_close("busy", busy.cpu().numpy(), o_busy)


SIZES = {16: 500, 64: 500, 128: 300, 256: 130, 512: 100}


@pytest.mark.parametrize("max_chunks", [16, 64, 128, 256, 512])
def test_simultaneous_completions_on_every_lds_layout(gpu, oracle, max_chunks):
    """All-Reduce plans of Alg. 1 on the tie-rich networks, one chunk capacity
    per LDS layout: up to 128 chunks the event loop of simulate_fast, beyond it
    simulate_packed.  Reaches the branch at the end of their delivery loops
    that takes the next completion of the same instant (the smallest
    chunk << 2 | dimension among the stages left in `done`), and the appends
    that keep every list in (arrival, chunk id) order when several chunks
    arrive at one instant.  The count below shows the inputs do that."""
    n = SIZES[max_chunks]
    b = w().dyadic_ties(n, seed=7000 + max_chunks, max_chunks=max_chunks)
    check_batch(gpu, oracle, b, workspace=False)
    # evidence that the instants with several completions are there
    o_orders, _ = oracle.plan_batch(b, threads=8)
    _, o_qo, _ = oracle.simulate_batch(b, o_orders, threads=8)
    sample = [i for i in range(n) if b.ndims[i] >= 2][:12]
    ties = [simultaneous_completions(b, i, o_orders, o_qo) for i in sample]
    assert sum(x > 0 for x in ties) >= 8 and sum(ties) >= 50, ties
    # the untilted ladder: every load ties after every chunk (baseline orders throughout)
    b2 = w().dyadic_ties(n // 2, seed=7100 + max_chunks, max_chunks=max_chunks, tilt=False)
    check_batch(gpu, oracle, b2, workspace=False)
    # the fused sweep runs the same loops without outputs (three schedulers, two thresholds)
    import torch
    keep = b.take(slice(0, n // 2))
    thr = np.array([0.0, 1 / 16])
    got = gpu.themis_sweep(gpu.to_device(keep), torch.from_numpy(thr).cuda(), 7)
    torch.cuda.synchronize()
    assert_close("sweep", got.cpu().numpy(), oracle.sweep(keep, thr, 7, threads=8))


@pytest.mark.parametrize("max_chunks", [16, 64, 128, 256, 512])
def test_simultaneous_completions_all_collective_types_and_delays(gpu, oracle, max_chunks):
    """The same branches with stand-alone Reduce-Scatter and All-Gather
    collectives mixed in, with and without fixed per-stage delays that are
    multiples of 2^-14 s (the kFix variants of the stage-start blocks), and with
    arbitrary orders instead of planned ones (all D! permutations inside one
    scenario, so chunks meet on every dimension in both phases)."""
    n = SIZES[max_chunks] // 2
    b = _with_collective_types(w().dyadic_ties(n, seed=7200 + max_chunks, max_chunks=max_chunks), 3)
    check_batch(gpu, oracle, b, workspace=False)
    _check_given_orders(gpu, oracle, b, _arbitrary_orders(b, 11))
    b = _dyadic_delays(b, 5)
    check_batch(gpu, oracle, b, workspace=False)
    _check_given_orders(gpu, oracle, b, _arbitrary_orders(b, 12))


def test_simultaneous_completions_in_traces(gpu, oracle):
    """Traces on the tie-rich networks (ranked-list path, simulate_trace_fast):
    collective sizes a power of two apart share resident sizes across
    collectives, several collectives are released at one instant, and release
    instants are multiples of the stage times, so releases coincide with each
    other and with completions (the latter hands the scenario to the generic
    path, which merges both kinds of arrivals by chunk id).  Reaches the
    same-instant branch of the trace loop's delivery and the release loop that
    lets every collective due at an instant join before any dispatch."""
    W = w()
    rng = np.random.default_rng(21)
    for max_chunks, max_coll, n in ((8, 6, 300), (16, 12, 120), (64, 4, 70)):
        b = W.dyadic_ties(n, seed=7300 + max_chunks, max_chunks=max_chunks)
        b.max_coll = max_coll
        b.n_coll = rng.integers(1, max_coll + 1, n).astype(np.uint32)
        chunk = b.size_bytes / b.chunks
        b.coll_size = np.ascontiguousarray(
            (chunk * b.chunks)[None, :] * 2.0 ** rng.integers(-2, 3, (max_coll, n)))
        b.release_time = None
        check_batch(gpu, oracle, b)                       # all released at t = 0
        # release instants on a grid of 2^-12 s (stage times are 2^-9 .. 2^-22 s)
        b.release_time = np.ascontiguousarray(rng.integers(0, 4, (max_coll, n)) * 2.0 ** -12)
        t = check_batch(gpu, oracle, b)
        assert np.isfinite(t).all()
        check_batch(gpu, oracle, _dyadic_delays(_with_collective_types(b, 9), 10))


def test_tie_rich_networks_with_other_npu_counts(gpu, oracle):
    """The table-driven loops (NPU counts that are not powers of two run the same
    event loop on per-order tables): NPU counts 3, 6 and 12 with bandwidths
    2^a * (P-1)/P keep the per-byte latencies powers of two, and sizes that are
    multiples of 3^4 * 2^m divide evenly, so equal times and sizes abound."""
    W = w()
    rng = np.random.default_rng(33)
    for max_chunks, n in ((64, 400), (128, 200), (256, 60)):
        b = W.dyadic_ties(n, seed=7400 + max_chunks, max_chunks=max_chunks)
        scale = (b.npus - 1.0) / b.npus
        a = b.bw / scale
        b.npus = np.ascontiguousarray(rng.choice([3, 6, 12, 4], (4, n)).astype(np.uint32))
        b.bw = np.ascontiguousarray(a * ((b.npus - 1.0) / b.npus))
        b.size_bytes = b.size_bytes * 81.0
        check_batch(gpu, oracle, _with_collective_types(b, 2), workspace=False)


def test_tie_rich_traces_with_other_npu_counts(gpu, oracle):
    """Traces on networks with NPU counts 3, 6 and 12 under both queue policies
    (division mode of the ranked-list path: one size rank per (dimension, phase,
    order) and collective, equal sizes sharing a rank): bandwidths 2^a * (P-1)/P
    keep the per-byte latencies powers of two and sizes that are multiples of
    3^4 * 2^m divide evenly, so equal resident sizes across orders, phases and
    collectives abound, as do equal times; with collectives released at one
    instant and at coinciding instants."""
    W = w()
    rng = np.random.default_rng(34)
    for max_chunks, max_coll, n in ((8, 6, 300), (16, 10, 120), (64, 3, 70)):
        b = W.dyadic_ties(n, seed=7900 + max_chunks, max_chunks=max_chunks)
        scale = (b.npus - 1.0) / b.npus
        a = b.bw / scale
        b.npus = np.ascontiguousarray(rng.choice([3, 6, 12, 4], (4, n)).astype(np.uint32))
        b.bw = np.ascontiguousarray(a * ((b.npus - 1.0) / b.npus))
        b.max_coll = max_coll
        b.n_coll = rng.integers(1, max_coll + 1, n).astype(np.uint32)
        b.coll_size = np.ascontiguousarray(
            (b.size_bytes * 81.0)[None, :] * 2.0 ** rng.integers(-2, 3, (max_coll, n)))
        b.release_time = None
        check_batch(gpu, oracle, _with_collective_types(b, 3))
        b.release_time = np.ascontiguousarray(rng.integers(0, 4, (max_coll, n)) * 2.0 ** -12)
        t = check_batch(gpu, oracle, b)
        assert np.isfinite(t).all()


@pytest.mark.parametrize("mapping", ["lane", "quad"])
def test_sweep_mappings_agree_with_the_oracle(gpu, oracle, mapping):
    """themis_sweep under each of its two lane mappings (one lane per evaluation;
    four lanes per evaluation, lane j owning dimension j), forced for every
    chunk capacity: the tie-rich networks reach the quad mapping's loop that
    appends the chunks of several stages ending at one instant one at a time,
    lowest chunk id first; the ragged batches (D 1..4, any C, scenarios without
    a fast path, a last wavefront with empty quads) its hand-over to the
    follow-up passes."""
    import torch
    W = w()
    thr = torch.tensor([0.0, 1.0 / 16.0, 0.5], dtype=torch.float64, device="cuda")
    gpu.themis_set_sweep_mapping({"lane": gpu.MAPPING_LANE, "quad": gpu.MAPPING_QUAD}[mapping])
    try:
        for mc, n in ((16, 150), (64, 150), (200, 90), (512, 70)):
            for b in (W.dyadic_ties(n, seed=7600 + mc, max_chunks=mc),
                      W.mixed(n + 3, seed=7700 + mc, max_chunks=mc, pow2=(mc != 200))):
                d = gpu.to_device(b)
                sw = gpu.themis_sweep(d, thr, 7)
                torch.cuda.synchronize()
                assert_close("sweep (%s, %d chunks)" % (mapping, mc), sw.cpu().numpy(),
                             oracle.sweep(b, thr.cpu().numpy(), 7, threads=8))
    finally:
        gpu.themis_set_sweep_mapping(gpu.MAPPING_AUTO)
