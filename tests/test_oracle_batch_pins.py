"""Pins of the oracle's batch drivers (sweep, trace mode of plan / simulate,
trace totals of the metrics) against values worked out by hand, closed forms,
Alg. 1 replayed with exact rationals and the independent schedule checker.

The drivers add only indexing to the single-scenario functions pinned in
test_oracle_pins.py -- which policy a sweep column gets, which threshold a
scenario gets, where a collective's row of order codes lies, which collectives
count towards a total -- so every case here is chosen so that a wrong index,
stride or column moves a value that is known independently of the oracle.
"""
import itertools
import math
from fractions import Fraction

import numpy as np
import pytest

from paper_2110_04478_amd import workloads as W
from schedule_checker import order_dims, rebuild_and_check

MB = 1e6
U = 2.0 ** -20   # time unit of the dyadic hand cases, seconds


def code_of(dims):
    return sum(k << (2 * j) for j, k in enumerate(dims))


# The 2x2 network of the hand case: P = (2, 2), BW = (2^30, 2^33) B/s, three
# chunks of 2^22 bytes.  Per-byte latencies (Sec. 4.5) are 2^-31 and 2^-34 s, so
# in units of 2^-20 s a stage on dim1 takes 2048 with a whole chunk resident
# and 1024 with half of it, on dim2 256 and 128.
#
# Baseline (every chunk dim1 first): dim1 serves 3 x (2048 + 2048) back to back
# -> T = 12288.
# Alg. 1: chunk 0 sees (0, 0) -> dim1 first, tracker (4096, 256); chunk 1 ->
# dim2 first, (6144, 768); chunk 2 -> dim2 first, (8192, 1280).
# Themis + FIFO: dim1 runs c0 RS [0, 2048], then by arrival c1 RS [2048, 3072]
# (arrived 256), c2 RS [3072, 4096] (512), c0 AG [4096, 6144] (2304), c1 AG
# [6144, 7168] (3072), c2 AG [7168, 8192] (4096); c2's All-Gather on dim2
# follows, 256 -> T = 8448.
# Themis + SCF: at 3072 dim1 holds c2 RS (half a chunk), c0 AG (half) and c1 AG
# (a quarter): the quarter goes first [3072, 4096], then c2 RS [4096, 5120]
# (half, earlier arrival than c0), c2 AG [5120, 6144] (quarter), c0 AG
# [6144, 8192]; every dim2 stage is over by then -> T = 8192.
HAND = dict(P=[2, 2], bw=[2.0 ** 30, 2.0 ** 33], S=3 * 2.0 ** 22, C=3,
            t_baseline=12288 * U, t_fifo=8448 * U, t_scf=8192 * U)


def hand_batch(n=1, **kw):
    return W.make_batch([2] * n, [HAND["P"]] * n, [HAND["bw"]] * n, HAND["S"], HAND["C"],
                        1, 0, 0.0, **kw)


# ---------------------------------------------------------------- sweep columns
def test_sweep_columns_hand_values(oracle):
    """Each scheduler bit of the policy mask must get its own column, in
    ascending bit order: baseline + FIFO, Alg. 1 + FIFO, Alg. 1 + SCF
    (Table 3 of the paper).  The three differ on the hand case above."""
    b = hand_batch()
    want = {1: HAND["t_baseline"], 2: HAND["t_fifo"], 4: HAND["t_scf"]}
    for mask in range(1, 8):
        t = oracle.sweep(b, [0.0], mask)
        cols = [want[bit] for bit in (1, 2, 4) if mask & bit]
        assert t.shape == (1, 1, len(cols))
        assert t[0, 0].tolist() == cols


def test_sweep_columns_follow_their_policy(oracle):
    """Every column of a sweep re-derived without the oracle's event loop: the
    plan by Alg. 1, then the time the independent checker rebuilds from the
    per-dimension orders under the policy that column must have (Sec. 4.3).  A
    column evaluated under the other policy, or with the other scheduler, gives
    another time on these networks."""
    rng = np.random.default_rng(31)
    nets = []
    while len(nets) < 6:
        D = int(rng.integers(2, 4))
        P = [int(2 ** rng.integers(1, 4)) for _ in range(D)]
        bw = [float(2.0 ** rng.integers(28, 34)) for _ in range(D)]
        C = int(rng.integers(3, 7))
        nets.append((D, P, bw, C, float(C * 2 ** 22)))
    distinct = 0
    for D, P, bw, C, S in nets:
        b = W.make_batch([D], [P], [bw], S, C, 1, 0, 0.0)
        t = oracle.sweep(b, [0.0], 7)[0, 0]
        exact = []
        for inter, intra in ((0, 0), (1, 0), (1, 1)):
            od = oracle.plan(P, bw, S, C, inter)[0]
            qo = oracle.simulate(P, bw, [S], C, intra, od)["queue_order"]
            T, _ = rebuild_and_check(P, bw, [S], C, intra, od, qo)
            exact.append(T)
        assert [Fraction(v) for v in t] == exact
        distinct += len(set(exact)) == 3
    assert distinct >= 2        # the cases do tell the three columns apart


def test_sweep_known_times_in_every_column(oracle):
    """Cases whose time does not depend on the scheduler: a 1-D ring
    (2(P-1)/P * S/B, Sec. 2.1 / 4.5), the 2-D scenario of the first benchmark
    configuration (713.03168 us by hand: t0 + 8 t1 + t0) and the paper's 4x4
    worked example, where the baseline takes 8 units (Sec. 3.3)."""
    thr = np.array([0.0, 1 / 16, 1.0])
    b = W.make_batch([1], [[8]], [[100e9]], 2.0 ** 30, 64, 1, 0, 0.0, W.THR_REL)
    t = oracle.sweep(b, thr, 7)
    assert t.shape == (1, 3, 3)
    assert t == pytest.approx(2.0 * 7 / 8 * 2.0 ** 30 / 100e9, rel=1e-13)
    t = oracle.sweep(W.config1(), thr, 7)
    assert t == pytest.approx(713.03168e-6, rel=1e-9)
    B0 = 100e9
    unit = 64 * MB * 0.75 / B0
    b = W.make_batch([2], [[4, 4]], [[B0, B0 / 2]], 256 * MB, 4, 1, 0, 0.0, W.THR_REL)
    t = oracle.sweep(b, thr, 1)
    assert (t / unit == 8.0).all()


def test_sweep_threshold_layout(oracle):
    """Per-scenario thresholds are laid out [n_thr][n]; shared ones [n_thr].
    Alg. 1's threshold test (line 19) decides between the baseline order
    (threshold +inf: 12288 units on the hand case with FIFO) and the sorted
    order (threshold 0: 8448), so each entry of the result shows which
    threshold the scenario was given."""
    n, n_thr = 3, 2
    b = hand_batch(n)
    inf = math.inf
    thr = np.array([[0.0, inf, inf],
                    [inf, 0.0, 0.0]])            # [n_thr][n], not symmetric
    assert thr.reshape(-1).tolist() != thr.T.reshape(-1).tolist()
    t = oracle.sweep(b, thr, W.SWEEP_THEMIS_FIFO, thr_per_scenario=True)
    want = np.where(np.isinf(thr.T), HAND["t_baseline"], HAND["t_fifo"])   # [n][n_thr]
    assert t[:, :, 0].tolist() == want.tolist()
    # shared thresholds: the same column for every scenario
    t = oracle.sweep(b, np.array([inf, 0.0, inf]), W.SWEEP_THEMIS_FIFO | W.SWEEP_THEMIS_SCF)
    assert t[:, :, 0].tolist() == [[HAND["t_baseline"], HAND["t_fifo"], HAND["t_baseline"]]] * n
    assert t[:, 1, 1].tolist() == [HAND["t_scf"]] * n
    # the baseline order under SCF, by hand: dim1 prefers the half-size
    # All-Gathers of c0 and c1 to c2's whole-chunk Reduce-Scatter, which so ends
    # at 10240; c2 then needs dim2 twice (256) before its last stage on dim1:
    # 10496 + 2048
    assert t[:, 0, 1].tolist() == [12544 * U] * n


def test_sweep_reads_each_scenario_s_own_fields(oracle):
    """Scenario i of a sweep takes column i of every [4][n] field: three
    different 1-D rings in one batch, each against its closed form."""
    P, B, S, C = [4, 8, 3], [25e9, 100e9, 77e9], [1e8, 2.0 ** 30, 123456789.0], [1, 64, 5]
    b = W.make_batch([1, 1, 1], [[p] for p in P], [[x] for x in B], S, C, 1, 0, 0.0,
                     max_chunks=64)
    t = oracle.sweep(b, [0.0, 0.5], 7)
    for i in range(3):
        assert t[i] == pytest.approx(2.0 * (P[i] - 1) / P[i] * S[i] / B[i], rel=1e-13)
    # a scenario with more chunks than the rows hold is invalid, the others are not
    b.chunks = b.chunks.copy()
    b.chunks[1] = 65
    t = oracle.sweep(b, [0.0], 7)
    assert np.isnan(t[1]).all() and np.isfinite(t[0]).all() and np.isfinite(t[2]).all()


# ---------------------------------------------------------------- trace mode
def _trace_batch(rng, n, max_coll, max_chunks, release):
    D = rng.integers(1, 4, n)
    P = [[int(2 ** rng.integers(1, 4)) for _ in range(D[i])] for i in range(n)]
    bw = [[float(2.0 ** rng.integers(28, 34)) for _ in range(D[i])] for i in range(n)]
    C = rng.integers(1, max_chunks, n)            # always below the row length
    Q = rng.integers(1, max_coll + 1, n)
    Q[0], Q[1] = max_coll, 1                       # both ends of the ragged range
    sizes = np.zeros((max_coll, n))
    rel = np.zeros((max_coll, n)) if release else None
    for i in range(n):
        for q in range(max_coll):
            # entries past n_coll[i] hold garbage the drivers must not read
            sizes[q, i] = float(C[i] * 2 ** int(rng.integers(18, 24))) if q < Q[i] else -1.0
            if release:
                rel[q, i] = float(rng.integers(0, 6)) * 2.0 ** -12 if q < Q[i] else math.nan
    b = W.make_batch(D, P, bw, 1.0, C, 1, rng.integers(0, 2, n), 1 / 16, W.THR_REL,
                     max_chunks=max_chunks, n_coll=Q, coll_size=sizes, release_time=rel)
    return b, D, P, bw, C, Q


def _replay_alg1(P, bw, S, C, f):
    """Alg. 1 with exact rationals (relative threshold f): orders and tracker."""
    D = len(P)
    coef = [Fraction(P[k] - 1, P[k]) / Fraction(bw[k]) for k in range(D)]
    load = [Fraction(0)] * D
    chunk = Fraction(S) / C
    orders = []
    for _ in range(C):
        lo = min(load)
        if max(load) - lo < f * chunk * coef[load.index(lo)]:
            want = list(range(D))
        else:
            want = sorted(range(D), key=lambda k: (load[k], k))
        orders.append(want)
        x = chunk
        for k in want:
            load[k] += 2 * x * coef[k]
            x /= P[k]
    return orders, load


@pytest.mark.parametrize("release", [False, True])
def test_trace_batch_drivers(oracle, release):
    """Traces through the batch drivers: ragged collective counts, rows longer
    than the chunk count, a different size per collective.  Orders
    [n][max_coll][max_chunks]: every collective planned on its own (the tracker
    starts afresh, Alg. 1 line 2) -- replayed with exact rationals; loads: the
    last collective's tracker.  Queue orders [n][4][2*slots] with chunk ids
    q*C + i: rebuilt and checked operation by operation by the independent
    checker (Sec. 4.3, 4.6.2), whose exact completion and busy times the
    batch's must equal."""
    rng = np.random.default_rng(4100 + release)
    n, max_coll, max_chunks = 10, 4, 7
    b, D, P, bw, C, Q = _trace_batch(rng, n, max_coll, max_chunks, release)
    orders, loads = oracle.plan_batch(b)
    assert orders.shape == (n, max_coll * max_chunks)
    rows = orders.reshape(n, max_coll, max_chunks)
    for i in range(n):
        for q in range(max_coll):
            if q >= Q[i]:
                assert (rows[i, q] == 0xFF).all()
                continue
            want, load = _replay_alg1(P[i], bw[i], b.coll_size[q, i], int(C[i]), Fraction(1, 16))
            assert [order_dims(int(c), int(D[i])) for c in rows[i, q, :C[i]]] == want
            assert (rows[i, q, C[i]:] == 0xFF).all()
            if q == Q[i] - 1:
                assert [Fraction(v) for v in loads[:D[i], i]] == load
                assert (loads[D[i]:, i] == 0.0).all()

    t, qo, busy = oracle.simulate_batch(b, orders)
    slots = max_coll * max_chunks
    assert qo.shape == (n, 4, 2 * slots)
    for i in range(n):
        G = int(Q[i] * C[i])
        compact = np.concatenate([rows[i, q, :C[i]] for q in range(Q[i])])
        lists = [qo[i, k, :2 * G].astype(np.int64) for k in range(D[i])]
        T, bz = rebuild_and_check(
            P[i], bw[i], [b.coll_size[q, i] for q in range(Q[i])], int(C[i]),
            int(b.intra_policy[i]), compact, lists,
            release=None if not release else [b.release_time[q, i] for q in range(Q[i])])
        assert Fraction(t[i]) == T
        assert [Fraction(v) for v in busy[:D[i], i]] == bz
        assert (qo[i, :D[i], 2 * G:] == 0xFFFF).all() and (qo[i, D[i]:] == 0xFFFF).all()


def test_trace_batch_one_dimensional_closed_form(oracle):
    """Collectives that share one dimension run back to back: the trace takes
    sum_q 2(P-1)/P * S_q / B (Sec. 2.1, 4.5), whatever their sizes, chunk
    counts and queue policy; the Ideal of Table 3 and the average bandwidth
    utilisation (Sec. 3) follow from the same total."""
    n, max_coll = 4, 5
    P, B = [8, 3, 2, 16], [100e9, 77e9, 400e9, 50e9]
    Q = [5, 3, 1, 4]
    rng = np.random.default_rng(5)
    sizes = rng.uniform(1e6, 1e9, (max_coll, n))
    b = W.make_batch([1] * n, [[p] for p in P], [[x] for x in B], 1.0, [3, 7, 64, 1], 1,
                     [0, 1, 1, 0], 0.0, max_chunks=64, n_coll=Q, coll_size=sizes)
    orders, _ = oracle.plan_batch(b)
    t, qo, busy = oracle.simulate_batch(b, orders)
    util, ideal = oracle.metrics_batch(b, t, busy)
    for i in range(n):
        total = sum(sizes[q, i] for q in range(Q[i]))
        exact = 2.0 * (P[i] - 1) / P[i] * total / B[i]
        assert t[i] == pytest.approx(exact, rel=1e-12)
        assert busy[0, i] == pytest.approx(exact, rel=1e-12)
        assert ideal[i] == pytest.approx(total / B[i], rel=1e-14)
        assert util[i] == pytest.approx(1.0, rel=1e-12)
        G = Q[i] * int(b.chunks[i])
        assert sorted(qo[i, 0, :2 * G].tolist()) == list(range(2 * G))


def test_trace_metrics_hand_value(oracle):
    """Ideal = all the bytes of the trace over the total bandwidth (Table 3),
    by hand: collectives of 1, 2 and 3 GB on (100 + 50) GB/s take 6/150 s, the
    first two alone 3/150 s; utilisation (Sec. 3) with both dimensions busy
    half of T is one half."""
    sizes = np.array([[1e9, 1e9], [2e9, 2e9], [3e9, 7e9]])       # [max_coll][n]
    b = W.make_batch([2, 2], [[4, 4]] * 2, [[100e9, 50e9]] * 2, 5e9, 4, 1, 0, 0.0,
                     n_coll=[3, 2], coll_size=sizes)
    t = np.array([0.08, 0.08])
    transfer = np.array([[0.04, 0.04], [0.04, 0.04], [0.0, 0.0], [0.0, 0.0]])
    util, ideal = oracle.metrics_batch(b, t, transfer)
    assert ideal.tolist() == [6e9 / 150e9, 3e9 / 150e9]
    assert util == pytest.approx(0.5, rel=1e-15)


# ---------------------------------------------------------------- optional per-scenario fields
@pytest.mark.parametrize("seed", range(4))
def test_batch_drivers_with_delays_and_collective_types(oracle, seed):
    """fixed_delay [4][n] and collective_type [n] through the batch drivers:
    every scenario's plan replayed by the single-collective planner's pinned
    rules (checked there with rationals) is not used here -- instead each
    scenario's queue orders go through the independent checker with that
    scenario's own delays and collective type, so a column or a row taken from
    a neighbour shows as a wrong time."""
    rng = np.random.default_rng(4300 + seed)
    n = 9
    D = rng.integers(1, 5, n)
    P = [[int(2 ** rng.integers(1, 4)) for _ in range(D[i])] for i in range(n)]
    bw = [[float(2.0 ** rng.integers(28, 34)) for _ in range(D[i])] for i in range(n)]
    C = rng.integers(1, 9, n)
    S = [float(C[i] * 2 ** int(rng.integers(18, 24))) for i in range(n)]
    fx = [[float(rng.integers(0, 9)) * 2.0 ** -14 for _ in range(D[i])] for i in range(n)]
    b = W.make_batch(D, P, bw, S, C, rng.integers(0, 2, n), rng.integers(0, 2, n), 0.0,
                     max_chunks=11, fixed_delay=fx)
    b.collective_type = rng.integers(0, 3, n).astype(np.uint8)
    orders, loads = oracle.plan_batch(b)
    t, qo, busy = oracle.simulate_batch(b, orders)
    for i in range(n):
        ct = int(b.collective_type[i])
        nops = (2 if ct == 0 else 1) * int(C[i])
        lists = [qo[i, k, :nops].astype(np.int64) for k in range(D[i])]
        T, bz = rebuild_and_check(P[i], bw[i], [S[i]], int(C[i]), int(b.intra_policy[i]),
                                  orders[i, :C[i]], lists, fixed_delay=fx[i], ctype=ct)
        assert Fraction(t[i]) == T
        assert [Fraction(v) for v in busy[:D[i], i]] == bz
        assert (qo[i, :, nops:] == 0xFFFF).all()
        # tracker: bytes moved (the checker's busy time less the delays) plus A_K
        stages = 2 if ct == 0 else 1
        for k in range(D[i]):
            moved = bz[k] - stages * int(C[i]) * Fraction(fx[i][k])
            assert Fraction(loads[k, i]) == moved + stages * Fraction(fx[i][k])
