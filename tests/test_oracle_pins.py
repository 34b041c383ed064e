"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these compare the oracle with itself: closed forms, the values the
paper prints for its worked example, exact rational arithmetic, an independent
schedule checker and brute-force enumeration.
"""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from schedule_checker import order_dims, rebuild_and_check

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
MB = 1e6


def read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            out.setdefault(key, []).append(vals)
    return out


def code_of(dims):
    return sum(k << (2 * j) for j, k in enumerate(dims))


# ---------------------------------------------------------------- latency model
@pytest.mark.parametrize("P,B,S,C", [
    (8, 100e9, 2.0 ** 30, 64), (4, 25e9, 100 * MB, 1), (2, 400e9, 3e8, 7),
    (16, 50e9, 2.0 ** 20, 512), (3, 77e9, 123456789.0, 5), (64, 12.5e9, 1e9, 64)])
def test_one_dimensional_ring_closed_form(oracle, P, B, S, C):
    """A 1-D All-Reduce moves 2(P-1)/P*S bytes per NPU (Sec. 2.1, 4.5): with
    one dimension nothing can overlap, so T = 2(P-1)/P * S/B whatever C is."""
    for inter, intra in itertools.product((0, 1), (0, 1)):
        orders, loads, _ = oracle.plan([P], [B], S, C, inter)
        assert (orders == 0).all()
        r = oracle.simulate([P], [B], [S], C, intra, orders)
        exact = 2.0 * (P - 1) / P * S / B
        assert r["t_done"] == pytest.approx(exact, rel=1e-13)
        assert loads[0] == pytest.approx(exact, rel=1e-13)
        assert r["busy"][0] == pytest.approx(exact, rel=1e-13)
        # the single queue is FIFO over ids whatever the policy says... for
        # FIFO every RS precedes nothing in particular, so only check counts
        assert sorted(r["queue_order"][0].tolist()) == list(range(2 * C))


def test_footnote_bytes_per_npu(oracle):
    """Sec. 4.5 footnote: a 4 MB chunk on a ring dimension sends (P-1)/P*4MB."""
    for P in (2, 4, 5, 8, 64):
        bw = 1e9
        coef = oracle.latency_coef([P], [bw])[0]
        assert coef * 4 * MB * bw == pytest.approx((P - 1) / P * 4 * MB, rel=1e-15)


def test_worked_example_stage_ratios(oracle):
    g = read_golden("worked_example_4x4.txt")
    ratios = [float(v) for v in g["stage_ratio"][0]]
    B0 = 100e9
    orders, loads, st = oracle.plan([4, 4], [B0, B0 / 2], 256 * MB, 4, inter_policy=0)
    unit = st[0][0]                       # 64 MB Reduce-Scatter on dim1
    stages = [st[0][0], st[0][1], st[0][1], st[0][0]]  # RS d1, RS d2, AG d2, AG d1
    assert [s / unit for s in stages] == ratios
    # Sec. 3.3 sets the unit of time as a Reduce-Scatter of 64 MB on dim1 and
    # gives the All-Gather that starts from 16 MB the same unit: the AG that
    # ends with 64 MB resident costs what the 64 MB RS does -- checked through
    # the simulator, whose dim1 must be busy exactly 8 units for 4 chunks
    r = oracle.simulate([4, 4], [B0, B0 / 2], [256 * MB], 4, 0, orders)
    assert r["busy"][0] / unit == 8.0 and r["busy"][1] / unit == 4.0
    # baseline: dim1 is the bottleneck and never idles
    assert r["t_done"] / unit == 8.0


def test_worked_example_themis_orders(oracle):
    g = read_golden("worked_example_4x4.txt")
    first = [int(v) - 1 for v in g["first_dim"][0]]
    B0 = 100e9
    orders, loads, st = oracle.plan([4, 4], [B0, B0 / 2], 256 * MB, 4, inter_policy=1)
    assert [order_dims(int(c), 2)[0] for c in orders] == first
    # load trajectory in paper units, by hand from the latency model:
    # (2,1) -> (2.5,5) -> (4.5,6) -> (6.5,7)
    unit = 64 * MB * 0.75 / B0
    want = [(2, 1), (2.5, 5), (4.5, 6), (6.5, 7)]
    for i, w in enumerate(want, start=1):
        _, ld, _ = oracle.plan([4, 4], [B0, B0 / 2], 64 * MB * i, i, inter_policy=1)
        assert ld[0] / unit == pytest.approx(w[0], rel=1e-14)
        assert ld[1] / unit == pytest.approx(w[1], rel=1e-14)


def test_equal_bandwidth_does_not_reduce_to_baseline(oracle):
    """P=(4,4), equal B: by hand loads go (2,.5) -> (2.5,2.5) -> (4.5,3) ->
    (5,5) in units of a full-chunk RS on dim1, so orders alternate."""
    orders, loads, _ = oracle.plan([4, 4], [64e9, 64e9], 2.0 ** 28, 4, 1)
    assert [order_dims(int(c), 2)[0] for c in orders] == [0, 1, 0, 1]
    unit = 2.0 ** 26 * 0.75 / 64e9
    assert loads[0] / unit == pytest.approx(5.0, rel=1e-14)
    assert loads[1] / unit == pytest.approx(5.0, rel=1e-14)


@pytest.mark.parametrize("P,Bgbps", [
    ((4, 4), (400, 100)),            # Sec. 3.3: BW(dim1) = 4*BW(dim2) for 4x4
    ((16, 8, 8), (800, 50, 6.25)),   # Sec. 6.1: 800 = 16*50 = 128*6.25 Gb/s
    ((2, 8, 8, 64), (1024, 512, 64, 8))])
def test_just_enough_bandwidth_reduces_to_baseline(oracle, P, Bgbps):
    """Sec. 3.3 / 6.3 'just enough' condition BW(dim1) = P1*BW(dim2) = ...,
    with the (P-1)/P factor the text leaves out folded into the bandwidths:
    all baseline stage times are then equal, every load ties after every
    chunk, and Alg. 1 must keep the baseline order for all chunks."""
    bw = [b * 1e9 / 8 * (p - 1) / p for p, b in zip(P, Bgbps)]
    D = len(P)
    orders, loads, st = oracle.plan(P, bw, 2.0 ** 30, 64, 1)
    assert (orders == code_of(range(D))).all()
    assert len({st[0][k] for k in range(D)}) == 1
    # and the arithmetic of the condition itself
    prod = 1
    for k in range(D):
        assert Bgbps[0] == prod * Bgbps[k]
        prod *= P[k]


def test_threshold_rule(oracle):
    """Alg. 1 line 19 is a strict '<'.  Worked example after chunk 1: loads
    (2,1) units, the least-loaded dimension is dim2 where a whole-chunk RS
    takes 2 units; so relative thresholds 0.5 (Threshold = 1.0 = difference)
    must still sort, anything above must fall back to the baseline order."""
    B0 = 100e9
    args = ([4, 4], [B0, B0 / 2], 256 * MB, 4, 1)
    first = lambda o: [order_dims(int(c), 2)[0] for c in o]
    assert first(oracle.plan(*args, threshold_mode=1, threshold=0.5)[0])[1] == 1
    assert first(oracle.plan(*args, threshold_mode=1, threshold=0.5 + 1e-9)[0])[1] == 0
    # absolute mode: difference is exactly one unit of time
    unit = 64 * MB * 0.75 / B0
    assert first(oracle.plan(*args, threshold_mode=0, threshold=unit)[0])[1] == 1
    assert first(oracle.plan(*args, threshold_mode=0, threshold=unit * 1.001)[0])[1] == 0
    # a huge threshold disables Themis entirely; paper default f = 1/16 keeps it
    assert first(oracle.plan(*args, threshold_mode=0, threshold=math.inf)[0]) == [0] * 4
    assert first(oracle.plan(*args, threshold_mode=1, threshold=1 / 16)[0]) == [0, 1, 0, 0]


def test_schedule_space_count():
    """Sec. 4.2 footnote: D=3, C=8 gives (3!*3!)^8 = 2821109907456 schedules."""
    assert (math.factorial(3) * math.factorial(3)) ** 8 == 2821109907456


# ---------------------------------------------------------------- conservation
def _rand_net(rng, D, dyadic):
    if dyadic:
        P = [int(2 ** rng.integers(1, 4)) for _ in range(D)]
        bw = [float(2.0 ** rng.integers(28, 34)) for _ in range(D)]
    else:
        P = [int(2 ** rng.integers(1, 5)) for _ in range(D)]
        bw = [float(rng.uniform(25e9, 400e9)) for _ in range(D)]
    return P, bw


@pytest.mark.parametrize("seed", range(12))
def test_load_conservation_exact(oracle, seed):
    """Sec. 4.5: N_K = sum of bytes each NPU sends on dim K; the tracker must
    hold 2 * B_K * N_K (RS + AG) whatever the orders are -- recomputed here
    from the emitted orders with exact rationals."""
    rng = np.random.default_rng(seed)
    D = int(rng.integers(1, 5))
    P = [int(rng.integers(2, 20)) for _ in range(D)]
    bw = [float(rng.uniform(10e9, 900e9)) for _ in range(D)]
    S = float(rng.integers(2 ** 20, 2 ** 32))
    C = int(rng.integers(1, 70))
    thr = float(rng.choice([0.0, 1 / 16, 0.3]))
    orders, loads, st = oracle.plan(P, bw, S, C, 1, 1, thr)
    exact = [Fraction(0)] * D
    for i in range(C):
        x = Fraction(S) / C
        for k in order_dims(int(orders[i]), D):
            t = Fraction(P[k] - 1, P[k]) * x / Fraction(bw[k])
            assert st[i][k] == pytest.approx(float(t), rel=1e-14)
            exact[k] += 2 * t
            x /= P[k]
    for k in range(D):
        assert loads[k] == pytest.approx(float(exact[k]), rel=1e-12)
    # and the simulator's busy time is the same total, summed in another order
    for intra in (0, 1):
        r = oracle.simulate(P, bw, [S], C, intra, orders)
        for k in range(D):
            assert r["busy"][k] == pytest.approx(float(exact[k]), rel=1e-12)
        assert r["t_done"] >= max(loads[:D]) * (1 - 1e-12)
        assert r["t_done"] >= S / sum(bw) * (1 - 1e-12)   # 'Ideal' of Table 3


def test_greedy_choice_is_argsort_of_exact_loads(oracle):
    """Replay Alg. 1 with exact rationals on dyadic inputs (where binary64 is
    exact too) and compare every chunk's order, including ties."""
    rng = np.random.default_rng(7)
    for _ in range(40):
        D = int(rng.integers(2, 5))
        P, bw = _rand_net(rng, D, dyadic=True)
        C = int(rng.integers(1, 33))
        S = float(C * 2 ** int(rng.integers(20, 26)))
        f = Fraction(int(rng.integers(0, 5)), 16)
        orders, loads, _ = oracle.plan(P, bw, S, C, 1, 1, float(f))
        coef = [Fraction(P[k] - 1, P[k]) / Fraction(bw[k]) for k in range(D)]
        load = [Fraction(0)] * D
        chunk = Fraction(S) / C
        for i in range(C):
            lo = min(load)
            kmin = load.index(lo)
            if max(load) - lo < f * chunk * coef[kmin]:
                want = list(range(D))
            else:
                want = sorted(range(D), key=lambda k: (load[k], k))
            assert order_dims(int(orders[i]), D) == want
            x = chunk
            for k in want:
                load[k] += 2 * x * coef[k]
                x /= P[k]
        assert [Fraction(v) for v in loads[:D]] == load


# ---------------------------------------------------------------- simulation
@pytest.mark.parametrize("seed", range(30))
def test_simulation_obeys_queue_rules_dyadic(oracle, seed):
    """Dyadic inputs make every time exactly representable, so ties between
    simultaneous events are real and the independent checker (exact rationals)
    must agree on every tie-break."""
    rng = np.random.default_rng(100 + seed)
    D = int(rng.integers(1, 5))
    P, bw = _rand_net(rng, D, dyadic=True)
    C = int(rng.integers(1, 13))
    S = float(C * 2 ** int(rng.integers(20, 26)))
    inter = int(rng.integers(0, 2))
    orders, loads, _ = oracle.plan(P, bw, S, C, inter, 1, float(rng.choice([0, 1 / 16])))
    if seed % 3 == 0:  # arbitrary (non-greedy) orders too
        perms = list(itertools.permutations(range(D)))
        orders = np.array([code_of(perms[rng.integers(len(perms))]) for _ in range(C)],
                          dtype=np.uint8)
    for intra in (0, 1):
        r = oracle.simulate(P, bw, [S], C, intra, orders)
        T, busy = rebuild_and_check(P, bw, [S], C, intra, orders, r["queue_order"])
        assert Fraction(r["t_done"]) == T
        assert [Fraction(v) for v in r["busy"][:D]] == busy


@pytest.mark.parametrize("seed", range(20))
def test_simulation_obeys_queue_rules_random(oracle, seed):
    rng = np.random.default_rng(500 + seed)
    D = int(rng.integers(2, 5))
    P, bw = _rand_net(rng, D, dyadic=False)
    C = int(rng.integers(2, 17))
    S = float(rng.integers(2 ** 20, 2 ** 32))
    orders, loads, _ = oracle.plan(P, bw, S, C, 1, 1, 1 / 16)
    for intra in (0, 1):
        r = oracle.simulate(P, bw, [S], C, intra, orders)
        T, busy = rebuild_and_check(P, bw, [S], C, intra, orders, r["queue_order"])
        assert r["t_done"] == pytest.approx(float(T), rel=1e-12)


@pytest.mark.parametrize("seed", range(8))
def test_trace_simulation_obeys_queue_rules(oracle, seed):
    """Several collectives sharing the queues, with and without staggered
    release times."""
    rng = np.random.default_rng(900 + seed)
    D = int(rng.integers(2, 4))
    P, bw = _rand_net(rng, D, dyadic=True)
    C, Q = int(rng.integers(1, 5)), int(rng.integers(2, 5))
    sizes = [float(C * 2 ** int(rng.integers(20, 25))) for _ in range(Q)]
    release = None
    if seed % 2:
        release = [float(rng.integers(0, 8)) * 2.0 ** -12 for _ in range(Q)]
    orders = np.concatenate([oracle.plan(P, bw, s, C, 1)[0] for s in sizes])
    for intra in (0, 1):
        r = oracle.simulate(P, bw, sizes, C, intra, orders, release)
        T, _ = rebuild_and_check(P, bw, sizes, C, intra, orders,
                                 r["queue_order"], release)
        assert Fraction(r["t_done"]) == T
        assert max(r["coll_done"]) == r["t_done"]


@pytest.mark.parametrize("D,C", [(2, 4), (3, 3), (2, 5)])
def test_brute_force_over_all_orders(oracle, D, C):
    """Tiny C: enumerate every assignment of Reduce-Scatter orders to chunks
    ((D!)^C of them, Sec. 4.1 observation 2 with the AG order tied to the
    reverse), check each simulated schedule with the independent checker, and
    that greedy Themis is never better than the optimum it is bounded by."""
    rng = np.random.default_rng(D * 10 + C)
    P, bw = _rand_net(rng, D, dyadic=True)
    S = float(C * 2 ** 22)
    perms = [code_of(p) for p in itertools.permutations(range(D))]
    themis = oracle.plan(P, bw, S, C, 1)[0]
    count = 0
    for intra in (0, 1):
        t_themis = oracle.simulate(P, bw, [S], C, intra, themis)["t_done"]
        best = math.inf
        for assign in itertools.product(perms, repeat=C):
            od = np.array(assign, dtype=np.uint8)
            r = oracle.simulate(P, bw, [S], C, intra, od)
            T, busy = rebuild_and_check(P, bw, [S], C, intra, od, r["queue_order"])
            assert Fraction(r["t_done"]) == T
            assert T >= max(busy)
            best = min(best, r["t_done"])
            count += 1
        assert best <= t_themis
        # no schedule beats the per-chunk critical path or the bandwidth bound
        assert best >= S / sum(bw)
    assert count == 2 * math.factorial(D) ** C


def test_worked_example_derived_schedules(oracle):
    """Not printed in the paper (its timing figure is not available as text):
    derived by hand from the model for the 4x4 example.  Baseline: dim1 runs
    c1..c4 RS then c1..c4 AG back to back (8 units)."""
    B0 = 100e9
    unit = 64 * MB * 0.75 / B0
    base = oracle.plan([4, 4], [B0, B0 / 2], 256 * MB, 4, 0)[0]
    r = oracle.simulate([4, 4], [B0, B0 / 2], [256 * MB], 4, 0, base)
    assert r["queue_order"][0].tolist() == [0, 2, 4, 6, 1, 3, 5, 7]
    rebuild_and_check([4, 4], [B0, B0 / 2], [256 * MB], 4, 0, base, r["queue_order"])
    assert r["t_done"] / unit == 8.0


def test_config1_by_hand(oracle):
    """2-D P=(4,8), B=(200,50) GB/s, 64 MiB in 4 chunks: RS times are
    16 MiB*(3/4)/200e9 and 4 MiB*(7/8)/50e9; dim2 is the heavier dimension
    from the first chunk on, so the ascending sort keeps dim1 first always."""
    P, bw, S, C = [4, 8], [200e9, 50e9], 64 * 2.0 ** 20, 4
    t0 = Fraction(16 * 2 ** 20) * Fraction(3, 4) / Fraction(200 * 10 ** 9)
    t1 = Fraction(4 * 2 ** 20) * Fraction(7, 8) / Fraction(50 * 10 ** 9)
    assert t1 > t0
    orders, loads, st = oracle.plan(P, bw, S, C, 1)
    assert orders.tolist() == [code_of([0, 1])] * 4
    assert loads[0] == pytest.approx(float(8 * t0), rel=1e-14)
    assert loads[1] == pytest.approx(float(8 * t1), rel=1e-14)
    for intra in (0, 1):
        r = oracle.simulate(P, bw, [S], C, intra, orders)
        T, _ = rebuild_and_check(P, bw, [S], C, intra, orders, r["queue_order"])
        # dim2 starts after one dim1 stage, works 8 stages back to back, and
        # the last chunk's AG on dim1 follows: t0 + 8*t1 + t0
        assert T == 2 * t0 + 8 * t1
        assert r["t_done"] == pytest.approx(float(T), rel=1e-14)
        assert r["t_done"] == pytest.approx(713.03168e-6, rel=1e-9)


# ---------------------------------------------------------------- paper aggregates
def test_paper_aggregates_trend(oracle):
    """Soft pin: the bandwidth-only model on the Table 2 topologies should land
    near the paper's averages (its simulator adds link latency)."""
    g = read_golden("paper_aggregates.txt")
    val = lambda k: float(g[k][0][0])
    sp_f, sp_s, ut_b, ut_f, ut_s = [], [], [], [], []
    for row in g["topology"]:
        bar = row.index("|")
        P = [int(v) for v in row[1:bar]]
        bw = [float(v) * 1e9 / 8 for v in row[bar + 1:]]
        for S in (100 * MB, 250 * MB, 500 * MB, 1000 * MB):
            res = {}
            for name, inter, intra in (("b", 0, 0), ("f", 1, 0), ("s", 1, 1)):
                od, ld, _ = oracle.plan(P, bw, S, 64, inter, 1, 1 / 16)
                T = oracle.simulate(P, bw, [S], 64, intra, od)["t_done"]
                util = sum(l * b for l, b in zip(ld, bw)) / (T * sum(bw))
                res[name] = (T, util)
            sp_f.append(res["b"][0] / res["f"][0])
            sp_s.append(res["b"][0] / res["s"][0])
            ut_b.append(res["b"][1]); ut_f.append(res["f"][1]); ut_s.append(res["s"][1])
    assert np.mean(sp_f) == pytest.approx(val("speedup_themis_fifo"), rel=0.05)
    assert np.mean(sp_s) == pytest.approx(val("speedup_themis_scf"), rel=0.05)
    assert np.max(sp_s) == pytest.approx(val("speedup_themis_scf_max"), rel=0.05)
    assert 100 * np.mean(ut_b) == pytest.approx(val("util_baseline"), abs=3.0)
    assert 100 * np.mean(ut_f) == pytest.approx(val("util_themis_fifo"), abs=4.0)
    assert 100 * np.mean(ut_s) == pytest.approx(val("util_themis_scf"), abs=4.0)


# ---------------------------------------------------------------- the checker bites
def test_checker_rejects_planted_mistakes(oracle):
    """The independent checker must fail on a wrong execution order, on the
    wrong policy and on wrong stage times, or it would pin nothing."""
    B0 = 100e9
    P, bw, S, C = [4, 4], [B0, B0 / 2], 256 * MB, 4
    orders = oracle.plan(P, bw, S, C, 1)[0]
    fifo = oracle.simulate(P, bw, [S], C, 0, orders)["queue_order"]
    scf = oracle.simulate(P, bw, [S], C, 1, orders)["queue_order"]
    assert fifo.tolist() != scf.tolist()
    with pytest.raises(AssertionError):
        rebuild_and_check(P, bw, [S], C, 1, orders, fifo)
    with pytest.raises(AssertionError):
        rebuild_and_check(P, bw, [S], C, 0, orders, scf)
    swapped = fifo.copy()
    swapped[0, [1, 2]] = swapped[0, [2, 1]]
    with pytest.raises(AssertionError):
        rebuild_and_check(P, bw, [S], C, 0, orders, swapped)
    # a transposed bandwidth pair changes which chunk arrives first
    with pytest.raises(AssertionError):
        rebuild_and_check(P, bw[::-1], [S], C, 0, orders, fifo)


# ---------------------------------------------------------------- fixed delay A_K
@pytest.mark.parametrize("P,B,S,C,a", [
    (8, 100e9, 2.0 ** 30, 64, 5e-6), (4, 25e9, 100 * MB, 1, 1e-3), (3, 77e9, 123456789.0, 5, 2e-7)])
def test_one_dimensional_closed_form_with_fixed_delay(oracle, P, B, S, C, a):
    """Sec. 4.5: Latency(dim) = A + N*B + idle.  One dimension never idles and
    every one of the 2C stages pays the fixed delay a, so
    T = 2*C*a + 2(P-1)/P * S/B."""
    orders, loads, _ = oracle.plan([P], [B], S, C, 1, fixed_delay=[a])
    r = oracle.simulate([P], [B], [S], C, 1, orders, fixed_delay=[a])
    exact = 2 * C * a + 2.0 * (P - 1) / P * S / B
    assert r["t_done"] == pytest.approx(exact, rel=1e-13)
    assert r["busy"][0] == pytest.approx(exact, rel=1e-13)
    # the tracker starts at A_K (one RS + one AG delay) and then adds bytes only
    assert loads[0] == pytest.approx(2 * a + 2.0 * (P - 1) / P * S / B, rel=1e-13)


def test_ring_all_reduce_step_count():
    """Sec. 4.5: a ring-based All-Reduce takes 2P-2 steps = RS + AG stage."""
    from paper_2110_04478_amd import workloads as W
    for p in (2, 4, 8, 16, 64):
        assert 2 * W.stage_steps("R", p) == 2 * p - 2
        assert W.stage_steps("S", p) == math.log2(p)
        assert W.stage_steps("F", p) == 1


def test_tracker_starts_at_fixed_delay(oracle):
    """Worked example with a fixed delay of 0.75 unit per stage on dim2 only:
    the tracker starts at (0, 1.5) units, so by hand the loads go
    (2,2.5) -> (4,3.5) -> (4.5,7.5) -> (6.5,8.5) and the chunks start from
    dim1, dim1, dim2, dim1 (without the delay: dim1, dim2, dim1, dim1)."""
    B0 = 100e9
    unit = 64 * MB * 0.75 / B0
    fx = [0.0, 0.75 * unit]
    orders, loads, _ = oracle.plan([4, 4], [B0, B0 / 2], 256 * MB, 4, 1, fixed_delay=fx)
    assert [order_dims(int(c), 2)[0] for c in orders] == [0, 0, 1, 0]
    assert loads[0] / unit == pytest.approx(6.5, rel=1e-13)
    assert loads[1] / unit == pytest.approx(8.5, rel=1e-13)
    # the baseline scheduler ignores the tracker but its stages still pay the delay
    base = oracle.plan([4, 4], [B0, B0 / 2], 256 * MB, 4, 0, fixed_delay=fx)[0]
    r = oracle.simulate([4, 4], [B0, B0 / 2], [256 * MB], 4, 0, base, fixed_delay=fx)
    assert r["busy"][1] / unit == pytest.approx(8 * 0.5 + 8 * 0.75, rel=1e-13)
    assert r["busy"][0] / unit == pytest.approx(8.0, rel=1e-13)


@pytest.mark.parametrize("seed", range(16))
def test_simulation_with_fixed_delay_obeys_queue_rules(oracle, seed):
    rng = np.random.default_rng(1300 + seed)
    D = int(rng.integers(1, 5))
    P, bw = _rand_net(rng, D, dyadic=True)
    C = int(rng.integers(1, 11))
    S = float(C * 2 ** int(rng.integers(20, 26)))
    fx = [float(rng.integers(0, 9)) * 2.0 ** -14 for _ in range(D)]
    orders, loads, _ = oracle.plan(P, bw, S, C, 1, 1, 1 / 16, fixed_delay=fx)
    # Alg. 1 replayed with exact rationals, tracker starting at A_K
    coef = [Fraction(P[k] - 1, P[k]) / Fraction(bw[k]) for k in range(D)]
    load = [2 * Fraction(fx[k]) for k in range(D)]
    chunk = Fraction(S) / C
    for i in range(C):
        lo = min(load)
        if max(load) - lo < Fraction(1, 16) * chunk * coef[load.index(lo)]:
            want = list(range(D))
        else:
            want = sorted(range(D), key=lambda k: (load[k], k))
        assert order_dims(int(orders[i]), D) == want
        x = chunk
        for k in want:
            load[k] += 2 * x * coef[k]
            x /= P[k]
    assert [Fraction(v) for v in loads[:D]] == load
    for intra in (0, 1):
        r = oracle.simulate(P, bw, [S], C, intra, orders, fixed_delay=fx)
        T, busy = rebuild_and_check(P, bw, [S], C, intra, orders, r["queue_order"],
                                    fixed_delay=fx)
        assert Fraction(r["t_done"]) == T
        assert [Fraction(v) for v in r["busy"][:D]] == busy


# ---------------------------------------------------------------- derived metrics
def test_utilization_and_ideal(oracle):
    """Sec. 3 definition of the average bandwidth utilisation and Table 3's
    Ideal, on cases with known answers: a 1-D All-Reduce uses its only
    dimension all the time; the baseline on the worked example keeps dim1
    (weight 2) busy 8 of 8 units and dim2 (weight 1) 4 of 8: (2*8 + 4)/(3*8)."""
    from paper_2110_04478_amd import workloads as W
    b = W.make_batch([1], [[8]], [[100e9]], 2.0 ** 30, 64, 1, 0, 0.0)
    od, ld = oracle.plan_batch(b)
    t, _, bz = oracle.simulate_batch(b, od)
    util, ideal = oracle.metrics_batch(b, t, bz)
    assert util[0] == pytest.approx(1.0, rel=1e-13)
    assert ideal[0] == pytest.approx(2.0 ** 30 / 100e9, rel=1e-15)
    B0 = 100e9
    b = W.make_batch([2], [[4, 4]], [[B0, B0 / 2]], 256 * MB, 4, 0, 0, 0.0)
    od, ld = oracle.plan_batch(b)
    t, _, bz = oracle.simulate_batch(b, od)
    util, ideal = oracle.metrics_batch(b, t, ld)
    assert util[0] == pytest.approx(20.0 / 24.0, rel=1e-13)
    assert ideal[0] == pytest.approx(256 * MB / (1.5 * B0), rel=1e-15)
    assert t[0] >= ideal[0]


# ---------------------------------------------------------------- stand-alone RS / AG
RS, AG = 1, 2


@pytest.mark.parametrize("P,B,S,C", [(8, 100e9, 2.0 ** 30, 64), (3, 77e9, 123456789.0, 5),
                                     (2, 400e9, 3e8, 7)])
def test_one_dimensional_reduce_scatter_and_all_gather(oracle, P, B, S, C):
    """Sec. 2.1: on P NPUs a Reduce-Scatter sends (P-1)/P of the resident data
    and leaves 1/P of it; an All-Gather that starts from S bytes per NPU ends
    with P*S and sends (P-1)*S.  An All-Reduce of S is the one followed by the
    other on S/P."""
    od, ld, _ = oracle.plan([P], [B], S, C, 1, ctype=RS)
    rs = oracle.simulate([P], [B], [S], C, 0, od, ctype=RS)
    assert rs["t_done"] == pytest.approx((P - 1) / P * S / B, rel=1e-13)
    assert ld[0] == pytest.approx((P - 1) / P * S / B, rel=1e-13)
    assert sorted(rs["queue_order"][0][:C].tolist()) == [2 * g for g in range(C)]
    od, ld, _ = oracle.plan([P], [B], S / P, C, 1, ctype=AG)
    ag = oracle.simulate([P], [B], [S / P], C, 0, od, ctype=AG)
    assert ag["t_done"] == pytest.approx((P - 1) * (S / P) / B, rel=1e-13)
    assert sorted(ag["queue_order"][0][:C].tolist()) == [2 * g + 1 for g in range(C)]
    od, _, _ = oracle.plan([P], [B], S, C, 1)
    ar = oracle.simulate([P], [B], [S], C, 0, od)
    assert ar["t_done"] == pytest.approx(rs["t_done"] + ag["t_done"], rel=1e-13)


@pytest.mark.parametrize("seed", range(10))
def test_single_chunk_all_reduce_is_rs_then_ag(oracle, seed):
    """With one chunk nothing overlaps: the baseline All-Reduce (RS dim1..dimD,
    AG dimD..dim1, Sec. 2.3) takes the Reduce-Scatter of S plus the All-Gather
    of what is left, S / (P_1*...*P_D), each with its own baseline order."""
    rng = np.random.default_rng(2000 + seed)
    D = int(rng.integers(1, 5))
    P, bw = _rand_net(rng, D, dyadic=True)
    S = float(2 ** int(rng.integers(24, 30)))
    prod = int(np.prod(P))
    od_ar = oracle.plan(P, bw, S, 1, 0)[0]
    od_rs = oracle.plan(P, bw, S, 1, 0, ctype=RS)[0]
    od_ag = oracle.plan(P, bw, S / prod, 1, 0, ctype=AG)[0]
    assert order_dims(int(od_rs[0]), D) == list(range(D))
    assert order_dims(int(od_ag[0]), D) == list(range(D))[::-1]
    t_ar = oracle.simulate(P, bw, [S], 1, 0, od_ar)["t_done"]
    t_rs = oracle.simulate(P, bw, [S], 1, 0, od_rs, ctype=RS)["t_done"]
    t_ag = oracle.simulate(P, bw, [S / prod], 1, 0, od_ag, ctype=AG)["t_done"]
    assert Fraction(t_ar) == Fraction(t_rs) + Fraction(t_ag)


@pytest.mark.parametrize("seed", range(24))
def test_stand_alone_collectives_plan_and_queue_rules(oracle, seed):
    """Alg. 1 for CT = Reduce-Scatter (ascending loads) and All-Gather
    (descending loads, ties to the higher dimension so that equal loads give
    dimD..dim1) replayed with exact rationals, and the simulation checked by
    the independent schedule checker."""
    rng = np.random.default_rng(2100 + seed)
    ctype = RS if seed % 2 else AG
    D = int(rng.integers(1, 5))
    P, bw = _rand_net(rng, D, dyadic=True)
    C = int(rng.integers(1, 12))
    S = float(C * 2 ** int(rng.integers(18, 24)))
    f = Fraction(int(rng.integers(0, 4)), 16)
    fx = [float(rng.integers(0, 5)) * 2.0 ** -14 for _ in range(D)] if seed % 3 == 0 else None
    orders, loads, _ = oracle.plan(P, bw, S, C, 1, 1, float(f), fixed_delay=fx, ctype=ctype)
    coef = [Fraction(P[k] - 1, P[k]) / Fraction(bw[k]) for k in range(D)]
    load = [Fraction(fx[k]) if fx else Fraction(0) for k in range(D)]
    chunk = Fraction(S) / C
    for i in range(C):
        lo = min(load)
        kmin = load.index(lo)
        whole = chunk * P[kmin] * coef[kmin] if ctype == AG else chunk * coef[kmin]
        asc = (list(range(D)) if max(load) - lo < f * whole
               else sorted(range(D), key=lambda k: (load[k], k)))
        want = asc[::-1] if ctype == AG else asc
        assert order_dims(int(orders[i]), D) == want
        x = chunk
        for k in want:
            if ctype == AG:
                x *= P[k]
                load[k] += x * coef[k]
            else:
                load[k] += x * coef[k]
                x /= P[k]
    assert [Fraction(v) for v in loads[:D]] == load
    for intra in (0, 1):
        r = oracle.simulate(P, bw, [S], C, intra, orders, fixed_delay=fx, ctype=ctype)
        T, busy = rebuild_and_check(P, bw, [S], C, intra, orders, r["queue_order"],
                                    fixed_delay=fx, ctype=ctype)
        assert Fraction(r["t_done"]) == T
        assert [Fraction(v) for v in r["busy"][:D]] == busy


# ---------------------------------------------------------------- exhaustive search
def test_exhaustive_search_against_python_enumeration(oracle):
    """The search must return the minimum over all (D!)^C assignments
    (Sec. 4.1) and the first assignment that reaches it; re-enumerated here
    with itertools, every schedule's time taken from the independent checker."""
    from paper_2110_04478_amd import workloads as W
    rng = np.random.default_rng(77)
    cases = [(2, 4), (3, 3), (2, 6), (4, 2), (1, 5)]
    for D, C in cases:
        P, bw = _rand_net(rng, D, dyadic=True)
        S = float(C * 2 ** 22)
        for intra in (0, 1):
            b = W.make_batch([D], [P], [bw], S, C, 1, intra, 0.0)
            best_t, best_orders = oracle.search_batch(b, math.factorial(D) ** C)
            perms = [code_of(p) for p in itertools.permutations(range(D))]  # lexicographic
            best, arg = None, None
            # chunk 0 is the least significant digit of the assignment number
            for rev in itertools.product(perms, repeat=C):
                od = np.array(rev[::-1], dtype=np.uint8)
                r = oracle.simulate(P, bw, [S], C, intra, od)
                T, _ = rebuild_and_check(P, bw, [S], C, intra, od, r["queue_order"])
                if best is None or T < best:
                    best, arg = T, od
            assert Fraction(best_t[0]) == best
            assert best_orders[0, :C].tolist() == arg.tolist()
            themis = oracle.plan(P, bw, S, C, 1)[0]
            assert best_t[0] <= oracle.simulate(P, bw, [S], C, intra, themis)["t_done"]
    # too many schedules for the given bound -> no answer
    b = W.make_batch([3], [[4, 4, 4]], [[1e9, 1e9, 1e9]], 2.0 ** 24, 4, 1, 0, 0.0)
    t, od = oracle.search_batch(b, 6 ** 4 - 1)
    assert np.isnan(t[0]) and (od == 0xFF).all()


def test_worked_example_optimum(oracle):
    """4x4 worked example, 4 chunks: over all 2^4 assignments the best
    schedule takes 8 units for both policies -- greedy Themis is optimal here,
    and so is the baseline (derived; the paper's timing figure is not
    available as text)."""
    from paper_2110_04478_amd import workloads as W
    B0 = 100e9
    unit = 64 * MB * 0.75 / B0
    for intra in (0, 1):
        b = W.make_batch([2], [[4, 4]], [[B0, B0 / 2]], 256 * MB, 4, 1, intra, 0.0)
        t, od = oracle.search_batch(b, 16)
        assert t[0] / unit == pytest.approx(8.0, rel=1e-13)


# ------------------------------------------------- bandwidth provisioning classes
def test_provisioning_classes_of_the_motivating_network(oracle):
    """Sec. 3.3 / 6.3: on a 4x4 network the baseline is balanced exactly when
    BW(dim1) = 4 BW(dim2); with BW(dim1) = 2 BW(dim2) (the worked example)
    dim2's extra bandwidth is wasted by the baseline; BW(dim1) = 8 BW(dim2)
    starves dim2."""
    from paper_2110_04478_amd import workloads as W
    b = W.make_batch([2, 2, 2], [[4, 4]] * 3, [[400e9, 100e9], [200e9, 100e9], [800e9, 100e9]],
                     256 * MB, 4, 1, 0, 0.0)
    cls = oracle.classify_batch(b)
    assert cls[0].tolist() == [oracle.JUST_ENOUGH, oracle.OVER_PROVISIONED, oracle.UNDER_PROVISIONED]
    assert (cls[1:] == 0xFF).all()          # pairs outside a 2-D network


def test_provisioning_class_uses_the_product_of_sizes_between_the_pair(oracle):
    """Sec. 6.3: dimL is compared against P_K * .. * P_{L-1}, the factor by
    which the chunk shrinks between the two dimensions -- not P_K alone, not
    including P_L."""
    from paper_2110_04478_amd import workloads as W
    # 2 x 8 x 4 x 16: shrink factors (1,2)=2 (1,3)=16 (1,4)=64 (2,3)=8 (2,4)=32 (3,4)=4
    P = [2, 8, 4, 16]
    base = 6400e9
    bw = [base, base / 2, base / 16, base / 64]           # all pairs balanced
    b = W.make_batch([4], [P], [bw], 1e9, 4, 1, 0, 0.0)
    assert oracle.classify_batch(b)[:, 0].tolist() == [0] * 6
    bw = [base, base / 2, base / 8, base / 64]            # dim3 doubled
    b = W.make_batch([4], [P], [bw], 1e9, 4, 1, 0, 0.0)
    #        (1,2) (1,3) (1,4) (2,3) (2,4) (3,4)
    assert oracle.classify_batch(b)[:, 0].tolist() == [0, 1, 0, 1, 0, 2]
    b = W.make_batch([3], [P[:3]], [bw[:3]], 1e9, 4, 1, 0, 0.0)
    assert oracle.classify_batch(b)[:, 0].tolist() == [0, 1, 0xFF, 1, 0xFF, 0xFF]


def test_provisioning_class_agrees_with_baseline_loads(oracle):
    """With equal NPU counts on every dimension the (P-1)/P factors cancel, so
    the sign of the baseline's load difference N_K - N_L (Alg. 1's tracker
    after a baseline plan) is the provisioning class of the pair: equal loads
    <=> just enough, dimK busier <=> dimL over-provisioned."""
    from paper_2110_04478_amd import workloads as W
    rng = np.random.default_rng(63)
    n = 300
    D = rng.integers(2, 5, n)
    p = 2 ** rng.integers(1, 5, n)
    P = [[int(p[i])] * int(D[i]) for i in range(n)]
    bw = []
    for i in range(n):
        top = float(2 ** rng.integers(30, 40))
        # balanced ladder, each rung randomly tilted by a power of two (exact in fp64)
        bw.append([top / p[i] ** k * float(2.0 ** rng.integers(-1, 2)) for k in range(D[i])])
    b = W.make_batch(D, P, bw, 2.0 ** 30, 8, 0, 0, 0.0)
    cls = oracle.classify_batch(b)
    _, loads = oracle.plan_batch(b)
    seen = set()
    for i in range(n):
        for pair, (K, L) in enumerate(oracle.PAIRS):
            if L >= D[i]:
                assert cls[pair, i] == 0xFF
                continue
            diff = loads[K, i] - loads[L, i]
            want = 0 if diff == 0 else (1 if diff > 0 else 2)
            assert cls[pair, i] == want
            seen.add(want)
    assert seen == {0, 1, 2}


def test_provisioning_class_rejects_invalid_networks(oracle):
    from paper_2110_04478_amd import workloads as W
    b = W.make_batch([2, 2, 0], [[4, 1], [4, 4], [4, 4]], [[1e9, 1e9], [1e9, -1.0], [1e9, 1e9]],
                     1e6, 4, 1, 0, 0.0)
    assert (oracle.classify_batch(b) == 0xFF).all()


def test_overflowing_times_are_reported_as_invalid(oracle):
    """A stage time beyond binary64 (bandwidth 1e-300 B/s) has no place in the
    model: NaN / all-ones, like an invalid scenario.  A stage too short to move
    the clock is legal and still obeys the 1-D closed form on its own
    dimension."""
    from paper_2110_04478_amd import workloads as W
    b = W.make_batch([2, 2, 1], [[4, 4], [4, 4], [4]], [[1e-300, 1e9], [1e3, 1e300], [1e-300]],
                     2.0 ** 30, 8, 1, 1, 0.0, max_chunks=8)
    od, _ = oracle.plan_batch(b)
    t, q, busy = oracle.simulate_batch(b, od)
    assert np.isnan(t[0]) and np.isnan(busy[:, 0]).all() and (q[0] == 0xFFFF).all()
    assert np.isnan(t[2])
    assert np.isfinite(t[1]) and (q[1][:2, :16] != 0xFFFF).all()
    # Themis sends every chunk but the first through the (free) dim2 first, so
    # dim1 serves one full chunk and seven quarter chunks, twice each; dim2's
    # 1e-291 s stages vanish next to that
    assert od[1].tolist() == [code_of([0, 1])] + [code_of([1, 0])] * 7
    assert busy[0, 1] == pytest.approx(2 * 0.75 * 2.0 ** 27 * (1 + 7 / 4) / 1e3, rel=1e-12)
    assert t[1] == pytest.approx(busy[0, 1], rel=1e-9)


def test_sweep_best_hand_values(oracle):
    """Best threshold and speed-up (Sec. 5.3, Sec. 6.1) on values worked out by
    hand: the lowest index among equal minima, NaN entries skipped, an all-NaN
    column, and the speed-up taken against the baseline column at a = 0."""
    nan = float("nan")
    #            a=0            a=1            a=2          (columns: baseline, Themis+FIFO, Themis+SCF)
    t = np.array([[[8.0, 7.0, 6.0], [8.0, 5.0, 6.0], [8.0, 5.0, 4.0]],
                  [[2.0, nan, nan], [2.0, 1.0, nan], [2.0, 0.5, nan]],
                  [[3.0, 3.0, 9.0], [3.0, 3.0, 9.0], [3.0, 3.0, 1.5]]])
    best_t, best_thr, speedup = oracle.sweep_best(t, baseline_col=0)
    assert best_t[0].tolist() == [8.0, 5.0, 4.0] and best_thr[0].tolist() == [0, 1, 2]
    assert speedup[0].tolist() == [1.0, 1.6, 2.0]
    assert best_t[1, :2].tolist() == [2.0, 0.5] and np.isnan(best_t[1, 2])
    assert best_thr[1].tolist() == [0, 2, 0xFFFFFFFF]
    assert speedup[1, :2].tolist() == [1.0, 4.0] and np.isnan(speedup[1, 2])
    assert best_thr[2].tolist() == [0, 0, 2] and speedup[2].tolist() == [1.0, 1.0, 2.0]
    # no baseline column: no speed-up
    assert oracle.sweep_best(t)[2] is None


def test_sweep_best_is_the_library_minimum(oracle):
    """Against numpy's minimum / argmin on a real sweep of the oracle: the best
    time is the minimum over the threshold axis, the index the first position
    of it, and no threshold beats the best one."""
    from paper_2110_04478_amd import workloads as W
    b = W.mixed(300, seed=11, max_chunks=24)
    thr = np.array([0.0, 1 / 64, 1 / 16, 1 / 4, 1.0])
    t = oracle.sweep(b, thr, 7, threads=4)
    best_t, best_thr, speedup = oracle.sweep_best(t, baseline_col=0)
    assert np.array_equal(best_t, t.min(axis=1))
    assert np.array_equal(best_thr, t.argmin(axis=1).astype(np.uint32))
    assert np.array_equal(speedup, t[:, 0, 0][:, None] / t.min(axis=1))
    assert (speedup[:, 0] == 1.0).all()          # the baseline against itself
    assert (t >= best_t[:, None, :]).all()
