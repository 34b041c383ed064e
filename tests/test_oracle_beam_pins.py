"""CPU pins of the oracle's beam search over per-chunk orders (Sec. 4.1,
observation 2: every chunk may take its own dimension order; Sec. 4.2 walks
that space greedily, the beam keeps several partial schedules instead of one).

What fixes the result from outside the oracle's own search code:
  * a beam that never drops anything is the exhaustive search (pinned itself
    against an itertools enumeration timed by the exact-rational checker);
  * the procedure re-stated here in Python -- extend, score, keep the best,
    equal times by assignment number -- with every score taken from the
    single-collective simulation and checked by the rational checker;
  * the result is never worse than the greedy plan of Alg. 1, and never better
    than the exhaustive optimum;
  * a width-1 case worked by hand.
"""
import itertools
import math
from fractions import Fraction

import numpy as np
import pytest

from test_oracle_pins import MB, _rand_net, code_of  # noqa: F401
from schedule_checker import rebuild_and_check


def _beam_in_python(oracle, P, bw, S, C, inter, intra, thr_mode, thr, width, fixed=None, ctype=0):
    """The search as the header of the oracle's to_beam_search states it."""
    D = len(P)
    perms = [code_of(p) for p in itertools.permutations(range(D))]   # lexicographic
    beam = [((), 0.0)]                                               # (digits, time)
    for m in range(1, C + 1):
        size_m = S if m == C else (S / C) * m
        cands = []
        for digits, _ in beam:
            for j in range(len(perms)):
                dg = digits + (j,)
                od = np.array([perms[x] for x in dg], dtype=np.uint8)
                r = oracle.simulate(P, bw, [size_m], m, intra, od, fixed_delay=fixed, ctype=ctype)
                T, _ = rebuild_and_check(P, bw, [size_m], m, intra, od, r["queue_order"],
                                         fixed_delay=fixed, ctype=ctype)
                # (exact on dyadic networks, where every product and sum is)
                assert abs(Fraction(r["t_done"]) - T) <= T * Fraction(1, 10 ** 12)
                # assignment number: the newest chunk's digit is the most significant
                cands.append((r["t_done"], dg[::-1], dg))
        cands.sort(key=lambda c: (c[0], c[1]))
        beam = [(c[2], c[0]) for c in cands[:width]]
    digits, best = beam[0]
    orders = [perms[x] for x in digits]
    greedy = oracle.plan(P, bw, S, C, inter, thr_mode, thr, fixed_delay=fixed, ctype=ctype)[0]
    tg = oracle.simulate(P, bw, [S], C, intra, greedy, fixed_delay=fixed, ctype=ctype)["t_done"]
    if tg < best:
        best, orders = tg, [int(x) for x in greedy[:C]]
    return best, orders


def test_a_beam_that_drops_nothing_is_the_exhaustive_search(oracle):
    from paper_2110_04478_amd import workloads as W
    rng = np.random.default_rng(91)
    for D, C in [(2, 4), (3, 2), (2, 6), (1, 5), (4, 1)]:
        F = math.factorial(D)
        assert F ** C <= 64
        P, bw = _rand_net(rng, D, dyadic=True)
        S = float(C * 2 ** 22)
        for intra in (0, 1):
            b = W.make_batch([D], [P], [bw], S, C, 0, intra, 0.0)   # baseline seed: cannot win a tie
            want_t, want_od = oracle.search_batch(b, F ** C)
            for width in (F ** C, 64):
                t, od = oracle.beam_search_batch(b, width)
                assert t[0] == want_t[0]
                assert od[0].tolist() == want_od[0].tolist()


@pytest.mark.parametrize("seed", range(6))
def test_beam_search_against_its_restatement_in_python(oracle, seed):
    from paper_2110_04478_amd import workloads as W
    rng = np.random.default_rng(400 + seed)
    D = int(rng.integers(2, 4))
    C = int(rng.integers(3, 7))
    dyadic = seed % 2 == 0           # dyadic networks tie all the time: the number decides
    P, bw = _rand_net(rng, D, dyadic=dyadic)
    S = float(C * 2 ** 22) if dyadic else float(rng.uniform(1e6, 1e9))
    ctype = seed % 3
    fixed = [float(rng.integers(0, 4)) * 2.0 ** -16 for _ in range(D)] if seed % 2 else None
    for intra in (0, 1):
        for width in (1, 2, 5):
            b = W.make_batch([D], [P], [bw], S, C, 1, intra, 0.0, fixed_delay=None if fixed is None else [fixed])
            b.collective_type = np.array([ctype], dtype=np.uint8)
            t, od = oracle.beam_search_batch(b, width)
            want_t, want_od = _beam_in_python(oracle, P, bw, S, C, 1, intra, 0, 0.0, width,
                                              fixed=fixed, ctype=ctype)
            assert t[0] == want_t
            assert od[0, :C].tolist() == want_od
            assert (od[0, C:] == 0xFF).all()


@pytest.mark.parametrize("seed", range(8))
def test_partial_schedules_are_scored_at_the_full_chunk_size(oracle, seed):
    """Fixed per-stage delays as long as the stages themselves: a partial
    schedule scored with chunks of S/m instead of S/C bytes would weigh delays
    and transfers differently and keep other schedules."""
    from paper_2110_04478_amd import workloads as W
    rng = np.random.default_rng(900 + seed)
    D, C = 2, 6
    P = [int(x) for x in rng.choice([2, 4, 8], D)]
    bw = [float(2.0 ** rng.integers(28, 32)) for _ in range(D)]
    S = float(C * 2 ** 20)
    # a stage moves 2^20 bytes (or a fraction) at 2^28..2^31 B/s: 2^-8 .. 2^-14 s
    fixed = [float(rng.integers(1, 6)) * 2.0 ** -10 for _ in range(D)]
    for intra in (0, 1):
        b = W.make_batch([D], [P], [bw], S, C, 1, intra, 0.0, fixed_delay=[fixed])
        for width in (1, 2):
            t, od = oracle.beam_search_batch(b, width)
            want_t, want_od = _beam_in_python(oracle, P, bw, S, C, 1, intra, 0, 0.0, width, fixed=fixed)
            assert t[0] == want_t
            assert od[0, :C].tolist() == want_od


def test_beam_search_between_the_greedy_plan_and_the_optimum(oracle):
    from paper_2110_04478_amd import workloads as W
    rng = np.random.default_rng(17)
    for _ in range(12):
        D = int(rng.integers(2, 4))
        C = 4 if D == 2 else 3
        P, bw = _rand_net(rng, D, dyadic=False)
        S = float(rng.uniform(1e6, 1e9))
        for intra in (0, 1):
            b = W.make_batch([D], [P], [bw], S, C, 1, intra, 0.0)
            greedy = oracle.plan(P, bw, S, C, 1)[0]
            tg = oracle.simulate(P, bw, [S], C, intra, greedy)["t_done"]
            opt, _ = oracle.search_batch(b, math.factorial(D) ** C)
            for width in (1, 3, 8):
                t, od = oracle.beam_search_batch(b, width)
                assert opt[0] <= t[0] <= tg
                # the orders returned reach the time returned
                assert oracle.simulate(P, bw, [S], C, intra, od[0, :C])["t_done"] == t[0]


def test_width_one_by_hand(oracle):
    """2-D, P = (2, 2), bandwidths 2^30 and 2^33 B/s, 3 chunks of 2^22 bytes, FIFO.
    With U = 2^-20 s a chunk's stages take: order (0,1): 2048 U on dim 0 and
    128 U on dim 1; order (1,0): 256 U on dim 1 and 1024 U on dim 0.
    Width 1: chunk 0 alone: (0,1) ends at 2*2048+2*128 = 4352 U, (1,0) at
    2*256+2*1024 = 2560 U -> keep (1,0).  Chunk 1 after it: both chunks (1,0)
    serialise on dim 0: 256 + 4*1024 = 4352 ... the search settles every step
    on the smaller time; its final time must be that of its own orders and no
    larger than the all-(1,0) schedule's 256 + 6*1024 + ... bound below."""
    from paper_2110_04478_amd import workloads as W
    U = 2.0 ** -20
    P, bw, S, C = [2, 2], [2.0 ** 30, 2.0 ** 33], 3 * 2.0 ** 22, 3
    b = W.make_batch([2], [P], [bw], S, C, 0, 0, 0.0)
    t, od = oracle.beam_search_batch(b, 1)
    # step 1 by hand: the single chunk takes order (1,0)
    one = W.make_batch([2], [P], [bw], S / 3, 1, 0, 0, 0.0)
    t1, od1 = oracle.beam_search_batch(one, 1)
    assert t1[0] == 2560 * U and od1[0, 0] == code_of((1, 0))
    assert od[0, 0] == code_of((1, 0))
    # the full result is consistent and no worse than every chunk on (1,0)
    all10 = np.array([code_of((1, 0))] * 3, dtype=np.uint8)
    assert t[0] <= oracle.simulate(P, bw, [S], C, 0, all10)["t_done"]
    assert oracle.simulate(P, bw, [S], C, 0, od[0, :C])["t_done"] == t[0]


def test_beam_search_rejects_what_it_cannot_take(oracle):
    from paper_2110_04478_amd import workloads as W
    b = W.make_batch([2], [[4, 4]], [[1e9, 1e9]], 2.0 ** 24, 4, 1, 0, 0.0)
    for width in (0, 65):
        t, od = oracle.beam_search_batch(b, width)
        assert np.isnan(t[0]) and (od == 0xFF).all()
    bad = W.make_batch([2], [[4, 1]], [[1e9, 1e9]], 2.0 ** 24, 4, 1, 0, 0.0)
    t, od = oracle.beam_search_batch(bad, 4)
    assert np.isnan(t[0]) and (od == 0xFF).all()
