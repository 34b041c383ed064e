"""Independent checker for a simulated schedule (used to pin the oracle).

It does not simulate.  Given the per-dimension executed-operation lists that a
simulator reports, it rebuilds every operation's start and end time from the
two precedence relations that any valid execution obeys (one operation at a
time per dimension, a chunk's stages one after another), and then verifies,
operation by operation, the rules of the paper's queue model (Sec. 4.3,
4.6.2): servers never idle while a chunk waits, and the chunk a dimension
starts is the first in FIFO or Smallest-Chunk-First order among those waiting
at that instant.  Stage times follow the latency model written out with exact
rationals (Sec. 4.5), independent of the oracle's floating point code.
"""
from fractions import Fraction


def order_dims(code, D):
    return [(code >> (2 * j)) & 3 for j in range(D)]


def exact_stage_times(npus, bw, chunk, dims):
    """Exact (time, size-before) of the D Reduce-Scatter stages of one chunk."""
    x = Fraction(chunk)
    out = []
    for k in dims:
        P = Fraction(int(npus[k]))
        out.append(((P - 1) / P * x / Fraction(bw[k]), x))
        x = x / P
    return out, x


def exact_all_gather_times(npus, bw, chunk, dims):
    """Exact (time, size-before) of the D stages of a stand-alone All-Gather:
    a stage on k grows the resident size by P_k and moves (P_k-1)/P_k of the
    grown size (Sec. 2.1, 4.5)."""
    y = Fraction(chunk)
    out = []
    for k in dims:
        P = Fraction(int(npus[k]))
        out.append(((P - 1) / P * (y * P) / Fraction(bw[k]), y))
        y = y * P
    return out


def rebuild_and_check(npus, bw, coll_sizes, C, intra_policy, orders,
                      queue_order, release=None, fixed_delay=None, ctype=0):
    """Returns (T, busy[D]) as Fractions after asserting the schedule is a
    valid execution under the policy.  queue_order[k] lists (g<<1|phase)."""
    D = len(npus)
    Q = len(coll_sizes)
    G = Q * C
    # stage table per chunk: list of (dim, phase, service, size_before)
    stages = []
    for g in range(G):
        q = g // C
        dims = order_dims(int(orders[g]), D)
        assert sorted(dims) == list(range(D))
        if ctype == 2:  # stand-alone All-Gather: D stages, phase bit 1
            ag = exact_all_gather_times(npus, bw, Fraction(coll_sizes[q]) / C, dims)
            if fixed_delay is not None:
                ag = [(t + Fraction(fixed_delay[k]), y) for (t, y), k in zip(ag, dims)]
            stages.append([(dims[j], 1, ag[j][0], ag[j][1]) for j in range(D)])
            continue
        rs, xD = exact_stage_times(npus, bw, Fraction(coll_sizes[q]) / C, dims)
        if fixed_delay is not None:  # A_K of Sec. 4.5: a fixed delay per stage on that dimension
            rs = [(t + Fraction(fixed_delay[k]), x) for (t, x), k in zip(rs, dims)]
        st = [(dims[j], 0, rs[j][0], rs[j][1]) for j in range(D)]
        if ctype == 0:  # All-Reduce: the All-Gather stages follow in reverse order
            y = xD
            for j in reversed(range(D)):
                st.append((dims[j], 1, rs[j][0], y))
                y = y * int(npus[dims[j]])
        stages.append(st)

    rel = [Fraction(0) if release is None else Fraction(release[g // C])
           for g in range(G)]
    # position of every (g, stage index) in its dimension's list
    per_chunk = 2 if ctype == 0 else 1
    nops = per_chunk * G
    queue_order = [list(row[:nops]) for row in queue_order]
    for k in range(D):
        ops = [int(e) for e in queue_order[k]]
        want = (list(range(2 * G)) if ctype == 0 else
                [2 * g + (1 if ctype == 2 else 0) for g in range(G)])
        assert sorted(ops) == want, "every (chunk, phase) exactly once per dimension"

    # iterative longest-path evaluation over the two precedence chains
    stage_idx = {}
    for g in range(G):
        for s, (k, ph, _, _) in enumerate(stages[g]):
            stage_idx[(k, g, ph)] = s
    start, end = {}, {}
    ptr = [0] * D
    free_at = [Fraction(0)] * D
    progressed = True
    done_ops = 0
    while progressed:
        progressed = False
        for k in range(D):
            while ptr[k] < nops:
                e = int(queue_order[k][ptr[k]])
                g, ph = e >> 1, e & 1
                s = stage_idx[(k, g, ph)]
                if s > 0 and (g, s - 1) not in end:
                    break
                ready = rel[g] if s == 0 else end[(g, s - 1)]
                b = max(free_at[k], ready)
                start[(g, s)] = b
                end[(g, s)] = b + stages[g][s][2]
                free_at[k] = end[(g, s)]
                ptr[k] += 1
                done_ops += 1
                progressed = True
    assert done_ops == D * nops, "executed order lists are not a consistent schedule"

    # policy conformance, operation by operation
    for k in range(D):
        prev_end = Fraction(0)
        served = set()
        for e in queue_order[k]:
            e = int(e)
            g, ph = e >> 1, e & 1
            s = stage_idx[(k, g, ph)]
            t0 = start[(g, s)]
            cands = []
            for g2 in range(G):
                for s2, (k2, ph2, _, size2) in enumerate(stages[g2]):
                    if k2 != k or (g2, s2) in served:
                        continue
                    arr = rel[g2] if s2 == 0 else end[(g2, s2 - 1)]
                    if arr <= t0:
                        key = ((size2, arr, g2) if intra_policy == 1 else (arr, g2))
                        cands.append((key, g2, s2, arr))
            assert cands, "dimension started a chunk that was not waiting"
            best = min(cands)
            assert (best[1], best[2]) == (g, s), (
                f"dim {k}: started chunk {g} stage {s} but {best[1]} stage "
                f"{best[2]} was first in queue order")
            if t0 > prev_end:  # the server idled: nobody may have been waiting
                assert all(c[3] == t0 for c in cands), "server idled with a chunk waiting"
            served.add((g, s))
            prev_end = end[(g, s)]

    T = max(end.values())
    busy = [sum((st[2] for g in range(G) for st in stages[g] if st[0] == k), Fraction(0))
            for k in range(D)]
    return T, busy
