"""ctypes front end of the C oracle (oracle/themis_oracle.c).

Test infrastructure: called by tests, the smoke check and the benchmark's CPU
baseline only.  Takes any object with the attributes of a scenario batch
(n, max_chunks, threshold_mode, ndims, npus, bw, size_bytes, chunks,
inter_policy, intra_policy, threshold, max_coll, n_coll, coll_size,
release_time as numpy arrays); it imports nothing from the GPU package.
"""
from __future__ import annotations

import ctypes as C
from concurrent.futures import ThreadPoolExecutor

import numpy as np

from . import build as _build

_lib = None

_u8p = C.POINTER(C.c_uint8)
_u16p = C.POINTER(C.c_uint16)
_u32p = C.POINTER(C.c_uint32)
_f64p = C.POINTER(C.c_double)


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(_build.build())
        L.to_plan.restype = C.c_int
        L.to_plan.argtypes = [C.c_int, _u32p, _f64p, _f64p, C.c_int, C.c_double, C.c_uint32,
                              C.c_int, C.c_int, C.c_double, _u8p, _f64p, _f64p]
        L.to_simulate.restype = C.c_int
        L.to_simulate.argtypes = [C.c_int, _u32p, _f64p, _f64p, C.c_int, C.c_uint32, _f64p,
                                  _f64p, C.c_uint32, C.c_int, _u8p, _f64p,
                                  _f64p, _u32p, _f64p]
        L.to_plan_batch.restype = None
        L.to_plan_batch.argtypes = [
            C.c_uint64, C.c_uint64, C.c_uint64, C.c_uint32, C.c_int, _u8p,
            _u32p, _f64p, _f64p, _u32p, _u8p, _f64p, _f64p, _u8p, C.c_uint32, _u32p,
            _f64p, _u8p, _f64p]
        L.to_simulate_batch.restype = None
        L.to_simulate_batch.argtypes = [
            C.c_uint64, C.c_uint64, C.c_uint64, C.c_uint32, _u8p, _u32p,
            _f64p, _f64p, _u32p, _u8p, _f64p, _u8p, C.c_uint32, _u32p, _f64p, _f64p,
            _u8p, _f64p, _u16p, _f64p]
        L.to_sweep.restype = None
        L.to_sweep.argtypes = [
            C.c_uint64, C.c_uint64, C.c_uint64, C.c_uint32, C.c_int, _u8p,
            _u32p, _f64p, _f64p, _u32p, _f64p, C.c_int, _f64p, C.c_int, C.c_uint,
            _f64p]
        L.to_metrics_batch.restype = None
        L.to_metrics_batch.argtypes = [
            C.c_uint64, C.c_uint64, C.c_uint64, _u8p, _f64p, _f64p, C.c_uint32,
            _u32p, _f64p, _f64p, _f64p, _f64p, _f64p]
        L.to_search_batch.restype = None
        L.to_search_batch.argtypes = [
            C.c_uint64, C.c_uint64, C.c_uint64, C.c_uint32, _u8p, _u32p, _f64p,
            _f64p, _u32p, _u8p, _f64p, _u8p, C.c_uint64, _f64p, _u8p]
        L.to_beam_search_batch.restype = None
        L.to_beam_search_batch.argtypes = [
            C.c_uint64, C.c_uint64, C.c_uint64, C.c_uint32, C.c_int, _u8p, _u32p, _f64p,
            _f64p, _u32p, _u8p, _u8p, _f64p, _f64p, _u8p, C.c_uint32, _f64p, _u8p]
        L.to_classify_batch.restype = None
        L.to_classify_batch.argtypes = [C.c_uint64, C.c_uint64, C.c_uint64, _u8p, _u32p, _f64p, _u8p]
        L.to_sweep_best.restype = None
        L.to_sweep_best.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, _f64p, C.c_int, _f64p, _u32p, _f64p]
        L.to_latency_coef.restype = None
        L.to_latency_coef.argtypes = [C.c_int, _u32p, _f64p, _f64p]
        _lib = L
    return _lib


def _p(a, ty):
    return None if a is None else a.ctypes.data_as(ty)


def _arr(a, dt):
    return np.ascontiguousarray(np.asarray(a, dtype=dt))


def _ranges(n, threads):
    threads = max(1, min(int(threads), n if n else 1))
    edges = np.linspace(0, n, threads + 1).astype(np.int64)
    return [(int(edges[t]), int(edges[t + 1])) for t in range(threads)
            if edges[t + 1] > edges[t]]


def _fan_out(fn, n, threads):
    rs = _ranges(n, threads)
    if len(rs) <= 1:
        for b, e in rs:
            fn(b, e)
        return
    # ctypes releases the GIL during the foreign call, so these run in parallel
    with ThreadPoolExecutor(max_workers=len(rs)) as ex:
        list(ex.map(lambda r: fn(*r), rs))


# -- single scenario --------------------------------------------------------
def latency_coef(npus, bw):
    P = _arr(npus, np.uint32)
    B = _arr(bw, np.float64)
    out = np.zeros(len(P))
    lib().to_latency_coef(len(P), _p(P, _u32p), _p(B, _f64p), _p(out, _f64p))
    return out


def _fixed4(fixed_delay, D):
    if fixed_delay is None:
        return None
    f = np.zeros(4)
    f[:D] = fixed_delay
    return f


ALL_REDUCE, REDUCE_SCATTER, ALL_GATHER = 0, 1, 2


def plan(npus, bw, size_bytes, chunks, inter_policy=1, threshold_mode=0,
         threshold=0.0, fixed_delay=None, ctype=ALL_REDUCE):
    """Alg. 1 for one collective.  Returns (orders u8[C], loads f64[4],
    stage_time f64[C,4]) or None if the inputs are invalid."""
    D = len(npus)
    P = np.zeros(4, np.uint32); P[:D] = npus
    B = np.ones(4); B[:D] = bw
    orders = np.zeros(chunks, np.uint8)
    loads = np.zeros(4)
    st = np.zeros((chunks, 4))
    fx = _fixed4(fixed_delay, D)
    ok = lib().to_plan(D, _p(P, _u32p), _p(B, _f64p), _p(fx, _f64p), int(ctype), float(size_bytes),
                       int(chunks), int(inter_policy), int(threshold_mode),
                       float(threshold), _p(orders, _u8p), _p(loads, _f64p),
                       _p(st, _f64p))
    return (orders, loads, st) if ok else None


def simulate(npus, bw, coll_sizes, chunks, intra_policy, orders, release=None,
             fixed_delay=None, ctype=ALL_REDUCE):
    """Queue simulation of one scenario (one or several collectives).
    Returns dict(t_done, coll_done, queue_order[D][2G], busy[4]) or None."""
    D = len(npus)
    P = np.zeros(4, np.uint32); P[:D] = npus
    B = np.ones(4); B[:D] = bw
    cs = _arr(np.atleast_1d(coll_sizes), np.float64)
    Q = len(cs)
    G = Q * int(chunks)
    od = _arr(orders, np.uint8).reshape(-1)
    assert od.shape[0] == G
    rl = None if release is None else _arr(release, np.float64)
    t = C.c_double(0.0)
    cd = np.zeros(Q)
    qo = np.zeros((4, 2 * G), np.uint32)
    busy = np.zeros(4)
    fx = _fixed4(fixed_delay, D)
    ok = lib().to_simulate(D, _p(P, _u32p), _p(B, _f64p), _p(fx, _f64p), int(ctype), Q, _p(cs, _f64p),
                           _p(rl, _f64p), int(chunks), int(intra_policy),
                           _p(od, _u8p), C.byref(t), _p(cd, _f64p),
                           _p(qo, _u32p), _p(busy, _f64p))
    if not ok:
        return None
    return dict(t_done=t.value, coll_done=cd, queue_order=qo[:D], busy=busy)


# -- batches ------------------------------------------------------------------
def _fixed(b):
    f = getattr(b, "fixed_delay", None)
    return None if f is None else _arr(f, np.float64)


def _ctype(b):
    c = getattr(b, "collective_type", None)
    return None if c is None else _arr(c, np.uint8)


def _trace(b):
    if getattr(b, "n_coll", None) is None:
        return 0, None, None, None
    return (int(b.max_coll), _arr(b.n_coll, np.uint32),
            _arr(b.coll_size, np.float64),
            None if b.release_time is None else _arr(b.release_time, np.float64))


def plan_batch(b, threads=1):
    """Returns (orders u8[n, slots], loads f64[4, n])."""
    mc, ncoll, csize, _ = _trace(b)
    slots = b.max_chunks * (mc if ncoll is not None else 1)
    orders = np.empty((b.n, slots), np.uint8)
    loads = np.empty((4, b.n))
    a = dict(ndims=_arr(b.ndims, np.uint8), npus=_arr(b.npus, np.uint32),
             bw=_arr(b.bw, np.float64), size=_arr(b.size_bytes, np.float64),
             chunks=_arr(b.chunks, np.uint32),
             inter=_arr(b.inter_policy, np.uint8),
             thr=_arr(b.threshold, np.float64))
    fx = _fixed(b)
    ct = _ctype(b)

    def run(lo, hi):
        lib().to_plan_batch(
            b.n, lo, hi, b.max_chunks, b.threshold_mode, _p(a["ndims"], _u8p),
            _p(a["npus"], _u32p), _p(a["bw"], _f64p), _p(a["size"], _f64p),
            _p(a["chunks"], _u32p), _p(a["inter"], _u8p), _p(a["thr"], _f64p),
            _p(fx, _f64p), _p(ct, _u8p), mc, _p(ncoll, _u32p), _p(csize, _f64p),
            _p(orders, _u8p), _p(loads, _f64p))
    _fan_out(run, b.n, threads)
    return orders, loads


def simulate_batch(b, orders, want_queue_order=True, threads=1):
    """Returns (t_done f64[n], queue_order u16[n,4,2*slots] or None,
    busy f64[4,n])."""
    mc, ncoll, csize, rel = _trace(b)
    slots = b.max_chunks * (mc if ncoll is not None else 1)
    od = _arr(orders, np.uint8).reshape(b.n, slots)
    t = np.empty(b.n)
    qo = np.empty((b.n, 4, 2 * slots), np.uint16) if want_queue_order else None
    busy = np.empty((4, b.n))
    a = dict(ndims=_arr(b.ndims, np.uint8), npus=_arr(b.npus, np.uint32),
             bw=_arr(b.bw, np.float64), size=_arr(b.size_bytes, np.float64),
             chunks=_arr(b.chunks, np.uint32),
             intra=_arr(b.intra_policy, np.uint8))
    fx = _fixed(b)
    ct = _ctype(b)

    def run(lo, hi):
        lib().to_simulate_batch(
            b.n, lo, hi, b.max_chunks, _p(a["ndims"], _u8p),
            _p(a["npus"], _u32p), _p(a["bw"], _f64p), _p(a["size"], _f64p),
            _p(a["chunks"], _u32p), _p(a["intra"], _u8p), _p(fx, _f64p), _p(ct, _u8p), mc,
            _p(ncoll, _u32p), _p(csize, _f64p), _p(rel, _f64p), _p(od, _u8p),
            _p(t, _f64p), _p(qo, _u16p), _p(busy, _f64p))
    _fan_out(run, b.n, threads)
    return t, qo, busy


def sweep(b, thr, policy_mask, thr_per_scenario=False, threads=1):
    """Returns t_done f64[n, n_thr, n_pol]."""
    thr = _arr(thr, np.float64)
    n_thr = thr.shape[0]
    n_pol = bin(policy_mask & 7).count("1")
    out = np.empty((b.n, n_thr, n_pol))
    a = dict(ndims=_arr(b.ndims, np.uint8), npus=_arr(b.npus, np.uint32),
             bw=_arr(b.bw, np.float64), size=_arr(b.size_bytes, np.float64),
             chunks=_arr(b.chunks, np.uint32))
    fx = _fixed(b)

    def run(lo, hi):
        lib().to_sweep(
            b.n, lo, hi, b.max_chunks, b.threshold_mode, _p(a["ndims"], _u8p),
            _p(a["npus"], _u32p), _p(a["bw"], _f64p), _p(a["size"], _f64p),
            _p(a["chunks"], _u32p), _p(fx, _f64p), n_thr, _p(thr, _f64p),
            1 if thr_per_scenario else 0, policy_mask, _p(out, _f64p))
    _fan_out(run, b.n, threads)
    return out


def metrics_batch(b, t_done, transfer, threads=1):
    """Average bandwidth utilisation and the Ideal time -> (util f64[n], ideal f64[n])."""
    mc, ncoll, csize, _ = _trace(b)
    t = _arr(t_done, np.float64)
    tr = _arr(transfer, np.float64)
    util = np.empty(b.n)
    ideal = np.empty(b.n)
    nd, bw, sz = _arr(b.ndims, np.uint8), _arr(b.bw, np.float64), _arr(b.size_bytes, np.float64)

    def run(lo, hi):
        lib().to_metrics_batch(b.n, lo, hi, _p(nd, _u8p), _p(bw, _f64p), _p(sz, _f64p), mc,
                               _p(ncoll, _u32p), _p(csize, _f64p), _p(t, _f64p), _p(tr, _f64p),
                               _p(util, _f64p), _p(ideal, _f64p))
    _fan_out(run, b.n, threads)
    return util, ideal


def search_batch(b, max_assignments, threads=1):
    """Exhaustive search over per-chunk orders -> (best_t f64[n], best_orders u8[n, max_chunks])."""
    best_t = np.empty(b.n)
    best_orders = np.empty((b.n, b.max_chunks), np.uint8)
    a = dict(ndims=_arr(b.ndims, np.uint8), npus=_arr(b.npus, np.uint32),
             bw=_arr(b.bw, np.float64), size=_arr(b.size_bytes, np.float64),
             chunks=_arr(b.chunks, np.uint32), intra=_arr(b.intra_policy, np.uint8))
    fx, ct = _fixed(b), _ctype(b)

    def run(lo, hi):
        lib().to_search_batch(
            b.n, lo, hi, b.max_chunks, _p(a["ndims"], _u8p), _p(a["npus"], _u32p),
            _p(a["bw"], _f64p), _p(a["size"], _f64p), _p(a["chunks"], _u32p),
            _p(a["intra"], _u8p), _p(fx, _f64p), _p(ct, _u8p), int(max_assignments),
            _p(best_t, _f64p), _p(best_orders, _u8p))
    _fan_out(run, b.n, threads)
    return best_t, best_orders


def beam_search_batch(b, width, threads=1):
    """Beam search over per-chunk orders, seeded with the greedy plan ->
    (best_t f64[n], best_orders u8[n, max_chunks])."""
    best_t = np.empty(b.n)
    best_orders = np.empty((b.n, b.max_chunks), np.uint8)
    a = dict(ndims=_arr(b.ndims, np.uint8), npus=_arr(b.npus, np.uint32),
             bw=_arr(b.bw, np.float64), size=_arr(b.size_bytes, np.float64),
             chunks=_arr(b.chunks, np.uint32), inter=_arr(b.inter_policy, np.uint8),
             intra=_arr(b.intra_policy, np.uint8), thr=_arr(b.threshold, np.float64))
    fx, ct = _fixed(b), _ctype(b)

    def run(lo, hi):
        lib().to_beam_search_batch(
            b.n, lo, hi, b.max_chunks, int(b.threshold_mode), _p(a["ndims"], _u8p),
            _p(a["npus"], _u32p), _p(a["bw"], _f64p), _p(a["size"], _f64p),
            _p(a["chunks"], _u32p), _p(a["inter"], _u8p), _p(a["intra"], _u8p),
            _p(a["thr"], _f64p), _p(fx, _f64p), _p(ct, _u8p), int(width),
            _p(best_t, _f64p), _p(best_orders, _u8p))
    _fan_out(run, b.n, threads)
    return best_t, best_orders


JUST_ENOUGH, OVER_PROVISIONED, UNDER_PROVISIONED = 0, 1, 2
PAIRS = ((0, 1), (0, 2), (0, 3), (1, 2), (1, 3), (2, 3))


def classify_batch(b):
    """Bandwidth provisioning class of every dimension pair (Sec. 6.3) -> u8[6, n]."""
    out = np.empty((6, b.n), np.uint8)
    nd, P, bw = _arr(b.ndims, np.uint8), _arr(b.npus, np.uint32), _arr(b.bw, np.float64)
    lib().to_classify_batch(b.n, 0, b.n, _p(nd, _u8p), _p(P, _u32p), _p(bw, _f64p), _p(out, _u8p))
    return out


def sweep_best(t_done, baseline_col=-1):
    """Best threshold per scenario and scheduler of a sweep result [n, n_thr, n_pol]
    (Sec. 5.3, Sec. 6.1) -> (best_t f64[n, n_pol], best_thr u32[n, n_pol],
    speedup f64[n, n_pol] or None)."""
    t = _arr(t_done, np.float64)
    n, n_thr, n_pol = t.shape
    best_t = np.empty((n, n_pol), np.float64)
    best_thr = np.empty((n, n_pol), np.uint32)
    speedup = np.empty((n, n_pol), np.float64) if baseline_col >= 0 else None
    lib().to_sweep_best(n, n_thr, n_pol, _p(t, _f64p), baseline_col, _p(best_t, _f64p),
                        _p(best_thr, _u32p), _p(speedup, _f64p) if speedup is not None else None)
    return best_t, best_thr, speedup
