"""Seeded synthetic scenario batches (host side, numpy only).

This module holds none of the method's arithmetic: it only draws the inputs --
network shapes, bandwidths, collective sizes, chunk counts, policies and
thresholds -- that both the CPU oracle and the GPU library are then given.
The shapes follow the paper's evaluation (Table 2: P_k between 4 and 64,
aggregate bandwidth 400-3000 Gb/s per NPU and dimension; Sec. 6.1: All-Reduce
of 100 MB-1 GB, 64 chunks by default, 4..512 in the sensitivity study).

Random numbers come from a counter-based generator: value k of scenario i is
splitmix64(seed + i*16 + k), so any sub-range of a batch can be regenerated
without the rest.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np

MAX_DIMS = 4
INTER_BASELINE, INTER_THEMIS = 0, 1
INTRA_FIFO, INTRA_SCF = 0, 1
THR_ABS, THR_REL = 0, 1
SWEEP_BASELINE, SWEEP_THEMIS_FIFO, SWEEP_THEMIS_SCF = 1, 2, 4
COLL_ALL_REDUCE, COLL_REDUCE_SCATTER, COLL_ALL_GATHER = 0, 1, 2

SEED_BASE = 0x211004478
MIB = float(2 ** 20)
GIB = float(2 ** 30)


@dataclass
class ScenarioBatch:
    """Structure-of-arrays description of n scenarios (host numpy arrays)."""
    n: int
    max_chunks: int
    threshold_mode: int
    ndims: np.ndarray         # u8  [n]
    npus: np.ndarray          # u32 [4, n]
    bw: np.ndarray            # f64 [4, n]  bytes/s
    size_bytes: np.ndarray    # f64 [n]
    chunks: np.ndarray        # u32 [n]
    inter_policy: np.ndarray  # u8  [n]
    intra_policy: np.ndarray  # u8  [n]
    threshold: np.ndarray     # f64 [n]
    max_coll: int = 0
    n_coll: Optional[np.ndarray] = None        # u32 [n]
    coll_size: Optional[np.ndarray] = None     # f64 [max_coll, n]
    release_time: Optional[np.ndarray] = None  # f64 [max_coll, n]
    fixed_delay: Optional[np.ndarray] = None   # f64 [4, n] seconds per stage, or None
    collective_type: Optional[np.ndarray] = None  # u8 [n] COLL_*, or None (All-Reduce)

    @property
    def slots(self) -> int:
        """Chunk slots per scenario in `orders` rows."""
        return self.max_chunks * (self.max_coll if self.n_coll is not None else 1)

    def take(self, idx) -> "ScenarioBatch":
        """Sub-batch of the scenarios in idx (slice or index array)."""
        idx = np.arange(self.n)[idx]
        opt = lambda a: None if a is None else np.ascontiguousarray(a[:, idx])
        return ScenarioBatch(
            n=len(idx), max_chunks=self.max_chunks,
            threshold_mode=self.threshold_mode,
            ndims=self.ndims[idx].copy(),
            npus=np.ascontiguousarray(self.npus[:, idx]),
            bw=np.ascontiguousarray(self.bw[:, idx]),
            size_bytes=self.size_bytes[idx].copy(),
            chunks=self.chunks[idx].copy(),
            inter_policy=self.inter_policy[idx].copy(),
            intra_policy=self.intra_policy[idx].copy(),
            threshold=self.threshold[idx].copy(),
            max_coll=self.max_coll,
            n_coll=None if self.n_coll is None else self.n_coll[idx].copy(),
            coll_size=opt(self.coll_size), release_time=opt(self.release_time),
            fixed_delay=opt(self.fixed_delay),
            collective_type=(None if self.collective_type is None
                             else self.collective_type[idx].copy()))


def make_batch(ndims, npus, bw, size_bytes, chunks, inter_policy, intra_policy,
               threshold, threshold_mode=THR_ABS, max_chunks=None,
               n_coll=None, coll_size=None, release_time=None,
               fixed_delay=None) -> ScenarioBatch:
    """Build a batch from per-scenario sequences; npus/bw are [n][<=4]."""
    ndims = np.asarray(ndims, dtype=np.uint8).reshape(-1)
    n = ndims.shape[0]
    P = np.full((MAX_DIMS, n), 2, dtype=np.uint32)
    B = np.ones((MAX_DIMS, n), dtype=np.float64)
    for i in range(n):
        row_p, row_b = list(npus[i]), list(bw[i])
        for k in range(min(len(row_p), MAX_DIMS)):
            P[k, i] = row_p[k]
        for k in range(min(len(row_b), MAX_DIMS)):
            B[k, i] = row_b[k]
    bc = lambda v, dt: np.ascontiguousarray(
        np.broadcast_to(np.asarray(v, dtype=dt), (n,)))
    chunks = bc(chunks, np.uint32)
    if max_chunks is None:
        max_chunks = int(chunks.max()) if n else 1
    mc = 0
    if n_coll is not None:
        n_coll = bc(n_coll, np.uint32)
        coll_size = np.ascontiguousarray(np.asarray(coll_size, dtype=np.float64))
        mc = coll_size.shape[0]
        if release_time is not None:
            release_time = np.ascontiguousarray(
                np.asarray(release_time, dtype=np.float64))
    return ScenarioBatch(
        n=n, max_chunks=int(max_chunks), threshold_mode=int(threshold_mode),
        ndims=ndims, npus=P, bw=B, size_bytes=bc(size_bytes, np.float64),
        chunks=chunks, inter_policy=bc(inter_policy, np.uint8),
        intra_policy=bc(intra_policy, np.uint8),
        threshold=bc(threshold, np.float64), max_coll=mc, n_coll=n_coll,
        coll_size=coll_size, release_time=release_time,
        fixed_delay=_fixed_rows(fixed_delay, n))


def _fixed_rows(fixed_delay, n):
    """[n][<=4] per-stage delays -> f64 [4, n] (missing dimensions 0)."""
    if fixed_delay is None:
        return None
    F = np.zeros((MAX_DIMS, n))
    for i in range(n):
        row = list(fixed_delay[i])
        F[:len(row), i] = row
    return F


# --------------------------------------------------------------------------
# counter-based random numbers
# --------------------------------------------------------------------------
_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def splitmix64(x: np.ndarray) -> np.ndarray:
    """splitmix64 finaliser of the 64-bit counters x (uint64 array)."""
    with np.errstate(over="ignore"):
        z = (x + np.uint64(0x9E3779B97F4A7C15)) & _M64
        z = ((z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)) & _M64
        z = ((z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)) & _M64
        return z ^ (z >> np.uint64(31))


def _u01(seed: int, i: np.ndarray, k: int, per: int = 16) -> np.ndarray:
    """Uniform [0,1) draw number k of scenario i (53-bit mantissa)."""
    with np.errstate(over="ignore"):
        ctr = (np.uint64(seed) + i.astype(np.uint64) * np.uint64(per)
               + np.uint64(k)) & _M64
    return (splitmix64(ctr) >> np.uint64(11)).astype(np.float64) * (1.0 / 2 ** 53)


def _log_uniform(u, lo, hi):
    return lo * np.exp(u * np.log(hi / lo))


def _const(n, v, dt):
    return np.full(n, v, dtype=dt)


# --------------------------------------------------------------------------
# the five benchmark configurations
# --------------------------------------------------------------------------
def config1() -> ScenarioBatch:
    """One 2-D scenario: ring P=4 at 200 GB/s, switch P=8 at 50 GB/s,
    64 MiB All-Reduce in 4 chunks, Themis + FIFO, threshold 0."""
    return make_batch([2], [[4, 8]], [[200e9, 50e9]], 64 * MIB, 4,
                      INTER_THEMIS, INTRA_FIFO, 0.0, THR_ABS)


def config2(n: int = 65536, seed: int = SEED_BASE + 2, first: int = 0,
            inter: int = INTER_THEMIS) -> ScenarioBatch:
    """3-D, P_k uniform in {2,4,8,16}, B_k log-uniform 25-400 GB/s, S
    log-uniform 1 MiB-1 GiB, C = 64, Themis + FIFO (or baseline)."""
    i = np.arange(first, first + n, dtype=np.uint64)
    P = np.full((MAX_DIMS, n), 2, dtype=np.uint32)
    B = np.ones((MAX_DIMS, n))
    for k in range(3):
        P[k] = (2 << np.minimum((_u01(seed, i, k) * 4).astype(np.int64), 3)
                ).astype(np.uint32)
        B[k] = _log_uniform(_u01(seed, i, 4 + k), 25e9, 400e9)
    S = np.floor(_log_uniform(_u01(seed, i, 8), MIB, GIB))
    return ScenarioBatch(
        n=n, max_chunks=64, threshold_mode=THR_ABS,
        ndims=_const(n, 3, np.uint8), npus=P, bw=B, size_bytes=S,
        chunks=_const(n, 64, np.uint32),
        inter_policy=_const(n, inter, np.uint8),
        intra_policy=_const(n, INTRA_FIFO, np.uint8),
        threshold=np.zeros(n))


def config3(n: int = 1 << 20, seed: int = SEED_BASE + 3,
            first: int = 0) -> ScenarioBatch:
    """4-D P=(2,8,8,64), nominal B=(250,200,100,50) GB/s jittered +/-20 %,
    S log-uniform 1 MiB-4 GiB, C = 64, Themis + SCF, relative threshold
    uniform in [0, 10 %]."""
    i = np.arange(first, first + n, dtype=np.uint64)
    P = np.empty((MAX_DIMS, n), dtype=np.uint32)
    B = np.empty((MAX_DIMS, n))
    for k, (p, b) in enumerate(zip((2, 8, 8, 64), (250e9, 200e9, 100e9, 50e9))):
        P[k] = p
        B[k] = b * (0.8 + 0.4 * _u01(seed, i, k))
    S = np.floor(_log_uniform(_u01(seed, i, 8), MIB, 4 * GIB))
    return ScenarioBatch(
        n=n, max_chunks=64, threshold_mode=THR_REL,
        ndims=_const(n, 4, np.uint8), npus=P, bw=B, size_bytes=S,
        chunks=_const(n, 64, np.uint32),
        inter_policy=_const(n, INTER_THEMIS, np.uint8),
        intra_policy=_const(n, INTRA_SCF, np.uint8),
        threshold=0.10 * _u01(seed, i, 9))


CONFIG4_THRESHOLDS = np.array([0.0, 1 / 64, 1 / 32, 1 / 16, 1 / 8, 1 / 4, 1 / 2, 1.0])


def config4(n: int = 65536, seed: int = SEED_BASE + 4,
            first: int = 0) -> ScenarioBatch:
    """4-D, P_k = 2^U{1..6}, B_k log-uniform 12.5-800 GB/s, S = 1 GiB,
    C = 512; meant for themis_sweep over CONFIG4_THRESHOLDS x {FIFO, SCF}."""
    i = np.arange(first, first + n, dtype=np.uint64)
    P = np.empty((MAX_DIMS, n), dtype=np.uint32)
    B = np.empty((MAX_DIMS, n))
    for k in range(4):
        e = 1 + np.minimum((_u01(seed, i, k) * 6).astype(np.int64), 5)
        P[k] = (1 << e).astype(np.uint32)
        B[k] = _log_uniform(_u01(seed, i, 4 + k), 12.5e9, 800e9)
    return ScenarioBatch(
        n=n, max_chunks=512, threshold_mode=THR_REL,
        ndims=_const(n, 4, np.uint8), npus=P, bw=B,
        size_bytes=_const(n, GIB, np.float64),
        chunks=_const(n, 512, np.uint32),
        inter_policy=_const(n, INTER_THEMIS, np.uint8),
        intra_policy=_const(n, INTRA_SCF, np.uint8),
        threshold=_const(n, 1 / 16, np.float64))


def config5(n: int = 16384, seed: int = SEED_BASE + 5, first: int = 0,
            n_coll: int = 200) -> ScenarioBatch:
    """3-D P=(8,16,32), B_k log-uniform 25-400 GB/s; a trace of n_coll
    All-Reduces with log-normal sizes (median 8 MiB, sigma 1.5, clamped to
    [64 KiB, 4 GiB]) released together at t = 0 and sharing the queues;
    C = 64 each, Themis + SCF, relative threshold 1/16."""
    i = np.arange(first, first + n, dtype=np.uint64)
    P = np.full((MAX_DIMS, n), 2, dtype=np.uint32)
    B = np.ones((MAX_DIMS, n))
    for k, p in enumerate((8, 16, 32)):
        P[k] = p
        B[k] = _log_uniform(_u01(seed, i, k), 25e9, 400e9)
    per = 16 + 2 * n_coll
    sizes = np.empty((n_coll, n))
    for q in range(n_coll):
        u1 = 1.0 - _u01(seed, i, 16 + 2 * q, per)      # (0,1]
        u2 = _u01(seed, i, 17 + 2 * q, per)
        z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)  # Box-Muller
        sizes[q] = np.clip(np.floor(8 * MIB * np.exp(1.5 * z)), 2.0 ** 16, 2.0 ** 32)
    return ScenarioBatch(
        n=n, max_chunks=64, threshold_mode=THR_REL,
        ndims=_const(n, 3, np.uint8), npus=P, bw=B,
        size_bytes=sizes[0].copy(), chunks=_const(n, 64, np.uint32),
        inter_policy=_const(n, INTER_THEMIS, np.uint8),
        intra_policy=_const(n, INTRA_SCF, np.uint8),
        threshold=_const(n, 1 / 16, np.float64),
        max_coll=n_coll, n_coll=_const(n, n_coll, np.uint32),
        coll_size=sizes, release_time=None)


def mixed(n: int, seed: int = SEED_BASE + 99, max_chunks: int = 64,
          pow2: bool = True, thr_mode: int = THR_REL) -> ScenarioBatch:
    """A ragged test batch: D in 1..4, C in 1..max_chunks, both policies, both
    schedulers, every field drawn per scenario.  pow2=False also draws NPU
    counts that are not powers of two."""
    i = np.arange(n, dtype=np.uint64)
    D = (1 + np.minimum((_u01(seed, i, 0) * 4).astype(np.int64), 3)).astype(np.uint8)
    P = np.full((MAX_DIMS, n), 2, dtype=np.uint32)
    B = np.ones((MAX_DIMS, n))
    for k in range(4):
        if pow2:
            e = 1 + np.minimum((_u01(seed, i, 1 + k) * 6).astype(np.int64), 5)
            P[k] = (1 << e).astype(np.uint32)
        else:
            P[k] = (2 + np.minimum((_u01(seed, i, 1 + k) * 23).astype(np.int64), 22)
                    ).astype(np.uint32)
        B[k] = _log_uniform(_u01(seed, i, 5 + k), 12.5e9, 800e9)
    S = np.floor(_log_uniform(_u01(seed, i, 9), MIB, 4 * GIB))
    C = (1 + np.minimum((_u01(seed, i, 10) * max_chunks).astype(np.int64),
                        max_chunks - 1)).astype(np.uint32)
    inter = (_u01(seed, i, 11) < 0.8).astype(np.uint8)
    intra = (_u01(seed, i, 12) < 0.5).astype(np.uint8)
    thr = _u01(seed, i, 13) * (0.25 if thr_mode == THR_REL else 1e-4)
    thr[_u01(seed, i, 14) < 0.3] = 0.0
    return ScenarioBatch(
        n=n, max_chunks=max_chunks, threshold_mode=thr_mode, ndims=D, npus=P,
        bw=B, size_bytes=S, chunks=C, inter_policy=inter, intra_policy=intra,
        threshold=thr)


def dyadic_ties(n: int, seed: int = SEED_BASE + 77, max_chunks: int = 64,
                tilt: bool = True) -> ScenarioBatch:
    """Networks on which many stages end at the very same binary64 instant:
    power-of-two NPU counts, bandwidths 2^a * (P-1)/P (so every per-byte latency
    is a power of two), chunks of 2^m bytes.  The exponents follow the paper's
    just-enough ladder (Sec. 3.3 / 6.3: BW(dim1) = P1 * BW(dim2) = ..., which
    makes the baseline's stage times equal on all dimensions), optionally
    tilted by a factor of two per dimension.  All stage times are then powers
    of two and every clock value an exact sum of them, so completions on
    different dimensions coincide again and again.  D in 1..4, both schedulers
    and queue policies, relative thresholds 0, 1/16 or 1/4 (which also make the
    threshold test of Alg. 1 hit exact equality)."""
    i = np.arange(n, dtype=np.uint64)
    D = (1 + np.minimum((_u01(seed, i, 0) * 5).astype(np.int64), 3)).astype(np.uint8)  # 4 twice as often
    P = np.full((MAX_DIMS, n), 2, dtype=np.uint32)
    B = np.ones((MAX_DIMS, n))
    a = 33.0 + np.floor(_u01(seed, i, 13) * 3)        # log2 of dim1's scaled bandwidth
    for k in range(4):
        e = 1 + np.minimum((_u01(seed, i, 1 + k) * 3).astype(np.int64), 2)   # P in {2, 4, 8}
        P[k] = (1 << e).astype(np.uint32)
        t = np.floor(_u01(seed, i, 5 + k) * 3) - 1 if tilt else 0.0
        p = P[k].astype(np.float64)
        B[k] = 2.0 ** (a + (t if k else 0.0)) * ((p - 1.0) / p)
        a = a - e                                      # the next rung of the ladder
    C = (1 + np.minimum((_u01(seed, i, 10) * max_chunks).astype(np.int64),
                        max_chunks - 1)).astype(np.uint32)
    C[_u01(seed, i, 14) < 0.4] = max_chunks            # many at the layout's capacity
    S = C.astype(np.float64) * 2.0 ** (20 + np.floor(_u01(seed, i, 9) * 5))
    inter = (_u01(seed, i, 11) < 0.8).astype(np.uint8)
    intra = (_u01(seed, i, 12) < 0.5).astype(np.uint8)
    thr = np.choose((_u01(seed, i, 15) * 3).astype(np.int64), [0.0, 1 / 16, 1 / 4])
    return ScenarioBatch(
        n=n, max_chunks=max_chunks, threshold_mode=THR_REL, ndims=D, npus=P,
        bw=B, size_bytes=S, chunks=C, inter_policy=inter, intra_policy=intra,
        threshold=thr)


# --------------------------------------------------------------------------
# the six 1024-NPU platforms of the paper's Table 2
# --------------------------------------------------------------------------
# name, sizes, per-dimension topology, aggregate bandwidth per NPU (Gb/s),
# step latency (ns).  R = ring, F = fully connected, S = switch.
TABLE2 = (
    ("2D-SW_SW", (16, 64), "SS", (1200, 800), (700, 1700)),
    ("3D-SW_SW_SW_homo", (16, 8, 8), "SSS", (800, 800, 800), (700, 700, 1700)),
    ("3D-SW_SW_SW_hetero", (16, 8, 8), "SSS", (1600, 800, 400), (700, 700, 1700)),
    ("3D-FC_Ring_SW", (8, 16, 8), "FRS", (1400, 800, 400), (700, 700, 1700)),
    ("4D-Ring_SW_SW_SW", (4, 4, 8, 8), "RSSS", (2000, 1600, 800, 400), (20, 700, 700, 1700)),
    ("4D-Ring_FC_Ring_SW", (4, 8, 4, 8), "RFRS", (3000, 1400, 1200, 800), (20, 700, 700, 1700)),
)


def stage_steps(topology: str, p: int) -> int:
    """Steps of one Reduce-Scatter (or All-Gather) stage of the topology-aware
    algorithm of the paper's Table 1: ring P-1 (so a ring All-Reduce takes
    2P-2, Sec. 4.5), direct on a fully connected dimension 1, halving-doubling
    on a switch log2 P."""
    if topology == "R":
        return p - 1
    if topology == "F":
        return 1
    if topology == "S":
        return int(p).bit_length() - 1
    raise ValueError(topology)


def table2(sizes_bytes=(100e6, 250e6, 500e6, 1000e6), chunks=64, inter=INTER_THEMIS,
           intra=INTRA_SCF, threshold=1 / 16, with_latency=True) -> ScenarioBatch:
    """One scenario per (Table 2 topology, All-Reduce size); fixed per-stage
    delay = steps x step latency when with_latency."""
    rows = [(t, s) for t in TABLE2 for s in sizes_bytes]
    fixed = None
    if with_latency:
        fixed = [[stage_steps(k, p) * lat * 1e-9 for k, p, lat in zip(t[2], t[1], t[4])]
                 for t, _ in rows]
    return make_batch(
        [len(t[1]) for t, _ in rows], [t[1] for t, _ in rows],
        [[g * 1e9 / 8 for g in t[3]] for t, _ in rows], [s for _, s in rows], chunks,
        inter, intra, threshold, THR_REL, fixed_delay=fixed)
