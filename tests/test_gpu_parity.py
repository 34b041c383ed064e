"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle
on the same seeded inputs.

Bar: order codes and per-dimension queue orders bit-exact; completion times,
loads and busy times within 1e-12 relative (binary64, the tolerance the
target states).
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

REL_TOL = 1e-12


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: the gpu-marked tests need an MI355X")
    from paper_2110_04478_amd import binding
    from paper_2110_04478_amd.csrc.build import ensure_built
    ensure_built()          # compiles only when no library is in the tree
    binding.lib()
    return binding


def w():
    from paper_2110_04478_amd import workloads
    return workloads


def assert_close(name, got, want):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    assert got.shape == want.shape, name
    nan_g, nan_w = np.isnan(got), np.isnan(want)
    assert np.array_equal(nan_g, nan_w), f"{name}: NaN pattern differs"
    g, x = got[~nan_g], want[~nan_w]
    with np.errstate(invalid="ignore"):   # equal infinities
        err = np.abs(g - x) / np.maximum(np.abs(x), np.finfo(np.float64).tiny)
    err[(g == x)] = 0.0
    assert err.size == 0 or err.max() <= REL_TOL, (
        f"{name}: max rel err {err.max():.3e} at {int(err.argmax())}, "
        f"{int((g != x).sum())} of {g.size} differ")


def widen_queue(q):
    q = q.cpu().numpy()
    if q.dtype == np.uint8:
        out = q.astype(np.uint16)
        out[q == 0xFF] = 0xFFFF
        return out
    return q.astype(np.uint16)


def run_gpu(gpu, batch, queue=True, workspace=True):
    import torch
    d = gpu.to_device(batch)
    orders, loads = gpu.themis_plan_batch(d)
    ws = gpu.alloc_workspace(gpu.themis_workspace_bytes(
        d.n, d.max_chunks, d.max_coll if d.n_coll is not None else 0)) if workspace else None
    t, qo, busy = gpu.themis_simulate_batch(d, orders, workspace=ws, want_queue_order=queue)
    torch.cuda.synchronize()
    return (orders.cpu().numpy(), loads.cpu().numpy(), t.cpu().numpy(),
            widen_queue(qo) if queue else None, busy.cpu().numpy())


def check_batch(gpu, oracle, batch, queue=True, threads=8, workspace=True):
    o_orders, o_loads = oracle.plan_batch(batch, threads=threads)
    o_t, o_qo, o_busy = oracle.simulate_batch(batch, o_orders, want_queue_order=queue,
                                              threads=threads)
    g_orders, g_loads, g_t, g_qo, g_busy = run_gpu(gpu, batch, queue, workspace)
    bad = np.nonzero((g_orders != o_orders).any(axis=1))[0]
    assert bad.size == 0, f"order codes differ in {bad.size} scenarios, first {bad[:5]}"
    assert_close("loads", g_loads, o_loads)
    if queue:
        badq = np.nonzero((g_qo != o_qo).reshape(batch.n, -1).any(axis=1))[0]
        assert badq.size == 0, f"queue orders differ in {badq.size} scenarios, first {badq[:5]}"
    assert_close("t_done", g_t, o_t)
    assert_close("busy", g_busy, o_busy)
    return g_t


def test_config1_single_scenario(gpu, oracle):
    t = check_batch(gpu, oracle, w().config1())
    assert t[0] == pytest.approx(713.03168e-6, rel=1e-9)


@pytest.mark.parametrize("inter", [1, 0])
def test_config2_shape(gpu, oracle, inter):
    check_batch(gpu, oracle, w().config2(n=4096 + 37, inter=inter))


def test_config3_shape(gpu, oracle):
    check_batch(gpu, oracle, w().config3(n=8192 + 5))


@pytest.mark.parametrize("n", [1, 63, 64, 65, 1000])
@pytest.mark.parametrize("thr_mode", [0, 1])
def test_ragged_mixed_batches(gpu, oracle, n, thr_mode):
    """D in 1..4, C in 1..64, both schedulers, both queue policies; batch
    sizes around the 64-lane wavefront boundary."""
    check_batch(gpu, oracle, w().mixed(n, seed=1234 + n, thr_mode=thr_mode))


@pytest.mark.parametrize("max_chunks", [8, 22, 64, 126])
@pytest.mark.parametrize("offset", [0, 1, 4, 8])
def test_queue_orders_at_any_address(gpu, oracle, max_chunks, offset):
    """The queue-order array may start at any byte: rows of whole wavefronts are
    put in place sixteen bytes at a time only where the address and the row
    length allow it, four or one at a time otherwise. 64 * 9 + 11 scenarios:
    whole wavefronts and a ragged last one; NPU counts that are not powers of
    two leave some scenarios of a wavefront to the second kernel."""
    import torch
    b = w().mixed(64 * 9 + 11, seed=77 + max_chunks, max_chunks=max_chunks, pow2=False)
    keep = np.arange(b.n) % 3 == 0          # two of three scenarios get powers of two
    b.npus = np.where(keep[None, :], b.npus,
                      1 << np.floor(np.log2(b.npus)).astype(np.int64)).astype(np.uint32)
    _with_collective_types(b, 5)
    o_orders, _ = oracle.plan_batch(b, threads=8)
    o_t, o_qo, _ = oracle.simulate_batch(b, o_orders, threads=8)
    d = gpu.to_device(b)
    orders, _ = gpu.themis_plan_batch(d)
    assert gpu.themis_queue_entry_bytes(max_chunks) == 1
    row = 4 * 2 * d.slots
    raw = torch.full((b.n * row + 64,), 0x5A, dtype=torch.uint8, device="cuda")
    qo = raw[offset:offset + b.n * row].view(b.n, 4, 2 * d.slots)
    ws = gpu.alloc_workspace(gpu.themis_workspace_bytes(d.n, d.max_chunks))
    t, _, _ = gpu.themis_simulate_batch(d, orders, queue_order=qo, workspace=ws)
    torch.cuda.synchronize()
    assert_close("t_done", t.cpu().numpy(), o_t)
    assert np.array_equal(widen_queue(qo), o_qo)
    host = raw.cpu().numpy()   # nothing outside the array was touched
    assert (host[:offset] == 0x5A).all() and (host[offset + b.n * row:] == 0x5A).all()


@pytest.mark.parametrize("max_chunks", [1, 7, 16, 17])
def test_small_chunk_counts(gpu, oracle, max_chunks):
    """C up to 16 runs on the 48-dword LDS layout (13 wavefronts per CU); 17 is
    the first size back on the 64-chunk layout; odd row lengths store queue
    entries bytewise."""
    b = w().mixed(900, seed=40 + max_chunks, max_chunks=max_chunks)
    check_batch(gpu, oracle, b)
    import torch
    thr = torch.tensor([0.0, 1 / 16, 1.0], dtype=torch.float64, device="cuda")
    want = oracle.sweep(b, thr.cpu().numpy(), 7, threads=8)
    d = gpu.to_device(b)
    ws = gpu.alloc_workspace(gpu.themis_workspace_bytes(d.n * 3 * 3, d.max_chunks))
    got = gpu.themis_sweep(d, thr, 7, workspace=ws)
    torch.cuda.synchronize()
    assert_close("sweep", got.cpu().numpy(), want)


def test_non_power_of_two_npus(gpu, oracle):
    check_batch(gpu, oracle, w().mixed(700, seed=77, pow2=False))


@pytest.mark.parametrize("ctype", [0, 1, 2])
def test_three_dimensional_networks_with_arbitrary_npu_counts(gpu, oracle, ctype):
    """NPU counts such as 3, 6, 12, 24, 72: resident sizes depend on the order
    of the divisions.  With at most 8 distinct order codes per scenario (always
    the case up to three dimensions) the LDS event loop runs on per-order-code
    tables; sizes that divide evenly make many equal Smallest-Chunk-First keys."""
    import torch
    W = w()
    n = 3000
    rng = np.random.default_rng(31 + ctype)
    b = W.config2(n=n)
    b.npus = np.ascontiguousarray(rng.choice([3, 6, 12, 24, 72, 5, 8], (4, n)).astype(np.uint32))
    b.ndims = rng.integers(1, 4, n).astype(np.uint8)
    b.intra_policy = rng.integers(0, 2, n).astype(np.uint8)
    b.size_bytes = np.where(rng.random(n) < 0.5, 2.0 ** rng.integers(24, 31, n) * 9.0, b.size_bytes)
    b.bw = np.ascontiguousarray(np.where(rng.random((4, n)) < 0.5,
                                         2.0 ** rng.integers(33, 37, (4, n)), b.bw))
    b.chunks = rng.choice([1, 7, 32, 64], n).astype(np.uint32)
    b.collective_type = np.full(n, ctype, np.uint8)
    if ctype:
        b.fixed_delay = np.ascontiguousarray(rng.uniform(0, 2e-6, (4, n)))
    check_batch(gpu, oracle, b, threads=16)
    thr = torch.tensor([0.0, 1 / 16], dtype=torch.float64, device="cuda")
    if ctype == 0:
        got = gpu.themis_sweep(gpu.to_device(b), thr, 7)
        torch.cuda.synchronize()
        assert_close("sweep", got.cpu().numpy(), oracle.sweep(b, thr.cpu().numpy(), 7, threads=16))


@pytest.mark.parametrize("max_chunks", [64, 100, 128])
def test_four_dimensional_networks_with_arbitrary_npu_counts(gpu, oracle, max_chunks):
    """4-D networks with NPU counts like 3, 6, 10, 48, 72: Themis plans use well
    over 8 distinct orders, random plans all 24 -- the variant with 64 size
    classes per dimension (up to 128 chunks; 8- and 16-bit queue entries).
    Evenly dividing sizes give equal keys.  No workspace is passed: nothing
    may be left to the generic scan."""
    import torch
    W = w()
    n = 1500 if max_chunks == 64 else 600
    rng = np.random.default_rng(57 + max_chunks)
    b = W.config3(n=n)
    b.max_chunks = max_chunks
    b.npus = np.ascontiguousarray(rng.choice([3, 6, 10, 12, 48, 72, 5, 4], (4, n)).astype(np.uint32))
    b.intra_policy = rng.integers(0, 2, n).astype(np.uint8)
    b.size_bytes = np.where(rng.random(n) < 0.5, 2.0 ** rng.integers(24, 31, n) * 45.0, b.size_bytes)
    b.bw = np.ascontiguousarray(np.where(rng.random((4, n)) < 0.5,
                                         2.0 ** rng.integers(33, 37, (4, n)), b.bw))
    b.chunks = rng.choice([5, 24, max_chunks - 1, max_chunks], n).astype(np.uint32)
    b.collective_type = rng.integers(0, 3, n).astype(np.uint8)
    b.fixed_delay = np.ascontiguousarray(rng.uniform(0, 2e-6, (4, n)) * (rng.random((4, n)) < 0.5))
    check_batch(gpu, oracle, b, threads=16, workspace=False)
    # arbitrary (not planned) orders: all 24 permutations in one scenario
    orders = np.full((n, b.max_chunks), 0xFF, np.uint8)
    perms = [sum(int(k) << (2 * j) for j, k in enumerate(p))
             for p in __import__("itertools").permutations(range(4))]
    for i in range(n):
        orders[i, :b.chunks[i]] = rng.choice(perms, int(b.chunks[i]))
    o_t, o_qo, o_busy = oracle.simulate_batch(b, orders, threads=16)
    d = gpu.to_device(b)
    t, qo, busy = gpu.themis_simulate_batch(d, torch.from_numpy(orders).cuda())
    torch.cuda.synchronize()
    assert_close("t_done", t.cpu().numpy(), o_t)
    assert np.array_equal(widen_queue(qo), o_qo)
    assert_close("busy", busy.cpu().numpy(), o_busy)
    b.collective_type = None
    thr = torch.tensor([0.0, 1 / 16], dtype=torch.float64, device="cuda")
    got = gpu.themis_sweep(gpu.to_device(b), thr, 7)
    torch.cuda.synchronize()
    assert_close("sweep", got.cpu().numpy(), oracle.sweep(b, thr.cpu().numpy(), 7, threads=16))


def test_single_collectives_run_without_a_workspace(gpu, oracle):
    """Single collectives of any chunk count run in LDS without a workspace,
    whatever the NPU counts (up to 64 chunks even the generic scan keeps its
    per-chunk arrays in LDS).  Only what no LDS path takes beyond 64 chunks
    (here: stage times too short to move the clock) needs the workspace and
    comes back as NaN / all-ones without it, next to unaffected scenarios."""
    import torch
    for mc in (9, 64, 100, 128, 200, 300, 512):
        b = w().mixed(500 if mc <= 128 else 150, seed=300 + mc, max_chunks=mc, pow2=False)
        o_orders, _ = oracle.plan_batch(b, threads=8)
        o_t, o_qo, o_busy = oracle.simulate_batch(b, o_orders, threads=8)
        d = gpu.to_device(b)
        orders, _ = gpu.themis_plan_batch(d)
        t, qo, busy = gpu.themis_simulate_batch(d, orders)          # no workspace
        thr = torch.tensor([0.0, 0.125], dtype=torch.float64, device="cuda")
        sw = gpu.themis_sweep(d, thr, 6)                            # no workspace
        torch.cuda.synchronize()
        assert not np.isnan(o_t).any()
        assert_close("t_done", t.cpu().numpy(), o_t)
        assert np.array_equal(widen_queue(qo), o_qo)
        assert_close("busy", busy.cpu().numpy(), o_busy)
        assert_close("sweep", sw.cpu().numpy(), oracle.sweep(b, thr.cpu().numpy(), 6, threads=8))
    W = w()
    P = [[4, 4], [4, 4], [4, 8]]
    bw = [[1e3, 1e300], [1e300, 1e3], [200e9, 50e9]]
    reps = 10
    b = W.make_batch([2, 2, 2] * reps, P * reps, bw * reps, 2.0 ** 30, [100, 70, 90] * reps, 1,
                     [1, 0, 1] * reps, 0.0, max_chunks=100)
    o_orders, _ = oracle.plan_batch(b, threads=8)
    o_t, _, _ = oracle.simulate_batch(b, o_orders, want_queue_order=False, threads=8)
    ordinary = np.arange(b.n) % 3 == 2
    d = gpu.to_device(b)
    orders, _ = gpu.themis_plan_batch(d)
    t, qo, _ = gpu.themis_simulate_batch(d, orders)                 # no workspace
    torch.cuda.synchronize()
    t = t.cpu().numpy()
    assert np.isfinite(o_t).all()
    assert np.isnan(t[~ordinary]).all() and (qo.cpu().numpy()[~ordinary] == 0xFF).all()
    assert_close("t_done of the LDS-path scenarios", t[ordinary], o_t[ordinary])
    check_batch(gpu, oracle, b)                                     # with a workspace


def test_large_chunk_counts(gpu, oracle):
    """C up to 512: the wide LDS layouts, 8- and 16-bit queue entries, odd
    row lengths."""
    check_batch(gpu, oracle, w().mixed(96, seed=5, max_chunks=512), threads=8)
    check_batch(gpu, oracle, w().config4(n=70))
    check_batch(gpu, oracle, w().mixed(200, seed=6, max_chunks=100))
    check_batch(gpu, oracle, w().mixed(200, seed=7, max_chunks=128))
    check_batch(gpu, oracle, w().mixed(200, seed=8, max_chunks=127))
    check_batch(gpu, oracle, w().mixed(200, seed=9, max_chunks=63))
    check_batch(gpu, oracle, w().mixed(130, seed=10, max_chunks=256))   # 320-dword layout
    check_batch(gpu, oracle, w().mixed(130, seed=11, max_chunks=129))
    check_batch(gpu, oracle, w().mixed(100, seed=12, max_chunks=257))   # first size on the 576-dword one


def test_empty_batch(gpu):
    import torch
    b = w().mixed(0)
    d = gpu.to_device(b)
    orders, loads = gpu.themis_plan_batch(d)
    t, qo, busy = gpu.themis_simulate_batch(d, orders)
    torch.cuda.synchronize()
    assert orders.shape[0] == 0 and t.shape[0] == 0


def test_invalid_scenarios_come_back_as_nan(gpu, oracle):
    b = w().mixed(256, seed=9)
    b.npus[1, 3] = 1             # P < 2 (only matters if D > 1)
    b.ndims[3] = 3
    b.bw[0, 10] = float("nan")
    b.bw[0, 11] = 0.0
    b.bw[0, 12] = float("inf")
    b.size_bytes[20] = -5.0
    b.chunks[30] = 0
    b.chunks[31] = b.max_chunks + 1
    b.ndims[40] = 0
    b.ndims[41] = 5
    b.threshold[50] = -1.0
    b.threshold[51] = float("nan")
    t = check_batch(gpu, oracle, b)
    for i in (3, 10, 11, 12, 20, 30, 31, 40, 41):
        assert np.isnan(t[i])
    assert np.isfinite(t[0])


def test_arbitrary_orders_are_accepted_and_malformed_ones_rejected(gpu, oracle):
    """themis_simulate_batch takes any valid permutation per chunk."""
    import torch
    b = w().mixed(300, seed=21)
    rng = np.random.default_rng(3)
    orders = np.full((b.n, b.slots), 0xFF, np.uint8)
    for i in range(b.n):
        D = int(b.ndims[i])
        for c in range(int(b.chunks[i])):
            perm = rng.permutation(D)
            orders[i, c] = sum(int(k) << (2 * j) for j, k in enumerate(perm))
    orders[7, 0] = 0xFF                      # malformed
    orders[8, 0] = 0x00 if b.ndims[8] > 1 else 0x01
    o_t, o_qo, o_busy = oracle.simulate_batch(b, orders, threads=8)
    d = gpu.to_device(b)
    ws = gpu.alloc_workspace(gpu.themis_workspace_bytes(d.n, d.max_chunks, 0))
    t, qo, busy = gpu.themis_simulate_batch(d, torch.from_numpy(orders).cuda(), workspace=ws)
    torch.cuda.synchronize()
    assert np.isnan(o_t[7]) and np.isnan(o_t[8])
    assert_close("t_done", t.cpu().numpy(), o_t)
    assert np.array_equal(widen_queue(qo), o_qo)
    assert_close("busy", busy.cpu().numpy(), o_busy)


@pytest.mark.gpu
@pytest.mark.parametrize("max_chunks", [200, 257, 512])
def test_arbitrary_orders_with_hundreds_of_chunks(gpu, oracle, max_chunks):
    """Any permutation per chunk, all three collective types and both queue
    policies on the LDS layouts for more than 128 chunks (16-bit queue
    entries), where a chunk's state is derived from its order, not stored."""
    import torch
    b = _with_collective_types(w().mixed(140, seed=300 + max_chunks, max_chunks=max_chunks), 31)
    b.chunks[:4] = [max_chunks, max_chunks - 1, 1, 2]
    rng = np.random.default_rng(max_chunks)
    orders = np.full((b.n, b.slots), 0xFF, np.uint8)
    for i in range(b.n):
        D = int(b.ndims[i])
        perms = np.argsort(rng.random((int(b.chunks[i]), D)), axis=1)
        orders[i, :perms.shape[0]] = (perms << (2 * np.arange(D))).sum(axis=1)
    o_t, o_qo, o_busy = oracle.simulate_batch(b, orders, threads=8)
    d = gpu.to_device(b)
    t, qo, busy = gpu.themis_simulate_batch(d, torch.from_numpy(orders).cuda())
    torch.cuda.synchronize()
    assert np.isfinite(o_t).all()
    assert_close("t_done", t.cpu().numpy(), o_t)
    assert np.array_equal(widen_queue(qo), o_qo)
    assert_close("busy", busy.cpu().numpy(), o_busy)


def test_trace_of_collectives_sharing_queues(gpu, oracle):
    b = w().config5(n=96, n_coll=6)
    check_batch(gpu, oracle, b)
    # staggered releases and ragged collective counts
    rng = np.random.default_rng(11)
    b = w().config5(n=70, n_coll=5)
    b.release_time = np.ascontiguousarray(rng.integers(0, 6, b.coll_size.shape) * 1e-4)
    b.n_coll = rng.integers(1, 6, b.n).astype(np.uint32)
    check_batch(gpu, oracle, b)


def _add_trace(b, rng, max_coll, pow2_sizes):
    """Turn a single-collective batch into a trace batch (in place)."""
    b.max_coll = max_coll
    b.n_coll = rng.integers(1, max_coll + 1, b.n).astype(np.uint32)
    if pow2_sizes:  # sizes a power of two apart: equal resident sizes across collectives
        base = b.size_bytes[None, :]
        b.coll_size = np.ascontiguousarray(base * 2.0 ** rng.integers(-3, 4, (max_coll, b.n)))
    else:
        b.coll_size = np.ascontiguousarray(np.floor(rng.uniform(2 ** 16, 2 ** 28, (max_coll, b.n))))
    b.release_time = None
    return b


def test_traces_ranked_list_path(gpu, oracle):
    """Traces released at t = 0 with power-of-two NPU counts take the ranked
    list path: ragged D, C, collective counts, both policies, equal resident
    sizes across collectives, and more collectives than the small tests."""
    rng = np.random.default_rng(5)
    b = _add_trace(w().mixed(200, seed=41, max_chunks=12), rng, 9, pow2_sizes=True)
    check_batch(gpu, oracle, b)
    b = _add_trace(w().mixed(130, seed=42, max_chunks=8), rng, 20, pow2_sizes=False)
    check_batch(gpu, oracle, b)
    b = w().config5(n=64, n_coll=24)
    b.intra_policy[::2] = 0           # half FIFO
    check_batch(gpu, oracle, b)
    # NPU counts that are not powers of two: the same path in division mode
    b = _add_trace(w().mixed(100, seed=43, max_chunks=8, pow2=False), rng, 5, pow2_sizes=False)
    check_batch(gpu, oracle, b)
    # the largest trace the ranked lists take (256 collectives) and one beyond it (generic path)
    b = _add_trace(w().mixed(40, seed=45, max_chunks=4), rng, 256, pow2_sizes=False)
    b.n_coll[:20] = 256
    check_batch(gpu, oracle, b, threads=16)
    b = _add_trace(w().mixed(12, seed=46, max_chunks=3), rng, 300, pow2_sizes=True)
    b.n_coll[:6] = 300
    check_batch(gpu, oracle, b, threads=16)
    # more wavefronts than CUs: the variant that keeps its bitmaps in the workspace
    b = _add_trace(w().mixed(256 * 64 + 700, seed=44, max_chunks=5), rng, 3, pow2_sizes=True)
    check_batch(gpu, oracle, b, threads=16)


def test_traces_on_networks_with_other_npu_counts(gpu, oracle):
    """NPU counts that are not powers of two in traces: the ranked-list loop
    takes them too, every stage time by the order's own divisions (and, for a
    stand-alone All-Gather, multiplications), one at a time as the latency model
    walks them, and under Smallest-Chunk-First with one size rank per
    (dimension, phase, order) of every collective.  Ragged D, C and collective
    counts, both policies, all collective types, with and without release times,
    fixed delays and queue orders; a trace with too many collectives for the
    ranks of a 4-D network goes to the generic path."""
    rng = np.random.default_rng(15)
    for seed, mc, ncoll in ((61, 8, 5), (62, 12, 9), (63, 64, 4)):
        b = _add_trace(w().mixed(160, seed=seed, max_chunks=mc, pow2=False), rng, ncoll, pow2_sizes=False)
        b.intra_policy[::2] = 0                   # half first-in-first-out
        check_batch(gpu, oracle, _with_collective_types(b, seed))
        check_batch(gpu, oracle, b, queue=False)
        b.release_time = np.ascontiguousarray(rng.integers(0, 5, b.coll_size.shape) * 2e-4)
        check_batch(gpu, oracle, _with_fixed_delay(b, seed + 1))
    # the config-5 shape on P = (6, 12, 24), both policies
    b = w().config5(n=80, n_coll=12)
    b.npus = np.ascontiguousarray(np.array([[6], [12], [24], [1]], dtype=np.uint32).repeat(b.n, axis=1))
    b.intra_policy[::2] = 0
    check_batch(gpu, oracle, b)
    # 4-D, 100 collectives: 100 x 48 ranks per dimension do not fit the lists (generic path), 80 do
    for ncoll in (100, 80):
        b = _add_trace(w().mixed(12, seed=64, max_chunks=4, pow2=False), rng, ncoll, pow2_sizes=False)
        b.ndims[:] = 4
        b.n_coll[:] = ncoll
        b.intra_policy[:] = 1
        check_batch(gpu, oracle, b, threads=16)


def test_traces_without_queue_orders(gpu, oracle):
    """Traces with neither release times, fixed delays nor queue orders asked
    for run a kernel compiled without those steps: times and busy times against
    the oracle, with the bitmaps in LDS and (more wavefronts than CUs) in the
    workspace."""
    rng = np.random.default_rng(6)
    b = _add_trace(w().mixed(300, seed=51, max_chunks=12), rng, 9, pow2_sizes=True)
    check_batch(gpu, oracle, _with_collective_types(b, 4), queue=False)
    b = _add_trace(w().mixed(150, seed=52, max_chunks=64), rng, 6, pow2_sizes=False)
    check_batch(gpu, oracle, b, queue=False)
    b = _add_trace(w().mixed(256 * 64 + 300, seed=53, max_chunks=5), rng, 3, pow2_sizes=True)
    check_batch(gpu, oracle, b, queue=False, threads=16)


def test_traces_with_staggered_releases(gpu, oracle):
    """Collectives released at different times (gradients of a back-propagation
    pass) on the ranked-list path: releases before, between and after the
    completions, several collectives per release instant, idle gaps, and a
    release that falls exactly on a completion (arrivals of both kinds at one
    instant are ordered by chunk id)."""
    rng = np.random.default_rng(77)
    # release instants on a coarse grid: many collectives share one
    b = _add_trace(w().mixed(300, seed=81, max_chunks=10), rng, 12, pow2_sizes=True)
    b.release_time = np.ascontiguousarray(rng.integers(0, 5, b.coll_size.shape) * 2e-4)
    check_batch(gpu, oracle, b)
    # continuous release times, long gaps (the queues drain in between), all three collective types
    b = _with_collective_types(_add_trace(w().mixed(300, seed=82, max_chunks=8), rng, 25, pow2_sizes=False), 83)
    b.release_time = np.ascontiguousarray(rng.uniform(0, 1, b.coll_size.shape) ** 4 * 5e-2)
    check_batch(gpu, oracle, b)
    # nothing released at t = 0, fixed delays
    b = _with_fixed_delay(w().config5(n=70, n_coll=9), 84)
    b.release_time = np.ascontiguousarray(rng.uniform(1e-5, 3e-3, b.coll_size.shape))
    b.intra_policy[::3] = 0
    check_batch(gpu, oracle, b)
    # exact coincidence: one dimension of two NPUs at 2^30 B/s, chunks of 2^20 bytes:
    # every stage takes 2^-11 s, and the second collective is released at 3 * 2^-11 s
    b = _add_trace(w().mixed(64, seed=85, max_chunks=4), rng, 3, pow2_sizes=True)
    b.release_time = np.zeros_like(b.coll_size)
    for i in range(0, 64, 2):
        b.ndims[i] = 1
        b.npus[0, i] = 2
        b.bw[0, i] = 2.0 ** 30
        b.chunks[i] = 4
        b.n_coll[i] = 3
        b.coll_size[:, i] = 4 * 2.0 ** 20
        b.release_time[:, i] = [0.0, 3 * 2.0 ** -11, 5 * 2.0 ** -11]
    t = check_batch(gpu, oracle, b)
    assert np.isfinite(t).all()


def test_trace_with_generic_only_workspace(gpu, oracle):
    """A workspace that only covers the generic area still gives exact results."""
    import torch
    b = w().config5(n=70, n_coll=4)
    d = gpu.to_device(b)
    orders, _ = gpu.themis_plan_batch(d)
    ws = gpu.alloc_workspace(d.n * d.slots * 20)
    t, qo, busy = gpu.themis_simulate_batch(d, orders, workspace=ws)
    torch.cuda.synchronize()
    o_orders, _ = oracle.plan_batch(b, threads=8)
    o_t, o_qo, o_busy = oracle.simulate_batch(b, o_orders, threads=8)
    assert_close("t_done", t.cpu().numpy(), o_t)
    assert np.array_equal(widen_queue(qo), o_qo)


def test_sweep_matches_oracle(gpu, oracle):
    import torch
    W = w()
    for b, thr, mask in (
            (W.config2(n=600), np.array([0.0]), W.SWEEP_BASELINE | W.SWEEP_THEMIS_FIFO),
            (W.config4(n=40), W.CONFIG4_THRESHOLDS, W.SWEEP_THEMIS_FIFO | W.SWEEP_THEMIS_SCF),
            (W.mixed(500, seed=31), np.array([0.0, 1 / 16, 0.5]), 7)):
        want = oracle.sweep(b, thr, mask, threads=8)
        d = gpu.to_device(b)
        n_pol = bin(mask).count("1")
        ws = gpu.alloc_workspace(gpu.themis_workspace_bytes(d.n * len(thr) * n_pol, d.max_chunks))
        got = gpu.themis_sweep(d, torch.from_numpy(thr).cuda(), mask, workspace=ws)
        torch.cuda.synchronize()
        assert_close("sweep t_done", got.cpu().numpy(), want)
    # per-scenario thresholds
    b = W.mixed(300, seed=32)
    thr = np.ascontiguousarray(np.random.default_rng(1).uniform(0, 0.3, (3, b.n)))
    want = oracle.sweep(b, thr, 6, thr_per_scenario=True, threads=8)
    d = gpu.to_device(b)
    ws = gpu.alloc_workspace(gpu.themis_workspace_bytes(d.n * 3 * 2, d.max_chunks))
    got = gpu.themis_sweep(d, torch.from_numpy(thr).cuda(), 6, thr_per_scenario=True, workspace=ws)
    torch.cuda.synchronize()
    assert_close("sweep t_done (per-scenario thr)", got.cpu().numpy(), want)
    # The baseline column is the same under every threshold (Alg. 1 looks at the
    # threshold only when Themis is on) and NaN exactly where the threshold
    # itself is not valid, whatever the first threshold is.
    for b in (W.config3(n=200), W.mixed(333, seed=33, max_chunks=512, pow2=False)):
        n = b.n
        for thr, per_scenario in ((np.array([1 / 16, -1.0, 0.5, float("nan")]), False),
                                  (np.array([-1.0, 0.25]), False),
                                  (np.where(np.random.default_rng(2).random((3, n)) < 0.3, -1.0, 0.1), True)):
            thr = np.ascontiguousarray(thr, dtype=np.float64)
            want = oracle.sweep(b, thr, 7, thr_per_scenario=per_scenario, threads=8)
            d = gpu.to_device(b)
            ws = gpu.alloc_workspace(gpu.themis_workspace_bytes(d.n * len(thr) * 3, d.max_chunks))
            got = gpu.themis_sweep(d, torch.from_numpy(thr).cuda(), 7,
                                   thr_per_scenario=per_scenario, workspace=ws)
            torch.cuda.synchronize()
            got = got.cpu().numpy()
            assert_close("sweep with thresholds that are not valid", got, want)
            base = got[:, :, 0]
            ok = ~np.isnan(base)
            first = np.where(ok.any(axis=1), base[np.arange(n), ok.argmax(axis=1)], np.nan)
            assert np.array_equal(np.where(ok, base, 0.0), np.where(ok, first[:, None], 0.0))


def test_sweep_best_matches_oracle(gpu, oracle):
    """Best threshold per scenario and scheduler and speed-up over the baseline
    (Sec. 5.3, Sec. 6.1), on a real sweep (with invalid scenarios: NaN rows)
    and on values with ties, NaN entries and all-NaN columns."""
    import torch
    W = w()
    b = W.mixed(1500, seed=91)
    b.bw[0, 7] = float("nan")
    b.chunks[9] = 0
    thr = np.array([0.0, 1 / 64, 1 / 16, 1 / 4, 1.0])
    d = gpu.to_device(b)
    for mask, col in ((7, 0), (6, -1), (3, 0), (4, -1)):
        t = gpu.themis_sweep(d, torch.from_numpy(thr).cuda(), mask)
        best_t, best_thr, speedup = gpu.themis_sweep_best(t, col)
        torch.cuda.synchronize()
        o_t, o_thr, o_s = oracle.sweep_best(t.cpu().numpy(), col)
        assert_close("best_t", best_t.cpu().numpy(), o_t)
        assert np.array_equal(best_thr.cpu().numpy(), o_thr)
        if col >= 0:
            assert_close("speedup", speedup.cpu().numpy(), o_s)
        else:
            assert speedup is None
        assert np.isnan(o_t[7]).all() and (o_thr[9] == 0xFFFFFFFF).all()
    rng = np.random.default_rng(5)
    t = rng.integers(1, 6, (4000, 7, 3)).astype(np.float64)      # many ties
    t[rng.random(t.shape) < 0.3] = np.nan
    t[::17, :, 1] = np.nan
    best_t, best_thr, speedup = gpu.themis_sweep_best(torch.from_numpy(t).cuda(), 0)
    torch.cuda.synchronize()
    o_t, o_thr, o_s = oracle.sweep_best(t, 0)
    assert_close("best_t", best_t.cpu().numpy(), o_t)
    assert np.array_equal(best_thr.cpu().numpy(), o_thr)
    assert_close("speedup", speedup.cpu().numpy(), o_s)
    # an empty batch is fine
    e = gpu.themis_sweep_best(torch.empty((0, 3, 2), dtype=torch.float64, device="cuda"), 0)
    assert e[0].shape == (0, 2)


def test_determinism_and_permutation_invariance(gpu):
    """The same scenario gives the same bits wherever it sits in the batch
    (the consistency requirement of Sec. 4.6: every NPU must derive exactly
    the same schedule)."""
    b = w().config3(n=2048)
    a = run_gpu(gpu, b)
    perm = np.random.default_rng(0).permutation(b.n)
    p = run_gpu(gpu, b.take(perm))
    assert np.array_equal(a[0][perm], p[0])
    assert np.array_equal(a[2][perm], p[2])
    assert np.array_equal(a[3][perm], p[3])
    again = run_gpu(gpu, b)
    assert all(np.array_equal(x, y) for x, y in zip(a, again))


def test_full_size_config3_sampled_and_invariants(gpu, oracle):
    """The 1,048,576-scenario configuration in the launch shape bench.py times:
    sampled scenarios against the oracle, and properties that hold for every
    scenario (Sec. 4.4: T >= max_K load_K; Table 3 Ideal: T >= S / sum B;
    every dimension executes each (chunk, phase) exactly once)."""
    import torch
    W = w()
    b = W.config3()
    d = gpu.to_device(b)
    orders, loads = gpu.themis_plan_batch(d)
    ws = gpu.alloc_workspace(gpu.themis_workspace_bytes(d.n, d.max_chunks))
    t, qo, busy = gpu.themis_simulate_batch(d, orders, workspace=ws)
    torch.cuda.synchronize()
    # -- invariants over the whole batch, evaluated with torch on the device
    assert bool(torch.isfinite(t).all())
    assert bool((t >= loads.max(dim=0).values * (1 - 1e-12)).all())
    ideal = d.size_bytes / d.bw.sum(dim=0)
    assert bool((t >= ideal).all())
    rel = ((busy - loads).abs() / loads).max().item()
    assert rel <= 1e-12, f"busy vs planned loads: {rel:.3e}"
    rows = torch.sort(qo.view(-1, 2 * d.slots), dim=1).values
    want = torch.arange(2 * d.slots, dtype=torch.uint8, device=rows.device)
    assert bool((rows == want).all()), "a dimension's executed list is not a permutation"
    del rows
    o = orders.to(torch.int32)
    seen = (1 << (o & 3)) | (1 << ((o >> 2) & 3)) | (1 << ((o >> 4) & 3)) | (1 << ((o >> 6) & 3))
    assert bool((seen == 15).all()), "an order code is not a permutation of the 4 dimensions"
    # -- sampled scenarios against the oracle, element by element
    idx = np.sort(np.random.default_rng(2110).choice(b.n, 4096, replace=False))
    sub = b.take(idx)
    o_orders, o_loads = oracle.plan_batch(sub, threads=8)
    o_t, o_qo, o_busy = oracle.simulate_batch(sub, o_orders, threads=8)
    sel = torch.from_numpy(idx).cuda()
    assert np.array_equal(orders[sel].cpu().numpy(), o_orders)
    assert np.array_equal(widen_queue(qo[sel]), o_qo)
    assert_close("t_done", t[sel].cpu().numpy(), o_t)
    assert_close("loads", loads[:, sel].cpu().numpy(), o_loads)
    assert_close("busy", busy[:, sel].cpu().numpy(), o_busy)


def test_full_size_config4_sweep_sampled_and_invariants(gpu, oracle):
    """The 512-chunk threshold sweep whole (65,536 scenarios x 8 thresholds x
    {FIFO, SCF}) in the launch shape bench.py times with --workload config4:
    sampled scenarios against the oracle, and T >= S / sum B (Table 3, Ideal)
    for every evaluation."""
    import torch
    W = w()
    b = W.config4()
    thr = W.CONFIG4_THRESHOLDS
    mask = W.SWEEP_THEMIS_FIFO | W.SWEEP_THEMIS_SCF
    d = gpu.to_device(b)
    got = gpu.themis_sweep(d, torch.from_numpy(thr).cuda(), mask)
    torch.cuda.synchronize()
    assert got.shape == (b.n, len(thr), 2)
    assert bool(torch.isfinite(got).all())
    ideal = d.size_bytes / d.bw.sum(dim=0)
    assert bool((got >= ideal[:, None, None]).all())
    idx = np.sort(np.random.default_rng(4478).choice(b.n, 48, replace=False))
    want = oracle.sweep(b.take(idx), thr, mask, threads=8)
    assert_close("sweep t_done", got[torch.from_numpy(idx).cuda()].cpu().numpy(), want)


def test_full_size_config5_traces_sampled_and_invariants(gpu, oracle):
    """The 16,384 traces of 200 collectives whole, in the launch shape bench.py
    times with --workload config5 (times and busy times, no queue orders):
    sampled scenarios against the oracle; T >= the busiest dimension's busy
    time (Sec. 4.4) and T >= sum S / sum B for every scenario."""
    import torch
    W = w()
    b = W.config5()
    d = gpu.to_device(b)
    orders, loads = gpu.themis_plan_batch(d)
    ws = gpu.alloc_workspace(gpu.themis_workspace_bytes(d.n, d.max_chunks, d.max_coll))
    t, _, busy = gpu.themis_simulate_batch(d, orders, workspace=ws, want_queue_order=False)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(t).all())
    assert bool((t >= busy.max(dim=0).values * (1 - 1e-12)).all())
    ideal = d.coll_size.sum(dim=0) / d.bw[:3].sum(dim=0)
    assert bool((t >= ideal).all())
    idx = np.sort(np.random.default_rng(2110).choice(b.n, 24, replace=False))
    sub = b.take(idx)
    o_orders, _ = oracle.plan_batch(sub, threads=8)
    o_t, _, o_busy = oracle.simulate_batch(sub, o_orders, want_queue_order=False, threads=8)
    sel = torch.from_numpy(idx).cuda()
    assert np.array_equal(orders[sel].cpu().numpy(), o_orders)
    assert_close("t_done", t[sel].cpu().numpy(), o_t)
    assert_close("busy", busy[:, sel].cpu().numpy(), o_busy)


def _with_fixed_delay(b, seed):
    rng = np.random.default_rng(seed)
    b.fixed_delay = np.ascontiguousarray(
        rng.uniform(0, 2e-5, (4, b.n)) * (rng.uniform(0, 1, (4, b.n)) < 0.7))
    return b


def test_fixed_delay_per_stage(gpu, oracle):
    """Fixed delay A_K (Sec. 4.5): tracker start and stage times, on every path
    (LDS layouts, generic, trace, sweep)."""
    import torch
    W = w()
    check_batch(gpu, oracle, W.table2())
    check_batch(gpu, oracle, W.table2(intra=W.INTRA_FIFO, chunks=512))
    check_batch(gpu, oracle, _with_fixed_delay(W.mixed(900, seed=51), 1))
    check_batch(gpu, oracle, _with_fixed_delay(W.mixed(300, seed=52, pow2=False), 2))
    check_batch(gpu, oracle, _with_fixed_delay(W.mixed(120, seed=53, max_chunks=200), 3))
    check_batch(gpu, oracle, _with_fixed_delay(W.config5(n=70, n_coll=7), 4))
    b = _with_fixed_delay(W.mixed(400, seed=54), 5)
    b.fixed_delay[1, 17] = -1.0          # invalid delay -> NaN scenario (if D > 1)
    b.ndims[17] = 3
    t = check_batch(gpu, oracle, b)
    assert np.isnan(t[17])
    thr = np.array([0.0, 1 / 16])
    want = oracle.sweep(b, thr, 7, threads=8)
    d = gpu.to_device(b)
    ws = gpu.alloc_workspace(gpu.themis_workspace_bytes(d.n * 2 * 3, d.max_chunks))
    got = gpu.themis_sweep(d, torch.from_numpy(thr).cuda(), 7, workspace=ws)
    torch.cuda.synchronize()
    assert_close("sweep with fixed delay", got.cpu().numpy(), want)


def test_metrics_match_oracle(gpu, oracle):
    import torch
    W = w()
    for b in (W.config3(n=5000), W.mixed(777, seed=61, pow2=False), W.config5(n=66, n_coll=5)):
        d = gpu.to_device(b)
        orders, loads = gpu.themis_plan_batch(d)
        ws = gpu.alloc_workspace(gpu.themis_workspace_bytes(
            d.n, d.max_chunks, d.max_coll if d.n_coll is not None else 0))
        t, _, busy = gpu.themis_simulate_batch(d, orders, workspace=ws, want_queue_order=False)
        util, ideal = gpu.themis_metrics_batch(d, t, busy)
        torch.cuda.synchronize()
        o_util, o_ideal = oracle.metrics_batch(b, t.cpu().numpy(), busy.cpu().numpy())
        assert_close("utilization", util.cpu().numpy(), o_util)
        assert_close("ideal", ideal.cpu().numpy(), o_ideal)
        u = util.cpu().numpy()
        assert np.all((u > 0) & (u <= 1 + 1e-12))
        # T >= Ideal (equality up to rounding for one dimension of two NPUs)
        assert np.all(t.cpu().numpy() >= ideal.cpu().numpy() * (1 - 1e-12))


def _with_collective_types(b, seed):
    b.collective_type = np.random.default_rng(seed).integers(0, 3, b.n).astype(np.uint8)
    return b


def test_stand_alone_reduce_scatter_and_all_gather(gpu, oracle):
    """Alg. 1's CollectiveType per scenario, on every path."""
    W = w()
    check_batch(gpu, oracle, _with_collective_types(W.mixed(1000, seed=71), 1))
    check_batch(gpu, oracle, _with_collective_types(W.mixed(1000, seed=72, thr_mode=0), 2))
    check_batch(gpu, oracle, _with_collective_types(W.mixed(400, seed=73, pow2=False), 3))
    check_batch(gpu, oracle, _with_collective_types(W.mixed(150, seed=74, max_chunks=300), 4))
    check_batch(gpu, oracle, _with_collective_types(_with_fixed_delay(W.mixed(500, seed=75), 6), 5))
    check_batch(gpu, oracle, _with_collective_types(W.config5(n=90, n_coll=8), 7))
    b = _with_collective_types(W.config3(n=3000), 8)
    check_batch(gpu, oracle, b)
    b = W.mixed(128, seed=76)
    b.collective_type = np.full(b.n, 1, np.uint8)
    b.collective_type[5] = 3               # not a collective type -> invalid scenario
    t = check_batch(gpu, oracle, b)
    assert np.isnan(t[5]) and np.isfinite(t[4])


def test_exhaustive_search_matches_oracle(gpu, oracle):
    """themis_search_batch: all (D!)^C assignments per scenario, best time and
    the first assignment that reaches it."""
    import torch
    W = w()
    rng = np.random.default_rng(8)
    n = 150
    D = rng.integers(1, 5, n)
    C = np.array([int(rng.integers(1, {1: 9, 2: 9, 3: 5, 4: 4}[int(d)])) for d in D])
    D[3], C[3] = 4, 8                     # 24^8 schedules: over the bound
    P = [[int(2 ** rng.integers(1, 5)) for _ in range(d)] for d in D]
    bw = [[float(rng.uniform(25e9, 400e9)) for _ in range(d)] for d in D]
    b = W.make_batch(D, P, bw, np.floor(rng.uniform(2 ** 20, 2 ** 30, n)), C, 1,
                     rng.integers(0, 2, n), 0.0, max_chunks=8)
    b.collective_type = rng.integers(0, 3, n).astype(np.uint8)
    bound = 24 ** 3
    want_t, want_od = oracle.search_batch(b, bound, threads=8)
    d = gpu.to_device(b)
    got_t, got_od = gpu.themis_search_batch(d, bound)
    torch.cuda.synchronize()
    assert np.isnan(want_t[3])
    assert_close("best_t", got_t.cpu().numpy(), want_t)
    assert np.array_equal(got_od.cpu().numpy(), want_od)
    # the same search with fixed per-stage delays, rows wide enough for the 64-chunk layout
    b2 = W.make_batch(D, P, bw, b.size_bytes, C, 1, b.intra_policy, 0.0, max_chunks=20)
    b2.fixed_delay = np.ascontiguousarray(rng.uniform(0, 5e-6, (4, n)))
    w2_t, w2_od = oracle.search_batch(b2, bound, threads=8)
    g2_t, g2_od = gpu.themis_search_batch(gpu.to_device(b2), bound)
    torch.cuda.synchronize()
    assert_close("best_t (fixed delay)", g2_t.cpu().numpy(), w2_t)
    assert np.array_equal(g2_od.cpu().numpy(), w2_od)
    # NPU counts that are not powers of two: the same search on per-order tables
    P3 = [[int(rng.choice([3, 5, 6, 12, 4])) for _ in range(d_)] for d_ in D]
    b3 = W.make_batch(D, P3, bw, b.size_bytes, C, 1, b.intra_policy, 0.0, max_chunks=8)
    b3.collective_type = b.collective_type
    w3_t, w3_od = oracle.search_batch(b3, bound, threads=8)
    g3_t, g3_od = gpu.themis_search_batch(gpu.to_device(b3), bound)
    torch.cuda.synchronize()
    assert np.isfinite(w3_t).sum() >= n - 2
    assert_close("best_t (other NPU counts)", g3_t.cpu().numpy(), w3_t)
    assert np.array_equal(g3_od.cpu().numpy(), w3_od)
    # the greedy plan can never beat the exhaustive optimum
    orders, _ = gpu.themis_plan_batch(d)
    t, _, _ = gpu.themis_simulate_batch(d, orders, want_queue_order=False)
    torch.cuda.synchronize()
    ok = ~np.isnan(want_t)
    assert np.all(t.cpu().numpy()[ok] >= want_t[ok])


def test_provisioning_classes_match_oracle(gpu, oracle):
    """themis_classify_batch on balanced ladders tilted by powers of two (all
    three classes, exact ties included), arbitrary networks and invalid ones."""
    import torch
    W = w()
    rng = np.random.default_rng(64)
    n = 5000
    D = rng.integers(1, 5, n)
    P, bw = [], []
    for i in range(n):
        p = [int(rng.integers(2, 65)) for _ in range(D[i])]
        if i % 2:
            top, b_i, shrink = float(2 ** rng.integers(30, 40)), [], 1.0
            for k in range(D[i]):
                b_i.append(top / shrink * float(2.0 ** rng.integers(-1, 2)))
                shrink *= p[k]
        else:
            b_i = [float(rng.uniform(1e9, 1e12)) for _ in range(D[i])]
        P.append(p); bw.append(b_i)
    P[7][0] = 1                            # invalid NPU count
    bw[9][D[9] - 1] = float("inf")         # invalid bandwidth
    b = W.make_batch(D, P, bw, 1e9, 4, 1, 0, 0.0)
    want = oracle.classify_batch(b)
    got = gpu.themis_classify_batch(gpu.to_device(b))
    torch.cuda.synchronize()
    assert (want[:, 7] == 0xFF).all() and (want[:, 9] == 0xFF).all()
    assert set(np.unique(want).tolist()) == {0, 1, 2, 0xFF}
    assert np.array_equal(got.cpu().numpy(), want)


def test_extreme_magnitudes_fall_back_to_the_generic_path(gpu, oracle):
    """Power-of-two networks whose stage times differ by hundreds of orders of
    magnitude: some stages are too short to move the clock, some times
    overflow.  The LDS path must notice and hand these scenarios to the generic
    path, lane by lane, next to ordinary scenarios in the same wavefront."""
    W = w()
    P = [[4, 4], [4, 4], [2, 8, 4], [4, 4], [4, 4], [4, 8], [2, 2, 2, 2]]
    bw = [[1e3, 1e300], [1e300, 1e3], [1e9, 1e290, 1e-5], [1e-300, 1e9], [1e9, 1e-300],
          [200e9, 50e9], [1e11, 1e-200, 1e200, 1e11]]
    reps = 20
    b = W.make_batch([len(p) for p in P] * reps, P * reps, bw * reps, 2.0 ** 30,
                     [8, 5, 8, 3, 8, 8, 6] * reps, 1, [1, 0, 1, 1, 0, 1, 1] * reps, 0.0,
                     max_chunks=8)
    check_batch(gpu, oracle, b)


def test_entry_points_replay_inside_a_hip_graph(gpu, oracle):
    """The C ABI allocates nothing and only launches kernels on the caller's
    stream, so plan + simulate + sweep can be captured into a HIP graph once and
    replayed; every replay (with eager work and synchronisations in between)
    must reproduce the eager, oracle-checked result bit for bit."""
    import torch
    b = w().mixed(3000, seed=77)           # includes scenarios that go to the generic kernel
    d = gpu.to_device(b)
    n = d.n
    orders = torch.empty((n, d.slots), dtype=torch.uint8, device="cuda")
    loads = torch.empty((4, n), dtype=torch.float64, device="cuda")
    t_done = torch.empty(n, dtype=torch.float64, device="cuda")
    busy = torch.empty((4, n), dtype=torch.float64, device="cuda")
    qo = torch.empty((n, 4, 2 * d.slots), dtype=torch.uint8, device="cuda")
    thr = torch.tensor([0.0, 0.25], dtype=torch.float64, device="cuda")
    sw = torch.empty((n, 2, 3), dtype=torch.float64, device="cuda")
    ws = gpu.alloc_workspace(gpu.themis_workspace_bytes(n * 6, d.max_chunks))

    def run():
        gpu.themis_plan_batch(d, orders, loads)
        gpu.themis_simulate_batch(d, orders, t_done, qo, busy, ws)
        gpu.themis_sweep(d, thr, 7, t_done=sw, workspace=ws)

    run()
    torch.cuda.synchronize()
    want = [x.clone() for x in (orders, loads, t_done, busy, qo, sw)]
    o_orders, _ = oracle.plan_batch(b, threads=8)
    o_t, _, _ = oracle.simulate_batch(b, o_orders, want_queue_order=False, threads=8)
    assert np.array_equal(want[0].cpu().numpy(), o_orders)
    assert_close("eager t_done", want[2].cpu().numpy(), o_t)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        run()                               # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            run()
    torch.cuda.synchronize()
    for rep in range(4):
        for x in (orders, loads, t_done, busy, qo, sw):
            x.fill_(7 if x.dtype == torch.uint8 else -1.0)   # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, got, ref in zip(("orders", "loads", "t_done", "busy", "queue_order", "sweep"),
                                  (orders, loads, t_done, busy, qo, sw), want):
            same = torch.equal(got, ref) if got.dtype == torch.uint8 else bool(
                ((got == ref) | (torch.isnan(got) & torch.isnan(ref))).all())
            assert same, f"replay {rep}: {name} differs from the eager run"


def test_kernel_launches_per_call(gpu):
    """How many kernels a call launches, counted as the nodes of a HIP graph
    captured around it: the planner one; the simulation and the sweep two (the
    LDS kernel and one follow-up kernel that holds the table passes and the
    generic pass), whatever the chunk capacity; three only for a batch of more
    than 2 x CUs wavefronts with up to 64 chunks and no workspace, whose generic
    pass keeps its 80 KiB of LDS to itself."""
    import ctypes as C
    import torch
    hip = C.CDLL("libamdhip64.so")

    def nodes(fn):
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            fn()                                             # warm-up: nothing lazy left to load
            side.synchronize()
            handle = C.c_void_p(side.cuda_stream)
            assert hip.hipStreamBeginCapture(handle, 2) == 0     # relaxed: other threads may call HIP
            try:
                fn()
            finally:
                graph = C.c_void_p()
                rc = hip.hipStreamEndCapture(handle, C.byref(graph))
            assert rc == 0 and graph.value
            count = C.c_size_t(0)
            assert hip.hipGraphGetNodes(graph, None, C.byref(count)) == 0
            hip.hipGraphDestroy(graph)
        torch.cuda.synchronize()
        return count.value

    cus = torch.cuda.get_device_properties(0).multi_processor_count
    thr = torch.tensor([0.0, 0.25], dtype=torch.float64, device="cuda")
    for max_chunks, n, with_ws, want in ((64, 3000, False, 2), (64, 3000, True, 2), (16, 500, False, 2),
                                         (128, 700, True, 2), (512, 300, True, 2),
                                         (64, 2 * cus * 64 + 64, True, 2), (64, 2 * cus * 64 + 64, False, 3)):
        b = w().mixed(n, seed=500 + max_chunks, max_chunks=max_chunks, pow2=(max_chunks != 128))
        d = gpu.to_device(b)
        orders = torch.empty((n, d.slots), dtype=torch.uint8, device="cuda")
        loads = torch.empty((4, n), dtype=torch.float64, device="cuda")
        t_done = torch.empty(n, dtype=torch.float64, device="cuda")
        busy = torch.empty((4, n), dtype=torch.float64, device="cuda")
        qo = torch.empty((n, 4, 2 * d.slots), dtype=torch.uint8 if max_chunks <= 127 else torch.int16,
                         device="cuda")
        sw = torch.empty((n, 2, 3), dtype=torch.float64, device="cuda")
        ws = gpu.alloc_workspace(gpu.themis_workspace_bytes(n * 6, d.max_chunks)) if with_ws else None
        assert nodes(lambda: gpu.themis_plan_batch(d, orders, loads)) == 1
        assert nodes(lambda: gpu.themis_simulate_batch(d, orders, t_done, qo, busy, ws)) == want, \
            (max_chunks, n, with_ws)
        assert nodes(lambda: gpu.themis_sweep(d, thr, 7, t_done=sw, workspace=ws)) == want, \
            (max_chunks, n, with_ws)


@pytest.mark.parametrize("max_chunks,pow2,thr_mode", [(2, True, 0), (64, True, 1), (64, False, 0),
                                                      (100, True, 1)])
def test_special_values(gpu, oracle, max_chunks, pow2, thr_mode):
    """Thresholds 0 / denormal / huge / infinite / negative / NaN, sizes of one
    byte, 2^60 bytes, 1e-300 bytes (halvings leave the normal range), zero and
    infinity, bandwidths 60 orders of magnitude apart: valid ones must match
    the oracle, invalid ones come back as NaN / all-ones on both sides."""
    n = 1200
    rng = np.random.default_rng(900 + max_chunks)
    b = w().mixed(n, seed=901 + max_chunks, max_chunks=max_chunks, pow2=pow2, thr_mode=thr_mode)
    sel = rng.random(n)
    thr = b.threshold.copy()
    thr[sel < 0.1] = np.inf if thr_mode == 0 else 1e300
    thr[(sel >= 0.1) & (sel < 0.2)] = 5e-324
    thr[(sel >= 0.2) & (sel < 0.25)] = -1.0
    thr[(sel >= 0.25) & (sel < 0.28)] = np.nan
    b.threshold = thr
    sel = rng.random(n)
    S = b.size_bytes.copy()
    S[sel < 0.1] = 1.0
    S[(sel >= 0.1) & (sel < 0.2)] = 2.0 ** 60
    S[(sel >= 0.2) & (sel < 0.25)] = 1e-300
    S[(sel >= 0.25) & (sel < 0.27)] = 0.0
    S[(sel >= 0.27) & (sel < 0.29)] = np.inf
    b.size_bytes = S
    sel = rng.random((4, n))
    bw = b.bw.copy()
    bw[sel < 0.03] = 1e-30
    bw[(sel >= 0.03) & (sel < 0.06)] = 1e30
    b.bw = np.ascontiguousarray(bw)
    t = check_batch(gpu, oracle, b, threads=16)
    assert 0 < int(np.isnan(t).sum()) < n


@pytest.mark.parametrize("ctype", [0, 1, 2])
def test_wavefronts_that_share_one_network(gpu, oracle, ctype):
    """Parameter studies put one topology into every lane of a wavefront, only
    bandwidths, sizes, chunk counts and thresholds differ: such wavefronts take
    what a stage does from an (order, stage) table the wavefront builds once.
    Every dimension count, both queue policies, each collective type, planned
    and arbitrary orders (all D! permutations inside a scenario), fixed delays,
    a ragged last wavefront, an invalid scenario inside a wavefront, and a
    batch whose wavefronts differ from each other (one table per wavefront)."""
    import torch
    W = w()
    rng = np.random.default_rng(600 + ctype)
    nets = [(1, [8]), (2, [4, 16]), (3, [2, 8, 4]), (4, [2, 8, 8, 64]), (4, [16, 2, 4, 4]), (3, [64, 2, 2])]
    parts = []
    for D, P in nets:
        for intra in (0, 1):
            n = 64 * 2 + (17 if (D, intra) == (4, 1) else 0)
            b = W.config3(n=n, seed=W.SEED_BASE + 100 * D + intra)
            b.ndims[:] = D
            b.npus[:, :] = 2
            for k in range(D):
                b.npus[k, :] = P[k]
            b.intra_policy[:] = intra
            b.chunks = rng.integers(1, 65, n).astype(np.uint32)
            b.chunks[:3] = [64, 1, 63]
            parts.append(b)
    cat = lambda f: np.concatenate([getattr(p, f) for p in parts], axis=-1)
    n = sum(p.n for p in parts)
    b = W.ScenarioBatch(n=n, max_chunks=64, threshold_mode=W.THR_REL, ndims=cat("ndims"),
                        npus=np.ascontiguousarray(cat("npus")), bw=np.ascontiguousarray(cat("bw")),
                        size_bytes=cat("size_bytes"), chunks=cat("chunks"),
                        inter_policy=cat("inter_policy"), intra_policy=cat("intra_policy"),
                        threshold=cat("threshold"))
    b.collective_type = np.full(n, ctype, np.uint8)
    b.bw[0, 70] = float("nan")            # an invalid scenario in the second wavefront
    t = check_batch(gpu, oracle, b)
    assert np.isnan(t[70]) and int(np.isnan(t).sum()) == 1
    check_batch(gpu, oracle, _with_fixed_delay(b, 7))
    # arbitrary orders
    orders = np.full((n, 64), 0xFF, np.uint8)
    for i in range(n):
        D = int(b.ndims[i])
        perms = np.argsort(rng.random((int(b.chunks[i]), D)), axis=1)
        orders[i, :perms.shape[0]] = (perms << (2 * np.arange(D))).sum(axis=1)
    o_t, o_qo, o_busy = oracle.simulate_batch(b, orders, threads=8)
    d = gpu.to_device(b)
    t, qo, busy = gpu.themis_simulate_batch(d, torch.from_numpy(orders).cuda())
    torch.cuda.synchronize()
    assert_close("t_done", t.cpu().numpy(), o_t)
    assert np.array_equal(widen_queue(qo), o_qo)
    assert_close("busy", busy.cpu().numpy(), o_busy)
    if ctype == 0:      # the fused sweep on the same wavefronts (times only)
        b.fixed_delay = None
        thr = np.array([0.0, 1 / 16])
        got = gpu.themis_sweep(gpu.to_device(b), torch.from_numpy(thr).cuda(), 7)
        torch.cuda.synchronize()
        assert_close("sweep", got.cpu().numpy(), oracle.sweep(b, thr, 7, threads=8))
