"""themis_simulate_batch_noalloc (the entry point for callers that cannot
allocate: its scratch is a device array inside the library) against
themis_simulate_batch with a caller workspace, through the C ABI: two calls in
a row, the second on a smaller batch, on inputs that do use the scratch --
traces (per-scenario queues live there) and single collectives of more than 64
chunks that only the generic path takes (its per-chunk arrays live there).

Bar as for every parity test: queue orders bit-exact, times within 1e-12
relative; the two entry points run the same kernels, so in fact every bit
agrees, and the oracle is checked beside them.
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
    ensure_built()
    binding.lib()
    return binding


def _close(name, got, want):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    assert np.array_equal(np.isnan(got), np.isnan(want)), f"{name}: NaN pattern differs"
    ok = ~np.isnan(want)
    err = np.abs(got[ok] - want[ok]) / np.maximum(np.abs(want[ok]), np.finfo(np.float64).tiny)
    assert err.size == 0 or err.max() <= REL_TOL, f"{name}: max rel err {err.max():.3e}"


def _widen(q):
    q = q.cpu().numpy()
    out = q.astype(np.uint16)
    if q.dtype == np.uint8:
        out[q == 0xFF] = 0xFFFF
    return out


def _batches():
    """(first, second): the second is smaller in scenarios, collectives and chunk slots."""
    from paper_2110_04478_amd import workloads as W
    rng = np.random.default_rng(17)
    # traces with staggered releases and ragged collective counts, both policies
    big = W.config5(n=300, n_coll=7)
    big.release_time = np.ascontiguousarray(rng.integers(0, 6, big.coll_size.shape) * 1e-4)
    big.n_coll = rng.integers(1, 8, big.n).astype(np.uint32)
    big.intra_policy[::3] = 0
    small = W.config5(n=70, n_coll=3)
    # single collectives of 100 chunk slots: bandwidths 297 orders of magnitude
    # apart make stages too short to move the clock, which no LDS path takes
    P = [[4, 4], [4, 4], [4, 8]]
    bw = [[1e3, 1e300], [1e300, 1e3], [200e9, 50e9]]
    reps = 12
    generic = W.make_batch([2, 2, 2] * reps, P * reps, bw * reps, 2.0 ** 30, [100, 70, 90] * reps,
                           1, [1, 0, 1] * reps, 0.0, max_chunks=100)
    return [big, generic], [small, generic.take(slice(0, 7))]


def _run_both(gpu, oracle, b):
    import torch
    d = gpu.to_device(b)
    orders, _ = gpu.themis_plan_batch(d)
    mc = d.max_coll if d.n_coll is not None else 0
    ws = gpu.alloc_workspace(gpu.themis_workspace_bytes(d.n, d.max_chunks, mc))
    t0, q0, z0 = gpu.themis_simulate_batch(d, orders, workspace=ws)
    torch.cuda.synchronize()
    # every buffer of the new call is allocated before it and is the caller's
    t1 = torch.full_like(t0, -1.0)
    q1 = torch.full_like(q0, 0x5A)
    z1 = torch.full_like(z0, -1.0)
    gpu.themis_simulate_batch_noalloc(d, orders, t1, q1, z1)
    torch.cuda.synchronize()
    print(f"no-alloc call: n={d.n} slots={d.slots} trace={d.n_coll is not None}", flush=True)
    _close("t_done", t1.cpu().numpy(), t0.cpu().numpy())
    _close("busy", z1.cpu().numpy(), z0.cpu().numpy())
    assert torch.equal(q1, q0), "queue orders differ between the two entry points"
    o_orders, _ = oracle.plan_batch(b, threads=8)
    o_t, o_q, o_z = oracle.simulate_batch(b, o_orders, threads=8)
    assert np.isfinite(o_t).all()
    _close("t_done vs oracle", t1.cpu().numpy(), o_t)
    _close("busy vs oracle", z1.cpu().numpy(), o_z)
    assert np.array_equal(_widen(q1), o_q)


def test_two_calls_in_a_row_the_second_smaller(gpu, oracle):
    first, second = _batches()
    for b in first:
        _run_both(gpu, oracle, b)
    for b in second:       # the scratch still holds what the larger calls left
        _run_both(gpu, oracle, b)


def test_requests_beyond_the_scratch_are_refused(gpu):
    import torch
    from paper_2110_04478_amd import workloads as W
    b = W.config5(n=2048, n_coll=200)
    d = gpu.to_device(b)
    assert gpu.themis_workspace_bytes(d.n, d.max_chunks, d.max_coll) > gpu.STATIC_SCRATCH_BYTES
    orders = torch.zeros((d.n, d.slots), dtype=torch.uint8, device="cuda")
    t = torch.full((d.n,), -1.0, dtype=torch.float64, device="cuda")
    with pytest.raises(gpu.ThemisError) as e:
        gpu.themis_simulate_batch_noalloc(d, orders, t, None, None)
    assert e.value.status == -4
    torch.cuda.synchronize()
    assert bool((t == -1.0).all())          # nothing was launched
    # up to 64 chunk slots a single collective needs no scratch: any batch size goes
    b = W.config3(n=100000)
    d = gpu.to_device(b)
    orders, _ = gpu.themis_plan_batch(d)
    t0, _, _ = gpu.themis_simulate_batch(d, orders, want_queue_order=False, want_busy=False)
    t1 = torch.empty_like(t0)
    gpu.themis_simulate_batch_noalloc(d, orders, t1, None, None)
    torch.cuda.synchronize()
    assert torch.equal(t0, t1)
