#!/usr/bin/env python3
"""Benchmark of the batched Themis evaluator on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic
scenarios resident in HBM: themis_plan_batch (Alg. 1) followed by
themis_simulate_batch (queue simulation) with every output requested (order
codes, final loads, completion times, per-dimension queue orders, busy times).
The workload is the 1,048,576-scenario 4-D configuration (P = (2,8,8,64),
C = 64, Themis + SCF, relative threshold).  Prints ONE JSON line.

--workload config4 / config5 time the two heavier configurations instead (the
512-chunk threshold sweep through themis_sweep, the 200-collective traces
through themis_plan_batch + themis_simulate_batch); they exist to profile the
wide-layout and trace kernels and print the same kind of line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

def device_peak(torch):
    """Vector issue peak of the device the run is on: compute units x 4 SIMDs x
    clock / 4 cycles per wave64 instruction, x 64 lanes.  Both figures come from
    the device properties (MI355X: 256 CUs, 2.4 GHz -> 39.3 Tlane-op/s, which is
    also the published 78.6 TFLOP/s of fp64 vector FMA)."""
    p = torch.cuda.get_device_properties(0)
    cus = int(p.multi_processor_count)
    khz = getattr(p, "clock_rate", None)
    if not khz:                       # older builds: ask the runtime
        import ctypes
        hip = ctypes.CDLL("libamdhip64.so")
        v = ctypes.c_int(0)
        rc = hip.hipDeviceGetAttribute(ctypes.byref(v), 5, 0)   # hipDeviceAttributeClockRate, kHz
        khz = v.value
        if rc != 0 or not 1e5 < khz < 1e7:
            sys.exit("bench.py: the runtime reports no usable clock rate (%d, status %d)" % (khz, rc))
    hz = float(khz) * 1e3
    return {"compute_units": cus, "clock_mhz_nominal": hz / 1e6,
            "wave_instr_per_s": cus * 4 * hz / 4, "lane_ops_per_s": cus * 4 * hz / 4 * 64}


def algorithmic_lane_ops(D, C):
    """Lane-operations one scenario needs, per kernel: the planner does about
    45 compare/select/flop operations per chunk (min/max over D loads, a
    D-element stable sort, D multiplies, divides and adds); the simulation
    handles 2*D*C chunk-stage events, each selecting the smallest key among
    up to C waiting chunks (one comparison per chunk)."""
    return {"plan": 45 * C, "simulate": 2 * D * C * C}


def profiled_figures(name):
    """Counter figures of an earlier rocprofv3 run of this file, kept as
    `key: value` lines between the markers of profiles/<name>.md together with
    the commit they were taken on.  None if the summary is not there."""
    path = os.path.join(ROOT, "profiles", name + ".md")
    if not os.path.exists(path):
        return None
    out, inside = {}, False
    for line in open(path):
        line = line.strip()
        if line.startswith("<!-- figures"):
            inside = True
        elif line.startswith("<!-- end figures"):
            inside = False
        elif inside and ":" in line:
            k, v = line.split(":", 1)
            try:
                out[k.strip()] = float(v)
            except ValueError:
                out[k.strip()] = v.strip()
    return out or None


def median(xs):
    xs = sorted(xs)
    return float(xs[len(xs) // 2]) if len(xs) % 2 else float(0.5 * (xs[len(xs) // 2 - 1] + xs[len(xs) // 2]))


def other_workload(args, np, torch, binding, workloads):
    """config4: one step = themis_sweep over 8 thresholds x {FIFO, SCF} of 65,536 scenarios
    with C = 512.  config5: one step = plan + simulate of 16,384 traces of 200 collectives."""
    dev = "cuda:0"
    if args.workload == "config4":
        n = args.scenarios if args.scenarios != 1 << 20 else 65536
        host = workloads.config4(n=n)
        D, C, Q = 4, 512, 1
        d = binding.to_device(host, dev)
        thr = torch.from_numpy(workloads.CONFIG4_THRESHOLDS).to(dev)
        mask = workloads.SWEEP_THEMIS_FIFO | workloads.SWEEP_THEMIS_SCF
        evals = n * len(workloads.CONFIG4_THRESHOLDS) * 2
        out = torch.empty((n, len(workloads.CONFIG4_THRESHOLDS), 2), dtype=torch.float64, device=dev)

        def step():
            binding.themis_sweep(d, thr, mask, t_done=out)
        name = ("config4: %d scenarios x 8 thresholds x {FIFO,SCF}, 4-D P_k=2^U{1..6}, C=512, "
                "themis_sweep, %s mapping" % (n, args.sweep_mapping))
        kernel = "sweep"
    else:
        n = args.scenarios if args.scenarios != 1 << 20 else 16384
        host = workloads.config5(n=n)
        if args.workload in ("config5fifo6", "config5scf6"):
            # the same traces on P = (6, 12, 24): NPU counts that are not powers of two on the
            # list path, under first-in-first-out or Smallest-Chunk-First
            host.npus = np.ascontiguousarray(np.array([[6], [12], [24], [1]], dtype=np.uint32).repeat(n, axis=1))
            if args.workload == "config5fifo6":
                host.intra_policy[:] = 0
        D, C, Q = 3, 64, host.max_coll
        d = binding.to_device(host, dev)
        evals = n
        orders = torch.empty((n, d.slots), dtype=torch.uint8, device=dev)
        loads = torch.empty((4, n), dtype=torch.float64, device=dev)
        out = torch.empty(n, dtype=torch.float64, device=dev)
        busy = torch.empty((4, n), dtype=torch.float64, device=dev)
        ws = binding.alloc_workspace(binding.themis_workspace_bytes(n, d.max_chunks, d.max_coll))

        def step():
            binding.themis_plan_batch(d, orders, loads)
            binding.themis_simulate_batch(d, orders, out, None, busy, ws, want_queue_order=False)
        name = ("config5: %d traces of %d All-Reduces, 3-D P=(8,16,32), C=64, Themis+SCF, "
                "plan + simulate (times and busy)" % (n, Q))
        if args.workload == "config5fifo6":
            name = name.replace("P=(8,16,32)", "P=(6,12,24)").replace("Themis+SCF", "Themis+FIFO").replace("config5", "config5fifo6")
        if args.workload == "config5scf6":
            name = name.replace("P=(8,16,32)", "P=(6,12,24)").replace("config5", "config5scf6")
        kernel = "simulate_trace"
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for e in evs:
        e[0].record()
        step()
        e[1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms = wall * 1e3 / args.steps
    kernel_ms = median([e[0].elapsed_time(e[1]) for e in evs])
    events = evals * 2 * D * C * Q
    peak = device_peak(torch)
    PEAK_LANE_OPS_PER_S = peak["lane_ops_per_s"]
    lane_ops = evals * Q * algorithmic_lane_ops(D, C)["simulate"]
    achieved = lane_ops / (kernel_ms * 1e-3)
    result = {
        "metric": "scenarios_per_sec", "value": n / (ms * 1e-3), "unit": "scenarios/s",
        "evaluations_per_sec": evals / (ms * 1e-3), "events_per_sec": events / (ms * 1e-3),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "kernel_ms": {kernel: kernel_ms, "statistic": "median of the per-step HIP-event times"},
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f64",
        "data": "synthetic", "config": {"workload": name},
        "nan_results": int(torch.isnan(out).sum().item()),
        "roofline": {"bound": "alu", "kernel": kernel, "achieved": achieved / 1e12,
                     "peak": PEAK_LANE_OPS_PER_S / 1e12, "unit": "Tlane-op/s",
                     "frac": achieved / PEAK_LANE_OPS_PER_S, "traffic": None,
                     "traffic_source": None, "compute_units": peak["compute_units"],
                     "clock_mhz_nominal": peak["clock_mhz_nominal"]},
    }
    if args.cpu_sample > 0:
        from oracle import themis_oracle
        m = min(n, 256 if args.workload == "config4" else 48)
        sample = host.take(slice(0, m))
        cores = min(os.cpu_count() or 1, 16)
        c0 = time.perf_counter()
        if args.workload == "config4":
            o = themis_oracle.sweep(sample, workloads.CONFIG4_THRESHOLDS, mask, threads=cores)
            g = out[:m].cpu().numpy()
        else:
            oo, _ = themis_oracle.plan_batch(sample, threads=cores)
            o, _, _ = themis_oracle.simulate_batch(sample, oo, want_queue_order=False, threads=cores)
            g = out[:m].cpu().numpy()
        cpu_s = time.perf_counter() - c0
        result["cpu_baseline"] = {
            "value": m / cpu_s, "unit": "scenarios/s", "cores": cores, "kind": "oracle",
            "sample": "first %d scenarios, %d threads, %.1f s" % (m, cores, cpu_s),
            "parity_on_sample": {"t_done_max_rel_err": float(np.max(np.abs(g - o) / o))}}
    return result


def small_workload(args, np, torch, binding, workloads):
    """Latency of the small cases, end to end (plan + simulate with every output): the single
    2-D scenario of the smallest configuration and the first 64 scenarios of the bench batch
    (one wavefront).  Per call: median over the timed steps of the HIP-event time around the
    two entry points, and the host's wall time per step with one synchronisation at the end."""
    dev = "cuda:0"
    rows = {}
    for name, host in (("config1: 1 scenario, 2-D P=(4,8), C=4", workloads.config1()),
                       ("64 scenarios of config3 (one wavefront)", workloads.config3(n=64))):
        n = host.n
        d = binding.to_device(host, dev)
        orders = torch.empty((n, d.slots), dtype=torch.uint8, device=dev)
        loads = torch.empty((4, n), dtype=torch.float64, device=dev)
        t = torch.empty(n, dtype=torch.float64, device=dev)
        busy = torch.empty((4, n), dtype=torch.float64, device=dev)
        qo = torch.empty((n, 4, 2 * d.slots), dtype=torch.uint8, device=dev)

        def step():
            binding.themis_plan_batch(d, orders, loads)
            binding.themis_simulate_batch(d, orders, t, qo, busy)
        for _ in range(max(args.warmup, 3)):
            step()
        torch.cuda.synchronize()
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
        t0 = time.perf_counter()
        for e in evs:
            e[0].record()
            step()
            e[1].record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        rows[name] = {"us_per_call_events_median": 1e3 * median([e[0].elapsed_time(e[1]) for e in evs]),
                      "us_per_call_wall": 1e6 * wall / args.steps,
                      "kernel_launches_per_call": "plan 1 + simulate 2",
                      "t_done_first": float(t[0].item())}
    return {"metric": "small_batch_latency", "unit": "us", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "dtype": "f64", "data": "synthetic", "higher_is_better": False,
            "config": {"workload": "small: config1 and one wavefront of config3, plan + simulate, all outputs"},
            "rows": rows}


def extras_workload(args, np, torch, binding, workloads):
    """The entry points beyond plan / simulate / sweep on the 4-D bench networks, each timed
    on its own with HIP events on the stream the kernels run on: per-stage fixed delays,
    stand-alone Reduce-Scatter / All-Gather, the derived metrics, the provisioning classes,
    the exhaustive search over per-chunk orders and the best threshold of a sweep."""
    dev = "cuda:0"
    n = args.scenarios
    rng = np.random.default_rng(workloads.SEED_BASE)
    rows = {}

    def timed(name, units, fn):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        for _ in range(args.steps):
            fn()
        ev1.record()
        torch.cuda.synchronize()
        ms = ev0.elapsed_time(ev1) / args.steps
        rows[name] = {"ms": ms, "per_sec": units / (ms * 1e-3)}

    base = workloads.config3(n=n)
    events = n * 512.0
    # fixed delays per stage (Sec. 4.4): tracker start and stage times
    host = workloads.config3(n=n)
    host.fixed_delay = np.ascontiguousarray(rng.uniform(0, 2e-6, (4, n)))
    d = binding.to_device(host, dev)
    orders, loads = binding.themis_plan_batch(d)
    qo = torch.empty((n, 4, 2 * d.slots), dtype=torch.uint8, device=dev)
    t = torch.empty(n, dtype=torch.float64, device=dev)
    busy = torch.empty((4, n), dtype=torch.float64, device=dev)
    timed("fixed_delay: plan", n, lambda: binding.themis_plan_batch(d, orders, loads))
    timed("fixed_delay: simulate, all outputs (events/s)", events,
          lambda: binding.themis_simulate_batch(d, orders, t, qo, busy))
    # stand-alone collectives (Alg. 1's CollectiveType): a third each of All-Reduce, RS, AG
    host = workloads.config3(n=n)
    host.collective_type = rng.integers(0, 3, n).astype(np.uint8)
    d2 = binding.to_device(host, dev)
    ev2 = float(((host.collective_type == 0) + 1).sum()) * 4 * 64
    timed("collective types: plan", n, lambda: binding.themis_plan_batch(d2, orders, loads))
    timed("collective types: simulate, all outputs (events/s)", ev2,
          lambda: binding.themis_simulate_batch(d2, orders, t, qo, busy))
    # derived metrics and provisioning classes
    d0 = binding.to_device(base, dev)
    binding.themis_plan_batch(d0, orders, loads)
    binding.themis_simulate_batch(d0, orders, t, qo, busy)
    timed("metrics (utilisation, Ideal)", n, lambda: binding.themis_metrics_batch(d0, t, busy))
    timed("provisioning classes", n, lambda: binding.themis_classify_batch(d0))
    # exhaustive search: 3-D, 4 chunks -> 6^4 = 1,296 schedules per scenario
    ns = max(1, n // 64)
    small = workloads.config2(n=ns)
    small.chunks[:] = 4
    small.max_chunks = 4
    ds = binding.to_device(small, dev)
    timed("search: %d scenarios x 1,296 schedules (schedules/s)" % ns, ns * 1296.0,
          lambda: binding.themis_search_batch(ds, 1296))
    # beam search at the paper's default chunk count: width 4 on the 4-D bench networks,
    # 64 steps x 4 x 24 partial schedules per scenario
    nb = max(1, n // 256)
    beam_host = workloads.config3(n=nb)
    db = binding.to_device(beam_host, dev)
    beam_ws = binding.alloc_workspace(binding.lib().themis_beam_workspace_bytes(nb, db.max_chunks, 4), dev)
    timed("beam search: %d scenarios, 64 chunks, width 4 (partial schedules/s)" % nb,
          nb * 64.0 * 4 * 24, lambda: binding.themis_beam_search_batch(db, 4, beam_ws))
    beam_t, _ = binding.themis_beam_search_batch(db, 4, beam_ws)
    g_orders, _ = binding.themis_plan_batch(db)
    greedy_t, _, _ = binding.themis_simulate_batch(db, g_orders, want_queue_order=False)
    torch.cuda.synchronize()
    gain = (greedy_t / beam_t).cpu().numpy()
    # best threshold of a sweep
    thr = torch.from_numpy(workloads.CONFIG4_THRESHOLDS).to(dev)
    sweep = binding.themis_sweep(d0, thr, 7)
    timed("sweep: 8 thresholds x 3 schedulers (results/s; 17 simulations per scenario, "
          "the baseline's once)", n * 24.0,
          lambda: binding.themis_sweep(d0, thr, 7, t_done=sweep))
    timed("sweep_best", n, lambda: binding.themis_sweep_best(sweep, 0))
    best_t, best_thr, speedup = binding.themis_sweep_best(sweep, 0)
    torch.cuda.synchronize()
    sp = speedup.cpu().numpy()
    return {"metric": "extras", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "dtype": "f64", "data": "synthetic",
            "config": {"workload": "extras: %d scenarios of the 4-D bench networks" % n},
            "rows": rows,
            "beam_width4_over_greedy_themis": {"mean": float(np.mean(gain)), "max": float(np.max(gain)),
                                               "scenarios_improved": int((gain > 1.0).sum()),
                                               "scenarios": int(nb)},
            "speedup_over_baseline_best_threshold": {
                "themis_fifo_mean": float(np.mean(sp[:, 1])), "themis_scf_mean": float(np.mean(sp[:, 2])),
                "themis_scf_max": float(np.max(sp[:, 2]))}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--scenarios", type=int, default=1 << 20,
                    help="batch size (default: the 1M-scenario configuration)")
    ap.add_argument("--cpu-sample", type=int, default=1 << 20,
                    help="scenarios the CPU oracle is timed on (0 = skip)")
    ap.add_argument("--no-queue-order", action="store_true",
                    help="do not request the per-dimension queue orders")
    ap.add_argument("--workload", choices=("config3", "config4", "config5", "config5fifo6", "config5scf6", "extras", "small"), default="config3")
    ap.add_argument("--sweep-mapping", choices=("auto", "lane", "quad"), default="auto",
                    help="lane mapping of themis_sweep's LDS kernel (auto: the library's choice)")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="MIB",
                    help="instead of the benchmark, run a plain device copy of MIB MiB "
                         "(known traffic, to calibrate the FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build evaluates one GPU's share on one GPU; "
                 "run with --gpus 1 (scenarios are independent: a batch shards by scenario range)")

    import numpy as np
    import torch
    from paper_2110_04478_amd import binding, workloads
    from paper_2110_04478_amd.csrc.build import ensure_built

    assert torch.cuda.is_available(), "bench.py needs an MI355X"
    ensure_built()          # compiles only when no library is in the tree
    torch.cuda.set_device(0)
    binding.themis_set_sweep_mapping({"auto": 0, "lane": 1, "quad": 2}[args.sweep_mapping])
    if args.copy_probe:
        src = torch.full((args.copy_probe << 20,), 7, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes_read": src.numel(), "copy_probe_bytes_written": dst.numel()}))
        return
    if args.workload == "small":
        print(json.dumps(small_workload(args, np, torch, binding, workloads)))
        return
    if args.workload == "extras":
        print(json.dumps(extras_workload(args, np, torch, binding, workloads)))
        return
    if args.workload != "config3":
        print(json.dumps(other_workload(args, np, torch, binding, workloads)))
        return
    n = args.scenarios
    host = workloads.config3(n=n)
    D, C = 4, 64
    torch.cuda.synchronize()
    h0 = time.perf_counter()
    d = binding.to_device(host, "cuda:0")
    torch.cuda.synchronize()
    h2d_ms = (time.perf_counter() - h0) * 1e3     # pageable host arrays, once; not part of any step

    # outputs and scratch are allocated once, outside the timed region
    orders = torch.empty((n, d.slots), dtype=torch.uint8, device="cuda:0")
    loads = torch.empty((4, n), dtype=torch.float64, device="cuda:0")
    t_done = torch.empty(n, dtype=torch.float64, device="cuda:0")
    busy = torch.empty((4, n), dtype=torch.float64, device="cuda:0")
    qo = None if args.no_queue_order else torch.empty(
        (n, 4, 2 * d.slots), dtype=torch.uint8, device="cuda:0")
    ws = binding.alloc_workspace(binding.themis_workspace_bytes(n, d.max_chunks))

    def step(ev=None):
        if ev:
            ev[0].record()
        binding.themis_plan_batch(d, orders, loads)
        if ev:
            ev[1].record()
        binding.themis_simulate_batch(d, orders, t_done, qo, busy, ws,
                                      want_queue_order=False)
        if ev:
            ev[2].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # HIP events on the stream the kernels are launched on (torch's current one)
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)]
              for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(events[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    plan_ms = median([e[0].elapsed_time(e[1]) for e in events])
    sim_ms = median([e[1].elapsed_time(e[2]) for e in events])
    step_ms = median([e[0].elapsed_time(e[2]) for e in events])
    ms_per_step = wall * 1e3 / args.steps

    peak = device_peak(torch)
    default_workload = n == (1 << 20) and qo is not None
    prof = profiled_figures("simulate_kernel_config3") if default_workload else None
    ops = algorithmic_lane_ops(D, C)
    achieved = ops["simulate"] * n / (sim_ms * 1e-3)
    result = {
        "metric": "scenarios_per_sec",
        "value": n / (ms_per_step * 1e-3),
        "unit": "scenarios/s",
        "events_per_sec": n * 2 * D * C / (ms_per_step * 1e-3),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "kernel_ms": {"plan": plan_ms, "simulate": sim_ms, "step": step_ms,
                      "statistic": "median of the per-step HIP-event times"},
        "h2d_ms_once": h2d_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64", "data": "synthetic",
        "config": {"workload": "config3: %d scenarios, 4-D P=(2,8,8,64), C=64, "
                               "Themis+SCF, relative threshold U[0,0.1]" % n,
                   "outputs": "orders,loads,t_done,busy" + ("" if qo is None else ",queue_order"),
                   "chunk_stage_events_per_scenario": 2 * D * C},
        "roofline": {
            "bound": "alu", "kernel": "simulate",
            "achieved": achieved / 1e12, "peak": peak["lane_ops_per_s"] / 1e12,
            "unit": "Tlane-op/s", "frac": achieved / peak["lane_ops_per_s"],
            "algorithmic_lane_ops_per_scenario": ops["simulate"],
            "compute_units": peak["compute_units"], "clock_mhz_nominal": peak["clock_mhz_nominal"],
            # what follows was not measured in this run: counters of an earlier
            # rocprofv3 run of this file, with the commit they were taken on
            "traffic": prof.get("traffic_bytes_per_launch") if prof else None,
            "traffic_source": ("profiles/simulate_kernel_config3.md @ %s" % prof.get("commit", "?"))
                              if prof else None,
            "profiled": prof,
        },
    }

    # the fused sweep entry point on the same batch (times only), for reference
    thr = torch.full((1,), 1.0 / 16.0, dtype=torch.float64, device="cuda:0")
    sw_out = torch.empty((n, 1, 1), dtype=torch.float64, device="cuda:0")
    for _ in range(3):
        binding.themis_sweep(d, thr, workloads.SWEEP_THEMIS_SCF, t_done=sw_out)
    torch.cuda.synchronize()
    sw_ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
    for e in sw_ev:
        e[0].record()
        binding.themis_sweep(d, thr, workloads.SWEEP_THEMIS_SCF, t_done=sw_out)
        e[1].record()
    torch.cuda.synchronize()
    sweep_ms = median([e[0].elapsed_time(e[1]) for e in sw_ev])
    sw_ops = (ops["plan"] + ops["simulate"]) * n / (sweep_ms * 1e-3)
    result["sweep_times_only"] = {
        "ms": sweep_ms, "evaluations_per_sec": n / (sweep_ms * 1e-3),
        "events_per_sec": n * 2 * D * C / (sweep_ms * 1e-3),
        "roofline": {"bound": "alu", "kernel": "sweep", "achieved": sw_ops / 1e12,
                     "peak": peak["lane_ops_per_s"] / 1e12, "unit": "Tlane-op/s",
                     "frac": sw_ops / peak["lane_ops_per_s"], "traffic": None, "traffic_source": None}}

    if args.cpu_sample > 0:
        from oracle import themis_oracle
        m = min(args.cpu_sample, n)
        sample = host.take(slice(0, m))
        cores = min(os.cpu_count() or 1, 16, m)
        c0 = time.perf_counter()
        o_orders, _ = themis_oracle.plan_batch(sample, threads=cores)
        o_t, _, _ = themis_oracle.simulate_batch(sample, o_orders, want_queue_order=qo is not None,
                                                 threads=cores)
        cpu_s = time.perf_counter() - c0
        # parity spot check on the sample while we have both results
        g_t = t_done[:m].cpu().numpy()
        rel = float(np.max(np.abs(g_t - o_t) / o_t))
        same_orders = bool(np.array_equal(orders[:m].cpu().numpy(), o_orders))
        result["cpu_baseline"] = {
            "value": m / cpu_s, "unit": "scenarios/s", "cores": cores, "kind": "oracle",
            "sample": "first %d scenarios of the same batch, plan+simulate, %d threads, %.1f s"
                      % (m, cores, cpu_s),
            "parity_on_sample": {"orders_equal": same_orders, "t_done_max_rel_err": rel},
        }
        # the same oracle on one core, on a 1/16 sub-sample
        m1 = max(1, m // 16)
        one = host.take(slice(0, m1))
        c1 = time.perf_counter()
        o1, _ = themis_oracle.plan_batch(one, threads=1)
        themis_oracle.simulate_batch(one, o1, want_queue_order=qo is not None, threads=1)
        one_s = time.perf_counter() - c1
        result["cpu_baseline_single_core"] = {
            "value": m1 / one_s, "unit": "scenarios/s", "cores": 1, "kind": "oracle",
            "sample": "first %d scenarios, %.1f s" % (m1, one_s)}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
