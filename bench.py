#!/usr/bin/env python3
"""Benchmark of the ABS-SGD hot path on one MI355X.

A step is one iteration of Algorithm 1 as one GPU sees it: the fused
sync-update of the delayed generation (K accumulators -> x, v), Step 2 of the
K workers (sum_k m_k micro-batch gradients into the current generation), and
the swap.  Inputs are resident in HBM before the timed region starts.

Prints ONE JSON line: whole-step throughput of the headline workload, its
dominant kernel against the HBM roofline, a table over the five stated
configurations, and the CPU oracle timed on the same box.

How Step 2 is issued (--accumulate):
  calls   one abs_ctx_accumulate call, one launch, per micro-batch gradient: every gradient
          is folded in as it arrives, g_b + 8 bytes per parameter each (default: the path
          the metric's byte count describes);
  rounds  one abs_ctx_accumulate_step call per iteration with fold = 1: one launch per
          round of gradients (every worker that still has one contributes one), the same
          traffic in max_k m_k launches instead of sum_k m_k;
  step    the same call with fold = 8: a worker's gradients of the iteration are folded in
          together (m_k g_b + 8 bytes per parameter), normally ONE launch for all workers:
          fewer bytes and fewer launches, for callers that hold a step's gradients at once.
Every line prices its time with the algorithmic bytes of its own mode.
"""
import argparse
import gc
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak

METRIC = "sync-update+accumulate GB/s and % of HBM peak; params/s per step"

STATED = ["cfg1_small", "cfg2_resnet18", "cfg3_resnet50_bf16", "cfg4_vgg16", "cfg5_gpt2_ragged_bf16"]
# buffers of these workloads fit the 256 MiB memory-side cache wholly or in good part, so their
# algorithmic GB/s is not an HBM rate (it can exceed the box's plain-copy rate)
CACHE_ASSISTED = {"cfg1_small", "cfg2_resnet18", "cfg3_resnet50_bf16", "paper_static", "paper_dynamic",
                  "paper_static_dynamic"}

MAX_BATCH = 8   # ABS_MAX_BATCH: gradients one accumulate launch folds in per worker


def measured_traffic(workload, kernel):
    """HBM-side bytes per launch of `kernel` in `workload`, from profiles/traffic.json (written by
    the profile summaries from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command).
    Returns (bytes or None, where it came from)."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    if not os.path.exists(path):
        return None, "profiles/traffic.json is absent"
    with open(path) as fh:
        table = json.load(fh)
    for row in table.get("rows", []):
        if row["workload"] == workload and row["kernel"] == kernel:
            return row["bytes_per_launch"], {"file": "profiles/traffic.json", "summary": row.get("summary"),
                                             "counters": table.get("counters"), "level": table.get("level")}
    return None, f"no row for {kernel} in {workload} in profiles/traffic.json"


def bytes_per_param(w, m_row, mode, extra_state=False, lars=False):
    """Algorithmic bytes per parameter in one step with micro-batch counts m_row: (accumulate,
    sync-update).  A launch reads each of the gradients it folds in once and reads + writes the
    fp32 accumulator once (a worker's first launch of a step only writes it); the sync-update
    reads K accumulators and reads + writes x and v (and a third state vector for the stored-
    iterate compensation and for Adam)."""
    gb = 4 if w.grad_dtype == "f32" else 2
    if mode in ("step", "batched"):
        acc = sum(int(m) * gb + 8 * (-(-int(m) // MAX_BATCH)) - 4 for m in m_row if m > 0)
    else:
        acc = sum(int(m) * (gb + 8) - 4 for m in m_row if m > 0)
    if lars:
        # K accumulators + x read, Gbar written; then Gbar, x, v read and x, v written
        return acc, (4 * w.K + 8) + 20
    return acc, 4 * w.K + 16 + (8 if extra_state else 0)


def dominant_kernel(w, mode):
    """The accumulate kernel: it moves most of a step's bytes in every workload.  Template
    arguments: bf16 gradients, streaming flavour, (most) gradients per launch and worker."""
    bf = "true" if w.grad_dtype == "bf16" else "false"
    kind = "ragged" if w.tensor_sizes is not None else "flat"
    if mode in ("step", "rounds"):
        return f"absk::accumulate_jobs_{kind}<{bf}, *, {'1' if mode == 'rounds' else '*'}>"
    return f"absk::accumulate_{kind}<{bf}, *, {'*' if mode == 'batched' else '1'}>"


def timed_region(run, plans, t0, steps, torch):
    """EXACTLY `steps` steps between two device synchronisations.  Returns (wall seconds,
    seconds the host needed to enqueue them)."""
    torch.cuda.synchronize()
    gc.disable()                       # a collection between two launches would idle the GPU for milliseconds
    try:
        t_start = time.perf_counter()
        for t in range(t0, t0 + steps):
            run.step(t, plans[t])
        t_issued = time.perf_counter()
        torch.cuda.synchronize()
        return time.perf_counter() - t_start, t_issued - t_start
    finally:
        gc.enable()


def kernel_event_pass(run, plans, t0, steps, torch):
    """Replay the timed steps on ONE stream with a HIP event pair per step around that step's
    accumulate launches and one around its sync-update launch, recorded on the stream the
    kernels run on.  Returns per step: accumulate bracket ms, the kernel launches in it (the
    library's own count: a long call goes in several launches), sync-update bracket ms (None for
    a step that applied nothing) and the kernel launches of that call."""
    import paper_2308_15164_amd as absgd
    ev = lambda: torch.cuda.Event(enable_timing=True)
    rows = []
    torch.cuda.synchronize()
    for t in range(t0, t0 + steps):
        es, e0, e1 = ev(), ev(), ev()
        n0 = absgd.abs_launch_count()
        es.record(run.s_acc)
        applied = run.sync_update()
        e0.record(run.s_acc)
        n1 = absgd.abs_launch_count()
        run.accumulate(plans[t])
        e1.record(run.s_acc)
        n2 = absgd.abs_launch_count()
        run.ctx.abs_swap_buffers()
        rows.append((e0, e1, n2 - n1, (es, e0) if applied else None, n1 - n0))
    torch.cuda.synchronize()
    return [(a.elapsed_time(b), n, s[0].elapsed_time(s[1]) if s else None, ns) for a, b, n, s, ns in rows]


def probe_ceilings(torch, Ks=(), nbytes=4 * 138_357_544, reps=20):
    """Copy / read / write / triad (two reads and one write in place: the steady accumulate's
    mix) rates of plain streaming kernels on this machine, and for each K in Ks a plain kernel with
    the sync-update's traffic (K + 2 vectors read, two of them written in place) and the same
    K + 2 vectors only read (what mixing a write stream into the reads costs).  Context for the
    roofline fractions; not part of the method.  Every vector is as long as the VGG16-sized
    parameter vector (553 MB): power-of-two sizes put all streams on the same DRAM banks at
    the same time and read 2-5 % low.  A probe is launched over sub-ranges, one launch per GiB
    moved, as the library cuts its own long calls (multi-GB launches run 4-7 % slower)."""
    import ctypes
    path = os.path.join(ROOT, "bench_probe", "libabs_probe.so")
    if not os.path.exists(path):
        return None
    L = ctypes.CDLL(path)
    vp, i64 = ctypes.c_void_p, ctypes.c_int64
    L.probe_copy.argtypes = [vp, vp, i64, vp]
    L.probe_read.argtypes = [vp, i64, vp, vp]
    L.probe_write.argtypes = [vp, i64, ctypes.c_float, vp]
    L.probe_triad.argtypes = [vp, vp, i64, ctypes.c_float, vp]
    a = torch.ones(nbytes // 4, device="cuda")
    b = torch.ones(nbytes // 4, device="cuda")
    sink = torch.zeros(4, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    out = {}

    def cuts(moved):
        """Sub-ranges of a vector, so that a probe is launched the way the library launches its own
        kernels: one launch per GiB moved (one below two), cut at multiples of 16 KiB."""
        n = max(1, moved // (1 << 30))
        edges = [(nbytes * i // n) // 16384 * 16384 for i in range(n)] + [nbytes]
        return [(edges[i], edges[i + 1] - edges[i]) for i in range(n)]

    def timed(fn, moved, warm=3):
        for i in range(warm):
            fn(i)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(reps):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return moved * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9

    pa, pb = a.data_ptr(), b.data_ptr()
    for name, one, moved in (("copy", lambda o, n: L.probe_copy(pa + o, pb + o, n, st), 2 * nbytes),
                             ("read", lambda o, n: L.probe_read(pa + o, n, sink.data_ptr(), st), nbytes),
                             ("write", lambda o, n: L.probe_write(pa + o, n, 1.0, st), nbytes),
                             ("triad", lambda o, n: L.probe_triad(pa + o, pb + o, n, 0.5, st), 3 * nbytes)):
        parts = cuts(moved)

        def fn(i, one=one, parts=parts):
            for o, n in parts:
                assert one(o, n) == 0
        out[name + "_GBs"] = timed(fn, moved)
    del a, b
    L.probe_mix.argtypes = [ctypes.POINTER(vp), ctypes.c_int, i64, vp]
    L.probe_readk.argtypes = [ctypes.POINTER(vp), ctypes.c_int, i64, vp, vp]
    for K in sorted(set(k for k in Ks if k in (4, 8, 16))):
        R = K + 2
        bufs = [torch.zeros(nbytes // 4, device="cuda") for _ in range(2 * R)]      # two sets, used in turn
        for name, moved, call in ((f"mix_{K}_workers_GBs", (R + 2) * nbytes,
                                   lambda ptrs, n: L.probe_mix(ptrs, R, n, st)),
                                  (f"read_only_{K}_workers_GBs", R * nbytes,
                                   lambda ptrs, n: L.probe_readk(ptrs, R, n, sink.data_ptr(), st))):
            parts = [[((vp * R)(*[t.data_ptr() + o for t in bufs[i * R:(i + 1) * R]]), n) for o, n in cuts(moved)]
                     for i in range(2)]

            def fn(i, call=call, parts=parts):
                for ptrs, n in parts[i % 2]:
                    assert call(ptrs, n) == 0
            out[name] = timed(fn, moved, warm=4)
        del bufs
    return out


def calibrate_copy(torch, nbytes=1 << 30, reps=10):
    """Only a plain copy of known size, for scaling the profiler's byte counters."""
    import ctypes
    L = ctypes.CDLL(os.path.join(ROOT, "bench_probe", "libabs_probe.so"))
    L.probe_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
    a = torch.ones(nbytes // 4, device="cuda")
    b = torch.ones(nbytes // 4, device="cuda")
    torch.cuda.synchronize()
    for _ in range(reps):
        L.probe_copy(a.data_ptr(), b.data_ptr(), nbytes, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    print(json.dumps({"calibration": "probe_copy_kernel", "bytes_read_per_launch": nbytes,
                      "bytes_written_per_launch": nbytes, "launches": reps}))


def _oracle_steps(orc, wl, w, x0, pool, sched, budget_s, mode):
    """Whole steps of the workload through the oracle until budget_s of wall time is spent."""
    import numpy as np
    P, K = x0.size, w.K
    x = x0.astype(np.float64)
    v = np.zeros(P)
    G = [[np.zeros(P) for _ in range(K)] for _ in range(2)]
    M = [[0] * K for _ in range(2)]
    cur, prev = 0, 1
    R = len(pool)
    done_bytes, done_steps, own_bytes = 0, 0, 0
    t_start = time.perf_counter()
    t = -1
    while True:
        t = (t + 1) % sched.shape[0]
        for i in range(K):
            orc.zero(G[cur][i])
            M[cur][i] = 0
            for j in range(int(sched[t, i])):
                orc.accumulate(G[cur][i], pool[wl.pool_index(w, t, i, j, R)], w.n)
                M[cur][i] += w.n
        orc.sync_update(x, v, G[prev], M[prev], w.lr, w.mu, w.wd)
        cur, prev = prev, cur
        a, s = bytes_per_param(w, sched[t], mode)
        done_bytes += (a + s) * P
        # what the oracle itself moves: double accumulators (zero pass, then read + write per
        # reference batch), all K of them read by the update, x and v in double
        gb = 4 if w.grad_dtype == "f32" else 2
        own_bytes += (8 * K + sum(int(m) for m in sched[t]) * (gb + 16) + 8 * K + 32) * P
        done_steps += 1
        if time.perf_counter() - t_start > budget_s:
            break
    return done_bytes, done_steps, time.perf_counter() - t_start, own_bytes


def cpu_baseline(w, x0, pool, sched, mode, budget_s=10.0):
    """The oracle as it stands, on the host cores, on a bounded run of the same workload: whole
    steps at full P, about budget_s of wall time with every core the box gives the process
    (OpenMP over the parameter index), then a few seconds on one thread."""
    import abs_workloads as wl
    from oracle import abs_oracle as orc

    threads = orc.max_threads()
    P = x0.size
    nbytes, steps, dt, own = _oracle_steps(orc, wl, w, x0, pool, sched, budget_s, mode)
    orc.set_threads(1)
    b1, s1, dt1, _ = _oracle_steps(orc, wl, w, x0, pool, sched, budget_s / 4, mode)
    orc.set_threads(threads)
    return {"value": nbytes / dt / 1e9, "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": f"{steps} whole steps of {w.name} at full P={P} (same inputs and m_k), "
                      f"{dt:.1f} s wall, OpenMP over the parameter index",
            "ms_per_step": dt / steps * 1e3, "params_per_s": P * steps / dt,
            # `value` prices the oracle's time with the same algorithmic bytes as the GPU line;
            # this is the oracle's own traffic
            "own_bytes_GBs": own / dt / 1e9,
            "single_thread": {"value": b1 / dt1 / 1e9, "unit": "GB/s", "ms_per_step": dt1 / s1 * 1e3,
                              "sample": f"{s1} whole steps, {dt1:.1f} s wall"}}


def stream_plans(absgd, w, mode, only=None):
    """(name, sync-update on a stream of its own, accumulate streams) to time, and the name of
    the plan whose time is `value`: the one the library's own rule names for this size."""
    plans = [("one stream", False, 1), ("accumulate | sync-update", True, 1)]
    if mode in ("calls", "batched"):
        for n in (2, 4):
            if n <= w.K:
                plans.append((f"{n} accumulate streams (workers balanced over them) | sync-update", True, n))
        n_sug = absgd.abs_suggest_accumulate_streams(w.P, w.K)
        chosen = "one stream" if n_sug == 1 else next(p[0] for p in plans if p[2] == n_sug)
    else:
        chosen = "one stream"          # a step call keeps all workers on one stream; two streams cannot add bandwidth
    if only is not None:
        plans = [p for p in plans if p[0] in only or p[0] == chosen]
    return plans, chosen


_INPUTS = {}     # workload name -> (x0, gradient pool) on the host


def measure(torch, absgd, wl, w, args, mode, K_steps, W, repeats, all_plans=True, variant=None):
    """Everything measured for one workload and one way of issuing Step 2."""
    from paper_2308_15164_amd.driver import DeviceRun
    variant = variant or {}
    total = W + K_steps
    sched = wl.schedule(w, total)
    if w.name not in _INPUTS:
        _INPUTS.clear()                                          # one workload's host arrays at a time
        # at least as many distinct gradient vectors as any worker folds in per step: no launch
        # reads one vector twice
        _INPUTS[w.name] = (wl.initial_params(w), wl.gradient_pool(w, pool=max(args.pool, int(sched.max()))))
    x0, pool = _INPUTS[w.name]
    lam = variant.get("lam")
    dcm = lam is not None and variant.get("dcm", False)
    adam, lars = variant.get("adam"), variant.get("lars")
    run = DeviceRun(w, x0, pool, sched, overlap=False, lam=lam, batched=(mode == "batched"),
                    lam_from_momentum=dcm, adam=adam, lars=lars,
                    step_fold={"step": MAX_BATCH, "rounds": 1}.get(mode))
    if adam:
        run.lr = 1e-3
    extra = (lam is not None and not dcm) or adam is not None      # a third state vector is moved
    calls = [run.plan_step(t) for t in range(total)]
    plans, chosen = stream_plans(absgd, w, mode, None if all_plans else ("one stream",))
    timings, issue = {}, {}
    for name, overlap, n_acc in plans:
        run.configure_streams(overlap, n_acc)
        timed_region(run, calls, 0, max(W, 3), torch)          # warm-up; also refills the delayed generation
        reps = [timed_region(run, calls, W, K_steps, torch) for _ in range(repeats)]
        timings[name] = [r[0] for r in reps]
        issue[name] = statistics.median(r[1] for r in reps)
    med = {k: statistics.median(v) for k, v in timings.items()}
    dt = med[chosen]
    fastest = min(med, key=med.get)

    # the kernels alone on the GPU: one stream, same steps, one event bracket per step and kernel
    run.configure_streams(False, 1)
    timed_region(run, calls, 0, max(W, 3), torch)
    rows = []
    for _ in range(repeats):
        rows += kernel_event_pass(run, calls, W, K_steps, torch)
    run.close()
    del run, calls
    torch.cuda.empty_cache()

    P = w.P
    bpp = [bytes_per_param(w, sched[t], mode, extra, lars is not None) for t in range(W, total)]
    step_bytes = sum((a + s) * P for a, s in bpp)
    acc_bytes = [a * P for a, _ in bpp] * repeats
    gbs = step_bytes / dt / 1e9
    launches = sum(r[1] for r in rows)
    kern_ms = sum(r[0] for r in rows) / launches
    kern_bytes = sum(acc_bytes) / launches
    achieved = kern_bytes / (kern_ms * 1e-3) / 1e9
    per_step_rate = [b / (r[0] * 1e-3) / 1e9 for b, r in zip(acc_bytes, rows)]
    sync_ms = [r[2] for r in rows if r[2] is not None]
    sync_launches = [r[3] for r in rows if r[2] is not None]
    sync_bytes = bpp[0][1] * P
    sync_med = statistics.median(sync_ms)
    sync_gbs = sync_bytes / (sync_med * 1e-3) / 1e9
    kname = dominant_kernel(w, mode)
    traffic, traffic_src = measured_traffic(w.name, kname)
    res = {
        "workload": w.name, "P": P, "K": w.K, "grad_dtype": w.grad_dtype, "accumulate": mode,
        "value": gbs, "pct_of_8TBs": 100.0 * gbs / HBM_PEAK_GBS,
        "ms_per_step": dt / K_steps * 1e3,
        "ms_per_step_repeats": [t / K_steps * 1e3 for t in timings[chosen]],
        "params_per_s": P * K_steps / dt,
        "algorithmic_bytes_per_step": step_bytes // K_steps,
        "plan": chosen,
        "ms_per_step_by_stream_plan": {k: v / K_steps * 1e3 for k, v in med.items()},
        "fastest_plan": {"name": fastest, "faster_than_chosen_by": med[chosen] / med[fastest] - 1.0},
        "overlap_speedup": med["one stream"] / min(v for k, v in med.items() if k != "one stream")
        if len(med) > 1 else None,
        "host_issue_ms_per_step": issue[chosen] / K_steps * 1e3,
        "cache_assisted": w.name in CACHE_ASSISTED,
        "accumulate_kernel": {
            "kernel": kname, "achieved": achieved, "frac": achieved / HBM_PEAK_GBS,
            "algorithmic_bytes_per_launch": kern_bytes, "avg_launch_ms": kern_ms,
            "launches_timed": launches, "launches_per_step": launches / len(rows),
            "median_step_rate": statistics.median(per_step_rate),
            "min_step_rate": min(per_step_rate), "max_step_rate": max(per_step_rate),
            "traffic": traffic, "traffic_source": traffic_src,
        },
        "sync_update_kernel": {
            "achieved": sync_gbs, "frac": sync_gbs / HBM_PEAK_GBS,
            "algorithmic_bytes_per_launch": sync_bytes, "median_launch_ms": sync_med,
            "min_launch_ms": min(sync_ms), "max_launch_ms": max(sync_ms), "launches_timed": len(sync_ms),
            # a call over several GB goes in several kernel launches over consecutive ranges
            "kernel_launches_per_call": sum(sync_launches) / len(sync_launches),
        },
    }
    return res, (x0, pool, sched)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--repeats", type=int, default=5, help="timed regions of --steps steps; the median is reported")
    ap.add_argument("--workload", default="cfg4_vgg16")
    ap.add_argument("--accumulate", default="calls", choices=["step", "rounds", "calls", "batched"],
                    help="how Step 2 is issued (see the module docstring); batched = one "
                         "abs_ctx_accumulate_batch call per worker")
    ap.add_argument("--pool", type=int, default=8, help="distinct gradient vectors resident in HBM")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-table", action="store_true", help="skip the table over the five stated configurations")
    ap.add_argument("--no-variants", action="store_true", help="skip the other ways of issuing Step 2")
    ap.add_argument("--only-chosen-plan", action="store_true",
                    help="time only the stream plan `value` comes from (with one stream, every kernel of the "
                         "command then runs alone on the GPU: what a profiler run wants)")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the plain streaming kernels (box_ceilings)")
    ap.add_argument("--cache-policy", default="-1,-1",
                    help="accumulate,update: -1 auto, 0 cached, 1 streaming (see abs_set_cache_policy)")
    ap.add_argument("--launch-tuning", default=None,
                    help="blocks_per_cu,max_rows_per_tile (see abs_set_launch_tuning); default: the library's")
    ap.add_argument("--compensation", type=float, default=None, metavar="LAMBDA",
                    help="also apply the delayed gradient compensation with this coefficient "
                         "(abs_sync_update_dc; +8 B/param); default: off, the four-part path of the headline metric")
    ap.add_argument("--compensation-from-momentum", action="store_true",
                    help="with --compensation: take x_t - x_{t-1} from the momentum (abs_sync_update_dcm; "
                         "no x_{t-1} buffer, no extra bytes)")
    ap.add_argument("--adam", action="store_true",
                    help="Adam (beta 0.9/0.999, eps 1e-8, lr 1e-3) as the update rule instead of momentum SGD "
                         "(abs_sync_update_adam; +8 B/param)")
    ap.add_argument("--lars", action="store_true",
                    help="LARS (trust 0.001) per tensor as the update rule (abs_sync_update_lars_mt; ragged "
                         "workloads only; 4K + 28 B/param)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run only a plain 1 GiB copy kernel (profiler counter calibration)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU: the K workers are K device-resident buffers and "
              "there are no collectives; --gpus must be 1", file=sys.stderr)
        return 2

    import torch
    import abs_workloads as wl
    import paper_2308_15164_amd as absgd

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    absgd.lib()
    if args.calibrate_copy:
        calibrate_copy(torch)
        return 0
    absgd.abs_set_cache_policy(*[int(v) for v in args.cache_policy.split(",")])
    if args.launch_tuning:
        absgd.abs_set_launch_tuning(*[int(v) for v in args.launch_tuning.split(",")])

    w = wl.WORKLOADS[args.workload]
    W, K_steps, R = args.warmup, args.steps, max(1, args.repeats)
    variant = {"lam": args.compensation, "dcm": args.compensation_from_momentum,
               "adam": (0.9, 0.999, 1e-8) if args.adam else None, "lars": 0.001 if args.lars else None}
    plain = args.compensation is None and not args.adam and not args.lars
    mode = args.accumulate

    head, (x0, pool, sched) = measure(torch, absgd, wl, w, args, mode, K_steps, W, R, variant=variant,
                                      all_plans=not args.only_chosen_plan)
    ak, sk = head["accumulate_kernel"], head["sync_update_kernel"]

    out = {
        "metric": METRIC,
        "value": head["value"],
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": K_steps,
        "warmup": W,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": w.name, "P": w.P, "K": w.K, "grad_dtype": w.grad_dtype,
            "samples_per_microbatch": w.n, "m_k": w.schedule + (str(list(w.ratio)) if w.ratio else ""),
            "tensors": 1 if w.tensor_sizes is None else len(w.tensor_sizes),
            "lr": w.lr, "mu": w.mu, "wd": w.wd, "gradient_pool": len(pool),
            "accumulate": mode, "compensation_lambda": args.compensation,
            "compensation_from_momentum": variant["dcm"] and args.compensation is not None,
            "update_rule": "adam" if args.adam else ("lars" if args.lars else "momentum sgd"),
            "streams": head["plan"] + ", double-buffered",
            "algorithmic_bytes_per_step": head["algorithmic_bytes_per_step"],
        },
        "timing": f"median of {R} timed regions of exactly {K_steps} steps, each between two device "
                  f"synchronisations, after {max(W, 3)} warm-up steps; kernel figures from HIP events on the "
                  f"kernels' own stream over the same steps x {R}",
        "repeats": R,
        "ms_per_step_repeats": head["ms_per_step_repeats"],
        # algorithmic bytes / time as a share of the published 8 TB/s; an HBM rate only where the
        # buffers exceed the memory-side cache (cache_assisted false)
        "pct_of_8TBs": head["pct_of_8TBs"],
        "cache_assisted": head["cache_assisted"],
        "params_per_s": head["params_per_s"],
        "overlap_speedup": head["overlap_speedup"],
        "ms_per_step_by_stream_plan": head["ms_per_step_by_stream_plan"],
        "fastest_plan": head["fastest_plan"],
        # time the host needed to enqueue a step (binding + launches + event joins): when it
        # approaches ms_per_step the workload is bound by launches, not by the kernels
        "host_issue_ms_per_step": head["host_issue_ms_per_step"],
        "roofline": {
            "bound": "hbm", "kernel": ak["kernel"], "achieved": ak["achieved"], "peak": HBM_PEAK_GBS,
            "unit": "GB/s", "frac": ak["frac"], "traffic": ak["traffic"], "traffic_source": ak["traffic_source"],
            "algorithmic_bytes_per_launch": ak["algorithmic_bytes_per_launch"],
            "avg_launch_ms": ak["avg_launch_ms"], "launches_timed": ak["launches_timed"],
            "launches_per_step": ak["launches_per_step"],
            "step_rate_GBs": {"median": ak["median_step_rate"], "min": ak["min_step_rate"],
                              "max": ak["max_step_rate"]},
            "measured": "HIP events around each step's accumulate launches on their stream, one-stream plan "
                        "(the kernel alone on the GPU), every timed step of every repeat, no step left out; "
                        "launches are kernel launches as the library counts them (abs_launch_count)",
        },
        "sync_update_kernel": dict(sk, unit="GB/s",
                                   measured="HIP events around the sync-update CALL of each step (its kernel "
                                            "launches: kernel_launches_per_call, consecutive ranges of one pass), "
                                            "one-stream plan; a bracket around one call also holds a few us of "
                                            "dispatch latency, so this is a lower bound on the kernels' rate (the "
                                            "kernel trace under profiles/ has their own durations)"),
    }

    table_Ks = {w.K}
    if plain and not args.no_variants:
        # the same workload with Step 2 issued the other ways (each priced with its own algorithmic bytes)
        out["accumulate_variants"] = {}
        for m in ("step", "rounds", "calls"):
            if m == mode:
                r = head
            else:
                r, _ = measure(torch, absgd, wl, w, args, m, K_steps, W, max(3, R // 2 + 1), all_plans=(m == "calls"))
            out["accumulate_variants"][m] = {
                k: r[k] for k in ("value", "pct_of_8TBs", "ms_per_step", "params_per_s", "plan",
                                  "algorithmic_bytes_per_step", "host_issue_ms_per_step")}
            out["accumulate_variants"][m]["accumulate_kernel_frac"] = r["accumulate_kernel"]["frac"]
            out["accumulate_variants"][m]["launches_per_step"] = (r["accumulate_kernel"]["launches_per_step"] +
                                                                  r["sync_update_kernel"]["kernel_launches_per_call"])
    if plain and not args.no_table:
        def row(r):
            return {"value": r["value"], "pct_of_8TBs": r["pct_of_8TBs"], "ms_per_step": r["ms_per_step"],
                    "params_per_s": r["params_per_s"], "plan": r["plan"],
                    "algorithmic_bytes_per_step": r["algorithmic_bytes_per_step"],
                    "accumulate_frac": r["accumulate_kernel"]["frac"], "sync_update_frac": r["sync_update_kernel"]["frac"],
                    "accumulate_launch_ms": r["accumulate_kernel"]["avg_launch_ms"],
                    "sync_update_launch_ms": r["sync_update_kernel"]["median_launch_ms"],
                    "launches_per_step": r["accumulate_kernel"]["launches_per_step"] + r["sync_update_kernel"]["kernel_launches_per_call"],
                    "host_issue_ms_per_step": r["host_issue_ms_per_step"]}
        out["per_config"] = {}
        for name in STATED:
            wc = wl.WORKLOADS[name]
            table_Ks.add(wc.K)
            r = head if name == w.name else measure(torch, absgd, wl, wc, args, mode, min(K_steps, 20), W, R,
                                                    all_plans=False)[0]
            entry = dict(row(r), P=wc.P, K=wc.K, grad_dtype=wc.grad_dtype, accumulate=mode,
                         cache_assisted=r["cache_assisted"])
            if mode != "step":
                # the same configuration with Step 2 as one job-list call per iteration
                rs = measure(torch, absgd, wl, wc, args, "step", min(K_steps, 20), W, R, all_plans=False)[0]
                entry["one_call_per_step"] = dict(row(rs), step_time_vs_separate_calls=rs["ms_per_step"] / r["ms_per_step"])
            out["per_config"][name] = entry

    ceil = None if args.no_ceilings else probe_ceilings(torch, table_Ks)
    out["box_ceilings"] = ceil
    if ceil:
        out["pct_of_box_copy_rate"] = 100.0 * head["value"] / ceil["copy_GBs"]
        out["pct_of_box_read_rate"] = 100.0 * head["value"] / ceil["read_GBs"]
        out["roofline"]["frac_of_box_triad"] = ak["achieved"] / ceil["triad_GBs"]
        mix = ceil.get(f"mix_{w.K}_workers_GBs")
        if mix:
            out["sync_update_kernel"]["frac_of_box_mix"] = sk["achieved"] / mix
        for name, row in out.get("per_config", {}).items():
            row["pct_of_box_copy"] = 100.0 * row["value"] / ceil["copy_GBs"]
            row["accumulate_vs_box_triad"] = row["accumulate_frac"] * HBM_PEAK_GBS / ceil["triad_GBs"]
            mix = ceil.get(f"mix_{row['K']}_workers_GBs")
            if mix:
                row["sync_update_vs_box_mix"] = row["sync_update_frac"] * HBM_PEAK_GBS / mix
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, x0, pool, sched[W:], mode)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
