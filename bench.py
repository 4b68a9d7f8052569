#!/usr/bin/env python3
"""Benchmark of the ABS-SGD hot path on one MI355X.

A step is one iteration of Algorithm 1 as one GPU sees it: the fused
sync-update of the delayed generation (K accumulators -> x, v) on one stream,
sum_k m_k accumulate calls into the current generation on another, and the
swap.  Inputs are resident in HBM before the timed region starts.

Prints ONE JSON line: whole-step throughput under the fastest stream plan, the dominant
kernel against the HBM roofline, and the CPU oracle timed on the same box.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak

METRIC = "sync-update+accumulate GB/s and % of HBM peak; params/s per step"

# HBM bytes per launch of the dominant kernel, from rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE runs of this same command, scaled by what the same counters read
# for a plain copy of known size (summaries under profiles/).  None = not measured.
MEASURED_TRAFFIC = {
    # FETCH_SIZE x 2.000 = 81.88 MB, WRITE_SIZE x 1.000 = 46.75 MB per launch (average over
    # the 12 read-modify-write and 4 overwrite launches of a step)
    ("cfg2_resnet18", "absk::accumulate_flat<false, *, 1>"): 128.63e6,
    # cfg4: 923.7 MB fetched + 553.4 MB written per launch (schedule average)
    ("cfg4_vgg16", "absk::accumulate_flat<false, *, 1>"): 1477.1e6,
}


MAX_BATCH = 8   # ABS_MAX_BATCH: gradients one accumulate launch folds in


def bytes_per_param(w, m_row, extra_state=False, batched=False, lars=False):
    """Algorithmic bytes per parameter in one step with micro-batch counts m_row:
    an accumulate reads one gradient element and reads+writes one fp32
    accumulator element (the first call of a step only writes it); the
    sync-update reads K accumulators and reads+writes x and v (and the previous
    iterate when the delayed gradient compensation is on)."""
    gb = 4 if w.grad_dtype == "f32" else 2
    if batched:
        # a worker's m gradients go in ceil(m / MAX_BATCH) launches: every gradient is read
        # once, the accumulator is written once per launch and read by all but the first
        acc = sum(int(m) * gb + 8 * (-(-int(m) // MAX_BATCH)) - 4 for m in m_row)
    else:
        acc = sum(int(m) * (gb + 8) - 4 for m in m_row)
    if lars:
        # K accumulators + x read, Gbar written; then Gbar, x, v read and x, v written
        return acc, (4 * w.K + 8) + 20
    return acc, 4 * w.K + 16 + (8 if extra_state else 0)


def accumulate_launches(m_row, batched):
    return sum(-(-int(m) // MAX_BATCH) if batched else int(m) for m in m_row)


def dominant_kernel(w, batched=False):
    """The accumulate kernel: it moves most of a step's bytes in every workload.
    Template arguments: bf16 gradients, streaming flavour, gradients per launch."""
    bf = "true" if w.grad_dtype == "bf16" else "false"
    kind = "ragged" if w.tensor_sizes is not None else "flat"
    return f"absk::accumulate_{kind}<{bf}, *, {'*' if batched else '1'}>"


HOST_ISSUE = {}    # seconds the host needed to enqueue the last timed region's steps


def time_steps(run, plans, t0, steps, torch, tag=None):
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for t in range(t0, t0 + steps):
        run.step(t, plans[t])
    t_issued = time.perf_counter()
    torch.cuda.synchronize()
    if tag is not None:
        HOST_ISSUE[tag] = t_issued - t_start
    return time.perf_counter() - t_start


def kernel_event_pass(run, plans, t0, steps, torch):
    """Replay the timed steps with ONE HIP event pair per step around that step's
    whole sequence of accumulate launches, recorded on the stream they run on
    (launches on one stream run back to back, so the bracket divided by the
    number of launches is the average launch duration; one pair per ~16
    launches keeps the events' own cost below 1 %).  The sync-update of the
    step runs concurrently on the other stream, as in the timed region."""
    ctx, n, gdt = run.ctx, run.w.n, run.gdt
    pairs, launches, sync_pairs = [], [], []
    torch.cuda.synchronize()
    for t in range(t0, t0 + steps):
        es = torch.cuda.Event(enable_timing=True)
        es.record(run.s_acc)
        applied = run.sync_update()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record(run.s_acc)
        if run.batched:
            per_worker = {}
            for k, g in plans[t]:
                per_worker.setdefault(k, []).append(g)
            for k, gs in per_worker.items():
                ctx.abs_accumulate_batch(k, gs, [n] * len(gs), grad_dtype=gdt)
            launches.append(sum(-(-len(gs) // MAX_BATCH) for gs in per_worker.values()))
        else:
            for k, g in plans[t]:
                ctx.abs_accumulate(k, g, n, grad_dtype=gdt)
            launches.append(len(plans[t]))
        e1.record(run.s_acc)
        pairs.append((e0, e1))
        if applied:
            sync_pairs.append((es, e0))      # one stream: the sync-update sits between these two
        ctx.abs_swap_buffers()
    torch.cuda.synchronize()
    return [a.elapsed_time(b) for a, b in pairs], launches, [a.elapsed_time(b) for a, b in sync_pairs]


def probe_ceilings(torch, K=None, nbytes=1 << 30, reps=20):
    """Copy / read / write / triad (a += s*b: the accumulate's two reads and one
    write) rates of plain streaming kernels on this machine (context for the roofline
    fraction; not part of the method)."""
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
    for name, fn, moved in (("copy", lambda: L.probe_copy(a.data_ptr(), b.data_ptr(), nbytes, st), 2 * nbytes),
                            ("read", lambda: L.probe_read(a.data_ptr(), nbytes, sink.data_ptr(), st), nbytes),
                            ("write", lambda: L.probe_write(a.data_ptr(), nbytes, 1.0, st), nbytes),
                            ("triad", lambda: L.probe_triad(a.data_ptr(), b.data_ptr(), nbytes, 0.0, st), 3 * nbytes)):
        for _ in range(3):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        out[name + "_GBs"] = moved * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9
    if K in (4, 8, 16):
        # a plain kernel with the sync-update's traffic: K + 2 vectors read, two of them written
        del a, b
        R, nb = K + 2, 1 << 28
        L.probe_mix.argtypes = [ctypes.POINTER(vp), ctypes.c_int, i64, vp]
        bufs = [torch.zeros(nb // 4, device="cuda") for _ in range(2 * R)]      # two sets, used in turn
        sets = [(vp * R)(*[t.data_ptr() for t in bufs[i * R:(i + 1) * R]]) for i in range(2)]
        for i in range(4):
            assert L.probe_mix(sets[i % 2], R, nb, st) == 0
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(reps):
            L.probe_mix(sets[i % 2], R, nb, st)
        e1.record()
        torch.cuda.synchronize()
        out[f"mix_{K}_workers_GBs"] = (R + 2) * nb * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9
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


def _oracle_steps(orc, wl, w, x0, pool, sched, budget_s, comp=False):
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
        a, s = bytes_per_param(w, sched[t])
        done_bytes += (a + s) * P
        # what the oracle itself moves: double accumulators (zero pass, then read + write per
        # reference batch), all K of them read by the update, x and v in double
        gb = 4 if w.grad_dtype == "f32" else 2
        own_bytes += (8 * K + sum(int(m) for m in sched[t]) * (gb + 16) + 8 * K + 32) * P
        done_steps += 1
        if time.perf_counter() - t_start > budget_s:
            break
    return done_bytes, done_steps, time.perf_counter() - t_start, own_bytes


def cpu_baseline(w, x0, pool, sched, budget_s=10.0):
    """The oracle as it stands, on the host cores, on a bounded run of the same
    workload: whole steps at full P, about budget_s of wall time with every core the
    box gives the process (OpenMP over the parameter index), then a few seconds on
    one thread."""
    import abs_workloads as wl
    from oracle import abs_oracle as orc

    threads = orc.max_threads()
    P = x0.size
    nbytes, steps, dt, own = _oracle_steps(orc, wl, w, x0, pool, sched, budget_s)
    orc.set_threads(1)
    b1, s1, dt1, _ = _oracle_steps(orc, wl, w, x0, pool, sched, budget_s / 4)
    orc.set_threads(threads)
    return {"value": nbytes / dt / 1e9, "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": f"{steps} whole steps of {w.name} at full P={P} (same inputs and m_k), "
                      f"{dt:.1f} s wall, OpenMP over the parameter index",
            "ms_per_step": dt / steps * 1e3, "params_per_s": P * steps / dt,
            # `value` uses the method's algorithmic bytes (as for the GPU); this is the oracle's own traffic
            "own_bytes_GBs": own / dt / 1e9,
            "single_thread": {"value": b1 / dt1 / 1e9, "unit": "GB/s", "ms_per_step": dt1 / s1 * 1e3,
                              "sample": f"{s1} whole steps, {dt1:.1f} s wall"}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg2_resnet18")
    ap.add_argument("--pool", type=int, default=8, help="distinct gradient vectors resident in HBM")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cache-policy", default="-1,-1",
                    help="accumulate,update: -1 auto, 0 cached, 1 streaming (see abs_set_cache_policy)")
    ap.add_argument("--launch-tuning", default=None,
                    help="blocks_per_cu,max_rows_per_tile (see abs_set_launch_tuning); default: the library's")
    ap.add_argument("--acc-streams", type=int, default=1,
                    help="streams the K workers' accumulations are spread over")
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
    ap.add_argument("--batched", action="store_true",
                    help="one abs_accumulate_batch call per worker and step instead of one abs_accumulate "
                         "per micro-batch (fewer bytes: the accumulator is read and written once)")
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
    from paper_2308_15164_amd.driver import DeviceRun

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
    W, K_steps = args.warmup, args.steps
    total = W + K_steps
    x0 = wl.initial_params(w)
    pool = wl.gradient_pool(w, pool=args.pool)
    sched = wl.schedule(w, total)

    # Stream plans.  The double buffer is in use in all of them; they differ in which
    # HIP streams carry the work.  Each plan is warmed up and timed over the same K steps.
    plans_wanted = [("one stream", False, 1), ("accumulate | sync-update", True, 1)]
    for n in (2, 4):
        if n <= w.K:
            plans_wanted.append((f"{n} accumulate streams (workers balanced over them) | sync-update", True, n))
    if args.acc_streams > 1:
        plans_wanted = [p for p in plans_wanted if p[2] in (1, args.acc_streams)]
    dcm = args.compensation is not None and args.compensation_from_momentum
    run = DeviceRun(w, x0, pool, sched, overlap=False, lam=args.compensation, batched=args.batched,
                    lam_from_momentum=dcm,
                    adam=(0.9, 0.999, 1e-8) if args.adam else None, lars=0.001 if args.lars else None)
    if args.adam:
        run.lr = 1e-3
    comp = (args.compensation is not None and not dcm) or args.adam    # a third state vector is moved
    calls = [run.plan_step(t) for t in range(total)]
    timings = {}
    for name, overlap, n_acc in plans_wanted:
        run.configure_streams(overlap, n_acc)
        time_steps(run, calls, 0, max(W, 1), torch)        # also refills the delayed generation
        timings[name] = time_steps(run, calls, W, K_steps, torch, tag=name)
    # `value` comes from the plan the library's own rule names for this size
    # (abs_suggest_accumulate_streams), not from whichever happened to win this run;
    # the fastest one is reported beside it
    fastest = min(timings, key=timings.get)
    n_sug = absgd.abs_suggest_accumulate_streams(w.P, w.K)
    best = "one stream" if n_sug == 1 else next((k for k in timings if k.startswith(f"{n_sug} accumulate streams")), None)
    if best is None or best not in timings:
        best = fastest
    dt = timings[best]
    dt_serial = timings["one stream"]
    dt_overlap = min(v for k, v in timings.items() if k != "one stream")

    # Dominant kernel (accumulate) alone on the GPU: the one-stream plan, same steps.
    run.configure_streams(False, 1)
    time_steps(run, calls, 0, max(W, 1), torch)
    bracket_ms, step_launches, sync_ms = kernel_event_pass(run, calls, W, K_steps, torch)
    run.close()
    del run, calls
    torch.cuda.empty_cache()

    step_bytes = 0
    for t in range(W, total):
        a, s_ = bytes_per_param(w, sched[t], comp, args.batched, args.lars)
        step_bytes += (a + s_) * w.P
    gbs = step_bytes / dt / 1e9
    # Algorithmic bytes per accumulate launch = the step's accumulate bytes
    # (sum_k [m_k (g_b + 8) - 4] per parameter) averaged over its sum_k m_k launches.
    # A step whose bracket is far off the others (a hiccup of the box) is left out: steps are
    # ranked by time per launch and the slowest twentieth dropped.
    step_acc_bytes = [bytes_per_param(w, sched[t], comp, args.batched, args.lars)[0] * w.P for t in range(W, total)]
    order = sorted(range(K_steps), key=lambda i: bracket_ms[i] / step_launches[i])
    keep = order[:max(1, K_steps - K_steps // 20)]
    launches = sum(step_launches[i] for i in keep)
    kern_ms = sum(bracket_ms[i] for i in keep) / launches
    kern_bytes = sum(step_acc_bytes[i] for i in keep) / launches
    achieved = kern_bytes / (kern_ms * 1e-3) / 1e9
    sync_ms = sorted(sync_ms)[:max(1, len(sync_ms) - len(sync_ms) // 20)]
    sync_avg_ms = sum(sync_ms) / len(sync_ms)
    sync_bytes = bytes_per_param(w, sched[W], comp, args.batched, args.lars)[1] * w.P
    sync_gbs = sync_bytes / (sync_avg_ms * 1e-3) / 1e9
    kname = dominant_kernel(w, args.batched)
    traffic = MEASURED_TRAFFIC.get((w.name, kname))

    out = {
        "metric": METRIC,
        "value": gbs,
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": K_steps,
        "warmup": W,
        "ms_per_step": dt / K_steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": w.name, "P": w.P, "K": w.K, "grad_dtype": w.grad_dtype,
            "samples_per_microbatch": w.n, "m_k": w.schedule + (str(list(w.ratio)) if w.ratio else ""),
            "tensors": 1 if w.tensor_sizes is None else len(w.tensor_sizes),
            "lr": w.lr, "mu": w.mu, "wd": w.wd, "gradient_pool": args.pool,
            "compensation_lambda": args.compensation, "compensation_from_momentum": dcm, "batched_accumulate": args.batched,
            "update_rule": "adam" if args.adam else ("lars" if args.lars else "momentum sgd"),
            "streams": best + ", double-buffered",
            "algorithmic_bytes_per_step": step_bytes // K_steps,
        },
        "pct_hbm_peak": 100.0 * gbs / HBM_PEAK_GBS,
        "params_per_s": w.P * K_steps / dt,
        "overlap_speedup": dt_serial / dt_overlap,
        "ms_per_step_by_stream_plan": {k: v / K_steps * 1e3 for k, v in timings.items()},
        # time the host needed to enqueue a step (binding + launches + event joins): when it
        # approaches ms_per_step the workload is bound by launches, not by the kernels
        "host_issue_ms_per_step": HOST_ISSUE[best] / K_steps * 1e3,
        "fastest_plan": {"name": fastest, "ms_per_step": timings[fastest] / K_steps * 1e3,
                         "is_the_chosen_one": fastest == best,
                         "faster_than_chosen_by": timings[best] / timings[fastest] - 1.0},
        "roofline": {
            "bound": "hbm", "kernel": kname, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
            "algorithmic_bytes_per_launch": kern_bytes, "avg_launch_ms": kern_ms,
            "launches_timed": launches,
            "measured": "HIP events around each step's accumulate launches, one-stream plan "
                        "(the kernel alone on the GPU), same steps as the timed region",
        },
        "sync_update_kernel": {
            "achieved": sync_gbs, "unit": "GB/s", "frac": sync_gbs / HBM_PEAK_GBS,
            "algorithmic_bytes_per_launch": sync_bytes, "avg_launch_ms": sync_avg_ms,
            "measured": "HIP events around the single sync-update launch of each step, one-stream plan, same "
                        "steps; a bracket around one launch also holds ~5 us of dispatch latency, so this is "
                        "a lower bound on the kernel's rate (the kernel trace under profiles/ has its own duration)",
        },
        "box_ceilings": probe_ceilings(torch, w.K),
    }
    if out["box_ceilings"]:
        out["pct_of_box_copy_rate"] = 100.0 * gbs / out["box_ceilings"]["copy_GBs"]
        # the dominant kernel against a plain kernel of its own read:write mix at 1 GiB per vector
        out["roofline"]["frac_of_box_triad"] = achieved / out["box_ceilings"]["triad_GBs"]
        mix = out["box_ceilings"].get(f"mix_{w.K}_workers_GBs")
        if mix:
            out["sync_update_kernel"]["frac_of_box_mix"] = sync_gbs / mix
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, x0, pool, sched[W:])
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
