#!/usr/bin/env python3
"""Throughput of the SPB worker step on one MI355X, swept over the backprop depth k.

A step is one full forward pass plus the backward pass truncated to the top k units (Sec. 2 of the
paper) on one synthetic batch that is already resident in HBM.  The timed region replays, for every
depth of the workload's sweep in turn, a HIP graph that holds exactly the kernels the two C-ABI calls
enqueue; `--steps` is the total number of timed steps, shared evenly between the depths.

Prints ONE JSON line: metric, value, unit, per-depth times, the roofline of the dominant kernel, the server-side
update and the CPU rate of the oracle.  Other modes: --table1, --emulate K, --round-robin (each prints one line too).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK = {"mfma_bf16": 2500.0, "mfma_f32": 157.3, "hbm": 8000.0}   # TFLOP/s, TFLOP/s, GB/s (MI355X, published)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--config", default="cfg5")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="budget of the oracle timing")
    ap.add_argument("--launch", choices=["auto", "graph", "eager"], default="auto",
                    help="how the timed steps are launched: replayed HIP graphs (launch-bound workloads: the perceptrons), "
                         "eagerly on one stream (the library then runs weight gradients on a second stream of its own, "
                         "which a graph replay does not profit from), or auto = graph for perceptrons, eager otherwise")
    ap.add_argument("--eager", action="store_true",
                    help="launch the timed steps eagerly instead of replaying HIP graphs (for counter collection, "
                         "which does not survive graph replay on this ROCm)")
    ap.add_argument("--table1", action="store_true",
                    help="print forward ms / backward ms / workspace GB against the percentage of units backpropagated, "
                         "in the shape of the paper's Table 1 (ResNet-101-style stack, batch 64), and exit")
    ap.add_argument("--emulate", type=int, default=0, metavar="K",
                    help="emulate one iteration of K workers time-multiplexed on this GPU (worker j backpropagates "
                         "ceil(j L / K) units, then the server-side update), against K complete workers, and exit")
    ap.add_argument("--round-robin", action="store_true",
                    help="keep all five configurations resident and run their steps in turn: cost of switching between "
                         "models whose parameters stay on the device, and exit")
    ap.add_argument("--jigsaw", action="store_true",
                    help="time every (configuration, depth) pair on this GPU, build a seeded synthetic job mix from them and "
                         "place it on a 45-device cluster task by task (Sec. 3) and as gangs, with and without SPB, and exit")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MIB",
                    help="run only a plain elementwise copy of this many MiB (10 launches) and exit: the reference "
                         "the HBM traffic counters are scaled by")
    return ap.parse_args()


def stored_traffic(kernel_name):
    """HBM bytes per launch of the roofline kernel from a counter summary kept under profiles/ (FETCH_SIZE and
    WRITE_SIZE of two profiler passes, scaled by a plain copy's readings).  Such a file ends with `key = value`
    lines: kernel, date, fetch_bytes_per_launch, write_bytes_per_launch, sources (file names under csrc/) and
    sources_sha256.  Returns None when no file covers this kernel or the kernel's sources have changed since."""
    import glob
    import hashlib
    csrc = os.path.join(ROOT, "paper_2111_10672_amd", "csrc")
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*_hbm_traffic.txt"))):
        rec = {}
        try:
            for line in open(path):
                if " = " in line and not line.startswith(" "):
                    key, val = line.split(" = ", 1)
                    rec[key.strip()] = val.strip()
            if rec.get("kernel") != kernel_name:
                continue
            h = hashlib.sha256()
            for fn in rec["sources"].split():
                h.update(open(os.path.join(csrc, fn), "rb").read())
            if rec["sources_sha256"] != h.hexdigest():
                continue
            return {"file": os.path.relpath(path, ROOT), "date": rec.get("date"),
                    "fetch": float(rec["fetch_bytes_per_launch"]), "write": float(rec["write_bytes_per_launch"])}
        except (OSError, KeyError, ValueError):
            continue
    return None


def table1(spb, torch, wl, reps):
    """Forward time, backward time and workspace against the share of units backpropagated, for the model and batch
    size of the paper's Table 1 (its numbers are a V100's and another framework's: context, not a target).  Forward
    time is `reps` forward passes between two events; backward time is the same for whole steps, minus that."""
    cfg = wl.get_config("resnet101_cifar")
    model = spb.SpbModel(cfg, wl.make_params(cfg, 0), "cuda:0")
    dev = {n: t.cuda() for n, t in wl.make_batch(cfg, 0).items()}
    L = model.n_units
    rows = []
    for pct in reversed(cfg["percents"]):
        k = -(-pct * L // 100)
        need = model.reserve(k)
        model.step(dev, k)
        torch.cuda.synchronize()
        e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        e[0].record()
        for _ in range(reps):
            model.forward(dev, k)
        e[1].record()
        for _ in range(reps):
            model.step(dev, k)
        e[2].record()
        torch.cuda.synchronize()
        fwd, both = e[0].elapsed_time(e[1]) / reps, e[1].elapsed_time(e[2]) / reps
        rows.append({"percent": pct, "units": k, "forward_ms": round(fwd, 4), "backward_ms": round(both - fwd, 4),
                     "workspace_gb": round(need / 1e9, 4)})
    model.close()
    print(json.dumps({"table": "forward / backward time and workspace vs share of units backpropagated",
                      "workload": "resnet101_cifar: bottleneck stack [3,4,23,3], 32x32 images, batch 64, bf16",
                      "units": L, "rows": rows}))


def emulate(spb, torch, wl, name, n_workers, reps):
    """One SPB iteration of K workers sharing this GPU in time (Sec. 2 and 3): each worker runs its step on its own
    batch at its own depth into its own gradient buffers, then the server-side update consumes them.  The same with
    K complete workers is ordinary data parallelism; the ratio is what SPB saves per iteration on one device."""
    cfg = wl.get_config(name)
    model = spb.SpbModel(cfg, wl.make_params(cfg, 0), "cuda:0")
    L = model.n_units
    batches = [{n: t.cuda() for n, t in wl.make_batch(cfg, 1 + j).items()} for j in range(n_workers)]
    grads = [[torch.zeros_like(g) for g in model.grads] for _ in range(n_workers)]
    vel = [torch.zeros_like(g) for g in model.grads]
    model.reserve(L)

    def iteration(depths):
        for j, k in enumerate(depths):
            spb.spb_bind_grads(model.handle, grads[j])
            model.step(batches[j], k)
        spb.spb_aggregate_update(model.handle, depths, grads, vel, 0.0, 0.9, 0.0, True, model.stream())   # rate 0: weights stay

    out = {"workload": name, "workers": n_workers, "units": L, "batch_per_worker": cfg["batch"]}
    for label, depths in (("spb", [spb.spb_worker_depth(model.handle, j, n_workers) for j in range(1, n_workers + 1)]),
                          ("full", [L] * n_workers)):
        for _ in range(3):
            iteration(depths)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            iteration(depths)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        out[label] = {"depths": depths, "ms_per_iteration": round(ms, 4),
                      "samples_per_s": round(n_workers * cfg["batch"] / (ms * 1e-3), 1)}
    out["iteration_time_ratio_spb_over_full"] = round(out["spb"]["ms_per_iteration"] / out["full"]["ms_per_iteration"], 4)
    model.close()
    print(json.dumps(out))


def round_robin(spb, torch, wl, reps):
    """Sec. 3 keeps the parameters of several jobs on the device and switches between them; here the five
    configurations stay resident (parameters, gradients, workspaces) and their steps run in turn at each one's
    shallowest depth.  Reported: every model's step time alone and the time of a whole turn."""
    names = ["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"]
    models, batches, depths = [], [], []
    for n in names:
        cfg = wl.get_config(n)
        m = spb.SpbModel(cfg, wl.make_params(cfg, 0), "cuda:0")
        k = wl.depth_sweep(cfg)[0]
        m.reserve(k)
        models.append(m); depths.append(k)
        batches.append({key: t.cuda() for key, t in wl.make_batch(cfg, 0).items()})

    def timed(fn):
        for _ in range(2):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    alone = [timed(lambda m=m, b=b, k=k: m.step(b, k)) for m, b, k in zip(models, batches, depths)]

    def turn():
        for m, b, k in zip(models, batches, depths):
            m.step(b, k)

    whole = timed(turn)
    resident = sum(m.workspace_bytes + sum(p.numel() * p.element_size() + g.numel() * 4 for p, g in zip(m.params, m.grads)) for m in models)
    for m in models:
        m.close()
    print(json.dumps({"models": names, "depths": depths, "step_ms_alone": [round(a, 4) for a in alone],
                      "sum_alone_ms": round(sum(alone), 4), "turn_ms": round(whole, 4),
                      "switching_overhead_ms": round(whole - sum(alone), 4), "resident_gb": round(resident / 1e9, 3)}))


def jigsaw_report(spb, torch, wl, reps, n_jobs=200, n_machines=45, seed=0):
    """Sec. 3-4.2: task-by-task placement of SPB jobs against gang scheduling of complete jobs, on a synthetic mix.
    Every (configuration, depth) pair is timed on this GPU (step time and workspace: what the paper's scheduler
    gets from profiling); jobs draw a configuration, a worker count with the paper's proportions (half the jobs
    one worker, the rest 2 / 4 / 8 / 16 as 10 / 20 / 15 / 5 %) and an iteration count; worker j of W
    backpropagates ceil(j L / W) units.  The cluster is `n_machines` copies of this GPU; moving a model costs its
    parameter bytes at 50 GB/s.  The placement itself is the library's spb_schedule_tasks."""
    import random
    import time as _time
    names = ["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"]
    step_ms, ws_bytes, model_bytes, units = {}, {}, {}, {}
    for n in names:
        cfg = wl.get_config(n)
        m = spb.SpbModel(cfg, wl.make_params(cfg, 0), "cuda:0")
        b = {key: t.cuda() for key, t in wl.make_batch(cfg, 0).items()}
        units[n] = m.n_units
        m.reserve(m.n_units)
        model_bytes[n] = sum(p.numel() * p.element_size() for p in m.params)
        for k in range(1, m.n_units + 1):
            for _ in range(2):
                m.step(b, k)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(reps):
                m.step(b, k)
            e1.record()
            torch.cuda.synchronize()
            step_ms[(n, k)] = e0.elapsed_time(e1) / reps
            ws_bytes[(n, k)] = spb.spb_workspace_size(m.handle, k)
        m.close()
    rng = random.Random(seed)
    hbm = 288e9
    jobs_spb, jobs_full = [], []
    for _ in range(n_jobs):
        n = rng.choice(names)
        u = rng.random()
        w = 1 if u < 0.5 else 2 if u < 0.6 else 4 if u < 0.8 else 8 if u < 0.95 else 16
        iters = rng.randint(20, 120)
        arrival = rng.uniform(0.0, 2.0)
        depths = [-(-j * units[n] // w) for j in range(1, w + 1)]
        common = dict(arrival=arrival, iterations=iters, model_size=float(model_bytes[n]))
        jobs_spb.append(dict(common, durations=[step_ms[(n, k)] * 1e-3 for k in depths],
                             resources=[ws_bytes[(n, k)] / hbm for k in depths]))
        full = units[n]
        jobs_full.append(dict(common, durations=[step_ms[(n, full)] * 1e-3] * w, resources=[ws_bytes[(n, full)] / hbm] * w))
    gamma = 1.0 / 50e9
    out = {"jobs": n_jobs, "machines": n_machines, "tasks": sum(len(j["durations"]) * j["iterations"] for j in jobs_spb)}
    for label, jobs, gang in (("spb_tasks", jobs_spb, False), ("spb_gang", jobs_spb, True),
                              ("full_tasks", jobs_full, False), ("full_gang", jobs_full, True)):
        t0 = _time.perf_counter()
        placed, makespan = spb.spb_schedule_tasks(jobs, n_machines, gamma=gamma, gang=gang)
        out[label] = {"makespan_s": round(makespan, 4), "moved_fraction": round(sum(p["moved"] for p in placed) / max(1, len(placed)), 5),
                      "placement_wall_s": round(_time.perf_counter() - t0, 3)}
    out["makespan_ratio_spb_tasks_over_full_gang"] = round(out["spb_tasks"]["makespan_s"] / out["full_gang"]["makespan_s"], 4)
    out["step_ms"] = {f"{n} k={k}": round(v, 4) for (n, k), v in step_ms.items()}
    print(json.dumps(out))


def server_update(spb, torch, wl, model, cfg, n_workers=4, reps=50):
    """The server side of an iteration (Sec. 2: per-layer average over the contributing workers, then the optimizer
    step) for 4 workers at depths ceil(j L / 4), timed outside the step's timed region: an HBM-bound kernel, reported
    as bytes it must move per second against the HBM peak."""
    names = [i["name"] for i in model.infos]
    depths = [spb.spb_worker_depth(model.handle, j, n_workers) for j in range(1, n_workers + 1)]
    grads = [[torch.zeros_like(g) for g in model.grads] for _ in range(n_workers)]
    vel = [torch.zeros_like(g) for g in model.grads]
    es = 4 if cfg["dtype"] == "f32" else 2
    nbytes = 0
    for info in model.infos:
        c = sum(1 for k in depths if info["unit"] >= model.n_units - k)
        if c:
            nbytes += info["numel"] * (4 * c + 8 + 2 * es)
    stream = model.stream()
    run = lambda: spb.spb_aggregate_update(model.handle, depths, grads, vel, 0.0, 0.9, 0.0, True, stream)   # rate 0: parameters stay as they are
    for _ in range(5):
        run()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        run()
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / reps
    return {"workers": n_workers, "depths": depths, "us": round(us, 2), "algorithmic_bytes": nbytes,
            "gbps": round(nbytes / us / 1e3, 1), "frac_hbm_peak": round(nbytes / us / 1e3 / PEAK["hbm"], 4)}


def cpu_model_name():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(wl, cfg, params, batch, depths, budget_s):
    """The oracle as it stands, exact float64 mode, on this host's cores, on a bounded sample of the benchmarked
    workload: whole depth sweeps for the perceptrons (milliseconds per step), ONE step at the deepest depth of the
    sweep for the large configurations (tens of seconds; the bottleneck CNN on the first 8 images of its batch)."""
    import oracle
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    common = {"unit": "samples/s", "cores": int(cores), "kind": "oracle", "cpu": cpu_model_name()}
    if cfg["family"] != "mlp":
        k = depths[-1]
        n = cfg["batch"]
        if cfg["family"] == "resnet_bottleneck" and cfg["batch"] > 8:
            n = 8
            batch = {name: t[:n] for name, t in batch.items()}
            cfg = dict(cfg, batch=n)
        t0 = time.perf_counter()
        oracle.spb_step(cfg, params, batch, k)
        elapsed = time.perf_counter() - t0
        return dict(common, value=n / elapsed, seconds=round(elapsed, 2),
                    sample=f"{cfg['name']}: one step (full forward, backward through the top {k} units) on "
                           f"{n} of the batch's {len(next(iter(batch.values()))) if n == cfg['batch'] else 64} samples, "
                           f"float64 exact mode, {elapsed:.1f} s")
    oracle.spb_step(cfg, params, batch, depths[-1])            # touch everything once, untimed
    t0 = time.perf_counter()
    sweeps = 0
    while True:
        for k in depths:
            oracle.spb_step(cfg, params, batch, k)
        sweeps += 1
        elapsed = time.perf_counter() - t0
        if elapsed >= budget_s or elapsed * (sweeps + 1) / sweeps > 2.5 * budget_s:
            break
    samples = sweeps * len(depths) * cfg["batch"]
    return dict(common, value=samples / elapsed, seconds=round(elapsed, 2),
                sample=f"{cfg['name']} full batch of {cfg['batch']}, {sweeps} sweep(s) over depths {depths}, "
                       f"float64 exact mode, {elapsed:.1f} s")


RIDGE = {"bf16": PEAK["mfma_bf16"] * 1e3 / PEAK["hbm"], "f32": PEAK["mfma_f32"] * 1e3 / PEAK["hbm"]}   # flop per byte


def is_backward_product(name):
    return any(tag in name for tag in ("dgrad", "wgrad", "attn_bwd"))


def product_roofline(rec, dtype, avg_us):
    """One product class against the roofline that bounds it: the matrix-core peak when its arithmetic intensity
    (flops over the bytes of each operand once plus the result once) is above the ridge, else that intensity times
    the HBM peak.  Both fractions are given either way."""
    mfma_peak = PEAK["mfma_f32" if dtype == "f32" else "mfma_bf16"]
    flops, nbytes = rec["flops"] / rec["launches"], rec["bytes"] / rec["launches"]
    ai = flops / nbytes
    tflops = flops / avg_us / 1e6
    gbps = nbytes / avg_us / 1e3
    roof = min(mfma_peak, ai * PEAK["hbm"] / 1e3)          # TFLOP/s this product could reach at best
    bound = "mfma" if ai >= RIDGE[dtype] else "hbm"
    out = {"kernel": rec["name"], "bound": bound, "arithmetic_intensity_flop_per_byte": round(ai, 1),
           "ridge_flop_per_byte": round(RIDGE[dtype], 1),
           "tflops": round(tflops, 2), "frac_of_mfma_peak": round(tflops / mfma_peak, 5),
           "frac_of_min_roof": round(tflops / roof, 5), "gbps_at_algorithmic_bytes": round(gbps, 1),
           "flops_per_launch": flops, "algorithmic_bytes_per_launch": nbytes, "avg_launch_us": round(avg_us, 3)}
    if bound == "mfma":
        out.update(achieved=round(tflops, 3), peak=mfma_peak, unit="TFLOP/s", frac=round(tflops / mfma_peak, 5))
    else:
        out.update(achieved=round(gbps, 2), peak=PEAK["hbm"], unit="GB/s", frac=round(gbps / PEAK["hbm"], 5))
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: the library runs one worker's step on ONE GPU; there is no multi-GPU path. "
              "Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2111_10672_amd as spb
    import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the SPB path has no host fallback.", file=sys.stderr)
        sys.exit(2)

    if args.calibrate_copy:
        n = args.calibrate_copy << 20
        src = torch.ones(n // 4, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.add(src, 0.0, out=dst)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(10):
            torch.add(src, 0.0, out=dst)      # one read and one write of n bytes per launch
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / 10
        print(json.dumps({"copy_bytes_read": n, "copy_bytes_written": n, "launches": 11, "us_per_launch": round(us, 2),
                          "gbps": round(2 * n / us / 1e3, 1), "frac_hbm_peak": round(2 * n / us / 1e3 / PEAK["hbm"], 4)}))
        return

    if args.table1:
        table1(spb, torch, wl, max(3, min(args.steps, 20)))
        return
    if args.emulate:
        emulate(spb, torch, wl, args.config, args.emulate, max(5, min(args.steps, 200)))
        return
    if args.round_robin:
        round_robin(spb, torch, wl, max(3, min(args.steps, 50)))
        return
    if args.jigsaw:
        jigsaw_report(spb, torch, wl, max(3, min(args.steps, 20)))
        return

    cfg = wl.get_config(args.config)
    depths = wl.depth_sweep(cfg)
    params, batch = wl.make_params(cfg, 0), wl.make_batch(cfg, 0)
    model = spb.SpbModel(cfg, params, "cuda:0")
    dev = {n: t.cuda() for n, t in batch.items()}
    model.reserve(max(depths))
    steps, warmup = max(1, args.steps), max(0, args.warmup)
    sweep = lambda i: depths[i % len(depths)]      # step i runs at this depth: the sweep is walked step by step

    # One HIP graph per depth: the kernels of spb_forward(k) + spb_backward_truncated(k), nothing else.
    # (graph capture needs a stream of its own; eager launches stay on the default stream, the only one the
    # counter-collection mode of the profiler copes with)
    eager = args.eager or args.launch == "eager" or (args.launch == "auto" and cfg["family"] != "mlp")
    stream = torch.cuda.current_stream() if eager else torch.cuda.Stream()
    graphs = {}
    with torch.cuda.stream(stream):
        for k in depths:
            model.step(dev, k)
        stream.synchronize()
        class Eager:
            def __init__(self, k):
                self.k = k

            def replay(self):
                model.step(dev, self.k)

        for k in depths:
            if eager:
                graphs[k] = Eager(k)
                continue
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=stream):
                model.step(dev, k)
            graphs[k] = g
        for i in range(warmup):
            graphs[sweep(i)].replay()
        stream.synchronize()
        # ---- timed region: exactly `steps` steps, depths taken in turn ------------------------------
        m0, m1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        m0.record(stream)
        for i in range(steps):
            graphs[sweep(i)].replay()
        m1.record(stream)
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        total_ms = m0.elapsed_time(m1)

        # ---- outside the timed region: each depth on its own (the sweep of the metric) ---------------
        per_depth = max(2, min(200, -(-steps // len(depths))))
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(len(depths) + 1)]
        marks[0].record(stream)
        for i, k in enumerate(depths):
            for _ in range(per_depth):
                graphs[k].replay()
            marks[i + 1].record(stream)
        torch.cuda.synchronize()
        depth_ms = [marks[i].elapsed_time(marks[i + 1]) / per_depth for i in range(len(depths))]

        # ---- the same steps launched eagerly, every kernel bracketed by HIP events on this stream ----
        timing_steps = max(2, min(50, per_depth))
        spb.spb_set_kernel_timing(model.handle, True)
        for _ in range(timing_steps):
            for k in depths:
                model.step(dev, k)
        stream.synchronize()
        kernels = spb.spb_read_kernel_timing(model.handle)
        # The roofline kernel is the backward product (input gradient or weight gradient) with the largest total
        # time.  Beside its in-step average (one event bracket per launch, which adds the dispatch latency of a
        # few microseconds), the same product back-to-back between two events.
        products = [r for r in kernels if r["flops"] > 0]
        backward = [r for r in products if is_backward_product(r["name"])]
        dom = max(backward or products or kernels, key=lambda r: r["total_ms"])
        back_to_back_us = None
        if dom["flops"] > 0:
            reps = 100
            spb.spb_replay_kernel(model.handle, dom["name"], 10, stream.cuda_stream)
            b0, b1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            b0.record(stream)
            spb.spb_replay_kernel(model.handle, dom["name"], reps, stream.cuda_stream)
            b1.record(stream)
            stream.synchronize()
            back_to_back_us = b0.elapsed_time(b1) * 1e3 / reps
        spb.spb_set_kernel_timing(model.handle, False)

    ms_per_step = total_ms / steps
    value = cfg["batch"] / (ms_per_step * 1e-3)
    dtype = "f32" if cfg["dtype"] == "f32" else "bf16"
    table = []
    for r in kernels:
        avg_us = r["total_ms"] / r["launches"] * 1e3
        row = {"name": r["name"], "launches_per_sweep": r["launches"] / timing_steps, "avg_us": round(avg_us, 3),
               "gbps": round(r["bytes"] / r["total_ms"] / 1e6, 2)}
        if r["flops"]:
            pr = product_roofline(r, dtype, avg_us)
            row.update(tflops=pr["tflops"], bound=pr["bound"], frac_of_mfma_peak=pr["frac_of_mfma_peak"],
                       frac_of_min_roof=pr["frac_of_min_roof"])
        else:
            row.update(bound="hbm", frac_of_hbm_peak=round(r["bytes"] / r["total_ms"] / 1e6 / PEAK["hbm"], 5))
        table.append(row)
    if dom["flops"] > 0:
        roofline = product_roofline(dom, dtype, dom["total_ms"] / dom["launches"] * 1e3)
        roofline["avg_launch_us_back_to_back"] = round(back_to_back_us, 3)
        roofline["tflops_back_to_back"] = round(dom["flops"] / dom["launches"] / back_to_back_us / 1e6, 2)
        rec = stored_traffic(dom["name"])
        roofline["traffic"] = rec["fetch"] + rec["write"] if rec else None
        if rec:
            roofline.update(traffic_unit="HBM bytes per launch (fetch + write)", traffic_fetch=rec["fetch"], traffic_write=rec["write"],
                            traffic_source=f"stored: {rec['file']} ({rec['date']}), kernel sources unchanged since")
    else:
        achieved = dom["bytes"] / dom["total_ms"] / 1e6
        roofline = {"kernel": dom["name"], "bound": "hbm", "achieved": round(achieved, 2), "peak": PEAK["hbm"],
                    "unit": "GB/s", "frac": round(achieved / PEAK["hbm"], 5), "traffic": None}
    # all backward products together: flops over the summed in-step time
    bwd_flops, bwd_ms = sum(r["flops"] for r in backward), sum(r["total_ms"] for r in backward)
    shape = cfg["dims"] if "dims" in cfg else {k: cfg[k] for k in ("layers", "hidden", "heads", "ffn", "seq", "vocab", "loss_rows") if k in cfg} or \
        {k: cfg[k] for k in ("image", "stage_blocks", "stage_widths", "classes")}

    out = {
        "metric": "SPB train-step samples/sec vs backprop depth k; % MFMA peak (bwd GEMMs)",
        "value": round(value, 1), "unit": "samples/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": round(ms_per_step, 6), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype, "data": "synthetic",
        "config": {"workload": f"{cfg['name']}: {cfg['family']} {shape} batch {cfg['batch']}, "
                               f"depth sweep k={depths} walked step by step (step i runs depth number i mod {len(depths)})",
                   "launch": "eager" if eager else "hip_graph_replay"},
        "samples_per_s_by_depth": {str(k): round(cfg["batch"] / (ms * 1e-3), 1) for k, ms in zip(depths, depth_ms)},
        "ms_by_depth": {str(k): round(ms, 6) for k, ms in zip(depths, depth_ms)},
        "workspace_bytes_by_depth": {str(k): spb.spb_workspace_size(model.handle, k) for k in depths},
        "wall_ms_timed_region": round(wall_ms, 3),
        "roofline": roofline,
        "backward_products_tflops": round(bwd_flops / bwd_ms / 1e9, 2) if bwd_ms else None,
        "backward_products_frac_of_mfma_peak": round(bwd_flops / bwd_ms / 1e9 / PEAK["mfma_f32" if dtype == "f32" else "mfma_bf16"], 5) if bwd_ms else None,
        "kernels": sorted(table, key=lambda r: -r["avg_us"] * r["launches_per_sweep"])[:24],
    }
    out["server_update"] = server_update(spb, torch, wl, model, cfg)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, cfg, params, batch, depths, args.cpu_seconds)
    model.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
