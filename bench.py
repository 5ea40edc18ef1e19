#!/usr/bin/env python3
"""Benchmark of the stitched fusion-group kernels on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--only NAME] [--full] [--no-cpu] [--no-traffic]

Prints ONE JSON line.  The headline workload is the largest of the five benchmark groups, LayerNorm
backward on fp32 [32768, 1024] (dx by two row reductions, dgamma and dbeta by column reductions over
all rows, one stitched plan): one step = one launch of the plan over one batch of synthetic input
already resident in HBM.  `value` is algorithmic bytes (every group input read once, every output
written once) per second of wall time over the timed steps.  Input buffers rotate over enough
distinct sets that the bytes touched between two uses of a set exceed the 256 MB last-level cache.

`roofline` is the same plan against the 8 TB/s HBM peak, from HIP events recorded on the launch
stream around the timed launches; `roofline.traffic` is measured in this run by two child runs under
rocprofv3 (FETCH_SIZE, then WRITE_SIZE), each scaled by what the counter reads for the plain copy
kernel.  `config.configs` carries all five benchmark groups measured in this run (microseconds by
events, fraction of peak, fraction of the copy kernel's rate on the same bytes, per-op baseline);
`cpu_baseline` is the CPU oracle timed on this machine's host cores, on one thread and on all of them.
`--full` adds the long per-group table (generated-kernel groups, tuner, bandwidth model, whole
programs through the fusion planner).
"""
from __future__ import annotations

import argparse
import json
import os
import subprocess
import sys
import tempfile
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_all_groups.md")
HEADLINE = "layernorm_bwd"

ROTATE_BYTES = 640 * 2**20     # bytes touched between reuses of one buffer set
TUNE = False                   # also time every group after fs_plan_tune (--full)
SPIN_UP_S = 0.05               # seconds of untimed launches before every timing loop (see time_plan; --spin-up)

TORCH_DT = None


def committed_traffic(name):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary, or None."""
    import re
    try:
        text = open(TRAFFIC_FILE).read()
    except OSError:
        return None
    m = re.search(r"traffic_bytes_per_launch\[%s\]\s*=\s*(\d+)" % re.escape(name), text)
    return int(m.group(1)) if m else None


def _torch_dt():
    global TORCH_DT
    import torch
    if TORCH_DT is None:
        TORCH_DT = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
    return TORCH_DT


def make_sets(ops, ins, algo_bytes, max_sets=8):
    """Device copies of the inputs and outputs, rotated so consecutive launches touch
    different memory.  Set 0 holds the seeded inputs; the others hold the same tensors
    with their leading dim rolled (same distribution, different addresses)."""
    import torch
    from workloads import inputs as wl_inputs
    dts = [op.dtype for op in ops if op.kind == "parameter"]
    outs = [(op.shape, op.dtype) for op in ops if op.kind == "output"]
    n_sets = max(1, min(max_sets, -(-ROTATE_BYTES // max(1, algo_bytes))))
    base = [wl_inputs.to_torch(a, dt, "cuda:0") for a, dt in zip(ins, dts)]
    sets = []
    for j in range(n_sets):
        lead = base[0].shape[0]
        tin = base if j == 0 else [torch.roll(t, 997 * j, 0).contiguous() if t.shape[0] == lead else t.clone()
                                   for t in base]
        tout = [torch.empty(shape, dtype=_torch_dt()[dt], device="cuda:0") for shape, dt in outs]
        sets.append((tin, tout))
    return sets


def time_plan(plan, sets, steps, warmup):
    """-> (wall ms per step, event ms per step).  Launches go to torch's current stream
    and the HIP events are recorded on that same stream."""
    import torch
    from paper_1911_11576_amd import BoundArgs
    bound = [BoundArgs(i, o) for i, o in sets]
    n = len(bound)
    stream = torch.cuda.current_stream().cuda_stream
    # Untimed spin-up before the warmup steps: after an idle stretch (the host builds the next
    # group's inputs) the first ~20 ms of launches measured up to 10% slower than the steady state.
    t_end = time.perf_counter() + SPIN_UP_S
    i = 0
    while time.perf_counter() < t_end:
        for _ in range(16):
            plan.launch_bound(bound[i % n], stream)
            i += 1
        torch.cuda.synchronize()
    for i in range(warmup):
        plan.launch_bound(bound[i % n], stream)
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for i in range(steps):
        plan.launch_bound(bound[i % n], stream)
    e1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    return (t1 - t0) * 1e3 / steps, e0.elapsed_time(e1) / steps


def time_copy(nbytes, steps, warmup):
    """Plain copy kernel moving `nbytes` in total (half read, half written)."""
    import torch
    from paper_1911_11576_amd import fs_stream_copy
    half = max(16, (nbytes // 2) // 16 * 16)
    n = max(1, min(8, -(-ROTATE_BYTES // (2 * half))))
    src = [torch.empty(half, dtype=torch.uint8, device="cuda:0").random_(0, 255) for _ in range(n)]
    dst = [torch.empty(half, dtype=torch.uint8, device="cuda:0") for _ in range(n)]
    # pointers and stream resolved once: small copies would otherwise time the Python wrapper
    stream = torch.cuda.current_stream().cuda_stream
    dp, sp = [t.data_ptr() for t in dst], [t.data_ptr() for t in src]
    t_end = time.perf_counter() + SPIN_UP_S
    i = 0
    while time.perf_counter() < t_end:
        for _ in range(16):
            fs_stream_copy(dp[i % n], sp[i % n], half, stream)
            i += 1
        torch.cuda.synchronize()
    for i in range(warmup):
        fs_stream_copy(dp[i % n], sp[i % n], half, stream)
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(steps):
        fs_stream_copy(dp[i % n], sp[i % n], half, stream)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps, 2 * half


def bandwidth_model(steps=100, warmup=10):
    """M(V) of the paper's model-based score (Section 4.3): achieved bandwidth of a plain
    streaming kernel as a function of the bytes it moves, measured with the copy kernel."""
    import torch
    table = []
    for mb in (1, 2, 4, 8, 16, 32, 64, 128, 256, 512, 1024):
        nbytes = mb << 20
        ms, moved = time_copy(nbytes, steps, warmup)
        table.append({"bytes": moved, "us": ms * 1e3, "gbs": moved / (ms * 1e-3) / 1e9})
        torch.cuda.empty_cache()
    return table


def bench_group(cfg, steps, warmup, with_per_op=True, build_kw=None):
    import torch
    from paper_1911_11576_amd import Plan
    from workloads import algorithmic_bytes
    ops, ins = cfg.build("full", **(build_kw or {}))
    algo = algorithmic_bytes(ops)
    sets = make_sets(ops, ins, algo)
    res = {"algorithmic_bytes": algo, "buffer_sets": len(sets)}
    with Plan(ops) as plan:
        info = plan.info()
        template = plan.describe()
        wall_ms, ev_ms = time_plan(plan, sets, steps, warmup)
    res.update(schedule=info["schedule"], n_kernels=info["n_kernels"], template=template, stitched_us=ev_ms * 1e3,
               stitched_wall_us=wall_ms * 1e3,
               stitched_gbs=algo / (ev_ms * 1e-3) / 1e9, stitched_frac_of_peak=algo / (ev_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
               lds_bytes=info["lds_bytes"], workspace_bytes=info["workspace_bytes"])
    # the same group after the tuner (Algorithm 3's loop over templates) has timed the schedule's launch
    # templates on one buffer set and kept the fastest
    if TUNE:
        try:
            with Plan.tune(ops, sets[0][0], sets[0][1], trials=30) as plan:
                twall, tev = time_plan(plan, sets, steps, warmup)
                res.update(tuned_us=tev * 1e3, tuned_frac_of_peak=algo / (tev * 1e-3) / 1e9 / HBM_PEAK_GBS,
                           tuned_options={k: v for k, v in plan.tuned.items() if k != "us"}, tuned_template=plan.describe())
        except Exception as e:   # the tuner is an extra: report, do not fail the bench
            res.update(tuned_error=str(e))
    if with_per_op:
        psteps = max(5, steps // 10)
        with Plan(ops, "per_op") as plan:
            pinfo = plan.info()
            pwall, pev = time_plan(plan, sets, psteps, max(2, warmup // 10))
        res.update(per_op_us=pev * 1e3, per_op_kernels=pinfo["n_kernels"], per_op_moved_bytes=pinfo["moved_bytes"],
                   speedup_vs_per_op=pev / ev_ms)
    cms, cbytes = time_copy(algo, steps, warmup)
    res.update(copy_us=cms * 1e3, copy_gbs=cbytes / (cms * 1e-3) / 1e9,
               stitched_frac_of_copy=(algo / ev_ms) / (cbytes / cms))
    del sets
    torch.cuda.empty_cache()
    return res, ev_ms, wall_ms


def compact(res):
    """The few figures of one group that go into the headline line."""
    r3 = lambda v: None if v is None else round(v, 3)
    return {"us": round(res["stitched_us"], 2), "frac": r3(res["stitched_frac_of_peak"]), "copy_frac": r3(res["stitched_frac_of_copy"]),
            "kernels": res["n_kernels"], "per_op_us": round(res.get("per_op_us", 0.0), 1), "per_op_kernels": res.get("per_op_kernels"),
            "speedup": round(res.get("speedup_vs_per_op", 0.0), 1), "bytes": res["algorithmic_bytes"]}


def bench_programs(steps=40, warmup=5):
    """Whole graphs through the fusion planner (Section 4) and the stitched groups it makes, against the
    same graph one kernel per op: a stack of five row-local layers (bias + GELU + residual + LayerNorm,
    no partition op between them) and the clipping of four gradient tensors by their global norm.  Device tensors are drawn by torch (seeded); results are checked elsewhere (tests)."""
    import torch
    from paper_1911_11576_amd import FusedProgram, Plan
    from workloads import graphs
    gen = torch.Generator(device="cuda:0").manual_seed(1911)
    rnd = lambda *shape: torch.randn(*shape, device="cuda:0", generator=gen)
    rows, cols, layers = 16384, 1024, 5
    shapes = [(4096, 1024), (1024,), (1024, 4096), (4096,)]
    cases = {
        "encoder_tail_stack_5_layers": (graphs.encoder_tail_stack(layers, rows, cols),
                                        [rnd(rows, cols)] + [0.5 * rnd(cols) for _ in range(3 * layers)]),
        "clip_by_global_norm_4_tensors": (graphs.clip_by_global_norm(shapes, 1.0), [rnd(*sh) for sh in shapes]),
    }

    def timed(fn):
        t_end = time.perf_counter() + SPIN_UP_S
        while time.perf_counter() < t_end:
            fn()
            torch.cuda.synchronize()
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / steps * 1e3

    out = {}
    for name, (ops, ins) in cases.items():
        with FusedProgram(ops) as prog:
            prog.bind(ins)
            fused_us = timed(prog.run_bound)
            res = {"ops": len(ops), "groups": len(prog.fusion.groups), "kernels": prog.n_kernels, "fused_us": fused_us,
                   "group_sizes": [len(g["members"]) for g in prog.fusion.groups]}
        # the same graph planned again with execution-based scores for the plan's patterns and the best other candidates
        prog, report = FusedProgram.measured(ops, top=8, trials=10)
        with prog:
            prog.bind(ins)
            res.update(measured_plan_us=timed(prog.run_bound), measured_plan_groups=len(prog.fusion.groups),
                       measured_plan_kernels=prog.n_kernels, measured_patterns=len(report),
                       measured_vs_model_us=[[len(o), round(m, 2), round(v, 2)] for o, m, v in report[:6]])
        with Plan(ops, "per_op") as plan:
            outs = [torch.empty(op.shape, dtype=_torch_dt()[op.dtype], device="cuda:0") for op in ops if op.kind == "output"]
            per_op_us = timed(lambda: plan.launch(ins, outs))
            res.update(per_op_kernels=plan.info()["n_kernels"], per_op_us=per_op_us, speedup_vs_per_op=per_op_us / fused_us)
        out[name] = res
        del ins
        torch.cuda.empty_cache()
    return out


# ---------------------------------------------------------------- CPU oracle timing

# rows (batch elements for config 3) of each benchmark group that one worker runs through the oracle
CPU_SAMPLE = {"layernorm_fwd": dict(rows=256, cols=768), "scaled_masked_softmax": dict(shape=(8192, 128), mask="full"),
              "causal_attention": dict(batch=32, seq=64, dim=64), "bias_gelu_residual_layernorm": dict(rows=1024, cols=1024),
              "layernorm_bwd": dict(rows=1024, cols=1024)}


def _cpu_worker(name):
    """One worker: the oracle on this group's sample, repeated for about a second; -> (bytes, seconds, reps)."""
    from threadpoolctl import threadpool_limits
    from oracle import interp
    from workloads import BY_NAME, algorithmic_bytes
    cfg = BY_NAME[name]
    ops, ins = cfg.build("full", **CPU_SAMPLE[name])
    nbytes = algorithmic_bytes(ops)
    with threadpool_limits(1):
        interp.run(ops, ins)           # untimed: pages and caches warm
        reps, total = 0, 0.0
        while total < 1.0 and reps < 200:
            t0 = time.perf_counter()
            interp.run(ops, ins)
            total += time.perf_counter() - t0
            reps += 1
    return nbytes, total, reps


def cpu_baseline():
    """The oracle as it stands, timed on the host cores before anything touches the GPU: every benchmark
    group on a bounded sample of its rows, first one worker on one thread, then as many workers as the
    box has cores (each on one thread, each on a sample of its own: rows are independent, and the column
    sums of config 5 are then sums over each worker's rows).  The headline figure is config 5 on all cores."""
    import multiprocessing as mp
    from workloads import CONFIGS
    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit():
        cores = max(1, min(cores, int(env)))       # the machine's CPU share, where nproc shows the whole host
    names = [c.name for c in CONFIGS]
    one, many = {}, {}
    ctx = mp.get_context("fork")
    with ctx.Pool(cores) as pool:
        pool.map(_cpu_worker, [names[0]] * cores)          # workers started and imports done before timing
        for name in names:
            nbytes, sec, reps = pool.apply(_cpu_worker, (name,))
            one[name] = round(nbytes * reps / sec / 1e9, 3)
            t0 = time.perf_counter()
            res = pool.map(_cpu_worker, [name] * cores, chunksize=1)
            wall = time.perf_counter() - t0
            # every worker ran for `sec_i`; they ran side by side, so the rate is the sum of the workers' rates
            many[name] = round(sum(b * r / s for b, s, r in res) / 1e9, 3)
            del wall
    cpu = None
    try:
        with open("/proc/cpuinfo") as f:
            cpu = next((l.split(":", 1)[1].strip() for l in f if l.startswith("model name")), None)
    except OSError:
        pass
    return {"value": many[HEADLINE], "unit": "GB/s", "cores": cores, "kind": "oracle",
            "sample": "per worker: " + ", ".join(f"{k} {v}" for k, v in CPU_SAMPLE.items()) +
                      "; about 1 s of repetitions each, one thread per worker, algorithmic bytes / time summed over the workers",
            "one_thread_gbs": one, "all_cores_gbs": many, "cpu_model": cpu}


# ---------------------------------------------------------------- HBM traffic by counters, in this run

def traffic_child(name):
    """Run under rocprofv3 by measure_traffic(): a few launches of the copy kernel on a known size, then a
    few launches of the group's plan.  Prints what the parent needs to find the dispatches."""
    global SPIN_UP_S
    SPIN_UP_S = 0.0
    import torch
    from paper_1911_11576_amd import Plan, fs_stream_copy
    from workloads import BY_NAME, algorithmic_bytes
    torch.cuda.set_device(0)
    half = 96 << 20
    src = torch.empty(half, dtype=torch.uint8, device="cuda:0").random_(0, 255)
    dst = torch.empty(half, dtype=torch.uint8, device="cuda:0")
    for _ in range(6):
        fs_stream_copy(dst, src, half)
    torch.cuda.synchronize()
    del src, dst
    cfg = BY_NAME[name]
    ops, ins = cfg.build("full")
    sets = make_sets(ops, ins, algorithmic_bytes(ops), max_sets=2)
    with Plan(ops) as plan:
        time_plan(plan, sets, 6, 2)
    print(json.dumps({"copy_half_bytes": half}))


def measure_traffic(name, timeout_s=150):
    """-> (bytes per launch of the group's kernels, detail) or (None, reason).  Two child runs under
    rocprofv3 --pmc, one counter each; per dispatch the counters are KiB; each is scaled by what it
    reads for the copy kernel, whose bytes are known."""
    import csv
    import statistics
    rocprof = "/opt/rocm/bin/rocprofv3"
    if not os.path.exists(rocprof):
        return None, "rocprofv3 not found"
    vals = {}
    with tempfile.TemporaryDirectory(prefix="fs_traffic_") as tmp:
        env = dict(os.environ, TMPDIR=tmp)
        for counter in ("FETCH_SIZE", "WRITE_SIZE"):
            cmd = ["timeout", "-s", "KILL", str(timeout_s), rocprof, "--pmc", counter, "-d", tmp, "-o", counter.lower(),
                   "--output-format", "csv", "--", sys.executable, os.path.join(ROOT, "bench.py"), "--traffic-child", name]
            try:
                r = subprocess.run(cmd, cwd=tmp, env=env, capture_output=True, text=True, timeout=timeout_s + 30)
            except (OSError, subprocess.TimeoutExpired) as e:
                return None, f"{counter}: {e}"
            if r.returncode != 0:
                return None, f"{counter}: rocprofv3 exited {r.returncode}: {(r.stderr or r.stdout)[-300:]}"
            path = None
            for dirpath, _, files in os.walk(tmp):
                for fn in files:
                    if fn.endswith("counter_collection.csv") and counter.lower() in fn:
                        path = os.path.join(dirpath, fn)
            if path is None:
                return None, f"{counter}: no counter_collection.csv written"
            per = {}
            for row in csv.DictReader(open(path)):
                if row["Counter_Name"] == counter:
                    per.setdefault(row["Kernel_Name"], []).append(float(row["Counter_Value"]))
            vals[counter] = per
    half = 96 << 20
    detail, total = {}, 0.0
    for counter in ("FETCH_SIZE", "WRITE_SIZE"):
        per = vals[counter]
        copy = [k for k in per if "stream_copy_kernel" in k]
        if not copy:
            return None, f"{counter}: copy kernel not in the trace"
        factor = (half / 1024.0) / statistics.median(per[copy[0]])
        detail[counter.lower() + "_factor"] = round(factor, 4)
        kib = 0.0
        for k, v in per.items():
            # the plan's kernels: hand-written stitched kernels, generated ones, and the combine kernel of a column reduction
            if k.startswith(("fs_row_", "fs_ew_")) or "stitch_kernel" in k or "col_combine" in k or "lnbwd" in k:
                kib += statistics.median(v)
                detail.setdefault("kernels", set()).add(k.split("(")[0])
        total += kib * factor * 1024.0
    detail["kernels"] = sorted(detail.get("kernels", []))
    return int(round(total)), detail


def main():
    global SPIN_UP_S, TUNE
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--only", default=None, help="time just this group as the headline (a config name)")
    ap.add_argument("--full", action="store_true", help="add the long per-group table: generated-kernel groups, tuner, bandwidth model, programs")
    ap.add_argument("--no-groups", action="store_true", help="headline group only")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--no-traffic", action="store_true", help="do not measure HBM traffic with rocprofv3 child runs (the committed figure is reported instead)")
    ap.add_argument("--spin-up", type=float, default=SPIN_UP_S,
                    help="seconds of untimed launches before each timing loop (0 for counter runs, which only need a few launches)")
    ap.add_argument("--traffic-child", default=None, help=argparse.SUPPRESS)
    args = ap.parse_args()
    if args.traffic_child:
        traffic_child(args.traffic_child)
        return
    SPIN_UP_S = max(0.0, args.spin_up)
    TUNE = args.full
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (one stitched kernel per fusion group; "
              "rows / batch elements would shard across GPUs without communication). "
              "Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    # the CPU oracle first: its worker processes are forked before this process touches the GPU
    cpu = None
    if not args.no_cpu:
        try:
            cpu = cpu_baseline()
        except Exception as e:
            cpu = {"value": None, "unit": "GB/s", "cores": 0, "kind": "oracle", "sample": f"failed: {e}"}
    import torch
    from workloads import BY_NAME, CONFIGS, EXTRA_GROUPS
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    head = BY_NAME[args.only or HEADLINE]
    res, ev_ms, wall_ms = bench_group(head, args.steps, args.warmup, with_per_op=True)
    algo = res["algorithmic_bytes"]
    groups = {head.name: res}
    if not args.no_groups:
        for cfg in CONFIGS:
            if cfg.name != head.name:
                groups[cfg.name] = bench_group(cfg, args.steps, max(5, args.warmup // 2))[0]
    traffic, traffic_detail = None, None
    if not args.no_traffic:
        torch.cuda.synchronize()
        traffic, traffic_detail = measure_traffic(head.name)
    traffic_source = "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE child runs of this command"
    if traffic is None:
        traffic_source = f"profiles/hbm_traffic_all_groups.md ({traffic_detail or 'in-run measurement switched off'})"
        traffic, traffic_detail = committed_traffic(head.name), None
    out = {
        "metric": "achieved HBM GB/s of the stitched fusion group (algorithmic bytes / time); fraction of 8 TB/s in roofline.frac",
        "value": algo / (wall_ms * 1e-3) / 1e9,
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": head.dtype, "data": "synthetic",
        "config": {"workload": f"config {head.index}: {head.name} {head.full} (largest of the five groups)", "algorithmic_bytes": algo,
                   "buffer_sets": res["buffer_sets"], "kernels_per_step": res["n_kernels"],
                   "speedup_vs_per_op": round(res.get("speedup_vs_per_op", 0.0), 2), "per_op_kernels": res.get("per_op_kernels"),
                   "configs": {f"cfg{BY_NAME[k].index}_{k}": compact(v) for k, v in sorted(groups.items(), key=lambda kv: BY_NAME[kv[0]].index)}},
        "roofline": {"bound": "hbm", "achieved": algo / (ev_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": algo / (ev_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                     "traffic_detail": traffic_detail,
                     "kernel_us": ev_ms * 1e3, "frac_of_copy_kernel": res["stitched_frac_of_copy"],
                     "note": "time of the whole plan per launch (row kernel + combine kernel where the plan has two), HIP events on the launch stream"},
    }
    if cpu is not None:
        out["cpu_baseline"] = cpu
    props = torch.cuda.get_device_properties(0)       # device facts as read at run time, not assumed
    out["device"] = {"name": props.name, "arch": getattr(props, "gcnArchName", None),
                     "compute_units": props.multi_processor_count,
                     "hbm_gib": round(props.total_memory / 2 ** 30, 1),
                     "lds_bytes_per_workgroup": getattr(props, "shared_memory_per_block", None),
                     "l2_bytes": getattr(props, "L2_cache_size", None),
                     "clock_khz": getattr(props, "clock_rate", None)}
    if args.full:
        kp = dict(shape=(64, 16, 128, 128), mask="key_padding")
        groups["scaled_masked_softmax_key_padding"] = bench_group(BY_NAME["scaled_masked_softmax"], args.steps,
                                                                  args.warmup, build_kw=kp)[0]
        for cfg in EXTRA_GROUPS:
            heavy = cfg.name == "multi_interest_pattern"        # 1.2 GB per launch, 11 ms unfused
            groups[cfg.name] = bench_group(cfg, max(20, args.steps // (25 if heavy else 4)), max(3, args.warmup // (10 if heavy else 2)))[0]
        out["groups"] = groups
        out["bandwidth_model"] = bandwidth_model()
        try:
            out["programs"] = bench_programs()
        except Exception as e:      # an extra beside the groups: report, do not fail the bench
            out["programs"] = {"error": str(e)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
