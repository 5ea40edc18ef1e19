#!/usr/bin/env python3
"""Benchmark of the stitched fusion-group kernels on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--only NAME] [--no-groups] [--no-cpu]

Prints ONE JSON line.  The headline workload is the scaled-masked-softmax group (fp32
scores [131072,128] with a full additive mask): one step = one launch of the stitched
plan over one batch of synthetic input already resident in HBM.  `value` is algorithmic
bytes (every group input read once, every output written once) per second of wall time
over the timed steps.  Input buffers rotate over enough distinct sets that the bytes
touched between two uses of a set exceed the 256 MB last-level cache.

`roofline` is the same kernel against the 8 TB/s HBM peak, from HIP events recorded on
the launch stream around the timed launches.  `groups` lists all five benchmark groups
(stitched, per-op baseline, speedup, plain-copy ceiling); `cpu_baseline` is the CPU
oracle timed on this machine's host cores.
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

HBM_PEAK_GBS = 8000.0
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_all_groups.md")


def measured_traffic(name):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary (FETCH_SIZE and
    WRITE_SIZE, each scaled by what it reads for the plain copy kernel), or None."""
    import re
    try:
        text = open(TRAFFIC_FILE).read()
    except OSError:
        return None
    m = re.search(r"traffic_bytes_per_launch\[%s\]\s*=\s*(\d+)" % re.escape(name), text)
    return int(m.group(1)) if m else None

ROTATE_BYTES = 640 * 2**20     # bytes touched between reuses of one buffer set
TUNE = True                    # also time every group after fs_plan_tune (--no-tune)
SPIN_UP_S = 0.05               # seconds of untimed launches before every timing loop (see time_plan; --spin-up)

TORCH_DT = None


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
    res.update(schedule=info["schedule"], template=template, stitched_us=ev_ms * 1e3, stitched_wall_us=wall_ms * 1e3,
               stitched_gbs=algo / (ev_ms * 1e-3) / 1e9, stitched_frac_of_peak=algo / (ev_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
               lds_bytes=info["lds_bytes"], workspace_bytes=info["workspace_bytes"])
    # the same group after the tuner (Algorithm 3's loop over templates) has timed the schedule's launch
    # templates on one buffer set and kept the fastest
    try:
        if not TUNE:
            raise RuntimeError("skipped (--no-tune)")
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
        with Plan(ops, "per_op") as plan:
            outs = [torch.empty(op.shape, dtype=_torch_dt()[op.dtype], device="cuda:0") for op in ops if op.kind == "output"]
            per_op_us = timed(lambda: plan.launch(ins, outs))
            res.update(per_op_kernels=plan.info()["n_kernels"], per_op_us=per_op_us, speedup_vs_per_op=per_op_us / fused_us)
        out[name] = res
        del ins
        torch.cuda.empty_cache()
    return out


def cpu_baseline(cfg):
    """The oracle as it stands on the host cores, on a bounded row sample of the headline
    workload (numpy runs its elementwise loops on one thread)."""
    from oracle import interp
    from workloads import algorithmic_bytes, graphs, inputs
    rows = 32768           # a quarter of the 131072 rows: a few seconds of CPU work
    ops = graphs.scaled_masked_softmax((rows, 128), 0.125, "full")
    ins = inputs.scaled_masked_softmax((rows, 128), "full")
    reps, t_total = 0, 0.0
    while t_total < 10.0 and reps < 50:
        t0 = time.perf_counter()
        interp.run(ops, ins)
        t_total += time.perf_counter() - t0
        reps += 1
    sec = t_total / reps
    cpu = None
    try:
        with open("/proc/cpuinfo") as f:
            cpu = next((l.split(":", 1)[1].strip() for l in f if l.startswith("model name")), None)
    except OSError:
        pass
    return {"value": algorithmic_bytes(ops) / sec / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"{rows} of 131072 rows of the same workload, {reps} repetitions, mean",
            "ms_per_sample": sec * 1e3, "cpu_model": cpu}


def main():
    global SPIN_UP_S, TUNE
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--only", default=None, help="time just this group as the headline (a config name)")
    ap.add_argument("--no-groups", action="store_true", help="skip the per-group table")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--spin-up", type=float, default=SPIN_UP_S,
                    help="seconds of untimed launches before each timing loop (0 for counter runs, which only need a few launches)")
    ap.add_argument("--no-tune", action="store_true", help="skip the timing of each group after the tuner (counter runs)")
    args = ap.parse_args()
    SPIN_UP_S = max(0.0, args.spin_up)
    TUNE = not args.no_tune
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (one stitched kernel per fusion group; "
              "rows / batch elements would shard across GPUs without communication). "
              "Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import torch
    from workloads import BY_NAME, CONFIGS, EXTRA_GROUPS
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    head = BY_NAME[args.only or "scaled_masked_softmax"]
    res, ev_ms, wall_ms = bench_group(head, args.steps, args.warmup, with_per_op=True)
    algo = res["algorithmic_bytes"]
    out = {
        "metric": "achieved HBM GB/s of the stitched fusion group (algorithmic bytes / time); fraction of 8 TB/s in roofline.frac",
        "value": algo / (wall_ms * 1e-3) / 1e9,
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": head.dtype, "data": "synthetic",
        "config": {"workload": f"{head.name} {head.full}", "algorithmic_bytes": algo,
                   "buffer_sets": res["buffer_sets"], "speedup_vs_per_op": res.get("speedup_vs_per_op"),
                   "per_op_kernels": res.get("per_op_kernels")},
        "roofline": {"bound": "hbm", "achieved": algo / (ev_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": algo / (ev_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "traffic": measured_traffic(head.name),
                     "kernel_us": ev_ms * 1e3, "frac_of_copy_kernel": res["stitched_frac_of_copy"]},
    }
    props = torch.cuda.get_device_properties(0)       # device facts as read at run time, not assumed
    out["device"] = {"name": props.name, "arch": getattr(props, "gcnArchName", None),
                     "compute_units": props.multi_processor_count,
                     "hbm_gib": round(props.total_memory / 2 ** 30, 1),
                     "lds_bytes_per_workgroup": getattr(props, "shared_memory_per_block", None),
                     "l2_bytes": getattr(props, "L2_cache_size", None),
                     "clock_khz": getattr(props, "clock_rate", None),
                     "memory_clock_khz": getattr(props, "memory_clock_rate", None),
                     "memory_bus_bits": getattr(props, "memory_bus_width", None)}
    if not args.no_groups:
        groups = {head.name: res}
        for cfg in CONFIGS:
            if cfg.name == head.name:
                continue
            steps = args.steps if cfg.index != 5 else max(20, args.steps // 4)
            groups[cfg.name] = bench_group(cfg, steps, max(5, args.warmup // 2))[0]
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
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(head)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
