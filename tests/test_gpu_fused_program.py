"""End to end: a computation graph larger than one fusion group is planned (Section 4), every
group becomes a stitched plan, the groups run in order on the GPU, and the program's outputs
are compared with the oracle's evaluation of the whole graph."""
import sys

import pytest
import torch

from oracle import interp
from paper_1911_11576_amd import FusedProgram, Plan
from workloads import TOLERANCE, graphs, inputs

from gpu_util import assert_close, to_device

pytestmark = pytest.mark.gpu


def announce(msg):
    sys.__stderr__.write(f"[gpu-case] {msg}\n")
    sys.__stderr__.flush()


@pytest.fixture(autouse=True)
def _need_gpu(device):
    yield


def _encoder_inputs(rows, cols, batch, seq):
    s, m = inputs.scaled_masked_softmax((batch, 1, seq, seq), "key_padding")
    x, bias, res, gamma, beta = inputs.bias_gelu_residual_layernorm(rows, cols, "f32")
    return [s.reshape(batch, seq, seq), m.reshape(batch, 1, seq), x, bias, res, gamma, beta]


def _run(ops, ins, **kw):
    dev_in = to_device(ops, ins)
    with FusedProgram(ops, **kw) as prog:
        outs = prog.run(dev_in)
        torch.cuda.synchronize()
        got = [t.to(torch.float64).cpu().numpy() for t in outs]
        return got, prog.n_kernels, len(prog.fusion.groups)


def test_encoder_tail_runs_as_a_few_stitched_groups():
    announce("fused program encoder tail")
    rows, cols, batch, seq = 300, 1024, 6, 128
    ops, ins = graphs.encoder_tail(rows, cols, batch, seq), _encoder_inputs(rows, cols, batch, seq)
    want = interp.run(ops, ins)
    got, n_kernels, n_groups = _run(ops, ins)
    for a, b in zip(got, want):
        assert_close(a, b, TOLERANCE["f32"], "encoder tail")
    with Plan(ops, "per_op") as p:
        unfused = p.info()["n_kernels"]
    assert n_kernels < unfused / 4          # 30-odd kernels become a handful
    # planning options change the grouping, never the result
    for kw in (dict(explore_budget=-1), dict(launch_us=10.0), dict(max_patterns=4)):
        again, _, _ = _run(ops, ins, **kw)
        for a, b in zip(again, want):
            assert_close(a, b, TOLERANCE["f32"], f"encoder tail {kw}")


def test_crossing_branches_after_cycle_repair():
    announce("fused program crossing branches")
    ops = graphs.crossing_branches(257, 512)
    ins = inputs.normal_tensors([(257, 512), (512,)], scale=0.5)
    want = interp.run(ops, ins)
    kinds = [op.kind for op in ops]
    b_chain = [kinds.index("tanh"), kinds.index("tanh") + 2, len(ops) - 3]
    for kw in ({}, dict(extra_patterns=[b_chain])):
        got, _, _ = _run(ops, ins, **kw)
        for a, b in zip(got, want):
            assert_close(a, b, TOLERANCE["f32"], f"crossing branches {kw}")


@pytest.mark.parametrize("rows,cols", [(300, 1024), (33, 4096), (517, 96)])
def test_encoder_tail_backward_is_one_group(rows, cols):
    """LayerNorm backward, GELU backward and the three parameter gradients of a Transformer block's
    tail: 38 per-op kernels; the planner makes one group of it, which runs as the row kernel
    with three packed column sums plus the combine kernel."""
    announce(f"fused program encoder tail backward {rows}x{cols}")
    ops, ins = graphs.encoder_tail_bwd(rows, cols), inputs.encoder_tail_bwd(rows, cols)
    want = interp.run(ops, ins)
    got, n_kernels, n_groups = _run(ops, ins)
    assert n_groups == 1 and n_kernels == 2
    for a, b in zip(got, want):
        assert_close(a, b, TOLERANCE["f32"], "encoder tail backward")


@pytest.mark.parametrize("name", ["layernorm_bwd", "multi_interest", "adam"])
def test_single_group_graphs_through_the_planner(name):
    announce(f"fused program {name}")
    if name == "layernorm_bwd":
        ops, ins = graphs.layernorm_bwd(517, 1024), inputs.layernorm_bwd(517, 1024)
    elif name == "multi_interest":
        ops, ins = graphs.multi_interest_pattern(7), inputs.multi_interest_pattern(7)
    else:
        ops, ins = graphs.adam_update((129, 512)), inputs.adam_update((129, 512))
    want = interp.run(ops, ins)
    got, _, _ = _run(ops, ins)
    for a, b in zip(got, want):
        assert_close(a, b, TOLERANCE["f32"], name)


@pytest.mark.parametrize("seed", range(16))
def test_random_programs_through_the_planner(seed):
    """Random graphs over full, per-row and per-column values with reductions over either dim as
    intermediates: the planner has to cut them into several dependent groups (a column-reduced value
    ends its group; its readers start new ones), every group runs as its stitched plan, and the
    program's outputs must match the oracle's evaluation of the whole graph."""
    import random
    rng = random.Random(100 + seed)
    rows, cols = [(600, 1024), (257, 96), (64, 4096), (1000, 30)][seed % 4]
    ops, pshapes = graphs.random_program(rng, rows, cols, n_ops=rng.randint(10, 40))
    ins = inputs.normal_tensors(pshapes, seed_offset=400 + seed)
    announce(f"random program seed {seed} {rows}x{cols}: {len(ops)} ops")
    want = interp.run(ops, ins)
    got, n_kernels, n_groups = _run(ops, ins, seed_bytes=1)      # every fusible op may seed the exploratory search
    for a, b in zip(got, want):
        assert_close(a, b, TOLERANCE["f32"], f"random program {seed}")
    with Plan(ops, "per_op") as p:
        assert n_kernels <= p.info()["n_kernels"]


@pytest.mark.parametrize("name", ["encoder_tail", "clip", "random"])
def test_planning_with_measured_scores(name):
    """Section 4.3's hybrid policy end to end: the plan's patterns and the best other candidates are built and
    timed against one kernel per op, the plan is made again with those measurements, and the program that comes
    out computes what the oracle computes.  The measured patterns carry their measurement, and the selection is
    the best one over the scores it was given."""
    import random
    announce(f"measured planning {name}")
    if name == "encoder_tail":
        rows, cols, batch, seq = 300, 1024, 6, 128
        ops, ins = graphs.encoder_tail(rows, cols, batch, seq), _encoder_inputs(rows, cols, batch, seq)
    elif name == "clip":
        shapes = [(300, 256), (1000,), (64, 64), (5, 7, 11)]
        ops, ins = graphs.clip_by_global_norm(shapes), inputs.normal_tensors(shapes, seed_offset=77)
    else:
        rng = random.Random(111)
        ops, pshapes = graphs.random_program(rng, 600, 1024, n_ops=30)
        ins = inputs.normal_tensors(pshapes, seed_offset=411)
    want = interp.run(ops, ins)
    prog, report = FusedProgram.measured(ops, top=6, trials=5)
    with prog:
        assert report and all(len(r) == 3 for r in report)
        by_ops = {tuple(p["ops"]): p for p in prog.fusion.patterns}
        for pat_ops, model_us, saved_us in report:
            p = by_ops[tuple(pat_ops)]
            assert p["measured"] and p["score_us"] == pytest.approx(saved_us)
            assert model_us >= 0
        chosen = [p for p in prog.fusion.patterns if p["chosen"]]
        assert all(p["score_us"] >= 0 for p in chosen)
        assert prog.fusion.total_score_us == pytest.approx(sum(p["score_us"] for p in chosen))
        outs = prog.run(to_device(ops, ins))
        torch.cuda.synchronize()
        for a, b in zip(outs, want):
            assert_close(a.to(torch.float64).cpu().numpy(), b, TOLERANCE["f32"], f"measured planning {name}")


def test_fused_program_as_a_captured_graph():
    """The groups of a planned graph recorded into one HIP graph: replayed with new input values and
    eager work in between, every replay against the oracle; and timed against launching group by group."""
    import random
    import time
    rng = random.Random(105)
    ops, pshapes = graphs.random_program(rng, 600, 1024, n_ops=rng.randint(10, 40))
    ins = inputs.normal_tensors(pshapes, seed_offset=405)
    announce(f"fused program as a graph: {len(ops)} ops")
    dev_in = to_device(ops, ins)
    with FusedProgram(ops, seed_bytes=1) as prog:
        graph, outs = prog.capture(dev_in)
        assert len(prog.plans) >= 3
        for rep, scale in enumerate([1.0, -0.5, 2.0]):
            cur = [inputs.round_to(a * scale, "f32") if k == 0 else a for k, a in enumerate(ins)]
            dev_in[0].copy_(to_device(ops, cur)[0])
            for t in outs:
                t.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for got, ref in zip(outs, interp.run(ops, cur)):
                assert_close(got.double().cpu().numpy(), ref, TOLERANCE["f32"], f"fused program graph replay {rep}")
        def timed(fn, n=200):
            for _ in range(10):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(n):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / n * 1e6
        eager_us, graph_us = timed(prog.run_bound), timed(graph.replay)
        announce(f"  {len(prog.plans)} groups, {prog.n_kernels} kernels: {eager_us:.1f} us launched one by one, {graph_us:.1f} us as a graph")


def test_fused_program_tuned_group_by_group():
    announce("fused program, tuned")
    rows, cols, batch, seq = 300, 1024, 6, 128
    ops, ins = graphs.encoder_tail(rows, cols, batch, seq), _encoder_inputs(rows, cols, batch, seq)
    want = interp.run(ops, ins)
    dev_in = to_device(ops, ins)
    with FusedProgram(ops) as prog:
        outs = prog.tune(dev_in, trials=3)
        torch.cuda.synchronize()
        for a, b in zip(outs, want):
            assert_close(a.double().cpu().numpy(), b, TOLERANCE["f32"], "tuned program, outputs of the tuning run")
        assert all(p.tuned is not None for p in prog.plans)
        again = prog.run(dev_in)
        torch.cuda.synchronize()
        for a, b in zip(again, want):
            assert_close(a.double().cpu().numpy(), b, TOLERANCE["f32"], "tuned program, ordinary run")


def test_plans_compared_by_execution():
    """Whole plans under different planning options, timed on the device; the fastest is kept and is still right."""
    import random
    announce("plans compared by execution")
    rng = random.Random(111)
    ops, pshapes = graphs.random_program(rng, 600, 1024, n_ops=36)
    ins = inputs.normal_tensors(pshapes, seed_offset=411)
    dev_in = to_device(ops, ins)
    prog, us, kw = FusedProgram.best_of(ops, dev_in, trials=5)
    try:
        assert us > 0 and isinstance(kw, dict)
        outs = prog.run_bound()
        torch.cuda.synchronize()
        for a, b in zip(outs, interp.run(ops, ins)):
            assert_close(a.double().cpu().numpy(), b, TOLERANCE["f32"], "best plan by execution")
    finally:
        prog.close()


@pytest.mark.parametrize("max_norm", [5.0, 1e6])
def test_clip_by_global_norm_passes_scalars_between_groups(max_norm):
    """Three tensors of different shapes, their global norm, every tensor scaled by the clipping
    factor: reductions down to scalars, scalar arithmetic as a group of its own, the factor broadcast
    back into one kernel of independent parts.  With max_norm far above the norm the factor is 1."""
    announce(f"fused program clip by global norm {max_norm}")
    shapes = [(300, 1024), (1024,), (64, 3, 50)]
    ops = graphs.clip_by_global_norm(shapes, max_norm)
    ins = inputs.normal_tensors(shapes, "f32", seed_offset=33)
    want = interp.run(ops, ins)
    got, n_kernels, n_groups = _run(ops, ins)
    for a, b in zip(got, want):
        assert_close(a, b, TOLERANCE["f32"], "clip by global norm")
    with Plan(ops, "per_op") as p:
        assert n_kernels < p.info()["n_kernels"]


@pytest.mark.parametrize("n_layers", [3, 8])
def test_stack_of_row_local_layers(n_layers):
    """Layers with no partition op between them: the planner makes one group of three layers (one row
    kernel with six reductions) and cuts eight layers into stretches of at most 128 ops."""
    announce(f"fused program stack of {n_layers} layers")
    rows, cols = 150, 512
    ops = graphs.encoder_tail_stack(n_layers, rows, cols)
    ins = inputs.normal_tensors([(rows, cols)] + [(cols,)] * (3 * n_layers), "f32", seed_offset=60, scale=0.7)
    want = interp.run(ops, ins)
    got, n_kernels, n_groups = _run(ops, ins)
    assert n_groups == (1 if n_layers == 3 else 2) and n_kernels == n_groups
    for a, b in zip(got, want):
        assert_close(a, b, TOLERANCE["f32"], f"stack of {n_layers} layers")


@pytest.mark.parametrize("name", ["causal_attention", "attention_residual_layernorm", "sigmoid_attention"])
def test_fine_grained_dots_are_fused_with_the_ops_around_them(name):
    """Section 5.1 composes batched GEMMs of fine granularity with the memory-intensive ops around them: the planner
    does not part the graph at such dots.  With the model's scores the whole graph is one group or two (the
    bandwidth table makes two small savings look a little better than one large one); with measured scores
    (Section 4.3's hybrid policy) it is one group and one kernel on the matrix unit."""
    from workloads import BY_NAME
    cfg = BY_NAME[name]
    announce(f"fused program around fine-grained dots: {name}")
    ops, ins = cfg.graph_fn(**cfg.full), cfg.input_fn(**cfg.full)
    want = interp.run(ops, ins)
    got, n_kernels, n_groups = _run(ops, ins)
    assert n_groups <= 2 and n_kernels <= 2
    for a, b in zip(got, want):
        assert_close(a, b, TOLERANCE[cfg.dtype], name)
    prog, report = FusedProgram.measured(ops)
    with prog:
        assert len(prog.fusion.groups) == 1 and prog.n_kernels == 1, [(len(r[0]), r[1], r[2]) for r in report]
        outs = prog.run(to_device(ops, ins))
        torch.cuda.synchronize()
        for a, b in zip(outs, want):
            assert_close(a.to(torch.float64).cpu().numpy(), b, TOLERANCE[cfg.dtype], name + " (measured plan)")
