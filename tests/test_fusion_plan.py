"""Fusion planning (Section 4): the oracle against hand-checked cases and the definitions, and
the library's planner against the oracle."""
import random

import pytest

from oracle import fusion as of
from paper_1911_11576_amd import FsError, FusionPlan, Plan, binding
from workloads import graphs
from workloads.graphs import Graph

TABLE = [(1 << 20, 500.0), (16 << 20, 2500.0), (256 << 20, 6000.0), (1 << 30, 6500.0)]
PHI = 3.0


# ---------------------------------------------------------------- oracle pins

def _chain():
    """x -> a = exp(x) -> b = a * 2 -> c = tanh(b) -> out; a also feeds a second output."""
    g = Graph()
    x = g.parameter("x", "f32", (1024, 1024))
    a = g.exp(x)
    b = g.multiply(a, g.constant(2.0))
    c = g.tanh(b)
    g.output(c)
    g.output(a)
    return g.ops, (a, b, c)


def test_oracle_traffic_and_saved_bytes_by_hand():
    ops, (a, b, c) = _chain()
    S = 1024 * 1024 * 4
    # one kernel per op: a reads x writes a; b reads a writes b; c reads b writes c  -> 6 S
    assert of.traffic(ops, [[a], [b], [c]]) == 6 * S
    # all three fused: read x, write a (an output) and c -> 3 S; b never leaves the chip
    assert of.traffic(ops, [[a, b, c]]) == 3 * S
    assert of.saved_bytes(ops, [a, b, c]) == 3 * S
    # b and c fused: read a, write c: saves b's write and read
    assert of.saved_bytes(ops, [b, c]) == 2 * S
    # a and b fused: a still has to be written (it is an output), its read by b is saved
    assert of.saved_bytes(ops, [a, b]) == 1 * S
    # an input read by two ops of the pattern is read once
    g = Graph()
    x = g.parameter("x", "f32", (256, 256))
    u, v = g.exp(x), g.tanh(x)
    g.output(g.add(u, v))
    s = 256 * 256 * 4
    assert of.saved_bytes(g.ops, [u, v, u + 2]) == (2 * s + 2 * s) + s      # u, v written+read; x read once instead of twice


def test_oracle_model_and_score():
    assert of.model_us(TABLE, 0) == 0.0
    assert of.model_us(TABLE, 1 << 20) == pytest.approx((1 << 20) / 500e9 * 1e6)
    assert of.model_us(TABLE, 1 << 10) == pytest.approx((1 << 10) / 500e9 * 1e6)       # below the table: first rate
    assert of.model_us(TABLE, 1 << 31) == pytest.approx((1 << 31) / 6500e9 * 1e6)      # above: last rate
    mid = 4 << 20                                                                     # halfway in log between 1 and 16 MiB
    assert of.model_us(TABLE, mid) == pytest.approx(mid / 1500e9 * 1e6)
    ops, (a, b, c) = _chain()
    S = 1024 * 1024 * 4
    assert of.score(ops, [a, b, c], TABLE, PHI) == pytest.approx(of.model_us(TABLE, 3 * S) + 2 * PHI)


def test_oracle_convexity_on_the_papers_cycle_example():
    # A -> B -> C and A -> C (the cyclic-dependence figure): fusing A and C puts B on a cycle
    g = Graph()
    x = g.parameter("x", "f32", (64, 64))
    A = g.exp(x)
    B = g.tanh(A)
    Cn = g.add(A, B)
    g.output(Cn)
    assert not of.is_convex(g.ops, [A, Cn])
    assert of.is_convex(g.ops, [A, B]) and of.is_convex(g.ops, [B, Cn]) and of.is_convex(g.ops, [A, B, Cn])
    assert not of.contraction_is_acyclic(g.ops, [[A, Cn]])
    assert of.contraction_is_acyclic(g.ops, [[A, B]])
    # looking through a broadcast: a per-row value used by a full op is a data-flow edge
    ops = graphs.log_softmax((8, 64))
    prod, cons = of.flow(ops)
    kinds = [op.kind for op in ops]
    mx = kinds.index("reduce_max")
    sub = kinds.index("subtract")
    assert mx in prod[sub] and sub in cons[mx]


def test_oracle_substitution_segments_and_brute_force():
    ops = graphs.log_softmax((8, 64))
    red = lambda op: op.kind in ("reduce_sum", "reduce_max")
    segs = of.substitution_segments(ops, red)
    kinds = [[ops[i].kind for i in s] for s in segs]
    assert kinds == [["subtract", "exp"], ["log", "subtract"]]       # what lies between the reductions
    assert of.substitution_segments(ops, lambda op: False) == [[i for i, op in enumerate(ops) if of.owns_kernel(op)]]
    # brute force: overlapping patterns exclude each other, the better combination wins
    ops, (a, b, c) = _chain()
    best, sets = of.best_selection(ops, [[a, b], [b, c], [a, b, c]], [5.0, 4.0, 8.0])
    assert best == 8.0 and sets == [(2,)]
    best, sets = of.best_selection(ops, [[a, b], [b, c], [a, b, c]], [5.0, 4.0, -1.0])
    assert best == 5.0 and sets == [(0,)]


# ---------------------------------------------------------------- the library's planner

def _check_plan(ops, fp, brute_force=True):
    owned = [i for i, op in enumerate(ops) if of.owns_kernel(op)]
    # every scored pattern: what the oracle computes for the same op set
    for p in fp.patterns:
        assert all(of.owns_kernel(ops[o]) for o in p["ops"])
        if p["score_us"] < 0:
            continue
        assert of.is_convex(ops, p["ops"])
        assert p["saved_bytes"] == of.saved_bytes(ops, p["ops"])
        assert p["score_us"] == pytest.approx(of.score(ops, p["ops"], TABLE, PHI), rel=1e-9)
    # Algorithm 1 under the four partition sets
    is_dot = lambda op: op.kind == "dot"
    is_red = lambda op: op.kind in ("reduce_sum", "reduce_max")
    not_row = lambda op: is_red(op) and op.axis != len(ops[op.operands[0]].shape) - 1
    # (a segment that was first met as a connected part of a larger one keeps that origin)
    have = {tuple(p["ops"]) for p in fp.patterns if p["origin"] in (0, 1)}
    for part in (is_dot, lambda op: is_dot(op) or not_row(op), lambda op: is_dot(op) or is_red(op)):
        for seg in of.substitution_segments(ops, part):
            if len(seg) <= 128:          # (a pattern holds at most 128 ops)
                assert tuple(seg) in have, seg
    # the plan: disjoint, acyclic, covers every kernel once, in data-flow order
    chosen = [p["ops"] for p in fp.patterns if p["chosen"]]
    flat = [o for c in chosen for o in c]
    assert len(flat) == len(set(flat))
    assert of.contraction_is_acyclic(ops, chosen)
    assert fp.total_score_us == pytest.approx(sum(p["score_us"] for p in fp.patterns if p["chosen"]))
    members = [o for g in fp.groups for o in g["members"]]
    assert sorted(members) == owned
    produced = {i for i, op in enumerate(ops) if op.kind == "parameter"}
    for g in fp.groups:
        assert set(g["input_of"]) <= produced, "a group runs before its inputs exist"
        produced |= set(g["output_of"])
        assert set(g["output_of"]) <= set(g["members"])
    for i, op in enumerate(ops):
        if op.kind == "output":
            src = op.operands[0]
            assert src in produced
    # optimal among its own candidates (brute force, small candidate sets only)
    cands = [p for p in fp.patterns if p["score_us"] >= 0]
    if brute_force and len(cands) <= 14:
        best, _ = of.best_selection(ops, [p["ops"] for p in cands], [p["score_us"] for p in cands])
        assert fp.total_score_us == pytest.approx(best)


GRAPHS = {
    "log_softmax": lambda: graphs.log_softmax((4096, 1024)),
    "layernorm_bwd": lambda: graphs.layernorm_bwd(4096, 1024),
    "encoder_tail": lambda: graphs.encoder_tail(4096, 1024, 64, 128),
    "crossing": lambda: graphs.crossing_branches(4096, 1024),
    "multi_interest": lambda: graphs.multi_interest_pattern(64),
    "adam": lambda: graphs.adam_update((4096, 1024)),
}


@pytest.mark.parametrize("name", sorted(GRAPHS))
def test_planner_against_the_oracle(name):
    ops = GRAPHS[name]()
    fp = FusionPlan(ops, launch_us=PHI, bandwidth=TABLE)
    _check_plan(ops, fp)
    # without the exploratory search the candidate set is small enough for the brute force
    fp2 = FusionPlan(ops, launch_us=PHI, bandwidth=TABLE, explore_budget=-1)
    assert all(p["origin"] != 2 for p in fp2.patterns)
    _check_plan(ops, fp2)
    assert fp.total_score_us >= fp2.total_score_us - 1e-9


def test_whole_groups_are_found_where_one_kernel_can_run_them():
    for ops in (graphs.log_softmax((4096, 1024)), graphs.layernorm_bwd(4096, 1024), graphs.adam_update((4096, 1024)),
                graphs.multi_interest_pattern(4096), graphs.bias_gelu_residual_layernorm(4096, 1024, "bf16")):
        fp = FusionPlan(ops)
        assert len(fp.groups) == 1 and fp.groups[0]["score_us"] > 0
        with Plan(fp.groups[0]["ops"]) as p:          # the group's own op list plans like the original
            assert p.info()["schedule"] != "per_op"
    fp = FusionPlan(graphs.encoder_tail(4096, 1024, 64, 128))
    big = max(fp.groups, key=lambda g: len(g["members"]))
    assert len(big["members"]) >= 20 and len(big["output_of"]) == 2       # the LayerNorm branch with both its outputs


def test_fine_grained_dots_do_not_part_the_graph():
    # a dot whose tile one workgroup's matrix-unit schedule holds (Section 5.1: batched GEMMs of fine granularity are
    # composed with the ops around them) is fusible; a larger one is a library call and parts the graph
    for ops, sched in ((graphs.causal_attention(512, 64, 64), "bdot_softmax"), (graphs.sigmoid_attention(512, 64, 64, 64, 64), "block_dot"),
                       (graphs.attention_residual_layernorm(512, 64, 64, 64), "block_dot")):
        fp = FusionPlan(ops)
        owned = [i for i, op in enumerate(ops) if of.owns_kernel(op)]
        whole = [p for p in fp.patterns if p["ops"] == owned]
        assert len(whole) == 1 and whole[0]["score_us"] > 0 and whole[0]["origin"] == 0      # found by the first substitution step
        with Plan(whole[0]["group_ops"]) as p:
            assert p.info()["schedule"] == sched and p.info()["n_kernels"] == 1
        # (the model may still prefer two groups: two small savings score a little higher than one large one)
        assert len(fp.groups) <= 2 and all(len(g["members"]) > 1 for g in fp.groups)
    fp = FusionPlan(graphs.attention_block(4, 64, 256, 64))          # 256 keys: beyond the fine-grained tile
    dots = [i for i, op in enumerate(graphs.attention_block(4, 64, 256, 64)) if op.kind == "dot"]
    for d in dots:
        assert any(g["members"] == [d] for g in fp.groups)


def test_cycle_repair_between_two_chains_that_feed_each_other():
    """Two chains that feed each other: each is a valid pattern, together they are cyclic.  The
    solver's first answer takes both; the repair forbids the pair and the second answer is the
    best acyclic selection.  The per-column chain is a connected same-shape part of the graph's one
    segment, so the planner meets the cycle on its own; supplying the chain changes nothing."""
    ops = graphs.crossing_branches(4096, 1024)
    kinds = [op.kind for op in ops]
    b_chain = [kinds.index("tanh"), kinds.index("tanh") + 2, len(ops) - 3]      # b1, n, b2
    assert [ops[i].shape for i in b_chain] == [(1024,)] * 3
    fp = FusionPlan(ops, launch_us=PHI, bandwidth=TABLE, extra_patterns=[b_chain])
    assert fp.solver_rounds == 2
    assert any(p["origin"] in (1, 3) and p["ops"] == sorted(b_chain) and p["score_us"] > 0 for p in fp.patterns)
    _check_plan(ops, fp)                      # acyclic, and the brute-force optimum over the same candidates
    own = FusionPlan(ops, launch_us=PHI, bandwidth=TABLE)
    assert own.solver_rounds == 2 and own.total_score_us == pytest.approx(fp.total_score_us)
    _check_plan(ops, own)
    # without that candidate nothing is cyclic: substitution segments of a graph cut only at its reductions
    assert FusionPlan(graphs.log_softmax((4096, 1024)), launch_us=PHI, bandwidth=TABLE).solver_rounds == 1


def test_scalars_between_groups_clip_by_global_norm():
    """A value reduced over everything feeds ops on the full tensors: no single kernel covers the
    graph.  The planner must fuse each tensor's square with its first reduction, the scalar
    arithmetic behind the reductions into one kernel, and the final scalings of all tensors into one
    kernel of independent parts -- and every group, scalar parameters included, must plan."""
    shapes = [(300, 1024), (1024,), (64, 3, 50)]
    ops = graphs.clip_by_global_norm(shapes, 5.0)
    fp = FusionPlan(ops, launch_us=PHI, bandwidth=TABLE)
    _check_plan(ops, fp, brute_force=False)
    kinds = lambda g: sorted(ops[o].kind for o in g["members"])
    assert ["add", "add", "divide", "divide", "maximum", "sqrt"] in [kinds(g) for g in fp.groups]
    assert ["multiply"] * len(shapes) in [kinds(g) for g in fp.groups]          # the scalings, packed
    assert sum(kinds(g) == ["multiply", "reduce_sum"] for g in fp.groups) == 2
    assert ["multiply", "reduce_sum", "reduce_sum"] in [kinds(g) for g in fp.groups]     # rank 3: two links of the chain merge
    assert len(fp.groups) == 7 < sum(1 for op in ops if of.owns_kernel(op))
    for g in fp.groups:
        with Plan(g["ops"]) as p:
            assert p.info()["schedule"] != "per_op"


def test_segments_longer_than_a_pattern_are_cut_into_stretches():
    """A stack of row-local layers with no partition op between them: up to the pattern size the whole
    stack is one group (one row kernel, rows stay in registers across the layers); beyond it the segment's
    consecutive stretches of that size are the candidates, and the plan is a few large groups -- not
    the pieces between reductions."""
    ops = graphs.encoder_tail_stack(3, 4096, 1024)
    fp = FusionPlan(ops, launch_us=PHI, bandwidth=TABLE)
    assert len(fp.groups) == 1
    _check_plan(ops, fp, brute_force=False)
    ops = graphs.encoder_tail_stack(12, 4096, 1024)
    owned = sum(1 for op in ops if of.owns_kernel(op))
    assert owned > 2 * 128
    fp = FusionPlan(ops, launch_us=PHI, bandwidth=TABLE)
    _check_plan(ops, fp, brute_force=False)
    assert len(fp.groups) <= 4 and max(len(g["members"]) for g in fp.groups) == 128
    for g in fp.groups:
        with Plan(g["ops"]) as p:
            assert p.info()["schedule"] == "row" and p.info()["n_kernels"] == 1


def test_random_elementwise_graphs():
    rng = random.Random(7)
    for trial in range(6):
        g = Graph()
        vals = [g.parameter(f"p{k}", "f32", (2048, 1024)) for k in range(2)]
        for _ in range(rng.randint(4, 9)):
            kind = rng.choice(["add", "multiply", "exp", "tanh", "subtract"])
            if kind in ("exp", "tanh"):
                vals.append(getattr(g, kind)(rng.choice(vals)))
            else:
                vals.append(getattr(g, kind)(rng.choice(vals), rng.choice(vals)))
        used = {o for op in g.ops for o in op.operands}
        for v in vals[2:]:
            if v not in used:
                g.output(v)
        if not any(op.kind == "output" for op in g.ops):
            g.output(vals[-1])
        fp = FusionPlan(g.ops, launch_us=PHI, bandwidth=TABLE, explore_budget=40)
        _check_plan(g.ops, fp)


@pytest.mark.parametrize("seed", range(10))
def test_random_programs_are_cut_into_valid_groups(seed):
    """Graphs that need several dependent groups (reductions over either dim as intermediates):
    scores against the oracle, disjointness, order, acyclicity; and the exploratory search must
    have found more than the substitution segments alone."""
    rng = random.Random(100 + seed)
    ops, _ = graphs.random_program(rng, 600, 1024, n_ops=rng.randint(10, 40))
    fp = FusionPlan(ops, launch_us=PHI, bandwidth=TABLE)
    _check_plan(ops, fp)
    assert all(p["score_us"] >= 0 for p in fp.patterns if p["origin"] == 2)      # the search only keeps valid patterns
    without = FusionPlan(ops, launch_us=PHI, bandwidth=TABLE, explore_budget=-1)
    assert fp.total_score_us >= without.total_score_us - 1e-9
    owned = sum(1 for op in ops if of.owns_kernel(op))
    assert len(fp.groups) <= max(2, (2 * owned) // 3)                            # it does fuse


def test_measured_scores_replace_the_models_and_the_selection_follows():
    """Section 4.3's hybrid policy: a pattern the caller has run carries the time it was measured to save; the
    selection is the brute-force optimum over the candidates with those figures in place of the model's."""
    ops = graphs.encoder_tail(4096, 1024, 64, 128)
    base = FusionPlan(ops, launch_us=PHI, bandwidth=TABLE, explore_budget=-1)
    usable = [p for p in base.patterns if p["score_us"] >= 0]
    assert len(usable) >= 3 and all("group_ops" in p and not p["measured"] for p in usable)
    for p in usable:      # a candidate's op list plans on its own, and stands for the same ops
        assert len(p["output_of"]) >= 1 and set(p["output_of"]) <= set(p["ops"])
    with Plan(usable[0]["group_ops"]) as plan:
        assert plan.info()["schedule"] != "per_op"
    assert all("group_ops" not in p for p in base.patterns if p["score_us"] < 0)
    chosen = [p for p in base.patterns if p["chosen"]]
    loser = max(chosen, key=lambda p: p["score_us"])
    others = [p for p in usable if not p["chosen"]]
    winner = others[0]
    # the best chosen pattern was measured to lose, one the model passed over to win big; one entry says nothing
    quiet = next(p for p in usable if p is not loser and p is not winner)
    extra = [loser["ops"], list(reversed(winner["ops"])), quiet["ops"]]
    fp = FusionPlan(ops, launch_us=PHI, bandwidth=TABLE, explore_budget=-1, extra_patterns=extra, extra_scores=[-4.0, 1e4, None])
    by_ops = {tuple(p["ops"]): p for p in fp.patterns}
    assert len(fp.patterns) == len(base.patterns)                      # the same candidates, not new ones
    lo, wi, silent = by_ops[tuple(loser["ops"])], by_ops[tuple(winner["ops"])], by_ops[tuple(quiet["ops"])]
    assert lo["measured"] and lo["score_us"] == -4.0 and not lo["chosen"]
    assert wi["measured"] and wi["score_us"] == 1e4 and wi["chosen"]
    assert not silent["measured"] and silent["score_us"] == pytest.approx(quiet["score_us"])
    for p in fp.patterns:
        if not p["measured"] and p["score_us"] >= 0:
            assert p["score_us"] == pytest.approx(of.score(ops, p["ops"], TABLE, PHI), rel=1e-9)
    cands = [p for p in fp.patterns if p["score_us"] >= 0]
    assert fp.total_score_us == pytest.approx(sum(p["score_us"] for p in cands if p["chosen"]))
    if len(cands) <= 16:
        best, _ = of.best_selection(ops, [p["ops"] for p in cands], [p["score_us"] for p in cands])
        assert fp.total_score_us == pytest.approx(best)
    # a measurement for a pattern no kernel can be built for changes nothing
    bad = next((p for p in base.patterns if p["score_us"] < 0), None)
    if bad is not None:
        fp2 = FusionPlan(ops, launch_us=PHI, bandwidth=TABLE, explore_budget=-1, extra_patterns=[bad["ops"]], extra_scores=[50.0])
        again = {tuple(p["ops"]): p for p in fp2.patterns}[tuple(bad["ops"])]
        assert again["score_us"] < 0 and not again["measured"] and not again["chosen"]
    with pytest.raises(ValueError):
        FusionPlan(ops, extra_patterns=[loser["ops"]], extra_scores=[1.0, 2.0])
    for bad_score in (float("inf"), -float("inf"), 1e300):
        with pytest.raises(FsError):
            FusionPlan(ops, extra_patterns=[loser["ops"]], extra_scores=[bad_score])


def test_planner_rejects_bad_input():
    ops = graphs.log_softmax((64, 64))
    with pytest.raises(FsError) as e:
        FusionPlan(ops, max_patterns=300)
    assert e.value.status == binding.FS_ERR_INVALID
    with pytest.raises(FsError) as e:
        FusionPlan(ops, bandwidth=[(100, 5.0), (50, 6.0)])
    assert e.value.status == binding.FS_ERR_INVALID
    with pytest.raises(FsError) as e:
        FusionPlan(ops, extra_patterns=[[0, 1]])        # a parameter owns no kernel
    assert e.value.status == binding.FS_ERR_INVALID
