"""GPU parity: the stitched kernels (and the per-op baseline), called through the C ABI,
against the CPU oracle, element by element on the same seeded inputs.

Bar: |gpu - oracle| <= tol + tol*|oracle| with tol = 1e-5 for fp32 groups and 2e-2 for
fp16/bf16 groups (the oracle is fp64 and unrounded)."""
import sys

import numpy as np
import pytest
import torch

from oracle import interp
from paper_1911_11576_amd import FsError, Plan
from paper_1911_11576_amd import binding
from workloads import BY_NAME, CONFIGS, TOLERANCE, graphs, inputs

from gpu_util import (alloc_outputs, assert_close, check_against_oracle, run_gpu,
                      to_device)

pytestmark = pytest.mark.gpu


def announce(msg):
    # names the case on the real stderr before any GPU work, so that it survives a dead box
    sys.__stderr__.write(f"[gpu-case] {msg}\n")
    sys.__stderr__.flush()


@pytest.fixture(autouse=True)
def _need_gpu(device):
    yield


# ---------------------------------------------------------------- the five configs, small

@pytest.mark.parametrize("cfg", CONFIGS, ids=lambda c: c.name)
def test_config_small_stitched(cfg):
    announce(f"small stitched {cfg.name}")
    ops, ins = cfg.build("small")
    check_against_oracle(ops, ins, "stitched", what=cfg.name)


@pytest.mark.parametrize("cfg", CONFIGS, ids=lambda c: c.name)
def test_config_small_per_op_baseline(cfg):
    """The unfused baseline rounds every intermediate to its declared dtype, as the oracle's
    storage-rounding mode does; it is held to the group tolerance except for the fp32
    column sums over many rows, whose per-op rounding alone exceeds 1e-5 absolute."""
    announce(f"small per_op {cfg.name}")
    ops, ins = cfg.build("small")
    want = interp.run(ops, ins)
    got = run_gpu(ops, ins, "per_op")
    tol = TOLERANCE[cfg.dtype]
    for i, (a, b) in enumerate(zip(got, want)):
        t = 1e-3 if (cfg.name == "layernorm_bwd" and b.ndim == 1) else tol
        assert_close(a, b, t, f"{cfg.name} per_op output {i}")


@pytest.mark.parametrize("cfg", CONFIGS, ids=lambda c: c.name)
def test_stitched_equals_per_op_on_gpu(cfg):
    announce(f"stitched vs per_op {cfg.name}")
    ops, ins = cfg.build("small")
    a = run_gpu(ops, ins, "stitched")
    b = run_gpu(ops, ins, "per_op")
    tol = TOLERANCE[cfg.dtype]
    for i, (x, y) in enumerate(zip(a, b)):
        t = 1e-3 if (cfg.name == "layernorm_bwd" and x.ndim == 1) else 2 * tol
        assert_close(x, y, t, f"{cfg.name} stitched vs per_op output {i}")


# ---------------------------------------------------------------- row schedule: shapes

@pytest.mark.parametrize("rows,cols", [(1, 4), (3, 8), (5, 24), (37, 100), (9, 256), (64, 768), (37, 1000),
                                       (11, 1536), (6, 2048), (130, 32)])
def test_layernorm_shapes_f32(rows, cols):
    announce(f"layernorm f32 {rows}x{cols}")
    check_against_oracle(graphs.layernorm_fwd(rows, cols), inputs.layernorm_fwd(rows, cols), what=f"ln {rows}x{cols}")


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("rows,cols", [(1, 8), (7, 40), (33, 512), (19, 1024), (5, 2048)])
def test_layernorm_shapes_16bit(rows, cols, dtype):
    announce(f"layernorm {dtype} {rows}x{cols}")
    check_against_oracle(graphs.layernorm_fwd(rows, cols, dtype), inputs.layernorm_fwd(rows, cols, dtype),
                         what=f"ln {dtype} {rows}x{cols}")


# The group with the GELU prologue has two stitched forms: the default is the generated kernel
# (mode "stitched"), the hand-written kernels serve mode "prebuilt"
GELU_LN_MODES = ["stitched", "prebuilt"]


@pytest.mark.parametrize("mode", GELU_LN_MODES)
@pytest.mark.parametrize("dtype,rows,cols", [("bf16", 203, 1024), ("f16", 33, 768), ("f32", 65, 1024),
                                             ("bf16", 4, 2048), ("f32", 3, 8)])
def test_bias_gelu_residual_layernorm_shapes(dtype, rows, cols, mode):
    announce(f"bias+gelu+res+ln {dtype} {rows}x{cols} {mode}")
    check_against_oracle(graphs.bias_gelu_residual_layernorm(rows, cols, dtype),
                         inputs.bias_gelu_residual_layernorm(rows, cols, dtype), mode, what=f"cfg4 {dtype} {rows}x{cols}")


@pytest.mark.parametrize("shape", [(1, 4), (3, 12), (1030, 128), (77, 64), (5, 1000), (9, 2048), (130, 32), (33, 16)])
@pytest.mark.parametrize("mask", ["full", "none"])
def test_softmax_shapes_f32(shape, mask):
    announce(f"softmax f32 {shape} mask={mask}")
    check_against_oracle(graphs.scaled_masked_softmax(shape, 0.125, mask),
                         inputs.scaled_masked_softmax(shape, mask), what=f"softmax {shape} {mask}")


@pytest.mark.parametrize("shape", [(3, 4, 16, 16), (2, 3, 5, 128), (4, 2, 7, 64)])
def test_softmax_key_padding_mask(shape):
    announce(f"softmax key_padding {shape}")
    check_against_oracle(graphs.scaled_masked_softmax(shape, 0.125, "key_padding"),
                         inputs.scaled_masked_softmax(shape, "key_padding"), what=f"softmax kp {shape}")


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_softmax_16bit(dtype):
    announce(f"softmax {dtype}")
    shape = (67, 128)
    # a mask of -1e4 is not representable in f16/bf16 exactly; the generator rounds it
    check_against_oracle(graphs.scaled_masked_softmax(shape, 0.125, "full", dtype),
                         inputs.scaled_masked_softmax(shape, "full", dtype), what=f"softmax {dtype}")


def test_softmax_fully_masked_rows_and_large_values():
    announce("softmax degenerate rows")
    shape = (8, 128)
    ops = graphs.scaled_masked_softmax(shape, 0.125, "full")
    s, m = inputs.scaled_masked_softmax(shape, "full")
    m[0, :] = -1e4          # fully padded row: still a softmax of the shifted row
    s[1, :] = 3.0           # constant row
    s[2, :] = 600.0         # exp would overflow without the max subtraction
    s[3, 5] = -700.0
    check_against_oracle(ops, [s, m], what="softmax degenerate")


# ---------------------------------------------------------------- row schedule, block-composed form

@pytest.mark.parametrize("rows,cols", [(3, 770), (5, 4096), (2, 3001), (7, 10007), (2, 16384), (1, 40000), (9, 1), (4, 3)])
def test_layernorm_long_or_unaligned_rows_f32(rows, cols):
    announce(f"layernorm block form f32 {rows}x{cols}")
    check_against_oracle(graphs.layernorm_fwd(rows, cols), inputs.layernorm_fwd(rows, cols), what=f"ln block {rows}x{cols}")


@pytest.mark.parametrize("mode", GELU_LN_MODES)
@pytest.mark.parametrize("dtype,rows,cols", [("bf16", 5, 4096), ("f16", 3, 3001), ("bf16", 2, 12), ("f16", 6, 8200)])
def test_gelu_layernorm_long_or_unaligned_rows_16bit(dtype, rows, cols, mode):
    announce(f"bias+gelu+res+ln block form {dtype} {rows}x{cols} {mode}")
    check_against_oracle(graphs.bias_gelu_residual_layernorm(rows, cols, dtype),
                         inputs.bias_gelu_residual_layernorm(rows, cols, dtype), mode, what=f"cfg4 block {dtype} {rows}x{cols}")


@pytest.mark.parametrize("shape,mask", [((5, 94), "full"), ((3, 4100), "full"), ((6, 2049), "none"), ((2, 3, 94, 94), "key_padding"),
                                        ((2, 2, 5, 4096), "key_padding"), ((4, 1), "full")])
def test_softmax_long_or_unaligned_rows(shape, mask):
    announce(f"softmax block form {shape} {mask}")
    check_against_oracle(graphs.scaled_masked_softmax(shape, 0.125, mask),
                         inputs.scaled_masked_softmax(shape, mask), what=f"softmax block {shape} {mask}")


@pytest.mark.parametrize("rows,cols", [(3, 2052), (5, 5000), (4, 8192), (2, 32768), (3, 20480)])
def test_layernorm_team_form_f32(rows, cols):
    announce(f"layernorm team form f32 {rows}x{cols}")
    check_against_oracle(graphs.layernorm_fwd(rows, cols), inputs.layernorm_fwd(rows, cols), what=f"ln team {rows}x{cols}")


@pytest.mark.parametrize("mode", GELU_LN_MODES)
@pytest.mark.parametrize("dtype,rows,cols", [("bf16", 3, 2056), ("f16", 5, 4096), ("bf16", 2, 32768), ("f16", 3, 12288)])
def test_gelu_layernorm_team_form_16bit(dtype, rows, cols, mode):
    announce(f"bias+gelu+res+ln team form {dtype} {rows}x{cols} {mode}")
    check_against_oracle(graphs.bias_gelu_residual_layernorm(rows, cols, dtype),
                         inputs.bias_gelu_residual_layernorm(rows, cols, dtype), mode, what=f"cfg4 team {dtype} {rows}x{cols}")


@pytest.mark.parametrize("shape,mask", [((5, 4096), "full"), ((2, 2, 3, 8192), "key_padding"), ((3, 16000), "none")])
def test_softmax_team_form(shape, mask):
    announce(f"softmax team form {shape} {mask}")
    check_against_oracle(graphs.scaled_masked_softmax(shape, 0.125, mask),
                         inputs.scaled_masked_softmax(shape, mask), what=f"softmax team {shape} {mask}")


def test_team_form_launch_options():
    announce("row team form options")
    ops, ins = graphs.layernorm_fwd(77, 8192), inputs.layernorm_fwd(77, 8192)
    ref = run_gpu(ops, ins)
    for opts in (dict(wg_size=256), dict(wg_size=1024), dict(grid=5), dict(wg_size=512, grid=3)):
        got = run_gpu(ops, ins, **opts)
        assert_close(got[0], ref[0], 1e-6, f"team form {opts}")


def test_block_form_launch_options():
    announce("row block form options")
    ops, ins = graphs.layernorm_fwd(300, 4096), inputs.layernorm_fwd(300, 4096)
    ref = run_gpu(ops, ins)
    for opts in (dict(wg_size=64), dict(wg_size=1024), dict(grid=7)):
        got = run_gpu(ops, ins, **opts)
        assert_close(got[0], ref[0], 1e-6, f"block form {opts}")


# ---------------------------------------------------------------- launch parameters

@pytest.mark.parametrize("opts", [dict(wg_size=64), dict(wg_size=512), dict(rows_per_wave=1), dict(rows_per_wave=2),
                                  dict(grid=7), dict(wg_size=128, rows_per_wave=4, grid=3)])
def test_row_schedule_launch_options_do_not_change_results(opts):
    announce(f"row options {opts}")
    shape = (1030, 128)
    ops, ins = graphs.scaled_masked_softmax(shape, 0.125, "full"), inputs.scaled_masked_softmax(shape, "full")
    ref = run_gpu(ops, ins)
    got = run_gpu(ops, ins, **opts)
    assert np.array_equal(ref[0], got[0])
    ops, ins = graphs.layernorm_fwd(517, 768), inputs.layernorm_fwd(517, 768)
    ref = run_gpu(ops, ins)
    got = run_gpu(ops, ins, **opts)
    assert np.array_equal(ref[0], got[0])


# ---------------------------------------------------------------- LayerNorm backward

# both forms of the group: the hand-written row kernel + combine kernel (default) and the generated
# row kernel + combine kernel (mode "generated")
LNBWD_MODES = ["stitched", "generated"]


@pytest.mark.parametrize("mode", LNBWD_MODES)
@pytest.mark.parametrize("rows,cols", [(1, 4), (5, 64), (517, 1024), (4099, 1000), (33, 768), (700, 256)])
def test_layernorm_bwd_shapes(rows, cols, mode):
    announce(f"layernorm_bwd {rows}x{cols} {mode}")
    check_against_oracle(graphs.layernorm_bwd(rows, cols), inputs.layernorm_bwd(rows, cols), mode, what=f"lnbwd {rows}x{cols}")


@pytest.mark.parametrize("mode", LNBWD_MODES)
@pytest.mark.parametrize("opts", [dict(grid=1), dict(grid=3, wg_size=64), dict(grid=100, wg_size=256), dict(grid=1024)])
def test_layernorm_bwd_launch_options(opts, mode):
    announce(f"layernorm_bwd options {opts} {mode}")
    rows, cols = 2100, 1024
    check_against_oracle(graphs.layernorm_bwd(rows, cols), inputs.layernorm_bwd(rows, cols), mode, what=f"lnbwd {opts}", **opts)


@pytest.mark.parametrize("mode", LNBWD_MODES)
def test_layernorm_bwd_is_bit_reproducible_and_reusable(mode):
    announce(f"layernorm_bwd determinism {mode}")
    rows, cols = 3000, 1024
    ops, ins = graphs.layernorm_bwd(rows, cols), inputs.layernorm_bwd(rows, cols)
    dev_in = to_device(ops, ins)
    runs = []
    with Plan(ops, mode) as plan:
        for _ in range(5):
            out = alloc_outputs(ops)
            plan.launch(dev_in, out)
            torch.cuda.synchronize()
            runs.append([t.cpu().numpy() for t in out])
    for r in runs[1:]:
        for a, b in zip(runs[0], r):
            assert np.array_equal(a, b)


@pytest.mark.parametrize("mode", LNBWD_MODES)
def test_layernorm_bwd_output_subsets(mode):
    announce(f"layernorm_bwd subsets {mode}")
    rows, cols = 300, 512
    full = graphs.layernorm_bwd(rows, cols)
    ins = inputs.layernorm_bwd(rows, cols)
    outs = [i for i, op in enumerate(full) if op.kind == "output"]
    for keep in ([0], [1, 2], [2], [0, 2]):
        ops = [op for i, op in enumerate(full) if op.kind != "output" or outs.index(i) in keep]
        check_against_oracle(ops, ins, mode, what=f"lnbwd outputs {keep}")


# ---------------------------------------------------------------- attention

@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("seq,dim", [(64, 64), (1, 32), (7, 64), (16, 32), (33, 64), (94, 64), (128, 32), (48, 128), (128, 64), (128, 128), (100, 128), (17, 32)])
def test_attention_shapes(seq, dim, dtype):
    announce(f"attention {dtype} seq={seq} dim={dim}")
    B = 5
    check_against_oracle(graphs.causal_attention(B, seq, dim, dtype), inputs.causal_attention(B, seq, dim, dtype),
                         what=f"attn {dtype} {seq}x{dim}")


def _attention_variant(B, S, d, causal, fill, dtype="f16"):
    g = graphs.Graph()
    q = g.parameter("q", dtype, (B, S, d))
    k = g.parameter("k", dtype, (B, S, d))
    v = g.parameter("v", dtype, (B, S, d))
    z = g.multiply(g.dot(q, k, transpose_b=True), g.constant(d ** -0.5))
    if causal:
        z = g.causal_mask(z, fill)
    zmax = g.reduce_max(z, -1)
    e = g.exp(g.subtract(z, g.row_broadcast(zmax, z)))
    p = g.divide(e, g.row_broadcast(g.reduce_sum(e, -1), e))
    o = g.dot(g.convert(p, dtype), v)
    g.output(g.convert(o, dtype))
    return g.ops


@pytest.mark.parametrize("causal,fill", [(False, 0.0), (True, -1e4), (True, -3.0)])
def test_attention_mask_variants(causal, fill):
    announce(f"attention causal={causal} fill={fill}")
    B, S, d = 3, 40, 64
    ops = _attention_variant(B, S, d, causal, fill)
    check_against_oracle(ops, inputs.causal_attention(B, S, d), what=f"attn causal={causal} fill={fill}")


# ---- schedule 3 with the elementwise ops around the two dots (Section 3.1's pattern shape): additive
# masks, an epilogue on O, a second output, unequal query and key lengths

ATTN_BLOCK_CASES = [
    # (batch, sq, sk, dim, dtype, kwargs)
    (3, 40, 72, 64, "f16", dict()),                                            # more keys than queries
    (2, 100, 24, 32, "bf16", dict()),                                          # more queries than keys
    (2, 16, 128, 128, "f16", dict(causal=True)),                               # one query tile, eight key tiles
    (3, 64, 64, 64, "f16", dict(mask="key")),                                  # key padding, vector mask loads
    (3, 50, 37, 64, "bf16", dict(mask="key")),                                 # ... ragged: scalar mask loads
    (2, 48, 64, 32, "f16", dict(mask="full")),
    (2, 33, 45, 64, "f16", dict(mask="full", causal=True)),
    (4, 64, 64, 64, "bf16", dict(mask="shared")),                              # one bias for the whole batch
    (2, 40, 40, 64, "f16", dict(mask="key", causal=True, mask_outside_causal=True)),
    (3, 64, 64, 64, "f16", dict(gate=True)),
    (3, 40, 72, 64, "bf16", dict(residual=True)),
    (2, 70, 50, 128, "f16", dict(gate=True, residual=True)),
    (3, 64, 64, 64, "f16", dict(lse=True, causal=True)),
    (2, 35, 90, 32, "bf16", dict(lse=True, mask="key")),
    (5, 64, 64, 64, "f16", dict(causal=True, mask="key", gate=True, residual=True, lse=True)),   # everything at once
    (2, 128, 128, 128, "bf16", dict(causal=True, mask="full", gate=True, residual=True, lse=True)),   # maximum sizes
    (1, 1, 1, 32, "f16", dict(lse=True, gate=True)),                           # a single score
]


@pytest.mark.parametrize("case", ATTN_BLOCK_CASES, ids=lambda c: f"{c[0]}x{c[1]}x{c[2]}x{c[3]}-{c[4]}-" + "+".join(sorted(c[5])))
def test_attention_with_prologue_and_epilogue(case):
    B, sq, sk, d, dtype, kw = case
    announce(f"attention block {case}")
    ops = graphs.attention_block(B, sq, sk, d, dtype, **kw)
    ins = inputs.attention_block(B, sq, sk, d, dtype, **kw)
    with Plan(ops) as plan:
        assert plan.info()["schedule"] == "bdot_softmax" and plan.info()["n_kernels"] == 1
    got, want = check_against_oracle(ops, ins, what=f"attention block {case}")
    if kw.get("lse"):
        assert got[1].shape == (B, sq)


# ---------------------------------------------------------------- full-size configs, bench launch shape

def test_full_size_layernorm_fwd():
    announce("full cfg1")
    ops, ins = BY_NAME["layernorm_fwd"].build("full")
    check_against_oracle(ops, ins, what="cfg1 full")


def test_full_size_softmax_whole_tensor():
    announce("full cfg2")
    cfg = BY_NAME["scaled_masked_softmax"]
    ops, ins = cfg.build("full")
    (got,) = run_gpu(ops, ins)
    (want,) = interp.run(ops, ins)
    assert_close(got, want, 1e-5, "cfg2 full, every element")
    # properties that hold for every row
    assert np.abs(got.sum(axis=1) - 1).max() < 1e-5
    assert got.min() >= 0 and not np.isnan(got).any()


def test_full_size_attention_whole_tensor():
    announce("full cfg3")
    cfg = BY_NAME["causal_attention"]
    ops, ins = cfg.build("full")
    (got,) = run_gpu(ops, ins)
    (want,) = interp.run(ops, ins)
    assert_close(got, want, 2e-2, "cfg3 full, every element")
    assert np.allclose(got[:, 0, :], ins[2][:, 0, :], atol=1e-3)   # first query row sees only V[0]
    assert not np.isnan(got).any()


@pytest.mark.parametrize("mode", GELU_LN_MODES)
def test_full_size_bias_gelu_ln_whole_tensor(mode):
    announce(f"full cfg4 {mode}")
    cfg = BY_NAME["bias_gelu_residual_layernorm"]
    ops, ins = cfg.build("full")
    (got,) = run_gpu(ops, ins, mode)
    (want,) = interp.run(ops, ins)
    assert_close(got, want, 2e-2, "cfg4 full, every element")
    assert not np.isnan(got).any()


@pytest.mark.parametrize("mode", LNBWD_MODES)
def test_full_size_layernorm_bwd(mode):
    announce(f"full cfg5 {mode}")
    cfg = BY_NAME["layernorm_bwd"]
    ops, ins = cfg.build("full")
    dx, dgamma, dbeta = run_gpu(ops, ins, mode)
    want_dx, want_dgamma, want_dbeta = interp.run(ops, ins)
    assert_close(dgamma, want_dgamma, 1e-5, "cfg5 full dgamma")
    assert_close(dbeta, want_dbeta, 1e-5, "cfg5 full dbeta")
    assert_close(dx, want_dx, 1e-5, "cfg5 full dx")


# ---------------------------------------------------------------- tuning (Algorithm 3's outer loop)

@pytest.mark.parametrize("cfg", CONFIGS, ids=lambda c: c.name)
def test_plan_tune_returns_a_correct_plan(cfg):
    announce(f"tune {cfg.name}")
    ops, ins = cfg.build("small")
    dev_in, dev_out = to_device(ops, ins), alloc_outputs(ops)
    plan = Plan.tune(ops, dev_in, dev_out, trials=3)
    try:
        assert plan.tuned["us"] > 0
        want = interp.run(ops, ins)
        tol = TOLERANCE[cfg.dtype]
        # the outputs already hold the winner's result
        torch.cuda.synchronize()
        for got, ref in zip(dev_out, want):
            assert_close(got.double().cpu().numpy(), ref, tol, f"tuned {cfg.name}")
        # and the returned plan is an ordinary plan
        fresh = alloc_outputs(ops)
        plan.launch(dev_in, fresh)
        torch.cuda.synchronize()
        for got, ref in zip(fresh, want):
            assert_close(got.double().cpu().numpy(), ref, tol, f"tuned relaunch {cfg.name}")
        # one stitched kernel; the generated form of a group with column reductions adds its combine kernel
        assert plan.info()["n_kernels"] <= (2 if plan.info()["schedule"] == "row_col" else 1)
    finally:
        plan.close()


def test_tuned_options_are_reused_by_later_plans(tmp_path):
    """'Optimize once, reuse': the winner of fs_plan_tune is what fs_plan_create builds for the same
    group from then on (launch parameters left open), also after a trip through the cache file."""
    from paper_1911_11576_amd import fs_tune_cache_clear, fs_tune_cache_load, fs_tune_cache_save, fs_tune_cache_size
    announce("tuning cache")
    ops, ins = graphs.rmsnorm((2048, 1024), "bf16"), inputs.normal_tensors([(2048, 1024), (1024,)], "bf16")
    dev_in, dev_out = to_device(ops, ins), alloc_outputs(ops)
    assert fs_tune_cache_size() == 0
    with Plan(graphs.rmsnorm((2047, 1024), "bf16")) as p:
        other_shape = p.describe()
    with Plan.tune(ops, dev_in, dev_out, trials=5) as tuned:
        winner = tuned.describe()
    assert fs_tune_cache_size() == 1
    with Plan(ops) as p:
        assert p.describe() == winner
    check_against_oracle(ops, ins, what="plan from the tuning cache")
    fs_tune_cache_save(tmp_path / "t.txt")
    fs_tune_cache_clear()
    fs_tune_cache_load(tmp_path / "t.txt")
    with Plan(ops) as p:
        assert p.describe() == winner
    # another shape of the same group is another entry
    with Plan(graphs.rmsnorm((2047, 1024), "bf16")) as p:
        assert p.describe() == other_shape


def test_plan_tune_rejects_unsupported_groups_and_bad_arguments():
    announce("tune errors")
    g = graphs.Graph()
    x = g.parameter("x", "f32", (4, 8, 6, 64))
    g.output(g.reduce_sum(g.exp(x), 1))       # a reduction over an outer dim that keeps the dims between: no stitched schedule
    t = torch.zeros(4, 8, 6, 64, device="cuda:0")
    with pytest.raises(FsError) as e:
        Plan.tune(g.ops, [t], [torch.empty(4, 6, 64, device="cuda:0")])
    assert e.value.status == binding.FS_ERR_UNSUPPORTED
    ops, ins = graphs.layernorm_fwd(4, 768), inputs.layernorm_fwd(4, 768)
    dev_in, dev_out = to_device(ops, ins), alloc_outputs(ops)
    with pytest.raises(FsError) as e:
        Plan.tune(ops, dev_in[:2], dev_out)
    assert e.value.status == binding.FS_ERR_INVALID
    with pytest.raises(FsError) as e:
        Plan.tune(ops, dev_in, dev_out, trials=0)
    assert e.value.status == binding.FS_ERR_INVALID


# ---------------------------------------------------------------- edge cases and error paths

def test_empty_inputs_launch_nothing_and_succeed():
    announce("empty inputs")
    for ops, ins in [(graphs.layernorm_fwd(0, 768), inputs.layernorm_fwd(0, 768)),
                     (graphs.causal_attention(0, 64, 64), inputs.causal_attention(0, 64, 64))]:
        for mode in ("stitched", "per_op"):
            out = run_gpu(ops, ins, mode)
            assert out[0].size == 0


def test_launch_rejects_bad_pointers_and_counts():
    announce("launch argument errors")
    ops, ins = graphs.layernorm_fwd(4, 768), inputs.layernorm_fwd(4, 768)
    dev_in, dev_out = to_device(ops, ins), alloc_outputs(ops)
    with Plan(ops) as plan:
        with pytest.raises(FsError) as e:
            plan.launch(dev_in[:2], dev_out)
        assert e.value.status == binding.FS_ERR_INVALID
        with pytest.raises(FsError) as e:
            plan.launch([dev_in[0].data_ptr() + 4, dev_in[1], dev_in[2]], dev_out)
        assert e.value.status == binding.FS_ERR_INVALID
        with pytest.raises(FsError) as e:
            plan.launch([0, dev_in[1], dev_in[2]], dev_out)
        assert e.value.status == binding.FS_ERR_INVALID
        plan.launch(dev_in, dev_out)      # the plan still works afterwards
        torch.cuda.synchronize()
    (want,) = interp.run(ops, ins)
    assert_close(dev_out[0].double().cpu().numpy(), want, 1e-5, "after errors")


def test_stream_copy_matches_source():
    announce("stream copy")
    src = torch.randint(0, 255, (3 * 1024 * 1024 + 16,), dtype=torch.uint8, device="cuda:0")
    dst = torch.zeros_like(src)
    binding.fs_stream_copy(dst, src, src.numel())
    torch.cuda.synchronize()
    assert torch.equal(src, dst)


def test_launch_on_a_side_stream():
    announce("side stream")
    ops, ins = graphs.layernorm_fwd(64, 768), inputs.layernorm_fwd(64, 768)
    dev_in, dev_out = to_device(ops, ins), alloc_outputs(ops)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    with Plan(ops) as plan:
        plan.launch(dev_in, dev_out, stream=s.cuda_stream)
        s.synchronize()
    (want,) = interp.run(ops, ins)
    assert_close(dev_out[0].double().cpu().numpy(), want, 1e-5, "side stream")


# ---------------------------------------------------------------- launches recorded into a HIP graph

@pytest.mark.parametrize("name", ["scaled_masked_softmax", "layernorm_bwd", "causal_attention", "multi_tensor_momentum"])
def test_launches_replay_from_a_captured_graph(name):
    """After one ordinary launch (which loads the kernels and allocates the plan's workspace) a launch is
    nothing but kernel launches on the caller's stream, so it can be recorded into a HIP graph.
    The graph is replayed three times, with eager work and new input values between the replays,
    and every replay is compared with the oracle."""
    announce(f"graph capture {name}")
    cfg = BY_NAME[name]
    ops, ins = cfg.build("small")
    tol = TOLERANCE[cfg.dtype]
    dev_in, dev_out = to_device(ops, ins), alloc_outputs(ops)
    with Plan(ops) as plan:
        plan.launch(dev_in, dev_out)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        with torch.cuda.graph(graph, stream=side):
            plan.launch(dev_in, dev_out)                      # torch's current stream is the capturing one here
        for rep in range(3):
            # new values in the same buffers: the first tensor is scaled, eagerly, between replays
            scale = [1.0, 0.5, -1.5][rep]
            cur = [a * scale if k == 0 else a for k, a in enumerate(ins)]
            cur[0] = inputs.round_to(cur[0], ops[0].dtype)
            dev_in[0].copy_(to_device(ops, cur)[0])
            for t in dev_out:
                t.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            want = interp.run(ops, cur)
            for got, ref in zip(dev_out, want):
                assert_close(got.double().cpu().numpy(), ref, tol, f"graph replay {rep} of {name}")
