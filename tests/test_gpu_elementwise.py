"""GPU parity of the generic elementwise schedule (thread composition + kernel packing)
against the CPU oracle, in both of its forms: the kernel generated for the group
(mode "stitched") and the register-program interpreter (mode "prebuilt")."""
import sys

import numpy as np
import pytest
import torch

from oracle import interp
from paper_1911_11576_amd import Plan
from workloads import graphs, inputs

from gpu_util import check_against_oracle, run_gpu, assert_close

pytestmark = pytest.mark.gpu


def announce(msg):
    sys.__stderr__.write(f"[gpu-case] {msg}\n")
    sys.__stderr__.flush()


@pytest.fixture(autouse=True)
def _need_gpu(device):
    yield


MODES = ["stitched", "prebuilt"]


def _rand(shape, seed, lo=-2.0, hi=2.0):
    return inputs.round_to(np.random.default_rng(seed).uniform(lo, hi, shape), "f32")


@pytest.mark.parametrize("mode", MODES)
def test_unary_chain_and_schedule_name(mode):
    announce(f"elementwise unary chain {mode}")
    g = graphs.Graph()
    x = g.parameter("x", "f32", (37, 64))
    g.output(g.exp(g.tanh(x)))
    with Plan(g.ops, mode) as p:
        info = p.info()
        assert info["schedule"] == "elementwise" and info["n_kernels"] == 1
        # interpreted, a pure chain lives in the accumulator: only the program is in LDS
        assert info["lds_bytes"] == (0 if mode == "stitched" else 2048)
    check_against_oracle(g.ops, [_rand((37, 64), 1)], mode, what="exp(tanh(x))")


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("dtype,rows,cols", [("bf16", 203, 1024), ("f16", 33, 768), ("f32", 65, 1000), ("bf16", 7, 30), ("f32", 5, 3),
                                             ("bf16", 19, 1028), ("f16", 3, 8)])
def test_bias_gelu_residual(dtype, rows, cols, mode):
    announce(f"elementwise bias+gelu+residual {dtype} {rows}x{cols} {mode}")
    check_against_oracle(graphs.bias_gelu_residual(rows, cols, dtype), inputs.bias_gelu_residual(rows, cols, dtype), mode,
                         what=f"bias_gelu_residual {dtype} {rows}x{cols}")


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("shape", [(1000,), (64, 1024), (3, 5, 7), (2, 3, 4, 8), (4099,), (300, 1024)])
def test_adam_update_three_packed_outputs(shape, mode):
    announce(f"elementwise adam {shape} {mode}")
    ops, ins = graphs.adam_update(shape), inputs.adam_update(shape)
    with Plan(ops, mode) as p:
        assert p.info()["schedule"] == "elementwise"
    check_against_oracle(ops, ins, mode, what=f"adam {shape}")


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("dtype,shape", [("f32", (33, 128)), ("f32", (4, 6, 100)), ("bf16", (17, 256)), ("f32", (9, 7)), ("f16", (2, 3, 5, 64)),
                                         ("bf16", (5, 12)), ("f32", (700, 1024))])
def test_row_and_column_broadcast_operands(dtype, shape, mode):
    announce(f"elementwise row/col broadcast {dtype} {shape} {mode}")
    check_against_oracle(graphs.scale_shift_rows_cols(shape, dtype), inputs.scale_shift_rows_cols(shape, dtype), mode,
                         what=f"rows_cols {dtype} {shape}")


@pytest.mark.parametrize("mode", MODES)
def test_diamond_reuse_many_live_values_and_constant_first_operand(mode):
    announce(f"elementwise diamond {mode}")
    g = graphs.Graph()
    a = g.parameter("a", "f32", (40, 96))
    b = g.parameter("b", "f32", (40, 96))
    s = g.add(a, b)                     # used three times
    d = g.subtract(a, b)                # used twice
    p = g.multiply(s, d)
    q = g.multiply(s, s)                # same value twice
    r = g.divide(g.constant(2.0), g.add(q, g.constant(1.0)))   # constant as first operand
    t = g.maximum(g.subtract(p, r), g.negate(d))
    u = g.add(g.add(t, s), g.multiply(a, a))                   # the same parameter twice
    g.output(u)
    g.output(r)
    ops = g.ops
    with Plan(ops, "prebuilt") as plan:
        assert plan.info()["lds_bytes"] > 2048
    check_against_oracle(ops, [_rand((40, 96), 2), _rand((40, 96), 3)], mode, what="diamond")


@pytest.mark.parametrize("mode", MODES)
def test_mid_graph_rounding_is_applied(mode):
    announce(f"elementwise mid-graph convert {mode}")
    g = graphs.Graph()
    x = g.parameter("x", "f32", (16, 64))
    y = g.convert(g.multiply(x, g.constant(1.0009765625)), "bf16")     # rounds here
    z = g.multiply(g.convert(y, "f32"), g.constant(3.0))
    g.output(z)
    xs = _rand((16, 64), 4)
    (got,) = run_gpu(g.ops, [xs], mode)
    (want,) = interp.run(g.ops, [xs], storage_rounding=True)
    assert_close(got, want, 1e-6, "mid-graph bf16 rounding")


@pytest.mark.parametrize("mode", MODES)
def test_key_padding_style_broadcast_rank4(mode):
    announce(f"elementwise rank-4 broadcast {mode}")
    g = graphs.Graph()
    s = g.parameter("s", "f32", (2, 3, 5, 64))
    m = g.parameter("m", "f32", (2, 1, 1, 64))
    g.output(g.add(g.multiply(s, g.constant(0.125)), g.broadcast(m, (2, 3, 5, 64), 0)))
    check_against_oracle(g.ops, [_rand((2, 3, 5, 64), 5), _rand((2, 1, 1, 64), 6)], mode, what="rank-4 broadcast")


def test_elementwise_matches_per_op_and_options():
    announce("elementwise vs per_op")
    ops, ins = graphs.adam_update((129, 512)), inputs.adam_update((129, 512))
    b = run_gpu(ops, ins, "per_op")
    for mode in MODES:
        a = run_gpu(ops, ins, mode)
        for x, y in zip(a, b):
            assert_close(x, y, 1e-6, f"{mode} vs per_op")
        for opts in (dict(wg_size=64), dict(wg_size=128), dict(grid=3), dict(rows_per_wave=2), dict(rows_per_wave=4)):
            c = run_gpu(ops, ins, mode, **opts)
            for x, y in zip(a, c):
                assert np.array_equal(x, y)


def test_long_chain_only_the_generated_kernel_takes():
    announce("elementwise 100-op chain")
    g = graphs.Graph()
    x = g.parameter("x", "f32", (33, 64))
    y = x
    for i in range(100):
        y = g.add(g.multiply(y, g.constant(0.99)), g.constant(0.01)) if i % 2 else g.tanh(y)
    g.output(y)
    check_against_oracle(g.ops, [_rand((33, 64), 9)], what="100-op chain")


def test_tuner_picks_among_generated_and_interpreted_forms():
    announce("elementwise tune")
    from gpu_util import to_device, alloc_outputs
    ops, ins = graphs.adam_update((256, 1024)), inputs.adam_update((256, 1024))
    dev_in, dev_out = to_device(ops, ins), alloc_outputs(ops)
    with Plan.tune(ops, dev_in, dev_out, trials=5) as plan:
        assert plan.info()["schedule"] == "elementwise" and plan.tuned["us"] > 0
    torch.cuda.synchronize()
    want = interp.run(ops, ins)
    for t, w in zip(dev_out, want):
        assert_close(t.to(torch.float64).cpu().numpy(), w, 1e-5, "tuned elementwise")


def test_empty_elementwise_group():
    announce("elementwise empty")
    ops = graphs.adam_update((0, 16))
    for mode in MODES:
        out = run_gpu(ops, inputs.adam_update((0, 16)), mode)
        assert all(o.size == 0 for o in out)


def _gelu_variants(shape, dtype, spelling, constants=(0.5, None, None)):
    """tanh-form GELU spelled with operands in different orders / associations, optionally with
    an interior value as a second output or with other constants than the usual ones."""
    from workloads.graphs import GELU_K0, GELU_K1, Graph
    half, k0, k1 = constants[0], constants[1] or GELU_K0, constants[2] or GELU_K1
    g = Graph()
    x = g.parameter("x", dtype, shape)
    h = x if dtype == "f32" else g.convert(x, "f32")
    if spelling == "usual":
        h3 = g.multiply(g.multiply(h, h), h)
        t = g.tanh(g.multiply(g.add(h, g.multiply(h3, g.constant(k1))), g.constant(k0)))
        y = g.multiply(g.multiply(h, g.constant(half)), g.add(t, g.constant(1.0)))
    elif spelling == "commuted":
        h3 = g.multiply(h, g.multiply(h, h))
        t = g.tanh(g.multiply(g.constant(k0), g.add(g.multiply(g.constant(k1), h3), h)))
        y = g.multiply(g.add(g.constant(1.0), t), g.multiply(g.constant(half), h))
    else:                                   # interior value is an output too: no idiom
        h3 = g.multiply(g.multiply(h, h), h)
        t = g.tanh(g.multiply(g.add(h, g.multiply(h3, g.constant(k1))), g.constant(k0)))
        y = g.multiply(g.multiply(h, g.constant(half)), g.add(t, g.constant(1.0)))
        g.output(t if dtype == "f32" else g.convert(t, dtype), "t")
    g.output(y if dtype == "f32" else g.convert(y, dtype), "y")
    return g.ops


@pytest.mark.parametrize("spelling", ["usual", "commuted", "interior_output"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_gelu_idiom_matches_the_spelled_out_ops(dtype, spelling):
    shape = (37, 260)
    ops = _gelu_variants(shape, dtype, spelling)
    x = np.random.default_rng(5).normal(0.0, 3.0, shape)
    x.flat[:8] = [0.0, -0.0, 40.0, -40.0, 1e4, -1e4, 1e-30, -3.0]      # saturated tanh on both sides, zero
    ins = [inputs.round_to(x, dtype)]
    announce(f"gelu idiom {dtype} {spelling}")
    got, want = check_against_oracle(ops, ins, what=f"gelu {spelling}")
    assert not np.isnan(np.asarray(got[-1], dtype=np.float64)).any()


def test_gelu_idiom_with_other_constants():
    shape = (5, 64)
    ops = _gelu_variants(shape, "f32", "usual", constants=(1.0, 0.5, 0.1))
    ins = [_rand(shape, 9, -3, 3)]
    announce("gelu idiom, other constants")
    check_against_oracle(ops, ins, what="gelu constants")


# ---------------------------------------------------------------- independent parts of different shapes, one kernel

@pytest.mark.parametrize("shapes,dtypes", [
    ([(1024, 1024), (1024,), (4096, 1024), (4096,), (3, 5, 7)], ["f32", "f32", "bf16", "f32", "f16"]),
    ([(7,), (300, 96)], None),
    ([(64, 64)] + [(k + 1,) for k in range(7)], None),                 # eight parts, 16 outputs
    ([(0,), (5, 8), (3, 0, 2)], None),                                 # empty tensors among them
])
def test_packed_parts_of_different_shapes(shapes, dtypes):
    ops = graphs.multi_tensor_momentum(shapes, dtypes=dtypes)
    ins = inputs.multi_tensor_momentum(shapes, dtypes)
    announce(f"packed elementwise parts {shapes}")
    with Plan(ops) as p:
        info = p.info()
        assert info["schedule"] == "elementwise" and info["n_kernels"] == 1
        assert f"packed in {len(shapes)} independent parts" in p.describe()
    check_against_oracle(ops, ins, what="packed parts")
    check_against_oracle(ops, ins, what="packed parts wg 64", wg_size=64)
    # the unfused baseline runs them as separate kernels
    with Plan(ops, "per_op") as p:
        assert p.info()["n_kernels"] >= 2 * len([s for s in shapes])


def test_packed_parts_share_an_input_and_mix_ops():
    """Two parts may read the same parameter (no computed value is shared), and need not apply the same ops."""
    g = graphs.Graph()
    x = g.parameter("x", "f32", (33, 100))
    s = g.parameter("s", "f32", (100,))
    t = g.parameter("t", "f32", (5, 100))
    g.output(g.multiply(g.tanh(x), g.col_broadcast(s, x)), "a")          # [33, 100]
    g.output(g.add(g.exp(g.negate(g.multiply(s, s))), g.constant(1.0)), "b")   # [100]
    g.output(g.maximum(t, g.col_broadcast(s, t)), "c")                   # [5, 100]
    ins = inputs.normal_tensors([(33, 100), (100,), (5, 100)])
    announce("packed parts sharing an input")
    with Plan(g.ops) as p:
        assert "packed in 3 independent parts" in p.describe()
    check_against_oracle(g.ops, ins, what="packed parts sharing an input")


# ---------------------------------------------------------------- updates in place

def test_update_in_place_where_the_kernel_reads_before_it_writes():
    """Optimizer-style updates: outputs given the very buffers of the parameters they replace."""
    from paper_1911_11576_amd import FsError, binding
    from gpu_util import to_device
    shapes = [(300, 96), (96,), (7, 5, 3)]
    ops, ins = graphs.multi_tensor_momentum(shapes), inputs.multi_tensor_momentum(shapes)
    want = interp.run(ops, ins)
    announce("in-place multi-tensor momentum")
    dev = to_device(ops, ins)                                   # p0 g0 m0 p1 g1 m1 ...
    outs = [dev[3 * (k // 2) + (0 if k % 2 == 0 else 2)] for k in range(2 * len(shapes))]      # p_k' -> p_k, m_k' -> m_k
    with Plan(ops) as p:
        p.launch(dev, outs)
        torch.cuda.synchronize()
    for got, ref in zip(outs, want):
        assert_close(got.double().cpu().numpy(), ref, 1e-5, "in-place momentum")
    # a generated row kernel: LayerNorm written over its input
    rows, cols = 203, 1024
    ops, ins = graphs.layernorm_fwd(rows, cols), inputs.layernorm_fwd(rows, cols)
    (want,) = interp.run(ops, ins)
    dev = to_device(ops, ins)
    with Plan(ops, "generated") as p:
        p.launch(dev, [dev[0]])
        torch.cuda.synchronize()
    assert_close(dev[0].double().cpu().numpy(), want, 1e-5, "in-place LayerNorm")
    # refused: the hand-written kernel, the per-op baseline, the streamed template, a parameter read through a broadcast
    dev = to_device(ops, ins)
    for kw in (dict(mode="prebuilt"), dict(mode="per_op"), dict(mode="generated", grid=3)):
        with Plan(ops, **kw) as p:
            with pytest.raises(FsError) as e:
                p.launch(dev, [dev[0]])
            assert e.value.status == binding.FS_ERR_INVALID and "in-place" in e.value.message
    g = graphs.Graph()
    x = g.parameter("x", "f32", (64, 64))
    v = g.parameter("v", "f32", (64,))
    g.output(g.add(g.tanh(v), g.constant(1.0)), "v2")             # [64], would overwrite what the other part still reads
    g.output(g.multiply(x, g.col_broadcast(v, x)), "y")
    dev = to_device(g.ops, inputs.normal_tensors([(64, 64), (64,)]))
    with Plan(g.ops) as p:
        with pytest.raises(FsError):
            p.launch(dev, [dev[1], torch.empty_like(dev[0])])


def test_tanh_of_fp32_groups_is_accurate_relative_to_its_value():
    """The generated kernels' tanh for fp32 groups (a short series near zero, the exponential form
    elsewhere): scaled by 1e4 the comparison bar 1e-5 + 1e-5*|ref| asks for about 1e-5 relative accuracy of
    tanh itself, from 1e-7 to saturation, both signs."""
    x = np.concatenate([np.logspace(-7, 1.5, 4093), -np.logspace(-7, 1.5, 4093), [0.0, -0.0, 0.3, -0.3, 0.29999998, 88.0, -1e6, 1e30]])
    x = inputs.round_to(x, "f32").reshape(2, -1)
    for build in ("elementwise", "row"):
        g = graphs.Graph()
        p = g.parameter("x", "f32", x.shape)
        t = g.multiply(g.tanh(p), g.constant(1e4))
        g.output(t, "t")
        if build == "row":
            g.output(g.reduce_max(t, -1), "m")
        announce(f"tanh accuracy, {build} group")
        with Plan(g.ops) as plan:
            assert "generated kernel" in plan.describe()
        check_against_oracle(g.ops, [x], what=f"tanh accuracy ({build})")


# ---------------------------------------------------------------- erf and logistic

@pytest.mark.parametrize("mode", MODES + ["per_op"])
@pytest.mark.parametrize("dtype,shape", [("bf16", (203, 1024)), ("f32", (33, 100)), ("f16", (5, 7, 9))])
def test_swiglu(dtype, shape, mode):
    ops = graphs.swiglu(shape, dtype)
    ins = inputs.normal_tensors([shape, shape], dtype, scale=3.0, seed_offset=61)
    announce(f"swiglu {dtype} {shape} {mode}")
    check_against_oracle(ops, ins, mode, what=f"swiglu {dtype} {shape}")


@pytest.mark.parametrize("mode", MODES + ["per_op"])
def test_erf_and_logistic_over_their_whole_range(mode):
    x = np.concatenate([np.linspace(-6.0, 6.0, 2041), [-100.0, -20.0, 20.0, 100.0, 0.0, -0.0, 1e-8]]).reshape(1, -1)
    x = inputs.round_to(np.repeat(x, 2, axis=0), "f32")
    g = graphs.Graph()
    p = g.parameter("x", "f32", x.shape)
    g.output(g.erf(p), "erf")
    g.output(g.logistic(p), "logistic")
    g.output(g.multiply(g.multiply(p, g.constant(0.5)), g.add(g.erf(g.multiply(p, g.constant(0.7071067811865476))), g.constant(1.0))), "gelu")
    announce(f"erf and logistic {mode}")
    check_against_oracle(g.ops, [x], mode, what="erf / logistic / exact gelu")
