"""Host-side checks of the C ABI that need no GPU: the library loads and exports what
include/fs.h declares, plans are recognised and sized, and malformed or unsupported
groups come back as status codes (the paper's "negative score", Section 4.3)."""
import ctypes
import os
import re

import pytest

from paper_1911_11576_amd import FsError, Plan, binding
from workloads import BY_NAME, CONFIGS, algorithmic_bytes, graphs
from workloads.graphs import Graph, Op

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "fs.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(fs_[a-z_]+)\s*\(", header))
    assert {"fs_plan_create", "fs_launch", "fs_destroy", "fs_last_error", "fs_plan_info",
            "fs_plan_describe", "fs_stream_copy"} <= names
    lib = binding.lib()
    for n in names:
        assert hasattr(lib, n), n


def test_a_caller_written_in_c(tmp_path):
    """include/fs.h is plain C (c99, pedantic, no warnings) and the library is usable from it: tests/abi_from_c.c
    describes a softmax group, plans it, reads the plan back and checks an error path."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler here")
    libdir = os.path.dirname(binding.lib()._name)
    exe = str(tmp_path / "abi_from_c")
    build = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(ROOT, "include"), "-o", exe,
                            os.path.join(ROOT, "tests", "abi_from_c.c"), "-L", libdir, "-lfusionstitch", "-Wl,-rpath," + libdir],
                           capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    run = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "schedule=1 kernels=1" in run.stdout and "refused:" in run.stdout


def test_struct_layout_matches_the_header():
    # int32 x4, int64 x4, int32 x3, int32, double
    assert ctypes.sizeof(binding.fs_op_desc) == 16 + 32 + 12 + 4 + 8
    assert binding.fs_op_desc.shape.offset == 16
    assert binding.fs_op_desc.operand.offset == 48
    assert binding.fs_op_desc.attr.offset == 64
    assert ctypes.sizeof(binding.fs_plan_options) == 16


@pytest.mark.parametrize("cfg", CONFIGS, ids=lambda c: c.name)
def test_configs_are_recognised(cfg):
    want = {"layernorm_fwd": "row", "scaled_masked_softmax": "row", "causal_attention": "bdot_softmax",
            "bias_gelu_residual_layernorm": "row", "layernorm_bwd": "row_col"}[cfg.name]
    ops = cfg.graph_fn(**cfg.full)
    with Plan(ops) as p:
        info = p.info()
        assert info["schedule"] == want
        # one stitched kernel; config 5's plan is the row kernel plus its combine kernel
        assert info["n_kernels"] == (2 if cfg.name == "layernorm_bwd" else 1)
        assert "cta_num=" in p.describe() and "cta_size=" in p.describe()
    with Plan(ops, "prebuilt") as p:          # the hand-written kernels: one launch each, config 5's row kernel plus its combine kernel
        assert p.info()["schedule"] == want and p.info()["n_kernels"] == (2 if cfg.name == "layernorm_bwd" else 1)
        assert "generated" not in p.describe()
    with Plan(ops, "per_op") as p:
        info = p.info()
        assert info["schedule"] == "per_op" and info["n_kernels"] >= 7
        assert info["moved_bytes"] > 3 * info["algorithmic_bytes"]
        assert info["workspace_bytes"] > 0


def test_plan_info_sizes():
    with Plan(BY_NAME["layernorm_bwd"].graph_fn(**BY_NAME["layernorm_bwd"].full), "prebuilt") as p:
        info = p.info()
        assert info["algorithmic_bytes"] == 402_927_616
        # 4 wavefronts x (dgamma, dbeta) x 1024 fp64 slots; one partial row of 2048 doubles per workgroup
        assert info["lds_bytes"] == 4 * 2 * 1024 * 8
        assert info["workspace_bytes"] == 256 * 2 * 1024 * 8
        assert info["moved_bytes"] == info["algorithmic_bytes"] + 2 * info["workspace_bytes"]
    with Plan(BY_NAME["layernorm_bwd"].graph_fn(**BY_NAME["layernorm_bwd"].full), "generated") as p:
        info = p.info()
        # generated: (dgamma, dbeta) x 1024 fp64 sums in LDS, 256 partial rows of them in the workspace
        assert info["lds_bytes"] == 2 * 1024 * 8 and info["workspace_bytes"] == 256 * 2 * 1024 * 8
        assert info["moved_bytes"] == info["algorithmic_bytes"] + 2 * info["workspace_bytes"]
    with Plan(BY_NAME["causal_attention"].graph_fn(**BY_NAME["causal_attention"].full)) as p:
        assert 0 < p.info()["lds_bytes"] <= 64 * 1024


def test_commuted_and_reassociated_spellings_are_recognised():
    # LayerNorm with mean spelled as multiply by 1/N, operands swapped, beta added first
    g = Graph()
    x = g.parameter("x", "f32", (16, 256))
    gamma = g.parameter("gamma", "f32", (256,))
    beta = g.parameter("beta", "f32", (256,))
    mean = g.multiply(g.constant(1.0 / 256), g.reduce_sum(x, 1))
    c = g.subtract(x, g.row_broadcast(mean, x))
    var = g.multiply(g.reduce_sum(g.multiply(c, c), 1), g.constant(1.0 / 256))
    rstd = g.rsqrt(g.add(g.constant(1e-6), var))
    y = g.add(g.col_broadcast(beta, x), g.multiply(g.col_broadcast(gamma, x), g.multiply(g.row_broadcast(rstd, x), c)))
    g.output(y)
    with Plan(g.ops) as p:
        assert p.info()["schedule"] == "row"
    # softmax without scale or mask
    with Plan(graphs.scaled_masked_softmax((8, 64), 1.0, "none")) as p:
        assert p.info()["schedule"] == "row"


def _expect(status, ops, **kw):
    with pytest.raises(FsError) as e:
        Plan(ops, **kw)
    assert e.value.status == status, e.value
    assert e.value.message
    return e.value.message


def test_unsupported_groups_return_unsupported_not_crash():
    g = Graph()
    x = g.parameter("x", "f32", (8, 64))
    g.output(g.reduce_sum(g.exp(x), 0))            # a lone column reduction: generated, partial rows + combine
    with Plan(g.ops) as p:
        assert p.info()["schedule"] == "row_col" and p.info()["n_kernels"] == 2
    _expect(binding.FS_ERR_UNSUPPORTED, g.ops, mode="prebuilt")   # no hand-written kernel matches it
    with Plan(g.ops, "per_op") as p:               # the per-op plan always exists
        assert p.info()["n_kernels"] == 3
    g = Graph()
    x = g.parameter("x", "f32", (4, 8, 64))
    g.output(g.reduce_sum(g.exp(x), 1))            # a sum over the dim before the last: column sums per run of rows
    with Plan(g.ops) as p:
        assert p.info()["schedule"] == "row_col" and p.info()["n_kernels"] == 1 and "per run of 8 rows" in p.describe()
    g = Graph()
    x = g.parameter("x", "f32", (4, 8, 64))
    g.output(g.reduce_max(g.exp(x), 1))            # maxima too
    with Plan(g.ops) as p:
        assert p.info()["schedule"] == "row_col" and p.info()["n_kernels"] == 1
    g = Graph()
    x = g.parameter("x", "f32", (4, 8, 6, 64))
    g.output(g.reduce_sum(g.exp(x), 1))            # a sum over a dim further out, the dims between kept: no stitched schedule
    _expect(binding.FS_ERR_UNSUPPORTED, g.ops)
    g = Graph()
    x = g.parameter("x", "f32", (8, 64))
    g.output(g.exp(g.tanh(x)))                     # any all-elementwise group stitches
    with Plan(g.ops) as p:
        assert p.info()["schedule"] == "elementwise"
    # the hand-written LayerNorm backward takes at most 1024 columns; beyond that the generated kernel
    with Plan(graphs.layernorm_bwd(8, 2048)) as p:
        assert p.info()["schedule"] == "row_col" and "generated kernel" in p.describe()
    _expect(binding.FS_ERR_UNSUPPORTED, graphs.layernorm_bwd(8, 2048), mode="prebuilt")
    # rows beyond one wavefront's registers: a team of wavefronts per row, column sums still packed
    with Plan(graphs.layernorm_bwd(64, 8192)) as p:
        assert p.info()["schedule"] == "row_col" and "CTA-S" in p.describe() and "cta_size=1024" in p.describe()
        assert p.info()["workspace_bytes"] == 2 * 4 * 8192 * 8          # 16 rows per workgroup: 4 partial rows
    # beyond the register templates the streamed template keeps the column sums as running values per thread
    with Plan(graphs.layernorm_bwd(8, 16384)) as p:
        assert p.info()["schedule"] == "row_col" and "streamed" in p.describe() and "column reduce x2" in p.describe()
        assert p.info()["n_kernels"] == 2 and p.info()["workspace_bytes"] == 2 * 8 * 16384 * 8     # one partial row per workgroup (8 rows: 8 workgroups)
    msg = _expect(binding.FS_ERR_UNSUPPORTED, graphs.layernorm_bwd(8, 32768))
    assert "column reductions" in msg and "registers" in msg
    # a reduction over the leading dim that keeps the inner dims is a column reduction of the same memory read as a matrix
    g = Graph()
    x = g.parameter("x", "f32", (4, 8, 64))
    g.output(g.reduce_sum(g.exp(x), 0))
    with Plan(g.ops) as p:
        assert p.info()["schedule"] == "row_col" and p.info()["n_kernels"] == 2
    # fp32 attention has no MFMA path
    _expect(binding.FS_ERR_UNSUPPORTED, graphs.causal_attention(2, 64, 64, "f32"))
    _expect(binding.FS_ERR_UNSUPPORTED, graphs.causal_attention(2, 256, 64))


def test_lds_volume_constraint():
    # the largest attention group the schedule takes keeps K (128 rows of 136 halves) and V (128 rows of 144)
    # in LDS, inside the budget
    with Plan(graphs.causal_attention(2, 128, 128)) as p:
        assert p.info()["lds_bytes"] == 2 * (128 * 136 + 128 * 144)
    # a row longer than the LDS row cache of the block-composed row form: without kernel
    # generation that is the end, with it the streamed template takes over
    msg = _expect(binding.FS_ERR_LDS, graphs.layernorm_fwd(4, 50000), mode="prebuilt")
    assert "LDS" in msg
    with Plan(graphs.layernorm_fwd(4, 50000)) as p:
        assert "streamed in" in p.describe()


def test_long_and_unaligned_rows_take_the_block_composed_form():
    for ops in (graphs.layernorm_fwd(4, 4096), graphs.layernorm_fwd(4, 770),
                graphs.scaled_masked_softmax((3, 94), 0.125, "full"),
                graphs.bias_gelu_residual_layernorm(5, 8192, "bf16")):
        with Plan(ops) as p:
            info = p.info()
            assert info["schedule"] == "row" and info["n_kernels"] == 1
            assert info["lds_bytes"] > 0 and "CTA" in p.describe()
    # rows that fit a wavefront's registers keep the register-resident form (no LDS)
    with Plan(graphs.layernorm_fwd(4, 2048)) as p:
        assert p.info()["lds_bytes"] == 0


def test_invalid_op_lists():
    ok = graphs.layernorm_fwd(4, 64)

    def mutate(i, **kw):
        ops = list(ok)
        ops[i] = ops[i]._replace(**kw)
        return ops
    _expect(binding.FS_ERR_INVALID, [])                                            # empty
    _expect(binding.FS_ERR_INVALID, mutate(4, operands=(7,)))                       # forward reference
    _expect(binding.FS_ERR_INVALID, mutate(3, axis=5))                              # reduce axis
    _expect(binding.FS_ERR_INVALID, mutate(0, shape=(4, 65)))                       # shape mismatch downstream
    _expect(binding.FS_ERR_INVALID, mutate(0, shape=(4, -64)))                      # negative extent
    _expect(binding.FS_ERR_INVALID, [op for op in ok if op.kind != "output"])       # no output
    _expect(binding.FS_ERR_INVALID, [Op("constant", "f32", (), (), -1, 1.0, ""),
                                     Op("output", "f32", (), (0,), -1, 0.0, "")])    # no parameter / const output
    _expect(binding.FS_ERR_INVALID, ok, wg_size=100)                                # bad launch option
    _expect(binding.FS_ERR_INVALID, ok, wg_size=-64)
    # raw ABI misuse: NULL out pointer, unknown kind/dtype, non-zero reserved field
    lib = binding.lib()
    arr = binding.marshal_ops(ok)
    assert lib.fs_plan_create(arr, len(arr), None, None) == binding.FS_ERR_INVALID
    out = ctypes.c_void_p()
    assert lib.fs_plan_create(None, 3, None, ctypes.byref(out)) == binding.FS_ERR_INVALID
    for field, val in (("kind", 99), ("dtype", 7), ("reserved", 1), ("rank", 9)):
        arr = binding.marshal_ops(ok)
        setattr(arr[2], field, val)
        assert lib.fs_plan_create(arr, len(arr), None, ctypes.byref(out)) == binding.FS_ERR_INVALID
        assert out.value is None
        assert binding.fs_last_error()
    assert lib.fs_destroy(None) == binding.FS_OK


def test_scalar_parameters_and_scalar_groups():
    """A rank-0 parameter is one element in device memory: arithmetic among scalars is an
    elementwise group of one element, and a scalar enters a larger shape through a broadcast."""
    g = graphs.Graph()
    a, b = g.parameter("a", "f32", ()), g.parameter("b", "f32", ())
    g.output(g.sqrt(g.add(a, g.multiply(b, g.constant(2.0)))))
    with Plan(g.ops) as p:
        info = p.info()
        assert info["schedule"] == "elementwise" and info["algorithmic_bytes"] == 12
    g = graphs.Graph()
    f, x = g.parameter("f", "f32", ()), g.parameter("x", "bf16", (33, 100))
    y = g.multiply(g.convert(x, "f32"), g.broadcast(f, (33, 100), 0))
    g.output(g.convert(y, "bf16"))
    with Plan(g.ops) as p:
        assert p.info()["schedule"] == "elementwise"
    with Plan(g.ops, "per_op") as p:
        assert p.info()["n_kernels"] >= 1
    # a scalar is not implicitly broadcast: only constants are
    g = graphs.Graph()
    f, x = g.parameter("f", "f32", ()), g.parameter("x", "f32", (8, 16))
    bad = g.ops + [Op("multiply", "f32", (8, 16), (1, 0), -1, 0.0, ""), Op("output", "f32", (8, 16), (2,), -1, 0.0, "")]
    _expect(binding.FS_ERR_INVALID, bad)


def test_chained_reductions_over_trailing_dims_are_one_reduction():
    """[.., B, C] reduced over C and then over B is a reduction over the B*C elements that lie
    together in memory: one row kernel, not a kernel per link -- as long as nothing in the group
    tells the two dims apart and a leading dim is left."""
    for ops in (graphs.norm_over_trailing_dims((32, 8, 96)), graphs.norm_over_trailing_dims((6, 4, 5, 32), 3, "bf16"),
                graphs.max_abs_over_trailing_dims((64, 3, 50), 2), graphs.max_abs_over_trailing_dims((6, 4, 5, 32), 3, "f16")):
        with Plan(ops) as p:
            info = p.info()
            assert info["schedule"] == "row" and info["n_kernels"] == 1
            assert info["algorithmic_bytes"] == algorithmic_bytes(ops)
    # not when the reduction would leave no row (everything down to a scalar) ...
    _expect(binding.FS_ERR_UNSUPPORTED, graphs.max_abs_over_trailing_dims((64, 50), 2))
    # ... or when an operand tells the trailing dims apart
    g = graphs.Graph()
    x, w = g.parameter("x", "f32", (32, 8, 96)), g.parameter("w", "f32", (96,))
    g.output(g.reduce_sum(g.reduce_sum(g.multiply(x, g.broadcast(w, (32, 8, 96), 2)), 2), 1))
    _expect(binding.FS_ERR_UNSUPPORTED, g.ops)
    # ... or when the inner result is wanted too
    g = graphs.Graph()
    x = g.parameter("x", "f32", (32, 8, 96))
    inner = g.reduce_sum(x, 2)
    g.output(inner)
    g.output(g.reduce_sum(inner, 1))
    _expect(binding.FS_ERR_UNSUPPORTED, g.ops)


def test_launch_without_plan_is_an_error_not_a_crash():
    lib = binding.lib()
    assert lib.fs_launch(None, None, 0, None, 0, None) == binding.FS_ERR_INVALID
    assert lib.fs_plan_info(None, None, None, None, None, None, None) == binding.FS_ERR_INVALID
    assert lib.fs_stream_copy(None, None, 24, None) == binding.FS_ERR_INVALID


# ---------------------------------------------------------------- elementwise schedule (host side)

def test_elementwise_groups_compile_to_one_kernel():
    ops = graphs.adam_update((64, 1024))
    with Plan(ops) as p:
        info = p.info()
        assert info["schedule"] == "elementwise" and info["n_kernels"] == 1
        assert info["workspace_bytes"] == 0
        # four parameters read once, three outputs written once
        assert info["algorithmic_bytes"] == 7 * 64 * 1024 * 4 == info["moved_bytes"]
        assert "THREAD_4" in p.describe() and "cta_size=256" in p.describe() and "generated kernel" in p.describe()
    with Plan(ops, "prebuilt") as p:         # the same group without run-time compilation
        assert p.info()["schedule"] == "elementwise" and "interpreted" in p.describe()
        assert p.info()["lds_bytes"] > 0
    with Plan(ops, "per_op") as q:
        assert q.info()["n_kernels"] > 8 and q.info()["moved_bytes"] > 3 * 7 * 64 * 1024 * 4
    # a last extent that is not a multiple of 4: one element per thread
    with Plan(graphs.adam_update((7, 5))) as p:
        assert "THREAD_4" not in p.describe()
    # widening converts are free: 16-bit storage, fp32 arithmetic
    with Plan(graphs.bias_gelu_residual(32, 1024, "bf16")) as p:
        assert p.info()["schedule"] == "elementwise" and "THREAD_8" in p.describe()   # 16-byte accesses
        assert p.info()["algorithmic_bytes"] == (3 * 32 * 1024 + 1024) * 2


def test_elementwise_limits_are_reported():
    g = Graph()
    x = g.parameter("x", "f32", (8, 64))
    y = x
    for _ in range(70):                      # longer than the register program may be
        y = g.tanh(y)
    g.output(y)
    with Plan(g.ops) as p:                   # the generated kernel has no such limit
        assert "generated kernel" in p.describe()
    e = _expect(binding.FS_ERR_UNSUPPORTED, g.ops, mode="prebuilt")
    assert "64 instructions" in str(e)
    g = Graph()
    x = g.parameter("x", "f32", (8, 64))
    g.output(g.exp(x))
    e = _expect(binding.FS_ERR_INVALID, g.ops, wg_size=512)
    assert "wg_size" in str(e)
    g = Graph()                               # a broadcast of a computed value is not elementwise ...
    x = g.parameter("x", "f32", (8, 64))
    v = g.parameter("v", "f32", (64,))
    g.output(g.add(x, g.col_broadcast(g.exp(v), x)))
    _expect(binding.FS_ERR_UNSUPPORTED, g.ops, mode="prebuilt")
    with Plan(g.ops) as p:                    # ... the row generator takes it: the per-column op is done per row
        assert p.info()["schedule"] == "row" and p.info()["n_kernels"] == 1
    g = Graph()                               # a computed value broadcast along another dim is nobody's
    x = g.parameter("x", "f32", (8, 64, 4))
    v = g.parameter("v", "f32", (64,))
    g.output(g.add(x, g.broadcast(g.exp(v), (8, 64, 4), 1)))
    _expect(binding.FS_ERR_UNSUPPORTED, g.ops)


# ---------------------------------------------------------------- generated row schedule (host side)

def test_row_groups_without_a_hand_written_kernel_get_a_generated_one():
    with Plan(graphs.log_softmax((300, 768))) as p:
        info = p.info()
        assert info["schedule"] == "row" and info["n_kernels"] == 1 and info["workspace_bytes"] == 0
        assert "generated kernel fs_row_" in p.describe() and "WARP" in p.describe()
        assert info["algorithmic_bytes"] == 2 * 300 * 768 * 4
    with Plan(graphs.log_softmax((300, 5))) as p:            # short unaligned rows: one thread per row
        assert "THREAD]" in p.describe()
    with Plan(graphs.log_softmax((3, 8192))) as p:           # long rows: one workgroup per row
        assert "CTA-S" in p.describe() and p.info()["lds_bytes"] > 0
    # the same source is compiled once per process: equal groups share a kernel name
    with Plan(graphs.rmsnorm((64, 256))) as a, Plan(graphs.rmsnorm((64, 256))) as b:
        assert a.describe() == b.describe()
    # full and per-row outputs in one tuple
    with Plan(graphs.layernorm_fwd_with_stats(64, 1024)) as p:
        assert p.info()["algorithmic_bytes"] == (2 * 64 * 1024 + 2 * 1024 + 2 * 64) * 4


def test_per_row_arithmetic_without_a_reduction_is_a_row_group():
    # ops of the full and of the per-row shape in one group: not an elementwise group (one shape),
    # the row generator takes it with the largest computed shape as the full shape
    with Plan(graphs.gated_rows((300, 96))) as p:
        info = p.info()
        assert info["schedule"] == "row" and info["n_kernels"] == 1
        assert info["algorithmic_bytes"] == (2 * 300 * 96 + 2 * 300 + 96) * 4
    with pytest.raises(FsError) as e:
        Plan(graphs.gated_rows((300, 96)), mode="prebuilt")
    assert e.value.status == binding.FS_ERR_UNSUPPORTED


def _gelu_group(extra_output):
    """tanh-form GELU of x + 1 on [64, 256]; optionally the tanh itself is a second output."""
    from workloads.graphs import GELU_K0, GELU_K1
    g = Graph()
    x = g.parameter("x", "f32", (64, 256))
    h = g.add(x, g.constant(1.0))
    h3 = g.multiply(g.multiply(h, h), h)
    t = g.tanh(g.multiply(g.add(h, g.multiply(h3, g.constant(GELU_K1))), g.constant(GELU_K0)))
    # operands commuted against the usual spelling
    g.output(g.multiply(g.add(g.constant(1.0), t), g.multiply(g.constant(0.5), h)), "y")
    if extra_output:
        g.output(t, "t")
    return g.ops


def test_gelu_idiom_is_generated_as_one_op():
    with Plan(_gelu_group(False)) as p:
        assert "x2 merged" in p.describe()          # the add and the GELU
    with Plan(_gelu_group(True)) as p:              # an interior value leaves the group: ops stay spelled out
        assert "x10 merged" in p.describe()
    with Plan(BY_NAME["bias_gelu_residual_layernorm"].build("small")[0]) as p:
        assert "elementwise x13" in p.describe()    # 21 with the GELU spelled out


def test_sum_over_all_leading_dims_is_one_column_reduction():
    def bias_grad(partial_is_output):
        g = Graph()
        dy = g.parameter("dy", "f32", (4, 50, 256))
        x = g.parameter("x", "f32", (4, 50, 256))
        dx = g.multiply(dy, g.tanh(x))
        g.output(dx, "dx")
        part = g.reduce_sum(dx, 0)                   # [50, 256]
        if partial_is_output:
            g.output(part, "partial")
        g.output(g.reduce_sum(part, 0), "dbias")     # [256]
        return g.ops
    with Plan(bias_grad(False)) as p:
        info = p.info()
        assert info["schedule"] == "row_col" and info["n_kernels"] == 2 and "column reduce x1" in p.describe()
    # the sum over only the first dim is neither a per-row nor a per-column value
    _expect(binding.FS_ERR_UNSUPPORTED, bias_grad(True))
    with Plan(bias_grad(True), mode="per_op") as p:
        assert p.info()["n_kernels"] >= 4


def test_generated_mode_and_prebuilt_mode_on_recognised_groups():
    ops, _ = BY_NAME["layernorm_fwd"].build("small")
    with Plan(ops) as p:
        assert "generated" not in p.describe()               # hand-written by default
    with Plan(ops, "generated") as p:
        assert p.info()["schedule"] == "row" and "generated kernel" in p.describe()
    with Plan(ops, "prebuilt") as p:
        assert "generated" not in p.describe()
    # without run-time compilation a row group that only the generator covers is unsupported
    _expect(binding.FS_ERR_UNSUPPORTED, graphs.log_softmax((8, 64)), mode="prebuilt")
    # lanes per row is the launch template of the generated kernels
    with Plan(graphs.log_softmax((300, 64)), rows_per_wave=16) as p:
        assert "THREAD_16" in p.describe()                   # 4 lanes per row, 16 elements per lane
    _expect(binding.FS_ERR_INVALID, graphs.log_softmax((300, 64)), rows_per_wave=3)
    # rows beyond the register templates are streamed in passes; Algorithm 4 lays out the LDS row buffers
    with Plan(graphs.log_softmax((2, 40000))) as p:
        assert "streamed in 3 passes" in p.describe() and "1 taken over" in p.describe()
        assert p.info()["lds_bytes"] <= 160 * 1024
    with Plan(graphs.log_softmax((2, 262144))) as p:
        assert "re-read per pass" in p.describe()
    with Plan(graphs.log_softmax((300, 64)), grid=8, wg_size=512) as p:
        assert "streamed" in p.describe() and "cta_num=8" in p.describe() and "cta_size=512" in p.describe()
    _expect(binding.FS_ERR_INVALID, graphs.log_softmax((300, 64)), wg_size=512)    # register templates: up to 256


def test_motivating_pattern_plans_as_one_kernel():
    ops = graphs.multi_interest_pattern(16384)
    with Plan(ops) as p:
        info = p.info()
        assert info["schedule"] == "row" and info["n_kernels"] == 1
        assert "reduce x3" in p.describe()                   # max, sum, and the second dot
        # two 552 MiB outputs, the inputs are megabytes
        assert info["algorithmic_bytes"] == 1201274880
        assert info["lds_bytes"] > 0                         # the staging tile of the dense stores
    with Plan(ops, "per_op") as q:
        assert q.info()["n_kernels"] == 13
        assert q.info()["moved_bytes"] > 6 * info["algorithmic_bytes"]


def test_tuning_cache_on_the_host(tmp_path):
    """The cache that fs_plan_tune fills: keys, file round trip, and its use by fs_plan_create
    when the caller leaves the launch parameters open."""
    from paper_1911_11576_amd import (fs_group_key, fs_tune_cache_clear, fs_tune_cache_load, fs_tune_cache_save,
                                      fs_tune_cache_size)
    fs_tune_cache_clear()
    ops = graphs.log_softmax((300, 768))
    key = fs_group_key(ops)
    assert key == fs_group_key(graphs.log_softmax((300, 768)))              # a function of the group alone
    assert key != fs_group_key(graphs.log_softmax((301, 768))) and key != fs_group_key(graphs.log_softmax((300, 768), "bf16"))
    with Plan(ops) as p:
        default = p.describe()
    with Plan(ops, rows_per_wave=2) as p:
        wide = p.describe()
    assert wide != default
    f = tmp_path / "tune.txt"
    f.write_text("fs-tune-cache 1\n%016x 0 0 2 0 12.500\n" % key)
    fs_tune_cache_load(f)
    assert fs_tune_cache_size() == 1
    with Plan(ops) as p:                                                    # launch parameters left open: the recorded ones
        assert p.describe() == wide
    with Plan(ops, rows_per_wave=1) as p:                                   # explicit options never look
        assert p.describe() == default
    with Plan(graphs.log_softmax((301, 768))) as p:                         # another group
        assert "THREAD_12" in p.describe()
    # round trip through a file
    g = tmp_path / "again.txt"
    fs_tune_cache_save(g)
    fs_tune_cache_clear()
    assert fs_tune_cache_size() == 0
    with Plan(ops) as p:
        assert p.describe() == default
    fs_tune_cache_load(g)
    assert fs_tune_cache_size() == 1 and g.read_text() == f.read_text()
    # recorded options that do not build (written by something else): the defaults, silently
    f.write_text("fs-tune-cache 1\n%016x 0 100 0 0 1.000\n" % key)
    fs_tune_cache_load(f)
    with Plan(ops) as p:
        assert p.describe() == default
    # malformed files merge nothing
    for text in ("", "something else\n", "fs-tune-cache 1\nzz 0 0 0 0 1\n", "fs-tune-cache 1\n%016x 1 0 0 0 1.0\n" % key,
                 "fs-tune-cache 1\n%016x 0 0 2 0\n" % key, "fs-tune-cache 1\n%016x 0 -1 2 0 1.0\n" % key):
        f.write_text(text)
        with pytest.raises(FsError) as e:
            fs_tune_cache_load(f)
        assert e.value.status == binding.FS_ERR_INVALID and "fs_tune_cache_load" in e.value.message
    with pytest.raises(FsError):
        fs_tune_cache_load(tmp_path / "missing.txt")
    with pytest.raises(FsError):
        fs_tune_cache_save(tmp_path / "no_such_dir" / "x.txt")
    assert fs_tune_cache_size() == 1
    fs_tune_cache_clear()


def test_compiled_kernels_are_kept_on_disk_between_processes(tmp_path):
    """The kernel cache directory: a generated kernel is compiled once, found in memory after that,
    and found on disk by a process (here: after dropping the in-memory copies) that has not compiled it."""
    import time
    from paper_1911_11576_amd import fs_kernel_cache_dir, fs_kernel_cache_drop_memory, fs_kernel_cache_stats
    ops = graphs.log_softmax((41, 1234))                       # a shape nothing else in the suite uses
    try:
        fs_kernel_cache_dir(tmp_path)
        fs_kernel_cache_drop_memory()
        s0 = fs_kernel_cache_stats()
        t0 = time.perf_counter()
        with Plan(ops) as p:
            first = p.describe()
        t_compile = time.perf_counter() - t0
        s1 = fs_kernel_cache_stats()
        assert s1["compiled"] == s0["compiled"] + 1 and s1["from_disk"] == s0["from_disk"]
        files = sorted(tmp_path.glob("fs_*.co"))
        assert len(files) == 1 and files[0].stat().st_size > 1000 and not list(tmp_path.glob("*.tmp.*"))
        with Plan(ops) as p:                                    # same process: memory
            assert p.describe() == first
        s2 = fs_kernel_cache_stats()
        assert s2["from_memory"] == s1["from_memory"] + 1 and s2["compiled"] == s1["compiled"]
        fs_kernel_cache_drop_memory()                           # as a new process would start
        t0 = time.perf_counter()
        with Plan(ops) as p:
            assert p.describe() == first                        # same code object: same size in the description
        t_disk = time.perf_counter() - t0
        s3 = fs_kernel_cache_stats()
        assert s3["from_disk"] == s2["from_disk"] + 1 and s3["compiled"] == s2["compiled"]
        assert t_disk < t_compile / 3, (t_disk, t_compile)
        # a damaged file is ignored and replaced
        files[0].write_bytes(files[0].read_bytes()[:200])
        fs_kernel_cache_drop_memory()
        with Plan(ops) as p:
            assert p.describe() == first
        s4 = fs_kernel_cache_stats()
        assert s4["compiled"] == s3["compiled"] + 1 and files[0].stat().st_size > 1000
        # ... and so is a file of the right length with one byte flipped in the middle of the code, or in the
        # identity text that says which source, options and compiler the code belongs to
        good = files[0].read_bytes()
        for at in (len(good) // 2 + 1000, 100):
            bad = bytearray(good)
            bad[min(at, len(bad) - 1)] ^= 0x40
            files[0].write_bytes(bytes(bad))
            fs_kernel_cache_drop_memory()
            before = fs_kernel_cache_stats()
            with Plan(ops) as p:
                assert p.describe() == first
            after = fs_kernel_cache_stats()
            assert after["compiled"] == before["compiled"] + 1 and after["from_disk"] == before["from_disk"], at
            assert files[0].read_bytes() == good                # replaced by the fresh compile
        s4 = fs_kernel_cache_stats()
        # without a directory nothing is read or written
        fs_kernel_cache_dir(None)
        fs_kernel_cache_drop_memory()
        for f in tmp_path.glob("fs_*.co"):
            f.unlink()
        with Plan(ops) as p:
            pass
        assert not list(tmp_path.glob("fs_*.co")) and fs_kernel_cache_stats()["compiled"] == s4["compiled"] + 1
    finally:
        fs_kernel_cache_dir(None)


def test_plans_are_created_concurrently_from_several_threads():
    """Plan creation is thread-safe: run-time compilation, the kernel and tuning caches, the per-thread
    error message."""
    import threading
    problems = []

    def work(k):
        try:
            for j in range(2):
                with Plan(graphs.log_softmax((50 + k, 96 + 8 * j))) as p:
                    assert "generated kernel" in p.describe() and p.info()["algorithmic_bytes"] == 2 * (50 + k) * (96 + 8 * j) * 4
                with pytest.raises(FsError) as e:                   # each thread sees its own message
                    Plan(graphs.log_softmax((50 + k, 96)), wg_size=100 + k)
                assert "wg_size" in e.value.message
        except Exception as exc:            # collected, not raised in the thread
            problems.append((k, repr(exc)))

    threads = [threading.Thread(target=work, args=(k,)) for k in range(4)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not problems, problems


# ---------------------------------------------------------------- schedule 3 with prologue and epilogue

def test_attention_block_forms_are_recognised():
    cases = [dict(), dict(causal=True), dict(mask="key"), dict(mask="full", causal=True), dict(mask="shared"),
             dict(mask="key", causal=True, mask_outside_causal=True), dict(gate=True), dict(residual=True),
             dict(gate=True, residual=True, lse=True), dict(lse=True, mask="key", causal=True)]
    for kw in cases:
        for sq, sk in ((64, 64), (40, 72), (100, 24)):
            with Plan(graphs.attention_block(3, sq, sk, 64, "f16", **kw)) as p:
                info, text = p.info(), p.describe()
                assert info["schedule"] == "bdot_softmax" and info["n_kernels"] == 1 and info["workspace_bytes"] == 0, (kw, sq, sk)
                assert ("add_mask" in text) == ("mask" in kw) and ("logsumexp" in text) == bool(kw.get("lse"))
                assert ("multiply_gate" in text) == bool(kw.get("gate")) and ("add_residual" in text) == bool(kw.get("residual"))
                # one wavefront per 16 query rows; V^T of the (padded) key tiles in LDS
                nq = 1 if sq <= 16 else 2 if sq <= 32 else 4 if sq <= 64 else 8
                nk = 2 if sk <= 32 else 4 if sk <= 64 else 8
                assert f"cta_size={64 * nq}" in text and info["lds_bytes"] == 2 * (nk * 16 * (64 + 8) + nk * 16 * (64 + 8))


def test_attention_block_forms_beyond_the_hand_written_kernel():
    # lengths beyond the fine-grained schedules: refused by both the hand-written kernel and the generator
    _expect(binding.FS_ERR_UNSUPPORTED, graphs.attention_block(2, 32, 200, 64))
    _expect(binding.FS_ERR_UNSUPPORTED, graphs.attention_block(2, 200, 32, 64))
    # a finite causal fill under a mask that is added afterwards (the fill value is shifted by the mask): not the
    # hand-written kernel's form -- the generated block-composed kernel takes it
    with Plan(graphs.attention_block(2, 32, 32, 64, causal=True, fill=-1e4, mask="key", mask_outside_causal=True)) as p:
        assert p.info()["schedule"] == "block_dot"
    # a mask inside the scale, scale * (dot + mask): likewise
    g = Graph()
    q = g.parameter("q", "f16", (2, 32, 64)); k = g.parameter("k", "f16", (2, 32, 64)); v = g.parameter("v", "f16", (2, 32, 64))
    m = g.parameter("m", "f32", (2, 32, 32))
    z = g.multiply(g.add(g.dot(q, k, transpose_b=True, dtype="f32"), m), g.constant(0.125))
    zmax = g.reduce_max(z, -1)
    e = g.exp(g.subtract(z, g.row_broadcast(zmax, z)))
    p = g.convert(g.divide(e, g.row_broadcast(g.reduce_sum(e, -1), e)), "f16")
    g.output(g.convert(g.dot(p, v, dtype="f32"), "f16"))
    with Plan(g.ops) as p:
        assert p.info()["schedule"] == "block_dot"


# ---------------------------------------------------------------- generated block composition around MFMA dots

def _dot_group(dtype="f16", kc=64, transpose_b=True, after=False, d=64):
    g = Graph()
    B, M, N = 2, 32, 48
    q = g.parameter("q", dtype, (B, M, kc))
    k = g.parameter("k", dtype, (B, N, kc) if transpose_b else (B, kc, N))
    v = g.parameter("v", dtype, (B, N, d))
    p = g.logistic(g.dot(q, k, transpose_b=transpose_b, dtype="f32"))
    o = g.dot(g.convert(p, dtype) if dtype != "f32" else p, v, dtype="f32")
    if after:
        o = g.multiply(o, g.constant(2.0))
    g.output(o)
    return g.ops


def test_block_dot_groups_are_generated_or_refused_with_a_reason():
    with Plan(_dot_group()) as p:
        info = p.info()
        assert info["schedule"] == "block_dot" and info["n_kernels"] == 1 and info["workspace_bytes"] == 0
        # V (64 keys of 64 + 8 halves), placed by the shared-memory planner, and behind it the first dot's second
        # operand (64 rows of 64 + 8 halves), which one wavefront per 16 rows loads for all
        assert info["lds_bytes"] == 2 * 64 * (64 + 8) + 2 * 64 * (64 + 8)
        assert "dot_1" in p.describe() and "dot_2" in p.describe() and "MFMA" in p.describe()
    assert "matrix unit" in _expect(binding.FS_ERR_UNSUPPORTED, _dot_group("f32"))            # fp32 dots have no MFMA path
    # the second operand stored [B, K, N] (contraction along its rows): kept in LDS as stored, whole 32-steps of rows
    # (64) of whole 16-column tiles (48 -> 64 columns, + 8 halves of padding)
    with Plan(_dot_group(transpose_b=False)) as p:
        assert p.info()["schedule"] == "block_dot" and p.info()["lds_bytes"] == 2 * 64 * (64 + 8) + 2 * 64 * (64 + 8)
    # elementwise ops after the consuming dot run on its accumulators (same kernel, same LDS), and so do
    # reductions over its rows; a reduction over another dim of its result does not
    with Plan(_dot_group(after=True)) as p:
        info = p.info()
        assert info["schedule"] == "block_dot" and info["n_kernels"] == 1 and info["lds_bytes"] == 2 * 64 * (64 + 8) + 2 * 64 * (64 + 8)
    g = Graph()
    q = g.parameter("q", "f16", (2, 32, 64)); k = g.parameter("k", "f16", (2, 48, 64)); v = g.parameter("v", "f16", (2, 48, 64))
    o = g.dot(g.convert(g.logistic(g.dot(q, k, transpose_b=True, dtype="f32")), "f16"), v, dtype="f32")
    g.output(g.reduce_sum(o, -1))
    with Plan(g.ops) as p:
        assert p.info()["schedule"] == "block_dot" and p.info()["n_kernels"] == 1
    g = Graph()
    q = g.parameter("q", "f16", (2, 32, 64)); k = g.parameter("k", "f16", (2, 48, 64)); v = g.parameter("v", "f16", (2, 48, 64))
    o = g.dot(g.convert(g.logistic(g.dot(q, k, transpose_b=True, dtype="f32")), "f16"), v, dtype="f32")
    g.output(g.reduce_sum(o, 1))
    assert "not over the last dim" in _expect(binding.FS_ERR_UNSUPPORTED, g.ops)
    # an operand of the ops after the dot with the wrong shape ([B, M, N] where [B, M, D] is needed)
    g = Graph()
    q = g.parameter("q", "f16", (2, 32, 64)); k = g.parameter("k", "f16", (2, 48, 64)); v = g.parameter("v", "f16", (2, 48, 32))
    w = g.parameter("w", "f32", (2, 32, 48))
    o = g.dot(g.convert(g.logistic(g.dot(q, k, transpose_b=True, dtype="f32")), "f16"), v, dtype="f32")
    bad = g._new("add", "f32", (2, 32, 32), (o, w))
    g.output(bad)
    _expect(binding.FS_ERR_INVALID, g.ops)        # the op list itself is malformed: operand shapes differ
    assert "32, 64 or 128" in _expect(binding.FS_ERR_UNSUPPORTED, _dot_group(d=48))
    assert "multiple of 8" in _expect(binding.FS_ERR_UNSUPPORTED, _dot_group(kc=20))
