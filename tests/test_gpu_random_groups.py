"""Parity fuzzing of the kernel generators: random groups (elementwise ops on full and per-row
values, reductions over the last dim, broadcasts back, optional column sums) are planned, run
on the GPU and compared with the CPU oracle, through every template that takes them."""
import random
import sys

import pytest

from paper_1911_11576_amd import FsError, Plan, binding
from workloads import graphs, inputs

from gpu_util import check_against_oracle

pytestmark = pytest.mark.gpu


def announce(msg):
    sys.__stderr__.write(f"[gpu-case] {msg}\n")
    sys.__stderr__.flush()


@pytest.fixture(autouse=True)
def _need_gpu(device):
    yield


SHAPES = [(37, 128), (5, 768), (3, 7, 64), (2, 3, 5, 32), (300, 8), (33, 100), (65, 30), (7, 770), (4, 4096), (129, 16)]


@pytest.mark.parametrize("seed", range(24))
def test_random_row_groups(seed):
    rng = random.Random(4242 + seed)
    shape = SHAPES[seed % len(SHAPES)]
    dtype = ["f32", "f32", "bf16", "f16"][seed % 4]
    ops, pshapes = graphs.random_row_group(rng, shape, dtype, n_ops=rng.randint(6, 16))
    ins = inputs.normal_tensors(pshapes, dtype, seed_offset=100 + seed)
    announce(f"random row group seed {seed} shape {shape} {dtype}: {len(ops)} ops")
    with Plan(ops) as p:
        schedule = p.info()["schedule"]
        assert schedule in ("row", "elementwise")
        streamed = "streamed" in p.describe()
    check_against_oracle(ops, ins, what=f"random group {seed}")
    if schedule == "row":
        if not streamed:
            check_against_oracle(ops, ins, what=f"random group {seed} streamed", grid=3)
        try:
            check_against_oracle(ops, ins, what=f"random group {seed} persistent", grid=2, rows_per_wave=1)
        except FsError as e:
            assert e.status == binding.FS_ERR_UNSUPPORTED      # rows too long for one wavefront's registers


@pytest.mark.parametrize("seed", range(15))
def test_random_groups_with_column_sums(seed):
    rng = random.Random(777 + seed)
    # (rank above 2: the sum over the rows is a chain of sums over the leading dim)
    shape = [(37, 128), (300, 8), (33, 100), (517, 1024), (65, 30), (5, 2048), (1000, 64), (129, 16),
             (40, 4096), (33, 3000), (9, 8192), (3, 7, 64), (2, 3, 5, 32), (2, 9, 4096), (4, 50, 100)][seed]
    ops, pshapes = graphs.random_row_group(rng, shape, "f32", n_ops=rng.randint(5, 12), column_sums=True)
    ins = inputs.normal_tensors(pshapes, "f32", seed_offset=200 + seed)
    announce(f"random group with column sum seed {seed} shape {shape}: {len(ops)} ops")
    with Plan(ops) as p:
        assert p.info()["schedule"] == "row_col" and p.info()["n_kernels"] == 2
    check_against_oracle(ops, ins, what=f"random column group {seed}")
    check_against_oracle(ops, ins, what=f"random column group {seed} grid 3", grid=3, wg_size=128)


@pytest.mark.parametrize("seed", range(12))
def test_random_groups_with_column_sums_per_run_of_rows(seed):
    """Random row groups whose extra outputs are sums over the innermost row dims ([B, S, H] over S;
    [B, N, S, H] over S, or over S and N): runs of 1 to 600 rows, one or several workgroups per run,
    rows of one wavefront and of a team."""
    rng = random.Random(4242 + seed)
    shape = [(37, 5, 128), (300, 7, 8), (3, 600, 100), (2, 3, 5, 32), (65, 2, 30), (5, 9, 2048), (1, 64, 64), (4, 1, 96),
             (6, 20, 4096), (2, 4, 50, 100), (700, 3, 64), (2, 2, 2, 2)][seed]
    dtype = ["f32", "bf16", "f16"][seed % 3]
    ops, pshapes = graphs.random_row_group(rng, shape, dtype, n_ops=rng.randint(4, 12), column_sums="runs")
    ins = inputs.normal_tensors(pshapes, dtype, seed_offset=400 + seed)
    announce(f"random group with column sums per run seed {seed} shape {shape} {dtype}: {len(ops)} ops")
    with Plan(ops) as p:
        assert p.info()["schedule"] == "row_col" and "per run of" in p.describe()
    check_against_oracle(ops, ins, what=f"random run-sum group {seed}")
    check_against_oracle(ops, ins, what=f"random run-sum group {seed} wg 128", wg_size=128)


@pytest.mark.parametrize("shape,dtype", [((300, 96), "f32"), ((7, 5, 33), "f32"), ((64, 2048), "bf16"), ((1000, 4), "f16")])
def test_per_row_arithmetic_without_a_reduction(shape, dtype):
    ops = graphs.gated_rows(shape, dtype)
    ins = inputs.normal_tensors([shape, shape[:-1], shape[-1:]], dtype, seed_offset=31)
    announce(f"gated rows {shape} {dtype}")
    check_against_oracle(ops, ins, what=f"gated rows {shape}")
    check_against_oracle(ops, ins, what=f"gated rows {shape} streamed", grid=5)


POOL = [(37, 128), (5, 768), (3, 7, 64), (2, 3, 5, 32), (300, 8), (33, 100), (65, 30), (7, 770), (4, 4096), (129, 16),
        (6, 40000), (50, 2), (9, 1), (3, 2, 2, 2), (17, 6000)]


@pytest.mark.parametrize("seed", range(45))
def test_random_groups_wide_pool(seed):
    """More shapes (rows of 1 or 2 elements, rows for the streamed template, rows for wavefront
    teams), all three dtypes, 3 to 24 ops, a column sum on every fourth rank-2 case."""
    rng = random.Random(9000 + seed)
    shape = POOL[seed % len(POOL)]
    dtype = ["f32", "bf16", "f16"][seed % 3]
    col = seed % 4 == 3 and len(shape) == 2
    ops, pshapes = graphs.random_row_group(rng, shape, dtype, n_ops=rng.randint(3, 24), column_sums=col)
    ins = inputs.normal_tensors(pshapes, dtype, seed_offset=300 + seed)
    announce(f"random group (wide pool) seed {seed} shape {shape} {dtype} column sum {col}: {len(ops)} ops")
    try:
        check_against_oracle(ops, ins, what=f"random group {seed}")
    except FsError as e:
        # the one documented limit this pool reaches
        assert e.status == binding.FS_ERR_UNSUPPORTED and "column reductions over rows longer" in e.message


@pytest.mark.parametrize("seed", range(20))
def test_random_packed_elementwise_parts(seed):
    """Independent elementwise computations of different shapes and dtypes in one op list: one kernel,
    each part on its own run of workgroups."""
    import numpy as np
    rng = random.Random(5000 + seed)
    ops, pshapes, pdtypes = graphs.random_elementwise_parts(rng)
    r = np.random.default_rng(seed)
    ins = [inputs.round_to(r.normal(0.0, 1.0, s), dt) for s, dt in zip(pshapes, pdtypes)]
    announce(f"random packed parts seed {seed}: {len(ops)} ops, shapes {pshapes[::3]}")
    with Plan(ops) as p:
        assert p.info()["schedule"] == "elementwise" and p.info()["n_kernels"] == 1
    check_against_oracle(ops, ins, what=f"random packed parts {seed}")


DOT_SHAPES = [(3, 64, 64, 64, 64), (2, 37, 52, 40, 32), (4, 16, 128, 32, 128), (2, 100, 36, 72, 64), (5, 1, 8, 16, 32),
              (2, 128, 128, 128, 64), (3, 50, 20, 24, 32), (2, 33, 100, 64, 128)]


@pytest.mark.parametrize("seed", range(32))
def test_random_groups_around_two_dots(seed):
    """dot -> random middle section -> dot -> random epilogue (elementwise ops and row reductions on the second
    dot's result), the first dot's second operand stored either way, f16 and bf16: all through the generated
    block-composed kernel (the hand-written attention kernel is not asked), one kernel each."""
    import numpy as np
    rng = random.Random(12000 + seed)
    B, M, N, Kc, D = DOT_SHAPES[seed % len(DOT_SHAPES)]
    dtype = ["f16", "bf16"][seed % 2]
    ops, params = graphs.random_dot_group(rng, B, M, N, Kc, D, dtype)
    r = np.random.Generator(np.random.PCG64(inputs.BASE_SEED + 400 + seed))
    ins = [inputs.round_to(r.normal(0.0, 1.0, shape), dt) for shape, dt in params]
    announce(f"random group around two dots, seed {seed} {B}x{M}x{N} K={Kc} D={D} {dtype}: {len(ops)} ops")
    with Plan(ops, "generated") as plan:
        assert plan.info()["schedule"] == "block_dot" and plan.info()["n_kernels"] == 1
    check_against_oracle(ops, ins, "generated", what=f"random dot group {seed}")
