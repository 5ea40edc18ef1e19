"""fs_launch_static -- the launch that allocates nothing -- against fs_launch, through the C ABI:
same kernels on the library's static scratch array instead of a plan-owned workspace, so the
outputs must be bit-identical.  Two calls in a row, the second on a smaller input: the array keeps
the first call's contents and the second call must not be disturbed by them."""
import numpy as np
import pytest
import torch

from gpu_util import alloc_outputs, assert_close, to_device
from oracle import interp
from paper_1911_11576_amd import FsError, Plan, binding
from workloads import BY_NAME, graphs

pytestmark = pytest.mark.gpu


def _both(ops, ins, mode):
    """-> (outputs of fs_launch, outputs of fs_launch_static), float64 numpy, same plan."""
    dev_in = to_device(ops, ins)
    ref, got = alloc_outputs(ops), alloc_outputs(ops)
    with Plan(ops, mode) as plan:
        assert plan.info()["workspace_bytes"] > 0          # the case the entry point exists for
        plan.launch(dev_in, ref)                           # also puts a generated kernel on the device
        torch.cuda.synchronize()
        plan.launch_static(dev_in, got)
        torch.cuda.synchronize()
    f = lambda ts: [t.to(torch.float64).cpu().numpy() for t in ts]
    return f(ref), f(got)


@pytest.mark.parametrize("mode", ["stitched", "generated"])
def test_static_launch_matches_fs_launch_twice_second_smaller(mode):
    cfg = BY_NAME["layernorm_bwd"]
    for rows in (1500, 203):                               # the second call is the smaller one
        print(f"fs_launch_static layernorm_bwd rows={rows} mode={mode}", flush=True)
        ops, ins = cfg.build("small", rows=rows)
        ref, got = _both(ops, ins, mode)
        want = interp.run(ops, ins)
        for r, g, w in zip(ref, got, want):
            assert np.array_equal(r, g)                    # same kernels, fixed summation order: bit-identical
            assert_close(g, w, 1e-5, f"static launch rows={rows} ({mode})")


def test_static_launch_per_op_plan_and_limits():
    # a per-op plan keeps its intermediates in scratch memory: small ones fit the static array
    ops, ins = BY_NAME["layernorm_fwd"].build("small")
    ref, got = _both(ops, ins, "per_op")
    for r, g in zip(ref, got):
        assert np.array_equal(r, g)
    # beyond the array: a clear error, nothing launched
    big = BY_NAME["layernorm_fwd"].graph_fn(rows=8192, cols=768)
    with Plan(big, "per_op") as plan:
        assert plan.info()["workspace_bytes"] > 8 * 2**20
        x = [torch.zeros(op.shape, device="cuda:0") for op in big if op.kind == "parameter"]
        y = [torch.zeros(op.shape, device="cuda:0") for op in big if op.kind == "output"]
        with pytest.raises(FsError) as e:
            plan.launch_static(x, y)
        assert e.value.status == binding.FS_ERR_UNSUPPORTED and "static array" in e.value.message
    # a generated kernel that was never launched is not on the device yet
    ops, ins = BY_NAME["layernorm_bwd"].build("small")
    with Plan(ops, "generated") as plan:
        with pytest.raises(FsError) as e:
            plan.launch_static(to_device(ops, ins), alloc_outputs(ops))
        assert e.value.status == binding.FS_ERR_INVALID and "fs_launch" in e.value.message
