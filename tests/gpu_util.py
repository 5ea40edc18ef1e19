"""Helpers for the GPU parity tests: run a group through the C ABI and compare with the
oracle element by element."""
import numpy as np
import torch

from paper_1911_11576_amd import Plan
from workloads import TOLERANCE, inputs as wl_inputs

_TORCH = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def param_dtypes(ops):
    return [op.dtype for op in ops if op.kind == "parameter"]


def output_specs(ops):
    return [(op.shape, op.dtype) for op in ops if op.kind == "output"]


def to_device(ops, ins, device="cuda:0"):
    return [wl_inputs.to_torch(a, dt, device) for a, dt in zip(ins, param_dtypes(ops))]


def alloc_outputs(ops, device="cuda:0"):
    # NaN-filled so that an element the kernel never writes fails the comparison
    return [torch.full(shape, float("nan"), dtype=_TORCH[dt], device=device) for shape, dt in output_specs(ops)]


def run_gpu(ops, ins, mode="stitched", launches=1, **opts):
    """-> list of float64 numpy outputs computed by the HIP library."""
    dev_in = to_device(ops, ins)
    dev_out = alloc_outputs(ops)
    with Plan(ops, mode, **opts) as plan:
        for _ in range(launches):
            plan.launch(dev_in, dev_out)
        torch.cuda.synchronize()
    return [t.to(torch.float64).cpu().numpy() for t in dev_out]


def group_dtype(ops):
    """Storage dtype that sets the comparison bar: 16-bit if any parameter or output is."""
    for op in ops:
        if op.kind in ("parameter", "output") and op.dtype != "f32":
            return op.dtype
    return "f32"


def assert_close(got, want, tol, what="", slack=None):
    """|got - want| <= tol + tol*|want| (+ slack, an array of further absolute room per element, when a caller
    derives one) for every element; NaN anywhere fails."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    if got.size == 0:
        return
    err = np.abs(got - want)
    bound = tol + tol * np.abs(want)
    if slack is not None:
        bound = bound + np.broadcast_to(np.asarray(slack, dtype=np.float64), want.shape)
    bad = ~(err <= bound)          # also true for NaN
    if bad.any():
        k = np.unravel_index(np.argmax(np.where(np.isnan(err), np.inf, err - bound)), err.shape)
        raise AssertionError(
            f"{what}: {int(bad.sum())} of {got.size} elements outside tol {tol}; worst at {k}: "
            f"got {got[k]!r} want {want[k]!r}")


def check_against_oracle(ops, ins, mode="stitched", tol=None, what="", **opts):
    from oracle import interp
    want = interp.run(ops, ins)
    got = run_gpu(ops, ins, mode, **opts)
    tol = TOLERANCE[group_dtype(ops)] if tol is None else tol
    for i, (a, b) in enumerate(zip(got, want)):
        assert_close(a, b, tol, f"{what} output {i} ({mode})")
    return got, want
