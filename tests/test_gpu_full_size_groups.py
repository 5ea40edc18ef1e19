"""The groups that `bench.py --full` times beyond the five configs, at the sizes it times them, against the
oracle: whole tensors where the oracle's float64 intermediates fit comfortably, batch slices where they do not
(the motivating pattern: 1.2 GB of outputs; its batch elements are independent)."""
import sys

import numpy as np
import pytest
import torch

from oracle import interp
from paper_1911_11576_amd import Plan
from workloads import BY_NAME, EXTRA_GROUPS, TOLERANCE

from gpu_util import alloc_outputs, assert_close, group_dtype, to_device

pytestmark = pytest.mark.gpu


def announce(msg):
    sys.__stderr__.write(f"[gpu-case] {msg}\n")
    sys.__stderr__.flush()


@pytest.fixture(autouse=True)
def _need_gpu(device):
    yield


def _run_stitched(ops, ins):
    dev_in, dev_out = to_device(ops, ins), alloc_outputs(ops)
    with Plan(ops) as plan:
        schedule = plan.info()["schedule"]
        plan.launch(dev_in, dev_out)
        torch.cuda.synchronize()
    return [t.to(torch.float64).cpu().numpy() for t in dev_out], schedule


def _long_sum_slack(ops, vals, j):
    """Further room for an fp32 output that is a sum of more than 2048 terms (the column sums over 16384 rows):
    every term t_i reaches the sum with the rounding of the fp32 chain that made it, a few units of 2^-24 * |t_i|,
    independent from term to term, so the sum is off by about 4 * 2^-24 * sqrt(sum t_i^2) whatever the order
    of the additions (the oracle itself, rounding every intermediate to fp32, misses 1e-5 on such sums by up to
    3e-5).  None for every other output."""
    src = ops[ops[j].operands[0]]
    if src.kind != "reduce_sum" or src.dtype != "f32":
        return None
    t = np.asarray(vals[src.operands[0]])
    if t.size // max(1, np.asarray(vals[j]).size) <= 2048:
        return None
    return 4.0 * 2.0 ** -24 * np.sqrt((t * t).sum(axis=src.axis))


WHOLE = [c.name for c in EXTRA_GROUPS if c.name != "multi_interest_pattern"]


@pytest.mark.parametrize("name", WHOLE)
def test_bench_group_at_full_size_whole_tensors(name):
    cfg = BY_NAME[name]
    announce(f"full size {name} {cfg.full}")
    ops, ins = cfg.build("full")
    got, schedule = _run_stitched(ops, ins)
    assert schedule != "per_op"
    vals = interp.run(ops, ins, keep=True)
    tol = TOLERANCE[group_dtype(ops)]
    outputs = [j for j, op in enumerate(ops) if op.kind == "output"]
    assert len(outputs) == len(got)
    for i, j in enumerate(outputs):
        assert_close(got[i], vals[j], tol, f"{name} at full size, output {i}", slack=_long_sum_slack(ops, vals, j))


def test_motivating_pattern_at_full_size_on_batch_slices():
    """Section 3.1's pattern with 16384 batch elements (552 MB of intermediates unfused, 1.2 GB of outputs):
    the stitched kernel runs all of it; the oracle evaluates three slices of 48 batch elements (first, middle,
    last: also the last workgroups of the grid) from the same inputs."""
    cfg = BY_NAME["multi_interest_pattern"]
    announce(f"full size multi_interest_pattern {cfg.full}")
    ops, ins = cfg.build("full")
    got, schedule = _run_stitched(ops, ins)
    assert schedule != "per_op"
    batch = cfg.full["batch"]
    small_kw = dict(cfg.full, batch=48)
    small_ops = cfg.graph_fn(**small_kw)
    tol = TOLERANCE[group_dtype(ops)]
    for lo in (0, batch // 2 - 24, batch - 48):
        part = [a[lo:lo + 48] for a in ins]
        assert all(p.shape[0] == 48 for p in part)
        want = interp.run(small_ops, part)
        assert len(want) == len(got)
        for i, (a, b) in enumerate(zip(got, want)):
            assert_close(a[lo:lo + 48], b, tol, f"motivating pattern, batch elements {lo}..{lo + 47}, output {i}")
    # nothing outside the slices is left unwritten or non-finite
    for a in got:
        assert np.isfinite(a).all()
