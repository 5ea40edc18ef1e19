"""Tensors of more than 2^31 elements: every index the kernels form must be 64-bit.  Inputs are drawn
on the device (seeded), the oracle checks sampled rows - the first, the last, rows around element
2^31 - plus properties that hold for every row."""
import sys

import numpy as np
import pytest
import torch

from oracle import interp
from paper_1911_11576_amd import Plan
from workloads import graphs
from workloads.graphs import Graph

from gpu_util import assert_close

pytestmark = pytest.mark.gpu
_TORCH = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def announce(msg):
    sys.__stderr__.write(f"[gpu-case] {msg}\n")
    sys.__stderr__.flush()


@pytest.fixture(autouse=True)
def _need_gpu(device):
    yield
    torch.cuda.empty_cache()


def _rows_to_check(rows, cols):
    at = (1 << 31) // cols          # the row that holds element 2^31
    idx = [0, 1, at - 1, at, at + 1, rows // 3, rows - 2, rows - 1]
    return np.unique(np.clip(np.array(idx, dtype=np.int64), 0, rows - 1))


def _device_normal(shape, dtype, seed, scale=1.0):
    g = torch.Generator(device="cuda:0")
    g.manual_seed(seed)
    t = torch.empty(shape, dtype=_TORCH[dtype], device="cuda:0")
    t.normal_(0.0, scale, generator=g)
    return t


def _host(t, idx=None):
    return (t if idx is None else t[torch.as_tensor(idx, device=t.device)]).to(torch.float64).cpu().numpy()


def test_elementwise_group_beyond_2_31_elements():
    rows, cols = (1 << 21) + 3, 1024                       # 2 147 486 720 elements, 4.3 GB per fp16 tensor
    def build(r):
        g = Graph()
        x = g.parameter("x", "f16", (r, cols))
        c = g.parameter("c", "f16", (cols,))
        xf, cf = g.convert(x, "f32"), g.convert(c, "f32")
        g.output(g.convert(g.add(g.multiply(g.tanh(xf), g.constant(0.5)), g.col_broadcast(cf, xf)), "f16"))
        return g.ops
    announce(f"elementwise {rows}x{cols} f16")
    x, c = _device_normal((rows, cols), "f16", 1), _device_normal((cols,), "f16", 2)
    y = torch.full((rows, cols), float("nan"), dtype=torch.float16, device="cuda:0")
    with Plan(build(rows)) as p:
        assert p.info()["schedule"] == "elementwise"
        p.launch([x, c], [y])
        torch.cuda.synchronize()
    idx = _rows_to_check(rows, cols)
    (want,) = interp.run(build(len(idx)), [_host(x, idx), _host(c)])
    assert_close(_host(y, idx), want, 2e-2, "elementwise beyond 2^31")
    assert not bool(torch.isnan(y).any())                  # every element was written


@pytest.mark.parametrize("form", ["generated log-softmax", "hand-written masked softmax"])
def test_row_groups_beyond_2_31_elements(form):
    rows, cols = (1 << 24) + 5, 128                        # 2 147 484 288 elements, 8.6 GB per fp32 tensor
    announce(f"{form} {rows}x{cols} f32")
    x = _device_normal((rows, cols), "f32", 3, scale=2.0)
    y = torch.full((rows, cols), float("nan"), dtype=torch.float32, device="cuda:0")
    idx = _rows_to_check(rows, cols)
    if form.startswith("generated"):
        build, ins = (lambda r: graphs.log_softmax((r, cols))), [x]
    else:
        m = _device_normal((rows, cols), "f32", 4)
        m = torch.where(m > 1.28, torch.full_like(m, -1e4), torch.zeros_like(m))      # about one in ten masked
        build, ins = (lambda r: graphs.scaled_masked_softmax((r, cols), 0.125, "full")), [x, m]
    with Plan(build(rows)) as p:
        assert ("generated kernel" in p.describe()) == form.startswith("generated")
        p.launch(ins, [y])
        torch.cuda.synchronize()
    (want,) = interp.run(build(len(idx)), [_host(t, idx) for t in ins])
    assert_close(_host(y, idx), want, 1e-5, f"{form} beyond 2^31")
    # every row: probabilities sum to one
    prob = y.exp() if form.startswith("generated") else y
    s = prob.sum(dim=1, dtype=torch.float64)
    assert float((s - 1).abs().max()) < 1e-5 and not bool(torch.isnan(s).any())
