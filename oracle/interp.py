"""CPU oracle: a per-op interpreter of a fusion group.  TEST INFRASTRUCTURE ONLY.

A fusion pattern is a sub-DAG of XLA-semantics tensor ops whose outputs form a
tuple (paper, Section 3.1 and Section 4.1).  Fusing changes only where the
intermediates live (registers / shared memory instead of off-chip memory,
Section 5.1); the values are those of running the ops one after another, which
is also what the execution-based score compares against (Section 4.3: the sum of
the single-op kernels K(Op_j) versus the fused K(P) of the *same* ops).  So the
oracle is that plain definition: walk the list in order; every op reads its
operands as whole tensors and materialises a whole result tensor.  No fusion, no
tiling, no reordering.

Arithmetic is float64 throughout.  Inputs arrive as float64 arrays that hold
values already rounded to their storage dtype.  In the default mode `convert`
is the identity, so the result is the un-rounded mathematical value of the group
on those inputs.  With `storage_rounding=True` every op result is rounded to the
op's declared dtype, which mimics a framework that runs one kernel per op.

This file shares no code with the HIP library and imports nothing from it.
Only tests, the smoke check and the bench's cpu_baseline leg may use it.

Parity pins (tests/test_oracle_*.py): brute-force scalar loops per op on tiny
inputs; LayerNorm rows have mean 0 and variance v/(v+eps); softmax rows sum to 1
and are shift invariant; attention with V=1 gives 1, with Q=0 gives causal prefix
means; gelu(x)-gelu(-x)=x; LayerNorm-backward against central finite differences;
every group against the matching PyTorch CPU library routine.
"""
from __future__ import annotations

import math

import numpy as np


def _round(a, dtype):
    if dtype == "f32":
        return a.astype(np.float32).astype(np.float64)
    if dtype == "f16":
        return a.astype(np.float16).astype(np.float64)
    if dtype == "bf16":
        # round-to-nearest-even on the upper 16 bits of the float32 pattern
        f = np.ascontiguousarray(a.astype(np.float32))
        u = f.view(np.uint32).astype(np.uint64)
        u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
        out = u.astype(np.uint32).view(np.float32).astype(np.float64)
        return np.where(np.isfinite(f), out, f.astype(np.float64))
    raise ValueError(dtype)


def _broadcast(a, shape, axis):
    # operand dim d sits at result dim axis+d; all other result dims are new
    full = [1] * len(shape)
    for d, e in enumerate(a.shape):
        full[axis + d] = e
    return np.broadcast_to(a.reshape(full), shape).copy()


def _causal_mask(a, fill):
    rows, cols = a.shape[-2], a.shape[-1]
    i = np.arange(rows)[:, None]
    j = np.arange(cols)[None, :]
    return np.where(j <= i, a, fill)


def _dot(a, b, transpose_b):
    if transpose_b:
        b = np.swapaxes(b, 1, 2)
    return np.matmul(a, b)


_BINARY = {
    "add": np.add, "subtract": np.subtract, "multiply": np.multiply,
    "divide": np.divide, "maximum": np.maximum,
}
_UNARY = {
    "negate": np.negative, "exp": np.exp, "log": np.log, "tanh": np.tanh,
    "sqrt": np.sqrt, "rsqrt": lambda a: 1.0 / np.sqrt(a),
    "erf": lambda a: _erf(a), "logistic": lambda a: 1.0 / (1.0 + np.exp(-a)),
}


def _erf(a):
    """erf(x) = (2/sqrt(pi)) * integral from 0 to x of exp(-t^2) dt, element by element from the C library."""
    return np.vectorize(math.erf, otypes=[np.float64])(np.asarray(a, dtype=np.float64))


def run(ops, inputs, storage_rounding=False, keep=False):
    """Evaluate the op list.  `inputs`: one float64 array per `parameter`, in order.
    Returns the list of output arrays (float64), or every op's value if `keep`."""
    vals = []
    outs = []
    it = iter(inputs)
    for op in ops:
        arg = [vals[i] for i in op.operands]
        k = op.kind
        if k == "parameter":
            v = np.asarray(next(it), dtype=np.float64)
            if v.shape != op.shape:
                raise ValueError(f"parameter {op.name}: shape {v.shape} != {op.shape}")
        elif k == "constant":
            v = np.float64(op.attr)
        elif k in _BINARY:
            v = _BINARY[k](arg[0], arg[1])
        elif k in _UNARY:
            v = _UNARY[k](arg[0])
        elif k == "convert":
            v = arg[0]
        elif k == "broadcast":
            v = _broadcast(arg[0], op.shape, op.axis)
        elif k == "reduce_sum":
            v = np.sum(arg[0], axis=op.axis)
        elif k == "reduce_max":
            v = np.max(arg[0], axis=op.axis)
        elif k == "dot":
            v = _dot(arg[0], arg[1], op.axis == 1)
        elif k == "causal_mask":
            v = _causal_mask(arg[0], op.attr)
        elif k == "output":
            v = arg[0]
            outs.append(np.array(v, dtype=np.float64))
        else:
            raise ValueError(f"unknown op kind {k}")
        if storage_rounding and k not in ("parameter", "output"):
            v = _round(np.asarray(v, dtype=np.float64), op.dtype)
        if np.shape(v) != op.shape:
            raise ValueError(f"op {len(vals)} ({k}): shape {np.shape(v)} != {op.shape}")
        vals.append(v)
    return vals if keep else outs
