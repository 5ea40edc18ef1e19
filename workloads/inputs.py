"""Seeded synthetic inputs for the five benchmark groups.

Every tensor is drawn from numpy's PCG64 with seed `BASE_SEED + config index`,
in fp64, in parameter order, and then rounded once to its storage dtype.  What is
returned is the rounded value held in a float64 array (so the oracle reads it
exactly) together with the storage dtype name (so the GPU side can allocate the
tensor in that dtype without a second rounding).

Distributions follow the benchmark configs; the second argument of N(.,.) is
read as a standard deviation.  Nothing here evaluates any op of a fusion group;
the only statistics computed are the saved per-row mean and reciprocal standard
deviation that a LayerNorm forward pass would hand to its backward pass, taken
with numpy's own `mean` / `var`.
"""
from __future__ import annotations

import numpy as np
import torch

BASE_SEED = 1911_11576

_TORCH = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def round_to(a, dtype):
    """Round an fp64 array to `dtype` storage (nearest even) and widen back."""
    a = np.ascontiguousarray(a, dtype=np.float64)
    if dtype == "f32":
        return a.astype(np.float32).astype(np.float64)
    if dtype == "f16":
        return a.astype(np.float16).astype(np.float64)
    if dtype == "bf16":
        t = torch.from_numpy(a.astype(np.float32)).to(torch.bfloat16)
        return t.to(torch.float64).numpy()
    raise ValueError(dtype)


def to_torch(a, dtype, device="cpu"):
    """Exact conversion of an already-rounded fp64 array to a storage tensor."""
    return torch.from_numpy(np.ascontiguousarray(a)).to(_TORCH[dtype]).to(device)


def _rng(config):
    return np.random.Generator(np.random.PCG64(BASE_SEED + config))


def layernorm_fwd(rows=256, cols=768, dtype="f32", seed_offset=1):
    r = _rng(seed_offset)
    x = r.normal(0.0, 1.0, (rows, cols))
    gamma = r.uniform(0.5, 1.5, (cols,))
    beta = r.normal(0.0, 0.1, (cols,))
    return [round_to(t, dtype) for t in (x, gamma, beta)]


def scaled_masked_softmax(shape=(131072, 128), mask="full", dtype="f32",
                          p_pad=0.1, mask_value=-1e4, seed_offset=2):
    r = _rng(seed_offset)
    s = round_to(r.normal(0.0, 2.0, shape), dtype)
    if mask == "none":
        return [s]
    mshape = shape if mask == "full" else (shape[0], 1, 1, shape[3])
    m = np.where(r.random(mshape) < p_pad, mask_value, 0.0)
    return [s, round_to(m, dtype)]


def causal_attention(batch=512, seq=64, dim=64, dtype="f16", seed_offset=3):
    r = _rng(seed_offset)
    return [round_to(r.normal(0.0, 1.0, (batch, seq, dim)), dtype) for _ in range(3)]


def attention_block(batch, sq, sk, dim, dtype="f16", mask=None, gate=False, residual=False, seed_offset=15, **_):
    """Inputs of graphs.attention_block in parameter order: q, k, v ~ N(0,1); an additive mask of 0 / -1e4
    (padding with probability 0.1) for "key" and "full", a bias ~ N(0,1) for "shared"; gate ~ U(0,1),
    residual ~ N(0,1)."""
    r = _rng(seed_offset)
    out = [round_to(r.normal(0.0, 1.0, (batch, n, dim)), dtype) for n in (sq, sk, sk)]
    if mask == "key":
        out.append(round_to(np.where(r.random((batch, 1, sk)) < 0.1, -1e4, 0.0), "f32"))
    elif mask == "full":
        out.append(round_to(np.where(r.random((batch, sq, sk)) < 0.1, -1e4, 0.0), "f32"))
    elif mask == "shared":
        out.append(round_to(r.normal(0.0, 1.0, (sq, sk)), "f32"))
    if gate:
        out.append(round_to(r.random((batch, sq, dim)), dtype))
    if residual:
        out.append(round_to(r.normal(0.0, 1.0, (batch, sq, dim)), dtype))
    return out


def sigmoid_attention(batch, sq, sk, kc, dim, dtype="bf16", seed_offset=16):
    """q, k ~ N(0,1); v ~ N(0, 0.25): the weights are not normalised and are rounded to 16 bits before the second
    dot, so v is drawn small enough for that rounding to stay well inside the 2e-2 bar on outputs near zero."""
    r = _rng(seed_offset)
    return [round_to(r.normal(0.0, 1.0, (batch, sq, kc)), dtype), round_to(r.normal(0.0, 1.0, (batch, sk, kc)), dtype),
            round_to(r.normal(0.0, 0.25, (batch, sk, dim)), dtype)]


def attention_residual_layernorm(batch, sq, sk, dim, dtype="f16", seed_offset=17):
    r = _rng(seed_offset)
    return [round_to(r.normal(0.0, 1.0, (batch, sq, dim)), dtype), round_to(r.normal(0.0, 1.0, (batch, dim, sk)), dtype),
            round_to(r.normal(0.0, 1.0, (batch, sk, dim)), dtype), round_to(r.normal(0.0, 1.0, (batch, sq, dim)), dtype),
            round_to(1.0 + r.normal(0.0, 0.02, (dim,)), "f32"), round_to(r.normal(0.0, 0.02, (dim,)), "f32")]


def bias_gelu_residual_layernorm(rows=16384, cols=1024, dtype="bf16", seed_offset=4):
    r = _rng(seed_offset)
    x = r.normal(0.0, 1.0, (rows, cols))
    bias = r.normal(0.0, 0.02, (cols,))
    res = r.normal(0.0, 1.0, (rows, cols))
    gamma = 1.0 + r.normal(0.0, 0.02, (cols,))
    beta = r.normal(0.0, 0.02, (cols,))
    return [round_to(t, dtype) for t in (x, bias, res, gamma, beta)]


def layernorm_bwd(rows=32768, cols=1024, dtype="f32", eps=1e-5, seed_offset=5):
    r = _rng(seed_offset)
    dy = round_to(r.normal(0.0, 1.0, (rows, cols)), dtype)
    x = round_to(r.normal(0.0, 1.0, (rows, cols)), dtype)
    gamma = round_to(1.0 + r.normal(0.0, 0.02, (cols,)), dtype)
    mean = round_to(np.mean(x, axis=1), dtype)
    rstd = round_to(1.0 / np.sqrt(np.var(x, axis=1) + eps), dtype)
    return [dy, x, gamma, mean, rstd]


def bias_gelu_residual(rows, cols, dtype="bf16", seed_offset=11):
    r = _rng(seed_offset)
    x = r.normal(0.0, 1.0, (rows, cols))
    bias = r.normal(0.0, 0.02, (cols,))
    res = r.normal(0.0, 1.0, (rows, cols))
    return [round_to(t, dtype) for t in (x, bias, res)]


def adam_update(shape, dtype="f32", seed_offset=12):
    r = _rng(seed_offset)
    p = r.normal(0.0, 1.0, shape)
    grad = r.normal(0.0, 0.1, shape)
    m = r.normal(0.0, 0.05, shape)
    v = r.uniform(1e-4, 1e-2, shape)
    return [round_to(t, dtype) for t in (p, grad, m, v)]


def scale_shift_rows_cols(shape, dtype="f32", seed_offset=13):
    r = _rng(seed_offset)
    x = r.normal(0.0, 1.5, shape)
    rowv = r.normal(0.0, 1.0, shape[:-1])
    colv = r.uniform(0.5, 1.5, (shape[-1],))
    return [round_to(t, dtype) for t in (x, rowv, colv)]


def normal_tensors(shapes, dtype="f32", seed_offset=20, scale=1.0):
    """One N(0, scale) tensor per shape, for the groups outside the five configs."""
    r = _rng(seed_offset)
    return [round_to(r.normal(0.0, scale, s), dtype) for s in shapes]


def multi_interest_pattern(batch, m=94, n=94, k=1, p_pad=0.1, seed_offset=8):
    r = _rng(seed_offset)
    x = r.normal(0.0, 1.0, (batch, m, k))
    y = r.normal(0.0, 1.0, (batch, k, n))
    mask = np.where(r.random((batch, 1, n)) < p_pad, -1e4, 0.0)
    v = r.normal(0.0, 1.0, (batch, n, 1))
    gate = r.uniform(0.0, 1.0, (batch, m, 1))
    return [round_to(t, "f32") for t in (x, y, mask, v, gate)]


def encoder_tail_bwd(rows, cols):
    """dy, x ~ N(0,1); bias ~ N(0,0.02); r ~ N(0,1) (stands for the saved LayerNorm input);
    gamma = 1 + N(0,0.02); mean and rstd of r as a forward pass would have saved them."""
    rng = _rng(40)
    dy = rng.standard_normal((rows, cols))
    x = rng.standard_normal((rows, cols))
    bias = 0.02 * rng.standard_normal(cols)
    r = round_to(rng.standard_normal((rows, cols)), "f32")
    gamma = 1.0 + 0.02 * rng.standard_normal(cols)
    r64 = r
    mean = r64.mean(axis=-1) if rows else np.zeros(0)
    rstd = 1.0 / np.sqrt(r64.var(axis=-1) + 1e-5) if rows else np.zeros(0)
    return [round_to(t, "f32") for t in (dy, x, bias)] + [r] + [round_to(t, "f32") for t in (gamma, mean, rstd)]


def multi_tensor_momentum(shapes, dtypes=None, seed_offset=41):
    """Per tensor: p ~ N(0,1), g ~ N(0,0.1), m ~ N(0,0.05), in parameter order."""
    r = _rng(seed_offset)
    dtypes = dtypes or ["f32"] * len(shapes)
    out = []
    for shape, dt in zip(shapes, dtypes):
        out += [round_to(r.normal(0.0, 1.0, shape), dt), round_to(r.normal(0.0, 0.1, shape), dt), round_to(r.normal(0.0, 0.05, shape), dt)]
    return out
