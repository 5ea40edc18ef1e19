"""Pins for the oracle on whole fusion groups: invariants, closed forms, special
cases, brute force, finite differences and the PyTorch CPU library routines.
None of these re-types the interpreter's formulas; each would fail for a dropped
term, a wrong sign, a wrong axis or a transposed operand in the group."""
import math

import numpy as np
import pytest
import torch

from oracle import interp
from workloads import CONFIGS, BY_NAME, graphs, inputs


def _t(a):
    return torch.from_numpy(np.ascontiguousarray(a))


# ------------------------------------------------------------------ LayerNorm fwd

def _ln_inputs(rows=6, cols=40, seed=0):
    r = np.random.default_rng(seed)
    return r.normal(0.3, 2.0, (rows, cols)), r.uniform(0.5, 1.5, cols), r.normal(0, 0.1, cols)


def test_layernorm_rows_have_mean0_and_closed_form_variance():
    x, gamma, beta = _ln_inputs()
    eps = 1e-5
    ops = graphs.layernorm_fwd(*x.shape, eps=eps)
    (xhat,) = interp.run(ops, [x, np.ones_like(gamma), np.zeros_like(beta)])
    assert np.abs(xhat.mean(axis=1)).max() < 1e-14
    v = x.var(axis=1)                       # biased
    assert np.allclose(xhat.var(axis=1), v / (v + eps), rtol=1e-12, atol=0)


def test_layernorm_constant_row_gives_beta_and_shift_invariance():
    x, gamma, beta = _ln_inputs()
    ops = graphs.layernorm_fwd(*x.shape)
    xc = np.full_like(x, 3.25)
    (y,) = interp.run(ops, [xc, gamma, beta])
    assert np.array_equal(y, np.broadcast_to(beta, x.shape))
    (y0,) = interp.run(ops, [x, gamma, beta])
    (y1,) = interp.run(ops, [x + np.arange(x.shape[0])[:, None], gamma, beta])
    assert np.allclose(y0, y1, rtol=0, atol=1e-12)


def test_layernorm_matches_torch_cpu():
    x, gamma, beta = _ln_inputs(9, 768, seed=3)
    (y,) = interp.run(graphs.layernorm_fwd(*x.shape), [x, gamma, beta])
    ref = torch.nn.functional.layer_norm(_t(x), (x.shape[1],), _t(gamma), _t(beta), 1e-5).numpy()
    assert np.allclose(y, ref, rtol=1e-12, atol=1e-12)


def test_layernorm_eps_is_inside_the_root():
    # one row [-1, 1]: mean 0, biased variance 1 -> y = x / sqrt(1 + eps)
    x = np.array([[-1.0, 1.0]])
    (y,) = interp.run(graphs.layernorm_fwd(1, 2, eps=3.0), [x, np.ones(2), np.zeros(2)])
    assert np.allclose(y, x / 2.0, rtol=1e-15)


# ------------------------------------------------------------------ softmax

def test_softmax_rows_sum_to_one_shift_invariant_and_masked_zero():
    ops = graphs.scaled_masked_softmax((50, 128), 0.125, "full")
    s, m = inputs.scaled_masked_softmax((50, 128), "full")
    m[:, 0] = 0.0                                      # every row keeps one open entry
    (p,) = interp.run(ops, [s, m])
    assert np.abs(p.sum(axis=1) - 1).max() < 1e-14
    assert p.min() >= 0 and p.max() <= 1
    assert np.all(p[m != 0] == 0.0)                    # exp(-1e4) underflows even in fp64
    (p2,) = interp.run(ops, [s + 8.0 * np.arange(50)[:, None], m])
    assert np.allclose(p, p2, rtol=1e-10, atol=1e-300)


def test_softmax_constant_row_and_fully_masked_row():
    ops = graphs.scaled_masked_softmax((2, 128), 0.125, "full")
    s = np.full((2, 128), 1.75)
    m = np.zeros((2, 128))
    m[1, :] = -1e4                                     # a fully padded row is still a softmax
    (p,) = interp.run(ops, [s, m])
    assert np.allclose(p, 1.0 / 128, rtol=1e-15)


def test_softmax_scale_then_mask_order_and_two_entry_closed_form():
    # row [a, b] with scale c and mask [0, mu]: p0 = 1 / (1 + exp(c*b + mu - c*a))
    a, b, c, mu = 0.7, -1.1, 0.125, -2.0
    ops = graphs.scaled_masked_softmax((1, 2), c, "full")
    (p,) = interp.run(ops, [np.array([[a, b]]), np.array([[0.0, mu]])])
    assert p[0, 0] == pytest.approx(1.0 / (1.0 + math.exp(c * b + mu - c * a)), rel=1e-14)


def test_softmax_matches_torch_cpu_full_and_key_padding():
    s, m = inputs.scaled_masked_softmax((70, 128), "full")
    (p,) = interp.run(graphs.scaled_masked_softmax((70, 128), 0.125, "full"), [s, m])
    ref = torch.softmax(_t(s) * 0.125 + _t(m), dim=-1).numpy()
    assert np.allclose(p, ref, rtol=1e-12, atol=1e-300)
    shape = (3, 4, 16, 16)
    s, m = inputs.scaled_masked_softmax(shape, "key_padding")
    assert m.shape == (3, 1, 1, 16)
    (p,) = interp.run(graphs.scaled_masked_softmax(shape, 0.125, "key_padding"), [s, m])
    ref = torch.softmax(_t(s) * 0.125 + _t(m), dim=-1).numpy()
    assert np.allclose(p, ref, rtol=1e-12, atol=1e-300)


# ------------------------------------------------------------------ attention

def test_attention_v_ones_gives_ones_and_row0_is_v0():
    B, S, d = 3, 16, 8
    q, k, v = inputs.causal_attention(B, S, d)
    ops = graphs.causal_attention(B, S, d)
    (o,) = interp.run(ops, [q, k, np.ones_like(v)])
    assert np.allclose(o, 1.0, rtol=1e-14)
    (o,) = interp.run(ops, [q, k, v])
    assert np.allclose(o[:, 0, :], v[:, 0, :], rtol=1e-15)


def test_attention_q_zero_gives_causal_prefix_means():
    B, S, d = 2, 12, 4
    q, k, v = inputs.causal_attention(B, S, d)
    (o,) = interp.run(graphs.causal_attention(B, S, d), [np.zeros_like(q), k, v])
    for b in range(B):
        for i in range(S):
            for c in range(d):
                want = sum(v[b, j, c] for j in range(i + 1)) / (i + 1)
                assert o[b, i, c] == pytest.approx(want, rel=1e-13, abs=1e-15)


def test_attention_brute_force_triple_loop():
    B, S, d = 2, 4, 4
    q, k, v = inputs.causal_attention(B, S, d)
    (o,) = interp.run(graphs.causal_attention(B, S, d), [q, k, v])
    for b in range(B):
        for i in range(S):
            w = []
            for j in range(i + 1):
                w.append(math.exp(sum(q[b, i, t] * k[b, j, t] for t in range(d)) / math.sqrt(d)))
            for c in range(d):
                want = sum(w[j] * v[b, j, c] for j in range(i + 1)) / sum(w)
                assert o[b, i, c] == pytest.approx(want, rel=1e-12, abs=1e-14)


def test_attention_matches_torch_sdpa():
    B, S, d = 4, 64, 64
    q, k, v = inputs.causal_attention(B, S, d)
    (o,) = interp.run(graphs.causal_attention(B, S, d), [q, k, v])
    ref = torch.nn.functional.scaled_dot_product_attention(
        _t(q), _t(k), _t(v), is_causal=True, scale=0.125).numpy()
    assert np.allclose(o, ref, rtol=1e-10, atol=1e-12)


# ------------------------------------------------------------------ bias + GELU + residual + LN

def _gelu_only_ops(cols):
    """The group with LayerNorm neutralised is not expressible; instead evaluate
    the group with keep=True and pick the gelu(x+bias)+residual node."""
    ops = graphs.bias_gelu_residual_layernorm(1, cols, dtype="f32")
    # the op feeding the first reduce_sum is r = gelu(h) + residual
    first_reduce = next(i for i, op in enumerate(ops) if op.kind == "reduce_sum")
    return ops, ops[first_reduce].operands[0]


def test_gelu_identities_and_limits():
    cols = 9
    ops, r_idx = _gelu_only_ops(cols)
    x = np.array([[0.0, 0.5, -0.5, 1.7, -1.7, 3.0, -3.0, 30.0, -30.0]])
    zeros = np.zeros(cols)
    vals = interp.run(ops, [x, zeros, np.zeros_like(x), np.ones(cols), zeros], keep=True)
    g = vals[r_idx][0]
    assert g[0] == 0.0
    for a, b in ((1, 2), (3, 4), (5, 6), (7, 8)):       # gelu(x) - gelu(-x) = x
        assert g[a] - g[b] == pytest.approx(x[0, a], rel=1e-14)
    assert g[7] == pytest.approx(30.0, rel=1e-15) and abs(g[8]) < 1e-300
    ref = torch.nn.functional.gelu(_t(x), approximate="tanh").numpy()[0]
    assert np.allclose(g, ref, rtol=1e-13, atol=1e-300)


def test_bias_and_residual_enter_where_they_should():
    cols = 8
    ops, r_idx = _gelu_only_ops(cols)
    rng = np.random.default_rng(5)
    x, bias, res = rng.normal(0, 1, (1, cols)), rng.normal(0, 1, cols), rng.normal(0, 1, (1, cols))
    vals = interp.run(ops, [x, bias, res, np.ones(cols), np.zeros(cols)], keep=True)
    ref = torch.nn.functional.gelu(_t(x + bias), approximate="tanh").numpy() + res
    assert np.allclose(vals[r_idx], ref, rtol=1e-13, atol=1e-15)


def test_cfg4_matches_torch_cpu_composition():
    rows, cols = 7, 1024
    ins = inputs.bias_gelu_residual_layernorm(rows, cols)
    (y,) = interp.run(graphs.bias_gelu_residual_layernorm(rows, cols), ins)
    x, bias, res, gamma, beta = map(_t, ins)
    r = torch.nn.functional.gelu(x + bias, approximate="tanh") + res
    ref = torch.nn.functional.layer_norm(r, (cols,), gamma, beta, 1e-5).numpy()
    assert np.allclose(y, ref, rtol=1e-11, atol=1e-12)


# ------------------------------------------------------------------ LayerNorm bwd

def _ln_loss(x, gamma, beta, dy, eps=1e-5):
    (y,) = interp.run(graphs.layernorm_fwd(*x.shape, eps=eps), [x, gamma, beta])
    return float(np.sum(dy * y))


def test_layernorm_bwd_against_central_finite_differences():
    rows, cols, eps = 3, 8, 1e-5
    rng = np.random.default_rng(11)
    x, dy = rng.normal(0, 1, (rows, cols)), rng.normal(0, 1, (rows, cols))
    gamma, beta = 1.0 + rng.normal(0, 0.2, cols), rng.normal(0, 0.2, cols)
    mean = x.mean(axis=1)
    rstd = 1.0 / np.sqrt(x.var(axis=1) + eps)
    dx, dgamma, dbeta = interp.run(graphs.layernorm_bwd(rows, cols), [dy, x, gamma, mean, rstd])
    h = 1e-6
    for i in range(rows):
        for j in range(cols):
            xp, xm = x.copy(), x.copy()
            xp[i, j] += h
            xm[i, j] -= h
            fd = (_ln_loss(xp, gamma, beta, dy) - _ln_loss(xm, gamma, beta, dy)) / (2 * h)
            assert dx[i, j] == pytest.approx(fd, rel=1e-6, abs=1e-8)
    for j in range(cols):
        gp, gm = gamma.copy(), gamma.copy()
        gp[j] += h
        gm[j] -= h
        fd = (_ln_loss(x, gp, beta, dy) - _ln_loss(x, gm, beta, dy)) / (2 * h)
        assert dgamma[j] == pytest.approx(fd, rel=1e-7, abs=1e-9)
        assert dbeta[j] == pytest.approx(sum(dy[i, j] for i in range(rows)), rel=1e-14)


def test_layernorm_bwd_row_invariants_and_torch_autograd():
    rows, cols = 33, 1024
    dy, x, gamma, mean, rstd = inputs.layernorm_bwd(rows, cols)
    dx, dgamma, dbeta = interp.run(graphs.layernorm_bwd(rows, cols), [dy, x, gamma, mean, rstd])
    xhat = (x - mean[:, None]) * rstd[:, None]
    assert np.abs(dx.sum(axis=1)).max() < 1e-4          # saved stats are fp32-rounded
    assert np.abs((dx * xhat).sum(axis=1)).max() < 1e-3
    # exact statistics -> invariants hold to fp64 rounding
    mean64 = x.mean(axis=1)
    rstd64 = 1.0 / np.sqrt(x.var(axis=1) + 1e-5)
    dx64, _, _ = interp.run(graphs.layernorm_bwd(rows, cols), [dy, x, gamma, mean64, rstd64])
    xhat64 = (x - mean64[:, None]) * rstd64[:, None]
    assert np.abs(dx64.sum(axis=1)).max() < 1e-11
    # sum_j dx*xhat = rstd * s2 * (1 - mean(xhat^2)) = rstd * s2 * eps * rstd^2: tiny, not 0
    s2 = (dy * gamma * xhat64).sum(axis=1)
    assert np.allclose((dx64 * xhat64).sum(axis=1), s2 * 1e-5 * rstd64 ** 3, rtol=1e-6, atol=1e-12)
    xt = _t(x).requires_grad_(True)
    gt = _t(gamma).requires_grad_(True)
    bt = torch.zeros(cols, dtype=torch.float64, requires_grad=True)
    y = torch.nn.functional.layer_norm(xt, (cols,), gt, bt, 1e-5)
    y.backward(_t(dy))
    assert np.allclose(dx64, xt.grad.numpy(), rtol=1e-9, atol=1e-12)
    assert np.allclose(dgamma, gt.grad.numpy(), rtol=0, atol=1e-4)   # fp32-rounded stats
    assert np.allclose(dbeta, bt.grad.numpy(), rtol=1e-13, atol=1e-12)


# ------------------------------------------------------------------ whole configs

@pytest.mark.parametrize("cfg", CONFIGS, ids=lambda c: c.name)
def test_storage_rounding_mode_stays_within_the_group_tolerance(cfg):
    """Rounding every intermediate to its declared dtype (what a one-kernel-per-op
    framework does) moves the answer by far less than the comparison bar."""
    from workloads import TOLERANCE
    ops, ins = cfg.build("small")
    exact = interp.run(ops, ins)
    stored = interp.run(ops, ins, storage_rounding=True)
    tol = TOLERANCE[cfg.dtype]
    for a, b in zip(exact, stored):
        if cfg.name == "layernorm_bwd" and a.ndim == 1:
            continue   # fp32 column sums over many rows: see the accumulation note in the design
        assert np.all(np.abs(a - b) <= tol + tol * np.abs(a))


def test_config_table_matches_the_benchmark_sizes():
    from workloads import algorithmic_bytes
    want = {"layernorm_fwd": 1_579_008, "scaled_masked_softmax": 201_326_592,
            "causal_attention": 16_777_216, "bias_gelu_residual_layernorm": 100_669_440,
            "layernorm_bwd": 402_927_616}
    for name, nbytes in want.items():
        cfg = BY_NAME[name]
        assert algorithmic_bytes(cfg.graph_fn(**cfg.full)) == nbytes
    ops = graphs.scaled_masked_softmax((64, 16, 128, 128), 0.125, "key_padding")
    assert algorithmic_bytes(ops) == 134_250_496
