"""Pins for the oracle's individual ops: brute-force scalar loops on tiny,
hand-checkable inputs, written independently of numpy's array routines."""
import math

import numpy as np
import pytest

from oracle import interp
from workloads.graphs import Graph


def _run1(build, *arrays):
    g = Graph()
    build(g)
    return interp.run(g.ops, [np.asarray(a, dtype=np.float64) for a in arrays])


def _ints(shape, lo=-4, hi=5, seed=0):
    return np.random.default_rng(seed).integers(lo, hi, shape).astype(np.float64)


@pytest.mark.parametrize("kind,fn", [
    ("add", lambda a, b: a + b), ("subtract", lambda a, b: a - b),
    ("multiply", lambda a, b: a * b), ("divide", lambda a, b: a / b),
    ("maximum", lambda a, b: a if a > b else b),
])
def test_binary_brute(kind, fn):
    a = _ints((3, 5), seed=1)
    b = _ints((3, 5), 1, 6, seed=2)

    def build(g):
        pa = g.parameter("a", "f32", a.shape)
        pb = g.parameter("b", "f32", b.shape)
        g.output(getattr(g, kind)(pa, pb))
    (out,) = _run1(build, a, b)
    for i in range(3):
        for j in range(5):
            assert out[i, j] == fn(a[i, j], b[i, j])


def test_subtract_and_divide_operand_order_with_constant():
    a = np.array([[1.0, 2.0, 4.0]])

    def build(g):
        pa = g.parameter("a", "f32", a.shape)
        g.output(g.subtract(g.constant(10.0), pa))
        g.output(g.subtract(pa, g.constant(10.0)))
        g.output(g.divide(g.constant(8.0), pa))
        g.output(g.divide(pa, g.constant(8.0)))
    o = _run1(build, a)
    assert o[0].tolist() == [[9.0, 8.0, 6.0]]
    assert o[1].tolist() == [[-9.0, -8.0, -6.0]]
    assert o[2].tolist() == [[8.0, 4.0, 2.0]]
    assert o[3].tolist() == [[0.125, 0.25, 0.5]]


@pytest.mark.parametrize("kind,fn", [
    ("negate", lambda a: -a), ("exp", math.exp), ("log", math.log), ("tanh", math.tanh),
    ("sqrt", math.sqrt), ("rsqrt", lambda a: 1.0 / math.sqrt(a)),
])
def test_unary_brute(kind, fn):
    a = _ints((2, 4), 1, 6, seed=3) / 2.0

    def build(g):
        g.output(getattr(g, kind)(g.parameter("a", "f32", a.shape)))
    (out,) = _run1(build, a)
    for i in range(2):
        for j in range(4):
            assert out[i, j] == pytest.approx(fn(a[i, j]), rel=1e-15, abs=0)


@pytest.mark.parametrize("axis", [0, 1, 2])
@pytest.mark.parametrize("kind", ["reduce_sum", "reduce_max"])
def test_reduce_brute(kind, axis):
    a = _ints((2, 3, 4), seed=4)

    def build(g):
        g.output(getattr(g, kind)(g.parameter("a", "f32", a.shape), axis))
    (out,) = _run1(build, a)
    rest = [d for d in range(3) if d != axis]
    assert out.shape == tuple(a.shape[d] for d in rest)
    for p in range(a.shape[rest[0]]):
        for q in range(a.shape[rest[1]]):
            vals = []
            for r in range(a.shape[axis]):
                idx = [0, 0, 0]
                idx[rest[0]], idx[rest[1]], idx[axis] = p, q, r
                vals.append(a[tuple(idx)])
            want = sum(vals) if kind == "reduce_sum" else max(vals)
            assert out[p, q] == want


def test_broadcast_row_col_and_unit_dims():
    r = np.array([1.0, 2.0, 3.0])            # per row
    c = np.array([10.0, 20.0, 30.0, 40.0])   # per column
    m = _ints((2, 1, 1, 4), seed=5)

    def build(g):
        pr = g.parameter("r", "f32", (3,))
        pc = g.parameter("c", "f32", (4,))
        pm = g.parameter("m", "f32", (2, 1, 1, 4))
        g.output(g.broadcast(pr, (3, 4), 0))
        g.output(g.broadcast(pc, (3, 4), 1))
        g.output(g.broadcast(pm, (2, 3, 5, 4), 0))
    o = _run1(build, r, c, m)
    for i in range(3):
        for j in range(4):
            assert o[0][i, j] == r[i]
            assert o[1][i, j] == c[j]
    for b in range(2):
        for h in range(3):
            for i in range(5):
                for j in range(4):
                    assert o[2][b, h, i, j] == m[b, 0, 0, j]


@pytest.mark.parametrize("transpose_b", [False, True])
def test_dot_brute(transpose_b):
    B, M, K, N = 2, 4, 3, 5
    a = _ints((B, M, K), seed=6)
    b = _ints((B, N, K) if transpose_b else (B, K, N), seed=7)

    def build(g):
        pa = g.parameter("a", "f16", a.shape)
        pb = g.parameter("b", "f16", b.shape)
        g.output(g.dot(pa, pb, transpose_b=transpose_b))
    (out,) = _run1(build, a, b)
    assert out.shape == (B, M, N)
    for t in range(B):
        for i in range(M):
            for j in range(N):
                acc = 0.0
                for k in range(K):
                    acc += a[t, i, k] * (b[t, j, k] if transpose_b else b[t, k, j])
                assert out[t, i, j] == acc


def test_causal_mask_brute():
    a = _ints((2, 4, 4), 1, 9, seed=8)

    def build(g):
        g.output(g.causal_mask(g.parameter("a", "f32", a.shape), -7.0))
    (out,) = _run1(build, a)
    for t in range(2):
        for i in range(4):
            for j in range(4):
                assert out[t, i, j] == (a[t, i, j] if j <= i else -7.0)


def test_convert_identity_by_default_and_rounds_in_storage_mode():
    a = np.array([[1.0 + 2.0 ** -10, 1.0 + 2.0 ** -9, 3.0 + 2.0 ** -7, 1e-8]])
    g = Graph()
    p = g.parameter("a", "f32", a.shape)
    g.output(g.convert(p, "bf16"))
    g.output(g.convert(p, "f16"))
    exact = interp.run(g.ops, [a])
    assert np.array_equal(exact[0], a) and np.array_equal(exact[1], a)
    st = interp.run(g.ops, [a], storage_rounding=True)
    # bf16 keeps 8 significant bits (spacing 2^-7 at 1, 2^-6 at 3): 1+2^-10 and
    # 1+2^-9 are below the half-way point 1+2^-8 -> 1; 3+2^-7 is exactly half-way
    # between 3 and 3+2^-6 -> ties to the even significand, 3
    assert st[0][0, 0] == 1.0
    assert st[0][0, 1] == 1.0
    assert st[0][0, 2] == 3.0
    # fp16 keeps 11 bits: 1+2^-10 is representable, 1+2^-9 too
    assert st[1][0, 0] == 1.0 + 2.0 ** -10
    assert st[1][0, 1] == 1.0 + 2.0 ** -9


def test_bf16_rounding_matches_torch_bit_for_bit():
    import torch
    a = np.random.default_rng(9).normal(0, 3, 4096)
    ours = interp._round(a, "bf16")
    ref = torch.from_numpy(a.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(ours, ref)


def test_shape_mismatch_is_an_error():
    g = Graph()
    g.output(g.parameter("a", "f32", (2, 3)))
    with pytest.raises(ValueError):
        interp.run(g.ops, [np.zeros((3, 2))])


def test_erf_against_its_integral_its_series_and_another_library():
    """erf(x) = 2/sqrt(pi) * integral_0^x exp(-t^2) dt: Simpson's rule with 20 000 panels, the Maclaurin series
    sum (-1)^n x^(2n+1) / (n! (2n+1)), scipy's routine, oddness and the limits."""
    from scipy import special
    x = np.array([[-3.0, -1.0, -0.5, 0.0], [0.25, 0.5, 1.0, 2.5]])

    def build(g):
        g.output(g.erf(g.parameter("a", "f32", x.shape)))
    (out,) = _run1(build, x)
    for xi, got in zip(x.ravel(), out.ravel()):
        t = np.linspace(0.0, xi, 20001)
        f = np.exp(-t * t)
        h = (xi - 0.0) / 20000
        simpson = h / 3.0 * (f[0] + f[-1] + 4.0 * f[1:-1:2].sum() + 2.0 * f[2:-1:2].sum()) * 2.0 / math.sqrt(math.pi)
        series = 2.0 / math.sqrt(math.pi) * sum((-1) ** n * xi ** (2 * n + 1) / (math.factorial(n) * (2 * n + 1)) for n in range(80))
        assert got == pytest.approx(simpson, abs=1e-12)
        assert got == pytest.approx(series, abs=1e-10)
        assert got == pytest.approx(float(special.erf(xi)), abs=1e-15)
    assert out[0, 3] == 0.0 and np.allclose(out[0, :3], -np.array([out_v for out_v in (1 - 2.209049699858544e-05, 0.8427007929497149, 0.5204998778130465)]), atol=1e-15)

    def far(g):
        g.output(g.erf(g.parameter("a", "f32", (1, 2))))
    (lim,) = _run1(far, np.array([[30.0, -30.0]]))
    assert lim.tolist() == [[1.0, -1.0]]


def test_logistic_identities():
    """1/(1+exp(-x)): value 1/2 at 0, s(x) + s(-x) = 1, s(x) = (1 + tanh(x/2))/2, limits 0 and 1."""
    x = np.array([[-40.0, -2.0, -0.5, 0.0], [0.5, 1.0, 3.0, 40.0]])

    def build(g):
        g.output(g.logistic(g.parameter("a", "f32", x.shape)))
    (s,) = _run1(build, x)
    (sm,) = _run1(build, -x)
    assert s[0, 3] == 0.5
    assert np.allclose(s + sm, 1.0, atol=1e-15)
    assert np.allclose(s, 0.5 * (1.0 + np.tanh(x / 2.0)), atol=1e-15)
    assert s[0, 0] == pytest.approx(math.exp(-40.0), rel=1e-12) and s[1, 3] == pytest.approx(1.0, abs=1e-15)
    assert s[1, 1] == pytest.approx(0.7310585786300049, abs=1e-15)        # 1/(1+1/e)
