"""Fusion-group op lists (the paper's "fusion pattern": a sub-DAG of XLA-semantics
ops with one or more outputs, Section 3.1 and Section 4.1).

This module only *describes* computations: it builds topologically ordered lists
of `Op` records.  It evaluates nothing and holds none of the method's
arithmetic.  Both the CPU oracle and the HIP library are handed the same lists
by the tests and the bench; neither imports this module.

Op semantics (shared vocabulary, defined here once):

  parameter            group input, dense row-major
  constant             rank-0 scalar with value `attr`; may be used directly as an
                       operand of a binary op (implicit scalar broadcast)
  add subtract multiply divide maximum          elementwise binary, equal shapes
  negate exp log tanh rsqrt sqrt                elementwise unary
  convert              change of storage dtype (value-preserving up to rounding)
  broadcast            operand dims map to result dims [axis, axis+rank(operand));
                       operand dims of extent 1 are expanded
  reduce_sum reduce_max   reduce over `axis`; that dim is removed from the shape
  dot                  batched matrix product a[B,M,K] x b[B,K,N];  axis=1 means b is
                       stored [B,N,K] (contraction over the last dim of both)
  causal_mask          x[..., i, j] kept where j <= i, else replaced by `attr`
  output               marks operand 0 as a group output (one element of the
                       paper's terminal `tuple`)
"""
from __future__ import annotations

from collections import namedtuple

Op = namedtuple("Op", "kind dtype shape operands axis attr name")

KINDS = (
    "parameter", "constant", "add", "subtract", "multiply", "divide", "maximum",
    "negate", "exp", "log", "tanh", "rsqrt", "sqrt", "convert", "broadcast",
    "reduce_sum", "reduce_max", "dot", "causal_mask", "output", "erf", "logistic",
)
DTYPES = ("f32", "f16", "bf16")


class Graph:
    """Builder for one fusion group.  Methods return the index of the new op."""

    def __init__(self):
        self.ops = []

    def _new(self, kind, dtype, shape, operands=(), axis=-1, attr=0.0, name=""):
        assert kind in KINDS and dtype in DTYPES
        self.ops.append(Op(kind, dtype, tuple(int(s) for s in shape),
                           tuple(int(o) for o in operands), int(axis), float(attr), name))
        return len(self.ops) - 1

    def dtype(self, i):
        return self.ops[i].dtype

    def shape(self, i):
        return self.ops[i].shape

    # leaves
    def parameter(self, name, dtype, shape):
        return self._new("parameter", dtype, shape, name=name)

    def constant(self, value, dtype="f32"):
        return self._new("constant", dtype, (), attr=value)

    # elementwise
    def _binary(self, kind, a, b):
        sa, sb = self.shape(a), self.shape(b)
        shape = sa if sa != () else sb
        assert sa == () or sb == () or sa == sb, (kind, sa, sb)
        dt = self.dtype(a) if sa != () else self.dtype(b)
        return self._new(kind, dt, shape, (a, b))

    def add(self, a, b): return self._binary("add", a, b)
    def subtract(self, a, b): return self._binary("subtract", a, b)
    def multiply(self, a, b): return self._binary("multiply", a, b)
    def divide(self, a, b): return self._binary("divide", a, b)
    def maximum(self, a, b): return self._binary("maximum", a, b)

    def _unary(self, kind, a):
        return self._new(kind, self.dtype(a), self.shape(a), (a,))

    def negate(self, a): return self._unary("negate", a)
    def exp(self, a): return self._unary("exp", a)
    def log(self, a): return self._unary("log", a)
    def tanh(self, a): return self._unary("tanh", a)
    def rsqrt(self, a): return self._unary("rsqrt", a)
    def sqrt(self, a): return self._unary("sqrt", a)
    def erf(self, a): return self._unary("erf", a)
    def logistic(self, a): return self._unary("logistic", a)

    def convert(self, a, dtype):
        return self._new("convert", dtype, self.shape(a), (a,))

    # shape ops
    def broadcast(self, a, shape, axis):
        sa = self.shape(a)
        assert axis + len(sa) <= len(shape)
        for d, e in enumerate(sa):
            assert e == 1 or e == shape[axis + d], (sa, shape, axis)
        return self._new("broadcast", self.dtype(a), shape, (a,), axis=axis)

    def _reduce(self, kind, a, axis):
        sa = self.shape(a)
        axis = axis % len(sa)
        return self._new(kind, self.dtype(a), sa[:axis] + sa[axis + 1:], (a,), axis=axis)

    def reduce_sum(self, a, axis): return self._reduce("reduce_sum", a, axis)
    def reduce_max(self, a, axis): return self._reduce("reduce_max", a, axis)

    def dot(self, a, b, transpose_b=False, dtype="f32"):
        sa, sb = self.shape(a), self.shape(b)
        assert len(sa) == 3 and len(sb) == 3 and sa[0] == sb[0]
        if transpose_b:
            assert sa[2] == sb[2]
            shape = (sa[0], sa[1], sb[1])
        else:
            assert sa[2] == sb[1]
            shape = (sa[0], sa[1], sb[2])
        return self._new("dot", dtype, shape, (a, b), axis=1 if transpose_b else 0)

    def causal_mask(self, a, fill):
        return self._new("causal_mask", self.dtype(a), self.shape(a), (a,), attr=fill)

    def output(self, a, name=""):
        return self._new("output", self.dtype(a), self.shape(a), (a,), name=name)

    # helper spellings used by several groups
    def row_broadcast(self, a, like):
        """[R...] per-row values -> shape of `like` (expanded along the last dim)."""
        return self.broadcast(a, self.shape(like), 0)

    def col_broadcast(self, a, like):
        """[C] per-column values -> shape of `like` (expanded along leading dims)."""
        return self.broadcast(a, self.shape(like), len(self.shape(like)) - 1)


# ----------------------------------------------------------------------------------
# The five groups of the benchmark.  Each returns a list[Op].
# ----------------------------------------------------------------------------------

def _layernorm_tail(g, r, gamma, beta, eps):
    """r -> layernorm(r) * gamma + beta over the last dim (biased variance, eps
    inside the root): row mean, subtract, square, row mean, rsqrt, scale, shift."""
    n = g.shape(r)[-1]
    mean = g.divide(g.reduce_sum(r, -1), g.constant(n))
    c = g.subtract(r, g.row_broadcast(mean, r))
    sq = g.multiply(c, c)
    var = g.divide(g.reduce_sum(sq, -1), g.constant(n))
    rstd = g.rsqrt(g.add(var, g.constant(eps)))
    xhat = g.multiply(c, g.row_broadcast(rstd, r))
    scaled = g.multiply(xhat, g.col_broadcast(gamma, r))
    return g.add(scaled, g.col_broadcast(beta, r))


def layernorm_fwd(rows, cols, dtype="f32", eps=1e-5):
    """Config 1: y = (x - mean) * rsqrt(var + eps) * gamma + beta."""
    g = Graph()
    x = g.parameter("x", dtype, (rows, cols))
    gamma = g.parameter("gamma", dtype, (cols,))
    beta = g.parameter("beta", dtype, (cols,))
    if dtype != "f32":
        x, gamma, beta = (g.convert(t, "f32") for t in (x, gamma, beta))
    y = _layernorm_tail(g, x, gamma, beta, eps)
    if dtype != "f32":
        y = g.convert(y, dtype)
    g.output(y, "y")
    return g.ops


def scaled_masked_softmax(shape, scale=0.125, mask="full", dtype="f32"):
    """Config 2: softmax over the last dim of (scores * scale + mask).

    mask="full": the mask has the shape of the scores.
    mask="key_padding": scores are [B,H,S,S] and the mask is [B,1,1,S].
    mask="none": no mask operand.
    """
    g = Graph()
    s = g.parameter("scores", dtype, shape)
    m = None
    if mask == "full":
        m = g.parameter("mask", dtype, shape)
    elif mask == "key_padding":
        assert len(shape) == 4
        m = g.parameter("mask", dtype, (shape[0], 1, 1, shape[3]))
    else:
        assert mask == "none"
    if dtype != "f32":
        s = g.convert(s, "f32")
        if m is not None:
            m = g.convert(m, "f32")
    z = g.multiply(s, g.constant(scale))
    if mask == "full":
        z = g.add(z, m)
    elif mask == "key_padding":
        z = g.add(z, g.broadcast(m, shape, 0))
    zmax = g.reduce_max(z, -1)
    e = g.exp(g.subtract(z, g.row_broadcast(zmax, z)))
    denom = g.reduce_sum(e, -1)
    p = g.divide(e, g.row_broadcast(denom, e))
    if dtype != "f32":
        p = g.convert(p, dtype)
    g.output(p, "p")
    return g.ops


def causal_attention(batch, seq, dim, dtype="f16", scale=None):
    """Config 3: O = softmax_rows(causal(Q K^T * scale)) V with fp32 accumulation."""
    if scale is None:
        scale = dim ** -0.5
    g = Graph()
    q = g.parameter("q", dtype, (batch, seq, dim))
    k = g.parameter("k", dtype, (batch, seq, dim))
    v = g.parameter("v", dtype, (batch, seq, dim))
    s = g.dot(q, k, transpose_b=True, dtype="f32")
    z = g.multiply(s, g.constant(scale))
    z = g.causal_mask(z, float("-inf"))
    zmax = g.reduce_max(z, -1)
    e = g.exp(g.subtract(z, g.row_broadcast(zmax, z)))
    denom = g.reduce_sum(e, -1)
    p = g.divide(e, g.row_broadcast(denom, e))
    p = g.convert(p, dtype)
    o = g.dot(p, v, transpose_b=False, dtype="f32")
    g.output(g.convert(o, dtype), "o")
    return g.ops


def attention_block(batch, sq, sk, dim, dtype="f16", scale=None, causal=False, fill=float("-inf"), mask=None,
                    gate=False, residual=False, lse=False, mask_outside_causal=False):
    """Schedule 3 with the elementwise ops the motivating pattern has around its two dots
    (Section 3.1): O = (softmax_rows(causal(Q K^T * scale + mask)) V) * gate + residual, optionally with a
    second output, the log-sum-exp of every score row.  mask: None, "key" ([batch, 1, sk], key padding),
    "full" ([batch, sq, sk]) or "shared" ([sq, sk], one bias for every batch element), fp32."""
    if scale is None:
        scale = dim ** -0.5
    g = Graph()
    q = g.parameter("q", dtype, (batch, sq, dim))
    k = g.parameter("k", dtype, (batch, sk, dim))
    v = g.parameter("v", dtype, (batch, sk, dim))
    z = g.multiply(g.dot(q, k, transpose_b=True, dtype="f32"), g.constant(scale))
    m = None
    if mask == "key":
        m = g.broadcast(g.parameter("mask", "f32", (batch, 1, sk)), (batch, sq, sk), 0)
    elif mask == "full":
        m = g.parameter("mask", "f32", (batch, sq, sk))
    elif mask == "shared":
        m = g.broadcast(g.parameter("mask", "f32", (sq, sk)), (batch, sq, sk), 1)
    if m is not None and not mask_outside_causal:
        z = g.add(z, m)
    if causal:
        z = g.causal_mask(z, fill)
    if m is not None and mask_outside_causal:
        z = g.add(m, z)
    zmax = g.reduce_max(z, -1)
    e = g.exp(g.subtract(z, g.row_broadcast(zmax, z)))
    denom = g.reduce_sum(e, -1)
    p = g.convert(g.divide(e, g.row_broadcast(denom, e)), dtype)
    o = g.dot(p, v, transpose_b=False, dtype="f32")
    if gate:
        o = g.multiply(o, g.convert(g.parameter("gate", dtype, (batch, sq, dim)), "f32"))
    if residual:
        o = g.add(o, g.convert(g.parameter("residual", dtype, (batch, sq, dim)), "f32"))
    g.output(g.convert(o, dtype), "o")
    if lse:
        g.output(g.add(g.log(denom), zmax), "lse")
    return g.ops


def sigmoid_attention(batch, sq, sk, kc, dim, dtype="bf16"):
    """A dot -> elementwise -> dot group that is no softmax attention: weights logistic(q k^T / sqrt(kc)), not
    normalised, returned as a second (fp32) output beside o = weights v.  The hand-written attention recogniser
    refuses it; the generated block-composed kernel runs both dots on the matrix unit."""
    g = Graph()
    q = g.parameter("q", dtype, (batch, sq, kc))
    k = g.parameter("k", dtype, (batch, sk, kc))
    v = g.parameter("v", dtype, (batch, sk, dim))
    w = g.logistic(g.multiply(g.dot(q, k, transpose_b=True, dtype="f32"), g.constant(kc ** -0.5)))
    o = g.dot(g.convert(w, dtype), v, transpose_b=False, dtype="f32")
    g.output(g.convert(o, dtype), "o")
    g.output(w, "weights")
    return g.ops


def attention_residual_layernorm(batch, sq, sk, dim, dtype="f16", eps=1e-5):
    """Softmax attention whose weights are normalised after the second dot (o = (exp(s - max) v) / sum), a residual,
    and LayerNorm over the head dim with gamma and beta: dot -> elementwise / reductions -> dot -> elementwise /
    reductions, one group.  x is stored [B, Sq, D], the keys as a weight matrix is, [B, D, Sk]."""
    g = Graph()
    q = g.parameter("q", dtype, (batch, sq, dim))
    kt = g.parameter("kt", dtype, (batch, dim, sk))
    v = g.parameter("v", dtype, (batch, sk, dim))
    res = g.parameter("res", dtype, (batch, sq, dim))
    gamma = g.parameter("gamma", "f32", (dim,))
    beta = g.parameter("beta", "f32", (dim,))
    s = g.multiply(g.dot(q, kt, transpose_b=False, dtype="f32"), g.constant(dim ** -0.5))
    e = g.exp(g.subtract(s, g.row_broadcast(g.reduce_max(s, -1), s)))
    den = g.reduce_sum(e, -1)
    o = g.dot(g.convert(e, dtype), v, transpose_b=False, dtype="f32")
    h = g.add(g.divide(o, g.row_broadcast(den, o)), g.convert(res, "f32"))
    y = _layernorm_tail(g, h, gamma, beta, eps)
    g.output(g.convert(y, dtype), "y")
    return g.ops


GELU_K0 = 0.7978845608028654   # sqrt(2/pi)
GELU_K1 = 0.044715


def bias_gelu_residual_layernorm(rows, cols, dtype="bf16", eps=1e-5):
    """Config 4: y = LayerNorm(gelu_tanh(x + bias) + residual) * gamma + beta,
    storage in `dtype`, all arithmetic in fp32."""
    g = Graph()
    x = g.parameter("x", dtype, (rows, cols))
    bias = g.parameter("bias", dtype, (cols,))
    res = g.parameter("residual", dtype, (rows, cols))
    gamma = g.parameter("gamma", dtype, (cols,))
    beta = g.parameter("beta", dtype, (cols,))
    if dtype != "f32":
        x, bias, res, gamma, beta = (g.convert(t, "f32") for t in (x, bias, res, gamma, beta))
    h = g.add(x, g.col_broadcast(bias, x))
    h3 = g.multiply(g.multiply(h, h), h)
    inner = g.multiply(g.add(h, g.multiply(h3, g.constant(GELU_K1))), g.constant(GELU_K0))
    t = g.tanh(inner)
    gelu = g.multiply(g.multiply(h, g.constant(0.5)), g.add(t, g.constant(1.0)))
    r = g.add(gelu, res)
    y = _layernorm_tail(g, r, gamma, beta, eps)
    if dtype != "f32":
        y = g.convert(y, dtype)
    g.output(y, "y")
    return g.ops


def layernorm_bwd(rows, cols, dtype="f32"):
    """Config 5: (dx, dgamma, dbeta) of LayerNorm from dy, x, gamma and the saved
    per-row mean and rstd.  Row reductions for dx, column reductions for the
    parameter gradients, 15 arithmetic ops."""
    assert dtype == "f32"
    g = Graph()
    dy = g.parameter("dy", dtype, (rows, cols))
    x = g.parameter("x", dtype, (rows, cols))
    gamma = g.parameter("gamma", dtype, (cols,))
    mean = g.parameter("mean", dtype, (rows,))
    rstd = g.parameter("rstd", dtype, (rows,))
    n = g.constant(cols)
    rstd_b = g.row_broadcast(rstd, x)
    xhat = g.multiply(g.subtract(x, g.row_broadcast(mean, x)), rstd_b)      # 2 ops
    gg = g.multiply(dy, g.col_broadcast(gamma, dy))                          # g = dy*gamma
    dbeta = g.reduce_sum(dy, 0)
    t = g.multiply(dy, xhat)
    dgamma = g.reduce_sum(t, 0)
    s1 = g.reduce_sum(gg, 1)
    gx = g.multiply(gg, xhat)
    s2 = g.reduce_sum(gx, 1)
    c1 = g.divide(s1, n)
    c2 = g.divide(s2, n)
    u = g.multiply(xhat, g.row_broadcast(c2, x))
    v = g.subtract(gg, g.row_broadcast(c1, x))
    w = g.subtract(v, u)
    dx = g.multiply(w, rstd_b)
    g.output(dx, "dx")
    g.output(dgamma, "dgamma")
    g.output(dbeta, "dbeta")
    return g.ops


# ----------------------------------------------------------------------------------
# All-elementwise groups (thread composition and kernel packing, Section 5.1).
# ----------------------------------------------------------------------------------

def bias_gelu_residual(rows, cols, dtype="bf16"):
    """y = gelu_tanh(x + bias) + residual: the prologue of config 4 as a group of its own."""
    g = Graph()
    x = g.parameter("x", dtype, (rows, cols))
    bias = g.parameter("bias", dtype, (cols,))
    res = g.parameter("residual", dtype, (rows, cols))
    if dtype != "f32":
        x, bias, res = (g.convert(t, "f32") for t in (x, bias, res))
    h = g.add(x, g.col_broadcast(bias, x))
    h3 = g.multiply(g.multiply(h, h), h)
    inner = g.multiply(g.add(h, g.multiply(h3, g.constant(GELU_K1))), g.constant(GELU_K0))
    gelu = g.multiply(g.multiply(h, g.constant(0.5)), g.add(g.tanh(inner), g.constant(1.0)))
    y = g.add(gelu, res)
    if dtype != "f32":
        y = g.convert(y, dtype)
    g.output(y, "y")
    return g.ops


def adam_update(shape, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, dtype="f32"):
    """Three packed outputs over one shape (the backward-phase gradient-accumulation
    pattern the paper packs): m' = b1*m + (1-b1)*g, v' = b2*v + (1-b2)*g*g,
    p' = p - lr * m' / (sqrt(v') + eps)."""
    g = Graph()
    p = g.parameter("p", dtype, shape)
    grad = g.parameter("grad", dtype, shape)
    m = g.parameter("m", dtype, shape)
    v = g.parameter("v", dtype, shape)
    m2 = g.add(g.multiply(m, g.constant(beta1)), g.multiply(grad, g.constant(1.0 - beta1)))
    v2 = g.add(g.multiply(v, g.constant(beta2)), g.multiply(g.multiply(grad, grad), g.constant(1.0 - beta2)))
    step = g.divide(g.multiply(m2, g.constant(lr)), g.add(g.sqrt(v2), g.constant(eps)))
    p2 = g.subtract(p, step)
    g.output(p2, "p")
    g.output(m2, "m")
    g.output(v2, "v")
    return g.ops


def swiglu(shape, dtype="bf16"):
    """y = silu(a) * b = a * logistic(a) * b: the gated activation of LLaMA-style MLPs, an
    all-elementwise group with two full operands."""
    g = Graph()
    a = g.parameter("a", dtype, shape)
    b = g.parameter("b", dtype, shape)
    af, bf = (a, b) if dtype == "f32" else (g.convert(a, "f32"), g.convert(b, "f32"))
    y = g.multiply(g.multiply(af, g.logistic(af)), bf)
    g.output(y if dtype == "f32" else g.convert(y, dtype), "y")
    return g.ops


def bias_gelu_erf_residual_layernorm(rows, cols, dtype="bf16", eps=1e-5):
    """Config 4 with the exact GELU, 0.5 h (1 + erf(h / sqrt 2)), in place of the tanh form."""
    g = Graph()
    x = g.parameter("x", dtype, (rows, cols))
    bias = g.parameter("bias", dtype, (cols,))
    res = g.parameter("residual", dtype, (rows, cols))
    gamma = g.parameter("gamma", dtype, (cols,))
    beta = g.parameter("beta", dtype, (cols,))
    if dtype != "f32":
        x, bias, res, gamma, beta = (g.convert(t, "f32") for t in (x, bias, res, gamma, beta))
    h = g.add(x, g.col_broadcast(bias, x))
    gelu = g.multiply(g.multiply(h, g.constant(0.5)), g.add(g.erf(g.multiply(h, g.constant(0.7071067811865476))), g.constant(1.0)))
    y = _layernorm_tail(g, g.add(gelu, res), gamma, beta, eps)
    g.output(y if dtype == "f32" else g.convert(y, dtype), "y")
    return g.ops


def multi_tensor_momentum(shapes, lr=1e-2, mu=0.9, dtypes=None):
    """The same update on several tensors of different shapes, as ONE group of independent parts
    (kernel packing of the backward phase's many small ops, Section 5.1): per tensor
    m' = mu*m + g, p' = p - lr*m'; parameters (p_k, g_k, m_k) and outputs (p'_k, m'_k) per tensor.
    `dtypes` gives each tensor's storage dtype (default all f32; the arithmetic is f32)."""
    g = Graph()
    dtypes = dtypes or ["f32"] * len(shapes)
    for k, (shape, dt) in enumerate(zip(shapes, dtypes)):
        p = g.parameter(f"p{k}", dt, shape)
        grad = g.parameter(f"g{k}", dt, shape)
        m = g.parameter(f"m{k}", dt, shape)
        pf, gf, mf = (p, grad, m) if dt == "f32" else tuple(g.convert(t, "f32") for t in (p, grad, m))
        m2 = g.add(g.multiply(mf, g.constant(mu)), gf)
        p2 = g.subtract(pf, g.multiply(m2, g.constant(lr)))
        g.output(p2 if dt == "f32" else g.convert(p2, dt), f"p{k}")
        g.output(m2 if dt == "f32" else g.convert(m2, dt), f"m{k}")
    return g.ops


def clip_by_global_norm(shapes, max_norm=1.0):
    """Gradient clipping over several tensors: n = sqrt(sum_k sum(g_k^2)), every g_k scaled by
    1 / max(1, n / max_norm).  Each tensor's sum of squares is spelled as a chain of reductions down
    to a scalar, the scalars are added, and the factor is broadcast back: a graph that no single
    group covers (a value reduced over everything feeds ops on the full tensors), so the planner
    has to cut it.  Parameters g_k, outputs the clipped g_k, in order."""
    g = Graph()
    params = [g.parameter(f"g{k}", "f32", shape) for k, shape in enumerate(shapes)]
    total = None
    for x in params:
        s = g.multiply(x, x)
        while len(g.shape(s)) > 0:
            s = g.reduce_sum(s, len(g.shape(s)) - 1)
        total = s if total is None else g.add(total, s)
    norm = g.sqrt(total)
    factor = g.divide(g.constant(1.0), g.maximum(g.divide(norm, g.constant(max_norm)), g.constant(1.0)))
    for k, x in enumerate(params):
        g.output(g.multiply(x, g.broadcast(factor, g.shape(x), 0)), f"g{k}")
    return g.ops


def norm_over_trailing_dims(shape, n_trailing=2, dtype="f32", eps=1e-5):
    """Normalisation of x over its last `n_trailing` dims jointly (a group or instance norm's
    statistics), every reduction spelled as a chain of reductions over one dim each:
    c = x - mean, y = c * rsqrt(mean(c^2) + eps); outputs (y, mean).  Parameter x."""
    g = Graph()
    x = g.parameter("x", dtype, shape)
    xf = x if dtype == "f32" else g.convert(x, "f32")
    count = 1
    for d in shape[len(shape) - n_trailing:]:
        count *= d

    def chain(v, reduce):
        for _ in range(n_trailing):
            v = reduce(v, len(g.shape(v)) - 1)
        return v
    mean = g.multiply(chain(xf, g.reduce_sum), g.constant(1.0 / count))
    c = g.subtract(xf, g.broadcast(mean, shape, 0))
    var = g.multiply(chain(g.multiply(c, c), g.reduce_sum), g.constant(1.0 / count))
    rstd = g.rsqrt(g.add(var, g.constant(eps)))
    y = g.multiply(c, g.broadcast(rstd, shape, 0))
    g.output(y if dtype == "f32" else g.convert(y, dtype), "y")
    g.output(mean, "mean")
    return g.ops


def max_abs_over_trailing_dims(shape, n_trailing, dtype="f32"):
    """max(x, -x) reduced over the last `n_trailing` dims by a chain of reduce_max ops."""
    g = Graph()
    x = g.parameter("x", dtype, shape)
    v = x if dtype == "f32" else g.convert(x, "f32")
    v = g.maximum(v, g.negate(v))
    for _ in range(n_trailing):
        v = g.reduce_max(v, len(g.shape(v)) - 1)
    g.output(v, "amax")
    return g.ops


def sequence_pool(shape, levels=1, dtype="f32", with_row_work=False, pool="sum"):
    """Sum pooling over the innermost row dims: x[.., S, H] -> tanh -> sum over S -> [.., H] (with
    levels=2, over the two dims before the last, each a reduction of its own).  With row work the
    pooled value is tanh(x - rowmax(x)), which is a second, full-size output.  `pool`: "sum", "max" or
    "both" (two pooled outputs).  Parameter x; outputs (full value if any, pooled...); pooled outputs are f32."""
    g = Graph()
    x = g.parameter("x", dtype, shape)
    v = x if dtype == "f32" else g.convert(x, "f32")
    if with_row_work:
        m = g.reduce_max(v, len(shape) - 1)
        v = g.tanh(g.subtract(v, g.broadcast(m, shape, 0)))
        g.output(v if dtype == "f32" else g.convert(v, dtype), "y")
    else:
        v = g.tanh(v)
    for kind in (("sum", "max") if pool == "both" else (pool,)):
        s = v
        for _ in range(levels):
            s = (g.reduce_sum if kind == "sum" else g.reduce_max)(s, len(g.shape(s)) - 2)
        g.output(s, "pooled_" + kind)
    return g.ops


def encoder_tail_stack(n_layers, rows, cols, eps=1e-5):
    """`n_layers` times bias + GELU(tanh) + residual + LayerNorm, each layer reading the one before:
    every op is local to a row, so any stretch of the list is a valid row group -- a planner test for
    segments longer than a pattern may be.  Parameters: x[rows, cols], then (bias, gamma, beta)[cols]
    per layer; one output."""
    g = Graph()
    cur = g.parameter("x", "f32", (rows, cols))
    for k in range(n_layers):
        b, ga, be = (g.parameter(f"{n}{k}", "f32", (cols,)) for n in ("bias", "gamma", "beta"))
        h = g.add(cur, g.col_broadcast(b, cur))
        inner = g.multiply(g.add(h, g.multiply(g.multiply(g.multiply(h, h), h), g.constant(0.044715))), g.constant(0.7978845608028654))
        gelu = g.multiply(g.multiply(h, g.constant(0.5)), g.add(g.tanh(inner), g.constant(1.0)))
        cur = _layernorm_tail(g, g.add(gelu, cur), ga, be, eps)
    g.output(cur, "y")
    return g.ops


def scale_shift_rows_cols(shape, dtype="f32"):
    """y = (x - rowv) * colv / (1 + exp(-x)) with a per-row and a per-column operand:
    broadcasts along either side folded into one elementwise group."""
    g = Graph()
    x = g.parameter("x", dtype, shape)
    rowv = g.parameter("rowv", dtype, shape[:-1])
    colv = g.parameter("colv", dtype, (shape[-1],))
    if dtype != "f32":
        x, rowv, colv = (g.convert(t, "f32") for t in (x, rowv, colv))
    a = g.multiply(g.subtract(x, g.row_broadcast(rowv, x)), g.col_broadcast(colv, x))
    sig = g.divide(g.constant(1.0), g.add(g.exp(g.negate(x)), g.constant(1.0)))
    y = g.multiply(a, sig)
    if dtype != "f32":
        y = g.convert(y, dtype)
    g.output(y, "y")
    return g.ops


# ----------------------------------------------------------------------------------
# Row groups outside the five configs (warp composition on other op mixes, Section 5.1).
# ----------------------------------------------------------------------------------

def _f32_in(g, dtype, *ts):
    return ts if dtype == "f32" else tuple(g.convert(t, "f32") for t in ts)


def bias_gelu_bwd(rows, cols, dtype="f32"):
    """Backward of y = gelu_tanh(x + bias): dx = dy * gelu'(h), dbias = column sums of dx.  An
    elementwise chain packed with a reduction over the rows and no row reduction at all
    (backward-phase packing, Section 5.1)."""
    g = Graph()
    dy = g.parameter("dy", dtype, (rows, cols))
    x = g.parameter("x", dtype, (rows, cols))
    b = g.parameter("bias", dtype, (cols,))
    dyf, xf, bf = _f32_in(g, dtype, dy, x, b)
    h = g.add(xf, g.col_broadcast(bf, xf))
    h2 = g.multiply(h, h)
    u = g.multiply(g.multiply(h, g.add(g.multiply(h2, g.constant(GELU_K1)), g.constant(1.0))), g.constant(GELU_K0))
    t = g.tanh(u)
    # d/dh [0.5 h (1 + t)] = 0.5 (1 + t) + 0.5 h (1 - t^2) k0 (1 + 3 k1 h^2)
    du = g.multiply(g.add(g.multiply(h2, g.constant(3.0 * GELU_K1)), g.constant(1.0)), g.constant(GELU_K0))
    dt = g.multiply(g.subtract(g.constant(1.0), g.multiply(t, t)), du)
    dg = g.add(g.multiply(g.add(t, g.constant(1.0)), g.constant(0.5)), g.multiply(g.multiply(h, g.constant(0.5)), dt))
    dx = g.multiply(dyf, dg)
    g.output(dx if dtype == "f32" else g.convert(dx, dtype), "dx")
    g.output(g.reduce_sum(dx, 0), "dbias")
    return g.ops


def gated_rows(shape, dtype="f32"):
    """Per-row arithmetic beside full arithmetic with no reduction: gate = tanh(rowv) * rowv + 1
    (computed once per row), y = x * gate + colv, and the gate itself as a second output."""
    g = Graph()
    x = g.parameter("x", dtype, shape)
    rowv = g.parameter("rowv", dtype, shape[:-1])
    colv = g.parameter("colv", dtype, (shape[-1],))
    xf, rf, cf = _f32_in(g, dtype, x, rowv, colv)
    gate = g.add(g.multiply(g.tanh(rf), rf), g.constant(1.0))
    y = g.add(g.multiply(xf, g.row_broadcast(gate, xf)), g.col_broadcast(cf, xf))
    g.output(y if dtype == "f32" else g.convert(y, dtype), "y")
    g.output(gate if dtype == "f32" else g.convert(gate, dtype), "gate")
    return g.ops


def log_softmax(shape, dtype="f32"):
    """y = x - max - log(sum(exp(x - max))) over the last dim."""
    g = Graph()
    x = g.parameter("x", dtype, shape)
    (xf,) = _f32_in(g, dtype, x)
    m = g.reduce_max(xf, -1)
    c = g.subtract(xf, g.row_broadcast(m, xf))
    lse = g.log(g.reduce_sum(g.exp(c), -1))
    y = g.subtract(c, g.row_broadcast(lse, xf))
    if dtype != "f32":
        y = g.convert(y, dtype)
    g.output(y, "y")
    return g.ops


def rmsnorm(shape, dtype="f32", eps=1e-6):
    """y = x * rsqrt(mean(x^2) + eps) * gamma."""
    g = Graph()
    x = g.parameter("x", dtype, shape)
    gamma = g.parameter("gamma", dtype, (shape[-1],))
    xf, gf = _f32_in(g, dtype, x, gamma)
    ms = g.divide(g.reduce_sum(g.multiply(xf, xf), -1), g.constant(shape[-1]))
    r = g.rsqrt(g.add(ms, g.constant(eps)))
    y = g.multiply(g.multiply(xf, g.row_broadcast(r, xf)), g.col_broadcast(gf, xf))
    if dtype != "f32":
        y = g.convert(y, dtype)
    g.output(y, "y")
    return g.ops


def rmsnorm_one_plus_weight(shape, dtype="bf16", eps=1e-6):
    """y = x * rsqrt(mean(x^2) + eps) * (1 + w): the scale vector is computed in the group from the
    per-column parameter (a [C]-shaped op whose result is broadcast over the rows)."""
    g = Graph()
    x = g.parameter("x", dtype, shape)
    w = g.parameter("w", dtype, (shape[-1],))
    xf, wf = _f32_in(g, dtype, x, w)
    ms = g.divide(g.reduce_sum(g.multiply(xf, xf), -1), g.constant(shape[-1]))
    inv = g.rsqrt(g.add(ms, g.constant(eps)))
    scale = g.add(wf, g.constant(1.0))
    y = g.multiply(g.multiply(xf, g.row_broadcast(inv, xf)), g.col_broadcast(scale, xf))
    g.output(y if dtype == "f32" else g.convert(y, dtype), "y")
    return g.ops


def l2_normalize_scaled(shape, dtype="f32"):
    """y = x * s / sqrt(sum(x^2)) with one scale s per row; also returns the norms."""
    g = Graph()
    x = g.parameter("x", dtype, shape)
    s = g.parameter("s", dtype, shape[:-1])
    xf, sf = _f32_in(g, dtype, x, s)
    norm = g.sqrt(g.reduce_sum(g.multiply(xf, xf), -1))
    y = g.divide(g.multiply(xf, g.row_broadcast(sf, xf)), g.row_broadcast(norm, xf))
    if dtype != "f32":
        y = g.convert(y, dtype)
    g.output(y, "y")
    g.output(norm, "norm")
    return g.ops


def layernorm_fwd_with_stats(rows, cols, dtype="f32", eps=1e-5):
    """LayerNorm forward that also returns the per-row mean and reciprocal standard deviation
    (what a training forward pass saves for the backward pass): a 3-tuple."""
    g = Graph()
    x = g.parameter("x", dtype, (rows, cols))
    gamma = g.parameter("gamma", dtype, (cols,))
    beta = g.parameter("beta", dtype, (cols,))
    xf, gf, bf = _f32_in(g, dtype, x, gamma, beta)
    mean = g.divide(g.reduce_sum(xf, -1), g.constant(cols))
    c = g.subtract(xf, g.row_broadcast(mean, xf))
    var = g.divide(g.reduce_sum(g.multiply(c, c), -1), g.constant(cols))
    rstd = g.rsqrt(g.add(var, g.constant(eps)))
    y = g.add(g.multiply(g.multiply(c, g.row_broadcast(rstd, xf)), g.col_broadcast(gf, xf)), g.col_broadcast(bf, xf))
    if dtype != "f32":
        y = g.convert(y, dtype)
    g.output(y, "y")
    g.output(mean, "mean")
    g.output(rstd, "rstd")
    return g.ops


def softmax_with_lse(shape, temperature=0.7, dtype="f32"):
    """p = softmax(x / T) over the last dim, plus the log-sum-exp of x / T per row."""
    g = Graph()
    x = g.parameter("x", dtype, shape)
    (xf,) = _f32_in(g, dtype, x)
    z = g.divide(xf, g.constant(temperature))
    m = g.reduce_max(z, -1)
    e = g.exp(g.subtract(z, g.row_broadcast(m, z)))
    ssum = g.reduce_sum(e, -1)
    p = g.divide(e, g.row_broadcast(ssum, z))
    lse = g.add(g.log(ssum), m)
    if dtype != "f32":
        p = g.convert(p, dtype)
    g.output(p, "p")
    g.output(lse, "lse")
    return g.ops


def row_sum_of_squares(shape, dtype="f32"):
    """One per-row output only: sum(x^2) over the last dim."""
    g = Graph()
    x = g.parameter("x", dtype, shape)
    (xf,) = _f32_in(g, dtype, x)
    g.output(g.reduce_sum(g.multiply(xf, xf), -1), "ss")
    return g.ops


def multi_interest_pattern(batch, m=94, n=94, k=1, scale=0.25, gain=0.5):
    """A stand-in for the paper's motivating example (Section 3.1; its figure is not
    available): two batched dots around nine elementwise ops and two reductions, with
    a four-element output tuple (subtract, divide, log_1, multiply_2).  dot_1 expands
    two small tensors into a [batch, m, n] tile (contraction length k, 1 in the sizes
    the paper quotes); dot_2 contracts the tile back to one value per row.

      dot_1      = x[B,m,k] . y[B,k,n]
      multiply   = dot_1 * scale
      add        = multiply + mask[B,1,n]
      reduce_max = max_n add
      subtract   = add - reduce_max            -> output
      exp        = exp(subtract)
      reduce_sum = sum_n exp
      divide     = exp / reduce_sum            -> output
      log        = log(reduce_sum)
      log_1      = log + reduce_max            -> output  [B,m]
      dot_2      = divide . v[B,n,1]           [B,m,1]
      multiply_1 = dot_2 * gate[B,m,1]
      multiply_2 = multiply_1 * gain           -> output  [B,m,1]
    """
    g = Graph()
    x = g.parameter("x", "f32", (batch, m, k))
    y = g.parameter("y", "f32", (batch, k, n))
    mask = g.parameter("mask", "f32", (batch, 1, n))
    v = g.parameter("v", "f32", (batch, n, 1))
    gate = g.parameter("gate", "f32", (batch, m, 1))
    full = (batch, m, n)
    dot_1 = g.dot(x, y)
    multiply = g.multiply(dot_1, g.constant(scale))
    add = g.add(multiply, g.broadcast(mask, full, 0))
    reduce_max = g.reduce_max(add, -1)
    subtract = g.subtract(add, g.row_broadcast(reduce_max, add))
    exp = g.exp(subtract)
    reduce_sum = g.reduce_sum(exp, -1)
    divide = g.divide(exp, g.row_broadcast(reduce_sum, add))
    log = g.log(reduce_sum)
    log_1 = g.add(log, reduce_max)
    dot_2 = g.dot(divide, v)
    multiply_1 = g.multiply(dot_2, gate)
    multiply_2 = g.multiply(multiply_1, g.constant(gain))
    g.output(subtract, "subtract")
    g.output(divide, "divide")
    g.output(log_1, "log_1")
    g.output(multiply_2, "multiply_2")
    return g.ops


def causal_softmax(shape, scale=0.125, dtype="f32"):
    """softmax over the last dim of causally masked scores [..., S, S] (keys right of the diagonal
    excluded): the middle of an attention block as a group of its own."""
    g = Graph()
    s = g.parameter("scores", dtype, shape)
    (sf,) = _f32_in(g, dtype, s)
    z = g.causal_mask(g.multiply(sf, g.constant(scale)), float("-inf"))
    m = g.reduce_max(z, -1)
    e = g.exp(g.subtract(z, g.row_broadcast(m, z)))
    p = g.divide(e, g.row_broadcast(g.reduce_sum(e, -1), z))
    if dtype != "f32":
        p = g.convert(p, dtype)
    g.output(p, "p")
    return g.ops


def causal_fill(shape, fill=-1e4, dtype="f32"):
    """y = causal_mask(x * 2, fill): an all-elementwise group with an index-dependent op."""
    g = Graph()
    x = g.parameter("x", dtype, shape)
    (xf,) = _f32_in(g, dtype, x)
    y = g.causal_mask(g.multiply(xf, g.constant(2.0)), fill)
    if dtype != "f32":
        y = g.convert(y, dtype)
    g.output(y, "y")
    return g.ops


# ----------------------------------------------------------------------------------
# Computation graphs larger than one fusion group (input of the fusion planner, Section 4).
# ----------------------------------------------------------------------------------

def encoder_tail(rows, cols, batch, seq, dtype="f32"):
    """Two independent branches of a Transformer block, as one graph:
      scores[batch, seq, seq] -> * scale -> + mask -> softmax                       -> p
      x[rows, cols] -> + bias -> gelu -> + residual -> layernorm -> * 2 -> tanh     -> y
                                                     and the row sums of y**2        -> ss
    The planner should find one stitched group per connected branch."""
    g = Graph()
    s = g.parameter("scores", dtype, (batch, seq, seq))
    m = g.parameter("mask", dtype, (batch, 1, seq))
    x = g.parameter("x", dtype, (rows, cols))
    bias = g.parameter("bias", dtype, (cols,))
    res = g.parameter("residual", dtype, (rows, cols))
    gamma = g.parameter("gamma", dtype, (cols,))
    beta = g.parameter("beta", dtype, (cols,))
    z = g.add(g.multiply(s, g.constant(0.125)), g.broadcast(m, (batch, seq, seq), 0))
    mx = g.reduce_max(z, -1)
    e = g.exp(g.subtract(z, g.row_broadcast(mx, z)))
    p = g.divide(e, g.row_broadcast(g.reduce_sum(e, -1), z))
    g.output(p, "p")
    h = g.add(x, g.col_broadcast(bias, x))
    h3 = g.multiply(g.multiply(h, h), h)
    inner = g.multiply(g.add(h, g.multiply(h3, g.constant(GELU_K1))), g.constant(GELU_K0))
    gelu = g.multiply(g.multiply(h, g.constant(0.5)), g.add(g.tanh(inner), g.constant(1.0)))
    r = g.add(gelu, res)
    ln = _layernorm_tail(g, r, gamma, beta, 1e-5)
    y = g.tanh(g.multiply(ln, g.constant(2.0)))
    g.output(y, "y")
    g.output(g.reduce_sum(g.multiply(y, y), -1), "ss")
    return g.ops


def encoder_tail_bwd(rows, cols):
    """Backward of y = LayerNorm(gelu_tanh(x + bias) + residual) from dy and what the forward pass
    saved (r = the LayerNorm input, its per-row mean and rstd): dr (= the residual's gradient), dx,
    and the three parameter gradients dgamma, dbeta, dbias -- two row reductions, three column
    reductions and two full outputs over the same rows."""
    g = Graph()
    dy = g.parameter("dy", "f32", (rows, cols))
    x = g.parameter("x", "f32", (rows, cols))
    bias = g.parameter("bias", "f32", (cols,))
    r = g.parameter("r", "f32", (rows, cols))
    gamma = g.parameter("gamma", "f32", (cols,))
    mean = g.parameter("mean", "f32", (rows,))
    rstd = g.parameter("rstd", "f32", (rows,))
    n = g.constant(cols)
    rstd_b = g.row_broadcast(rstd, r)
    xhat = g.multiply(g.subtract(r, g.row_broadcast(mean, r)), rstd_b)
    gg = g.multiply(dy, g.col_broadcast(gamma, dy))
    dbeta = g.reduce_sum(dy, 0)
    dgamma = g.reduce_sum(g.multiply(dy, xhat), 0)
    c1 = g.divide(g.reduce_sum(gg, -1), n)
    c2 = g.divide(g.reduce_sum(g.multiply(gg, xhat), -1), n)
    dr = g.multiply(g.subtract(g.subtract(gg, g.row_broadcast(c1, gg)), g.multiply(xhat, g.row_broadcast(c2, gg))), rstd_b)
    h = g.add(x, g.col_broadcast(bias, x))
    h2 = g.multiply(h, h)
    u = g.multiply(g.multiply(h, g.add(g.multiply(h2, g.constant(GELU_K1)), g.constant(1.0))), g.constant(GELU_K0))
    t = g.tanh(u)
    du = g.multiply(g.add(g.multiply(h2, g.constant(3.0 * GELU_K1)), g.constant(1.0)), g.constant(GELU_K0))
    dt = g.multiply(g.subtract(g.constant(1.0), g.multiply(t, t)), du)
    dg = g.add(g.multiply(g.add(t, g.constant(1.0)), g.constant(0.5)), g.multiply(g.multiply(h, g.constant(0.5)), dt))
    dx = g.multiply(dr, dg)
    g.output(dr, "dr")
    g.output(dx, "dx")
    g.output(dgamma, "dgamma")
    g.output(dbeta, "dbeta")
    g.output(g.reduce_sum(dx, 0), "dbias")
    return g.ops


def crossing_branches(rows, cols):
    """Two chains that feed each other, so that fusing each chain on its own would make the
    contracted graph cyclic (the situation of the paper's cyclic-dependence figure, Section 4.1):
      a1 = exp(x); m = a1 * 2; a2 = m + colbc(b1); c = colsum(a1)      (full shape + column sum)
      b1 = tanh(v); n = b1 * 3; b2 = n + c                               (per-column values)
    a2 reads b1, b2 reads c: {a1, m, a2, c} and {b1, n, b2} are each convex, together cyclic."""
    g = Graph()
    x = g.parameter("x", "f32", (rows, cols))
    v = g.parameter("v", "f32", (cols,))
    a1 = g.exp(x)
    m = g.multiply(a1, g.constant(2.0))
    b1 = g.tanh(v)
    n = g.multiply(b1, g.constant(3.0))
    a2 = g.add(m, g.col_broadcast(b1, m))
    c = g.reduce_sum(a1, 0)
    b2 = g.add(n, c)
    g.output(a2, "a2")
    g.output(b2, "b2")
    return g.ops


# ----------------------------------------------------------------------------------
# Random groups (parity fuzzing of the kernel generators).
# ----------------------------------------------------------------------------------

def random_row_group(rng, shape, dtype="f32", n_ops=12, column_sums=False):
    """A random DAG over one full shape: elementwise ops on full and per-row values, reductions
    over the last dim, per-row values broadcast back, a per-row and a per-column operand;
    values are kept tame (tanh before exp, sums divided by the row length) so that every op
    list is well conditioned.  `rng` is a random.Random.  Returns (ops, parameter shapes)."""
    g = Graph()
    rowshape, ncol = tuple(shape[:-1]), shape[-1]
    x = g.parameter("x", dtype, shape)
    y = g.parameter("y", dtype, shape)
    rv = g.parameter("rv", dtype, rowshape) if rowshape else None
    cv = g.parameter("cv", dtype, (ncol,))
    conv = (lambda t: t) if dtype == "f32" else (lambda t: g.convert(t, "f32"))
    full = [conv(x), conv(y)]
    rows = [conv(rv)] if rv is not None else []
    cvf = conv(cv)
    colvals = [cvf]                # per-column values: the parameter and what is computed from it
    for _ in range(n_ops):
        kind = rng.choice(["bin", "bin", "un", "reduce", "rowop", "bcast_row", "bcast_col", "const", "colop"])
        if kind == "bin":
            a, b = rng.choice(full), rng.choice(full)
            full.append(getattr(g, rng.choice(["add", "subtract", "multiply", "maximum"]))(a, b))
        elif kind == "un":
            a = rng.choice(full)
            op = rng.choice(["tanh", "negate", "exp_tanh", "square_plus"])
            if op == "exp_tanh":
                full.append(g.exp(g.tanh(a)))
            elif op == "square_plus":
                full.append(g.rsqrt(g.add(g.multiply(a, a), g.constant(1.0))))
            else:
                full.append(getattr(g, op)(a))
        elif kind == "reduce" and rowshape:
            a = rng.choice(full)
            if rng.random() < 0.5:
                rows.append(g.divide(g.reduce_sum(a, -1), g.constant(ncol)))
            else:
                rows.append(g.reduce_max(g.tanh(a), -1))
        elif kind == "rowop" and len(rows) >= 1:
            a, b = rng.choice(rows), rng.choice(rows)
            rows.append(getattr(g, rng.choice(["add", "multiply", "maximum"]))(g.tanh(a), b))
        elif kind == "bcast_row" and rows:
            full.append(getattr(g, rng.choice(["add", "multiply", "subtract"]))(rng.choice(full), g.row_broadcast(rng.choice(rows), full[0])))
        elif kind == "bcast_col":
            full.append(getattr(g, rng.choice(["add", "multiply"]))(rng.choice(full), g.col_broadcast(rng.choice(colvals), full[0])))
        elif kind == "const":
            full.append(getattr(g, rng.choice(["add", "multiply"]))(rng.choice(full), g.constant(rng.choice([0.5, -1.25, 2.0]))))
        elif kind == "colop" and len(shape) >= 2 and tuple(shape[:-1]) != (ncol,):
            a = rng.choice(colvals)
            colvals.append(rng.choice([lambda: g.add(g.tanh(a), g.constant(1.0)), lambda: g.multiply(a, rng.choice(colvals)),
                                       lambda: g.maximum(g.negate(a), cvf)])())
    out = full[-1]
    if out in (full[0], full[1]):
        out = g.add(full[0], full[1])
    g.output(out if dtype == "f32" else g.convert(out, dtype))
    computed_rows = [r for r in rows if g.ops[r].kind not in ("parameter", "convert")]
    if computed_rows:
        g.output(computed_rows[-1])
    if column_sums == "runs" and len(shape) >= 3:
        # sums over the innermost row dims only, each link over the dim before the last:
        # [B, N, S, H] -> [B, N, H] (-> [B, H]); two values summed the same way
        levels = rng.randint(1, len(shape) - 2)
        for _ in range(rng.randint(1, 2)):
            c = g.tanh(rng.choice(full))
            for _ in range(levels):
                c = g.reduce_sum(c, len(g.shape(c)) - 2)
            g.output(c)
    elif column_sums and len(shape) >= 2:
        c = g.tanh(rng.choice(full))
        for _ in range(len(shape) - 1):          # one sum per leading dim: [B, S, H] -> [S, H] -> [H]
            c = g.reduce_sum(c, 0)
        g.output(c)
    pshapes = [shape, shape] + ([rowshape] if rowshape else []) + [(ncol,)]
    return g.ops, pshapes


def random_program(rng, rows, cols, n_ops=30):
    """A random graph larger than one fusion group, over full [rows, cols], per-row [rows] and
    per-column [cols] values: elementwise ops on each class, reductions over the last dim and over
    the rows as INTERMEDIATES (their results are broadcast back into later full ops), so that a
    fusion plan has to cut it into several dependent groups.  Values stay tame (tanh before exp and
    before every reduction, sums divided by their length).  `rng` is a random.Random.
    Returns (ops, parameter shapes)."""
    g = Graph()
    x = g.parameter("x", "f32", (rows, cols))
    y = g.parameter("y", "f32", (rows, cols))
    rv = g.parameter("rv", "f32", (rows,))
    cv = g.parameter("cv", "f32", (cols,))
    full, rws, cls = [x, y], [rv], [cv]
    for _ in range(n_ops):
        kind = rng.choice(["bin", "bin", "un", "rsum", "rmax", "csum", "rowop", "colop", "bcast_row", "bcast_col", "const"])
        if kind == "bin":
            full.append(getattr(g, rng.choice(["add", "subtract", "multiply", "maximum"]))(rng.choice(full), rng.choice(full)))
        elif kind == "un":
            a = rng.choice(full)
            full.append(rng.choice([lambda: g.tanh(a), lambda: g.exp(g.tanh(a)), lambda: g.rsqrt(g.add(g.multiply(a, a), g.constant(1.0)))])())
        elif kind == "rsum":
            rws.append(g.divide(g.reduce_sum(g.tanh(rng.choice(full)), -1), g.constant(cols)))
        elif kind == "rmax":
            rws.append(g.reduce_max(g.tanh(rng.choice(full)), -1))
        elif kind == "csum":
            cls.append(g.divide(g.reduce_sum(g.tanh(rng.choice(full)), 0), g.constant(rows)))
        elif kind == "rowop":
            rws.append(getattr(g, rng.choice(["add", "multiply", "maximum"]))(g.tanh(rng.choice(rws)), rng.choice(rws)))
        elif kind == "colop":
            cls.append(getattr(g, rng.choice(["add", "multiply", "maximum"]))(g.tanh(rng.choice(cls)), rng.choice(cls)))
        elif kind == "bcast_row":
            full.append(getattr(g, rng.choice(["add", "multiply", "subtract"]))(rng.choice(full), g.row_broadcast(rng.choice(rws), x)))
        elif kind == "bcast_col":
            full.append(getattr(g, rng.choice(["add", "multiply"]))(rng.choice(full), g.col_broadcast(rng.choice(cls), x)))
        else:
            full.append(getattr(g, rng.choice(["add", "multiply"]))(rng.choice(full), g.constant(rng.choice([0.5, -1.25, 2.0]))))
    out = full[-1] if len(full) > 2 else g.add(x, y)
    g.output(out, "full")
    computed = lambda lst: [v for v in lst if g.ops[v].kind != "parameter"]
    seen = {out}
    for lst, name in ((rws, "row"), (cls, "col")):
        c = [v for v in computed(lst) if v not in seen]
        if c:
            g.output(c[-1], name)
            seen.add(c[-1])
    # only what reaches an output stays (parameters all stay: they are the launch's inputs)
    ops = g.ops
    live = [op.kind in ("output", "parameter") for op in ops]
    for i in range(len(ops) - 1, -1, -1):
        if live[i]:
            for o in ops[i].operands:
                live[o] = True
    renumber, kept = {}, []
    for i, op in enumerate(ops):
        if live[i]:
            renumber[i] = len(kept)
            kept.append(Op(op.kind, op.dtype, op.shape, tuple(renumber[o] for o in op.operands), op.axis, op.attr, op.name))
    return kept, [(rows, cols), (rows, cols), (rows,), (cols,)]


def random_dot_group(rng, B, M, N, Kc, D, dtype="f16"):
    """A random group around two batched dots: x[B,M,K] . w (stored [B,N,K] or [B,K,N]) -> a random middle section
    on the [B,M,N] tile that ends in bounded weights (softmax, scaled sigmoid or normalised relu^2) -> . v[B,N,D]
    -> a random epilogue on the [B,M,D] result (residual, per-column gate, per-row values of either section, row
    reductions over D, tanh).  Outputs: the last value, a per-row value, sometimes the second dot's own result.
    `rng` is a random.Random.  Returns (ops, [(shape, dtype) per parameter])."""
    g = Graph()
    kn = rng.random() < 0.5
    x = g.parameter("x", dtype, (B, M, Kc))
    w = g.parameter("w", dtype, (B, Kc, N) if kn else (B, N, Kc))
    v = g.parameter("v", dtype, (B, N, D))
    bias = g.parameter("bias", "f32", (N,))
    temp = g.parameter("temp", "f32", (B, M))
    res = g.parameter("res", dtype, (B, M, D))
    gate = g.parameter("gate", "f32", (D,))
    params = [((B, M, Kc), dtype), ((B, Kc, N) if kn else (B, N, Kc), dtype), ((B, N, D), dtype), ((N,), "f32"), ((B, M), "f32"),
              ((B, M, D), dtype), ((D,), "f32")]
    s = g.multiply(g.dot(x, w, transpose_b=not kn, dtype="f32"), g.constant(Kc ** -0.5))
    rows = [g.tanh(temp)]
    for _ in range(rng.randint(0, 3)):
        kind = rng.choice(["bias", "temp", "tanh", "const"])
        if kind == "bias":
            s = g.add(s, g.col_broadcast(bias, s))
        elif kind == "temp":
            s = g.multiply(s, g.row_broadcast(rows[0], s))
        elif kind == "tanh":
            s = g.multiply(g.tanh(s), g.constant(2.0))
        else:
            s = g.add(s, g.constant(rng.choice([0.5, -1.0])))
    form = rng.choice(["softmax", "sigmoid", "relu2"])
    if form == "softmax":
        smax = g.reduce_max(s, -1)
        e = g.exp(g.subtract(s, g.row_broadcast(smax, s)))
        den = g.reduce_sum(e, -1)
        rows += [smax, g.log(den)]
        p = g.divide(e, g.row_broadcast(den, e))
    elif form == "sigmoid":
        p = g.multiply(g.logistic(s), g.constant(1.0 / N))
        rows.append(g.reduce_sum(p, -1))
    else:
        r = g.maximum(s, g.constant(0.0))
        r2 = g.add(g.multiply(r, r), g.constant(1e-2))
        den = g.reduce_sum(r2, -1)
        rows.append(g.divide(den, g.constant(float(N))))
        p = g.divide(r2, g.row_broadcast(den, r2))
    o = g.dot(g.convert(p, dtype), v, dtype="f32")
    dot_result = o
    resf = g.convert(res, "f32")
    for _ in range(rng.randint(1, 6)):
        kind = rng.choice(["res", "gate", "row", "tanh", "center", "const", "scale_by_max"])
        if kind == "res":
            o = g.add(o, resf)
        elif kind == "gate":
            o = g.multiply(o, g.col_broadcast(gate, o))
        elif kind == "row":
            o = getattr(g, rng.choice(["add", "multiply"]))(o, g.row_broadcast(g.tanh(rng.choice(rows)), o))
        elif kind == "tanh":
            o = g.tanh(o)
        elif kind == "center":
            mean = g.divide(g.reduce_sum(o, -1), g.constant(float(D)))
            rows.append(mean)
            o = g.subtract(o, g.row_broadcast(mean, o))
        elif kind == "const":
            o = getattr(g, rng.choice(["add", "multiply", "maximum"]))(o, g.constant(rng.choice([0.5, -0.75, 1.5])))
        else:
            mx = g.reduce_max(g.tanh(o), -1)
            rows.append(mx)
            o = g.multiply(o, g.row_broadcast(g.add(mx, g.constant(1.5)), o))
    out_dtype = rng.choice([dtype, "f32"])
    g.output(o if out_dtype == "f32" else g.convert(o, out_dtype))
    g.output(rows[-1])
    if rng.random() < 0.4 and o != dot_result:
        g.output(dot_result)
    return g.ops, params


def random_elementwise_parts(rng, n_parts=None):
    """Several independent all-elementwise computations of different shapes and dtypes in one op
    list (the kernel packing case): per part two full operands, a per-column operand broadcast in,
    a random chain of ops, one or two outputs.  Returns (ops, parameter shapes, parameter dtypes)."""
    g = Graph()
    shapes_pool = [(37, 128), (5,), (3, 7, 64), (300, 8), (33, 100), (1,), (64, 64), (2, 3, 5, 32), (129, 16), (4096,)]
    n_parts = n_parts or rng.randint(2, 6)
    pshapes, pdtypes, n_out = [], [], 0
    for k in range(n_parts):
        shape = rng.choice(shapes_pool)
        dt = rng.choice(["f32", "f32", "bf16", "f16"])
        a = g.parameter(f"a{k}", dt, shape)
        b = g.parameter(f"b{k}", dt, shape)
        c = g.parameter(f"c{k}", dt, shape[-1:])
        pshapes += [shape, shape, shape[-1:]]
        pdtypes += [dt, dt, dt]
        conv = (lambda t: t) if dt == "f32" else (lambda t: g.convert(t, "f32"))
        vals = [conv(a), conv(b)]
        cb = g.broadcast(conv(c), shape, len(shape) - 1) if len(shape) > 1 else conv(c)
        for _ in range(rng.randint(2, 8)):
            kind = rng.choice(["bin", "bin", "un", "col", "const"])
            if kind == "bin":
                vals.append(getattr(g, rng.choice(["add", "subtract", "multiply", "maximum"]))(rng.choice(vals), rng.choice(vals)))
            elif kind == "un":
                v = rng.choice(vals)
                vals.append(rng.choice([lambda: g.tanh(v), lambda: g.exp(g.tanh(v)), lambda: g.negate(v),
                                        lambda: g.rsqrt(g.add(g.multiply(v, v), g.constant(1.0)))])())
            elif kind == "col":
                vals.append(getattr(g, rng.choice(["add", "multiply"]))(rng.choice(vals), cb))
            else:
                vals.append(getattr(g, rng.choice(["add", "multiply"]))(rng.choice(vals), g.constant(rng.choice([0.5, -1.25, 2.0]))))
        outs = [vals[-1]] if len(vals) < 4 or n_out >= 14 or rng.random() < 0.5 else [vals[-1], vals[-3]]
        for o in dict.fromkeys(outs):
            if o in (vals[0], vals[1]):
                o = g.add(vals[0], vals[1])
            g.output(o if dt == "f32" else g.convert(o, dt))
            n_out += 1
    return g.ops, pshapes, pdtypes
