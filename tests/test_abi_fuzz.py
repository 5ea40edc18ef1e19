"""Descriptor fuzzing of the host entry points: op lists of the benchmark groups with fields mutated
at random (kinds, dtypes, ranks, extents, wiring, attributes, options, counts).  Every call must
answer with a status and, on failure, a message -- never crash, never hand out a plan it reports
as failed.  Seeded; runs on the CPU."""
import ctypes as C
import random

from paper_1911_11576_amd import binding
from paper_1911_11576_amd.binding import fs_fusion_options, fs_plan_options, lib, marshal_ops
from workloads import graphs


def _bases():
    return [graphs.layernorm_fwd(8, 64), graphs.scaled_masked_softmax((2, 2, 8, 16), 0.125, "key_padding"),
            graphs.layernorm_bwd(8, 64), graphs.causal_attention(2, 16, 32), graphs.adam_update((8, 16)),
            graphs.multi_interest_pattern(2, 6, 6, 1), graphs.bias_gelu_bwd(8, 32), graphs.multi_tensor_momentum([(4, 8), (5,)]),
            graphs.sequence_pool((3, 5, 16), 1, "f32", True, "both"), graphs.sequence_pool((2, 3, 4, 8), 2, "bf16"),
            graphs.norm_over_trailing_dims((4, 3, 8)), graphs.max_abs_over_trailing_dims((2, 3, 4, 8), 3, "f16"),
            graphs.clip_by_global_norm([(4, 8), (5,)], 1.0), _dots_with_an_epilogue()]


def _dots_with_an_epilogue():
    """dot -> exp -> row sum -> dot -> division by the row sum -> gate -> residual: the generated block-composed form
    with ops after its second dot."""
    g = graphs.Graph()
    q = g.parameter("q", "f16", (2, 16, 32)); k = g.parameter("k", "f16", (2, 24, 32)); v = g.parameter("v", "f16", (2, 24, 32))
    res = g.parameter("res", "f16", (2, 16, 32)); gate = g.parameter("gate", "f32", (32,))
    e = g.exp(g.dot(q, k, transpose_b=True, dtype="f32"))
    den = g.reduce_sum(e, -1)
    o = g.dot(g.convert(e, "f16"), v, dtype="f32")
    o = g.add(g.multiply(g.divide(o, g.row_broadcast(den, o)), g.col_broadcast(gate, o)), g.convert(res, "f32"))
    g.output(g.convert(o, "f16"))
    return g.ops


def _mutate(rng, arr):
    n = len(arr)
    for _ in range(rng.randint(1, 3)):
        d = arr[rng.randrange(n)]
        f = rng.choice(["kind", "dtype", "rank", "axis", "shape", "operand", "attr", "reserved"])
        if f == "kind":
            d.kind = rng.choice([-1, 0, 1, 5, 14, 15, 17, 18, 19, 20, 99, 2**31 - 1])
        elif f == "dtype":
            d.dtype = rng.choice([-1, 0, 1, 2, 3, 77])
        elif f == "rank":
            d.rank = rng.choice([-1, 0, 1, 2, 3, 4, 5, 100])
        elif f == "axis":
            d.axis = rng.choice([-5, -1, 0, 1, 2, 3, 4, 9])
        elif f == "shape":
            d.shape[rng.randrange(4)] = rng.choice([-1, 0, 1, 2, 7, 64, 2**20, 2**40, 2**62])
        elif f == "operand":
            d.operand[rng.randrange(3)] = rng.choice([-2, -1, 0, 1, n - 1, n, n + 5, 2**30])
        elif f == "attr":
            d.attr = rng.choice([0.0, float("nan"), float("inf"), -1e30])
        else:
            d.reserved = rng.choice([0, 1])


def test_mutated_op_lists_never_crash_plan_creation():
    rng = random.Random(20191111)
    bases = _bases()
    seen = {}
    for _ in range(1500):
        arr = marshal_ops(rng.choice(bases))
        n = len(arr)
        _mutate(rng, arr)
        # mostly without run-time compilation (fast); some in the default and the per-op mode
        opt = fs_plan_options(rng.choice([2, 2, 2, 2, 1, 0]), rng.choice([0, 0, 64, 100, 256, 4096, -1]),
                              rng.choice([0, 0, 1, 3, 64, -2]), rng.choice([0, 0, 1, 7, 2**30, -1]))
        count = rng.choice([n, n - 1, 1, 0, -1]) if rng.random() < 0.1 else n
        out = C.c_void_p()
        st = lib().fs_plan_create(arr, count, C.byref(opt), C.byref(out))
        seen[st] = seen.get(st, 0) + 1
        if st == binding.FS_OK:
            assert out.value and lib().fs_plan_describe(out)
            assert lib().fs_destroy(out) == binding.FS_OK
        else:
            assert not out.value and binding.fs_last_error()
            assert st in (binding.FS_ERR_INVALID, binding.FS_ERR_UNSUPPORTED, binding.FS_ERR_LDS)
    assert seen.get(binding.FS_OK, 0) > 20 and seen.get(binding.FS_ERR_INVALID, 0) > 500       # the mutations bite, and not always


def test_mutated_op_lists_never_crash_the_fusion_planner():
    rng = random.Random(4)
    bases = _bases()
    ok = 0
    for _ in range(300):
        arr = marshal_ops(rng.choice(bases))
        _mutate(rng, arr)
        opt = fs_fusion_options()
        opt.launch_us = rng.choice([0.0, 2.5, -1.0, float("nan")])
        opt.max_patterns = rng.choice([0, 0, 4, 256, 1000, -3])
        opt.explore_budget = rng.choice([0, -1, 5, 10**6])
        # caller-supplied patterns (valid or not) with measured scores of every kind
        keep = None
        if rng.random() < 0.5:
            n_extra = rng.randint(1, 3)
            sizes = [rng.randint(1, 5) for _ in range(n_extra)]
            flat = [rng.randint(-1, len(arr) + 1) for _ in range(sum(sizes))]
            scores = [rng.choice([float("nan"), float("inf"), -float("inf"), -3.0, 0.0, 7.5, 1e300]) for _ in range(n_extra)]
            keep = ((C.c_int32 * n_extra)(*sizes), (C.c_int32 * len(flat))(*flat), (C.c_double * n_extra)(*scores))
            opt.n_extra, opt.extra_sizes, opt.extra_ops = n_extra, keep[0], keep[1]
            if rng.random() < 0.7:
                opt.extra_scores = keep[2]
        out = C.c_void_p()
        st = lib().fs_fusion_create(arr, len(arr), C.byref(opt), C.byref(out))
        if st == binding.FS_OK:
            ok += 1
            n_groups, n_pat = C.c_int32(), C.c_int32()
            assert lib().fs_fusion_info(out, C.byref(n_groups), C.byref(n_pat), None, None) == binding.FS_OK and n_groups.value >= 1
            for k in range(-1, n_pat.value + 1):        # every candidate as an op list, and both ends past the range
                a, b, c, m = C.c_int32(), C.c_int32(), C.c_int32(), C.c_int32()
                st2 = lib().fs_fusion_pattern_group_size(out, k, C.byref(a), C.byref(b), C.byref(c), C.byref(m))
                assert (st2 == binding.FS_OK) == (0 <= k < n_pat.value)
                if st2 == binding.FS_OK and a.value:
                    gops = (binding.fs_op_desc * a.value)()
                    assert lib().fs_fusion_pattern_group(out, k, gops, None, None) == binding.FS_OK
            assert lib().fs_fusion_destroy(out) == binding.FS_OK
        else:
            assert not out.value and binding.fs_last_error()
    assert ok > 5


def test_extents_whose_product_wraps_are_refused():
    """Two (or more) extents that are each below 2^40 but whose product is not, up to products that wrap a
    64-bit integer to 0 or to something small: FS_ERR_INVALID, never an "empty" or a small tensor."""
    for shape in ([2**32, 2**32, 1, 1], [2**32, 2**32, 2**32, 2**32], [2**33, 2**31 + 1, 2, 1], [2**21, 2**21, 2**21, 2],
                  [2**39, 4, 1, 1], [3, 2**39, 1, 1]):
        for kind in ("parameter", "add"):
            ops = graphs.adam_update((8, 16))
            arr = marshal_ops(ops)
            target = next(i for i, op in enumerate(ops) if op.kind == kind)
            arr[target].rank = 4
            for k in range(4):
                arr[target].shape[k] = shape[k]
            out = C.c_void_p()
            st = lib().fs_plan_create(arr, len(arr), None, C.byref(out))
            assert st == binding.FS_ERR_INVALID and not out.value, (shape, kind, st)
            assert "too large" in binding.fs_last_error() or "shape" in binding.fs_last_error()
    # a zero extent still makes a legal, empty tensor whatever the other extents are
    ops = graphs.layernorm_fwd(0, 64)
    with binding.Plan(ops) as p:
        assert p.info()["algorithmic_bytes"] == 2 * 64 * 4
