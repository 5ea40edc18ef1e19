"""ctypes binding of include/fs.h: same entry points, argument marshalling only.

Every step of the path runs in the HIP library.  PyTorch appears here only as the
owner of device memory and streams (`tensor.data_ptr()`, the current stream's
handle).  If the built library is missing, loading fails loudly: there is no CPU
or eager fallback.
"""
from __future__ import annotations

import ctypes as C
import os

FS_MAX_RANK = 4
LIB_PATH = os.environ.get("FS_LIB_PATH") or os.path.join(os.path.dirname(os.path.abspath(__file__)),
                                                        "libfusionstitch.so")

FS_OK, FS_ERR_INVALID, FS_ERR_UNSUPPORTED, FS_ERR_LDS, FS_ERR_HIP, FS_ERR_NOMEM = range(6)
STATUS_NAMES = ["FS_OK", "FS_ERR_INVALID", "FS_ERR_UNSUPPORTED", "FS_ERR_LDS", "FS_ERR_HIP", "FS_ERR_NOMEM"]
FS_MODE_STITCHED, FS_MODE_PER_OP, FS_MODE_STITCHED_PREBUILT, FS_MODE_STITCHED_GENERATED = 0, 1, 2, 3
SCHEDULE_NAMES = ["per_op", "row", "row_col", "bdot_softmax", "elementwise", "block_dot"]

DTYPES = {"f32": 0, "f16": 1, "bf16": 2}
OPKINDS = {name: i for i, name in enumerate((
    "parameter", "constant", "add", "subtract", "multiply", "divide", "maximum", "negate",
    "exp", "log", "tanh", "rsqrt", "sqrt", "convert", "broadcast", "reduce_sum", "reduce_max",
    "dot", "causal_mask", "output", "erf", "logistic"))}


class fs_op_desc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("dtype", C.c_int32), ("rank", C.c_int32), ("axis", C.c_int32),
                ("shape", C.c_int64 * FS_MAX_RANK), ("operand", C.c_int32 * 3),
                ("reserved", C.c_int32), ("attr", C.c_double)]


class fs_plan_options(C.Structure):
    _fields_ = [("mode", C.c_int32), ("wg_size", C.c_int32), ("rows_per_wave", C.c_int32),
                ("grid", C.c_int32)]


class fs_fusion_options(C.Structure):
    _fields_ = [("launch_us", C.c_double), ("max_patterns", C.c_int32), ("explore_budget", C.c_int32),
                ("seed_bytes", C.c_int64), ("bw_bytes", C.POINTER(C.c_int64)), ("bw_gbs", C.POINTER(C.c_double)),
                ("n_bw", C.c_int32), ("n_extra", C.c_int32), ("extra_sizes", C.POINTER(C.c_int32)),
                ("extra_ops", C.POINTER(C.c_int32)), ("extra_scores", C.POINTER(C.c_double))]


class FsError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"{STATUS_NAMES[status] if 0 <= status < 6 else status}: {message}")
        self.status = status
        self.message = message


_lib = None


def lib():
    """The loaded shared library (loaded on first use)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is not built: run `python -m paper_1911_11576_amd.build` "
                "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        L.fs_plan_create.argtypes = [C.POINTER(fs_op_desc), i32, C.POINTER(fs_plan_options), C.POINTER(vp)]
        L.fs_plan_create.restype = i32
        L.fs_launch.argtypes = [vp, C.POINTER(vp), i32, C.POINTER(vp), i32, vp]
        L.fs_launch.restype = i32
        L.fs_launch_static.argtypes = [vp, C.POINTER(vp), i32, C.POINTER(vp), i32, vp]
        L.fs_launch_static.restype = i32
        L.fs_destroy.argtypes = [vp]
        L.fs_destroy.restype = i32
        L.fs_last_error.argtypes = []
        L.fs_last_error.restype = C.c_char_p
        L.fs_plan_info.argtypes = [vp, C.POINTER(i32), C.POINTER(i32), C.POINTER(i64), C.POINTER(i64),
                                   C.POINTER(i64), C.POINTER(i64)]
        L.fs_plan_info.restype = i32
        L.fs_plan_describe.argtypes = [vp]
        L.fs_plan_describe.restype = C.c_char_p
        L.fs_plan_tune.argtypes = [C.POINTER(fs_op_desc), i32, C.POINTER(vp), i32, C.POINTER(vp), i32, vp, i32,
                                   C.POINTER(vp), C.POINTER(fs_plan_options), C.POINTER(C.c_double)]
        L.fs_plan_tune.restype = i32
        L.fs_stream_copy.argtypes = [vp, vp, i64, vp]
        L.fs_stream_copy.restype = i32
        L.fs_kernel_cache_dir.argtypes = [C.c_char_p]
        L.fs_kernel_cache_dir.restype = i32
        L.fs_kernel_cache_stats.argtypes = [C.POINTER(i64), C.POINTER(i64), C.POINTER(i64)]
        L.fs_kernel_cache_stats.restype = i32
        L.fs_kernel_cache_drop_memory.argtypes = []
        L.fs_kernel_cache_drop_memory.restype = i32
        L.fs_group_key.argtypes = [C.POINTER(fs_op_desc), i32, C.POINTER(C.c_uint64)]
        L.fs_group_key.restype = i32
        L.fs_tune_cache_size.argtypes = []
        L.fs_tune_cache_size.restype = i32
        L.fs_tune_cache_clear.argtypes = []
        L.fs_tune_cache_clear.restype = i32
        L.fs_tune_cache_save.argtypes = [C.c_char_p]
        L.fs_tune_cache_save.restype = i32
        L.fs_tune_cache_load.argtypes = [C.c_char_p]
        L.fs_tune_cache_load.restype = i32
        L.fs_shared_plan.argtypes = [C.POINTER(i32), C.POINTER(i64), C.POINTER(C.c_uint8), i32, C.POINTER(i64),
                                     C.POINTER(i32), C.POINTER(i64)]
        L.fs_shared_plan.restype = i32
        L.fs_fusion_create.argtypes = [C.POINTER(fs_op_desc), i32, C.POINTER(fs_fusion_options), C.POINTER(vp)]
        L.fs_fusion_create.restype = i32
        L.fs_fusion_destroy.argtypes = [vp]
        L.fs_fusion_destroy.restype = i32
        L.fs_fusion_info.argtypes = [vp, C.POINTER(i32), C.POINTER(i32), C.POINTER(C.c_double), C.POINTER(i32)]
        L.fs_fusion_info.restype = i32
        L.fs_fusion_group_size.argtypes = [vp, i32, C.POINTER(i32), C.POINTER(i32), C.POINTER(i32), C.POINTER(i32),
                                           C.POINTER(C.c_double)]
        L.fs_fusion_group_size.restype = i32
        L.fs_fusion_group.argtypes = [vp, i32, C.POINTER(fs_op_desc), C.POINTER(i32), C.POINTER(i32), C.POINTER(i32)]
        L.fs_fusion_group.restype = i32
        L.fs_fusion_pattern.argtypes = [vp, i32, C.POINTER(i32), C.POINTER(i32), i32, C.POINTER(i32), C.POINTER(i64),
                                        C.POINTER(C.c_double), C.POINTER(i32)]
        L.fs_fusion_pattern.restype = i32
        L.fs_fusion_pattern_group_size.argtypes = [vp, i32, C.POINTER(i32), C.POINTER(i32), C.POINTER(i32), C.POINTER(i32)]
        L.fs_fusion_pattern_group_size.restype = i32
        L.fs_fusion_pattern_group.argtypes = [vp, i32, C.POINTER(fs_op_desc), C.POINTER(i32), C.POINTER(i32)]
        L.fs_fusion_pattern_group.restype = i32
        _lib = L
    return _lib


def fs_last_error():
    return lib().fs_last_error().decode()


def _check(status):
    if status != FS_OK:
        raise FsError(status, fs_last_error())


def marshal_ops(ops):
    """Sequence of records with fields kind, dtype, shape, operands, axis, attr ->
    a C array of fs_op_desc."""
    arr = (fs_op_desc * len(ops))()
    for d, op in zip(arr, ops):
        d.kind = OPKINDS[op.kind]
        d.dtype = DTYPES[op.dtype]
        d.rank = len(op.shape)
        d.axis = op.axis if op.axis >= 0 else 0
        for k in range(FS_MAX_RANK):
            d.shape[k] = op.shape[k] if k < len(op.shape) else 0
        for k in range(3):
            d.operand[k] = op.operands[k] if k < len(op.operands) else -1
        d.reserved = 0
        d.attr = op.attr
    return arr


def fs_plan_create(ops, mode=FS_MODE_STITCHED, wg_size=0, rows_per_wave=0, grid=0):
    """-> opaque plan handle (int).  `ops` may be a marshalled array or op records."""
    arr = ops if isinstance(ops, C.Array) else marshal_ops(ops)
    opt = fs_plan_options(mode, wg_size, rows_per_wave, grid)
    out = C.c_void_p()
    _check(lib().fs_plan_create(arr, len(arr), C.byref(opt), C.byref(out)))
    return out.value


def _pointers(tensors):
    arr = (C.c_void_p * max(1, len(tensors)))()
    for i, t in enumerate(tensors):
        arr[i] = t if isinstance(t, int) else t.data_ptr()
    return arr


def fs_launch(plan, inputs, outputs, stream=None):
    """inputs/outputs: device tensors (anything with .data_ptr()) or raw addresses.
    stream: a hipStream_t address; None = torch's current stream."""
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    _check(lib().fs_launch(plan, _pointers(inputs), len(inputs), _pointers(outputs), len(outputs), stream))


def fs_launch_static(plan, inputs, outputs, stream=None):
    """fs_launch without any allocation: the plan's scratch memory is the library's static device array."""
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    _check(lib().fs_launch_static(plan, _pointers(inputs), len(inputs), _pointers(outputs), len(outputs), stream))


def fs_plan_tune(ops, inputs, outputs, stream=None, trials=20):
    """-> (plan handle, winning options as a dict, microseconds per launch)."""
    arr = ops if isinstance(ops, C.Array) else marshal_ops(ops)
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    out, opt, us = C.c_void_p(), fs_plan_options(), C.c_double()
    _check(lib().fs_plan_tune(arr, len(arr), _pointers(inputs), len(inputs), _pointers(outputs), len(outputs),
                              stream, trials, C.byref(out), C.byref(opt), C.byref(us)))
    return out.value, {"wg_size": opt.wg_size, "rows_per_wave": opt.rows_per_wave, "grid": opt.grid}, us.value


def fs_destroy(plan):
    _check(lib().fs_destroy(plan))


def fs_plan_info(plan):
    sched, nk = C.c_int32(), C.c_int32()
    lds, ws, algo, moved = C.c_int64(), C.c_int64(), C.c_int64(), C.c_int64()
    _check(lib().fs_plan_info(plan, C.byref(sched), C.byref(nk), C.byref(lds), C.byref(ws),
                              C.byref(algo), C.byref(moved)))
    return {"schedule": SCHEDULE_NAMES[sched.value], "n_kernels": nk.value, "lds_bytes": lds.value,
            "workspace_bytes": ws.value, "algorithmic_bytes": algo.value, "moved_bytes": moved.value}


def fs_plan_describe(plan):
    return lib().fs_plan_describe(plan).decode()


def fs_shared_plan(operands, req_bytes, is_output=None):
    """Algorithm 4 on a DAG given as per-op operand lists (indices of earlier ops) and shared-
    space requests in bytes.  -> (offsets, shares_with, total_bytes)."""
    n = len(operands)
    ops = (C.c_int32 * (3 * max(n, 1)))(*([-1] * (3 * max(n, 1))))
    for i, lst in enumerate(operands):
        assert len(lst) <= 3
        for j, o in enumerate(lst):
            ops[3 * i + j] = o
    req = (C.c_int64 * max(n, 1))(*req_bytes) if n else (C.c_int64 * 1)()
    outs = None if is_output is None else (C.c_uint8 * max(n, 1))(*[1 if b else 0 for b in is_output])
    off = (C.c_int64 * max(n, 1))()
    shr = (C.c_int32 * max(n, 1))()
    total = C.c_int64(0)
    _check(lib().fs_shared_plan(ops, req, outs, n, off, shr, C.byref(total)))
    return list(off[:n]), list(shr[:n]), total.value


def fs_kernel_cache_dir(path):
    """Directory for compiled kernels shared between processes (None turns it off)."""
    _check(lib().fs_kernel_cache_dir(None if path is None else str(path).encode()))


def fs_kernel_cache_stats():
    """-> dict(compiled, from_memory, from_disk): where generated kernels came from so far."""
    c, m, d = C.c_int64(), C.c_int64(), C.c_int64()
    _check(lib().fs_kernel_cache_stats(C.byref(c), C.byref(m), C.byref(d)))
    return {"compiled": c.value, "from_memory": m.value, "from_disk": d.value}


def fs_kernel_cache_drop_memory():
    _check(lib().fs_kernel_cache_drop_memory())


def fs_group_key(ops):
    """Key of a group in the tuning cache (an int)."""
    arr = ops if isinstance(ops, C.Array) else marshal_ops(ops)
    key = C.c_uint64()
    _check(lib().fs_group_key(arr, len(arr), C.byref(key)))
    return key.value


def fs_tune_cache_size():
    return lib().fs_tune_cache_size()


def fs_tune_cache_clear():
    _check(lib().fs_tune_cache_clear())


def fs_tune_cache_save(path):
    _check(lib().fs_tune_cache_save(str(path).encode()))


def fs_tune_cache_load(path):
    _check(lib().fs_tune_cache_load(str(path).encode()))


def fs_stream_copy(dst, src, nbytes, stream=None):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    _check(lib().fs_stream_copy(dst if isinstance(dst, int) else dst.data_ptr(),
                                src if isinstance(src, int) else src.data_ptr(), nbytes, stream))


class BoundArgs:
    """Pointer arrays of one (inputs, outputs) set, marshalled once so that repeated
    launches of the same buffers cost a single foreign call.  Keeps the tensors alive."""

    def __init__(self, inputs, outputs):
        self.keep = (list(inputs), list(outputs))
        self.n_in, self.n_out = len(inputs), len(outputs)
        self.in_ptrs, self.out_ptrs = _pointers(inputs), _pointers(outputs)


class Plan:
    """Owner of one fs_plan handle."""

    def __init__(self, ops, mode="stitched", wg_size=0, rows_per_wave=0, grid=0, _handle=None):
        self._h = _handle
        if _handle is None:
            m = {"stitched": FS_MODE_STITCHED, "per_op": FS_MODE_PER_OP, "prebuilt": FS_MODE_STITCHED_PREBUILT,
                 "generated": FS_MODE_STITCHED_GENERATED}[mode]
            self._h = fs_plan_create(ops, m, wg_size, rows_per_wave, grid)
        self.tuned = None

    @classmethod
    def tune(cls, ops, inputs, outputs, stream=None, trials=20):
        """The fastest of the schedule's launch templates for these buffers (fs_plan_tune)."""
        h, opts, us = fs_plan_tune(ops, inputs, outputs, stream, trials)
        plan = cls(ops, _handle=h)
        plan.tuned = dict(opts, us=us)
        return plan

    def launch(self, inputs, outputs, stream=None):
        fs_launch(self._h, inputs, outputs, stream)

    def launch_static(self, inputs, outputs, stream=None):
        fs_launch_static(self._h, inputs, outputs, stream)

    def launch_bound(self, bound, stream):
        """Launch with pre-marshalled arguments (see BoundArgs) on an explicit stream handle."""
        st = lib().fs_launch(self._h, bound.in_ptrs, bound.n_in, bound.out_ptrs, bound.n_out, stream)
        if st != FS_OK:
            raise FsError(st, fs_last_error())

    def info(self):
        return fs_plan_info(self._h)

    def describe(self):
        return fs_plan_describe(self._h)

    def close(self):
        if self._h is not None:
            h, self._h = self._h, None
            fs_destroy(h)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()


# ---------------------------------------------------------------- fusion planning (Section 4)

_KIND_NAMES = {v: k for k, v in OPKINDS.items()}
_DTYPE_NAMES = {v: k for k, v in DTYPES.items()}


class FusionPlan:
    """fs_fusion_create on a computation graph (op records as for Plan).

    .groups     list of dicts in execution order: ops (marshalled fs_op_desc array, ready for
                fs_plan_create), input_of / output_of (indices into the original list), members
                (the original ops it fuses), score_us
    .patterns   every scored candidate: ops, origin, saved_bytes, score_us, chosen, measured, and (where a
                stitched plan exists for it) group_ops / input_of / output_of like a group's

    extra_scores: per extra pattern the microseconds it was measured to save (None or NaN: the model's score).
    """

    def __init__(self, ops, launch_us=0.0, max_patterns=0, explore_budget=0, seed_bytes=0, bandwidth=None, extra_patterns=None,
                 extra_scores=None):
        arr = ops if isinstance(ops, C.Array) else marshal_ops(ops)
        opt = fs_fusion_options()
        opt.launch_us, opt.max_patterns, opt.explore_budget, opt.seed_bytes = launch_us, max_patterns, explore_budget, seed_bytes
        keep = None
        if bandwidth:
            bb = (C.c_int64 * len(bandwidth))(*[int(b) for b, _ in bandwidth])
            gg = (C.c_double * len(bandwidth))(*[float(g) for _, g in bandwidth])
            opt.bw_bytes, opt.bw_gbs, opt.n_bw = bb, gg, len(bandwidth)
            keep = (bb, gg)
        keep2 = None
        if extra_patterns:
            sizes = (C.c_int32 * len(extra_patterns))(*[len(p) for p in extra_patterns])
            flat = [o for p in extra_patterns for o in p]
            eo = (C.c_int32 * len(flat))(*flat)
            opt.n_extra, opt.extra_sizes, opt.extra_ops = len(extra_patterns), sizes, eo
            keep2 = (sizes, eo)
            if extra_scores is not None:
                if len(extra_scores) != len(extra_patterns):
                    raise ValueError("extra_scores: one entry per extra pattern")
                es = (C.c_double * len(extra_scores))(*[float("nan") if v is None else float(v) for v in extra_scores])
                opt.extra_scores = es
                keep2 = (sizes, eo, es)
        h = C.c_void_p()
        _check(lib().fs_fusion_create(arr, len(arr), C.byref(opt), C.byref(h)))
        del keep, keep2
        try:
            ng, npat, total, rounds = C.c_int32(), C.c_int32(), C.c_double(), C.c_int32()
            _check(lib().fs_fusion_info(h, C.byref(ng), C.byref(npat), C.byref(total), C.byref(rounds)))
            self.total_score_us, self.solver_rounds = total.value, rounds.value
            self.groups, self.patterns = [], []
            for g in range(ng.value):
                n_ops, n_in, n_out, n_mem, score = C.c_int32(), C.c_int32(), C.c_int32(), C.c_int32(), C.c_double()
                _check(lib().fs_fusion_group_size(h, g, C.byref(n_ops), C.byref(n_in), C.byref(n_out), C.byref(n_mem), C.byref(score)))
                gops = (fs_op_desc * max(1, n_ops.value))()
                gin, gout = (C.c_int32 * max(1, n_in.value))(), (C.c_int32 * max(1, n_out.value))()
                gmem = (C.c_int32 * max(1, n_mem.value))()
                _check(lib().fs_fusion_group(h, g, gops, gin, gout, gmem))
                trimmed = (fs_op_desc * n_ops.value)(*gops[:n_ops.value])
                self.groups.append(dict(ops=trimmed, input_of=list(gin[:n_in.value]), output_of=list(gout[:n_out.value]),
                                        members=list(gmem[:n_mem.value]), score_us=score.value))
            for k in range(npat.value):
                n_ops, origin, saved, score, chosen = C.c_int32(), C.c_int32(), C.c_int64(), C.c_double(), C.c_int32()
                _check(lib().fs_fusion_pattern(h, k, C.byref(n_ops), None, 0, None, None, None, None))      # its size first
                buf = (C.c_int32 * max(1, n_ops.value))()
                _check(lib().fs_fusion_pattern(h, k, C.byref(n_ops), buf, n_ops.value, C.byref(origin), C.byref(saved), C.byref(score), C.byref(chosen)))
                pat = dict(ops=list(buf[:n_ops.value]), n_ops=n_ops.value, origin=origin.value,
                           saved_bytes=saved.value, score_us=score.value, chosen=bool(chosen.value))
                l_ops, l_in, l_out, measured = C.c_int32(), C.c_int32(), C.c_int32(), C.c_int32()
                _check(lib().fs_fusion_pattern_group_size(h, k, C.byref(l_ops), C.byref(l_in), C.byref(l_out), C.byref(measured)))
                pat["measured"] = bool(measured.value)
                if l_ops.value:
                    gops = (fs_op_desc * l_ops.value)()
                    gin, gout = (C.c_int32 * max(1, l_in.value))(), (C.c_int32 * max(1, l_out.value))()
                    _check(lib().fs_fusion_pattern_group(h, k, gops, gin, gout))
                    pat.update(group_ops=gops, input_of=list(gin[:l_in.value]), output_of=list(gout[:l_out.value]))
                self.patterns.append(pat)
        finally:
            lib().fs_fusion_destroy(h)


def describe_group_ops(arr):
    """The ops of a marshalled list as (kind, dtype, shape, operands) tuples, for logs and tests."""
    out = []
    for d in arr:
        nop = 0 if d.kind in (OPKINDS["parameter"], OPKINDS["constant"]) else 2 if (2 <= d.kind <= 6 or d.kind == OPKINDS["dot"]) else 1
        out.append((_KIND_NAMES[d.kind], _DTYPE_NAMES[d.dtype], tuple(d.shape[:d.rank]), tuple(d.operand[:nop])))
    return out


class FusedProgram:
    """A whole computation graph run as the groups its fusion plan chose: one Plan per group,
    intermediates between groups in device tensors.  Inputs: one tensor per parameter op of the
    original list, in order; outputs: one per output op."""

    def __init__(self, ops, fusion=None, **fusion_options):
        import torch
        self._torch = torch
        self.ops = list(ops)
        self.fusion = fusion if fusion is not None else FusionPlan(self.ops, **fusion_options)
        self.param_ops = [i for i, op in enumerate(self.ops) if op.kind == "parameter"]
        self.output_ops = [i for i, op in enumerate(self.ops) if op.kind == "output"]
        self.plans = []
        for g in self.fusion.groups:
            try:
                plan = Plan(g["ops"])
            except FsError as e:
                if e.status != FS_ERR_UNSUPPORTED:
                    raise
                plan = Plan(g["ops"], "per_op")       # an op left alone that no stitched schedule takes (a lone dot)
            self.plans.append(plan)
        self.n_kernels = sum(p.info()["n_kernels"] for p in self.plans)

    def run(self, inputs, stream=None):
        torch = self._torch
        dt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
        values = {i: t for i, t in zip(self.param_ops, inputs)}
        for g, plan in zip(self.fusion.groups, self.plans):
            gin = [values[i] for i in g["input_of"]]
            gout = []
            for i in g["output_of"]:
                op = self.ops[i]
                t = torch.empty(op.shape, dtype=dt[op.dtype], device=gin[0].device if gin else "cuda:0")
                values[i] = t
                gout.append(t)
            plan.launch(gin, gout, stream)
        return [values[self.ops[i].operands[0]] for i in self.output_ops]

    @classmethod
    def best_of(cls, ops, inputs, option_sets=None, trials=20):
        """The execution-based side of Section 4.3 at the level of whole plans: build the program under
        each set of planning options, time it on the given inputs (HIP events, `trials` runs after two
        warm-ups), keep the fastest.  -> (program, microseconds per run, the winning options)."""
        import torch
        if option_sets is None:
            option_sets = [dict(), dict(explore_budget=-1), dict(seed_bytes=1), dict(launch_us=10.0), dict(launch_us=0.5)]
        best = None
        for kw in option_sets:
            prog = cls(ops, **kw)
            prog.bind(inputs)
            for _ in range(2):
                prog.run_bound()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(trials):
                prog.run_bound()
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / trials
            if best is None or us < best[1]:
                if best is not None:
                    best[0].close()
                best = (prog, us, dict(kw))
            else:
                prog.close()
        return best

    @classmethod
    def measured(cls, ops, top=12, trials=20, device="cuda:0", **fusion_options):
        """The hybrid scoring policy of Section 4.3.  Plan with the model's scores; build the plan's
        patterns and the `top` best other candidates, time each stitched and as one kernel per op on
        buffers of the right shapes, and plan again with the measured savings in place of the model's
        for those patterns.  -> (program, list of (pattern ops, model score, measured score))."""
        import torch
        ops = list(ops)
        dt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
        first = FusionPlan(ops, **fusion_options)
        ranked = sorted((p for p in first.patterns if p["score_us"] >= 0 and "group_ops" in p),
                        key=lambda p: (not p["chosen"], -p["score_us"]))
        n_chosen = sum(1 for p in ranked if p["chosen"])
        picked = ranked[:n_chosen + top]

        def timed(plan, gin, gout):
            for _ in range(2):
                plan.launch(gin, gout)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(trials):
                plan.launch(gin, gout)
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e3 / trials

        report = []
        for p in picked:
            shapes = [(ops[i].shape, ops[i].dtype) for i in p["input_of"]]
            gin = [torch.randn(sh, dtype=torch.float32, device=device).to(dt[d]) for sh, d in shapes]
            gout = [torch.empty(ops[i].shape, dtype=dt[ops[i].dtype], device=device) for i in p["output_of"]]
            with Plan(p["group_ops"]) as fused, Plan(p["group_ops"], "per_op") as apart:
                saved = timed(apart, gin, gout) - timed(fused, gin, gout)
            report.append((p["ops"], p["score_us"], saved))
        kw = dict(fusion_options)
        extra = list(kw.pop("extra_patterns", None) or [])
        scores = list(kw.pop("extra_scores", None) or [None] * len(extra))
        second = FusionPlan(ops, extra_patterns=extra + [r[0] for r in report], extra_scores=scores + [r[2] for r in report], **kw)
        return cls(ops, fusion=second), report

    def tune(self, inputs, trials=10):
        """Time every group's launch templates on the program's own data (fs_plan_tune, group by group in
        execution order) and keep the winners.  -> the program's outputs, as run() would return them."""
        torch = self._torch
        dt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
        values = {i: t for i, t in zip(self.param_ops, inputs)}
        for k, g in enumerate(self.fusion.groups):
            gin = [values[i] for i in g["input_of"]]
            gout = []
            for i in g["output_of"]:
                op = self.ops[i]
                values[i] = torch.empty(op.shape, dtype=dt[op.dtype], device=gin[0].device if gin else "cuda:0")
                gout.append(values[i])
            if self.plans[k].info()["schedule"] == "per_op":
                self.plans[k].launch(gin, gout)
                continue
            tuned = Plan.tune(g["ops"], gin, gout, trials=trials)      # leaves the group's outputs written
            self.plans[k].close()
            self.plans[k] = tuned
        self.n_kernels = sum(p.info()["n_kernels"] for p in self.plans)
        return [values[self.ops[i].operands[0]] for i in self.output_ops]

    def bind(self, inputs):
        """Fix the program's buffers: the given input tensors, and one freshly allocated tensor per value
        that crosses a group boundary.  -> the output tensors; run_bound() then launches every group on
        those buffers without allocating, which is what a HIP graph capture needs."""
        torch = self._torch
        dt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
        values = {i: t for i, t in zip(self.param_ops, inputs)}
        device = inputs[0].device if inputs else "cuda:0"
        self._bound = []
        for g, plan in zip(self.fusion.groups, self.plans):
            gin = [values[i] for i in g["input_of"]]
            gout = []
            for i in g["output_of"]:
                op = self.ops[i]
                values[i] = torch.empty(op.shape, dtype=dt[op.dtype], device=device)
                gout.append(values[i])
            self._bound.append((plan, BoundArgs(gin, gout)))
        self._bound_outputs = [values[self.ops[i].operands[0]] for i in self.output_ops]
        return self._bound_outputs

    def run_bound(self, stream=None):
        if stream is None:
            stream = self._torch.cuda.current_stream().cuda_stream
        for plan, args in self._bound:
            plan.launch_bound(args, stream)
        return self._bound_outputs

    def capture(self, inputs):
        """bind(inputs), one ordinary run (kernels loaded, workspaces allocated), then the same launches
        recorded into a HIP graph.  -> (graph, outputs): graph.replay() recomputes the outputs from whatever
        the input tensors hold then."""
        torch = self._torch
        outs = self.bind(inputs)
        self.run_bound()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=torch.cuda.Stream()):
            self.run_bound()
        return graph, outs

    def close(self):
        for p in self.plans:
            p.close()
        self.plans = []
        self._bound = []

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()
