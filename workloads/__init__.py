"""Neutral description of the benchmark workloads: op lists and seeded inputs.

Imported by the tests and the bench only; neither the oracle nor the HIP library
depends on it.
"""
from __future__ import annotations

from . import graphs, inputs

ITEMSIZE = {"f32": 4, "f16": 2, "bf16": 2}
# comparison bar |gpu - ref| <= atol + rtol*|ref| for a group by its storage dtype
TOLERANCE = {"f32": 1e-5, "f16": 2e-2, "bf16": 2e-2}


def algorithmic_bytes(ops):
    """Bytes a group must move: every parameter read once, every output written once."""
    total = 0
    for op in ops:
        if op.kind in ("parameter", "output"):
            n = 1
            for e in op.shape:
                n *= e
            total += n * ITEMSIZE[op.dtype]
    return total


class Config:
    def __init__(self, index, name, graph_fn, input_fn, full, small, dtype):
        self.index, self.name = index, name
        self.graph_fn, self.input_fn = graph_fn, input_fn
        self.full, self.small, self.dtype = full, small, dtype

    def build(self, size="full", **override):
        kw = dict(self.full if size == "full" else self.small)
        kw.update(override)
        ops = self.graph_fn(**kw)
        ins = self.input_fn(**kw)
        return ops, ins


CONFIGS = [
    Config(1, "layernorm_fwd", graphs.layernorm_fwd, inputs.layernorm_fwd,
           dict(rows=256, cols=768), dict(rows=37, cols=768), "f32"),
    Config(2, "scaled_masked_softmax", graphs.scaled_masked_softmax,
           inputs.scaled_masked_softmax,
           dict(shape=(131072, 128), mask="full"), dict(shape=(1030, 128), mask="full"), "f32"),
    Config(3, "causal_attention", graphs.causal_attention, inputs.causal_attention,
           dict(batch=512, seq=64, dim=64), dict(batch=5, seq=64, dim=64), "f16"),
    Config(4, "bias_gelu_residual_layernorm", graphs.bias_gelu_residual_layernorm,
           inputs.bias_gelu_residual_layernorm,
           dict(rows=16384, cols=1024), dict(rows=203, cols=1024), "bf16"),
    Config(5, "layernorm_bwd", graphs.layernorm_bwd, inputs.layernorm_bwd,
           dict(rows=32768, cols=1024), dict(rows=517, cols=1024), "f32"),
]
def _log_softmax_inputs(shape, dtype="f32"):
    return inputs.normal_tensors([shape], dtype, scale=3.0)


def _rmsnorm_inputs(shape, dtype="f32"):
    return inputs.normal_tensors([shape, shape[-1:]], dtype)


def _sequence_pool_inputs(shape, levels=1, dtype="f32", with_row_work=False):
    return inputs.normal_tensors([shape], dtype, seed_offset=14)


def _ln_stats_inputs(rows, cols, dtype="f32"):
    return inputs.layernorm_fwd(rows, cols, dtype)


# Groups measured beside the five, all run by generated kernels: all-elementwise groups (the
# packing pattern of the backward phase, Section 5.1), row groups that no hand-written kernel
# matches, the stand-in for the paper's motivating example (Section 3.1) at the sizes it
# quotes, and the backward tail of a Transformer block (two row reductions, three column sums and
# two full outputs packed over the same rows), and the momentum update of a Transformer layer's eight
# parameter tensors as one group of independent parts of different shapes, and sequence pooling
# ([B, S, H] summed over S: column sums per run of rows), and two groups around dots on the matrix unit: the
# attention kernel with a key mask, gate, residual and log-sum-exp output, a dot -> logistic -> dot group
# that only the generated block-composed kernel takes, and attention with the normalisation, a residual and a
# LayerNorm after the second dot (keys stored [B, D, Sk]).  Not benchmark configs, so not in CONFIGS.
EXTRA_GROUPS = [
    Config(6, "adam_update_packed", graphs.adam_update, inputs.adam_update,
           dict(shape=(16384, 1024)), dict(shape=(129, 512)), "f32"),
    Config(7, "bias_gelu_residual", graphs.bias_gelu_residual, inputs.bias_gelu_residual,
           dict(rows=16384, cols=1024, dtype="bf16"), dict(rows=203, cols=1024, dtype="bf16"), "bf16"),
    Config(8, "log_softmax", graphs.log_softmax, _log_softmax_inputs,
           dict(shape=(131072, 128)), dict(shape=(1030, 128)), "f32"),
    Config(9, "rmsnorm", graphs.rmsnorm, _rmsnorm_inputs,
           dict(shape=(16384, 1024), dtype="bf16"), dict(shape=(203, 1024), dtype="bf16"), "bf16"),
    Config(10, "layernorm_fwd_with_stats", graphs.layernorm_fwd_with_stats, _ln_stats_inputs,
           dict(rows=16384, cols=1024), dict(rows=203, cols=1024), "f32"),
    Config(11, "multi_interest_pattern", graphs.multi_interest_pattern, inputs.multi_interest_pattern,
           dict(batch=16384, m=94, n=94, k=1), dict(batch=7, m=94, n=94, k=1), "f32"),
    Config(12, "encoder_tail_bwd", graphs.encoder_tail_bwd, inputs.encoder_tail_bwd,
           dict(rows=16384, cols=1024), dict(rows=203, cols=1024), "f32"),
    Config(13, "multi_tensor_momentum", graphs.multi_tensor_momentum, inputs.multi_tensor_momentum,
           dict(shapes=[(1024, 1024), (1024,), (1024, 1024), (1024,), (4096, 1024), (4096,), (1024,), (1024,)]),
           dict(shapes=[(33, 100), (100,), (7,), (64, 64)]), "f32"),
    Config(14, "sequence_pool", graphs.sequence_pool, _sequence_pool_inputs,
           dict(shape=(16384, 50, 128)), dict(shape=(37, 50, 128)), "f32"),
    Config(15, "attention_block", graphs.attention_block, inputs.attention_block,
           dict(batch=512, sq=64, sk=64, dim=64, dtype="f16", causal=True, mask="key", gate=True, residual=True, lse=True),
           dict(batch=3, sq=40, sk=72, dim=64, dtype="f16", causal=True, mask="key", gate=True, residual=True, lse=True), "f16"),
    Config(16, "sigmoid_attention", graphs.sigmoid_attention, inputs.sigmoid_attention,
           dict(batch=512, sq=64, sk=64, kc=64, dim=64, dtype="bf16"), dict(batch=3, sq=40, sk=72, kc=64, dim=64, dtype="bf16"), "bf16"),
    Config(17, "attention_residual_layernorm", graphs.attention_residual_layernorm, inputs.attention_residual_layernorm,
           dict(batch=512, sq=64, sk=64, dim=64, dtype="f16"), dict(batch=3, sq=40, sk=72, dim=64, dtype="f16"), "f16"),
]
BY_NAME = {c.name: c for c in CONFIGS + EXTRA_GROUPS}
