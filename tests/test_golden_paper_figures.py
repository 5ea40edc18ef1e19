"""The figures the paper prints for its motivating example (Section 3.1) and for its shared-memory
example (Section 5.4), kept as a text fixture, against the stand-in workload and the oracles: the
workload has the op and output counts and the tensor sizes the text gives, and the shared-memory
oracle arrives at the one tile the text arrives at."""
import os

import numpy as np

from oracle import interp, shared_memory as osm
from workloads import graphs, inputs

HERE = os.path.dirname(os.path.abspath(__file__))


def _figures():
    out = {}
    with open(os.path.join(HERE, "golden", "paper_figures.txt")) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if line:
                name, value = (t.strip() for t in line.split("=", 1))
                out[name] = int(value)
    return out


ELEMENTWISE = ("add", "subtract", "multiply", "divide", "maximum", "negate", "exp", "log", "tanh", "rsqrt", "sqrt", "erf", "logistic")


def test_motivating_pattern_has_the_papers_counts_and_sizes():
    fig = _figures()
    ops = graphs.multi_interest_pattern(16384)
    kinds = [op.kind for op in ops]
    assert sum(k in ELEMENTWISE for k in kinds) == fig["motivating.elementwise_ops"]
    assert sum(k in ("reduce_sum", "reduce_max") for k in kinds) == fig["motivating.reductions"]
    assert kinds.count("dot") == fig["motivating.batched_gemms"]
    assert kinds.count("output") == fig["motivating.outputs"]
    dot_1 = next(op for op in ops if op.kind == "dot")
    assert dot_1.shape[1:] == (fig["shared.tile_rows"], fig["shared.tile_cols"])
    result_bytes = int(np.prod(dot_1.shape)) * fig["shared.bytes_per_element"]
    assert round(result_bytes / 2 ** 20) == fig["motivating.dot_1_result_MB"]
    input_bytes = sum(int(np.prod(ops[i].shape)) * 4 for i in dot_1.operands)
    assert round(input_bytes / 1e6) == fig["motivating.dot_1_inputs_MB"]


def test_motivating_pattern_outputs_are_the_named_ops():
    """divide, a log-derived value, a multiply and subtract are the four outputs; the oracle runs the
    pattern on a small batch and the softmax-like part behaves like one (rows of `divide` sum to 1)."""
    ops = graphs.multi_interest_pattern(3)
    out_kinds = [ops[op.operands[0]].kind for op in ops if op.kind == "output"]
    assert sorted(out_kinds) == ["add", "divide", "multiply", "subtract"]     # log_1 = log(...) + max
    outs = interp.run(ops, inputs.multi_interest_pattern(3))
    divide = outs[out_kinds.index("divide")]
    assert np.allclose(divide.sum(axis=-1), 1.0, atol=1e-12)


def test_shared_memory_example_needs_one_tile():
    fig = _figures()
    tile = fig["shared.tile_rows"] * fig["shared.tile_cols"] * fig["shared.bytes_per_element"]
    # x, y, dot_1(x, y), bias, add(dot_1, bias), reduce(add), subtract(add, reduce)
    operands = [[], [], [0, 1], [], [2, 3], [4], [4, 5]]
    req = [0, 0, tile, 0, tile, 0, 0]
    offset, shares, total = osm.plan(operands, req)
    assert total == fig["shared.tiles_after_sharing"] * tile
    assert shares[4] == 2 and offset[4] == offset[2]
