"""Shared-memory optimisation (Algorithm 4, Section 5.4): the oracle against the paper's own
example and the definition of dominance, and the library's planner against the oracle."""
import random

import pytest

from oracle import shared_memory as osm
from paper_1911_11576_amd import FsError, binding, fs_shared_plan

TILE = 94 * 94 * 4      # the shared space the paper's example quotes for dot_1 and for add


def paper_example():
    """The part of the motivating example the paper's text fixes (Section 5.4): dot_1 and add
    each need 94*94*4 bytes of shared space, and add can reuse dot_1's.  Ops: 0 x, 1 y,
    2 dot_1(x, y), 3 bias, 4 add(dot_1, bias), 5 reduce(add), 6 subtract(add, reduce)."""
    operands = [[], [], [0, 1], [], [2, 3], [4], [4, 5]]
    req = [0, 0, TILE, 0, TILE, 0, 0]
    return operands, req


def test_oracle_reproduces_the_papers_example():
    operands, req = paper_example()
    offset, shares, total = osm.plan(operands, req)
    assert shares[4] == 2                   # add takes over dot_1's space
    assert offset[4] == offset[2] == 0
    assert total == TILE                    # one tile instead of two
    assert osm.valid_sharing(operands, req, offset)


def test_oracle_dominance_is_the_definition_on_hand_checked_graphs():
    # diamond: 0 -> 1, 0 -> 2, (1, 2) -> 3; root uses 3
    operands = [[], [0], [0], [1, 2]]
    dom = osm.dominators(operands)
    assert dom[3][0] and dom[3][1] and dom[3][2]
    assert not dom[1][0] and not dom[2][0]          # 0 is reached around either branch
    # a second output that reads 0 directly: 3 no longer dominates 0
    dom = osm.dominators(operands, is_output=[True, False, False, True])
    assert not dom[3][0] and dom[3][1]
    # chain: every later op dominates every earlier one
    chain = [[], [0], [1], [2]]
    dom = osm.dominators(chain)
    assert all(dom[a][b] for a in range(4) for b in range(a))
    assert not any(dom[b][a] for a in range(4) for b in range(a))
    # dead op (no path from the root): nothing dominates it, it dominates nothing reachable
    dom = osm.dominators([[], [0], [0]], is_output=[False, True, False])
    assert not any(dom[a][2] for a in range(3)) and not dom[2][0]


def test_oracle_does_not_share_what_is_still_needed():
    # 0 needs space and is read by 1 (needs space) and later by 2: 1 must not take 0's space
    operands = [[], [0], [0, 1]]
    req = [100, 100, 0]
    offset, shares, total = osm.plan(operands, req)
    assert shares[1] == -1 and offset[1] != offset[0] and total == 200
    assert osm.valid_sharing(operands, req, offset)
    # without the late read, it does
    operands = [[], [0], [1]]
    offset, shares, total = osm.plan(operands, [100, 100, 0])
    assert shares[1] == 0 and total == 100
    # the checker itself: overlapping live values are reported
    assert not osm.valid_sharing([[], [0], [0, 1]], [100, 100, 0], [0, 0, -1])
    # a smaller space is not shared by a larger request, but is reclaimed for a later small one
    operands = [[], [0], [1], [2]]
    offset, shares, total = osm.plan(operands, [50, 100, 0, 40])
    assert shares[1] == -1 and total == 150 and offset[3] in (0, 50)


def _random_dag(rng, n):
    operands = []
    for i in range(n):
        k = 0 if i == 0 else rng.choice([0, 1, 1, 2, 2, 3])
        operands.append(sorted(rng.sample(range(i), min(k, i))))
    req = [rng.choice([0, 0, 64, 128, 256]) for _ in range(n)]
    return operands, req


@pytest.mark.parametrize("seed", range(40))
def test_oracle_plans_are_valid_on_random_graphs(seed):
    rng = random.Random(seed)
    operands, req = _random_dag(rng, rng.randint(2, 24))
    offset, shares, total = osm.plan(operands, req)
    assert osm.valid_sharing(operands, req, offset)
    assert total <= sum(r for r in req if r > 0)
    for i, r in enumerate(req):
        assert (offset[i] >= 0) == (r > 0)
        if offset[i] >= 0:
            assert offset[i] + r <= total


# ---------------------------------------------------------------- the library's planner

def test_library_planner_on_the_papers_example():
    operands, req = paper_example()
    offset, shares, total = fs_shared_plan(operands, req)
    assert total == TILE and shares[4] == 2 and offset[2] == offset[4] == 0
    assert offset[0] == offset[5] == -1


@pytest.mark.parametrize("seed", range(60))
def test_library_planner_matches_the_oracle(seed):
    rng = random.Random(1000 + seed)
    operands, req = _random_dag(rng, rng.randint(1, 32))
    outs = None
    if seed % 3 == 0:       # explicit outputs, possibly leaving dead ops
        outs = [rng.random() < 0.3 for _ in operands]
        outs[-1] = True
    got = fs_shared_plan(operands, req, outs)
    want = osm.plan(operands, req, outs)
    assert got[0] == want[0] and got[1] == want[1] and got[2] == want[2]
    assert osm.valid_sharing(operands, req, got[0], outs)


def test_library_planner_rejects_bad_graphs():
    with pytest.raises(FsError) as e:
        fs_shared_plan([[1], [0]], [0, 0])          # operand not earlier than its user
    assert e.value.status == binding.FS_ERR_INVALID
    assert fs_shared_plan([], []) == ([], [], 0)
