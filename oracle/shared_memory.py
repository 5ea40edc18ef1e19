"""Oracle for the shared-memory optimisation (paper Section 5.4, Algorithm 4).

Test infrastructure only: imported by tests/, never by the product path.

Two things are written out here, both from the paper's description and independent of the
library's code:

  dominators()     the dominance relation of the data-flow graph seen from the group's
                   root, by its plain definition: a dominates b iff removing a leaves b
                   unreachable from the root (one graph search per op; slow and obvious)
  plan()           Algorithm 4's walk: ops in execution order; an op without a request
                   passes on its operands' allocation information; an op with a request
                   collects that information, shares the first space whose owner it
                   dominates, reclaims the other dominated ones, otherwise allocates

and a checker, valid_sharing(), for the property the algorithm exists to guarantee: no
space is handed to a new owner while a value it held can still be read.
"""
from __future__ import annotations


def users_of(operands, is_output=None):
    n = len(operands)
    users = [[] for _ in range(n)]
    for i, ops in enumerate(operands):
        for o in ops:
            users[o].append(i)
    if is_output is None:
        is_output = [len(users[i]) == 0 for i in range(n)]
    return users, list(is_output)


def reachable_from_root(operands, is_output, removed=None):
    """Ops reachable from the root along user -> operand edges, with `removed` taken out."""
    n = len(operands)
    seen = [False] * n
    stack = [i for i in range(n) if is_output[i] and i != removed]
    for i in stack:
        seen[i] = True
    while stack:
        v = stack.pop()
        for o in operands[v]:
            if o != removed and not seen[o]:
                seen[o] = True
                stack.append(o)
    return seen


def dominators(operands, is_output=None):
    """dom[a][b] = True iff a != b, b is reachable from the root, and every path from the
    root to b passes through a."""
    n = len(operands)
    _, is_output = users_of(operands, is_output)
    base = reachable_from_root(operands, is_output)
    dom = [[False] * n for _ in range(n)]
    for a in range(n):
        without = reachable_from_root(operands, is_output, removed=a)
        for b in range(n):
            if a != b and base[b] and not without[b]:
                dom[a][b] = True
    return dom


def plan(operands, req_bytes, is_output=None):
    """Algorithm 4.  -> (offset per op or -1, shares_with per op or -1, total bytes).

    Where the paper is silent: a space is shared only if it is at least as large as the
    request; a request that shares nothing first looks for the smallest reclaimed space
    that fits and only then takes fresh space at the end of the footprint; the operands'
    allocation information is visited in increasing op index."""
    n = len(operands)
    dom = dominators(operands, is_output)
    space = [None] * n            # (offset, bytes) an op currently owns
    offset = [-1] * n
    shares = [-1] * n
    info = [set() for _ in range(n)]
    reclaimed = []
    total = 0
    for inst in range(n):
        prev_allocs = set()
        for o in operands[inst]:
            prev_allocs |= info[o]
        if req_bytes[inst] <= 0:
            info[inst] = prev_allocs
            continue
        shared = False
        keep = set()
        for prev in sorted(prev_allocs):
            if space[prev] is None:
                continue
            if dom[inst][prev]:
                if not shared and space[prev][1] >= req_bytes[inst]:
                    space[inst] = space[prev]
                    shares[inst] = prev
                    shared = True
                else:
                    reclaimed.append(space[prev])
                space[prev] = None
            else:
                keep.add(prev)
        if not shared:
            fits = [s for s in reclaimed if s[1] >= req_bytes[inst]]
            if fits:
                best = min(fits, key=lambda s: s[1])
                reclaimed.remove(best)
                space[inst] = best
            else:
                space[inst] = (total, req_bytes[inst])
                total += req_bytes[inst]
        offset[inst] = space[inst][0]
        info[inst] = keep | {inst}
    return offset, shares, total


def valid_sharing(operands, req_bytes, offset, is_output=None):
    """True iff no two requests whose values are alive at the same time overlap in space.
    A value is alive from the op that produces it to its last user that the root reaches
    (ops the root does not reach are never run); outputs stay alive to the end."""
    n = len(operands)
    users, is_output = users_of(operands, is_output)
    live = reachable_from_root(operands, is_output)
    users = [[u for u in us if live[u]] for us in users]
    last = [max(users[i]) if users[i] else i for i in range(n)]
    for i in range(n):
        if is_output[i]:
            last[i] = n
    reqs = [i for i in range(n) if req_bytes[i] > 0 and live[i]]
    for x in reqs:
        for y in reqs:
            if x >= y:
                continue
            overlap_space = offset[x] < offset[y] + req_bytes[y] and offset[y] < offset[x] + req_bytes[x]
            # y is produced while x is still needed by an op after y (x's own last use may be y itself:
            # an op may overwrite its operand's space in place)
            alive_together = last[x] > y
            if overlap_space and alive_together:
                return False
    return True
