"""Oracle for fusion planning (paper Section 4).

Test infrastructure only: imported by tests/, never by the product path.

Written from the paper's definitions, independently of the library:

  flow()              who reads whose result, seen through ops that own no kernel (constants,
                      broadcasts): the data-flow graph between kernels
  is_convex()         fusing a set of ops keeps the graph acyclic iff no path leaves the set
                      and returns to it (the cyclic-dependence condition of Section 4.1 / 4.2)
  traffic()           off-chip bytes moved when every listed kernel reads its inputs once and
                      writes its results once; saved_bytes() = one kernel per op minus one kernel
                      for the whole pattern: the V of the model-based score
  model_us()          M(V): bytes over the bandwidth read off a (bytes, GB/s) table, interpolated
                      linearly in log(bytes)
  score()             f(P) = M(V) + (N - 1) * phi
  substitution_segments()   Algorithm 1: ops between adjacent partition ops, in list order
  best_selection()    the ILP of Section 4.1 by brute force: the subset of pairwise disjoint
                      patterns with the largest total score whose contraction leaves a DAG
"""
from __future__ import annotations

import itertools
import math

ITEMSIZE = {"f32": 4, "f16": 2, "bf16": 2}
FREE = ("constant", "broadcast")


def nbytes(op):
    n = 1
    for e in op.shape:
        n *= e
    return n * ITEMSIZE[op.dtype]


def owns_kernel(op):
    return op.kind not in ("parameter", "output") + FREE


def flow(ops):
    """-> (producers, consumers): per op index, the kernel-owning ops / parameters it reads,
    and the kernel-owning ops / output ops that read it, looking through free ops."""
    n = len(ops)
    sources = [None] * n
    producers = [[] for _ in range(n)]
    consumers = [[] for _ in range(n)]
    for i, op in enumerate(ops):
        ins = []
        for a in op.operands:
            for s in sources[a]:
                if s not in ins:
                    ins.append(s)
        if op.kind in FREE:
            sources[i] = ins
            continue
        sources[i] = [i]
        if op.kind == "parameter":
            continue
        producers[i] = ins
        for s in ins:
            consumers[s].append(i)
    return producers, consumers


def is_convex(ops, members):
    """No path from a member through a non-member back to a member."""
    _, consumers = flow(ops)
    inside = set(members)
    for start in members:
        frontier = [c for c in consumers[start] if c not in inside]
        seen = set(frontier)
        while frontier:
            v = frontier.pop()
            for c in consumers[v]:
                if c in inside:
                    return False
                if c not in seen:
                    seen.add(c)
                    frontier.append(c)
    return True


def traffic(ops, kernels):
    """Bytes moved by a list of kernels (each a set of op indices run as one kernel): every
    kernel reads each distinct outside value it needs once and writes each of its results that
    someone outside it reads once."""
    producers, consumers = flow(ops)
    total = 0
    for k in kernels:
        k = set(k)
        reads = set()
        for o in k:
            for p in producers[o]:
                if p not in k:
                    reads.add(p)
        total += sum(nbytes(ops[p]) for p in reads)
        for o in k:
            if any(c not in k for c in consumers[o]):
                total += nbytes(ops[o])
    return total


def saved_bytes(ops, members):
    return traffic(ops, [[o] for o in members]) - traffic(ops, [list(members)])


def model_us(table, nbytes_moved):
    if nbytes_moved <= 0:
        return 0.0
    if nbytes_moved <= table[0][0]:
        gbs = table[0][1]
    elif nbytes_moved >= table[-1][0]:
        gbs = table[-1][1]
    else:
        for (b0, g0), (b1, g1) in zip(table, table[1:]):
            if nbytes_moved <= b1:
                t = (math.log(nbytes_moved) - math.log(b0)) / (math.log(b1) - math.log(b0))
                gbs = g0 + t * (g1 - g0)
                break
    return nbytes_moved / (gbs * 1e9) * 1e6


def score(ops, members, table, launch_us):
    return model_us(table, saved_bytes(ops, members)) + (len(members) - 1) * launch_us


def substitution_segments(ops, is_partition):
    """Algorithm 1: walk the kernel-owning ops in list order; a partition op closes the current
    segment and stands alone; segments of two or more ops are patterns."""
    out, seg = [], []
    for i, op in enumerate(ops):
        if not owns_kernel(op):
            continue
        if is_partition(op):
            if len(seg) >= 2:
                out.append(seg)
            seg = []
        else:
            seg.append(i)
    if len(seg) >= 2:
        out.append(seg)
    return out


def contraction_is_acyclic(ops, chosen):
    """Contract every chosen pattern to one node, keep the other kernels as they are: DAG?"""
    _, consumers = flow(ops)
    group = {}
    for g, members in enumerate(chosen):
        for o in members:
            group[o] = ("p", g)
    nodes, edges = set(), set()
    for i, op in enumerate(ops):
        if not owns_kernel(op):
            continue
        a = group.get(i, ("o", i))
        nodes.add(a)
        for c in consumers[i]:
            if not owns_kernel(ops[c]):
                continue
            b = group.get(c, ("o", c))
            if a != b:
                edges.add((a, b))
    indeg = {v: 0 for v in nodes}
    for _, b in edges:
        indeg[b] += 1
    ready = [v for v in nodes if indeg[v] == 0]
    done = 0
    while ready:
        v = ready.pop()
        done += 1
        for a, b in edges:
            if a == v:
                indeg[b] -= 1
                if indeg[b] == 0:
                    ready.append(b)
    return done == len(nodes)


def best_selection(ops, patterns, scores):
    """Brute force over all subsets of the candidate patterns (keep it to ~16 candidates)."""
    best, best_sets = 0.0, []
    idx = [k for k, s in enumerate(scores) if s >= 0]
    for r in range(len(idx) + 1):
        for combo in itertools.combinations(idx, r):
            used = set()
            ok = True
            for k in combo:
                if used & set(patterns[k]):
                    ok = False
                    break
                used |= set(patterns[k])
            if not ok or not contraction_is_acyclic(ops, [patterns[k] for k in combo]):
                continue
            total = sum(scores[k] for k in combo)
            if total > best + 1e-9:
                best, best_sets = total, [combo]
            elif abs(total - best) <= 1e-9:
                best_sets.append(combo)
    return best, best_sets
