"""Static candidate-tree topologies (inputs to `ht_set_tree`), as plain Python lists.

A tree is `(parent, rank)`: `parent[0] == -1`, `0 <= parent[v] < v`; `rank[v]` says which of the
top-r candidates of its level node v carries (root rank is 0 and unused).
"""
from __future__ import annotations

from itertools import product
from typing import List, Sequence, Tuple

from .generators import _key, _mix_py, GOLDEN


def tree_depths(parent: Sequence[int]) -> List[int]:
    depth = [0] * len(parent)
    for v in range(1, len(parent)):
        depth[v] = depth[parent[v]] + 1
    return depth


def prune_tree(branching: Sequence[int], size: int) -> Tuple[List[int], List[int]]:
    """Best-`size` sub-tree of the full top-b_1 x ... x top-b_k product tree.

    A node is a rank path (r_1..r_j); its score is prod(r_i + 1) (smaller = more likely under a
    rank-independence prior).  The `size` nodes smallest by (score, depth, path) are kept, which
    is ancestor-closed because every prefix has a score no larger and a smaller depth.  If the
    full tree is smaller than `size`, b_1 is widened until it is large enough.  Nodes are then
    numbered by (depth, path), so parents precede children.
    """
    branching = list(branching)
    if size < 1:
        raise ValueError("size must be >= 1")

    def full_count(b):
        total, level = 1, 1
        for x in b:
            level *= x
            total += level
        return total

    while full_count(branching) < size:
        branching[0] += 1

    nodes = [()]
    for j in range(1, len(branching) + 1):
        nodes.extend(product(*[range(b) for b in branching[:j]]))

    def score(path):
        s = 1
        for r in path:
            s *= r + 1
        return s

    kept = sorted(nodes, key=lambda p: (score(p), len(p), p))[:size]
    kept.sort(key=lambda p: (len(p), p))
    index = {p: i for i, p in enumerate(kept)}
    parent = [-1 if not p else index[p[:-1]] for p in kept]
    rank = [0 if not p else p[-1] for p in kept]
    return parent, rank


def random_tree(seed: int, size: int, max_depth: int) -> Tuple[List[int], List[int]]:
    """Each node attaches to a uniformly chosen earlier node whose depth is below `max_depth`."""
    parent, depth, rank, nchild = [-1], [0], [0], [0]
    key = _key(seed, 0x7EE)
    for v in range(1, size):
        eligible = [u for u in range(v) if depth[u] < max_depth]
        h = _mix_py(key + v * GOLDEN)
        p = eligible[(h >> 33) % len(eligible)]
        parent.append(p)
        depth.append(depth[p] + 1)
        rank.append(nchild[p])
        nchild[p] += 1
        nchild.append(0)
    return parent, rank


def chain_tree(size: int) -> Tuple[List[int], List[int]]:
    return [v - 1 for v in range(size)], [0] * size


def star_tree(size: int) -> Tuple[List[int], List[int]]:
    return [-1] + [0] * (size - 1), [0] + list(range(size - 1))
