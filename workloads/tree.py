"""Static draft-tree topologies (App. B "Static Tree Structures").

The paper's figure of the tree is not available as text; it only says the tree
is fixed, left-heavy ("more nodes to the left branches") and has 26 or ~58
drafted nodes.  This generator builds a left-heavy, ancestor-closed tree from
per-depth branching caps and a node budget:

  * enumerate the full tree with branching ``b_1..b_K``; a node is its path
    ``(r_1..r_d)`` with ``0 <= r_i < b_i`` (``r_i`` = rank among siblings);
  * cost of a node = ``sum_i i * r_i`` (1-based depth ``i``), so right-hand and
    deep right-hand branches are the first to be dropped;
  * keep the ``N`` cheapest by (cost, depth, path), renumber 1..N by
    (depth, path); row 0 is the root (the last committed token).

Rows are therefore in BFS order, ``parent[i] < i``, and the children of a row
are consecutive in index order (their static try-order).
"""
from itertools import product
from typing import List, Sequence

import numpy as np


def static_tree(branching: Sequence[int], n_nodes: int) -> np.ndarray:
    """Return ``parent`` (int32, length n_nodes+1, parent[0] = -1)."""
    nodes = []
    for d in range(1, len(branching) + 1):
        for path in product(*[range(b) for b in branching[:d]]):
            cost = sum((i + 1) * r for i, r in enumerate(path))
            nodes.append((cost, d, path))
    if n_nodes > len(nodes):
        raise ValueError("node budget exceeds the full tree")
    nodes.sort()
    kept = sorted(nodes[:n_nodes], key=lambda t: (t[1], t[2]))
    index = {(): 0}
    for i, (_, _, path) in enumerate(kept):
        index[path] = i + 1
    parent = np.full(n_nodes + 1, -1, dtype=np.int32)
    for _, _, path in kept:
        parent[index[path]] = index[path[:-1]]
    return parent


def tree_depths(parent: np.ndarray) -> np.ndarray:
    depth = np.zeros(len(parent), dtype=np.int32)
    for i in range(1, len(parent)):
        depth[i] = depth[parent[i]] + 1
    return depth


def children_lists(parent: np.ndarray) -> List[List[int]]:
    kids: List[List[int]] = [[] for _ in range(len(parent))]
    for i in range(1, len(parent)):
        kids[int(parent[i])].append(i)
    return kids
