"""Draft-tree topologies encoded as parent-index arrays.

A tree with N nodes is an int32 array ``parent`` with ``parent[0] == -1`` (the root, i.e. the
pending committed token) and ``0 <= parent[i] < i`` for every other node, so nodes are numbered
in an order in which every ancestor precedes its descendants.
"""
from __future__ import annotations

import numpy as np


def chain_tree(n: int) -> np.ndarray:
    """The chain draft the paper measures (Section 1, Section 4.2): parents [-1, 0, 1, ...]."""
    if n < 1:
        raise ValueError("a tree needs at least the root")
    return np.arange(-1, n - 1, dtype=np.int32)


def validate_parents(parent) -> None:
    parent = np.asarray(parent)
    if parent.ndim != 1 or parent.size == 0:
        raise ValueError("parent must be a non-empty 1-d array")
    if parent[0] != -1:
        raise ValueError("node 0 must be the root (parent -1)")
    for i in range(1, parent.size):
        if not (0 <= parent[i] < i):
            raise ValueError(f"parent[{i}]={parent[i]} must lie in [0, {i})")


def tree_depths(parent) -> np.ndarray:
    parent = np.asarray(parent)
    depth = np.zeros(parent.size, dtype=np.int32)
    for i in range(1, parent.size):
        depth[i] = depth[parent[i]] + 1
    return depth


def seeded_tree(seed: int, n_nodes: int = 60, levels: int = 6, root_fanout: int = 10,
                max_fanout: int = 4) -> np.ndarray:
    """A breadth-first numbered tree: one root with ``root_fanout`` children, ``levels`` levels
    counting the root's, ``n_nodes`` nodes in all, every other internal node with between 1 and
    ``max_fanout`` children drawn from the seed."""
    if levels < 2 or n_nodes < 1 + root_fanout + (levels - 2):
        raise ValueError("not enough nodes for the requested shape")
    rng = np.random.default_rng(seed)
    rest = n_nodes - 1 - root_fanout
    n_lower = levels - 2
    if n_lower == 0 and rest != 0:
        raise ValueError("nodes left over with no level to put them on")
    # level sizes: each lower level has >= 1 node and at most max_fanout per node above it
    for _ in range(10000):
        sizes = [1] * n_lower
        left = rest - n_lower
        ok = True
        # hand out the remaining nodes one at a time to a random level that still has room
        while left > 0:
            room = []
            prev = root_fanout
            for lv in range(n_lower):
                if sizes[lv] < max_fanout * prev:
                    room.append(lv)
                prev = sizes[lv]
            if not room:
                ok = False
                break
            sizes[int(rng.choice(room))] += 1
            left -= 1
        if not ok:
            continue
        prev = root_fanout
        for lv in range(n_lower):
            if sizes[lv] > max_fanout * prev:
                ok = False
            prev = sizes[lv]
        if ok:
            break
    else:
        raise ValueError("could not fit the level sizes")
    parent = [-1] + [0] * root_fanout
    level_nodes = list(range(1, 1 + root_fanout))
    for lv in range(n_lower):
        want = sizes[lv]
        # children per node of the level above: 0..max_fanout each, summing to `want`
        counts = np.zeros(len(level_nodes), dtype=np.int64)
        for _ in range(want):
            room = np.flatnonzero(counts < max_fanout)
            counts[int(rng.choice(room))] += 1
        new_nodes = []
        for node, c in zip(level_nodes, counts):
            for _ in range(int(c)):
                new_nodes.append(len(parent))
                parent.append(node)
        level_nodes = new_nodes
    out = np.asarray(parent, dtype=np.int32)
    validate_parents(out)
    assert out.size == n_nodes
    assert int(tree_depths(out).max()) == levels - 1
    return out
