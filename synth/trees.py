"""Draft-tree shapes as (parent, depth) int32 arrays in topological order.

Node 0 is the root (the last committed token); parent[0] = -1, parent[i] < i,
depth[i] = depth[parent[i]] + 1.  Only shapes and random ids are made here.
"""
from __future__ import annotations

import itertools

import numpy as np

from .model import MATRIX_IDS


def _depths(parent: np.ndarray) -> np.ndarray:
    depth = np.zeros(len(parent), dtype=np.int32)
    for i in range(1, len(parent)):
        depth[i] = depth[parent[i]] + 1
    return depth


def is_valid_tree(parent, depth) -> bool:
    parent = np.asarray(parent)
    depth = np.asarray(depth)
    if len(parent) < 1 or len(parent) != len(depth):
        return False
    if parent[0] != -1 or depth[0] != 0:
        return False
    for i in range(1, len(parent)):
        if not (0 <= parent[i] < i) or depth[i] != depth[parent[i]] + 1:
            return False
    return True


def chain_tree(n: int):
    """n nodes in a single line: node i hangs under node i-1."""
    parent = np.arange(-1, n - 1, dtype=np.int32)
    return parent, _depths(parent)


def complete_binary_tree(levels: int):
    """Complete binary tree with `levels` levels below the root (2^(levels+1)-1 nodes)."""
    n = 2 ** (levels + 1) - 1
    parent = np.array([-1] + [(i - 1) // 2 for i in range(1, n)], dtype=np.int32)
    return parent, _depths(parent)


def random_tree(n: int, max_depth: int, seed: int):
    """parent[i] uniform over the earlier nodes whose depth is below max_depth."""
    rng = np.random.Generator(np.random.SFC64(
        np.random.SeedSequence((seed, n, MATRIX_IDS["tree"]))))
    parent = np.full(n, -1, dtype=np.int32)
    depth = np.zeros(n, dtype=np.int32)
    for i in range(1, n):
        cand = np.flatnonzero(depth[:i] < max_depth)
        parent[i] = cand[rng.integers(0, len(cand))]
        depth[i] = depth[parent[i]] + 1
    return parent, depth


def product_tree_pruned(branching=(4, 3, 2, 2, 1, 1), keep: int = 63):
    """Top-k product tree cut down to its `keep` most likely nodes.

    The full tree gives every node at level k `branching[k]` children ranked
    0..b-1.  A node scores the product of 1/(1+rank) along its path; the `keep`
    best nodes are kept (ties: breadth-first index), which is closed under
    ancestors because scores never increase along a path.  Returns
    (parent, depth, rank) renumbered breadth-first; rank[0] = 0.
    """
    nodes = [(-1, 0, 0, 1.0)]  # parent index in `nodes`, depth, rank, score
    frontier = [0]
    for b in branching:
        nxt = []
        for p in frontier:
            for r in range(b):
                nodes.append((p, nodes[p][1] + 1, r, nodes[p][3] / (1.0 + r)))
                nxt.append(len(nodes) - 1)
        frontier = nxt
    order = sorted(range(len(nodes)), key=lambda i: (-nodes[i][3], i))[:keep]
    kept = sorted(order)  # breadth-first order is the construction order
    new_index = {old: new for new, old in enumerate(kept)}
    parent = np.array([-1 if nodes[o][0] < 0 else new_index[nodes[o][0]] for o in kept],
                      dtype=np.int32)
    depth = np.array([nodes[o][1] for o in kept], dtype=np.int32)
    rank = np.array([nodes[o][2] for o in kept], dtype=np.int32)
    return parent, depth, rank


def chain_with_corrections(gamma: int, correction_positions):
    """The tree shape of a cascaded draft: root, a main chain of `gamma` draft
    tokens (node i+1 carries draft position i), and for each position i in
    `correction_positions` one extra leaf that is a sibling of draft position i.
    Returns (parent, depth, main_node[gamma], corr_node{i: node})."""
    parent = [-1] + list(range(gamma))
    main_node = list(range(1, gamma + 1))
    corr_node = {}
    for i in sorted(correction_positions):
        assert 0 <= i < gamma
        corr_node[i] = len(parent)
        parent.append(i)  # node i is the parent of draft position i (node i+1)
    parent = np.array(parent, dtype=np.int32)
    return parent, _depths(parent), np.array(main_node, dtype=np.int32), corr_node


def distinct_sibling_tokens(parent, vocab: int, seed: int) -> np.ndarray:
    """Uniform random token ids with no two siblings sharing an id."""
    rng = np.random.Generator(np.random.SFC64(
        np.random.SeedSequence((seed, len(parent), MATRIX_IDS["tree_tokens"]))))
    n = len(parent)
    tok = np.zeros(n, dtype=np.int32)
    used = {}
    for i in range(n):
        taken = used.setdefault(int(parent[i]), set())
        while True:
            t = int(rng.integers(0, vocab))
            if t not in taken:
                break
        taken.add(t)
        tok[i] = t
    return tok


def all_parent_arrays(n: int):
    """Every topologically ordered tree on n nodes: parent[i] ranges over [0, i)."""
    for tail in itertools.product(*[range(i) for i in range(1, n)]):
        parent = np.array((-1,) + tail, dtype=np.int32)
        yield parent, _depths(parent)


def relabel_topological(parent, seed: int):
    """A random renumbering that keeps parents before children.
    Returns (new_parent, new_depth, old_of_new) with old_of_new[new] = old."""
    rng = np.random.Generator(np.random.SFC64(np.random.SeedSequence((seed, 99))))
    n = len(parent)
    children = {i: [] for i in range(n)}
    for i in range(1, n):
        children[int(parent[i])].append(i)
    ready = [0]
    old_of_new = []
    while ready:
        j = int(rng.integers(0, len(ready)))
        node = ready.pop(j)
        old_of_new.append(node)
        ready.extend(children[node])
    new_of_old = {old: new for new, old in enumerate(old_of_new)}
    new_parent = np.array([-1 if parent[o] < 0 else new_of_old[int(parent[o])]
                           for o in old_of_new], dtype=np.int32)
    return new_parent, _depths(new_parent), np.array(old_of_new, dtype=np.int32)
