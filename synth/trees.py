"""Draft-tree topologies as parent arrays (inputs to both sides).

A template is a parent array over R rows: rows 0..T-1 are the token tree in
level (breadth-first) order with the root (last emitted token) as row 0, rows
T..R-1 are mask tokens.  A group of n mask tokens attached to node v is the chain
v -> m_1 -> ... -> m_n, so a single parent array describes tree and mask rows
alike.  Only the *shape* is produced here; depths, ancestor sets, sibling ranks
and everything else derived from it are computed independently by each side.
"""
from dataclasses import dataclass
import numpy as np


@dataclass
class Template:
    parent: np.ndarray    # int32 [R], parent[0] = -1, parent[i] < i
    is_mask: np.ndarray   # uint8 [R]
    n_tree: int           # T
    n_mask: int           # n (mask tokens per group)

    @property
    def rows(self):
        return int(self.parent.shape[0])


def random_tree(T, max_depth, seed):
    """parent[i] uniform over earlier rows whose depth < max_depth; rows are then
    relabelled into level order (stable), as the flattened tree requires."""
    rng = np.random.default_rng(seed)
    parent = [-1]
    depth = [0]
    for i in range(1, T):
        ok = [j for j in range(i) if depth[j] < max_depth]
        p = int(ok[rng.integers(len(ok))])
        parent.append(p)
        depth.append(depth[p] + 1)
    order = sorted(range(T), key=lambda i: (depth[i], i))
    new_id = {old: new for new, old in enumerate(order)}
    out = np.full(T, -1, np.int32)
    for old in range(1, T):
        out[new_id[old]] = new_id[parent[old]]
    return out


def full_branching_tree(ks, T=None):
    """Every node of level i-1 has ks[i-1] children; level order; optionally
    truncated to the first T rows."""
    parent = [-1]
    level = [0]
    for k in ks:
        nxt = []
        for p in level:
            for _ in range(k):
                nxt.append(len(parent))
                parent.append(p)
        level = nxt
    if T is not None:
        parent = parent[:T]
    return np.asarray(parent, np.int32)


def efficient_tree_parents(n, k):
    """Level i holds k candidates, all children of the first candidate of level
    i-1 (the root for level 1): 1 + n*k rows."""
    parent = [-1]
    anchor = 0
    for _ in range(n):
        first = len(parent)
        parent.extend([anchor] * k)
        anchor = first
    return np.asarray(parent, np.int32)


def chain_tree(T):
    return np.arange(-1, T - 1, dtype=np.int32)


def star_tree(T):
    p = np.zeros(T, np.int32)
    p[0] = -1
    return p


def attach_mask_groups(tree_parent, attach_nodes, n_mask):
    """Append one chain of n_mask mask rows per entry of attach_nodes."""
    tree_parent = np.asarray(tree_parent, np.int32)
    T = tree_parent.shape[0]
    parent = list(tree_parent)
    for v in attach_nodes:
        prev = int(v)
        for _ in range(n_mask):
            parent.append(prev)
            prev = len(parent) - 1
    parent = np.asarray(parent, np.int32)
    is_mask = np.zeros(parent.shape[0], np.uint8)
    is_mask[T:] = 1
    return Template(parent, is_mask, T, n_mask)
