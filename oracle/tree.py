"""Token-tree logic of the streamlined generation-and-verification loop
(Sec. 3.2, Appendix B, Algorithm 1), on plain Python lists / numpy ints.

Row conventions (shared input format, see the template description): row 0 is the
root = the last emitted token, rows 1..T-1 the draft tree in level order, rows
T..R-1 mask tokens; a mask group hanging off node v is the chain v->m_1->...->m_n.
"""
import numpy as np


class Derived:
    """Everything read off a parent array."""
    pass


def derive_template(parent, is_mask, n_mask):
    parent = [int(p) for p in parent]
    is_mask = [int(m) for m in is_mask]
    R = len(parent)
    T = R - sum(is_mask)
    if R == 0 or parent[0] != -1 or is_mask[0]:
        raise ValueError("row 0 must be the root")
    if any(is_mask[:T]) or not all(is_mask[T:]):
        raise ValueError("tree rows must precede mask rows")
    d = Derived()
    d.parent, d.is_mask, d.R, d.T, d.n_mask = parent, is_mask, R, T, n_mask
    d.depth = [0] * R
    d.children = [[] for _ in range(R)]      # tree children only, in row order
    d.rank = [0] * R                          # index among the parent's tree children
    d.mask_index = [-1] * R                   # 0-based index inside its group
    d.group = [-1] * R                        # group id of a mask row
    d.group_attach = []                       # node each group hangs off
    d.group_of_node = [-1] * T
    for i in range(1, R):
        p = parent[i]
        if not (0 <= p < i):
            raise ValueError("parent[i] must satisfy 0 <= parent[i] < i")
        d.depth[i] = d.depth[p] + 1
        if not is_mask[i]:
            if is_mask[p]:
                raise ValueError("a draft token cannot hang off a mask token")
            d.rank[i] = len(d.children[p])
            d.children[p].append(i)
        elif not is_mask[p]:
            if d.group_of_node[p] != -1:
                raise ValueError("at most one mask group per node")
            d.group[i] = len(d.group_attach)
            d.group_of_node[p] = d.group[i]
            d.group_attach.append(p)
            d.mask_index[i] = 0
        else:
            if p != i - 1:
                raise ValueError("a mask group must occupy consecutive rows")
            d.group[i] = d.group[p]
            d.mask_index[i] = d.mask_index[p] + 1
    d.G = len(d.group_attach)
    for g in range(d.G):
        rows = [i for i in range(R) if d.group[i] == g]
        if len(rows) != n_mask or rows != list(range(rows[0], rows[0] + n_mask)):
            raise ValueError("every mask group must be a chain of exactly n_mask rows")
    d.group_rows = [[i for i in range(R) if d.group[i] == g] for g in range(d.G)]
    d.tree_depth = max(d.depth[:T])
    d.kmax = max([len(c) for c in d.children[:T]] + [1])
    return d


def ancestors_or_self(parent, r):
    """Rows on the path root..r, increasing: what row r attends to inside the pass
    (Sec. 3.2: tokens attend to their ancestors in the tree)."""
    out = []
    while r >= 0:
        out.append(r)
        r = int(parent[r])
    return out[::-1]


def anc_bitsets(parent):
    """Ancestor-or-self sets as ceil(R/64) 64-bit words per row (bit j of word j//64)."""
    R = len(parent)
    W = (R + 63) // 64
    bits = np.zeros((R, W), np.uint64)
    for r in range(R):
        for j in ancestors_or_self(parent, r):
            bits[r, j // 64] |= np.uint64(1) << np.uint64(j % 64)
    return bits


def efficient_tree(n, k):
    """Parent array of the efficient token tree (Sec. 3.2, Fig. 4): level i holds
    the top-k of mask token i, and only the top-1 node of a level has children."""
    parent = [-1]
    top1 = 0
    for _ in range(n):
        first = len(parent)
        for _j in range(k):
            parent.append(top1)
        top1 = first
    return parent


def build_tree_tokens(d, root_token, cand, group=0, shift=0):
    """Token of every row for the next pass.

    cand[g*n + i][j] is the j-th ranked prediction of mask i of group g from the
    previous pass.  A draft row at depth dv with sibling rank j carries the j-th
    prediction of mask (dv - 1 + shift) of the chosen group; `shift` > 0 is the
    straightforward scheme where the masks sat on the previous root and the first
    `shift` of them are stale after `shift` accepted drafts (Fig. 3).  Rows for
    which no prediction exists are inactive (-1).  Mask rows carry their mask index.
    """
    cand = np.asarray(cand)
    tok = [-1] * d.R
    tok[0] = int(root_token)
    for v in range(1, d.T):
        lvl = d.depth[v] - 1 + shift
        if lvl < d.n_mask and d.rank[v] < cand.shape[1]:
            tok[v] = int(cand[group * d.n_mask + lvl][d.rank[v]])
    for v in range(d.T, d.R):
        tok[v] = d.mask_index[v]
    return tok


def accept_walk(d, tokens, greedy):
    """Greedy verification (Sec. 3.2; Algorithm 1's inner loops on a general tree).

    greedy[v] is the model's own top-1 at tree row v.  Starting at the root, move
    to the child that carries the current node's greedy token (lowest row if
    several) until none does.  Returns (path, bonus): the accepted rows, root
    first, and the greedy token of the last one -- the autoregressive output that
    is always accepted.
    """
    v = 0
    path = [0]
    while True:
        a = int(greedy[v])
        nxt = None
        for c in d.children[v]:
            if tokens[c] >= 0 and tokens[c] == a:
                nxt = c
                break
        if nxt is None:
            return path, a
        path.append(nxt)
        v = nxt


def next_group_and_shift(d, path):
    """Which mask group feeds the next tree (Algorithm 1, last step: the group on
    the last accepted candidate, or on the last input token if none was accepted).
    If that node has no group of its own, the root's group is used and its first
    len(path)-1 predictions are dropped as stale."""
    g = d.group_of_node[path[-1]]
    if g >= 0:
        return g, 0
    return d.group_of_node[0], len(path) - 1


def algorithm1_verify(greedy_of_row, cand):
    """Verification of one pass on an efficient tree, in Algorithm 1's own terms.

    cand[i][j]: j-th candidate of mask i (n x k).  Rows: 0 is the last token of
    the result sequence, candidate (i, j) sits at row 1 + i*k + j (the tree
    flattened along its depth).  Returns (emitted tokens, last accepted row).
    """
    n, k = len(cand), len(cand[0])
    emitted = []
    last = 0
    a = int(greedy_of_row[0])
    for i in range(n):
        hit = -1
        for j in range(k):
            if a == int(cand[i][j]):
                hit = j
                break
        if hit < 0:
            break
        emitted.append(a)                 # candidate (i, hit) accepted
        last = 1 + i * k + hit
        a = int(greedy_of_row[last])      # its own prediction becomes the AR output
        if hit != 0:
            break                         # only the top-1 candidate has children
    emitted.append(a)
    return emitted, last


def compact_kv(cache_k, cache_v, new_k, new_v, path):
    """Append the accepted rows' K/V (root first) to the cache of every layer."""
    out_k, out_v = [], []
    for l in range(len(cache_k)):
        out_k.append(np.concatenate([cache_k[l], new_k[l][path]], 0))
        out_v.append(np.concatenate([cache_v[l], new_v[l][path]], 0))
    return out_k, out_v
