"""Pins for the oracle's tree logic (CPU only)."""
import itertools
import numpy as np
import pytest

import oracle
import synth
from oracle.tree import (derive_template, ancestors_or_self, anc_bitsets, efficient_tree,
                         build_tree_tokens, accept_walk, algorithm1_verify, next_group_and_shift)
from helpers import read_paper_facts, all_parent_arrays

FACTS = read_paper_facts()


def _tmpl(parent, attach, n):
    t = synth.attach_mask_groups(parent, attach, n)
    return t, derive_template(t.parent, t.is_mask, n)


def test_efficient_tree_sizes_match_paper_closed_forms():
    """n*k+1 mask groups (one per draft node plus the last input token)."""
    for n, k in [(int(FACTS["fig4_n"]), int(FACTS["fig4_k"])),
                 (int(FACTS["default_n_small"]), int(FACTS["default_k"])),
                 (int(FACTS["default_n_large"]), int(FACTS["default_k"]))]:
        p = efficient_tree(n, k)
        assert len(p) == n * k + 1
        t, d = _tmpl(p, range(len(p)), n)
        assert d.G == n * k + 1                       # Algorithm 1: M x (n*k+1)
        assert d.R == (n * k + 1) * (1 + n)
        # only the top-1 node of each level has children; each level has k nodes
        for lvl in range(1, n + 1):
            nodes = [v for v in range(d.T) if d.depth[v] == lvl]
            assert len(nodes) == k
            assert [d.rank[v] for v in nodes] == list(range(k))
            for v in nodes:
                assert (len(d.children[v]) > 0) == (d.rank[v] == 0 and lvl < n)
    assert len(efficient_tree(3, 5)) * 4 == 64 and len(efficient_tree(4, 5)) * 5 == 105
    assert list(synth.efficient_tree_parents(4, 3)) == efficient_tree(4, 3)


def test_ancestor_sets_exhaustive_small_trees():
    """Every parent array with up to 6 rows: bitset == brute-force reachability."""
    for T in range(1, 7):
        for parent in all_parent_arrays(T):
            bits = anc_bitsets(parent)
            # brute force: j is an ancestor-or-self of r iff repeated parent steps from r hit j
            for r in range(T):
                reach = set()
                x = r
                for _ in range(T):
                    if x < 0:
                        break
                    reach.add(x)
                    x = parent[x]
                got = {j for j in range(T) if (int(bits[r, 0]) >> j) & 1}
                assert got == reach
                assert ancestors_or_self(parent, r) == sorted(reach)


def test_ancestor_bitsets_multiword():
    parent = list(synth.chain_tree(130))
    bits = anc_bitsets(parent)
    assert bits.shape == (130, 3)
    assert int(bits[129, 0]) == 2 ** 64 - 1 and int(bits[129, 1]) == 2 ** 64 - 1 and int(bits[129, 2]) == 3
    assert int(bits[64, 1]) == 1 and int(bits[63, 1]) == 0


def _brute_force_accept(d, tokens, greedy):
    """Longest root-to-node path whose tokens equal the successive greedy outputs;
    among equal-token siblings the lowest row wins, which makes it unique."""
    best = [0]

    def rec(path):
        nonlocal best
        v = path[-1]
        seen = set()
        for c in d.children[v]:
            if tokens[c] >= 0 and tokens[c] == greedy[v] and tokens[c] not in seen:
                seen.add(tokens[c])
                if len(path) + 1 > len(best):
                    best = path + [c]
                rec(path + [c])
    rec([0])
    return best


def test_accept_walk_equals_bruteforce_on_random_trees():
    rng = np.random.default_rng(0)
    lens = set()
    for trial in range(300):
        T = int(rng.integers(1, 12))
        parent = synth.random_tree(T, 4, trial)
        t, d = _tmpl(parent, [0], 3)
        vocab = 4                                   # tiny vocab -> many matches and duplicates
        tokens = list(rng.integers(0, vocab, size=T)) + [0, 1, 2]
        for v in range(1, T):
            if rng.random() < 0.15:
                tokens[v] = -1                      # inactive rows never match
        greedy = list(rng.integers(0, vocab, size=T))
        path, bonus = accept_walk(d, tokens, greedy)
        assert path == _brute_force_accept(d, tokens, greedy)
        assert bonus == greedy[path[-1]]
        assert 1 <= len(path) <= d.tree_depth + 1
        for a, b in zip(path, path[1:]):
            assert d.parent[b] == a and tokens[b] == greedy[a]
        lens.add(len(path))
    assert lens >= {1, 2, 3}


def test_accept_walk_equals_algorithm1_on_efficient_trees():
    """The general walk and the paper's own loop agree on efficient trees, for all
    acceptance patterns including 'accepted a non-top-1 candidate, stop'."""
    rng = np.random.default_rng(1)
    seen_lens = set()
    for n, k in [(3, 5), (4, 3), (4, 5), (1, 1), (2, 1)]:
        parent = efficient_tree(n, k)
        t, d = _tmpl(parent, range(len(parent)), n)
        for trial in range(200):
            vocab = 6
            cand = np.stack([rng.permutation(vocab)[:k] if k <= vocab else rng.integers(0, vocab, k)
                             for _ in range(n)]).astype(np.int32)
            tokens = build_tree_tokens(d, 7, cand, group=0, shift=0)
            # row of candidate (i, j) is 1 + i*k + j, the tree flattened along its depth
            for i in range(n):
                for j in range(k):
                    assert tokens[1 + i * k + j] == cand[i, j]
            greedy = list(rng.integers(0, vocab, size=d.T))
            path, bonus = accept_walk(d, tokens, greedy)
            emitted, last = algorithm1_verify(greedy, cand)
            assert [tokens[c] for c in path[1:]] + [bonus] == emitted
            assert path[-1] == last
            assert 1 <= len(emitted) <= n + 1
            seen_lens.add(len(emitted))
            g, s = next_group_and_shift(d, path)
            assert d.group_attach[g] == last and s == 0     # group on the last accepted token
    assert seen_lens >= {1, 2, 3, 4}


def test_fig3_tokens_per_pass_bound():
    m = int(FACTS["fig3_mask_tokens"])
    per_pass = [int(x) for x in FACTS["fig3_tokens_per_pass"].split()]
    assert all(1 <= x <= m + 1 for x in per_pass)
    # a chain of M drafts (straightforward decoding) can emit at most M + 1 tokens, and exactly
    # reproduces each of the figure's counts for a suitable number of correct drafts
    parent = synth.chain_tree(m + 1)
    t, d = _tmpl(parent, [0], m)
    for want in per_pass:
        greedy = [10, 11, 12, 13]
        tokens = [5] + [10 + i if i < want - 1 else 99 for i in range(m)] + [0, 1, 2]
        path, bonus = accept_walk(d, tokens, greedy)
        assert len(path) == want and bonus == greedy[want - 1]
        g, s = next_group_and_shift(d, path)
        assert g == 0 and s == want - 1               # first c mask outputs are stale (Fig. 3)


def test_build_tree_tokens_shift_and_inactive_rows():
    parent = synth.full_branching_tree([2, 2, 1])
    t, d = _tmpl(parent, [0], 3)
    cand = np.arange(12, dtype=np.int32).reshape(3, 4) + 100
    tok = build_tree_tokens(d, 9, cand, 0, 0)
    assert tok[0] == 9
    assert tok[1:3] == [100, 101]                     # level 1 <- mask 0, ranks 0,1
    assert tok[3:7] == [104, 105, 104, 105]           # level 2 <- mask 1 under both parents
    assert tok[7:11] == [108, 108, 108, 108]
    assert tok[11:] == [0, 1, 2]                      # mask rows carry their index
    tok = build_tree_tokens(d, 9, cand, 0, 2)         # two stale masks: only level 1 usable
    assert tok[1:3] == [108, 109] and all(x == -1 for x in tok[3:11])


def test_template_validation_rejects_bad_shapes():
    with pytest.raises(ValueError):
        derive_template([-1, 1], [0, 0], 1)           # parent[i] >= i
    with pytest.raises(ValueError):
        derive_template([0, 0], [0, 0], 1)            # root must have parent -1
    with pytest.raises(ValueError):
        derive_template([-1, 0, 0], [0, 1, 0], 1)     # mask row before a tree row
    with pytest.raises(ValueError):
        derive_template([-1, 0, 1], [0, 1, 1], 3)     # group shorter than n_mask
    with pytest.raises(ValueError):
        derive_template([-1, 0, 0], [0, 1, 1], 1)     # two groups on one node


def test_prompt_prefix_parameter_fraction():
    """Per-layer K and V prefix of width Hkv*hd plus n mask embeddings reproduces the
    paper's ~0.06 % at 7B and roughly ten times less at 70B."""
    c7, c70 = synth.get_config("7b", n_mask=3), synth.get_config("70b", n_mask=4)

    def extra(c):
        return c.n_prompt * c.n_layers * 2 * c.kv_dim + c.n_mask * c.d_model

    def total(c):
        return c.weight_bytes(1) + c.vocab * c.d_model
    f7 = 100.0 * extra(c7) / total(c7)
    f70 = 100.0 * extra(c70) / total(c70)
    assert abs(f7 - float(FACTS["param_fraction_7b_percent"])) < 0.005
    assert 8 <= f7 / f70 <= 20
