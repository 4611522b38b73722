"""Host-side logic of bench.py, checked on the CPU against the oracle's tree rules
(Sec. 3.2, Algorithm 1): the planted candidate tables must make the verification accept
exactly the planted number of draft tokens, for every template of the sweep."""
import os
import sys

import numpy as np
import pytest

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import bench  # noqa: E402
import synth  # noqa: E402
from oracle.tree import derive_template, build_tree_tokens, accept_walk  # noqa: E402


@pytest.mark.parametrize("tree", sorted(bench.TREES))
def test_planted_walk_is_accepted_to_its_depth(tree):
    cfg = synth.get_config("7b")
    tin = bench.workload_template(synth, cfg, "7b", tree)
    d = derive_template(tin.parent, tin.is_mask, cfg.n_mask)
    children, depth_max = bench.tree_shape(tin)
    assert depth_max == max(d.depth[: d.T])
    for v in range(d.T):                       # sibling order = candidate column
        for j, c in enumerate(children[v]):
            assert d.rank[c] == j and d.parent[c] == v
    seen = set()
    for seed in range(40):
        rng = np.random.default_rng(seed)
        cont = rng.integers(0, cfg.vocab, depth_max + 2).tolist()
        depth_ok, col = bench.planted_walk(children, depth_max, cfg.n_mask, rng)
        cand = synth.planted_candidates(cont, cfg.n_mask, d.kmax, depth_ok, col, cfg.vocab, 50 + seed)
        root = int(rng.integers(0, cfg.vocab))
        tokens = build_tree_tokens(d, root, cand)
        # a model that continues the reference: a row whose root path spells cont[:depth]
        # predicts cont[depth]; every other row predicts a token no candidate carries
        greedy = []
        for r in range(d.T):
            path, v = [], r
            while v > 0:
                path.append(tokens[v])
                v = d.parent[v]
            path = path[::-1]
            greedy.append(cont[len(path)] if path == cont[: len(path)] else -7)
        acc_path, bonus = accept_walk(d, tokens, greedy)
        assert len(acc_path) == depth_ok + 1, (tree, seed, depth_ok, acc_path)
        assert bonus == cont[depth_ok]
        seen.add(depth_ok)
    assert len(seen) >= min(3, depth_max + 1)


def test_row_counts_of_the_sweep():
    cfg = synth.get_config("7b")
    rows = {t: bench.workload_template(synth, cfg, "7b", t).rows for t in bench.TREES}
    assert rows["full64"] == 68 and rows["efficient"] == 25 and rows["efficient-pernode"] == 105
    assert rows["full64-pernode"] == 320 and rows["full16"] == 20 and rows["full34-pernode"] == 170
