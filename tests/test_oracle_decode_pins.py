"""Pins for the oracle's whole step and decode loop (CPU only)."""
import numpy as np
import pytest
import torch

import oracle
import synth
from oracle.model import forward_rows, rope_rotate, rmsnorm
from oracle.tree import derive_template, ancestors_or_self
from oracle.decode import ar_greedy, bita_decode, prefill, BitaState, bita_step
from helpers import textbook_causal_attention

CFG = synth.get_config("tiny")


def _model(cfg=CFG, seed=0, **kw):
    w = synth.SynthWeights(cfg, seed=seed, **kw)
    return oracle.OracleModel(cfg, w), w


def _config1_template(seed=0):
    parent = synth.random_tree(8, 3, seed)
    return synth.attach_mask_groups(parent, [0], CFG.n_mask)


def _planted(cfg, d, stream, n_emitted, step, kmax):
    """Plant the known greedy continuation down to a step-dependent depth.  After
    n_emitted tokens the root's own successor is stream[n_emitted]."""
    rng = np.random.default_rng(1000 + step)
    depth_ok = int(rng.integers(0, d.tree_depth + 1))
    column = rng.integers(0, kmax, size=cfg.n_mask)
    cont = stream[n_emitted:]
    return synth.planted_candidates(cont, cfg.n_mask, kmax, depth_ok, column, cfg.vocab, 77 + step)


@pytest.mark.parametrize("mode", ["free", "planted"])
@pytest.mark.parametrize("topology", ["config1", "efficient_per_node", "full"])
def test_bita_stream_is_token_identical_to_ar_greedy(mode, topology):
    """The paper's losslessness claim: greedy BiTA output == plain AR greedy output."""
    model, _ = _model()
    ctx = synth.random_context(CFG.vocab, 64 if topology == "config1" else 24, 0)
    if topology == "config1":
        tmpl = _config1_template()
        steps = 16
    elif topology == "efficient_per_node":
        p = synth.efficient_tree_parents(CFG.n_mask, 3)
        tmpl = synth.attach_mask_groups(p, range(len(p)), CFG.n_mask)
        steps = 6
    else:
        p = synth.full_branching_tree([2, 2, 1])
        tmpl = synth.attach_mask_groups(p, [0], CFG.n_mask)
        steps = 8
    d = derive_template(tmpl.parent, tmpl.is_mask, tmpl.n_mask)
    ref = ar_greedy(model, ctx, steps * (d.tree_depth + 1) + 2)
    cand_fn = None
    if mode == "planted":
        cand_fn = lambda t, n_out: _planted(CFG, d, ref, n_out, t, d.kmax)  # noqa: E731
    out, trace, st = bita_decode(model, tmpl, ctx, steps, cand_fn)
    assert out == ref[: len(out)]
    lens = [r["n_acc"] for r in trace]
    assert all(1 <= n <= d.tree_depth + 1 for n in lens)
    assert sum(lens) == len(out)
    if mode == "planted":
        assert max(lens) >= 3 and len(set(lens)) >= 2  # several acceptance lengths exercised
    # committed cache == cache of a plain causal pass over the same tokens
    full = list(ctx) + out
    ck, cv = prefill(model, full[: st.cache_k[0].shape[0] + 1])
    for l in range(CFG.n_layers):
        assert np.allclose(st.cache_k[l], ck[l], rtol=1e-9, atol=1e-12)
        assert np.allclose(st.cache_v[l], cv[l], rtol=1e-9, atol=1e-12)


def test_garbage_drafts_never_change_the_stream():
    model, _ = _model()
    ctx = synth.random_context(CFG.vocab, 20, 5)
    tmpl = _config1_template(3)
    d = derive_template(tmpl.parent, tmpl.is_mask, tmpl.n_mask)
    ref = ar_greedy(model, ctx, 12)
    rng = np.random.default_rng(9)
    out, _, _ = bita_decode(model, tmpl, ctx, 6,
                            lambda t, n: rng.integers(0, CFG.vocab, size=(CFG.n_mask, d.kmax)).astype(np.int32))
    assert out == ref[: len(out)]


def test_tree_rows_equal_per_path_causal_decoding():
    """Tree attention == textbook causal attention over [cache | root..row path]:
    each row's logits must equal those of the last token of a plain causal pass over
    its own path, and its layer-0 attention output is recomputed here from scratch."""
    cfg = synth.get_config("tiny_gqa")
    model, w = _model(cfg, seed=2)
    ctx = synth.random_context(cfg.vocab, 12, 2)
    ck, cv = prefill(model, ctx)
    Lc = ck[0].shape[0]
    parent = synth.random_tree(9, 3, 4)
    tmpl = synth.attach_mask_groups(parent, [0, 2], cfg.n_mask)
    d = derive_template(tmpl.parent, tmpl.is_mask, tmpl.n_mask)
    rng = np.random.default_rng(3)
    tokens = list(rng.integers(0, cfg.vocab, size=d.T)) + [d.mask_index[r] for r in range(d.T, d.R)]
    pos = [Lc + d.depth[r] for r in range(d.R)]
    vis = [ancestors_or_self(d.parent, r) for r in range(d.R)]
    logits, nk, nv = forward_rows(model, tokens, d.is_mask, d.mask_index, pos, vis, ck, cv)
    for r in range(d.T):
        path = ancestors_or_self(d.parent, r)
        seq = list(ctx[:-1]) + [tokens[j] for j in path]
        n = len(seq)
        z = np.zeros((0, cfg.n_kv_heads, cfg.head_dim))
        lg, _, _ = forward_rows(model, seq, [0] * n, [-1] * n, list(range(n)),
                                [list(range(i + 1)) for i in range(n)],
                                [z] * cfg.n_layers, [z] * cfg.n_layers)
        assert np.allclose(lg[-1], logits[r], rtol=1e-9, atol=1e-11)
    # layer-0 attention of every row, rebuilt with the textbook routine (mask rows get the prefix
    # as extra leading keys that every position of their private sequence may see)
    x = np.stack([model.w("mask_emb")[d.mask_index[r]] if d.is_mask[r] else model.w("tok_emb")[tokens[r]]
                  for r in range(d.R)])
    h = rmsnorm(x, model.w("attn_norm", 0), cfg.rms_eps)
    Hq, Hkv, hd = cfg.n_heads, cfg.n_kv_heads, cfg.head_dim
    q = (h @ model.w("wq", 0).T).reshape(d.R, Hq, hd)
    for r in range(d.R):
        q[r] = rope_rotate(q[r], pos[r], cfg.rope_theta)
    assert np.allclose(nk[0], np.stack([rope_rotate((h[r] @ model.w("wk", 0).T).reshape(Hkv, hd), pos[r],
                                                    cfg.rope_theta) for r in range(d.R)]))
    from oracle.model import attend_row
    for r in range(d.R):
        path = ancestors_or_self(d.parent, r)
        ks = [ck[0], nk[0][path]]
        vs = [cv[0], nv[0][path]]
        if d.is_mask[r]:
            ks.insert(0, np.transpose(model.w("prompt_k", 0), (1, 0, 2)))
            vs.insert(0, np.transpose(model.w("prompt_v", 0), (1, 0, 2)))
        K, V = np.concatenate(ks), np.concatenate(vs)
        n = K.shape[0]
        Q = np.zeros((n, Hq, hd)); Q[-1] = q[r]
        ref = textbook_causal_attention(Q, K, V)[-1]
        got = attend_row(q[r], K, V, Hq, Hkv)
        assert np.allclose(ref, got, rtol=1e-11, atol=1e-13)


def test_chain_and_star_special_cases():
    model, _ = _model()
    ctx = synth.random_context(CFG.vocab, 10, 7)
    ck, cv = prefill(model, ctx)
    Lc = ck[0].shape[0]
    toks = [int(ctx[-1]), 5, 9, 33]
    # star: every child alone with the root == independent two-token continuations
    star = synth.star_tree(4)
    vis = [ancestors_or_self(star, r) for r in range(4)]
    lg_star, _, _ = forward_rows(model, toks, [0] * 4, [-1] * 4, [Lc, Lc + 1, Lc + 1, Lc + 1], vis, ck, cv)
    for c in (1, 2, 3):
        lg, _, _ = forward_rows(model, [toks[0], toks[c]], [0, 0], [-1, -1], [Lc, Lc + 1], [[0], [0, 1]], ck, cv)
        assert np.allclose(lg[1], lg_star[c], rtol=1e-10, atol=1e-12)
        assert np.allclose(lg[0], lg_star[0], rtol=1e-10, atol=1e-12)


def test_prefix_and_mask_embeddings_touch_mask_rows_only():
    """Prompt tokens influence only the mask tokens (Sec. 3.1): changing the prefix or
    the mask embeddings leaves every ordinary row's logits bit-identical and does
    change the mask rows'."""
    model, w = _model(seed=1)
    ctx = synth.random_context(CFG.vocab, 16, 1)
    tmpl = _config1_template(1)
    d = derive_template(tmpl.parent, tmpl.is_mask, tmpl.n_mask)
    cand = np.random.default_rng(0).integers(0, CFG.vocab, size=(CFG.n_mask, d.kmax)).astype(np.int32)
    st = BitaState(model, ctx)
    base = bita_step(model, d, st, cand)
    w2 = w.clone_cpu()
    g = torch.Generator().manual_seed(4)
    for l in range(CFG.n_layers):
        w2.set("prompt_k", l, torch.randn(CFG.n_kv_heads, CFG.n_prompt, CFG.head_dim, generator=g))
        w2.set("prompt_v", l, torch.randn(CFG.n_kv_heads, CFG.n_prompt, CFG.head_dim, generator=g))
    w2.set("mask_emb", None, torch.randn(CFG.n_mask, CFG.d_model, generator=g) * 0.5)
    model2 = oracle.OracleModel(CFG, w2)
    st2 = BitaState(model2, ctx)
    pert = bita_step(model2, d, st2, cand)
    assert np.array_equal(base["logits"][: d.T], pert["logits"][: d.T])
    assert np.abs(base["logits"][d.T:] - pert["logits"][d.T:]).max() > 1e-3
    # with P = 0 the mask rows only lose the prefix keys; ordinary rows again identical
    cfg0 = synth.get_config("tiny", n_prompt=0)
    w0 = w.clone_cpu(); w0.cfg = cfg0
    for l in range(CFG.n_layers):
        w0.set("prompt_k", l, torch.zeros(CFG.n_kv_heads, 0, CFG.head_dim))
        w0.set("prompt_v", l, torch.zeros(CFG.n_kv_heads, 0, CFG.head_dim))
    m0 = oracle.OracleModel(cfg0, w0)
    r0 = bita_step(m0, d, BitaState(m0, ctx), cand)
    assert np.array_equal(base["logits"][: d.T], r0["logits"][: d.T])


def test_planted_mistakes_are_caught():
    """Sanity of the pins themselves: typical slips, planted in a copy of the oracle's
    inputs, break token identity with AR greedy or the per-path equality."""
    model, _ = _model()
    ctx = synth.random_context(CFG.vocab, 16, 0)
    ck, cv = prefill(model, ctx)
    Lc = ck[0].shape[0]
    toks = [int(ctx[-1]), 5, 9]
    chain = synth.chain_tree(3)
    good, _, _ = forward_rows(model, toks, [0] * 3, [-1] * 3, [Lc, Lc + 1, Lc + 2],
                              [ancestors_or_self(chain, r) for r in range(3)], ck, cv)
    # (a) sibling leak: row 2 also sees row 1's sibling
    star = synth.star_tree(3)
    leak, _, _ = forward_rows(model, toks, [0] * 3, [-1] * 3, [Lc, Lc + 1, Lc + 1],
                              [[0], [0, 1], [0, 1, 2]], ck, cv)
    ok, _, _ = forward_rows(model, toks, [0] * 3, [-1] * 3, [Lc, Lc + 1, Lc + 1],
                            [ancestors_or_self(star, r) for r in range(3)], ck, cv)
    assert np.abs(leak[2] - ok[2]).max() > 1e-6
    # (b) position off by one
    bad, _, _ = forward_rows(model, toks, [0] * 3, [-1] * 3, [Lc, Lc + 1, Lc + 3],
                             [ancestors_or_self(chain, r) for r in range(3)], ck, cv)
    assert np.abs(bad[2] - good[2]).max() > 1e-6
