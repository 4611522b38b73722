"""Pins for the oracle's model arithmetic (CPU only)."""
import numpy as np
import pytest
import torch

import oracle
import synth
from oracle.model import rmsnorm, rope_rotate, silu, attend_row, forward_rows, topk_desc, argmax_low
from helpers import textbook_causal_attention


def _hf_model(cfg, w):
    from transformers import LlamaConfig, LlamaForCausalLM
    hc = LlamaConfig(hidden_size=cfg.d_model, intermediate_size=cfg.d_ffn,
                     num_hidden_layers=cfg.n_layers, num_attention_heads=cfg.n_heads,
                     num_key_value_heads=cfg.n_kv_heads, vocab_size=cfg.vocab,
                     rms_norm_eps=cfg.rms_eps, rope_theta=cfg.rope_theta,
                     max_position_embeddings=512, tie_word_embeddings=False,
                     attention_bias=False, mlp_bias=False, head_dim=cfg.head_dim,
                     attn_implementation="eager")
    m = LlamaForCausalLM(hc).to(torch.float64).eval()
    sd = m.state_dict()

    def put(key, name, layer=None):
        sd[key].copy_(w.torch(name, layer).to(torch.float64))
    put("model.embed_tokens.weight", "tok_emb")
    put("model.norm.weight", "final_norm")
    put("lm_head.weight", "lm_head")
    for l in range(cfg.n_layers):
        p = f"model.layers.{l}."
        for hf, mine in (("self_attn.q_proj", "wq"), ("self_attn.k_proj", "wk"),
                         ("self_attn.v_proj", "wv"), ("self_attn.o_proj", "wo"),
                         ("mlp.gate_proj", "w_gate"), ("mlp.up_proj", "w_up"),
                         ("mlp.down_proj", "w_down"), ("input_layernorm", "attn_norm"),
                         ("post_attention_layernorm", "ffn_norm")):
            put(p + hf + ".weight", mine, l)
    return m


def _weights_with_random_gains(cfg, seed):
    w = synth.SynthWeights(cfg, seed=seed)
    g = torch.Generator().manual_seed(seed + 100)
    for l in range(cfg.n_layers):
        for nm in ("attn_norm", "ffn_norm"):
            w.set(nm, l, 1 + 0.3 * torch.randn(cfg.d_model, generator=g))
    w.set("final_norm", None, 1 + 0.3 * torch.randn(cfg.d_model, generator=g))
    return w


@pytest.mark.parametrize("name", ["tiny", "tiny_gqa"])
def test_causal_forward_matches_huggingface_llama(name):
    """Whole-model pin: RMSNorm gains and eps, rotary pairing, GQA head mapping,
    SwiGLU and LM head against an independent LLaMA implementation.  The library
    evaluates its rotary table in float32, hence 1e-5 rather than 1e-12."""
    cfg = synth.get_config(name)
    w = _weights_with_random_gains(cfg, 3)
    ctx = synth.random_context(cfg.vocab, 24, 1)
    with torch.no_grad():
        ref = _hf_model(cfg, w)(torch.tensor(ctx[None].astype(np.int64))).logits[0].numpy()
    om = oracle.OracleModel(cfg, w)
    z = np.zeros((0, cfg.n_kv_heads, cfg.head_dim))
    n = len(ctx)
    lg, _, _ = forward_rows(om, list(ctx), [0] * n, [-1] * n, list(range(n)),
                            [list(range(r + 1)) for r in range(n)],
                            [z] * cfg.n_layers, [z] * cfg.n_layers)
    assert np.abs(ref).max() > 0.5
    assert np.abs(lg - ref).max() < 1e-5


def test_rmsnorm_closed_forms():
    d = 64
    g = np.linspace(0.5, 1.5, d)
    # constant vector c: c / sqrt(c^2 + eps) * g
    c = 3.0
    out = rmsnorm(np.full(d, c), g, 1e-5)
    assert np.allclose(out, c / np.sqrt(c * c + 1e-5) * g, rtol=1e-14)
    # against torch's rms_norm
    x = np.random.default_rng(0).normal(size=(5, d))
    ref = torch.nn.functional.rms_norm(torch.tensor(x), (d,), torch.tensor(g), 1e-5).numpy()
    assert np.allclose(rmsnorm(x, g, 1e-5), ref, rtol=1e-13, atol=1e-15)
    # zero vector stays zero (inactive rows)
    assert np.all(rmsnorm(np.zeros(d), g, 1e-5) == 0)


def test_rope_properties():
    rng = np.random.default_rng(1)
    hd, theta = 64, 10000.0
    q, k = rng.normal(size=hd), rng.normal(size=hd)
    # position 0 is the identity
    assert np.array_equal(rope_rotate(q, 0, theta), q)
    # norm preserving
    assert np.isclose(np.linalg.norm(rope_rotate(q, 37, theta)), np.linalg.norm(q), rtol=1e-13)
    # scores depend on the position difference only
    a = rope_rotate(q, 100, theta) @ rope_rotate(k, 93, theta)
    b = rope_rotate(q, 1007, theta) @ rope_rotate(k, 1000, theta)
    assert np.isclose(a, b, rtol=1e-9, atol=1e-11)
    # first pair rotates by exactly pos radians, last pair by pos * theta^(-(hd-2)/hd)
    e = np.zeros(hd); e[0] = 1.0
    r = rope_rotate(e, 2, theta)
    assert np.isclose(r[0], np.cos(2.0)) and np.isclose(r[hd // 2], np.sin(2.0))
    e = np.zeros(hd); e[hd // 2 - 1] = 1.0
    ang = 5 * theta ** (-(hd - 2) / hd)
    r = rope_rotate(e, 5, theta)
    assert np.isclose(r[hd // 2 - 1], np.cos(ang)) and np.isclose(r[hd - 1], np.sin(ang))


def test_silu_and_swiglu_against_torch():
    x = np.linspace(-6, 6, 41)
    assert np.allclose(silu(x), torch.nn.functional.silu(torch.tensor(x)).numpy(), rtol=1e-14)


def test_attend_row_matches_textbook_last_row():
    rng = np.random.default_rng(2)
    n, Hq, Hkv, hd = 9, 4, 2, 16
    q = rng.normal(size=(n, Hq, hd)); k = rng.normal(size=(n, Hkv, hd)); v = rng.normal(size=(n, Hkv, hd))
    ref = textbook_causal_attention(q, k, v)
    for r in range(n):
        out = attend_row(q[r], k[: r + 1], v[: r + 1], Hq, Hkv)
        assert np.allclose(out, ref[r], rtol=1e-12, atol=1e-14)
    # and against torch SDPA with GQA expanded by hand
    tq = torch.tensor(q).permute(1, 0, 2)[None]
    tk = torch.tensor(np.repeat(k, Hq // Hkv, axis=1)).permute(1, 0, 2)[None]
    tv = torch.tensor(np.repeat(v, Hq // Hkv, axis=1)).permute(1, 0, 2)[None]
    sd = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].permute(1, 0, 2).numpy()
    assert np.allclose(ref, sd, rtol=1e-10, atol=1e-12)


def test_attend_row_single_key_returns_value():
    rng = np.random.default_rng(3)
    q = rng.normal(size=(4, 8)); k = rng.normal(size=(1, 4, 8)); v = rng.normal(size=(1, 4, 8))
    assert np.allclose(attend_row(q, k, v, 4, 4), v[0])


def test_topk_and_argmax_tie_rules():
    row = np.array([1.0, 5.0, 3.0, 5.0, 2.0, 3.0], np.float32)
    assert argmax_low(row) == 1
    ids, vals = topk_desc(row, 4)
    assert list(ids) == [1, 3, 2, 5] and list(vals) == [5.0, 5.0, 3.0, 3.0]
    # against a stable sort on random data with many ties
    rng = np.random.default_rng(4)
    for _ in range(20):
        r = rng.integers(0, 8, size=50).astype(np.float32)
        ids, vals = topk_desc(r, 7)
        order = sorted(range(50), key=lambda i: (-r[i], i))[:7]
        assert list(ids) == order
        assert argmax_low(r) == order[0]


def test_absent_rows_are_zero_and_invisible():
    """A tree row without a candidate (negative token) is absent from the pass: zero hidden
    state, zero K/V, zero logits, and the rows that are present compute exactly what they
    compute in a pass from which the absent rows are removed."""
    cfg = synth.get_config("tiny")
    om = oracle.OracleModel(cfg, synth.SynthWeights(cfg, seed=3, norm_std=0.3, prefix_std=1.0))
    rng = np.random.default_rng(0)
    ck = [rng.normal(size=(5, cfg.n_kv_heads, cfg.head_dim)) for _ in range(cfg.n_layers)]
    cv = [rng.normal(size=(5, cfg.n_kv_heads, cfg.head_dim)) for _ in range(cfg.n_layers)]
    # root, two children, a grandchild of the second child, one mask row on the root; row 2 and its child 3 absent
    parent = [-1, 0, 0, 2, 0]
    is_mask = [0, 0, 0, 0, 1]
    tokens = [7, 11, -1, -1, 0]
    pos = [5, 6, 6, 7, 6]
    vis = [[0], [0, 1], [0, 2], [0, 2, 3], [0, 4]]
    lg, k, v = oracle.forward_rows(om, tokens, is_mask, [-1, -1, -1, -1, 0], pos, vis, ck, cv)
    for r in (2, 3):
        assert np.all(lg[r] == 0)
        assert all(np.all(k[l][r] == 0) and np.all(v[l][r] == 0) for l in range(cfg.n_layers))
    keep = [0, 1, 4]
    lg2, k2, v2 = oracle.forward_rows(om, [7, 11, 0], [0, 0, 1], [-1, -1, 0], [5, 6, 6], [[0], [0, 1], [0, 2]], ck, cv)
    # (equal up to the summation order of the library matmul at another row count)
    assert np.allclose(lg[keep], lg2, rtol=1e-11, atol=1e-13)
    for l in range(cfg.n_layers):
        assert np.allclose(k[l][keep], k2[l], rtol=1e-11, atol=1e-13) and np.allclose(v[l][keep], v2[l], rtol=1e-11, atol=1e-13)
