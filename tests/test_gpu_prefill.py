"""Context prefill through the C ABI (chunked chain passes) against the oracle's single
causal pass: committed K/V, context counters and the first greedy token."""
import numpy as np
import pytest
import torch

import oracle
import synth
from oracle.model import argmax_low
from gpu_util import dev_i32, read_cache

pytestmark = pytest.mark.gpu

KV_TOL = 3e-2         # same bar as the step tests put on a pass' K/V rows
MARGIN = 6e-2


@pytest.fixture(scope="module")
def bita():
    import paper_2401_12522_amd as b
    b.lib()
    return b


def _oracle_causal(om, toks):
    """K/V and last-row logits of one causal pass over toks from an empty cache."""
    cfg = om.cfg
    n = len(toks)
    ck = [np.zeros((0, cfg.n_kv_heads, cfg.head_dim)) for _ in range(cfg.n_layers)]
    cv = [np.zeros((0, cfg.n_kv_heads, cfg.head_dim)) for _ in range(cfg.n_layers)]
    vis = [list(range(r + 1)) for r in range(n)]
    logits, k, v = oracle.forward_rows(om, list(toks), [0] * n, [-1] * n, list(range(n)), vis, ck, cv)
    return k, v, logits[n - 1]


def _margin(row):
    s = np.sort(row)
    return s[-1] - s[-2]


@pytest.mark.parametrize("cfg_name,n_ctx,chunk", [("tiny", 150, 64), ("tiny_gqa", 150, 256), ("tiny_gqa", 97, 17),
                                                  ("tiny", 600, 512)])      # 512 rows: the largest template
def test_prefill_chunks_match_one_causal_pass(bita, cfg_name, n_ctx, chunk):
    cfg = synth.get_config(cfg_name)
    w = synth.SynthWeights(cfg, seed=3)
    om = oracle.OracleModel(cfg, w)
    smax = 256 if n_ctx <= 256 else 640
    model = bita.Model(cfg, w, max_pos=smax + 64)
    kv = bita.KVState(cfg, cfg.n_layers, 1, smax, chunk)
    ctx = synth.random_context(cfg.vocab, n_ctx, 11)
    nxt = bita.prefill(model, kv, 0, dev_i32(ctx[None]), chunk)
    torch.cuda.synchronize()
    assert int(kv.ctx_len[0]) == n_ctx
    k, v, last = _oracle_causal(om, ctx)
    gk, gv = read_cache(kv)
    for l in range(cfg.n_layers):
        assert gk[l].shape == k[l].shape
        assert np.abs(gk[l] - k[l]).max() <= KV_TOL
        assert np.abs(gv[l] - v[l]).max() <= KV_TOL
    # slots past the context stay untouched (the cache starts zeroed)
    assert not kv.k_cache[:, 0, :, n_ctx:].any() and not kv.v_cache[:, 0, :, n_ctx:].any()
    if _margin(last) > MARGIN:
        assert int(nxt[0]) == argmax_low(last)
    else:
        assert 0 <= int(nxt[0]) < cfg.vocab


def test_prefill_ragged_batch_in_two_calls(bita):
    """Three sequences of different lengths (one empty), filled by two calls: the second call
    appends to what the first committed.  Each sequence equals its own causal pass."""
    cfg = synth.get_config("tiny_gqa")
    w = synth.SynthWeights(cfg, seed=5)
    om = oracle.OracleModel(cfg, w)
    smax, chunk, B = 256, 48, 3
    model = bita.Model(cfg, w, max_pos=smax + 64)
    kv = bita.KVState(cfg, cfg.n_layers, B, smax, chunk)
    lens = [131, 37, 0]
    first = [60, 37, 0]                                  # tokens handed over by the first call
    ctxs = [synth.random_context(cfg.vocab, max(n, 1), 40 + b)[:n] for b, n in enumerate(lens)]

    def padded(parts):
        width = max(max(len(p) for p in parts), 1)
        out = np.full((B, width), -7, np.int32)           # padding is never read as a token
        for b, p in enumerate(parts):
            out[b, :len(p)] = p
        return dev_i32(out)
    n1 = bita.prefill(model, kv, 0, padded([c[:f] for c, f in zip(ctxs, first)]), chunk, seq_len=dev_i32(first))
    torch.cuda.synchronize()
    assert kv.ctx_len.cpu().tolist() == first
    rest = [len(c) - f for c, f in zip(ctxs, first)]
    n2 = bita.prefill(model, kv, max(first), padded([c[f:] for c, f in zip(ctxs, first)]), chunk, seq_len=dev_i32(rest))
    torch.cuda.synchronize()
    assert kv.ctx_len.cpu().tolist() == lens
    assert int(n1[2]) == -1 and int(n2[2]) == -1          # an empty sequence has no next token
    assert int(n2[1]) == -1                               # nothing of sequence 1 in the second call
    for b in range(B):
        if lens[b] == 0:
            continue
        k, v, last = _oracle_causal(om, ctxs[b])
        gk, gv = read_cache(kv, b=b)
        for l in range(cfg.n_layers):
            assert np.abs(gk[l] - k[l]).max() <= KV_TOL
            assert np.abs(gv[l] - v[l]).max() <= KV_TOL
        got = int(n2[b]) if rest[b] > 0 else int(n1[b])
        if _margin(last) > MARGIN:
            assert got == argmax_low(last)


def test_prefill_rejects_what_does_not_fit(bita):
    cfg = synth.get_config("tiny")
    w = synth.SynthWeights(cfg, seed=1)
    model = bita.Model(cfg, w, max_pos=96)
    kv = bita.KVState(cfg, cfg.n_layers, 1, 64, 32)
    toks = dev_i32(synth.random_context(cfg.vocab, 80, 2)[None])
    with pytest.raises(bita.BitaError) as e:
        bita.prefill(model, kv, 0, toks, 32)              # 80 tokens into 64 slots
    assert e.value.code == -3
    with pytest.raises(bita.BitaError) as e:
        bita.prefill(model, kv, 0, toks[:, :40].contiguous(), 33)   # scratch holds 32 rows
    assert e.value.code == -1
    # an empty context is a no-op, not an error
    nxt = bita.prefill(model, kv, 0, torch.zeros((1, 0), dtype=torch.int32, device="cuda"), 32)
    torch.cuda.synchronize()
    assert int(nxt[0]) == -1
    assert int(kv.ctx_len[0]) == 0 and not kv.k_cache.any()


def test_prompt_to_tokens_on_the_device_alone(bita):
    """The whole decoder with no oracle data on the device: prefill of the full prompt gives the
    first token, then the first step runs with no candidates (Algorithm 1, t = 1: only the root
    and its mask rows are live) and later steps draft for themselves.  The emitted stream is the
    oracle's autoregressive greedy stream wherever its top-2 margin is decisive."""
    cfg = synth.get_config("tiny")
    tin = synth.attach_mask_groups(synth.random_tree(8, 3, 0), [0], cfg.n_mask)
    w = synth.SynthWeights(cfg, seed=0)
    om = oracle.OracleModel(cfg, w)
    d = oracle.tree.derive_template(tin.parent, tin.is_mask, tin.n_mask)
    smax, steps = 256, 12
    model = bita.Model(cfg, w, max_pos=smax + 64)
    tmpl = bita.TreeTemplate(tin.parent, tin.is_mask, tin.n_tree, tin.n_mask)
    kv = bita.KVState(cfg, cfg.n_layers, 1, smax, max(tmpl.rows, 32))
    ctx = synth.random_context(cfg.vocab, 64, 0)
    # oracle: greedy stream and margins, one token per pass
    ck, cv = oracle.decode.prefill(om, ctx)
    ref, margins = [], []
    last = int(ctx[-1])
    for _ in range(steps * (d.tree_depth + 1) + 2):
        lg, k, v = oracle.forward_rows(om, [last], [0], [-1], [ck[0].shape[0]], [[0]], ck, cv)
        ck, cv = oracle.compact_kv(ck, cv, k, v, [0])
        last = argmax_low(lg[0])
        ref.append(last)
        margins.append(_margin(lg[0]))
    # device: prompt -> first token -> steps
    first = bita.prefill(model, kv, 0, dev_i32(ctx[None]), 32)
    emitted = [int(first[0])]
    kv.resize_rows(cfg.n_layers, cfg, tmpl.rows)
    buf = bita.StepBuffers(model, tmpl, 1, d.kmax)
    buf.bonus.copy_(first)
    buf.next_shift[0] = cfg.n_mask                       # t = 1: no candidates yet
    lens = []
    for t in range(steps):
        hint = len(ctx) + t * (d.tree_depth + 1)
        bita.decode_step(model, kv, hint, tmpl, buf, 1, buf.bonus, buf.topk_ids, buf.next_group, buf.next_shift)
        torch.cuda.synchronize()
        na = int(buf.n_acc[0])
        if t == 0:
            assert na == 1 and buf.token[0, 1:tmpl.n_tree].cpu().tolist() == [-1] * (tmpl.n_tree - 1)
        lens.append(na)
        emitted.extend(buf.emitted[0, :na].cpu().tolist())
    low = [i for i in range(len(emitted)) if margins[i] <= MARGIN]
    upto = low[0] if low else len(emitted)
    assert upto >= 8, "seed gives an early near-tie; pick another"
    assert emitted[:upto] == ref[:upto]
    assert int(kv.ctx_len[0]) == len(ctx) + sum(lens)


def test_prefill_and_first_step_replay_from_one_graph(bita):
    """bita_prefill allocates nothing and never waits for the stream once the model holds its
    chain templates: prefill of the prompt and the first step are captured into one HIP graph
    and replayed on reset state three times, with eager work in between; every replay gives the
    eager run's bits, and the tokens are the oracle's greedy ones where its margin is decisive."""
    cfg = synth.get_config("tiny_gqa")
    tin = synth.attach_mask_groups(synth.random_tree(8, 3, 0), [0], cfg.n_mask)
    w = synth.SynthWeights(cfg, seed=2, norm_std=0.3, prefix_std=1.0)
    om = oracle.OracleModel(cfg, w)
    d = oracle.tree.derive_template(tin.parent, tin.is_mask, tin.n_mask)
    smax, chunk, n_ctx = 256, 32, 75                     # two full chunks and a ragged one of 11 rows
    model = bita.Model(cfg, w, max_pos=smax + 64)
    tmpl = bita.TreeTemplate(tin.parent, tin.is_mask, tin.n_tree, tin.n_mask)
    kv = bita.KVState(cfg, cfg.n_layers, 1, smax, chunk)
    kv_step = bita.KVState.__new__(bita.KVState)         # the same memory, laid out for the step's rows
    kv_step.__dict__.update(kv.__dict__)
    kv_step.resize_rows(cfg.n_layers, cfg, tmpl.rows)
    ctx = synth.random_context(cfg.vocab, n_ctx, 5)
    toks = dev_i32(ctx[None])
    ws = bita.prefill_workspace(model, 1, chunk)
    first = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    buf = bita.StepBuffers(model, tmpl, 1, d.kmax, want_logits=True)
    shift0 = dev_i32([cfg.n_mask])                       # t = 1: no candidates yet

    def reset():
        kv.ctx_len.zero_(); kv.k_cache.zero_(); kv.v_cache.zero_(); first.fill_(-1)

    def run():
        bita.prefill(model, kv, 0, toks, chunk, workspace=ws, next_token=first)
        bita.decode_step(model, kv_step, n_ctx, tmpl, buf, 1, first, buf.topk_ids, None, shift0)

    bita.prefill_prepare(model, n_ctx, chunk)
    reset()
    run()                                                # eager
    torch.cuda.synchronize()
    eager = [first.clone(), buf.logits.clone(), buf.bonus.clone(), kv.k_cache.clone(), kv.ctx_len.clone()]
    assert int(kv.ctx_len[0]) == n_ctx + 1
    graph = torch.cuda.CUDAGraph()
    st = torch.cuda.Stream()
    reset()
    with torch.cuda.stream(st):
        with torch.cuda.graph(graph, stream=st):
            run()
    torch.cuda.synchronize()
    for rep in range(3):
        reset()
        buf.logits.fill_(7.0)
        (torch.ones(1 << 20, device="cuda") * 3).sum().item()   # the program's own eager work between replays
        graph.replay()
        torch.cuda.synchronize()
        got = [first, buf.logits, buf.bonus, kv.k_cache, kv.ctx_len]
        for a, b_ in zip(eager, got):
            assert torch.equal(a, b_), rep
    # against the oracle: the token after the prompt
    _, _, last = _oracle_causal(om, [int(x) for x in ctx])
    if _margin(last) > MARGIN:
        assert int(first[0]) == argmax_low(last)


def test_prefill_on_a_capturing_stream_needs_its_templates(bita):
    """A capturing stream that finds no chain template is refused, not served by an allocation."""
    cfg = synth.get_config("tiny")
    w = synth.SynthWeights(cfg, seed=1)
    model = bita.Model(cfg, w, max_pos=128)
    kv = bita.KVState(cfg, cfg.n_layers, 1, 96, 32)
    toks = dev_i32(synth.random_context(cfg.vocab, 50, 2)[None])
    ws = bita.prefill_workspace(model, 1, 32)
    first = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    bita.prefill(model, kv, 0, toks, 32, workspace=ws, next_token=first)      # eager: creates 32 and 18
    torch.cuda.synchronize()
    kv.ctx_len.zero_()
    graph, st = torch.cuda.CUDAGraph(), torch.cuda.Stream()
    torch.cuda.synchronize()
    with pytest.raises(bita.BitaError) as e:
        with torch.cuda.stream(st):
            with torch.cuda.graph(graph, stream=st):
                bita.prefill(model, kv, 0, toks, 29, workspace=ws, next_token=first)   # chunks of 29 and 21: unknown
    assert e.value.code == -1 and "bita_prefill_prepare" in str(e.value)
    torch.cuda.synchronize()
    assert int(kv.ctx_len[0]) == 0
