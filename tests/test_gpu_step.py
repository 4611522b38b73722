"""Whole-step parity (GPU) on the small configuration: tokens, logits, selections,
acceptance and K/V commit against the oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import synth
from oracle.model import topk_desc, argmax_low
from oracle.tree import derive_template, accept_walk, next_group_and_shift
from oracle.decode import ar_greedy, BitaState, bita_step
from gpu_util import dev_i32, load_cache, read_cache, round_state

pytestmark = pytest.mark.gpu

LOGIT_TOL = 3e-2      # max-abs, bf16 path
MARGIN = 6e-2         # argmax must agree wherever the oracle's top-2 gap exceeds this


@pytest.fixture(scope="module")
def bita():
    import paper_2401_12522_amd as b
    b.lib()
    return b


def _setup(bita, cfg_name, tmpl_in, seed=0, smax=256, batch=1):
    cfg = synth.get_config(cfg_name)
    w = synth.SynthWeights(cfg, seed=seed)
    om = oracle.OracleModel(cfg, w)
    model = bita.Model(cfg, w, max_pos=smax + 64)
    tmpl = bita.TreeTemplate(tmpl_in.parent, tmpl_in.is_mask, tmpl_in.n_tree, tmpl_in.n_mask)
    kv = bita.KVState(cfg, cfg.n_layers, batch, smax, tmpl.rows)
    d = derive_template(tmpl_in.parent, tmpl_in.is_mask, tmpl_in.n_mask)
    return cfg, w, om, model, tmpl, kv, d


def _check_selection_bit_exact(buf, d, logits_gpu, b=0):
    """Given the GPU's own fp32 logits, argmax and top-k must equal the oracle's selection
    rule applied to exactly those numbers."""
    for r in range(d.T):
        assert int(buf.argmax[b, r]) == argmax_low(logits_gpu[r])
    for g in range(d.G):
        for i, r in enumerate(d.group_rows[g]):
            ids, vals = topk_desc(logits_gpu[r], buf.kmax)
            assert buf.topk_ids[b, g * d.n_mask + i].cpu().tolist() == list(ids)
            assert np.array_equal(buf.topk_val[b, g * d.n_mask + i].cpu().numpy(), vals)


def _top2_margin(row):
    s = np.sort(row)
    return s[-1] - s[-2]


@pytest.mark.parametrize("cfg_name,topology", [("tiny", "config1"), ("tiny_gqa", "config1"),
                                               ("tiny", "per_node"), ("tiny", "full")])
def test_step_by_step_against_oracle(bita, cfg_name, topology):
    """Each step starts from the oracle's (bf16-representable) cache, so one step's
    rounding cannot compound into the next comparison."""
    base = synth.get_config(cfg_name)
    if topology == "config1":
        tin = synth.attach_mask_groups(synth.random_tree(8, 3, 0), [0], base.n_mask)
    elif topology == "per_node":
        p = synth.efficient_tree_parents(base.n_mask, 3)
        tin = synth.attach_mask_groups(p, range(len(p)), base.n_mask)
    else:
        tin = synth.attach_mask_groups(synth.full_branching_tree([3, 2, 2, 1]), [0], base.n_mask)
    cfg, w, om, model, tmpl, kv, d = _setup(bita, cfg_name, tin)
    ctx = synth.random_context(cfg.vocab, 64, 0)
    steps = 16 if topology == "config1" else 6
    ref_stream = ar_greedy(om, ctx, steps * (d.tree_depth + 1) + 1)
    st = round_state(BitaState(om, ctx))
    buf = bita.StepBuffers(model, tmpl, 1, d.kmax, want_logits=True)
    out = []
    seen = set()
    for t in range(steps):
        rng = np.random.default_rng(100 + t)
        depth_ok = int(rng.integers(0, d.tree_depth + 1))
        cand = synth.planted_candidates(ref_stream[len(out):], cfg.n_mask, d.kmax, depth_ok,
                                        np.zeros(cfg.n_mask, int) if topology == "per_node" else rng.integers(0, d.kmax, cfg.n_mask),
                                        cfg.vocab, 7 + t)
        cand_full = np.tile(cand, (max(d.G, 1), 1))
        Lc = load_cache(kv, st.cache_k, st.cache_v)
        root = st.root_token
        st_before_k, st_before_v = [x.copy() for x in st.cache_k], [x.copy() for x in st.cache_v]
        ref = bita_step(om, d, st, cand)
        bita.decode_step(model, kv, Lc, tmpl, buf, 1, dev_i32([root]), dev_i32(cand_full[None]))
        torch.cuda.synchronize()
        assert buf.token[0].cpu().tolist() == ref["tokens"]
        lg = buf.logits[0].cpu().numpy()
        assert np.isfinite(lg).all()
        err = np.abs(lg - ref["logits"]).max()
        assert err <= LOGIT_TOL, (t, err)
        _check_selection_bit_exact(buf, d, lg)
        gpu_greedy = buf.argmax[0].cpu().tolist()
        for r in range(d.T):
            if _top2_margin(ref["logits"][r]) > MARGIN:
                assert gpu_greedy[r] == ref["greedy"][r], (t, r)
        # acceptance is integer-exact given the same greedy tokens: replay the oracle's walk
        # on the GPU's own argmax (identical to the oracle's wherever the margin is decisive)
        path, bonus = accept_walk(d, ref["tokens"], gpu_greedy)
        na = len(path)
        assert int(buf.n_acc[0]) == na and buf.path[0, :na].cpu().tolist() == path
        assert int(buf.bonus[0]) == bonus
        assert buf.emitted[0, :na].cpu().tolist() == [ref["tokens"][c] for c in path[1:]] + [bonus]
        assert (int(buf.next_group[0]), int(buf.next_shift[0])) == next_group_and_shift(d, path)
        assert int(kv.ctx_len[0]) == Lc + na
        if gpu_greedy == ref["greedy"]:
            assert path == ref["path"] and bonus == ref["bonus"]
        # committed rows are bit copies of the pass' own K/V rows ...
        for l in range(cfg.n_layers):
            assert torch.equal(kv.k_cache[l, 0][:, Lc:Lc + na], kv.k_tree[l, 0][:, path])
            assert torch.equal(kv.v_cache[l, 0][:, Lc:Lc + na], kv.v_tree[l, 0][:, path])
            # ... and the pass' K/V rows match the oracle's to bf16 resolution
            got_k = kv.k_tree[l, 0].permute(1, 0, 2).to(torch.float64).cpu().numpy()
            got_v = kv.v_tree[l, 0].permute(1, 0, 2).to(torch.float64).cpu().numpy()
            assert np.abs(got_k - ref["new_k"][l]).max() < 3e-2
            assert np.abs(got_v - ref["new_v"][l]).max() < 3e-2
        # cache slots below ctx_len untouched
        ks, vs = read_cache(kv)
        for l in range(cfg.n_layers):
            assert np.array_equal(ks[l][:Lc], st_before_k[l]) and np.array_equal(vs[l][:Lc], st_before_v[l])
        seen.add(na)
        out.extend(ref["emitted"])
        round_state(st)
    assert out == ref_stream[: len(out)]
    assert len(seen) >= 2


@pytest.mark.parametrize("mode", ["free", "planted"])
def test_autonomous_gpu_loop_reproduces_ar_greedy(bita, mode):
    """16 steps on the device with no host round trip inside a step: the emitted stream is
    token-identical to plain autoregressive greedy decoding (the method is lossless)."""
    base = synth.get_config("tiny")
    tin = synth.attach_mask_groups(synth.random_tree(8, 3, 0), [0], base.n_mask)
    cfg, w, om, model, tmpl, kv, d = _setup(bita, "tiny", tin)
    ctx = synth.random_context(cfg.vocab, 64, 0)
    steps = 16
    n_ref = steps * (d.tree_depth + 1) + 1
    # oracle AR stream with its margins
    ck, cv = oracle.decode.prefill(om, ctx)
    ref, margins = [], []
    last = int(ctx[-1])
    for _ in range(n_ref):
        lg, k, v = oracle.forward_rows(om, [last], [0], [-1], [ck[0].shape[0]], [[0]], ck, cv)
        ck, cv = oracle.compact_kv(ck, cv, k, v, [0])
        last = argmax_low(lg[0])
        ref.append(last)
        margins.append(_top2_margin(lg[0]))
    st0 = round_state(BitaState(om, ctx))
    Lc0 = load_cache(kv, st0.cache_k, st0.cache_v)
    buf = bita.StepBuffers(model, tmpl, 1, d.kmax)
    buf.bonus[0] = int(ctx[-1])
    buf.next_shift[0] = cfg.n_mask            # first pass: no candidates yet, all drafts inactive
    emitted, lens = [], []
    planted = []
    pos = 0
    if mode == "planted":
        # acceptance lengths follow from the plan, so every table can be prepared up front
        for t in range(steps):
            rng = np.random.default_rng(500 + t)
            depth_ok = int(rng.integers(0, d.tree_depth + 1))
            planted.append((pos, depth_ok, rng.integers(0, d.kmax, cfg.n_mask)))
            pos += 0  # actual advance is read back below; tables are built lazily per step
    for t in range(steps):
        hint = Lc0 + t * (d.tree_depth + 1)
        if mode == "free":
            bita.decode_step(model, kv, hint, tmpl, buf, 1, buf.bonus, buf.topk_ids, buf.next_group, buf.next_shift)
        else:
            _, depth_ok, col = planted[t]
            cand = synth.planted_candidates(ref[len(emitted):], cfg.n_mask, d.kmax, depth_ok, col, cfg.vocab, 9 + t)
            bita.decode_step(model, kv, hint, tmpl, buf, 1, buf.bonus, dev_i32(cand[None]))
        torch.cuda.synchronize()
        na = int(buf.n_acc[0])
        lens.append(na)
        emitted.extend(buf.emitted[0, :na].cpu().tolist())
    n_ok = len(emitted)
    low = [i for i in range(n_ok) if margins[i] <= MARGIN]
    upto = low[0] if low else n_ok
    assert upto >= 8, "seed gives an early near-tie; pick another"
    assert emitted[:upto] == ref[:upto]
    assert int(kv.ctx_len[0]) == Lc0 + sum(lens)
    assert all(1 <= n <= d.tree_depth + 1 for n in lens)
    if mode == "planted" and not low:
        assert max(lens) >= 3


def test_batched_steps_with_ragged_contexts_and_accepts(bita):
    """Batch 3, independent sequences: different context lengths, planted drafts of different
    depths per sequence and step.  Every sequence's stream equals its own autoregressive greedy
    stream, its context counter advances by its own accepted lengths, and the committed K/V
    equal the oracle's causal-pass cache."""
    base = synth.get_config("tiny_gqa")
    tin = synth.attach_mask_groups(synth.random_tree(8, 3, 3), [0], base.n_mask)
    B = 3
    cfg, w, om, model, tmpl, kv, d = _setup(bita, "tiny_gqa", tin, batch=B)
    ctx_lens, ctx_seeds = [40, 64, 57], [31, 105, 56]    # seeds whose first 33 greedy tokens have decisive margins
    steps = 8
    n_ref = steps * (d.tree_depth + 1) + 1
    refs, margins, ctxs, Lc0 = [], [], [], []
    for b in range(B):
        ctx = synth.random_context(cfg.vocab, ctx_lens[b], ctx_seeds[b])
        ctxs.append(ctx)
        ck, cv = oracle.decode.prefill(om, ctx)
        ref, mar = [], []
        last = int(ctx[-1])
        for _ in range(n_ref):
            lg, k, v = oracle.forward_rows(om, [last], [0], [-1], [ck[0].shape[0]], [[0]], ck, cv)
            ck, cv = oracle.compact_kv(ck, cv, k, v, [0])
            last = argmax_low(lg[0])
            ref.append(last)
            mar.append(_top2_margin(lg[0]))
        refs.append(ref)
        margins.append(mar)
        st0 = round_state(BitaState(om, ctx))
        Lc0.append(load_cache(kv, st0.cache_k, st0.cache_v, b=b))
    buf = bita.StepBuffers(model, tmpl, B, d.kmax)
    for b in range(B):
        buf.bonus[b] = int(ctxs[b][-1])
        buf.next_shift[b] = cfg.n_mask
    emitted = [[] for _ in range(B)]
    lens = [[] for _ in range(B)]
    for t in range(steps):
        hint = max(Lc0[b] + sum(lens[b]) for b in range(B))
        cand = np.zeros((B, cfg.n_mask, d.kmax), np.int32)
        for b in range(B):
            rng = np.random.default_rng(900 + 10 * t + b)
            depth_ok = int(rng.integers(0, d.tree_depth + 1))
            col = rng.integers(0, d.kmax, cfg.n_mask)
            cand[b] = synth.planted_candidates(refs[b][len(emitted[b]):], cfg.n_mask, d.kmax, depth_ok, col,
                                               cfg.vocab, 77 + 10 * t + b)
        bita.decode_step(model, kv, hint, tmpl, buf, B, buf.bonus, dev_i32(cand))
        torch.cuda.synchronize()
        for b in range(B):
            na = int(buf.n_acc[b])
            lens[b].append(na)
            emitted[b].extend(buf.emitted[b, :na].cpu().tolist())
    for b in range(B):
        low = [i for i in range(len(emitted[b])) if margins[b][i] <= MARGIN]
        upto = low[0] if low else len(emitted[b])
        assert upto >= 6, "seed gives an early near-tie; pick another"
        assert emitted[b][:upto] == refs[b][:upto]
        assert int(kv.ctx_len[b]) == Lc0[b] + sum(lens[b])
        assert all(1 <= n <= d.tree_depth + 1 for n in lens[b])
        if not low:
            # committed cache == the oracle's cache after feeding the same tokens causally
            toks = np.concatenate([ctxs[b][:-1], [ctxs[b][-1]], np.array(emitted[b][:-1], dtype=ctxs[b].dtype)])[: int(kv.ctx_len[b])]
            ck, cv = oracle.decode.prefill(om, np.concatenate([toks, [0]]))
            gk, gv = read_cache(kv, b=b)
            for l in range(cfg.n_layers):
                assert np.abs(gk[l] - ck[l]).max() <= LOGIT_TOL
                assert np.abs(gv[l] - cv[l]).max() <= LOGIT_TOL
    assert len({tuple(x) for x in lens}) >= 2, "the sequences should not all accept alike"


def test_topology_may_change_every_step(bita):
    """The template is an argument of the step, not state: an efficient tree, a full tree, a
    per-node-group tree and a chain take turns on one KV state (Sec. 3.3 compares these
    topologies).  The candidates, group and shift a step hands over come from the previous
    step's template; every step is compared with the oracle run through the same sequence."""
    cfg = synth.get_config("tiny")
    n = cfg.n_mask
    eff = synth.efficient_tree_parents(n, 3)
    tins = [synth.attach_mask_groups(eff, [0], n),
            synth.attach_mask_groups(synth.full_branching_tree([3, 2, 2, 1]), [0], n),
            synth.attach_mask_groups(eff, range(len(eff)), n),
            synth.attach_mask_groups(synth.chain_tree(n + 1), [0], n)]
    w = synth.SynthWeights(cfg, seed=0)
    om = oracle.OracleModel(cfg, w)
    smax = 256
    model = bita.Model(cfg, w, max_pos=smax + 64)
    ds = [derive_template(t.parent, t.is_mask, t.n_mask) for t in tins]
    tmpls = [bita.TreeTemplate(t.parent, t.is_mask, t.n_tree, t.n_mask) for t in tins]
    KMAX = max(d.kmax for d in ds)
    bufs = [bita.StepBuffers(model, t, 1, KMAX, want_logits=True) for t in tmpls]
    kv = bita.KVState(cfg, cfg.n_layers, 1, smax, max(t.rows for t in tmpls))
    ctx = synth.random_context(cfg.vocab, 64, 0)
    ref_stream = ar_greedy(om, ctx, 12 * (n + 1) + 1)
    st = round_state(BitaState(om, ctx))
    out, seen = [], set()
    for t in range(12):
        i = (t * 3 + t // 4) % 4                          # 0 3 2 1 1 0 3 2 2 1 0 3: each follows several others
        d, tmpl, buf = ds[i], tmpls[i], bufs[i]
        kv.resize_rows(cfg.n_layers, cfg, tmpl.rows)
        Lc = load_cache(kv, st.cache_k, st.cache_v)
        root = st.root_token
        if t % 2 == 1:                                    # a planted draft, so that some steps accept deep
            rng = np.random.default_rng(300 + t)
            cand = synth.planted_candidates(ref_stream[len(out):], n, KMAX, int(rng.integers(1, d.tree_depth + 1)),
                                            np.zeros(n, int), cfg.vocab, 40 + t)
            group, shift = 0, 0
            ref = bita_step(om, d, st, cand, kmax=KMAX)
        else:                                             # what the previous step (another template) left
            if st.cand is None:
                cand, group, shift = np.full((n, KMAX), -1, np.int32), 0, n
            else:
                cand, group, shift = st.cand, st.group, st.shift
            ref = bita_step(om, d, st, kmax=KMAX)
        bita.decode_step(model, kv, Lc, tmpl, buf, 1, dev_i32([root]), dev_i32(np.asarray(cand)[None]),
                         dev_i32([group]), dev_i32([shift]))
        torch.cuda.synchronize()
        assert buf.token[0].cpu().tolist() == ref["tokens"], t
        lg = buf.logits[0].cpu().numpy()
        assert np.abs(lg - ref["logits"]).max() <= LOGIT_TOL, t
        _check_selection_bit_exact(buf, d, lg)
        gpu_greedy = buf.argmax[0].cpu().tolist()
        path, bonus = accept_walk(d, ref["tokens"], gpu_greedy)
        na = len(path)
        assert int(buf.n_acc[0]) == na and buf.path[0, :na].cpu().tolist() == path and int(buf.bonus[0]) == bonus
        assert (int(buf.next_group[0]), int(buf.next_shift[0])) == next_group_and_shift(d, path)
        assert int(kv.ctx_len[0]) == Lc + na
        for l in range(cfg.n_layers):
            assert torch.equal(kv.k_cache[l, 0][:, Lc:Lc + na], kv.k_tree[l, 0][:, path])
        decisive = all(_top2_margin(ref["logits"][r]) > MARGIN for r in range(d.T))
        if decisive:
            assert gpu_greedy == ref["greedy"] and path == ref["path"]
        seen.add((i, na))
        out.extend(ref["emitted"])
        round_state(st)
    assert out == ref_stream[: len(out)]                  # lossless whatever the topology
    assert len({i for i, _ in seen}) == 4 and max(na for _, na in seen) >= 2
