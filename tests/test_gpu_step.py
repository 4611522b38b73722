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

LOGIT_TOL = 3e-2      # max-abs, bf16 path: the stated tolerance
MARGIN = 6e-2         # argmax must agree wherever the oracle's top-2 gap exceeds this
# Regression bounds, about ten times what the path delivers on these cases (measured: logits
# 6e-6 .. 1.2e-5 at the small shape, also with random norm gains and an O(1) prompt prefix).
# The stated tolerance above is what the problem allows; these catch a kernel that got worse.
TINY_LOGIT_REGRESSION = 1e-4


@pytest.fixture(scope="module")
def bita():
    import paper_2401_12522_amd as b
    b.lib()
    return b


def _setup(bita, cfg_name, tmpl_in, seed=0, smax=256, batch=1, gains=False):
    """gains: every RMSNorm gain drawn as 1 + 0.3 N(0, 1) (a distinct vector per layer and norm)
    and an O(1) prompt prefix instead of unit gains and an N(0, 0.02) prefix."""
    cfg = synth.get_config(cfg_name)
    w = synth.SynthWeights(cfg, seed=seed, norm_std=0.3, prefix_std=1.0) if gains else synth.SynthWeights(cfg, seed=seed)
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


@pytest.mark.parametrize("cfg_name,topology,gains", [
    ("tiny", "config1", False), ("tiny_gqa", "config1", False), ("tiny", "per_node", False), ("tiny", "full", False),
    ("tiny", "config1", True), ("tiny_gqa", "config1", True), ("tiny", "per_node", True)])
def test_step_by_step_against_oracle(bita, cfg_name, topology, gains):
    """Each step starts from the oracle's (bf16-representable) cache, so one step's
    rounding cannot compound into the next comparison.  The `gains` cases draw every RMSNorm
    gain at random (attention norm, FFN norm and final norm of every layer all different) and
    an O(1) prompt prefix: a gain that is ignored, taken from the wrong norm or indexed wrongly,
    or a prefix that mask rows do not weigh as the oracle does, fails the logits bound."""
    base = synth.get_config(cfg_name)
    if topology == "config1":
        tin = synth.attach_mask_groups(synth.random_tree(8, 3, 0), [0], base.n_mask)
    elif topology == "per_node":
        p = synth.efficient_tree_parents(base.n_mask, 3)
        tin = synth.attach_mask_groups(p, range(len(p)), base.n_mask)
    else:
        tin = synth.attach_mask_groups(synth.full_branching_tree([3, 2, 2, 1]), [0], base.n_mask)
    cfg, w, om, model, tmpl, kv, d = _setup(bita, cfg_name, tin, gains=gains)
    ctx = synth.random_context(cfg.vocab, 64, 0)
    steps = 16 if topology == "config1" else 6
    worst = 0.0
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
        worst = max(worst, err)
        assert err <= LOGIT_TOL, (t, err)
        assert err <= TINY_LOGIT_REGRESSION, (t, err)
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
            # tighter: the resolution of the bf16 cache format at the largest value stored
            kv_tol = 2.0 ** -8 * max(np.abs(ref["new_k"][l]).max(), np.abs(ref["new_v"][l]).max()) + 1e-5
            assert np.abs(got_k - ref["new_k"][l]).max() <= kv_tol
            assert np.abs(got_v - ref["new_v"][l]).max() <= kv_tol
        # cache slots below ctx_len untouched
        ks, vs = read_cache(kv)
        for l in range(cfg.n_layers):
            assert np.array_equal(ks[l][:Lc], st_before_k[l]) and np.array_equal(vs[l][:Lc], st_before_v[l])
        seen.add(na)
        out.extend(ref["emitted"])
        round_state(st)
    assert out == ref_stream[: len(out)]
    assert len(seen) >= 2
    print(f"{cfg_name}/{topology}/gains={gains}: worst logits max-abs err {worst:.3e}", flush=True)


def test_same_step_twice_is_bit_identical(bita):
    """The kernels reduce in a fixed order and use no floating-point atomics: the same step on
    the same state gives the same bits (logits, pass-row K/V, selections, acceptance), also when
    the workspace holds other data beforehand (nothing is read before it is written)."""
    base = synth.get_config("tiny_gqa")
    tin = synth.attach_mask_groups(synth.random_tree(20, 4, 2), [0, 3], base.n_mask)
    B = 2
    cfg, w, om, model, tmpl, kv, d = _setup(bita, "tiny_gqa", tin, batch=B, gains=True)
    lens = [64, 37]
    cands = []
    for b in range(B):
        st = round_state(BitaState(om, synth.random_context(cfg.vocab, lens[b] + 1, 7 + b)))
        load_cache(kv, st.cache_k, st.cache_v, b=b)
        cands.append(np.tile(np.random.default_rng(3 + b).integers(0, cfg.vocab, size=(cfg.n_mask, d.kmax)), (d.G, 1)))
    roots, cand = dev_i32([11, 12]), dev_i32(np.stack(cands))
    groups, shifts = dev_i32([1, 0]), dev_i32([0, 1])
    runs = []
    for fill in (0x00, 0xFF, 0x7F):
        buf = bita.StepBuffers(model, tmpl, B, d.kmax, want_logits=True)
        buf.workspace.fill_(fill)                       # 0xFF.. = NaN patterns, 0x7F7F.. = huge values
        kv.ctx_len[:] = dev_i32(lens)
        kv.k_tree.fill_(1.5); kv.v_tree.fill_(-2.5)
        bita.decode_step(model, kv, max(lens), tmpl, buf, B, roots, cand, groups, shifts)
        torch.cuda.synchronize()
        runs.append([buf.logits.clone(), kv.k_tree.clone(), kv.v_tree.clone(), buf.argmax.clone(), buf.topk_ids.clone(),
                     buf.topk_val.clone(), buf.path.clone(), buf.n_acc.clone(), buf.bonus.clone(), kv.ctx_len.clone(),
                     kv.k_cache.clone(), kv.v_cache.clone()])
        assert torch.isfinite(buf.logits).all()
    for other in runs[1:]:
        for a, b_ in zip(runs[0], other):
            assert torch.equal(a, b_)


def test_ffn_width_with_an_odd_number_of_half_ksteps(bita):
    """d_ffn = 8208 = 16 * 513: the down projection's activation slab ends in a half-filled k-step,
    and 2 * 8208 / 16 = 1026 gate/up tiles select the 48-feature workgroup shape, whose 171
    workgroups end exactly at the last feature.  The workspace starts as NaN bit patterns: the
    empty half must be cleared by the step itself."""
    cfg = synth.get_config("tiny", d_ffn=8208)
    tin = synth.attach_mask_groups(synth.full_branching_tree([4, 3, 2, 1], 64), [0], cfg.n_mask)
    w = synth.SynthWeights(cfg, seed=4, norm_std=0.3, prefix_std=1.0)
    om = oracle.OracleModel(cfg, w)
    model = bita.Model(cfg, w, max_pos=256)
    tmpl = bita.TreeTemplate(tin.parent, tin.is_mask, tin.n_tree, tin.n_mask)
    kv = bita.KVState(cfg, cfg.n_layers, 1, 128, tmpl.rows)
    d = derive_template(tin.parent, tin.is_mask, tin.n_mask)
    ctx = synth.random_context(cfg.vocab, 50, 1)
    st = round_state(BitaState(om, ctx))
    Lc = load_cache(kv, st.cache_k, st.cache_v)
    cand = np.random.default_rng(2).integers(0, cfg.vocab, size=(cfg.n_mask, d.kmax)).astype(np.int32)
    buf = bita.StepBuffers(model, tmpl, 1, d.kmax, want_logits=True)
    buf.workspace.fill_(0xFF)
    ref = bita_step(om, d, st, cand)
    bita.decode_step(model, kv, Lc, tmpl, buf, 1, dev_i32([int(ctx[-1])]), dev_i32(cand[None]))
    torch.cuda.synchronize()
    lg = buf.logits[0].cpu().numpy()
    assert np.isfinite(lg).all()
    err = np.abs(lg - ref["logits"]).max()
    print(f"d_ffn 8208: logits max-abs err {err:.3e}", flush=True)
    assert err <= TINY_LOGIT_REGRESSION * 10, err


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
    per-node-group tree and a chain take turns on one KV state (Sec. 4.3.4 / Table 4 compare these
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
