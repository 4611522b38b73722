"""The benchmark configurations at their FULL size (GPU): LLaMA-2-7B-shaped, 32 layers, 1024-token
context and LLaMA-2-70B-shaped, 80 layers, 2048-token context; 64-node tree + 4 mask rows, batch 1,
the launch configuration bench.py times (prefill through bita_prefill, then tree steps).

The oracle cannot produce a 1024-token cache of a 7B-shaped model in test time, so these are
checks of properties that hold at any size (the element-wise parity against the oracle is in
test_gpu_llama_shapes.py, at the same widths and the full 7B depth with a short context):
  * lossless: the stream emitted by tree steps with planted drafts equals the stream of plain
    one-token-per-pass greedy decoding with the same kernels (Sec. 3.2), token by token; where the
    two disagree the one-row pass' own top-2 margin must be a near-tie (two summation orders);
  * accepted lengths are the planted ones and lie in 1..depth+1, the context counter advances by
    them, every committed K/V row is a bit copy of the pass' row, slots below the old context
    length are untouched;
  * the mask rows' logits change when the prompt prefix changes, the tree rows' logits do not
    (prompt tokens influence mask tokens only, Sec. 3.1)."""
import numpy as np
import pytest
import torch

import synth

pytestmark = pytest.mark.gpu


def _children(tin):
    ch = [[] for _ in range(tin.n_tree)]
    depth = [0] * tin.n_tree
    for v in range(1, tin.n_tree):
        ch[int(tin.parent[v])].append(v)
        depth[v] = depth[int(tin.parent[v])] + 1
    return ch, max(depth)


@pytest.mark.parametrize("name,ctx_n,steps", [("7b", 1024, 24), ("70b", 2048, 8)])
def test_full_size_tree_steps_are_lossless(name, ctx_n, steps):
    import paper_2401_12522_amd as bita
    from paper_2401_12522_amd import binding as B
    cfg = synth.get_config(name)
    tin = synth.attach_mask_groups(synth.full_branching_tree([4, 3, 2, 1], 64), [0], cfg.n_mask)
    children, depth_max = _children(tin)
    smax = ctx_n + (steps + 2) * (depth_max + 1) + 64
    w = synth.SynthWeights(cfg, seed=5, device="cuda", prefix_std=0.5)
    model = bita.Model(cfg, w, max_pos=smax + 64, free_source=True)
    tmpl = bita.TreeTemplate(tin.parent, tin.is_mask, tin.n_tree, cfg.n_mask)
    kv = bita.KVState(cfg, cfg.n_layers, 1, smax, 64)
    ctx = synth.random_context(cfg.vocab, ctx_n, 11)
    toks = torch.tensor(ctx[None, :-1], dtype=torch.int32, device="cuda").contiguous()
    B.prefill(model, kv, 0, toks, 64)
    torch.cuda.synchronize()
    ctx0 = int(kv.ctx_len[0])
    assert ctx0 == ctx_n - 1
    kv.resize_rows(cfg.n_layers, cfg, tmpl.rows)
    kmax = tmpl.kmax
    # ---- reference: one row per pass, restarted from the tree state after a near-tie
    t1 = synth.attach_mask_groups(np.array([-1], np.int32), [], cfg.n_mask)
    tm1 = B.TreeTemplate(t1.parent, t1.is_mask, 1, cfg.n_mask)
    kv_ref = bita.KVState(cfg, cfg.n_layers, 1, smax, 1)
    b1 = B.StepBuffers(model, tm1, 1, 1, want_logits=True)

    def reference_from(kv_now, root_now, n):
        kv_ref.k_cache.copy_(kv_now.k_cache)
        kv_ref.v_cache.copy_(kv_now.v_cache)
        kv_ref.ctx_len.copy_(kv_now.ctx_len)
        b1.bonus.copy_(root_now)
        toks_, margins_ = [], []
        for _ in range(n):
            B.decode_step(model, kv_ref, smax - 8, tm1, b1, 1, b1.bonus, None)
            top2 = torch.topk(b1.logits[0, 0], 2).values
            toks_.append(int(b1.bonus[0]))
            margins_.append(float(top2[0] - top2[1]))
        return toks_, margins_

    # ---- tree steps with planted drafts
    buf = B.StepBuffers(model, tmpl, 1, kmax, want_logits=True)
    root = torch.tensor([int(ctx[-1])], dtype=torch.int32, device="cuda")
    n_ref = (depth_max + 1) * 4
    (ref, margins), pos = reference_from(kv, root, n_ref), 0
    compared = near_ties = 0
    for t in range(steps):
        if len(ref) - pos < depth_max + 2:
            (ref, margins), pos = reference_from(kv, root, n_ref), 0
        rng = np.random.default_rng(300 + t)
        depth_ok = int(rng.integers(0, depth_max + 1))
        col, v = np.zeros(cfg.n_mask, int), 0
        for i in range(depth_ok):
            if not children[v]:                              # the truncated last level
                depth_ok = i
                break
            col[i] = int(rng.integers(0, len(children[v])))
            v = children[v][col[i]]
        cand = synth.planted_candidates(ref[pos:], cfg.n_mask, kmax, depth_ok, col, cfg.vocab, 70 + t)
        Lc = int(kv.ctx_len[0])
        k_before = kv.k_cache[:, 0, :, :Lc].clone()
        B.decode_step(model, kv, smax - 8, tmpl, buf, 1, root, torch.tensor(cand[None], dtype=torch.int32, device="cuda"))
        torch.cuda.synchronize()
        na = int(buf.n_acc[0])
        em = buf.emitted[0, :na].cpu().tolist()
        path = buf.path[0, :na].cpu().tolist()
        assert 1 <= na <= depth_max + 1
        assert int(kv.ctx_len[0]) == Lc + na
        assert torch.equal(kv.k_cache[:, 0, :, :Lc], k_before)
        assert torch.equal(kv.k_cache[:, 0][:, :, Lc:Lc + na], kv.k_tree[:, 0][:, :, path])
        assert torch.equal(kv.v_cache[:, 0][:, :, Lc:Lc + na], kv.v_tree[:, 0][:, :, path])
        assert torch.isfinite(buf.logits).all()
        want = ref[pos:pos + na]
        root = buf.bonus.clone()
        if em != want:
            # a token decided differently by the 68-row and the one-row pass: it must be a near-tie
            # of the one-row pass' own two best logits; the reference restarts from the tree state
            i = next(j for j in range(na) if em[j] != want[j])
            assert margins[pos + i] < 2e-3, (t, i, margins[pos + i])
            compared += i
            near_ties += 1
            (ref, margins), pos = reference_from(kv, root, n_ref), 0
            continue
        assert na == depth_ok + 1, (t, na, depth_ok)      # the planted walk, no more, no less
        compared += na
        pos += na
    print(f"{name}: {compared} tokens of the tree stream equal the one-row stream, {near_ties} near-ties", flush=True)
    assert near_ties <= steps // 3 and compared >= steps
    del kv_ref
    # ---- prompt tokens influence mask tokens only
    cand = np.random.default_rng(1).integers(0, cfg.vocab, size=(cfg.n_mask, kmax)).astype(np.int32)
    cand_d = torch.tensor(cand[None], dtype=torch.int32, device="cuda")
    B.build_tree(tmpl, root, cand_d, None, None, 1, buf.token)
    B.verify_step(model, kv, smax - 8, tmpl, buf, 1)
    torch.cuda.synchronize()
    lg0 = buf.logits[0].clone()
    for t_ in model._keep:                                  # scale every prompt-prefix tensor in place
        if isinstance(t_, torch.Tensor) and t_.dtype == torch.bfloat16 and tuple(t_.shape) == (cfg.n_kv_heads, cfg.n_prompt, cfg.head_dim):
            t_.mul_(-1.5)
    B.verify_step(model, kv, smax - 8, tmpl, buf, 1)
    torch.cuda.synchronize()
    lg1 = buf.logits[0]
    T = tmpl.n_tree
    assert torch.equal(lg0[:T], lg1[:T])
    assert (lg0[T:] - lg1[T:]).abs().max() > 1e-3
