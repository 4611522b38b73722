"""Decode loops: plain autoregressive greedy decoding (the exact result the method
must reproduce, Sec. 1 and 3.2) and the BiTA loop of Algorithm 1.
"""
import numpy as np
from .model import forward_rows, argmax_low, topk_desc
from .tree import (derive_template, ancestors_or_self, build_tree_tokens, accept_walk,
                   next_group_and_shift, compact_kv)


def _empty_cache(cfg):
    z = np.zeros((0, cfg.n_kv_heads, cfg.head_dim), np.float64)
    return [z.copy() for _ in range(cfg.n_layers)], [z.copy() for _ in range(cfg.n_layers)]


def prefill(model, context):
    """K/V of context[:-1] by a causal pass (a chain, every row sees all earlier ones)."""
    cfg = model.cfg
    ck, cv = _empty_cache(cfg)
    n = len(context) - 1
    if n <= 0:
        return ck, cv
    vis = [list(range(r + 1)) for r in range(n)]
    _, k, v = forward_rows(model, list(context[:n]), [0] * n, [-1] * n, list(range(n)), vis, ck, cv)
    return k, v


def ar_greedy(model, context, n_new, return_cache=False):
    """y_{t+1} = argmax F(x_0..x_t), one token per pass."""
    ck, cv = prefill(model, context)
    last = int(context[-1])
    out = []
    for _ in range(n_new):
        Lc = ck[0].shape[0]
        logits, k, v = forward_rows(model, [last], [0], [-1], [Lc], [[0]], ck, cv)
        ck, cv = compact_kv(ck, cv, k, v, [0])
        last = argmax_low(logits[0])
        out.append(last)
    if return_cache:
        return out, ck, cv
    return out


class BitaState:
    """What one sequence carries between passes."""

    def __init__(self, model, context):
        self.cache_k, self.cache_v = prefill(model, context)
        self.root_token = int(context[-1])
        self.cand = None        # [G*n][kmax] from the previous pass
        self.group = 0
        self.shift = 0


def bita_step(model, d, state, cand_override=None, kmax=None):
    """One pass: build the tree, score it, verify, commit K/V, pick next candidates.

    Returns a dict with everything the HIP path is compared against.
    """
    cfg = model.cfg
    kmax = d.kmax if kmax is None else kmax
    Lc = state.cache_k[0].shape[0]
    if cand_override is not None:
        cand, group, shift = np.asarray(cand_override), 0, 0
    elif state.cand is None:          # first pass: no drafts yet, every draft row inactive
        cand, group, shift = np.full((max(d.G, 1) * d.n_mask, kmax), -1, np.int32), 0, d.n_mask
    else:
        cand, group, shift = state.cand, state.group, state.shift
    tokens = build_tree_tokens(d, state.root_token, cand, group, shift)
    pos = [Lc + d.depth[r] for r in range(d.R)]
    vis = [ancestors_or_self(d.parent, r) for r in range(d.R)]
    logits, k, v = forward_rows(model, tokens, d.is_mask, d.mask_index, pos, vis,
                                state.cache_k, state.cache_v)
    greedy = [argmax_low(logits[r]) for r in range(d.T)]
    topk_ids = np.zeros((d.G * d.n_mask, kmax), np.int32)
    topk_val = np.zeros((d.G * d.n_mask, kmax), np.float64)
    for g in range(d.G):
        for i, r in enumerate(d.group_rows[g]):
            topk_ids[g * d.n_mask + i], topk_val[g * d.n_mask + i] = topk_desc(logits[r], kmax)
    path, bonus = accept_walk(d, tokens, greedy)
    emitted = [tokens[c] for c in path[1:]] + [bonus]
    state.cache_k, state.cache_v = compact_kv(state.cache_k, state.cache_v, k, v, path)
    state.root_token = bonus
    state.cand = topk_ids
    if d.G > 0:
        state.group, state.shift = next_group_and_shift(d, path)
    return dict(tokens=tokens, logits=logits, greedy=greedy, topk_ids=topk_ids, topk_val=topk_val,
                path=path, n_acc=len(path), bonus=bonus, emitted=emitted, new_k=k, new_v=v,
                ctx_len=Lc)


def bita_decode(model, template, context, n_steps, cand_fn=None):
    """Run n_steps passes.  cand_fn(step, n_emitted) may return a candidate table
    to plant instead of the model's own mask predictions."""
    d = derive_template(template.parent, template.is_mask, template.n_mask)
    st = BitaState(model, context)
    out, trace = [], []
    for t in range(n_steps):
        override = cand_fn(t, len(out)) if cand_fn is not None else None
        res = bita_step(model, d, st, override)
        out.extend(res["emitted"])
        trace.append(res)
    return out, trace, st
