"""The frozen decoder forward F(T, O, C, M; P) of Algorithm 1, row by row.

float64 throughout.  The paper fixes the architecture only as "LLaMA-2"
(Sec. 4.1.2); the constants are the public LLaMA-2 ones: RMSNorm (eps 1e-5),
rotary embeddings with base 10000 in the half-split pairing (i, i+hd/2), SwiGLU,
no biases, untied LM head, grouped-query attention where query head h reads
key/value head h // (Hq/Hkv).
"""
import numpy as np

F64 = np.float64


def rmsnorm(x, gain, eps):
    """x * rsqrt(mean(x^2) + eps) * gain over the last axis."""
    x = np.asarray(x, F64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(gain, F64)


def rope_rotate(x, pos, theta):
    """Rotary embedding of x[..., hd] at integer position pos (scalar).

    Pair (i, i + hd/2) is rotated by the angle pos * theta^(-2i/hd).
    """
    x = np.asarray(x, F64)
    hd = x.shape[-1]
    half = hd // 2
    i = np.arange(half, dtype=F64)
    ang = F64(pos) * theta ** (-2.0 * i / hd)
    c, s = np.cos(ang), np.sin(ang)
    lo, hi = x[..., :half], x[..., half:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


def silu(x):
    return x / (1.0 + np.exp(-x))


def attend_row(q, keys, values, n_heads, n_kv_heads):
    """Softmax attention of one query row over an explicit key list.

    q: [Hq, hd]; keys, values: [nk, Hkv, hd] in the order the row sees them.
    Returns [Hq, hd].  Scale 1/sqrt(hd).
    """
    hd = q.shape[-1]
    rep = n_heads // n_kv_heads
    out = np.empty_like(q)
    for h in range(n_heads):
        g = h // rep
        s = keys[:, g, :] @ q[h] / np.sqrt(F64(hd))
        s = s - s.max()
        p = np.exp(s)
        p = p / p.sum()
        out[h] = p @ values[:, g, :]
    return out


class OracleModel:
    """Weights upcast to float64 on use.  `source.get(name, layer)` returns the
    tensor as a numpy array shaped [out][in] (y = x @ W.T); prompt_k/prompt_v are
    [Hkv][P][hd]."""

    def __init__(self, cfg, source, cache_layers=True):
        self.cfg = cfg
        self.src = source
        self._cache = {} if cache_layers else None

    def w(self, name, layer=None):
        key = (name, layer)
        if self._cache is not None and key in self._cache:
            return self._cache[key]
        a = np.asarray(self.src.get(name, layer), F64)
        if self._cache is not None:
            self._cache[key] = a
        return a


def forward_rows(model, tokens, is_mask, mask_index, pos, visible_rows, cache_k, cache_v,
                 n_layers=None, return_hidden=False):
    """One pass of the decoder over R query rows of one sequence.

    tokens[r]      token id of an ordinary row (ignored for mask rows); a negative
                   id marks a row that is absent from this pass (a draft position
                   for which no candidate exists, Sec. 3.2 / Fig. 3: the mask
                   predictions that an accept made stale are dropped): it has no
                   embedding and attends to nothing, so its hidden state, its K/V
                   and its logits are zero, and no present row ever sees it (its
                   descendants are absent too).
    is_mask[r]     1 for a mask-token row: it is embedded with mask_emb[mask_index[r]]
                   (Sec. 3.1) and additionally sees the per-layer prompt prefix
                   (Sec. 3.2, tree-based attention).
    pos[r]         rotary position of the row.
    visible_rows[r] increasing list of rows j <= r of this pass that row r attends
                   to (its tree ancestors and itself).
    cache_k/v[l]   [Lc, Hkv, hd] keys/values of the tokens already in the result
                   sequence; every row sees all of them.
    Key order per row: prompt prefix (mask rows only, used as stored: no rotary,
    no projection), cached tokens 0..Lc-1, then the visible rows of this pass.

    Returns logits [R, V] and the per-layer K, V of the R rows ([L][R, Hkv, hd]).
    """
    cfg = model.cfg
    L = cfg.n_layers if n_layers is None else n_layers
    R = len(tokens)
    Hq, Hkv, hd = cfg.n_heads, cfg.n_kv_heads, cfg.head_dim
    tok_emb, mask_emb = model.w("tok_emb"), model.w("mask_emb")
    x = np.zeros((R, cfg.d_model), F64)
    for r in range(R):
        if is_mask[r]:
            x[r] = mask_emb[mask_index[r]]
        elif tokens[r] >= 0:
            x[r] = tok_emb[tokens[r]]
    new_k, new_v = [], []
    for l in range(L):
        h = rmsnorm(x, model.w("attn_norm", l), cfg.rms_eps)
        q = (h @ model.w("wq", l).T).reshape(R, Hq, hd)
        k = (h @ model.w("wk", l).T).reshape(R, Hkv, hd)
        v = (h @ model.w("wv", l).T).reshape(R, Hkv, hd)
        for r in range(R):
            q[r] = rope_rotate(q[r], pos[r], cfg.rope_theta)
            k[r] = rope_rotate(k[r], pos[r], cfg.rope_theta)
        pk, pv = model.w("prompt_k", l), model.w("prompt_v", l)     # [Hkv, P, hd]
        attn = np.zeros((R, Hq, hd), F64)
        for r in range(R):
            if not is_mask[r] and tokens[r] < 0:
                continue                                   # absent row: nothing to attend with
            parts_k, parts_v = [], []
            if is_mask[r] and cfg.n_prompt > 0:
                parts_k.append(np.transpose(pk, (1, 0, 2)))
                parts_v.append(np.transpose(pv, (1, 0, 2)))
            parts_k.append(np.asarray(cache_k[l], F64))
            parts_v.append(np.asarray(cache_v[l], F64))
            vis = list(visible_rows[r])
            parts_k.append(k[vis])
            parts_v.append(v[vis])
            attn[r] = attend_row(q[r], np.concatenate(parts_k, 0), np.concatenate(parts_v, 0),
                                 Hq, Hkv)
        x = x + attn.reshape(R, Hq * hd) @ model.w("wo", l).T
        h2 = rmsnorm(x, model.w("ffn_norm", l), cfg.rms_eps)
        gate = h2 @ model.w("w_gate", l).T
        up = h2 @ model.w("w_up", l).T
        x = x + (silu(gate) * up) @ model.w("w_down", l).T
        new_k.append(k)
        new_v.append(v)
    if return_hidden:
        return x, new_k, new_v
    logits = rmsnorm(x, model.w("final_norm"), cfg.rms_eps) @ model.w("lm_head").T
    return logits, new_k, new_v


def argmax_low(row):
    """Greedy choice: largest value, lowest index on ties."""
    row = np.asarray(row)
    return int(np.flatnonzero(row == row.max())[0])


def topk_desc(row, k):
    """Indices and values of the k largest entries, ordered by value descending
    and by index ascending among equal values."""
    row = np.asarray(row)
    idx = np.lexsort((np.arange(row.shape[0]), -row))[:k]
    return idx.astype(np.int32), row[idx]
