"""Shared test helpers (no method arithmetic of the product; the brute-force
references here are written independently of both the oracle and the HIP path)."""
import os
import numpy as np


def read_paper_facts():
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_facts.txt")
    facts = {}
    with open(path) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if "=" in line:
                k, v = line.split("=", 1)
                facts[k.strip()] = v.strip()
    return facts


def textbook_causal_attention(q, k, v):
    """Standard causal softmax attention over one sequence.
    q: [n, Hq, hd], k, v: [n, Hkv, hd]; returns [n, Hq, hd] (float64)."""
    n, Hq, hd = q.shape
    Hkv = k.shape[1]
    out = np.zeros_like(q, dtype=np.float64)
    for h in range(Hq):
        g = h // (Hq // Hkv)
        s = q[:, h, :] @ k[:, g, :].T / np.sqrt(hd)
        s = np.where(np.tril(np.ones((n, n), bool)), s, -np.inf)
        p = np.exp(s - s.max(axis=1, keepdims=True))
        p /= p.sum(axis=1, keepdims=True)
        out[:, h, :] = p @ v[:, g, :]
    return out


def all_parent_arrays(T):
    """Every parent array with parent[0] = -1 and parent[i] < i."""
    def rec(prefix):
        i = len(prefix)
        if i == T:
            yield list(prefix)
            return
        for p in range(i):
            yield from rec(prefix + [p])
    yield from rec([-1])
