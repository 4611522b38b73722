"""Helpers for the GPU parity tests: move oracle-side data to the device and back."""
import numpy as np
import torch

import synth


def dev_i32(a):
    return torch.tensor(np.asarray(a), dtype=torch.int32, device="cuda")


def load_cache(kv, cache_k, cache_v, b=0):
    """cache_k[l]: [Lc, Hkv, hd] float arrays holding bf16-representable values."""
    Lc = cache_k[0].shape[0]
    for l in range(len(cache_k)):
        kv.k_cache[l, b, :, :Lc] = torch.tensor(cache_k[l]).permute(1, 0, 2).to(torch.bfloat16)
        kv.v_cache[l, b, :, :Lc] = torch.tensor(cache_v[l]).permute(1, 0, 2).to(torch.bfloat16)
    kv.ctx_len[b] = Lc
    return Lc


def read_cache(kv, b=0):
    Lc = int(kv.ctx_len[b])
    ks = [kv.k_cache[l, b, :, :Lc].permute(1, 0, 2).to(torch.float64).cpu().numpy() for l in range(kv.k_cache.shape[0])]
    vs = [kv.v_cache[l, b, :, :Lc].permute(1, 0, 2).to(torch.float64).cpu().numpy() for l in range(kv.v_cache.shape[0])]
    return ks, vs


def round_state(st):
    st.cache_k = [synth.bf16_round(x) for x in st.cache_k]
    st.cache_v = [synth.bf16_round(x) for x in st.cache_v]
    return st
