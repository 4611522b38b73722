"""Seeded random-init weights, generated once and handed as the same bytes to
both the CPU oracle and the HIP path.

Every matrix, embedding, prompt-prefix tensor and mask embedding is drawn from
N(0, 0.02) (the paper initialises its learnable embeddings that way, Sec. 4.1.2)
with a per-tensor seed, then rounded once to bf16.  Norm gains are 1.0 by default
(`norm_std` = 0); a positive `norm_std` draws every gain as 1 + norm_std * N(0, 1), a
distinct seeded vector per layer and norm, so that a kernel that ignored a gain, or
read the wrong one, shows in the parity tests.  Matrices are stored
`[out_features][in_features]`, i.e. y = x @ W.T.
"""
import numpy as np
import torch

_TENSOR_IDS = {
    "tok_emb": 1, "mask_emb": 2, "lm_head": 3, "final_norm": 4,
    "wq": 10, "wk": 11, "wv": 12, "wo": 13, "w_gate": 14, "w_up": 15, "w_down": 16,
    "attn_norm": 17, "ffn_norm": 18, "prompt_k": 19, "prompt_v": 20,
}
LAYER_TENSORS = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down",
                 "attn_norm", "ffn_norm", "prompt_k", "prompt_v")
GLOBAL_TENSORS = ("tok_emb", "mask_emb", "lm_head", "final_norm")


def tensor_seed(seed, layer, name):
    """Distinct 63-bit seed per (global seed, layer, tensor)."""
    layer = -1 if layer is None else layer
    x = (seed * 1000003 + (layer + 1) * 7919 + _TENSOR_IDS[name] * 104729) & 0x7FFFFFFFFFFFFFFF
    return x


def tensor_shape(cfg, name):
    d, hd = cfg.d_model, cfg.head_dim
    return {
        "tok_emb": (cfg.vocab, d), "mask_emb": (cfg.n_mask, d), "lm_head": (cfg.vocab, d),
        "final_norm": (d,), "attn_norm": (d,), "ffn_norm": (d,),
        "wq": (cfg.n_heads * hd, d), "wk": (cfg.n_kv_heads * hd, d), "wv": (cfg.n_kv_heads * hd, d),
        "wo": (d, cfg.n_heads * hd), "w_gate": (cfg.d_ffn, d), "w_up": (cfg.d_ffn, d),
        "w_down": (d, cfg.d_ffn),
        "prompt_k": (cfg.n_kv_heads, cfg.n_prompt, hd), "prompt_v": (cfg.n_kv_heads, cfg.n_prompt, hd),
    }[name]


class SynthWeights:
    """Lazily generated bf16 tensors keyed by (name, layer).

    device="cpu" draws with torch's CPU generator (reproducible anywhere; used for
    the small cases and stored fixtures).  device="cuda" draws on the GPU for the
    7B-70B shapes, where host generation would take minutes; the values then differ
    from the CPU draw but oracle and HIP path still see identical bytes, because
    the oracle reads them back through `numpy()`.
    """

    def __init__(self, cfg, seed=0, device="cpu", std=0.02, prefix_std=None, keep=True, norm_std=0.0):
        self.cfg, self.seed, self.device, self.std = cfg, seed, torch.device(device), std
        self.prefix_std = std if prefix_std is None else prefix_std
        self.norm_std = norm_std
        self.keep = keep
        self._store = {}

    def torch(self, name, layer=None):
        key = (name, layer)
        if key in self._store:
            return self._store[key]
        shape = tensor_shape(self.cfg, name)
        if name.endswith("norm") and self.norm_std == 0.0:
            t = torch.ones(shape, dtype=torch.bfloat16, device=self.device)
        elif name.endswith("norm"):
            g = torch.Generator(device=self.device)
            g.manual_seed(tensor_seed(self.seed, layer, name))
            t = torch.randn(shape, generator=g, device=self.device, dtype=torch.float32)
            t = (1.0 + self.norm_std * t).to(torch.bfloat16)
        else:
            g = torch.Generator(device=self.device)
            g.manual_seed(tensor_seed(self.seed, layer, name))
            std = self.prefix_std if name.startswith("prompt_") else self.std
            t = torch.randn(shape, generator=g, device=self.device, dtype=torch.float32)
            t = (t * std).to(torch.bfloat16)
        if self.keep:
            self._store[key] = t
        return t

    def set(self, name, layer, tensor):
        """Replace a tensor (tests perturb the prefix / mask embeddings this way)."""
        self._store[(name, layer)] = tensor.to(torch.bfloat16).to(self.device)

    def numpy(self, name, layer=None):
        """fp32 numpy copy holding exactly the bf16 values."""
        return self.torch(name, layer).to(torch.float32).cpu().numpy()

    # the oracle's weight-source protocol
    get = numpy

    def clone_cpu(self):
        other = SynthWeights(self.cfg, self.seed, "cpu", self.std, self.prefix_std, norm_std=self.norm_std)
        other._store = {k: v.cpu().clone() for k, v in self._store.items()}
        return other
