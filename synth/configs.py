"""Model shapes of the synthetic workloads (LLaMA-2-shaped decoders).

The paper evaluates LLaMA-2 7B/13B/70B chat models with 16 prompt tokens and 3-4
mask tokens (Sec. 4.1.2); only the *shapes* are reproduced here, with random
weights.  `tiny` is the case the CPU oracle finishes in seconds.
"""
from dataclasses import dataclass, asdict


@dataclass(frozen=True)
class ModelCfg:
    name: str
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    n_prompt: int        # P: prompt-prefix tokens per layer
    n_mask: int          # n: mask tokens per group
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0

    def as_dict(self):
        return asdict(self)

    @property
    def q_dim(self):
        return self.n_heads * self.head_dim

    @property
    def kv_dim(self):
        return self.n_kv_heads * self.head_dim

    def weight_bytes(self, bytes_per_el=2):
        """Bytes of the matrices one step streams: all layers + LM head."""
        per_layer = (self.d_model * (self.q_dim + 2 * self.kv_dim)
                     + self.q_dim * self.d_model + 3 * self.d_model * self.d_ffn)
        return bytes_per_el * (self.n_layers * per_layer + self.vocab * self.d_model)

    def kv_bytes(self, ctx_lens, bytes_per_el=2):
        """Bytes of cached K and V the step sweeps, plus the prompt prefix once."""
        per_tok = 2 * self.kv_dim * bytes_per_el * self.n_layers
        return per_tok * (sum(ctx_lens) + self.n_prompt)


CONFIGS = {
    "tiny": ModelCfg("tiny", 2, 256, 4, 4, 64, 688, 1024, 8, 4),
    "tiny_gqa": ModelCfg("tiny_gqa", 2, 256, 4, 2, 64, 688, 1024, 8, 4),
    "7b": ModelCfg("7b", 32, 4096, 32, 32, 128, 11008, 32000, 16, 4),
    "13b": ModelCfg("13b", 40, 5120, 40, 40, 128, 13824, 32000, 16, 4),
    "70b": ModelCfg("70b", 80, 8192, 64, 8, 128, 28672, 32000, 16, 4),
}


def get_config(name, **overrides):
    cfg = CONFIGS[name]
    if overrides:
        d = cfg.as_dict()
        d.update(overrides)
        cfg = ModelCfg(**d)
    return cfg
