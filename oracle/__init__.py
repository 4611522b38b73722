"""CPU oracle for the BiTA tree-verify step -- TEST INFRASTRUCTURE ONLY.

Plain numpy, float64 arithmetic, no blocking or fusion: every function follows the
definition or the algorithm step it cites so it can be checked against the paper
by eye.  Nothing in the product path may import this package; it is used by the
tests, by the smoke check and by the benchmark's CPU-baseline leg.  It shares no
code with the HIP path.

What pins it (tests marked "not gpu"):
  * model arithmetic (RMSNorm, RoPE, GQA attention, SwiGLU, LM head) against the
    Hugging Face LLaMA implementation on the same random weights, plus closed
    forms (RoPE relative-position property, RMSNorm of a constant vector);
  * tree attention against textbook causal attention over each root-to-node path;
  * the whole decode loop against plain autoregressive greedy decoding (the
    paper's losslessness claim), free-running and with planted drafts;
  * the acceptance walk against a brute-force longest-matching-path search and
    against a transcription of Algorithm 1 on efficient trees;
  * tree sizes against the paper's closed forms (n*k+1 mask groups);
  * the prompt-prefix parameter count against the paper's 0.06 % figure.
Numeric logit values themselves are not printed anywhere in the paper: for them
parity is pinned only through the Hugging Face cross-check above.
"""
from .model import (OracleModel, rmsnorm, rope_rotate, silu, attend_row,   # noqa: F401
                    forward_rows, topk_desc, argmax_low)
from .tree import (derive_template, ancestors_or_self, anc_bitsets, efficient_tree,  # noqa: F401
                   build_tree_tokens, accept_walk, algorithm1_verify, compact_kv)
from .decode import ar_greedy, bita_decode, BitaState                        # noqa: F401
