"""Contexts and planted draft candidates.

With random weights the mask rows' own top-k never predicts the model's greedy
continuation, so a free-running loop always accepts nothing.  To exercise every
acceptance length the harness can plant candidates instead: given a token stream
known to be the greedy continuation, it writes that stream into the candidate
table down to a seeded depth at a seeded column and fills the rest with tokens
that differ from the continuation.
"""
import numpy as np


def random_context(vocab, length, seed):
    rng = np.random.default_rng(seed)
    return rng.integers(0, vocab, size=length, dtype=np.int64).astype(np.int32)


def planted_candidates(continuation, n_levels, kmax, depth_ok, column, vocab, seed):
    """cand[level][col] for one step.

    continuation[i] is the greedy token i+1 positions after the current root's
    own successor... precisely: continuation[0] is the token the root will emit,
    continuation[1] the one after it, and so on.  Level i (0-based) of the tree
    must carry continuation[i] to be accepted.  The true token is written at
    `column[i]` for i < depth_ok; every other entry differs from the true token of
    its level.
    """
    rng = np.random.default_rng(seed)
    cand = np.empty((n_levels, kmax), np.int32)
    for i in range(n_levels):
        true_tok = int(continuation[i]) if i < len(continuation) else -2
        for j in range(kmax):
            t = int(rng.integers(0, vocab))
            while t == true_tok:
                t = int(rng.integers(0, vocab))
            cand[i, j] = t
        if i < depth_ok and true_tok >= 0:
            cand[i, int(column[i]) % kmax] = true_tok
    return cand
