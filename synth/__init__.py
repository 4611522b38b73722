"""Seeded synthetic inputs for the BiTA tree-verify step.

This package produces *data only*: model shapes, random-init weights, draft-tree
parent arrays, contexts and planted-draft schedules.  It contains none of the
method's arithmetic (no attention, no acceptance walk, no ancestor sets), so the
CPU oracle and the HIP path can both be fed from it without sharing any logic.
"""
from .configs import ModelCfg, CONFIGS, get_config            # noqa: F401
from .weights import SynthWeights, tensor_seed                # noqa: F401
from .trees import (random_tree, full_branching_tree, efficient_tree_parents,  # noqa: F401
                    chain_tree, star_tree, attach_mask_groups, Template)
from .drafts import random_context, planted_candidates        # noqa: F401


def bf16_round(a):
    """Round a float array to the nearest bf16 value (ties to even), returned as float64.
    A data-conditioning helper: both sides are handed tensors that are exactly
    representable in bf16 so that storage precision is not charged as error."""
    import numpy as np
    import torch
    t = torch.as_tensor(np.asarray(a, dtype=np.float64)).to(torch.float32).to(torch.bfloat16)
    return t.to(torch.float64).numpy()
