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
