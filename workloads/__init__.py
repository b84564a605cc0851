"""Seeded synthetic inputs for the tree-verification step of speculative decoding.

This module only *draws* inputs (draft-tree shapes, ragged prefix lengths, image/text span
maps, permuted page tables, Q/K/V and weight tensors, draft/target token ids).  It holds none of
the arithmetic of the verification step itself, so it can serve both the CPU oracle and the
GPU library without coupling them.
"""
from .trees import chain_tree, seeded_tree, tree_depths, validate_parents
from .drafters import random_drafter, replay_drafter
from .draft import make_draft_logits
from .meta import make_meta_inputs
from .configs import (
    CONFIG_NAMES,
    VerifyInputs,
    make_verify_inputs,
    make_config,
    make_lmhead_inputs,
    plant_draft_ids,
    ToyWeights,
    make_toy_weights,
    widen,
)

__all__ = [
    "chain_tree",
    "seeded_tree",
    "tree_depths",
    "validate_parents",
    "CONFIG_NAMES",
    "VerifyInputs",
    "make_verify_inputs",
    "make_config",
    "make_lmhead_inputs",
    "plant_draft_ids",
    "ToyWeights",
    "make_toy_weights",
    "widen",
    "random_drafter",
    "replay_drafter",
    "make_draft_logits",
    "make_meta_inputs",
]
