"""LM head followed by a per-row argmax (oracle, float64).

The target's choice for the token that follows a node is the vocabulary entry with the largest
logit (greedy verification, Section 1 / Section 4.1 of the paper); ties go to the lowest id.
"""
from __future__ import annotations

import numpy as np


def lmhead_logits_ref(hidden, weight):
    """logits[m, v] = sum_k hidden[m, k] * weight[v, k]  (weight in nn.Linear layout [V, K])."""
    return np.asarray(hidden, dtype=np.float64) @ np.asarray(weight, dtype=np.float64).T


def lmhead_argmax_ref(hidden, weight):
    """(ids int32[M], max_logit float64[M]); the lowest id among equal maxima wins."""
    logits = lmhead_logits_ref(hidden, weight)
    ids = np.argmax(logits, axis=1)  # numpy returns the first (lowest) index of the maximum
    return ids.astype(np.int32), logits[np.arange(logits.shape[0]), ids]
