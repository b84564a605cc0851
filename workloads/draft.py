"""Seeded stand-ins for the draft model's outputs (inputs of the draft tree's construction)."""
from __future__ import annotations

import numpy as np


def make_draft_logits(seed, M, V, ties=False):
    """float32 [M, V] logits shaped like a language model's next-token scores: a few tokens carry
    most of the mass (logit falling with the logarithm of a token's rank under a per-row random
    permutation) plus noise.  ties=True rounds to multiples of 1/4, which plants many equal
    logits (also among the best)."""
    rng = np.random.default_rng(seed)
    out = np.empty((M, V), dtype=np.float32)
    base = (-1.2 * np.log1p(np.arange(V))).astype(np.float32)
    for m in range(M):
        row = base[rng.permutation(V)] + rng.normal(0, 0.7, size=V).astype(np.float32) + np.float32(rng.normal(0, 3))
        out[m] = np.round(row * 4) / 4 if ties else row
    return out
