"""Seeded stand-ins for the inputs of the draft model's intermediate layer: per-token features of
all target layers, meta queries and projection weights (random: the trained ones are not
available).  Values are rounded to bf16 so that the CPU and the GPU side start from the same
numbers."""
from __future__ import annotations

import numpy as np
import torch


def _bf16(a):
    return torch.from_numpy(np.asarray(a, dtype=np.float32)).to(torch.bfloat16)


def make_meta_inputs(seed, S, L, D, H, Q, peaked=False):
    """Returns a dict of bf16 torch tensors (CPU): feats [S, L, D] (hidden states of the L layers:
    unit scale, with a per-layer offset so that layers differ systematically as residual streams
    do), f_q [Q, D], w_q / w_k / w_v / w_o [D, D] (scale D^-1/2), w_fc1 [D, Q * D].
    peaked=True scales the queries up so that the softmax over the layers is far from uniform."""
    rng = np.random.default_rng(seed)
    layer_shift = rng.normal(0, 0.5, (1, L, D))
    feats = rng.normal(0, 1, (S, L, D)) + layer_shift
    f_q = rng.normal(0, 4.0 if peaked else 1.0, (Q, D))
    w = lambda n, k: rng.normal(0, k ** -0.5, (n, k))
    return dict(feats=_bf16(feats), f_q=_bf16(f_q), w_q=_bf16(w(D, D)), w_k=_bf16(w(D, D)), w_v=_bf16(w(D, D)),
                w_o=_bf16(w(D, D)), w_fc1=_bf16(w(D, Q * D)))
