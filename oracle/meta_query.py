"""The draft model's intermediate layer: target-feature aggregation with meta queries (oracle).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Section 3.1.1, Eq. (1): Q learnable meta queries f_q [Q, D] attend, for every token i, over the
features f_i [L, D] that the L target layers produced for that token (keys and values), and the
Q outputs are flattened into one vector of Q * D numbers per token.  Section 3.1.2 adds a skip
connection around this cross-attention whose residuals are a low-, a middle- and a high-level
feature of the same token, zero-initialises the attention's last projection (so that at the start
of training the layer's output IS those three features, side by side) and feeds the result to
fc1, the fully connected layer that brings Q * D back down to D; fc2 later joins a D-vector with
the token embedding by concatenation at every drafting step.

The paper fixes neither the attention's inner form nor its sizes.  Reading taken here: ordinary
multi-head attention with H heads of size d = D / H, projections without bias in the layout
y = x W^T, scores scaled by 1 / sqrt(d), softmax over the L layers:

  q = f_q W_q^T                     [Q, D]   (the same for every token)
  k_i = f_i W_k^T,  v_i = f_i W_v^T [L, D]
  o_i[:, head h] = softmax(q_h k_{i,h}^T / sqrt(d)) v_{i,h}
  f_c^i = flatten(o_i W_o^T + f_i[residual_layers])       (residual_layers: Q layer indices)

Everything in float64.  The paper's quality figures for this layer (Table 1, the ablation rows) need training and
stay parity unpinned; what is pinned is the arithmetic above (see tests/test_oracle_meta_query.py).
"""
from __future__ import annotations

import numpy as np


def meta_query_attn_ref(f_q, feats, w_q, w_k, w_v, w_o, H, residual_layers=None):
    """f_q [Q, D]; feats [S, L, D]; w_q, w_k, w_v, w_o [D, D].  Returns F_c [S, Q * D]."""
    f_q = np.asarray(f_q, dtype=np.float64)
    feats = np.asarray(feats, dtype=np.float64)
    w_q, w_k, w_v, w_o = (np.asarray(w, dtype=np.float64) for w in (w_q, w_k, w_v, w_o))
    Q, D = f_q.shape
    S, L, _ = feats.shape
    assert D % H == 0
    d = D // H
    q = f_q @ w_q.T
    out = np.zeros((S, Q, D), dtype=np.float64)
    for i in range(S):
        k = feats[i] @ w_k.T
        v = feats[i] @ w_v.T
        o = np.zeros((Q, D), dtype=np.float64)
        for h in range(H):
            sl = slice(h * d, (h + 1) * d)
            sc = q[:, sl] @ k[:, sl].T / np.sqrt(d)       # [Q, L]
            sc = sc - sc.max(axis=1, keepdims=True)
            p = np.exp(sc)
            p = p / p.sum(axis=1, keepdims=True)
            o[:, sl] = p @ v[:, sl]
        y = o @ w_o.T
        if residual_layers is not None:
            y = y + feats[i, np.asarray(residual_layers, dtype=np.int64), :]
        out[i] = y
    return out.reshape(S, Q * D)


def fc_concat_ref(a, b, w):
    """fc over the concatenation [a, b] along the feature axis: w [N, Ka + Kb]."""
    x = np.concatenate([np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)], axis=1)
    return x @ np.asarray(w, dtype=np.float64).T
