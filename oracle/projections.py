"""The target's projections around the tree-verify attention (oracle, float64).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

The paper's verification step is one parallel pass of the target model over the drafted tokens
(Section 1); in a decoder layer that pass is, around the attention: the query/key/value
projection of the nodes' hidden states, the rotary position embedding of queries and keys at
each node's position (a node at depth t below the pending token sits at position L + t, the
position it would have in sequential decoding), and the output projection; the rest of the
layer is the root-mean-square normalisation in front of the attention and of the feed-forward
block, and the gated-SiLU feed-forward block itself.  The paper gives no model dimensions; shapes and the rotate-half rotary convention are those of the toy decoder here
(and of the decoder family BAGEL builds on).
"""
from __future__ import annotations

import numpy as np


def tree_positions_ref(node_offset, parent, prefix_len):
    """positions[n] = prefix_len[b] + depth(n): where node n would sit in sequential decoding."""
    node_offset = np.asarray(node_offset)
    parent = np.asarray(parent)
    pos = np.zeros(int(node_offset[-1]), dtype=np.int64)
    for b in range(len(node_offset) - 1):
        n0, n1 = int(node_offset[b]), int(node_offset[b + 1])
        for i in range(n0, n1):
            p = int(parent[i])
            pos[i] = int(prefix_len[b]) if p < 0 else pos[n0 + p] + 1
    return pos


def rope_ref(x, positions, theta):
    """Rotary embedding, rotate-half convention: dimension d < D/2 is paired with d + D/2 and the
    pair is rotated by the angle positions * theta^(-d / (D/2)).  x [T, H, D] -> [T, H, D]."""
    x = np.asarray(x, dtype=np.float64)
    half = x.shape[-1] // 2
    inv_freq = float(theta) ** (-np.arange(half, dtype=np.float64) / half)
    ang = np.asarray(positions, dtype=np.float64)[:, None] * inv_freq[None, :]
    cos, sin = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * cos - x2 * sin, x2 * cos + x1 * sin], axis=-1)


def qkv_rope_project_ref(hidden, w_qkv, bias, positions, Hq, Hkv, D, theta):
    """hidden [T, K]; w_qkv [(Hq + 2 Hkv) D, K] (nn.Linear layout: rows = q heads, then k heads,
    then v heads); bias [(Hq + 2 Hkv) D] or None.  Returns q [T, Hq, D] and k [T, Hkv, D] with the
    rotary embedding applied, v [T, Hkv, D] without."""
    y = np.asarray(hidden, dtype=np.float64) @ np.asarray(w_qkv, dtype=np.float64).T
    if bias is not None:
        y = y + np.asarray(bias, dtype=np.float64)[None, :]
    T = y.shape[0]
    q = y[:, :Hq * D].reshape(T, Hq, D)
    k = y[:, Hq * D:(Hq + Hkv) * D].reshape(T, Hkv, D)
    v = y[:, (Hq + Hkv) * D:].reshape(T, Hkv, D)
    return rope_ref(q, positions, theta), rope_ref(k, positions, theta), v


def linear_ref(x, w, residual=None):
    """out[t, n] = sum_k x[t, k] w[n, k] (+ residual[t, n])."""
    y = np.asarray(x, dtype=np.float64) @ np.asarray(w, dtype=np.float64).T
    return y if residual is None else y + np.asarray(residual, dtype=np.float64)


def rmsnorm_ref(x, weight, eps):
    """Root-mean-square normalisation of every row: out[t, :] = x[t, :] / sqrt(mean_k x[t, k]^2 +
    eps) * weight.  x [T, K], weight [K]."""
    x = np.asarray(x, dtype=np.float64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + float(eps)) * np.asarray(weight, dtype=np.float64)[None, :]


def swiglu_ref(x, w_gate_up):
    """The gated-SiLU half of the feed-forward block: w_gate_up [2 F, K] holds the gate
    projection's F rows, then the up projection's F rows (nn.Linear layout);
    out[t, f] = silu(x[t] . w_gate[f]) * (x[t] . w_up[f]),  silu(z) = z / (1 + exp(-z)).  The down
    projection with the residual is linear_ref."""
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w_gate_up, dtype=np.float64)
    F = w.shape[0] // 2
    g = x @ w[:F].T
    u = x @ w[F:].T
    return g / (1.0 + np.exp(-g)) * u
