"""Stochastic (sampling) acceptance of a verified draft tree (oracle, exact integers).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

The paper states only that the target validates the drafted tokens and that the output is
lossless (Section 1, Section 4.1 "Setup"); it cites EAGLE-3 for the procedure.  Under sampling,
lossless means that the emitted tokens are distributed exactly as the target model's own
samples.  The published rule that achieves this is speculative sampling (accept a drafted token x
with probability min(1, p(x) / q(x)), p the target's and q the draft's distribution at that
position; after a rejection continue with the residual distribution max(p - q, 0) renormalised),
applied to several candidates per position by trying the children of a node one after the other,
each against the residual left by its rejected siblings, with the rejected token removed from q
(the candidates were drawn without replacement).  When no child is accepted (or the node has
none) the step's last token is drawn from the current residual (from p itself at a leaf).

Reading taken here, so that every decision is exactly reproducible on any hardware: all
probabilities are fixed-point integers, fix(p) = floor(p * 2^30) (exact for float32 inputs), the
uniform random numbers are 32-bit integers supplied by the caller, and every quantity a decision
depends on is an integer expression whose value does not depend on summation order:

  S(p) = sum_v p_v
  accept child with token x   iff   u * q_x * S(p) < 2^32 * p_x * S(q)
  after a rejection           r_v = max(p_v * S(q) - q_v * S(p), 0),  p_v <- r_v // max(S(r) >> 30, 1),
                              q_x <- 0                      (p unchanged when S(r) = 0)
  last token                  the smallest v with  p_0 + ... + p_v > (u_bonus * S(p)) >> 32

The sampled distribution differs from the real-valued rule by the truncation only (below 1e-6 in
total variation for vocabularies up to 2^18).  Node 0 is the pending committed token and is
always on the path, as in the greedy rule; the outputs have the greedy rule's layout.
"""
from __future__ import annotations

import numpy as np

FIX_BITS = 30


def to_fixed(p):
    """floor(p * 2^30) as Python-int-safe int64 (negative and NaN entries count as 0)."""
    p = np.asarray(p, dtype=np.float64)
    p = np.where(p > 0, p, 0.0)
    return np.minimum(np.floor(p * float(1 << FIX_BITS)), float((1 << 31) - 1)).astype(np.int64)


def accepts(u, p_x, q_x, s_p, s_q):
    """The acceptance test, in exact integers (u is a 32-bit uniform integer)."""
    return int(u) * int(q_x) * int(s_p) < (1 << 32) * int(p_x) * int(s_q)


def residual(p, q, s_p, s_q):
    """Fixed-point residual distribution after a rejection (int64 arrays; every product stays
    below 2^62 because entries and sums stay below 2^31, so int64 arithmetic is exact)."""
    assert 0 <= s_p < (1 << 31) and 0 <= s_q < (1 << 31) and int(p.max(initial=0)) <= (1 << 31)
    r = np.maximum(p * np.int64(s_q) - q * np.int64(s_p), 0)
    s_r = int(r.sum())  # <= s_p * s_q < 2^62
    if s_r == 0:
        return p
    return r // np.int64(max(s_r >> FIX_BITS, 1))


def inverse_cdf(p, u):
    """Smallest v with p_0 + ... + p_v > (u * S(p)) >> 32; -1 when S(p) = 0."""
    s_p = int(p.sum())
    if s_p == 0:
        return -1
    t = (int(u) * s_p) >> 32
    return int(np.searchsorted(np.cumsum(p), t, side="right"))


def tree_accept_sample_ref(node_offset, parent, draft_ids, p_target, q_draft, u_accept, u_bonus, max_path):
    """Returns accept_len[B], accept_path[B,max_path], out_tokens[B,max_path], bonus_id[B].

    p_target, q_draft: float [total_nodes, V]: the target's / the draft's distribution of the token
    that FOLLOWS each node.  u_accept uint32[total_nodes]: the uniform used when that node is tried
    as a child; u_bonus uint32[B]: the uniform of the step's last token.  A path is cut at max_path
    nodes (the node at that depth is treated as a leaf).  A sequence without nodes emits nothing
    (accept_len 0, bonus -1)."""
    node_offset = np.asarray(node_offset)
    parent = np.asarray(parent)
    draft_ids = np.asarray(draft_ids)
    B = node_offset.shape[0] - 1
    accept_len = np.zeros(B, dtype=np.int32)
    accept_path = np.full((B, max_path), -1, dtype=np.int32)
    out_tokens = np.full((B, max_path), -1, dtype=np.int32)
    bonus_id = np.full(B, -1, dtype=np.int32)
    for b in range(B):
        n0, n1 = int(node_offset[b]), int(node_offset[b + 1])
        n = n1 - n0
        if n == 0:
            continue
        par = parent[n0:n1]
        cur = 0
        path = [0]
        while True:
            p = to_fixed(p_target[n0 + cur])
            q = to_fixed(q_draft[n0 + cur])
            children = [c for c in range(cur + 1, n) if int(par[c]) == cur] if len(path) < max_path else []
            taken = None
            for c in children:
                x = int(draft_ids[n0 + c])
                s_p, s_q = int(p.sum()), int(q.sum())
                if accepts(u_accept[n0 + c], p[x], q[x], s_p, s_q):
                    taken = c
                    break
                p = residual(p, q, s_p, s_q)
                q = q.copy()
                q[x] = 0
            if taken is None:
                bonus = inverse_cdf(p, u_bonus[b])
                break
            path.append(taken)
            cur = taken
        ln = len(path)
        accept_len[b] = ln
        accept_path[b, :ln] = path
        out_tokens[b, :ln - 1] = draft_ids[n0 + np.array(path[1:], dtype=np.int64)] if ln > 1 else []
        out_tokens[b, ln - 1] = bonus
        bonus_id[b] = bonus
    return accept_len, accept_path, out_tokens, bonus_id
