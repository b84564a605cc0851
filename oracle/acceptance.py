"""Greedy acceptance of a verified draft tree (oracle, integers only).

Node 0 is the pending committed token and is always accepted.  A non-root node matches when
its draft id equals the target's argmax at its parent; it is accepted when it and all its
ancestors match.  The step keeps the deepest accepted node (lowest id among equals), emits the
draft ids along its path after the root plus the target's token at that node (the bonus token).
The number of emitted tokens is the per-step acceptance length whose mean the paper reports as
tau (Table 1, following EAGLE-3).

Second reading of the root (optional ``prev_target``): node 0 is itself a guess for the token
the target chose at the end of the previous step, and matches iff draft_ids[0] equals that
token.  A matching root gives exactly the result above.  A rejected root invalidates every
node (all were computed on a wrong context): nothing is accepted, nothing is emitted, the
pending token stays prev_target.  A sequence without nodes behaves the same way with no
pending token known (-1).
"""
from __future__ import annotations

import numpy as np


def tree_accept_ref(node_offset, parent, draft_ids, target_ids, max_path, prev_target=None):
    """Returns accept_len[B], accept_path[B,max_path], out_tokens[B,max_path], bonus_id[B]
    (int32; paths hold tree-local node ids, unused entries are -1).  prev_target int[B] or None:
    when given, the root of sequence b is accepted only if draft_ids[root] == prev_target[b];
    otherwise accept_len[b] = 0 and bonus_id[b] = prev_target[b]."""
    node_offset = np.asarray(node_offset)
    parent = np.asarray(parent)
    draft_ids = np.asarray(draft_ids)
    target_ids = np.asarray(target_ids)
    B = node_offset.shape[0] - 1
    accept_len = np.zeros(B, dtype=np.int32)
    accept_path = np.full((B, max_path), -1, dtype=np.int32)
    out_tokens = np.full((B, max_path), -1, dtype=np.int32)
    bonus_id = np.zeros(B, dtype=np.int32)
    for b in range(B):
        n0, n1 = int(node_offset[b]), int(node_offset[b + 1])
        par = parent[n0:n1]
        d_ids = draft_ids[n0:n1]
        t_ids = target_ids[n0:n1]
        n = n1 - n0
        if n == 0 or (prev_target is not None and int(d_ids[0]) != int(prev_target[b])):
            # no node, or a root that is not the token the target had chosen: nothing is valid
            bonus_id[b] = -1 if prev_target is None else int(prev_target[b])
            continue
        acc = np.zeros(n, dtype=bool)
        depth = np.zeros(n, dtype=np.int64)
        acc[0] = True
        for i in range(1, n):
            p = int(par[i])
            depth[i] = depth[p] + 1
            acc[i] = acc[p] and (d_ids[i] == t_ids[p])
        best = 0
        for i in range(n):
            if acc[i] and depth[i] > depth[best]:  # strict: the lowest id among equal depths stays
                best = i
        path = []
        x = best
        while x >= 0:
            path.append(x)
            x = int(par[x])
        path = path[::-1]
        ln = len(path)
        if ln > max_path:
            raise ValueError("max_path is smaller than an accepted path")
        accept_len[b] = ln
        accept_path[b, :ln] = path
        out_tokens[b, :ln - 1] = d_ids[path[1:]]
        out_tokens[b, ln - 1] = t_ids[best]
        bonus_id[b] = t_ids[best]
    return accept_len, accept_path, out_tokens, bonus_id
