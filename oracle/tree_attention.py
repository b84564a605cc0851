"""Tree-masked attention of draft nodes over a paged prefix KV cache (oracle, float64).

Definition (Section 1 of the paper states only that the target validates the drafted tokens in
one parallel pass; for that pass to reproduce what the target would compute token by token,
each drafted token must see exactly the context it would have had in sequential decoding):
node i of a tree attends to every prefix position and to the tree nodes on its own
root-to-i path, itself included, and to nothing else.
"""
from __future__ import annotations

import numpy as np


def ancestors(parent, i):
    """Node ids on the path root..i (ascending, i included) of a tree-local parent array."""
    path = []
    x = int(i)
    while x >= 0:
        path.append(x)
        x = int(parent[x])
    return path[::-1]


def tree_attn_ref(q, k_tree, v_tree, k_pool, v_pool, block_table, prefix_len, node_offset,
                  parent, softmax_scale, nodes=None):
    """out[n, h, :], lse[n, h] for every node n (or only the global node ids in ``nodes``).

    q [T, Hq, D]; k_tree, v_tree [T, Hkv, D]; pools [blocks, Hkv, page, D];
    block_table [B, max_blocks]; prefix_len [B]; node_offset [B+1]; parent [T] tree-local.
    Prefix position p of sequence b lives at pool[block_table[b, p // page], kv_head, p % page].
    Query head h uses kv head h // (Hq // Hkv).  All arithmetic in float64.
    """
    q = np.asarray(q, dtype=np.float64)
    k_tree = np.asarray(k_tree, dtype=np.float64)
    v_tree = np.asarray(v_tree, dtype=np.float64)
    k_pool = np.asarray(k_pool, dtype=np.float64)
    v_pool = np.asarray(v_pool, dtype=np.float64)
    block_table = np.asarray(block_table)
    prefix_len = np.asarray(prefix_len)
    node_offset = np.asarray(node_offset)
    parent = np.asarray(parent)
    T, Hq, D = q.shape
    Hkv = k_tree.shape[1]
    page = k_pool.shape[2]
    G = Hq // Hkv
    B = prefix_len.shape[0]
    want = range(T) if nodes is None else [int(n) for n in nodes]
    out = np.zeros((len(want), Hq, D))
    lse = np.zeros((len(want), Hq))
    seq_of = np.searchsorted(node_offset, np.arange(T), side="right") - 1
    cache = {}
    for row, n in enumerate(want):
        b = int(seq_of[n])
        L = int(prefix_len[b])
        n0 = int(node_offset[b])
        par_b = parent[n0:int(node_offset[b + 1])]
        if b not in cache:
            # the prefix keys/values of sequence b, read position by position through the table
            pos = np.arange(L)
            blk = block_table[b, pos // page]
            cache = {b: (k_pool[blk, :, pos % page, :], v_pool[blk, :, pos % page, :])}  # [L,Hkv,D]
        kp, vp = cache[b]
        anc = [n0 + a for a in ancestors(par_b, n - n0)]
        for g in range(Hkv):
            heads = slice(g * G, (g + 1) * G)  # the query heads that share kv head g
            keys = np.concatenate([kp[:, g, :], k_tree[anc, g, :]], axis=0)  # allowed keys A(i)
            vals = np.concatenate([vp[:, g, :], v_tree[anc, g, :]], axis=0)
            s = softmax_scale * (q[n, heads] @ keys.T)  # [G, |A|]
            m = s.max(axis=1, keepdims=True)
            e = np.exp(s - m)
            denom = e.sum(axis=1, keepdims=True)
            out[row, heads] = (e @ vals) / denom
            lse[row, heads] = (m + np.log(denom))[:, 0]
    return out, lse
