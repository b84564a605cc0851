"""Appending the accepted nodes' K/V to the paged cache (oracle, bit copies).

After a verification step the accepted path's keys and values become ordinary context: the
paper's context management keeps everything that is part of the committed sequence in the KV
cache (Section 4.1 "Setup").  The j-th node of the accepted path goes to position L + j.
"""
from __future__ import annotations

import numpy as np


def kv_compact_ref(k_tree, v_tree, k_pool, v_pool, block_table, prefix_len, node_offset,
                   accept_len, accept_path):
    """Returns (k_pool', v_pool', out_slots[B,max_path], new_len[B]).  Pools are copied, never
    modified in place; arrays may be of any dtype (bf16 is passed as its 16-bit pattern) and are
    copied bit for bit.  out_slots[b, j] = physical_block * page + offset of position L_b + j."""
    k_pool = np.array(k_pool, copy=True)
    v_pool = np.array(v_pool, copy=True)
    block_table = np.asarray(block_table)
    accept_path = np.asarray(accept_path)
    page = k_pool.shape[2]
    B, max_path = accept_path.shape
    out_slots = np.full((B, max_path), -1, dtype=np.int32)
    new_len = np.zeros(B, dtype=np.int32)
    for b in range(B):
        L = int(prefix_len[b])
        for j in range(int(accept_len[b])):
            p = L + j
            blk = int(block_table[b, p // page])
            src = int(node_offset[b]) + int(accept_path[b, j])
            k_pool[blk, :, p % page, :] = k_tree[src]
            v_pool[blk, :, p % page, :] = v_tree[src]
            out_slots[b, j] = blk * page + p % page
        new_len[b] = L + int(accept_len[b])
    return k_pool, v_pool, out_slots, new_len
