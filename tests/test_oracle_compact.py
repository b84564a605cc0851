"""Pins for the KV-compaction oracle: gather-back, untouched bytes, page-boundary crossing."""
import os

import numpy as np
import pytest

import workloads as W
from oracle import kv_compact_ref


def _bits(t):
    return t.view(dtype=__import__("torch").int16).numpy() if t.dtype == __import__("torch").bfloat16 else t.numpy()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("L0", [11, 13, 15, 16, 0])
def test_gather_back_and_nothing_else_changes(dtype, L0):
    trees = [W.seeded_tree(1, n_nodes=12, levels=5, root_fanout=2, max_fanout=3), W.chain_tree(5)]
    inp = W.make_verify_inputs(7, dtype, 4, 2, 8, [L0, 30], trees, page=16, poison=False)
    kt, vt, kp, vp = map(_bits, (inp.k_tree, inp.v_tree, inp.k_pool, inp.v_pool))
    accept_len = np.array([5, 3], dtype=np.int32)
    # any ancestor-closed path works for this function; use a real leaf path of depth 4
    par = trees[0]
    leaf = int(np.flatnonzero(W.tree_depths(par) == 4)[0])
    p0 = []
    x = leaf
    while x >= 0:
        p0.append(x); x = int(par[x])
    accept_path = np.array([p0[::-1], [0, 1, 2, -1, -1]], dtype=np.int32)
    k2, v2, slots, new_len = kv_compact_ref(kt, vt, kp, vp, inp.block_table.numpy(), inp.prefix_len.numpy(),
                                            inp.node_offset.numpy(), accept_len, accept_path)
    assert list(new_len) == [L0 + 5, 33]
    touched = np.zeros(kp.shape[:1] + kp.shape[2:3], dtype=bool)  # [block, offset]
    for b in range(2):
        L = int(inp.prefix_len[b])
        for j in range(accept_len[b]):
            p = L + j
            blk = int(inp.block_table[b, p // 16])
            src = int(inp.node_offset[b]) + accept_path[b, j]
            assert np.array_equal(k2[blk, :, p % 16], kt[src]) and np.array_equal(v2[blk, :, p % 16], vt[src])
            assert slots[b, j] == blk * 16 + p % 16
            touched[blk, p % 16] = True
        assert (slots[b, accept_len[b]:] == -1).all()
    keep = ~touched
    assert np.array_equal(k2.transpose(0, 2, 1, 3)[keep], kp.transpose(0, 2, 1, 3)[keep])
    assert np.array_equal(v2.transpose(0, 2, 1, 3)[keep], vp.transpose(0, 2, 1, 3)[keep])
    assert touched.sum() == 8
    # inputs were not modified in place
    assert np.array_equal(kp, _bits(inp.k_pool))


def test_hand_worked_slots():
    """Literal slot numbers for a permuted three-page table (tests/golden/kv_compact_hand_example.txt)."""
    rec = {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "kv_compact_hand_example.txt")):
        if line.strip() and not line.startswith("#"):
            key, *vals = line.split()
            rec[key] = [int(v) for v in vals]
    page, L, path = rec["page"][0], rec["prefix_len"][0], rec["path"]
    rng = np.random.default_rng(0)
    kt = rng.integers(-2**15, 2**15, size=(10, 2, 8)).astype(np.int16)
    vt = rng.integers(-2**15, 2**15, size=(10, 2, 8)).astype(np.int16)
    kp = rng.integers(-2**15, 2**15, size=(8, 2, page, 8)).astype(np.int16)
    vp = rng.integers(-2**15, 2**15, size=(8, 2, page, 8)).astype(np.int16)
    k2, v2, slots, new_len = kv_compact_ref(kt, vt, kp, vp, np.array([rec["block_table"]]), [L], [0, 10],
                                            [len(path)], np.array([path + [-1]]))
    assert list(slots[0]) == rec["out_slots"] + [-1] and list(new_len) == rec["new_len"]
    for node, slot in zip(path, rec["out_slots"]):
        assert np.array_equal(k2[slot // page, :, slot % page], kt[node])
        assert np.array_equal(v2[slot // page, :, slot % page], vt[node])
    changed = (k2 != kp).any(axis=(1, 3))  # [block, offset]
    assert sorted(map(tuple, np.argwhere(changed))) == sorted((s // page, s % page) for s in rec["out_slots"])
