"""GPU parity: hb_tree_accept and hb_kv_compact are bit-exact against the oracle."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import tree_accept_ref, kv_compact_ref
from parity import bits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def step():
    import paper_2509_18824_amd.step as s
    return s


def _accept_both(step, trees, draft, target, max_path):
    off = np.concatenate([[0], np.cumsum([len(t) for t in trees])]).astype(np.int32)
    par = np.concatenate(trees).astype(np.int32)
    ref = tree_accept_ref(off, par, draft, target, max_path)
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.int32)).cuda()
    got = step.tree_accept(t(off), t(par), t(draft), t(target), max_path, max(len(x) for x in trees))
    torch.cuda.synchronize()
    for g, r, name in zip(got, ref, ("accept_len", "accept_path", "out_tokens", "bonus_id")):
        assert np.array_equal(g.cpu().numpy(), r), name
    return ref


def test_config0_chain_with_seeded_matching_prefix(step):
    rng = np.random.default_rng(0)
    for trial in range(8):
        target = rng.integers(0, 1000, size=4)
        k = int(rng.integers(0, 4))
        draft = np.array([5] + [target[i - 1] if i <= k else (target[i - 1] + 1) % 1000 for i in range(1, 4)])
        ref = _accept_both(step, [W.chain_tree(4)], draft, target, 4)
        assert ref[0][0] == 1 + k


def test_planted_paths_on_batches_of_trees(step):
    for seed, tree_kind in [(1, "tree"), (2, "tree"), (3, "chain8")]:
        trees = [W.seeded_tree(seed * 100 + b) if tree_kind == "tree" else W.chain_tree(8) for b in range(16)]
        total = sum(len(t) for t in trees)
        target = np.random.default_rng(seed).integers(0, 152064, size=total)
        draft, planted = W.plant_draft_ids(seed, trees, target, 152064)
        ref = _accept_both(step, trees, draft, target, 8)
        assert list(ref[0]) == [d + 1 for d in planted]


def test_random_small_vocab_with_duplicates_and_ties(step):
    rng = np.random.default_rng(4)
    for trial in range(20):
        B = int(rng.integers(1, 6))
        trees = []
        for _ in range(B):
            n = int(rng.integers(1, 65))
            trees.append(np.array([-1] + [int(rng.integers(0, i)) for i in range(1, n)], dtype=np.int32))
        total = sum(len(t) for t in trees)
        draft = rng.integers(0, 3, size=total)
        target = rng.integers(0, 3, size=total)
        _accept_both(step, trees, draft, target, 64)


@pytest.mark.parametrize("dtype,Hkv,D", [("bf16", 4, 128), ("f32", 1, 64), ("bf16", 2, 64)])
def test_compaction_is_a_bit_exact_scatter(step, dtype, Hkv, D):
    trees = [W.seeded_tree(b) for b in range(6)]
    lens = [11, 12, 13, 14, 15, 16]  # accepted paths cross a page boundary in most sequences
    inp = W.make_verify_inputs(3, dtype, Hkv * 2, Hkv, D, lens, trees, poison=False)
    total = inp.total_nodes
    target = np.random.default_rng(1).integers(0, 500, size=total)
    draft, planted = W.plant_draft_ids(1, trees, target, 500, want_depth=[0, 1, 2, 3, 4, 5])
    alen, apath, _, _ = tree_accept_ref(inp.node_offset.numpy(), inp.parent.numpy(), draft, target, inp.max_path)
    ref_k, ref_v, ref_slots, ref_len = kv_compact_ref(bits(inp.k_tree), bits(inp.v_tree), bits(inp.k_pool),
                                                      bits(inp.v_pool), inp.block_table.numpy(),
                                                      inp.prefix_len.numpy(), inp.node_offset.numpy(), alen, apath)
    dev = step.to_device(inp)
    desc = step.desc_for(inp)
    slots, new_len = step.kv_compact(desc, dev, torch.from_numpy(alen).cuda(), torch.from_numpy(apath).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(slots.cpu().numpy(), ref_slots)
    assert np.array_equal(new_len.cpu().numpy(), ref_len)
    assert np.array_equal(bits(dev.k_pool), ref_k) and np.array_equal(bits(dev.v_pool), ref_v)
