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


def _accept_both(step, trees, draft, target, max_path, prev_target=None):
    off = np.concatenate([[0], np.cumsum([len(t) for t in trees])]).astype(np.int32)
    par = np.concatenate(trees).astype(np.int32)
    ref = tree_accept_ref(off, par, draft, target, max_path, prev_target=prev_target)
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.int32)).cuda()
    got = step.tree_accept(t(off), t(par), t(draft), t(target), max_path, max(max(len(x) for x in trees), 1),
                           prev_target=None if prev_target is None else t(prev_target))
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


def test_root_as_a_guess_and_sequences_without_nodes(step):
    """prev_target makes the root one more guess (a rejected root voids the tree); a sequence
    whose tree is empty, also the last of the batch, emits nothing.  Compaction then appends
    nothing for those sequences."""
    rng = np.random.default_rng(11)
    for trial in range(12):
        B = int(rng.integers(1, 7))
        trees = []
        for b in range(B):
            n = int(rng.integers(0, 20)) if (trial + b) % 3 else 0
            trees.append(np.array(([-1] + [int(rng.integers(0, i)) for i in range(1, n)]) if n else [], dtype=np.int32))
        if all(len(t) == 0 for t in trees):
            trees[0] = W.chain_tree(3)
        total = sum(len(t) for t in trees)
        draft = rng.integers(0, 3, size=total)
        target = rng.integers(0, 3, size=total)
        prev = rng.integers(0, 3, size=B)
        ref = _accept_both(step, trees, draft, target, 20, prev_target=prev)
        ref0 = _accept_both(step, trees, draft, target, 20)
        for b, t in enumerate(trees):
            if len(t) == 0:
                assert ref[0][b] == 0 and ref[3][b] == prev[b] and ref0[0][b] == 0 and ref0[3][b] == -1
    # compaction with empty and voided sequences: whole pools compared
    trees = [W.seeded_tree(1), np.array([], dtype=np.int32), W.chain_tree(4), np.array([], dtype=np.int32)]
    inp = W.make_verify_inputs(5, "bf16", 4, 2, 64, [14, 20, 15, 3], trees, poison=False)
    target = np.random.default_rng(2).integers(0, 50, size=inp.total_nodes)
    draft, _ = W.plant_draft_ids(2, [trees[0], trees[2]], target, 50, want_depth=[3, 2])
    prev = np.array([draft[0], 7, (draft[len(trees[0])] + 1) % 50, 9])  # sequence 2: rejected root
    alen, apath, _, bonus = tree_accept_ref(inp.node_offset.numpy(), inp.parent.numpy(), draft, target,
                                            inp.max_path, prev_target=prev)
    assert list(alen) == [4, 0, 0, 0] and list(bonus[1:]) == [7, prev[2], 9]
    ref_k, ref_v, ref_slots, ref_len = kv_compact_ref(bits(inp.k_tree), bits(inp.v_tree), bits(inp.k_pool),
                                                      bits(inp.v_pool), inp.block_table.numpy(),
                                                      inp.prefix_len.numpy(), inp.node_offset.numpy(), alen, apath)
    dev = step.to_device(inp)
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.int32)).cuda()
    got = step.tree_accept(dev.node_offset, dev.parent, t(draft), t(target), inp.max_path, 60, prev_target=t(prev))
    assert np.array_equal(got[0].cpu().numpy(), alen) and np.array_equal(got[1].cpu().numpy(), apath)
    slots, new_len = step.kv_compact(step.desc_for(inp), dev, got[0], got[1])
    torch.cuda.synchronize()
    assert np.array_equal(slots.cpu().numpy(), ref_slots) and np.array_equal(new_len.cpu().numpy(), ref_len)
    assert np.array_equal(bits(dev.k_pool), ref_k) and np.array_equal(bits(dev.v_pool), ref_v)


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


def test_compaction_of_all_layers_in_one_launch(step):
    """hb_kv_compact_layers: three layers with their own tree K/V and pools, one launch; every
    layer's pools must equal the oracle's scatter of that layer's tensors, bit for bit."""
    import paper_2509_18824_amd as hb
    trees = [W.seeded_tree(b) for b in range(5)]
    lens = [11, 30, 13, 47, 15]
    layers = [W.make_verify_inputs(40 + l, "bf16", 8, 4, 128, lens, trees, poison=False) for l in range(3)]
    inp = layers[0]
    target = np.random.default_rng(3).integers(0, 500, size=inp.total_nodes)
    draft, _ = W.plant_draft_ids(3, trees, target, 500, want_depth=[0, 5, 2, 3, 1])
    alen, apath, _, _ = tree_accept_ref(inp.node_offset.numpy(), inp.parent.numpy(), draft, target, inp.max_path)
    devs = [step.to_device(x) for x in layers]
    # the page table and lengths are shared by the layers (those of layer 0)
    refs = [kv_compact_ref(bits(x.k_tree), bits(x.v_tree), bits(x.k_pool), bits(x.v_pool), inp.block_table.numpy(),
                           inp.prefix_len.numpy(), inp.node_offset.numpy(), alen, apath) for x in layers]
    table = lambda ts: torch.tensor([t.data_ptr() for t in ts], dtype=torch.int64, device="cuda")
    B, max_path = apath.shape
    slots = torch.full((B, max_path), -7, dtype=torch.int32, device="cuda")
    new_len = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    d0 = devs[0]
    hb.hb_kv_compact_layers(step.desc_for(inp), 3, table([d.k_tree for d in devs]), table([d.v_tree for d in devs]),
                            table([d.k_pool for d in devs]), table([d.v_pool for d in devs]), d0.block_table,
                            d0.prefix_len, d0.node_offset, torch.from_numpy(alen).cuda(), torch.from_numpy(apath).cuda(),
                            max_path, slots, new_len)
    torch.cuda.synchronize()
    assert np.array_equal(slots.cpu().numpy(), refs[0][2]) and np.array_equal(new_len.cpu().numpy(), refs[0][3])
    for d, (ref_k, ref_v, _, _) in zip(devs, refs):
        assert np.array_equal(bits(d.k_pool), ref_k) and np.array_equal(bits(d.v_pool), ref_v)
