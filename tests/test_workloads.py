"""Structure checks for the seeded input generators (no method arithmetic involved)."""
import numpy as np
import pytest
import torch

import workloads as W


@pytest.mark.parametrize("seed", range(6))
def test_seeded_tree_shape(seed):
    par = W.seeded_tree(seed)
    W.validate_parents(par)
    depth = W.tree_depths(par)
    assert len(par) == 60 and depth.max() == 5
    counts = np.bincount(par[1:], minlength=60)
    assert counts[0] == 10 and counts[1:].max() <= 4
    assert (np.diff(depth) >= 0).all()  # breadth-first numbering
    assert np.array_equal(W.seeded_tree(seed), par)


def test_chain_and_validation():
    assert W.chain_tree(4).tolist() == [-1, 0, 1, 2]
    with pytest.raises(ValueError):
        W.validate_parents([-1, 1])
    with pytest.raises(ValueError):
        W.validate_parents([0, 0])


def test_config_shapes_and_paging():
    c = W.make_config(2, scale_down=16)
    assert c.B == 16 and c.Hq == 28 and c.Hkv == 4 and c.D == 128 and c.page == 16
    assert c.q.dtype == torch.bfloat16 and c.softmax_scale == 1.0
    assert c.total_nodes == 960 and c.max_path == 6
    bt = c.block_table.numpy()
    used = []
    for b in range(c.B):
        L = int(c.prefix_len[b])
        n_pages = -(-(L + c.max_path) // 16)
        used += bt[b, :n_pages].tolist()
        assert (bt[b, n_pages:] == c.poison_block).all()
        # slots past L hold NaN, slots before L are finite
        last = bt[b, (L - 1) // 16]
        assert torch.isfinite(c.k_pool[last, :, : (L - 1) % 16 + 1].float()).all()
        if L % 16:
            assert torch.isnan(c.k_pool[last, :, L % 16:].float()).all()
    assert len(set(used)) == len(used) and c.poison_block not in used
    assert torch.isnan(c.k_pool[c.poison_block].float()).all()


def test_config0_matches_its_description():
    c = W.make_config(0)
    assert (c.dtype, c.B, c.Hq, c.Hkv, c.D) == ("f32", 1, 4, 1, 64)
    assert int(c.prefix_len[0]) == 256 and c.parent.tolist() == [-1, 0, 1, 2]
    assert c.softmax_scale == pytest.approx(1 / 8)


def test_long_context_spans():
    c = W.make_config(3, scale_down=64)
    assert c.B == 2 and len(c.spans[0]) == 8
    assert all(e - s == (32768 // 64) // 16 for s, e in c.spans[0])


def test_planted_ids_have_distinct_siblings():
    trees = [W.seeded_tree(3)]
    tgt = np.random.default_rng(0).integers(0, 50, size=60)
    ids, planted = W.plant_draft_ids(1, trees, tgt, 50, want_depth=[4])
    par = trees[0]
    for p in range(60):
        kids = np.flatnonzero(par == p)
        assert len(set(ids[kids].tolist())) == len(kids)
