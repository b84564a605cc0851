"""Pins for the attention oracle: a hand-worked example, closed forms, per-branch brute force
through a library attention routine, and invariances that any correct implementation has."""
import os

import numpy as np
import pytest
import torch

import workloads as W
from oracle import tree_attn_ref, ancestors

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _call(inp, **kw):
    return tree_attn_ref(W.widen(inp.q), W.widen(inp.k_tree), W.widen(inp.v_tree),
                         W.widen(inp.k_pool), W.widen(inp.v_pool), inp.block_table.numpy(),
                         inp.prefix_len.numpy(), inp.node_offset.numpy(), inp.parent.numpy(),
                         inp.softmax_scale, **kw)


def _small(seed=3, poison=True, Hq=4, Hkv=2, D=8, lens=(37, 5), dtype="f32", trees=None):
    trees = trees or [W.seeded_tree(seed, n_nodes=9, levels=4, root_fanout=2, max_fanout=3),
                      W.chain_tree(5)]
    return W.make_verify_inputs(seed, dtype, Hq, Hkv, D, list(lens), trees, page=4, poison=poison)


def test_hand_worked_example():
    rows = [l.split() for l in open(os.path.join(GOLD, "tree_attn_hand_example.txt"))
            if l.strip() and not l.startswith("#")]
    ln = np.log
    k_pool = np.zeros((1, 1, 16, 2)); v_pool = np.zeros((1, 1, 16, 2))
    k_pool[0, 0, 0] = (0, 0); k_pool[0, 0, 1] = (ln(2), 0)
    v_pool[0, 0, 0] = (1, 0); v_pool[0, 0, 1] = (0, 1)
    k_pool[0, 0, 2:] = np.nan; v_pool[0, 0, 2:] = np.nan  # slots past L must be ignored
    k_tree = np.array([[ln(3), 0], [0, 0], [ln(4), 0]])[:, None, :]
    v_tree = np.array([[1, 1], [2, 0], [0, 2]], dtype=float)[:, None, :]
    q = np.tile(np.array([1.0, 0.0]), (3, 1, 1))
    out, lse = tree_attn_ref(q, k_tree, v_tree, k_pool, v_pool, np.array([[0]]), np.array([2]),
                             np.array([0, 3]), np.array([-1, 0, 0]), 1.0)
    for node, o0, o1, el in rows:
        i = int(node)
        assert out[i, 0] == pytest.approx([float(o0), float(o1)], abs=1e-14)
        assert np.exp(lse[i, 0]) == pytest.approx(float(el), rel=1e-14)


def test_ancestors_helper():
    par = [-1, 0, 0, 1, 3, 2]
    assert ancestors(par, 4) == [0, 1, 3, 4]
    assert ancestors(par, 5) == [0, 2, 5]
    assert ancestors(par, 0) == [0]


def test_zero_keys_give_mean_of_allowed_values_and_log_count():
    inp = _small()
    inp.k_pool = torch.where(torch.isnan(inp.k_pool), inp.k_pool, torch.zeros_like(inp.k_pool))
    inp.k_tree = torch.zeros_like(inp.k_tree)
    out, lse = _call(inp)
    vt = W.widen(inp.v_tree); vp = W.widen(inp.v_pool)
    off = inp.node_offset.numpy(); G = inp.Hq // inp.Hkv
    for b, par in enumerate(inp.trees()):
        L = int(inp.prefix_len[b])
        pref = np.stack([vp[int(inp.block_table[b, p // inp.page]), :, p % inp.page] for p in range(L)])
        for i in range(len(par)):
            anc = ancestors(par, i)
            allv = np.concatenate([pref, vt[[off[b] + a for a in anc]]])  # [cnt, Hkv, D]
            for h in range(inp.Hq):
                assert np.allclose(out[off[b] + i, h], allv[:, h // G].mean(0), atol=1e-13)
                assert lse[off[b] + i, h] == pytest.approx(np.log(L + len(anc)), abs=1e-13)


def test_constant_values_come_back_whatever_the_scores():
    inp = _small()
    c = 0.625
    inp.v_pool = torch.where(torch.isnan(inp.v_pool), inp.v_pool, torch.full_like(inp.v_pool, c))
    inp.v_tree = torch.full_like(inp.v_tree, c)
    out, _ = _call(inp)
    assert np.allclose(out, c, atol=1e-14)


def test_one_dominant_key_returns_its_value():
    inp = _small(lens=(37, 9))
    # plant a key parallel to query (node 3, head 1) with a score 40 above the rest
    n, h, p = 3, 1, 11
    g = h // (inp.Hq // inp.Hkv)
    qv = inp.q[n, h].double()
    blk = int(inp.block_table[0, p // inp.page])
    inp.k_pool[blk, g, p % inp.page] = (qv * (60.0 / (inp.softmax_scale * qv.dot(qv)))).float()
    out, _ = _call(inp, nodes=[n])
    assert np.allclose(out[0, h], W.widen(inp.v_pool[blk, g, p % inp.page]), atol=1e-6)


def _sdpa_branch(inp, b, i):
    """Ordinary causal attention over prefix + path-to-node via torch's library routine."""
    off = inp.node_offset.numpy(); par = inp.trees()[b]
    L = int(inp.prefix_len[b]); G = inp.Hq // inp.Hkv
    path = [off[b] + a for a in ancestors(par, i)]
    pos = np.arange(L)
    blk = inp.block_table[b].numpy()[pos // inp.page]
    kp = inp.k_pool.double()[blk, :, pos % inp.page]  # [L, Hkv, D]
    vp = inp.v_pool.double()[blk, :, pos % inp.page]
    ks = torch.cat([kp, inp.k_tree.double()[path]]).permute(1, 0, 2)  # [Hkv, S, D]
    vs = torch.cat([vp, inp.v_tree.double()[path]]).permute(1, 0, 2)
    S = ks.shape[1]
    qs = torch.zeros((inp.Hq, S, inp.D), dtype=torch.float64)
    qs[:, L:, :] = inp.q.double()[path].permute(1, 0, 2)
    ks = ks.repeat_interleave(G, dim=0); vs = vs.repeat_interleave(G, dim=0)
    o = torch.nn.functional.scaled_dot_product_attention(qs[None], ks[None], vs[None], is_causal=True,
                                                         scale=inp.softmax_scale)[0]
    return o[:, L:, :].permute(1, 0, 2).numpy()  # rows for every node of the path


@pytest.mark.parametrize("seed", [1, 2])
def test_every_node_equals_causal_attention_over_its_own_branch(seed):
    inp = _small(seed=seed)
    out, _ = _call(inp)
    off = inp.node_offset.numpy()
    for b, par in enumerate(inp.trees()):
        for i in range(len(par)):
            branch = _sdpa_branch(inp, b, i)
            assert np.allclose(out[off[b] + i], branch[-1], atol=1e-12), (b, i)


def test_single_node_tree_is_plain_decode_attention_and_chain_is_causal():
    inp = _small(trees=[W.chain_tree(1), W.chain_tree(6)], lens=(21, 16))
    out, _ = _call(inp)
    # chain: one SDPA call yields all rows at once (bottom-right aligned causal mask)
    for b, n_nodes in enumerate((1, 6)):
        rows = _sdpa_branch(inp, b, n_nodes - 1)
        o0 = int(inp.node_offset[b])
        assert np.allclose(out[o0:o0 + n_nodes], rows, atol=1e-12)


def test_poison_in_forbidden_slots_never_reaches_the_output():
    clean = _small(poison=False)
    dirty = _small(poison=True)
    # also poison tree K/V of one sequence's nodes as seen from the *other* sequence: nothing to
    # do (they are never addressed); and non-ancestor nodes: compare against a copy where the
    # non-ancestors of node i hold NaN
    o_clean, l_clean = _call(clean)
    o_dirty, l_dirty = _call(dirty)
    assert np.array_equal(o_clean, o_dirty) and np.array_equal(l_clean, l_dirty)
    off = dirty.node_offset.numpy()
    for b, par in enumerate(dirty.trees()):
        for i in range(len(par)):
            anc = set(ancestors(par, i))
            kt = dirty.k_tree.clone(); vt = dirty.v_tree.clone()
            for j in range(len(par)):
                if j not in anc:
                    kt[off[b] + j] = float("inf"); vt[off[b] + j] = float("nan")
            alt = tree_attn_ref(W.widen(dirty.q), W.widen(kt), W.widen(vt), W.widen(dirty.k_pool),
                                W.widen(dirty.v_pool), dirty.block_table.numpy(), dirty.prefix_len.numpy(),
                                dirty.node_offset.numpy(), dirty.parent.numpy(), dirty.softmax_scale,
                                nodes=[off[b] + i])
            assert np.array_equal(alt[0][0], o_dirty[off[b] + i])


def test_physical_page_shuffle_changes_nothing():
    inp = _small(poison=False)
    base, lse = _call(inp)
    perm = np.random.default_rng(9).permutation(inp.num_blocks)  # new id of old page p is perm[p]
    inv = np.argsort(perm)
    inp.k_pool = inp.k_pool[torch.from_numpy(inv)]
    inp.v_pool = inp.v_pool[torch.from_numpy(inv)]
    inp.block_table = torch.from_numpy(perm[inp.block_table.numpy()].astype(np.int32))
    again, lse2 = _call(inp)
    assert np.array_equal(base, again) and np.array_equal(lse, lse2)


def test_empty_prefix_uses_the_tree_only():
    inp = _small(lens=(0, 3))
    out, lse = _call(inp)
    # root of sequence 0 sees only itself
    assert np.allclose(out[0], W.widen(inp.v_tree)[0].repeat(inp.Hq // inp.Hkv, axis=0), atol=1e-14)
    assert np.allclose(lse[0], inp.softmax_scale * np.einsum(
        "hd,hd->h", W.widen(inp.q)[0], W.widen(inp.k_tree)[0].repeat(inp.Hq // inp.Hkv, axis=0)), atol=1e-13)


def test_split_merge_identity_holds_in_float64():
    """Splitting the key set anywhere and merging (m, l, O) partials reproduces the whole
    (the online-softmax identity the split-K design relies on)."""
    rng = np.random.default_rng(5)
    s = rng.standard_normal(50) * 3
    v = rng.standard_normal((50, 4))
    whole = (np.exp(s - s.max()) @ v) / np.exp(s - s.max()).sum()
    for cut in (1, 17, 49):
        parts = []
        for sl in (slice(0, cut), slice(cut, 50)):
            m = s[sl].max(); e = np.exp(s[sl] - m)
            parts.append((m, e.sum(), e @ v[sl]))
        m = max(p[0] for p in parts)
        l = sum(p[1] * np.exp(p[0] - m) for p in parts)
        o = sum(p[2] * np.exp(p[0] - m) for p in parts) / l
        assert np.allclose(o, whole, atol=1e-12)
