"""GPU parity: hb_tree_accept_sample is bit-exact against the oracle (every decision of the rule
is an integer expression, so there is exactly one correct result)."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import tree_accept_ref, tree_accept_sample_ref

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def step():
    import paper_2509_18824_amd.step as s
    return s


def _u32(rng, n):
    return rng.integers(0, 2 ** 32, size=n, dtype=np.uint64).astype(np.uint32)


def _both(step, trees, draft, P, Q, u_acc, u_bon, max_path):
    off = np.concatenate([[0], np.cumsum([len(t) for t in trees])]).astype(np.int32)
    par = (np.concatenate(trees) if len(off) > 1 and off[-1] > 0 else np.zeros(0)).astype(np.int32)
    P32, Q32 = P.astype(np.float32), Q.astype(np.float32)
    ref = tree_accept_sample_ref(off, par, draft, P32, Q32, u_acc, u_bon, max_path)
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.int32)).cuda()
    bits = lambda a: torch.from_numpy(np.asarray(a, dtype=np.uint32).view(np.int32)).cuda()
    got = step.tree_accept_sample(t(off), t(par), t(draft), torch.from_numpy(P32).cuda(), torch.from_numpy(Q32).cuda(),
                                  bits(u_acc), bits(u_bon), max_path, max(max((len(x) for x in trees), default=1), 1))
    torch.cuda.synchronize()
    for g, r, name in zip(got, ref, ("accept_len", "accept_path", "out_tokens", "bonus_id")):
        assert np.array_equal(g.cpu().numpy(), r), (name, g.cpu().numpy(), r)
    return ref


def _draw_drafts(rng, trees, Q, V):
    """Children of a node carry distinct tokens drawn from the node's q without replacement."""
    off = np.concatenate([[0], np.cumsum([len(t) for t in trees])])
    draft = np.zeros(off[-1], dtype=np.int64)
    for b, t in enumerate(trees):
        for node in range(len(t)):
            kids = [c for c in range(len(t)) if t[c] == node]
            if kids:
                q = Q[off[b] + node].astype(np.float64)
                toks = rng.choice(V, size=len(kids), replace=False, p=q / q.sum())
                draft[off[b] + np.array(kids)] = toks
    return draft


@pytest.mark.parametrize("V", [7, 300, 4097])
def test_random_trees_and_distributions(step, V):
    rng = np.random.default_rng(V)
    for trial in range(6):
        B = int(rng.integers(1, 7))
        trees = []
        for _ in range(B):
            n = int(rng.integers(1, 40))
            par = [-1]
            for i in range(1, n):
                free = [x for x in range(i) if par.count(x) < min(V, 5)]
                par.append(int(rng.choice(free)))
            trees.append(np.array(par, dtype=np.int32))
        total = sum(len(t) for t in trees)
        # peaked target, flatter draft that resembles it: acceptances and rejections both happen
        logits = rng.standard_normal((total, V)) * 2.0
        P = np.exp(logits); P /= P.sum(1, keepdims=True)
        Qm = np.exp(0.7 * logits + 0.8 * rng.standard_normal((total, V))); Qm /= Qm.sum(1, keepdims=True)
        draft = _draw_drafts(rng, trees, Qm, V)
        ref = _both(step, trees, draft, P, Qm, _u32(rng, total), _u32(rng, B), 8)
        assert (ref[0] >= 1).all()


def test_acceptance_statistics_are_sane_on_chains(step):
    """8-node chains drafted from q = p: every node is accepted, whatever the uniforms; with an
    unrelated q most chains stop early.  (Bit-exactness against the oracle is checked inside.)"""
    rng = np.random.default_rng(5)
    V, B = 2000, 16
    trees = [W.chain_tree(8) for _ in range(B)]
    P = rng.dirichlet(np.full(V, 0.05), size=8 * B)
    draft = _draw_drafts(rng, trees, P, V)
    ref = _both(step, trees, draft, P, P.copy(), _u32(rng, 8 * B), _u32(rng, B), 8)
    assert (ref[0] == 8).all()
    Q = rng.dirichlet(np.full(V, 0.05), size=8 * B)
    draft = _draw_drafts(rng, trees, Q, V)
    ref = _both(step, trees, draft, P, Q, _u32(rng, 8 * B), _u32(rng, B), 8)
    assert ref[0].mean() < 3.0


def test_one_hot_distributions_equal_greedy_acceptance_and_edge_cases(step):
    rng = np.random.default_rng(9)
    V = 50
    trees = [W.seeded_tree(3), np.array([], dtype=np.int32), W.chain_tree(1), W.seeded_tree(4, n_nodes=64)]
    off = np.concatenate([[0], np.cumsum([len(t) for t in trees])])
    total = int(off[-1])
    target = rng.integers(0, V, size=total)
    draft, _ = W.plant_draft_ids(7, [trees[0], trees[2], trees[3]], np.concatenate([target[:60], target[60:]]), V)
    P = np.zeros((total, V)); P[np.arange(total), target] = 1.0
    Q = np.full((total, V), 1.0 / V)
    ref = _both(step, trees, draft, P, Q, _u32(rng, total), _u32(rng, 4), 7)
    want = tree_accept_ref(off, np.concatenate(trees), draft, target, 7)
    for g, w in zip(ref, want):
        assert np.array_equal(g, w)
    assert ref[0][1] == 0 and ref[3][1] == -1  # the sequence without nodes emits nothing
    # zero rows: nothing can be accepted and no last token exists (-1); max_path = 1: root only
    Z = np.zeros((total, V))
    ref = _both(step, trees, draft, Z, Q, _u32(rng, total), _u32(rng, 4), 7)
    assert list(ref[0]) == [1, 0, 1, 1] and list(ref[3]) == [-1, -1, -1, -1]
    _both(step, trees, draft, P, Q, _u32(rng, total), _u32(rng, 4), 1)


def test_full_vocabulary_chains(step):
    """The shape the paper measures: 8-node chains, batch 16, vocabulary 152064."""
    rng = np.random.default_rng(11)
    V, B = 152064, 16
    trees = [W.chain_tree(8) for _ in range(B)]
    logits = (rng.standard_normal((8 * B, V)) * 3.0).astype(np.float32)
    P = np.exp(logits - logits.max(1, keepdims=True)); P /= P.sum(1, keepdims=True)
    noise = rng.standard_normal((8 * B, V)).astype(np.float32)
    Q = np.exp(0.9 * logits + 0.6 * noise); Q /= Q.sum(1, keepdims=True)
    draft = _draw_drafts(rng, trees, Q, V)
    ref = _both(step, trees, draft, P, Q, _u32(rng, 8 * B), _u32(rng, B), 8)
    assert 1.0 < ref[0].mean() < 8.0
