"""Pins for the sampling-acceptance oracle.

* Losslessness, the property the rule exists for: over the draft's own sampling of the candidate
  tokens (without replacement) and over all values of the uniforms, the token emitted after a
  node is distributed as the target's p.  Checked by exhaustive enumeration on a coarse grid of
  uniforms, with p and q chosen so that the acceptance thresholds fall on the grid.
* One-hot distributions reduce the rule to greedy acceptance: must equal tree_accept_ref.
* Closed forms: q == p accepts everything; a target that excludes the drafted token rejects it
  and emits its own token.
* A hand-worked example with literal integers (tests/golden/tree_accept_sample_hand_example.txt).
"""
import itertools
import os

import numpy as np
import pytest

import workloads as W
from oracle import tree_accept_ref, tree_accept_sample_ref

GOLD = os.path.join(os.path.dirname(__file__), "golden")
GRID_BITS = 6  # uniforms on a grid of 64 values; as 32-bit integers: g << 26


def _grid(g):
    return np.uint32(g << (32 - GRID_BITS))


def _emitted_distribution(p, q, n_children):
    """Exact distribution (on the uniform grid) of the token emitted right after the root of a
    tree whose root has n_children candidate children drawn from q without replacement."""
    V = len(p)
    out = np.zeros(V)
    G = 1 << GRID_BITS
    parent = [-1] + [0] * n_children
    # target / draft distributions of the token after every node (only the root's matter for the
    # first emitted token; the children get p as well so that a bonus can be drawn after them)
    P = np.tile(np.asarray(p, dtype=np.float64), (n_children + 1, 1))
    Q = np.tile(np.asarray(q, dtype=np.float64), (n_children + 1, 1))
    for toks in itertools.permutations(range(V), n_children):
        w = 1.0
        rest = 1.0
        for t in toks:  # probability of drawing this ordered candidate set without replacement
            w *= q[t] / rest
            rest -= q[t]
        if w == 0.0:
            continue
        draft = [0] + list(toks)
        for us in itertools.product(range(G), repeat=n_children + 1):
            u_acc = np.array([0] + [_grid(g) for g in us[:n_children]], dtype=np.uint32)
            alen, path, otoks, bonus = tree_accept_sample_ref([0, n_children + 1], parent, draft, P, Q, u_acc,
                                                             np.array([_grid(us[-1])], dtype=np.uint32), 2)
            first = otoks[0, 0]  # an accepted child's token, or the token drawn from the residual
            out[first] += w / G ** (n_children + 1)
    return out


def test_single_candidate_emits_the_target_distribution():
    # q on {1/2, 1/4, 1/4}; p multiples of 1/16: every ratio p_x / q_x is a multiple of 1/8
    p = [3 / 16, 9 / 16, 4 / 16]
    q = [1 / 2, 1 / 4, 1 / 4]
    got = _emitted_distribution(p, q, 1)
    assert np.abs(got - np.array(p)).max() <= 1.5 / (1 << GRID_BITS), got


@pytest.mark.parametrize("p,q", [([3 / 16, 9 / 16, 4 / 16], [1 / 2, 1 / 4, 1 / 4]),
                                 ([10 / 16, 1 / 16, 5 / 16], [1 / 4, 1 / 2, 1 / 4]),
                                 ([1 / 4, 1 / 2, 1 / 4], [1 / 4, 1 / 2, 1 / 4])])
def test_two_candidates_without_replacement_emit_the_target_distribution(p, q):
    global GRID_BITS
    old, GRID_BITS = GRID_BITS, 4  # three uniforms: 16^3 grid points per ordered candidate pair
    try:
        got = _emitted_distribution(p, q, 2)
        # the grid is coarse (1/16): thresholds of the second round do not fall on it exactly
        assert np.abs(got - np.array(p)).max() <= 0.07, got
    finally:
        GRID_BITS = old


def _one_hot(ids, V):
    out = np.zeros((len(ids), V))
    out[np.arange(len(ids)), ids] = 1.0
    return out


@pytest.mark.parametrize("seed", range(10))
def test_one_hot_distributions_reduce_to_greedy_acceptance(seed):
    rng = np.random.default_rng(seed)
    B = int(rng.integers(1, 5))
    V = 4
    trees = []
    for _ in range(B):
        n = int(rng.integers(1, 20))
        par = [-1]
        for i in range(1, n):  # at most V children per node: siblings carry distinct tokens
            free = [x for x in range(i) if par.count(x) < V]
            par.append(int(rng.choice(free)))
        trees.append(np.array(par))
    off = np.concatenate([[0], np.cumsum([len(t) for t in trees])])
    par = np.concatenate(trees)
    draft = rng.integers(0, V, size=off[-1])
    target = rng.integers(0, V, size=off[-1])
    for b, t in enumerate(trees):  # candidates are drawn without replacement
        for node in range(len(t)):
            kids = [c for c in range(len(t)) if t[c] == node]
            for k, c in enumerate(kids):
                draft[off[b] + c] = (draft[off[b] + kids[0]] + k) % V
    P = _one_hot(target, V)
    # the draft distribution at a node: uniform over its children's tokens (any q with q_x > 0 works)
    Q = np.full((off[-1], V), 1.0 / V)
    u_acc = rng.integers(0, 2 ** 32, size=off[-1], dtype=np.uint64).astype(np.uint32)
    u_bon = rng.integers(0, 2 ** 32, size=B, dtype=np.uint64).astype(np.uint32)
    got = tree_accept_sample_ref(off, par, draft, P, Q, u_acc, u_bon, 20)
    want = tree_accept_ref(off, par, draft, target, 20)
    for g, w in zip(got, want):
        assert np.array_equal(g, w)


def test_identical_distributions_accept_the_whole_chain_and_excluded_tokens_are_rejected():
    rng = np.random.default_rng(3)
    V, n = 50, 6
    P = rng.dirichlet(np.ones(V), size=n)
    draft = rng.integers(0, V, size=n)
    u = rng.integers(0, 2 ** 32, size=n, dtype=np.uint64).astype(np.uint32)
    alen, path, toks, bonus = tree_accept_sample_ref([0, n], W.chain_tree(n), draft, P, P.copy(), u, u[:1], n)
    assert alen[0] == n and list(path[0]) == list(range(n)) and list(toks[0, :n - 1]) == list(draft[1:])
    assert 0 <= bonus[0] < V and toks[0, n - 1] == bonus[0]
    # the target gives the drafted token of node 2 probability 0: the chain stops after node 1 and
    # the last token comes from the target's distribution at node 1 without that token
    P2 = P.copy()
    P2[1, draft[2]] = 0.0
    P2[1] /= P2[1].sum()
    alen, path, toks, bonus = tree_accept_sample_ref([0, n], W.chain_tree(n), draft, P2, P.copy(), u, u[:1], n)
    assert alen[0] == 2 and list(path[0, :2]) == [0, 1] and bonus[0] != draft[2]
    # max_path cuts the chain: the node at that depth is a leaf
    alen, path, toks, bonus = tree_accept_sample_ref([0, n], W.chain_tree(n), draft, P, P.copy(), u, u[:1], 3)
    assert alen[0] == 3 and list(path[0]) == [0, 1, 2]


def test_hand_worked_example():
    rec = {}
    for line in open(os.path.join(GOLD, "tree_accept_sample_hand_example.txt")):
        if line.strip() and not line.startswith("#"):
            key, *vals = line.split()
            rec[key] = vals
    V = 4
    p = np.array([[float(x) for x in rec["p_root"]], [float(x) for x in rec["p_node1"]], [0.25] * V, [0.25] * V])
    q = np.array([[float(x) for x in rec["q_root"]], [0.25] * V, [0.25] * V, [0.25] * V])
    parent = [int(x) for x in rec["parent"]]
    draft = [int(x) for x in rec["draft"]]
    for case in ("a", "b", "c"):
        u_acc = np.array([int(x) for x in rec[f"u_accept_{case}"]], dtype=np.uint32)
        u_bon = np.array([int(rec[f"u_bonus_{case}"][0])], dtype=np.uint32)
        d = [int(x) for x in rec.get(f"draft_{case}", rec["draft"])]
        alen, path, toks, bonus = tree_accept_sample_ref([0, 4], parent, d, p, q, u_acc, u_bon, 3)
        assert list(path[0, :alen[0]]) == [int(x) for x in rec[f"path_{case}"]], case
        assert list(toks[0, :alen[0]]) == [int(x) for x in rec[f"tokens_{case}"]], case
