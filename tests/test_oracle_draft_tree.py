"""Pins of the draft-tree construction oracle (oracle/draft_tree.py): a library routine, a
hand-worked example, brute force over all token paths, and invariants."""
import itertools
import os

import numpy as np
import pytest
import torch

from oracle.draft_tree import DraftTreeRef, build_draft_tree_ref, topk_logprob_ref

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "draft_tree_hand_example.txt")


def _golden():
    out = {}
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, *vals = line.split()
        out[key] = [float(v) if "." in v else int(v) for v in vals]
    return out


def test_topk_against_the_library_routines():
    rng = np.random.default_rng(5)
    x = rng.normal(0, 3, size=(7, 1000)).astype(np.float32)
    ids, logp = topk_logprob_ref(x, 10)
    t = torch.from_numpy(x).double()
    vals, tid = torch.topk(t, 10, dim=1)  # values are distinct here, so the order is unique
    assert np.array_equal(ids, tid.numpy().astype(np.int32))
    ref = torch.log_softmax(t, dim=1).gather(1, tid).numpy()
    assert np.abs(logp - ref).max() < 1e-12
    assert (logp <= 0).all() and (np.diff(logp, axis=1) <= 0).all()


def test_topk_equal_logits_go_to_the_lower_token_id():
    x = np.zeros((1, 50), dtype=np.float32)
    x[0, [40, 7, 23]] = 2.0
    x[0, 31] = 3.0
    ids, logp = topk_logprob_ref(x, 5)
    assert ids[0].tolist() == [31, 7, 23, 40, 0]
    assert abs(np.exp(topk_logprob_ref(x, 50)[1]).sum() - 1.0) < 1e-12  # a distribution


def test_hand_worked_example():
    g = _golden()
    K, T = g["K"][0], g["T"][0]
    for N in (4, 6):
        tree = DraftTreeRef(K, T)
        f0, s0 = tree.grow(np.array(g["ids0"]).reshape(1, K), np.array(g["logp0"], dtype=np.float32).reshape(1, K))
        assert f0 == [0, 1] and s0 == [0, 0]
        f1, s1 = tree.grow(np.array(g["ids1"]).reshape(K, K), np.array(g["logp1"], dtype=np.float32).reshape(K, K))
        assert f1 == g["frontier1"] and s1 == g["slots1"]
        parent, ids, depth, anc, cand, score = tree.finalize(N, g["root"][0])
        assert parent.tolist() == g[f"N{N}_parent"]
        assert ids.tolist() == g[f"N{N}_ids"]
        assert depth.tolist() == g[f"N{N}_depth"]
        assert [int(a) for a in anc] == g[f"N{N}_anc"]
        assert cand.tolist() == g[f"N{N}_cand"]


class _TableModel:
    """A seeded 'draft model' over a tiny vocabulary: a distribution per token path."""

    def __init__(self, seed, V, K):
        self.seed, self.V, self.K = seed, V, K

    def dist(self, path):
        rng = np.random.default_rng([self.seed] + [int(t) for t in path])
        return rng.normal(0, 2, size=self.V).astype(np.float32)

    def __call__(self, path):
        ids, logp = topk_logprob_ref(self.dist(path)[None, :], self.K)
        return ids[0], logp[0].astype(np.float32)


def _path_of(node, parent, ids):
    out = []
    while node >= 0:
        out.append(int(ids[node]))
        node = int(parent[node])
    return tuple(reversed(out))


@pytest.mark.parametrize("seed", range(6))
def test_two_levels_keep_exactly_the_most_probable_paths(seed):
    """With K equal to the vocabulary size and two levels nothing is pruned before the final
    re-ranking, so the tree must hold the N - 1 most probable of ALL token paths of length 1 and
    2 (enumerated here from the model's distributions, scored in float64)."""
    V = K = 4
    model = _TableModel(seed, V, K)
    root = 2
    N = 9
    parent, ids, depth, anc, cand, score = build_draft_tree_ref(model, K, 2, N, root)
    got = {_path_of(i, parent, ids) for i in range(1, len(parent))}
    scored = []
    for n in (1, 2):
        for toks in itertools.product(range(V), repeat=n):
            s, path = 0.0, [root]
            for t in toks:
                x = model.dist(path).astype(np.float64)
                s += x[t] - (x.max() + np.log(np.exp(x - x.max()).sum()))
                path.append(t)
            scored.append((s, tuple(path)))
    scored.sort(key=lambda e: -e[0])
    assert scored[N - 2][0] - scored[N - 1][0] > 1e-4  # the cut is clear of float32 rounding
    assert got == {p for _, p in scored[: N - 1]}


@pytest.mark.parametrize("seed", range(6))
def test_deeper_trees_against_a_search_over_token_paths(seed):
    """Three and four levels: the same search written over sets of token paths (no candidate
    indices, no arrays), plus the structural invariants."""
    V, K, T, N = 7, 3, 4 - seed % 2, 14
    model = _TableModel(100 + seed, V, K)
    root = 1
    parent, ids, depth, anc, cand, score = build_draft_tree_ref(model, K, T, N, root)
    # search over paths: every candidate is (score, path); expanded = best K of a level
    pool, expanded = {}, [(np.float32(0), (root,))]
    for level in range(T):
        fresh = []
        for s, p in expanded:
            cid, clp = model(list(p))
            for t, lp in zip(cid, clp):
                fresh.append((np.float32(s + lp), p + (int(t),)))
        for s, p in fresh:
            pool[p] = s
        expanded = fresh if level == 0 else sorted(fresh, key=lambda e: -float(e[0]))[:K]
    best = sorted(pool.items(), key=lambda e: -float(e[1]))[: N - 1]
    assert {p for p, _ in best} == {_path_of(i, parent, ids) for i in range(1, len(parent))}
    # invariants
    n = len(parent)
    assert n == N and parent[0] == -1 and depth[0] == 0 and ids[0] == root
    for i in range(1, n):
        p = int(parent[i])
        assert 0 <= p < i and depth[i] == depth[p] + 1 and depth[i] <= T
        assert score[i] <= (score[p] if p > 0 else 0.0)
        assert int(anc[i]) == int(anc[p]) | (1 << i)
    for p in range(n):  # siblings carry distinct tokens
        kids = [int(ids[i]) for i in range(1, n) if parent[i] == p]
        assert len(kids) == len(set(kids))
    # the greedy chain (the most probable token at every level) is always kept
    path = [root]
    for _ in range(T):
        path.append(int(model(path)[0][0]))
        assert tuple(path) in {_path_of(i, parent, ids) for i in range(1, n)}


def test_equal_scores_keep_the_lower_candidate_index():
    """Uniform distributions: every candidate of a level has the same score, so the order of
    candidate indices decides everything."""
    K, T, N = 3, 3, 9
    lp = np.full(K, -np.log(8.0), dtype=np.float32)
    parent, ids, depth, anc, cand, score = build_draft_tree_ref(lambda path: (np.arange(K) + 10 * len(path), lp), K, T, N, 0)
    # level 1: candidates 0..2 (kept), level 2: 3..11, frontier = 3, 4, 5 (children of slot 0); kept: 3..7
    assert cand.tolist() == [-1, 0, 1, 2, 3, 4, 5, 6, 7]
    assert parent.tolist() == [-1, 0, 0, 0, 1, 1, 1, 2, 2]
    assert depth.max() == 2
