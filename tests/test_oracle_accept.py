"""Pins for the acceptance oracle: a hand-worked tree, the chain closed form, brute-force
enumeration of every root-to-node path, and invariants."""
import os

import numpy as np
import pytest

import workloads as W
from oracle import tree_accept_ref

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_hand_worked_example():
    rec = {}
    for line in open(os.path.join(GOLD, "tree_accept_hand_example.txt")):
        if line.strip() and not line.startswith("#"):
            key, *vals = line.split()
            rec[key] = [int(v) for v in vals]
    n = len(rec["parent"])
    alen, path, toks, bonus = tree_accept_ref([0, n], rec["parent"], rec["draft"], rec["target"], 5)
    assert alen[0] == rec["accept_len"][0]
    assert list(path[0, :alen[0]]) == rec["path"] and path[0, alen[0]:].tolist() == [-1]
    assert list(toks[0, :alen[0]]) == rec["tokens"] and toks[0, alen[0]:].tolist() == [-1]
    assert bonus[0] == rec["bonus"][0]
    # second reading of the root: a matching root changes nothing, a rejected root voids the step
    ok = tree_accept_ref([0, n], rec["parent"], rec["draft"], rec["target"], 5, prev_target=rec["prev_ok"])
    assert ok[0][0] == alen[0] and np.array_equal(ok[1], path) and np.array_equal(ok[2], toks) and ok[3][0] == bonus[0]
    bad = tree_accept_ref([0, n], rec["parent"], rec["draft"], rec["target"], 5, prev_target=rec["prev_bad"])
    assert bad[0][0] == rec["bad_accept_len"][0] and bad[3][0] == rec["bad_bonus"][0]
    assert (bad[1] == -1).all() and (bad[2] == -1).all()


@pytest.mark.parametrize("n,k", [(4, 0), (4, 1), (4, 3), (8, 5), (1, 0)])
def test_chain_accepts_one_plus_matching_prefix(n, k):
    rng = np.random.default_rng(n * 10 + k)
    target = rng.integers(0, 1000, size=n)
    draft = np.zeros(n, dtype=np.int64)
    draft[0] = 3
    for i in range(1, n):
        draft[i] = target[i - 1] if i <= k else (target[i - 1] + 1) % 1000
    alen, path, toks, bonus = tree_accept_ref([0, n], W.chain_tree(n), draft, target, n)
    assert alen[0] == 1 + k
    assert list(path[0, :1 + k]) == list(range(1 + k))
    assert list(toks[0, :1 + k]) == list(target[:1 + k])
    assert bonus[0] == target[k]


def _brute(parent, draft, target):
    """Enumerate every node's root path; keep the deepest fully matching, lowest end node."""
    best = None
    for end in range(len(parent)):
        path = []
        x = end
        while x >= 0:
            path.append(x); x = parent[x]
        path = path[::-1]
        if all(draft[c] == target[p] for p, c in zip(path[:-1], path[1:])):
            if best is None or len(path) > len(best):
                best = path
    return best


@pytest.mark.parametrize("seed", range(12))
def test_matches_enumeration_on_random_trees(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(2, 14))
    parent = np.array([-1] + [int(rng.integers(0, i)) for i in range(1, n)])
    vocab = 3  # tiny vocabulary: many accidental matches, duplicate sibling ids, ties in depth
    draft = rng.integers(0, vocab, size=n); target = rng.integers(0, vocab, size=n)
    alen, path, toks, bonus = tree_accept_ref([0, n], parent, draft, target, n)
    want = _brute(parent.tolist(), draft.tolist(), target.tolist())
    assert alen[0] == len(want) and list(path[0, :alen[0]]) == want
    assert list(toks[0, :alen[0]]) == [int(draft[c]) for c in want[1:]] + [int(target[want[-1]])]
    assert bonus[0] == toks[0, alen[0] - 1]
    # invariants: ascending, ancestor-closed
    p = path[0, :alen[0]]
    assert all(parent[p[j]] == p[j - 1] for j in range(1, len(p))) and p[0] == 0


def test_duplicate_sibling_ids_resolve_to_lowest_node():
    parent = [-1, 0, 0, 1, 2]
    draft = [9, 4, 4, 6, 6]
    target = [4, 6, 6, 1, 2]
    alen, path, toks, bonus = tree_accept_ref([0, 5], parent, draft, target, 3)
    assert alen[0] == 3 and list(path[0]) == [0, 1, 3] and bonus[0] == 1


def test_batch_and_planted_paths():
    trees = [W.seeded_tree(s) for s in range(5)]
    off = np.concatenate([[0], np.cumsum([len(t) for t in trees])])
    target = np.random.default_rng(0).integers(0, 1000, size=off[-1])
    draft, planted = W.plant_draft_ids(0, trees, target, 1000, want_depth=[0, 1, 3, 5, 2])
    alen, path, toks, bonus = tree_accept_ref(off, np.concatenate(trees), draft, target, 6)
    assert list(alen) == [d + 1 for d in planted]
    for b in range(5):
        assert (path[b, alen[b]:] == -1).all() and (toks[b, alen[b]:] == -1).all()


def test_max_path_too_small_is_an_error():
    with pytest.raises(ValueError):
        tree_accept_ref([0, 3], [-1, 0, 1], [1, 5, 6], [5, 6, 7], 2)


def test_root_as_a_guess_matches_enumeration_and_empty_trees_emit_nothing():
    """With prev_target the root is one more link of the chain: prepend a virtual node whose
    target is prev_target and the first reading must give the same path shifted by one."""
    rng = np.random.default_rng(5)
    for _ in range(20):
        n = int(rng.integers(1, 10))
        parent = np.array([-1] + [int(rng.integers(0, i)) for i in range(1, n)])
        draft = rng.integers(0, 3, size=n); target = rng.integers(0, 3, size=n)
        prev = int(rng.integers(0, 3))
        alen, path, toks, bonus = tree_accept_ref([0, n], parent, draft, target, n + 1, prev_target=[prev])
        # virtual root (id 0) in front: its target is prev, old node i becomes i + 1
        vpar = np.concatenate([[-1], parent + 1]); vpar[1] = 0
        want = _brute(vpar.tolist(), [0] + draft.tolist(), [prev] + target.tolist())
        assert alen[0] == len(want) - 1
        assert list(path[0, :alen[0]]) == [x - 1 for x in want[1:]]
        if alen[0] == 0:
            assert bonus[0] == prev and (toks[0] == -1).all()
        else:
            assert bonus[0] == target[want[-1] - 1] and toks[0, alen[0] - 1] == bonus[0]
    # a sequence without nodes between two ordinary ones
    alen, path, toks, bonus = tree_accept_ref([0, 2, 2, 4], [-1, 0, -1, 0], [1, 5, 1, 9], [5, 6, 9, 2], 3)
    assert list(alen) == [2, 0, 2] and bonus[1] == -1 and (path[1] == -1).all() and (toks[1] == -1).all()
