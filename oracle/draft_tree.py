"""Construction of the draft token tree from the draft model's outputs (oracle).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

The paper drafts with a small model trained in the EAGLE-3 manner (Section 3.1) and says nothing
about how the drafted tokens are arranged; its measurements use chains (Section 4.2).  The
reading taken here is the published dynamic draft tree of the EAGLE line of work, restated:

  * The draft model is run level by level.  Level 0 is the root (the pending committed token).
    Running the draft on a node gives a distribution over the next token; its K most probable
    tokens become the node's candidate children.  A candidate's score is the log-probability of
    its whole path: score(child) = score(parent) + log p(child | path to parent), score(root) = 0.
  * Of a level's candidates only the K with the highest scores are run through the draft model
    again (the frontier); level 1 has exactly K candidates, so all of them are.
  * After T levels all candidates (K + (T - 1) K^2) are re-ranked by score and the N - 1 best
    are kept; with the root they form the tree that the target verifies.  Scores never increase
    along a path, so the kept set contains every kept node's parent.
  * Kept nodes are numbered in candidate order (level by level, within a level by frontier slot
    and then by the child's rank), which puts every parent before its children.

Precision and ties, so that the integer outputs are unique: log-probabilities enter as float32
values and a score is ONE float32 addition, score(parent) + logp, rounded to nearest; of two
equal scores the candidate with the lower candidate index ranks first; of two equal logits the
lower token id ranks first.

Candidate indices: level 1 holds candidates 0 .. K-1 (child rank j of the root at index j); level
l + 1 (l >= 1) holds K + (l - 1) K^2 + f K + j for frontier slot f (best first) and child rank j.
"""
from __future__ import annotations

import numpy as np


def topk_logprob_ref(logits, k):
    """Top-k tokens of each row and their log-probabilities.

    logits [M, V] (any float type; widened exactly to float64).  Returns ids int32 [M, k] ordered
    by (logit descending, token id ascending) and logp float64 [M, k] = logit - logsumexp(row)."""
    x = np.asarray(logits, dtype=np.float64)
    M, V = x.shape
    assert 1 <= k <= V
    ids = np.zeros((M, k), dtype=np.int32)
    logp = np.zeros((M, k), dtype=np.float64)
    for m in range(M):
        row = x[m]
        mx = row.max()
        lse = mx + np.log(np.exp(row - mx).sum())
        order = np.lexsort((np.arange(V), -row))  # last key is the primary one
        ids[m] = order[:k]
        logp[m] = row[order[:k]] - lse
    return ids, logp


class DraftTreeRef:
    """The candidate pool of ONE sequence, grown level by level."""

    def __init__(self, K, T):
        self.K, self.T = int(K), int(T)
        self.level = 0
        self.score = []    # float32 per candidate
        self.token = []    # int per candidate
        self.parent = []   # candidate index of the parent, -1 = the root
        self.frontier = []  # candidate indices that the draft model runs on next, best first

    def grow(self, child_ids, child_logp):
        """One level.  child_ids / child_logp [F, K]: the K best tokens (and their float32
        log-probabilities, none above 0) after each of the F nodes the draft model just ran on:
        F = 1 (the root) at level 0, else the K frontier nodes in frontier order.
        Returns (frontier candidate indices, frontier slot of each one's parent)."""
        K = self.K
        child_ids = np.asarray(child_ids)
        child_logp = np.asarray(child_logp, dtype=np.float32)
        F = 1 if self.level == 0 else K
        assert self.level < self.T and child_ids.shape == (F, K) and child_logp.shape == (F, K)
        assert not np.isnan(child_logp).any() and (child_logp <= 0).all()
        first = len(self.score)
        assert first == (0 if self.level == 0 else K + (self.level - 1) * K * K)
        for f in range(F):
            par = -1 if self.level == 0 else self.frontier[f]
            base = np.float32(0.0) if par < 0 else self.score[par]
            for j in range(K):
                self.score.append(np.float32(base + child_logp[f, j]))  # one float32 addition
                self.token.append(int(child_ids[f, j]))
                self.parent.append(par)
        new = list(range(first, len(self.score)))
        if self.level == 0:
            picked = new
        else:
            picked = sorted(new, key=lambda c: (-float(self.score[c]), c))[:K]
        slots = [(c - first) // K for c in picked]
        self.frontier = picked
        self.level += 1
        return list(picked), slots

    def finalize(self, N, root_token):
        """Keep the N - 1 best candidates; returns parent, draft_ids, depth (int32 [n]), the
        ancestor masks (uint64 [n], bit j of entry i set iff node j is i or an ancestor of i),
        the candidate index of every node (-1 for the root) and the nodes' scores (float32)."""
        C = len(self.score)
        keep = sorted(range(C), key=lambda c: (-float(self.score[c]), c))[: max(0, min(N - 1, C))]
        keep.sort()
        n = 1 + len(keep)
        assert n <= 64
        node_of = {-1: 0}
        for i, c in enumerate(keep):
            node_of[c] = i + 1
        parent = np.full(n, -1, dtype=np.int32)
        ids = np.zeros(n, dtype=np.int32)
        depth = np.zeros(n, dtype=np.int32)
        anc = np.zeros(n, dtype=np.uint64)
        cand = np.full(n, -1, dtype=np.int32)
        score = np.zeros(n, dtype=np.float32)
        ids[0] = root_token
        anc[0] = np.uint64(1)
        for i, c in enumerate(keep, start=1):
            p = node_of[self.parent[c]]  # KeyError would mean a kept node whose parent was dropped
            parent[i] = p
            ids[i] = self.token[c]
            depth[i] = depth[p] + 1
            anc[i] = anc[p] | (np.uint64(1) << np.uint64(i))
            cand[i] = c
            score[i] = self.score[c]
        return parent, ids, depth, anc, cand, score


def build_draft_tree_ref(draft_fn, K, T, N, root_token):
    """Whole construction for one sequence.  draft_fn(path_tokens) -> (ids [K], logp float32 [K]):
    the draft model's K best next tokens after the token path (root first)."""
    tree = DraftTreeRef(K, T)
    paths = [[int(root_token)]]
    for level in range(T):
        out = [draft_fn(p) for p in paths]
        child_ids = np.stack([np.asarray(o[0]) for o in out])
        child_logp = np.stack([np.asarray(o[1], dtype=np.float32) for o in out])
        frontier, slots = tree.grow(child_ids, child_logp)
        paths = [paths[s] + [tree.token[c]] for c, s in zip(frontier, slots)]
    return tree.finalize(N, root_token)
