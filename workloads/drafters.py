"""Seeded stand-ins for a draft model, used by the greedy-losslessness check.

A drafter maps (committed tokens, tree parent array) to one draft token id per node (entry 0,
the root, is the pending committed token and is not a guess).  None of them looks at the target
model; ``replay`` and ``corrupting`` are handed the reference stream they should imitate.
"""
from __future__ import annotations

import numpy as np


def _children(parent):
    ch = {}
    for i in range(1, len(parent)):
        ch.setdefault(int(parent[i]), []).append(i)
    return ch


def random_drafter(seed: int, vocab: int):
    """Uniformly random ids (siblings distinct): almost nothing is ever accepted."""
    rng = np.random.default_rng(seed * 16 + 12)

    def draft(tokens, parent):
        ids = np.zeros(len(parent), dtype=np.int32)
        ids[0] = tokens[-1]
        for _, kids in _children(parent).items():
            picks = rng.choice(vocab, size=len(kids), replace=False)
            for c, t in zip(kids, picks):
                ids[c] = int(t)
        return ids

    return draft


def replay_drafter(seed: int, vocab: int, prompt_len: int, stream, wrong_after=None):
    """Replays a given continuation ``stream`` (the tokens that follow the prompt): along the
    path that always descends into the tallest subtree every node carries the stream's token for its depth; all other nodes are
    distinct distractors.  With ``wrong_after=(lo, hi)`` the replay turns wrong after a seeded
    number of correct levels in [lo, hi] at every step (a drafter that is right for a while)."""
    rng = np.random.default_rng(seed * 16 + 13)
    stream = [int(t) for t in stream]

    def draft(tokens, parent):
        n = len(parent)
        ids = np.zeros(n, dtype=np.int32)
        ids[0] = tokens[-1]
        done = len(tokens) - prompt_len  # stream tokens already committed
        good_levels = n if wrong_after is None else int(rng.integers(wrong_after[0], wrong_after[1] + 1))
        ch = _children(parent)
        height = np.zeros(n, dtype=np.int64)
        for i in range(n - 1, 0, -1):
            height[parent[i]] = max(height[parent[i]], height[i] + 1)
        depth = np.zeros(n, dtype=np.int64)
        on_path = np.zeros(n, dtype=bool)
        on_path[0] = True
        for p in range(n):
            kids = ch.get(p, [])
            if not kids:
                continue
            d = int(depth[p]) + 1
            for c in kids:
                depth[c] = d
            idx = done + d - 1
            truth = stream[idx] if idx < len(stream) else -1
            used = set()
            if on_path[p] and truth >= 0 and d <= good_levels:
                heir = max(kids, key=lambda c: (height[c], -c))  # tallest subtree, lowest id
                ids[heir] = truth
                on_path[heir] = True
                used.add(truth)
                rest = [c for c in kids if c != heir]
            else:
                rest = kids
            for c in rest:
                while True:
                    cand = int(rng.integers(0, vocab))
                    if cand != truth and cand not in used:
                        break
                ids[c] = cand
                used.add(cand)
        return ids

    return draft
