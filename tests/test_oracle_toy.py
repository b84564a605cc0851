"""Pins for the toy decoder and the greedy-losslessness property (paper Section 1 and
Section 4.1 "Setup": verification by the target leaves its outputs unchanged)."""
import numpy as np
import pytest

import workloads as W
from oracle import ToyDecoderRef

PROMPT_LEN, N_NEW = 10, 32


@pytest.fixture(scope="module")
def setup():
    w = W.make_toy_weights(0)
    dec = ToyDecoderRef(w)
    prompt = [int(t) for t in np.random.default_rng(100).integers(0, w.vocab, size=PROMPT_LEN)]
    stream, margin = dec.greedy_ar(prompt, N_NEW)
    return w, dec, prompt, stream, margin


def test_cached_decoding_equals_whole_sequence_causal_forward(setup):
    w, dec, prompt, stream, margin = setup
    logits = dec.full_forward(prompt + stream)
    assert np.argmax(logits, axis=1)[PROMPT_LEN - 1:-1].tolist() == stream
    assert margin > 1e-3  # precondition for comparing with an fp32 implementation


def test_rope_is_a_rotation_and_relative():
    from oracle.toy_decoder import _rope
    rng = np.random.default_rng(0)
    x = rng.standard_normal((3, 2, 8)); y = rng.standard_normal((3, 2, 8))
    a = _rope(x, [5, 9, 2], 10000.0); b = _rope(y, [5, 9, 2], 10000.0)
    assert np.allclose((a * a).sum(-1), (x * x).sum(-1))
    # dot products depend only on the position difference
    a2 = _rope(x, [15, 19, 12], 10000.0); b2 = _rope(y, [15, 19, 12], 10000.0)
    assert np.allclose(np.einsum("thd,shd->tsh", a, b), np.einsum("thd,shd->tsh", a2, b2))
    assert np.allclose(_rope(x, [0, 0, 0], 10000.0), x)


def _tree(step):
    return W.seeded_tree(step, n_nodes=16, levels=5, root_fanout=3, max_fanout=3)


@pytest.mark.parametrize("kind", ["random", "replay", "corrupting"])
@pytest.mark.parametrize("topology", ["tree", "chain4"])
def test_speculative_decoding_emits_the_autoregressive_stream(setup, kind, topology):
    w, dec, prompt, stream, _ = setup
    drafter = {
        "random": W.random_drafter(1, w.vocab),
        "replay": W.replay_drafter(1, w.vocab, PROMPT_LEN, stream),
        "corrupting": W.replay_drafter(1, w.vocab, PROMPT_LEN, stream, wrong_after=(0, 4)),
    }[kind]
    tree = _tree if topology == "tree" else (lambda step: W.chain_tree(4))
    table = np.random.default_rng(3).permutation(8)[None, :]
    out, lens = dec.spec_decode(prompt, N_NEW, drafter, tree, table)
    assert out == stream
    if kind == "replay":
        full = 5 if topology == "tree" else 4
        assert all(l == full for l in lens[:-1])  # a perfect drafter is accepted to full depth
    if kind == "random":
        assert np.mean(lens) < 1.5
