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


def test_bf16_rounding_hook():
    """round_bf16 against torch's conversion (library routine), incl. ties and negative values; with
    the hook on, cached decoding still equals the whole-sequence forward and speculative decoding
    still emits the plain greedy stream (the hook rounds the same quantities in every mode)."""
    import torch
    from oracle.toy_decoder import round_bf16
    x = np.concatenate([np.random.default_rng(0).standard_normal(2000) * 37.0,
                        [1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -1.0 - 2.0 ** -8, 0.0, 2.0 ** -130, 65280.0]])
    want = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(round_bf16(x), want)
    w = W.make_toy_weights(3, lm_head_bf16=True)
    ref = ToyDecoderRef(w, quant=round_bf16)
    prompt = [int(t) for t in np.random.default_rng(5).integers(0, w.vocab, size=12)]
    stream, margin = ref.greedy_ar(prompt, 10)
    full = ref.full_forward(prompt + stream[:-1])
    assert [int(np.argmax(full[len(prompt) - 1 + i])) for i in range(10)] == stream
    out, _ = ref.spec_decode(prompt, 10, W.random_drafter(2, w.vocab), lambda s: W.chain_tree(4),
                             np.random.default_rng(1).permutation(8))
    assert out == stream


def test_dense_rounding_hook():
    """With the dense layers' hand-overs rounded as well (quant_dense) and bf16-representable
    weights, the three decoding modes still agree (the hook rounds the same quantities in every
    mode); the default (identity) leaves the decoder as it was; the rounding is really applied
    (the logits differ from the unrounded decoder's, slightly)."""
    from oracle.toy_decoder import round_bf16
    w = W.make_toy_weights(4, weights_bf16=True)
    for a in [w.embed, w.lm_head, *w.wq, *w.w_down]:
        assert np.array_equal(round_bf16(a), a)
    ref = ToyDecoderRef(w, quant=round_bf16, quant_dense=round_bf16)
    prompt = [int(t) for t in np.random.default_rng(6).integers(0, w.vocab, size=12)]
    stream, _ = ref.greedy_ar(prompt, 10)
    full = ref.full_forward(prompt + stream[:-1])
    assert [int(np.argmax(full[len(prompt) - 1 + i])) for i in range(10)] == stream
    out, _ = ref.spec_decode(prompt, 10, W.random_drafter(2, w.vocab), lambda s: W.seeded_tree(s, n_nodes=16, levels=4, root_fanout=4),
                             np.random.default_rng(1).permutation(8))
    assert out == stream
    plain = ToyDecoderRef(w, quant=round_bf16)
    l0, l1 = plain.full_forward(prompt), ref.full_forward(prompt)
    assert np.array_equal(ToyDecoderRef(w, quant=round_bf16, quant_dense=lambda a: a).full_forward(prompt), l0)
    d = np.abs(l0 - l1).max()
    assert 0 < d < 2.0  # the logits spread over tens of units
