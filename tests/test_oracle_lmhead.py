"""Pins for the LM-head argmax oracle: brute-force loops, planted winners, exact ties."""
import numpy as np

from oracle import lmhead_argmax_ref, lmhead_logits_ref


def test_matches_python_loops_on_tiny_input():
    rng = np.random.default_rng(0)
    h = rng.standard_normal((3, 5)); w = rng.standard_normal((7, 5))
    ids, mx = lmhead_argmax_ref(h, w)
    for m in range(3):
        best, best_v = -np.inf, -1
        for v in range(7):
            acc = 0.0
            for k in range(5):
                acc += h[m, k] * w[v, k]
            if acc > best:
                best, best_v = acc, v
        assert ids[m] == best_v and abs(mx[m] - best) < 1e-12


def test_planted_row_wins():
    rng = np.random.default_rng(1)
    h = rng.standard_normal((4, 32)); w = rng.standard_normal((100, 32)) * 0.02
    plant = [17, 0, 99, 42]
    for m, v in enumerate(plant):
        w[v] = h[m] * 3.0  # logit = 3 |h|^2, far above everything else
    ids, mx = lmhead_argmax_ref(h, w)
    assert list(ids) == plant
    assert np.allclose(mx, 3.0 * (h * h).sum(1))


def test_exact_tie_goes_to_lowest_id():
    rng = np.random.default_rng(2)
    h = rng.standard_normal((2, 8)); w = rng.standard_normal((20, 8)) * 0.01
    w[11] = h[0]; w[5] = h[0]; w[13] = h[0]
    ids, _ = lmhead_argmax_ref(h, w)
    assert ids[0] == 5


def test_weight_layout_is_vocab_by_hidden():
    h = np.array([[1.0, 0.0, 0.0]]); w = np.zeros((4, 3)); w[2, 0] = 1.0; w[0, 2] = 5.0
    assert lmhead_argmax_ref(h, w)[0][0] == 2
    assert lmhead_logits_ref(h, w).shape == (1, 4)
