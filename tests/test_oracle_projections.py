"""Pins for the projection oracle: a hand-worked rotation, the rotation's invariants (norm, the
relative-position property, identity at position 0), agreement with torch's linear in float64,
positions on chains and on a literal tree."""
import os

import numpy as np
import torch

import workloads as W
from oracle import tree_positions_ref, rope_ref, qkv_rope_project_ref, linear_ref

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_hand_worked_rotation():
    rec = {}
    for line in open(os.path.join(GOLD, "rope_hand_example.txt")):
        if line.strip() and not line.startswith("#"):
            key, *vals = line.split()
            rec[key] = [float(v) for v in vals]
    out = rope_ref(np.array(rec["x"]).reshape(1, 1, 4), rec["position"], rec["theta"][0])
    assert np.allclose(out.ravel(), rec["out"], atol=1e-15)


def test_rotation_invariants():
    rng = np.random.default_rng(0)
    x, y = rng.standard_normal((5, 3, 128)), rng.standard_normal((5, 3, 128))
    pos = np.array([7, 100, 32768, 0, 4095])
    a, b = rope_ref(x, pos, 1e6), rope_ref(y, pos, 1e6)
    assert np.allclose(np.linalg.norm(a, axis=-1), np.linalg.norm(x, axis=-1))
    # <rope(x, m), rope(y, n)> depends on m - n only
    a2, b2 = rope_ref(x, pos + 11, 1e6), rope_ref(y, pos[::-1].copy() + 11, 1e6)
    b1 = rope_ref(y, pos[::-1].copy(), 1e6)
    assert np.allclose((a * b1).sum(-1), (a2 * b2).sum(-1), atol=1e-9)
    assert np.allclose(rope_ref(x, np.zeros(5), 1e6), x)
    # two successive rotations add their positions
    assert np.allclose(rope_ref(rope_ref(x, pos, 1e4), pos * 2, 1e4), rope_ref(x, pos * 3, 1e4), atol=1e-8)
    # same convention as the toy decoder's rotary embedding (pinned separately)
    from oracle.toy_decoder import _rope
    assert np.allclose(_rope(x, pos, 1e4), rope_ref(x, pos, 1e4))


def test_projection_equals_linear_layer_then_split_then_rotation():
    rng = np.random.default_rng(1)
    T, K, Hq, Hkv, D = 9, 40, 6, 2, 8
    h = rng.standard_normal((T, K)); w = rng.standard_normal(((Hq + 2 * Hkv) * D, K)); bias = rng.standard_normal((Hq + 2 * Hkv) * D)
    pos = rng.integers(0, 500, size=T)
    q, k, v = qkv_rope_project_ref(h, w, bias, pos, Hq, Hkv, D, 1e4)
    y = torch.nn.functional.linear(torch.from_numpy(h), torch.from_numpy(w), torch.from_numpy(bias)).numpy()
    assert np.allclose(v, y[:, (Hq + Hkv) * D:].reshape(T, Hkv, D))
    assert np.allclose(q, rope_ref(y[:, :Hq * D].reshape(T, Hq, D), pos, 1e4))
    assert np.allclose(k, rope_ref(y[:, Hq * D:(Hq + Hkv) * D].reshape(T, Hkv, D), pos, 1e4))
    # at position 0 the projection is the plain linear layer
    q0, k0, _ = qkv_rope_project_ref(h, w, None, np.zeros(T), Hq, Hkv, D, 1e4)
    y0 = h @ w.T
    assert np.allclose(q0.reshape(T, -1), y0[:, :Hq * D]) and np.allclose(k0.reshape(T, -1), y0[:, Hq * D:(Hq + Hkv) * D])
    r = rng.standard_normal((T, 5)); wo = rng.standard_normal((5, K))
    assert np.allclose(linear_ref(h, wo, r), torch.nn.functional.linear(torch.from_numpy(h), torch.from_numpy(wo)).numpy() + r)


def test_positions():
    # a chain of n nodes behind a prefix of L tokens sits at L, L + 1, ...
    assert list(tree_positions_ref([0, 5], W.chain_tree(5), [100])) == [100, 101, 102, 103, 104]
    # literal tree: depths 0 1 1 2 2 3; second sequence empty, third a single node
    par = [-1, 0, 0, 1, 2, 4, -1]
    assert list(tree_positions_ref([0, 6, 6, 7], par, [10, 99, 0])) == [10, 11, 11, 12, 12, 13, 0]
    t = W.seeded_tree(3)
    assert np.array_equal(tree_positions_ref([0, len(t)], t, [7]), 7 + W.tree_depths(t))


def test_rmsnorm_pins():
    """Unit mean square for eps = 0 and unit weight; scale invariance; a constant row maps to
    +-weight; a hand-worked row; eps as an added variance; torch's rms_norm in float64; the toy
    decoder's own normalisation (pinned separately by the losslessness tests)."""
    from oracle import rmsnorm_ref
    rng = np.random.default_rng(3)
    x, w = rng.standard_normal((6, 40)), rng.standard_normal(40)
    y = rmsnorm_ref(x, np.ones(40), 0.0)
    assert np.allclose((y * y).mean(-1), 1.0)
    assert np.allclose(rmsnorm_ref(7.5 * x, w, 0.0), rmsnorm_ref(x, w, 0.0))
    assert np.allclose(rmsnorm_ref(np.full((1, 40), -3.0), w, 0.0), -w[None, :])
    # x = (3, 4): mean square 12.5; with eps = 3.5 the divisor is 4
    assert np.allclose(rmsnorm_ref([[3.0, 4.0]], [2.0, -1.0], 3.5), [[1.5, -1.0]])
    t = torch.nn.functional.rms_norm(torch.from_numpy(x), (40,), torch.from_numpy(w), eps=1e-6)
    assert np.allclose(rmsnorm_ref(x, w, 1e-6), t.numpy(), atol=1e-14)
    from oracle.toy_decoder import _rms_norm
    assert np.allclose(_rms_norm(x, w), rmsnorm_ref(x, w, 1e-6))


def test_swiglu_pins():
    """silu's closed forms (silu(0) = 0, silu(z) - silu(-z) = z, silu(z) -> z for large z), a
    hand-worked entry, gate and up are not interchangeable, torch's silu in float64, the toy
    decoder's feed-forward block."""
    from oracle import swiglu_ref
    # one token, K = 1, F = 2: gate pre-activations (0, ln 3), up pre-activations (5, 2)
    out = swiglu_ref([[1.0]], [[0.0], [np.log(3.0)], [5.0], [2.0]])
    assert np.allclose(out, [[0.0, np.log(3.0) / (1.0 + 1.0 / 3.0) * 2.0]])
    z = np.linspace(-6, 6, 25)
    s_pos = swiglu_ref(np.ones((25, 1)), np.concatenate([z[:, None], np.ones((25, 1))]))[0]      # silu(z) * 1
    s_neg = swiglu_ref(np.ones((25, 1)), np.concatenate([-z[:, None], np.ones((25, 1))]))[0]
    assert np.allclose(s_pos - s_neg, z)
    assert abs(swiglu_ref([[1.0]], [[40.0], [1.0]])[0, 0] - 40.0) < 1e-12
    rng = np.random.default_rng(4)
    x, w = rng.standard_normal((5, 16)), rng.standard_normal((2 * 12, 16))
    got = swiglu_ref(x, w)
    tx, tw = torch.from_numpy(x), torch.from_numpy(w)
    ref = torch.nn.functional.silu(tx @ tw[:12].T) * (tx @ tw[12:].T)
    assert np.allclose(got, ref.numpy(), atol=1e-13)
    swapped = swiglu_ref(x, np.concatenate([w[12:], w[:12]]))
    assert not np.allclose(got, swapped)
    from oracle.toy_decoder import _silu
    assert np.allclose(_silu(x @ w[:12].T) * (x @ w[12:].T), got)
