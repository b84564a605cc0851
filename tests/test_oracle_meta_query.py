"""Pins of the meta-query cross-attention oracle (oracle/meta_query.py): the library's multi-head
attention, the zero-initialisation property the paper states (Section 3.1.2), closed forms."""
import numpy as np
import torch

from oracle.meta_query import fc_concat_ref, meta_query_attn_ref
from oracle.projections import linear_ref


def _case(seed, S=5, L=6, D=32, H=4, Q=3):
    rng = np.random.default_rng(seed)
    f_q = rng.normal(0, 1, (Q, D))
    feats = rng.normal(0, 1, (S, L, D))
    ws = [rng.normal(0, D ** -0.5, (D, D)) for _ in range(4)]
    return f_q, feats, ws


def test_against_the_library_multi_head_attention():
    f_q, feats, (wq, wk, wv, wo) = _case(1)
    S, L, D = feats.shape
    Q, H = f_q.shape[0], 4
    t = lambda a: torch.from_numpy(np.asarray(a)).double()
    query = t(f_q)[:, None, :].expand(Q, S, D)          # the same queries for every token
    kv = t(feats).transpose(0, 1)                        # [L, S, D]
    ref, _ = torch.nn.functional.multi_head_attention_forward(
        query, kv, kv, D, H, in_proj_weight=torch.cat([t(wq), t(wk), t(wv)]), in_proj_bias=None, bias_k=None,
        bias_v=None, add_zero_attn=False, dropout_p=0.0, out_proj_weight=t(wo), out_proj_bias=None, need_weights=False)
    got = meta_query_attn_ref(f_q, feats, wq, wk, wv, wo, H).reshape(S, Q, D)
    assert np.abs(got - ref.transpose(0, 1).numpy()).max() < 1e-12


def test_zero_initialised_output_projection_passes_the_three_feature_levels_through():
    """Section 3.1.2: with the attention's last projection at zero, what reaches fc1 is the low-,
    middle- and high-level feature of each token, side by side."""
    f_q, feats, (wq, wk, wv, wo) = _case(2)
    layers = [0, 3, 5]
    got = meta_query_attn_ref(f_q, feats, wq, wk, wv, np.zeros_like(wo), 4, residual_layers=layers)
    want = np.concatenate([feats[:, l, :] for l in layers], axis=1)
    assert np.array_equal(got, want)
    # and the residual is added, not substituted, otherwise
    full = meta_query_attn_ref(f_q, feats, wq, wk, wv, wo, 4, residual_layers=layers)
    assert np.abs((full - meta_query_attn_ref(f_q, feats, wq, wk, wv, wo, 4)) - want).max() < 1e-12


def test_closed_forms():
    f_q, feats, (wq, wk, wv, wo) = _case(3)
    S, L, D = feats.shape
    # keys at zero: every layer gets weight 1 / L
    got = meta_query_attn_ref(f_q, feats, wq, np.zeros_like(wk), wv, wo, 4).reshape(S, -1, D)
    want = (feats.mean(axis=1) @ wv.T) @ wo.T
    assert np.abs(got - want[:, None, :]).max() < 1e-12
    # one layer: the softmax is 1
    one = meta_query_attn_ref(f_q, feats[:, :1], wq, wk, wv, wo, 4).reshape(S, -1, D)
    assert np.abs(one - ((feats[:, 0] @ wv.T) @ wo.T)[:, None, :]).max() < 1e-12
    # a planted layer whose key matches a query head strongly takes all of that head's weight
    H, d = 4, D // 4
    eye = np.eye(D)
    feats2 = feats.copy()
    feats2[:, 2, :d] = 60.0 * f_q[1, :d] / np.linalg.norm(f_q[1, :d])
    got = meta_query_attn_ref(f_q, feats2, eye, eye, eye, eye, H).reshape(S, -1, D)
    assert np.abs(got[:, 1, :d] - feats2[:, 2, :d]).max() < 1e-6
    # heads are independent: changing head 3's key columns leaves heads 0..2 of the pre-projection
    # output alone (identity output projection shows them)
    feats3 = feats.copy()
    feats3[:, :, 3 * d:] += 1.0
    a = meta_query_attn_ref(f_q, feats, eye, eye, eye, eye, H).reshape(S, -1, D)
    b = meta_query_attn_ref(f_q, feats3, eye, eye, eye, eye, H).reshape(S, -1, D)
    assert np.abs(a[:, :, :3 * d] - b[:, :, :3 * d]).max() < 1e-12 and np.abs(a[:, :, 3 * d:] - b[:, :, 3 * d:]).max() > 0.1


def test_fc_over_a_concatenation_is_the_sum_of_two_linear_layers():
    rng = np.random.default_rng(4)
    a, b = rng.normal(size=(7, 16)), rng.normal(size=(7, 24))
    w = rng.normal(size=(10, 40))
    assert np.abs(fc_concat_ref(a, b, w) - (linear_ref(a, w[:, :16]) + linear_ref(b, w[:, 16:]))).max() < 1e-12
    assert np.array_equal(fc_concat_ref(a, b, np.zeros_like(w)), np.zeros((7, 10)))  # zero-initialised fc2
