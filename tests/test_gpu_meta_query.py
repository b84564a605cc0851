"""GPU parity of the draft model's intermediate layer (meta-query cross-attention, Section 3.1.1,
Eq. 1, with the skip connection and fc1 of Section 3.1.2) against the float64 oracle.

Tolerance: the path is bf16 with fp32 accumulation; the projected values, the attention output
before the output projection and the layer's output are each rounded to bf16 (relative 2^-9), so
outputs of unit scale carry errors of a few 1e-3 in the worst element; asserted: relative L2
error <= 1e-2 and max-abs error <= 2e-2 * (1 + max |reference|), the bar of the attention tests."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import fc_concat_ref, linear_ref, meta_query_attn_ref

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def S():
    import paper_2509_18824_amd.step as s
    return s


def _close(got, ref, what):
    got = got.float().cpu().numpy().astype(np.float64)
    err = np.abs(got - ref)
    rel = np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-30)
    assert rel <= 1e-2 and err.max() <= 2e-2 * (1 + np.abs(ref).max()), (what, rel, err.max())
    return rel


def _run(S, seed, n_tok, L, D, H, Q, layers, peaked=False, zero_wo=False):
    x = W.make_meta_inputs(seed, n_tok, L, D, H, Q, peaked=peaked)
    if zero_wo:
        x["w_o"] = torch.zeros_like(x["w_o"])
    g = {k: v.cuda() for k, v in x.items()}
    layer = S.MetaQueryLayer(g["f_q"], g["w_q"], g["w_k"], g["w_v"], g["w_o"], g["w_fc1"], H, residual_layers=layers)
    f_c, out = layer.run(g["feats"])
    torch.cuda.synchronize()
    w = {k: v.float().numpy().astype(np.float64) for k, v in x.items()}
    ref_c = meta_query_attn_ref(w["f_q"], w["feats"], w["w_q"], w["w_k"], w["w_v"], w["w_o"], H, residual_layers=layers)
    _close(f_c, ref_c, "f_c")
    _close(out, linear_ref(ref_c, w["w_fc1"]), "fc1")
    return f_c, ref_c, x


@pytest.mark.parametrize("n_tok,L,D,H,Q,layers", [
    (5, 6, 256, 2, 3, [0, 2, 5]),        # small: one row tile, layers in one column tile
    (3, 28, 512, 4, 3, [1, 13, 27]),     # 28 layers (two column tiles, the second ragged)
    (7, 32, 768, 3, 4, None),            # 32 layers, four queries, no skip connection
    (2, 17, 1024, 32, 3, [0, 8, 16]),    # 96 (head, query) rows: every row tile
    (1, 1, 256, 2, 1, [0]),              # one layer, one head, one query
    (9, 5, 4352, 34, 2, [0, 4]),         # 17 slices of D over 9 workgroup columns (two slices each, the last one), a ragged
                                         # second token group, more than 4096 features (two column blocks in the mixing)
    (150, 4, 256, 2, 2, None),           # many tokens, a single slice
])
def test_small_shapes(S, n_tok, L, D, H, Q, layers):
    _run(S, 3 + n_tok, n_tok, L, D, H, Q, layers)
    _run(S, 13 + n_tok, n_tok, L, D, H, Q, layers, peaked=True)


def test_target_model_shape(S):
    """28 layers of hidden size 3584, 28 heads of 128, three queries: the 96 tokens that a
    batch of 16 sequences commits per step at most."""
    _run(S, 40, 96, 28, 3584, 28, 3, [2, 14, 27])
    _run(S, 41, 24, 28, 3584, 28, 3, [2, 14, 27], peaked=True)


def test_prefill_scale_on_sampled_tokens(S):
    """1024 tokens of the target model's shape (one workgroup column per two slices of D in the
    score kernel, 128 token groups); every token is independent of the others, so the oracle
    checks 24 sampled ones."""
    n_tok, L, D, H, Q, layers = 1024, 28, 3584, 28, 3, [2, 14, 27]
    x = W.make_meta_inputs(77, n_tok, L, D, H, Q)
    g = {k: v.cuda() for k, v in x.items()}
    layer = S.MetaQueryLayer(g["f_q"], g["w_q"], g["w_k"], g["w_v"], g["w_o"], g["w_fc1"], H, residual_layers=layers)
    f_c, out = layer.run(g["feats"])
    torch.cuda.synchronize()
    pick = np.sort(np.random.default_rng(5).choice(n_tok, 24, replace=False))
    pick[0], pick[-1] = 0, n_tok - 1
    w = {k: v.float().numpy().astype(np.float64) for k, v in x.items() if k != "feats"}
    feats = x["feats"][torch.from_numpy(pick)].float().numpy().astype(np.float64)
    ref_c = meta_query_attn_ref(w["f_q"], feats, w["w_q"], w["w_k"], w["w_v"], w["w_o"], H, residual_layers=layers)
    _close(f_c[torch.from_numpy(pick).cuda()], ref_c, "f_c")
    _close(out[torch.from_numpy(pick).cuda()], linear_ref(ref_c, w["w_fc1"]), "fc1")


def test_zero_initialised_output_projection_passes_the_feature_levels_through(S):
    """Section 3.1.2: with W_o at zero the layer's output is the three residual features, bit for bit."""
    f_c, ref_c, x = _run(S, 50, 9, 28, 512, 4, 3, [0, 13, 27], zero_wo=True)
    want = torch.cat([x["feats"][:, l, :] for l in (0, 13, 27)], dim=1)
    assert torch.equal(f_c.cpu(), want)


def test_fc_over_a_concatenation(S):
    rng = np.random.default_rng(7)
    bf = lambda a: torch.from_numpy(a.astype(np.float32)).to(torch.bfloat16)
    a, b = bf(rng.normal(size=(33, 512))), bf(rng.normal(size=(33, 512)))
    w = bf(rng.normal(0, 1024 ** -0.5, size=(512, 1024)))
    out = S.fc_concat(a.cuda(), b.cuda(), w[:, :512].contiguous().cuda(), w[:, 512:].contiguous().cuda())
    torch.cuda.synchronize()
    f = lambda t: t.float().numpy().astype(np.float64)
    _close(out, fc_concat_ref(f(a), f(b), f(w)), "fc2")
