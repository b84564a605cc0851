"""GPU parity: positions, rotary table, fused QKV projection + rotary embedding, output projection
against the float64 oracle.

Tolerances (bf16 outputs of fp32-accumulated products of bf16 inputs): the result is rounded once
to bf16 (relative 2^-9 = 2e-3); fp32 accumulation over K <= 3584 terms adds well under 1e-5
relative to the sum of magnitudes.  Tested as: max abs error <= 1e-2 * (1 + |ref|) elementwise and
relative L2 error <= 4e-3."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import tree_positions_ref, rope_ref, qkv_rope_project_ref, linear_ref, rmsnorm_ref, swiglu_ref

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hb():
    import paper_2509_18824_amd as m
    return m


def _close(got, ref, label):
    got = W.widen(got)
    err = np.abs(got - ref)
    assert np.isfinite(got).all(), label
    assert (err <= 1e-2 * (1.0 + np.abs(ref))).all(), f"{label}: max abs err {err.max():.3e}"
    rel = np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-30)
    assert rel <= 4e-3, f"{label}: rel L2 {rel:.3e}"


def test_positions_and_rope_table(hb):
    rng = np.random.default_rng(0)
    trees = [W.seeded_tree(1), np.array([], dtype=np.int32), W.chain_tree(8), W.seeded_tree(2, n_nodes=64), W.chain_tree(1)]
    off = np.concatenate([[0], np.cumsum([len(t) for t in trees])]).astype(np.int32)
    par = np.concatenate(trees).astype(np.int32)
    L = np.array([32768, 5, 0, 4095, 17], dtype=np.int32)
    t = lambda a: torch.from_numpy(a).cuda()
    pos = torch.full((int(off[-1]),), -1, dtype=torch.int32, device="cuda")
    hb.hb_tree_positions(len(trees), 64, t(off), t(par), t(L), pos)
    ref = tree_positions_ref(off, par, L)
    assert np.array_equal(pos.cpu().numpy(), ref)
    for theta in (1e4, 1e6):
        cos = torch.empty((pos.numel(), 64), dtype=torch.float32, device="cuda")
        sin = torch.empty_like(cos)
        hb.hb_rope_table(128, theta, pos, cos, sin)
        ang = ref[:, None].astype(np.float64) * theta ** (-np.arange(64) / 64.0)
        assert np.abs(cos.cpu().numpy() - np.cos(ang)).max() <= 2e-7
        assert np.abs(sin.cpu().numpy() - np.sin(ang)).max() <= 2e-7


@pytest.mark.parametrize("T,K,Hq,Hkv,bias", [(960, 3584, 28, 4, True), (128, 3584, 28, 4, False), (77, 128, 2, 1, True),
                                             (300, 320, 3, 3, False), (300, 320, 3, 3, True), (1, 64, 1, 1, True), (513, 192, 8, 2, True),
                                             (100, 256, 2, 1, True), (1, 512, 1, 1, True), (16, 768, 3, 3, False),
                                             (128, 1024, 4, 2, True)])
def test_qkv_projection_with_rotary_embedding(hb, T, K, Hq, Hkv, bias):
    _qkv_case(hb, T, K, Hq, Hkv, bias, False)


@pytest.mark.parametrize("T,K,Hq,Hkv,bias", [(128, 3584, 28, 4, True), (100, 256, 2, 1, True), (1, 512, 1, 1, False),
                                             (64, 768, 3, 3, True), (65, 1024, 4, 2, False), (300, 320, 3, 3, True),
                                             (288, 3584, 28, 4, True), (200, 1024, 3, 1, False), (512, 2048, 2, 2, True),
                                             (513, 2048, 2, 1, True)])
def test_qkv_projection_split_over_k(hb, T, K, Hq, Hkv, bias):
    """The workspace variant: at most 512 tokens take the split-K path when K has enough steps
    (one or several hidden tiles per weight tile and K part), up to 1024 tokens when the cost
    model expects a gain, anything else the ordinary one."""
    _qkv_case(hb, T, K, Hq, Hkv, bias, True)


def _qkv_case(hb, T, K, Hq, Hkv, bias, with_workspace):
    g = torch.Generator().manual_seed(T * 7 + K)
    hidden = torch.randn((T, K), generator=g).to(torch.bfloat16)
    w = (torch.randn(((Hq + 2 * Hkv) * 128, K), generator=g) * (1.0 / np.sqrt(K))).to(torch.bfloat16)
    b = (torch.randn((Hq + 2 * Hkv) * 128, generator=g) * 0.5).to(torch.bfloat16) if bias else None
    pos = torch.randint(0, 40000, (T,), generator=g, dtype=torch.int32)
    theta = 1e6
    cos = torch.empty((T, 64), dtype=torch.float32, device="cuda")
    sin = torch.empty_like(cos)
    hb.hb_rope_table(128, theta, pos.cuda(), cos, sin)
    q = torch.full((T, Hq, 128), float("nan"), dtype=torch.bfloat16, device="cuda")
    k = torch.full((T, Hkv, 128), float("nan"), dtype=torch.bfloat16, device="cuda")
    v = torch.full((T, Hkv, 128), float("nan"), dtype=torch.bfloat16, device="cuda")
    if with_workspace:
        nbytes = hb.hb_proj_workspace_bytes(T, K, (Hq + 2 * Hkv) * 128)
        assert nbytes == 0 if (K < 512 or T > 1024) else (nbytes > 0 or T > 512)
        ws = torch.full((max(nbytes, 16),), 0xFF, dtype=torch.uint8, device="cuda")  # NaN patterns: nothing may be read unwritten
        hb.hb_qkv_rope_project_ws(hidden.cuda(), w.cuda(), None if b is None else b.cuda(), cos, sin, q, k, v, ws)
    else:
        hb.hb_qkv_rope_project(hidden.cuda(), w.cuda(), None if b is None else b.cuda(), cos, sin, q, k, v)
    torch.cuda.synchronize()
    rq, rk, rv = qkv_rope_project_ref(W.widen(hidden), W.widen(w), None if b is None else W.widen(b), pos.numpy(),
                                      Hq, Hkv, 128, theta)
    _close(q, rq, "q"); _close(k, rk, "k"); _close(v, rv, "v")


@pytest.mark.parametrize("T,K,N,res", [(960, 3584, 3584, True), (128, 3584, 3584, False), (50, 64, 4, True),
                                       (333, 448, 1000, False), (700, 256, 260, True),
                                       (128, 3584, 3584, True), (37, 256, 20, True), (5, 512, 1000, False),
                                       (96, 10752, 3584, False), (1, 256, 4, True)])
def test_output_projection(hb, T, K, N, res):
    _out_case(hb, T, K, N, res, False)


@pytest.mark.parametrize("T,K,N,res", [(128, 3584, 3584, True), (96, 10752, 3584, False), (37, 256, 20, True),
                                       (5, 512, 1000, False), (1, 1024, 4, True), (64, 2048, 260, True),
                                       (129, 512, 512, True), (288, 3584, 3584, True), (300, 1024, 520, False),
                                       (512, 2048, 260, True), (450, 768, 2052, True), (960, 18944, 3584, True),
                                       (768, 9472, 520, False), (1024, 4096, 260, True), (1025, 4096, 260, True)])
def test_output_projection_split_over_k(hb, T, K, N, res):
    _out_case(hb, T, K, N, res, True)


def _out_case(hb, T, K, N, res, with_workspace):
    g = torch.Generator().manual_seed(T + K + N)
    x = torch.randn((T, K), generator=g).to(torch.bfloat16)
    w = (torch.randn((N, K), generator=g) * (1.0 / np.sqrt(K))).to(torch.bfloat16)
    r = torch.randn((T, N), generator=g).to(torch.bfloat16) if res else None
    out = torch.full((T, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    if with_workspace:
        nbytes = hb.hb_proj_workspace_bytes(T, K, N)
        ws = torch.full((max(nbytes, 16),), 0xFF, dtype=torch.uint8, device="cuda")
        hb.hb_out_project_ws(x.cuda(), w.cuda(), None if r is None else r.cuda(), out, ws)
    else:
        hb.hb_out_project(x.cuda(), w.cuda(), None if r is None else r.cuda(), out)
    torch.cuda.synchronize()
    _close(out, linear_ref(W.widen(x), W.widen(w), None if r is None else W.widen(r)), "out")


@pytest.mark.parametrize("T,K,eps", [(960, 3584, 1e-6), (128, 3584, 1e-6), (1, 8, 0.0), (7, 8200, 1e-5), (33, 72, 1e-2),
                                     (5, 16384, 1e-6)])
def test_rmsnorm(hb, T, K, eps):
    """Rows that fit the registers a thread keeps (K <= 8192), longer ones, the shortest."""
    g = torch.Generator().manual_seed(T + K)
    x = (torch.randn((T, K), generator=g) * 3.0 + 0.5).to(torch.bfloat16)
    w = (1.0 + 0.3 * torch.randn(K, generator=g)).to(torch.bfloat16)
    out = torch.full((T, K), float("nan"), dtype=torch.bfloat16, device="cuda")
    hb.hb_rmsnorm(x.cuda(), w.cuda(), eps, out)
    torch.cuda.synchronize()
    _close(out, rmsnorm_ref(W.widen(x), W.widen(w), eps), "rmsnorm")
    xin = x.cuda()
    hb.hb_rmsnorm(xin, w.cuda(), eps, xin)   # in place
    torch.cuda.synchronize()
    assert torch.equal(xin, out)


@pytest.mark.parametrize("T,K,F,ws", [(960, 3584, 18944, False), (128, 3584, 18944, True), (128, 3584, 18944, False),
                                      (77, 128, 132, True), (300, 320, 100, False), (1, 64, 4, True),
                                      (513, 192, 520, True), (40, 1024, 260, True), (288, 2048, 1000, True)])
def test_gated_silu_projection(hb, T, K, F, ws):
    """Gate and up projection in one pass with silu(gate) * up in the epilogue: the feed-forward
    width of the target model's shape for trees (960 tokens) and chains (128 tokens, split over K),
    ragged feature counts (the last tile holds fewer than 128 features), a single token."""
    g = torch.Generator().manual_seed(T * 3 + K + F)
    x = torch.randn((T, K), generator=g).to(torch.bfloat16)
    w = (torch.randn((2 * F, K), generator=g) * (1.5 / np.sqrt(K))).to(torch.bfloat16)
    out = torch.full((T, F), float("nan"), dtype=torch.bfloat16, device="cuda")
    wsp = None
    if ws:
        nbytes = hb.hb_proj_workspace_bytes(T, K, 2 * F)
        wsp = torch.full((max(nbytes, 16),), 0xFF, dtype=torch.uint8, device="cuda")
    hb.hb_swiglu_project(x.cuda(), w.cuda(), out, wsp)
    torch.cuda.synchronize()
    _close(out, swiglu_ref(W.widen(x), W.widen(w)), "swiglu")


@pytest.mark.parametrize("scale_down,K,tree", [(16, 512, "tree"), (1, 3584, "tree"), (1, 3584, "chain8")])
def test_projected_qkv_feed_the_attention(hb, scale_down, K, tree):
    """hidden -> QKV + rotary -> tree-verify attention -> output projection, against the oracle
    chained the same way on the bf16 tensors the GPU hands from step to step; also one whole layer
    of the batch-16 workload at full size (960 tree tokens, and 128 tokens of 8-node chains, which
    take the split-K projections; hidden size 3584, prefixes of 1024-4096 tokens)."""
    import paper_2509_18824_amd.step as S
    from oracle import tree_attn_ref
    inp = W.make_config(4, scale_down=scale_down, tree=tree)
    T, Hq, Hkv, D = inp.total_nodes, inp.Hq, inp.Hkv, inp.D
    g = torch.Generator().manual_seed(5)
    hidden = torch.randn((T, K), generator=g).to(torch.bfloat16)
    wqkv = (torch.randn(((Hq + 2 * Hkv) * D, K), generator=g) / np.sqrt(K)).to(torch.bfloat16)
    wo = (torch.randn((K, Hq * D), generator=g) / np.sqrt(Hq * D)).to(torch.bfloat16)
    dev = S.to_device(inp)
    pos = torch.empty(T, dtype=torch.int32, device="cuda")
    hb.hb_tree_positions(inp.B, 64, dev.node_offset, dev.parent, dev.prefix_len, pos)
    cos = torch.empty((T, 64), dtype=torch.float32, device="cuda"); sin = torch.empty_like(cos)
    hb.hb_rope_table(D, 1e6, pos, cos, sin)
    ws = S.alloc_workspace(max(hb.hb_proj_workspace_bytes(T, K, (Hq + 2 * Hkv) * D), hb.hb_proj_workspace_bytes(T, Hq * D, K)))
    hb.hb_qkv_rope_project_ws(hidden.cuda(), wqkv.cuda(), None, cos, sin, dev.q, dev.k_tree, dev.v_tree, ws)
    desc = S.desc_for(inp)
    out, _ = S.tree_verify_attn(desc, dev, want_lse=False)
    y = torch.empty((T, K), dtype=torch.bfloat16, device="cuda")
    hb.hb_out_project_ws(out.view(T, -1), wo.cuda(), hidden.cuda(), y, ws)
    torch.cuda.synchronize()
    ref_pos = tree_positions_ref(inp.node_offset.numpy(), inp.parent.numpy(), inp.prefix_len.numpy())
    rq, rk, rv = qkv_rope_project_ref(W.widen(hidden), W.widen(wqkv), None, ref_pos, Hq, Hkv, D, 1e6)
    _close(dev.q, rq, "q"); _close(dev.k_tree, rk, "k"); _close(dev.v_tree, rv, "v")
    ref_attn, _ = tree_attn_ref(W.widen(dev.q), W.widen(dev.k_tree), W.widen(dev.v_tree), W.widen(inp.k_pool),
                                W.widen(inp.v_pool), inp.block_table.numpy(), inp.prefix_len.numpy(),
                                inp.node_offset.numpy(), inp.parent.numpy(), inp.softmax_scale)
    got_attn = W.widen(out)
    assert np.linalg.norm(got_attn - ref_attn) / np.linalg.norm(ref_attn) <= 1e-2
    _close(y, linear_ref(got_attn.reshape(T, -1), W.widen(wo), W.widen(hidden)), "layer output")
