"""GPU parity of the draft tree's construction: hb_topk_logprob (token ids exact, log-probabilities
within 2e-5 of the float64 definition: float32 exp/log and a float32 sum over the vocabulary),
hb_tree_grow and hb_tree_finalize (bit-exact: integer outputs, and scores that are one float32
addition each)."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import DraftTreeRef, topk_logprob_ref

pytestmark = pytest.mark.gpu

LOGP_TOL = 2e-5


@pytest.fixture(scope="module")
def S():
    import paper_2509_18824_amd.step as s
    return s


def _topk_case(S, x, k, bf16=False):
    t = torch.from_numpy(x).cuda()
    if bf16:
        t = t.to(torch.bfloat16)
        x = t.float().cpu().numpy()
    ids, logp = S.topk_logprob(t.contiguous(), k)
    torch.cuda.synchronize()
    rid, rlogp = topk_logprob_ref(x, k)
    assert np.array_equal(ids.cpu().numpy(), rid)
    got = logp.cpu().numpy()
    assert np.abs(got - rlogp).max() <= LOGP_TOL, np.abs(got - rlogp).max()
    assert (got <= 0).all()


@pytest.mark.parametrize("M,V,k", [(5, 1000, 4), (3, 2049, 32), (7, 33, 8), (3, 1001, 5), (1, 16384, 10),
                                   (2, 16385, 10), (40, 32000, 10), (1, 7, 7)])
def test_topk_small_shapes(S, M, V, k):
    _topk_case(S, W.make_draft_logits(11 + M, M, V), k)


@pytest.mark.parametrize("M,V,k", [(4, 5000, 16), (2, 40000, 10)])
def test_topk_equal_logits_go_to_the_lower_token_id(S, M, V, k):
    _topk_case(S, W.make_draft_logits(21, M, V, ties=True), k)
    x = np.zeros((2, 3000), dtype=np.float32)  # everything equal, signed zeros mixed in
    x[0, ::2] = -0.0
    _topk_case(S, x, 9)
    x = np.full((1, 2500), -np.inf, dtype=np.float32)  # -inf entries are ordinary, just last
    x[0, [2000, 17]] = [1.0, 1.0]
    ids, logp = S.topk_logprob(torch.from_numpy(x).cuda(), 4)
    assert ids.cpu().numpy().tolist() == [[17, 2000, 0, 1]]
    assert np.allclose(logp.cpu().numpy()[0, :2], -np.log(2.0), atol=1e-6) and np.isneginf(logp.cpu().numpy()[0, 2:]).all()


@pytest.mark.parametrize("M,V,k,bf16,ties", [(3, 16388, 10, False, False),   # last chunk: a single 16-byte vector
                                              (70, 32768, 12, True, True),     # bf16, more than a thousand chunks
                                              (600, 4096, 10, False, False),   # one chunk per row, two rounds of rows
                                              (33, 40008, 32, True, False)])   # bf16, last chunk of one vector, k = 32
def test_topk_rows_of_whole_vectors(S, M, V, k, bf16, ties):
    """Rows that consist of whole 16-byte vectors (vector loads all the way, no ragged end), with
    a last chunk of a single vector, many more chunks than resident workgroups, bf16 and ties."""
    _topk_case(S, W.make_draft_logits(41 + M, M, V, ties=ties), k, bf16=bf16)


def test_topk_full_vocabulary_every_row_of_a_level(S):
    """The shape of one level of the batch-16 workload: 160 rows (16 sequences x 10 frontier
    nodes) over the vocabulary of 152064, float32; and the root level's 16 rows in bf16."""
    _topk_case(S, W.make_draft_logits(31, 160, 152064), 10)
    _topk_case(S, W.make_draft_logits(32, 16, 152064), 10, bf16=True)


def _grow_both(S, B, K, T, N, V, seed, ties=False, uniform=False):
    builder = S.DraftTreeBuilder(B, K, T)
    refs = [DraftTreeRef(K, T) for _ in range(B)]
    for level in range(T):
        F = 1 if level == 0 else K
        if uniform:
            ids = torch.arange(K, dtype=torch.int32).repeat(B * F, 1).cuda() + 100 * level
            logp = torch.full((B * F, K), -2.0, dtype=torch.float32).cuda()
        else:
            logits = torch.from_numpy(W.make_draft_logits(seed * 100 + level, B * F, V, ties=ties)).cuda()
            ids, logp = S.topk_logprob(logits, K)
        frontier, slot = builder.grow(ids, logp)
        torch.cuda.synchronize()
        ids_h = ids.cpu().numpy().reshape(B, F, K)
        logp_h = logp.cpu().numpy().reshape(B, F, K)
        for b in range(B):
            rf, rs = refs[b].grow(ids_h[b], logp_h[b])
            assert frontier[b].cpu().numpy().tolist() == rf, (level, b)
            assert slot[b].cpu().numpy().tolist() == rs, (level, b)
    root = torch.arange(B, dtype=torch.int32).cuda() + 7
    out = builder.finalize(N, root)
    torch.cuda.synchronize()
    n = N
    h = {k: v.cpu().numpy() for k, v in out.items()}
    assert h["node_offset"].tolist() == [b * n for b in range(B + 1)]
    import paper_2509_18824_amd as hb
    for b in range(B):
        parent, ids, depth, anc, cand, score = refs[b].finalize(N, 7 + b)
        sl = slice(b * n, (b + 1) * n)
        assert len(parent) == n
        assert np.array_equal(h["parent"][sl], parent), b
        assert np.array_equal(h["draft_ids"][sl], ids), b
        assert np.array_equal(h["depth"][sl], depth), b
        assert np.array_equal(h["anc_mask"][sl].view(np.uint64), anc), b
        assert np.array_equal(h["node_cand"][sl], cand), b
        assert np.array_equal(h["node_score"][sl].view(np.uint32), score.view(np.uint32)), b
        hb.hb_tree_validate_host(h["parent"][sl].tolist())
    return h


def test_tree_of_the_batch16_workload_shape(S):
    """16 sequences, 10 children per node, 5 levels, 60 nodes: the tree shape the verification
    workloads use."""
    h = _grow_both(S, 16, 10, 5, 60, 32000, seed=1)
    assert h["depth"].max() <= 5 and h["depth"].max() >= 2


@pytest.mark.parametrize("B,K,T,N", [(1, 1, 5, 6), (3, 2, 2, 4), (2, 4, 3, 1), (2, 3, 3, 22), (5, 8, 4, 64),
                                     (2, 32, 2, 40), (1, 7, 1, 8)])
def test_tree_shapes_and_edges(S, B, K, T, N):
    """Chains (K = 1), root-only trees (N = 1), everything kept (N - 1 = all candidates), the
    widest node (K = 32), the largest tree (64 nodes), a single level."""
    h = _grow_both(S, B, K, T, N, 5000, seed=B + K + T)
    if K == 1:
        assert h["parent"].tolist() == [-1, 0, 1, 2, 3, 4]


def test_tree_with_equal_scores(S):
    _grow_both(S, 2, 3, 3, 9, 0, seed=0, uniform=True)
    _grow_both(S, 4, 6, 4, 48, 3000, seed=9, ties=True)


def test_tree_build_replays_from_a_hip_graph(S):
    """Top-k, growth of every level and finalisation only enqueue kernels (no allocation, no
    memset): captured once, replayed on changing logits with eager builds in between, every replay
    equals the eager build bit for bit."""
    import paper_2509_18824_amd as hb
    B, K, T, N, V = 4, 5, 3, 24, 6000
    levels = [torch.empty((B * (1 if l == 0 else K), V), dtype=torch.float32, device="cuda") for l in range(T)]
    ids = [torch.empty((x.shape[0], K), dtype=torch.int32, device="cuda") for x in levels]
    lps = [torch.empty((x.shape[0], K), dtype=torch.float32, device="cuda") for x in levels]
    ws = S.alloc_workspace(hb.hb_topk_logprob_workspace_bytes(B * K, V, K))
    builder = S.DraftTreeBuilder(B, K, T)
    root = torch.arange(B, dtype=torch.int32, device="cuda")
    n = B * N
    i32 = lambda m: torch.empty(m, dtype=torch.int32, device="cuda")
    outs = [i32(B + 1), i32(n), i32(n), i32(n), torch.empty(n, dtype=torch.int64, device="cuda"), i32(n),
            torch.empty(n, dtype=torch.float32, device="cuda")]

    def build():
        for l in range(T):
            hb.hb_topk_logprob(levels[l], K, ids[l], lps[l], ws)
            hb.hb_tree_grow(B, K, T, l, ids[l], lps[l], builder.cand_score, builder.cand_token, builder.cand_parent,
                            builder.frontier, builder.frontier_slot)
        hb.hb_tree_finalize(B, K, T, N, builder.cand_score, builder.cand_token, builder.cand_parent, root, *outs)

    def fill(seed):
        for l, x in enumerate(levels):
            x.copy_(torch.from_numpy(W.make_draft_logits(seed * 10 + l, x.shape[0], V)))

    fill(0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        build()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        build()
    seen = set()
    for seed in (1, 2, 3):
        fill(seed)
        build()
        torch.cuda.synchronize()
        eager = [t.clone() for t in outs]
        for t in outs:
            t.zero_()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(eager, outs):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))
        hb.hb_tree_validate_host(outs[1][:N].cpu().tolist())
        seen.add(tuple(outs[2].cpu().tolist()))
    assert len(seen) == 3  # the logits, and with them the trees, did change between replays
