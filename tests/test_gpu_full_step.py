"""GPU end-to-end checks: the full verification step of the batch-16 workload against the
oracle, and greedy losslessness on the toy decoder with the GPU kernels in the loop."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import ToyDecoderRef, tree_accept_ref, kv_compact_ref, lmhead_logits_ref
from parity import bits, check_attn, oracle_attn

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def S():
    import paper_2509_18824_amd.step as s
    return s


@pytest.mark.parametrize("tree", ["tree", "chain8"])
def test_full_step_scaled(S, tree):
    """Attention -> LM head -> acceptance -> compaction on a scaled copy of the full-step
    workload (vocab 8192 instead of 152064 so the oracle covers every node).  Two passes, as in
    the benchmark: pass 1 yields the target ids, the host plants draft ids along a seeded path,
    pass 2 is the step under test."""
    inp = W.make_config(4, scale_down=8, tree=tree)
    V = 8192
    _, weight = W.make_lmhead_inputs(44, 1, inp.Hq * inp.D, V, dtype="bf16")
    dev = S.to_device(inp)
    desc = S.desc_for(inp)
    k_pool0, v_pool0 = bits(dev.k_pool).copy(), bits(dev.v_pool).copy()
    wdev = weight.cuda()
    dummy = torch.zeros(inp.total_nodes, dtype=torch.int32, device="cuda")
    stp = S.VerifyStep(desc, dev, wdev, dummy, inp.max_path)
    stp.run(compact=False)
    torch.cuda.synchronize()
    target = stp.target_ids.cpu().numpy()
    draft, planted = W.plant_draft_ids(4, inp.trees(), target, V)
    stp.draft_ids.copy_(torch.from_numpy(draft))
    stp.run(compact=True)
    torch.cuda.synchronize()

    # attention against the oracle
    ref_out, ref_lse = oracle_attn(inp)
    check_attn(inp, stp.out, None, ref=(ref_out, ref_lse), label="full step attention")
    # LM head: the oracle is fed the GPU's bf16 hidden states (decouples it from attention rounding)
    hidden = W.widen(stp.out.view(inp.total_nodes, -1))
    logits = lmhead_logits_ref(hidden, W.widen(weight))
    order = np.argsort(-logits, axis=1, kind="stable")[:, :2]
    r = np.arange(inp.total_nodes)
    margin = logits[r, order[:, 0]] - logits[r, order[:, 1]]
    eps = 1e-4 * np.linalg.norm(hidden, axis=1) * 0.02 * np.sqrt(hidden.shape[1])
    got = stp.target_ids.cpu().numpy()
    clear = margin > eps
    assert (got[clear] == order[clear, 0]).all() and clear.mean() > 0.95
    assert np.logical_or(got == order[:, 0], got == order[:, 1]).all()
    # acceptance and compaction: bit exact given the same target ids
    alen, apath, otoks, bonus = tree_accept_ref(inp.node_offset.numpy(), inp.parent.numpy(), draft, got, inp.max_path)
    assert np.array_equal(stp.accept_len.cpu().numpy(), alen)
    assert np.array_equal(stp.accept_path.cpu().numpy(), apath)
    assert np.array_equal(stp.out_tokens.cpu().numpy(), otoks)
    assert np.array_equal(stp.bonus.cpu().numpy(), bonus)
    assert list(alen) == [d + 1 for d in planted]
    rk, rv, rslots, rlen = kv_compact_ref(bits(inp.k_tree), bits(inp.v_tree), k_pool0, v_pool0,
                                          inp.block_table.numpy(), inp.prefix_len.numpy(),
                                          inp.node_offset.numpy(), alen, apath)
    assert np.array_equal(stp.out_slots.cpu().numpy(), rslots)
    assert np.array_equal(stp.new_len.cpu().numpy(), rlen)
    assert np.array_equal(bits(dev.k_pool), rk) and np.array_equal(bits(dev.v_pool), rv)


@pytest.mark.parametrize("kind", ["random", "replay", "corrupting"])
@pytest.mark.parametrize("topology", ["tree", "chain4"])
def test_greedy_losslessness_on_the_toy_decoder(kind, topology):
    """Speculative decoding with the GPU kernels emits exactly the oracle's plain greedy
    autoregressive stream (paper Section 1, Section 4.1 'Setup')."""
    from toy_gpu import ToyDecoderGpu
    w = W.make_toy_weights(0)
    ref = ToyDecoderRef(w)
    prompt = [int(t) for t in np.random.default_rng(100).integers(0, w.vocab, size=40)]
    n_new = 48
    stream, margin = ref.greedy_ar(prompt, n_new)
    assert margin > 1e-3  # fp32 reordering cannot flip an argmax
    drafter = {
        "random": W.random_drafter(1, w.vocab),
        "replay": W.replay_drafter(1, w.vocab, len(prompt), stream),
        "corrupting": W.replay_drafter(1, w.vocab, len(prompt), stream, wrong_after=(0, 4)),
    }[kind]
    tree = (lambda s: W.seeded_tree(s, n_nodes=16, levels=5, root_fanout=3, max_fanout=3)) \
        if topology == "tree" else (lambda s: W.chain_tree(4))
    table = np.random.default_rng(3).permutation(16)
    gpu = ToyDecoderGpu(w, n_blocks=16)
    out, lens = gpu.spec_decode(prompt, n_new, drafter, tree, table)
    assert out == stream
    if kind == "replay":
        full = 5 if topology == "tree" else 4
        assert all(l == full for l in lens[:-1])


def _bf16_toy():
    """A toy whose verification step runs on the matrix-core kernels (bf16, head_dim 128, 8 query /
    2 kv heads, vocabulary 4096), with a seed and prompt for which the plain greedy stream of its
    exact description (float64 arithmetic, bf16 rounding where the kernels' interfaces round) keeps
    a top-1 margin of at least 1.0 logit at every step: about 3 % of the logits' spread and more
    than an order of magnitude above what bf16 rounding noise (one step in the last place of some
    attention outputs and hidden states) moves a logit by.  The seed search is deterministic."""
    from oracle.toy_decoder import round_bf16
    for seed in range(200):
        w = W.make_toy_weights(seed, d=256, n_layers=2, Hq=8, Hkv=2, Dh=128, ffn=512, vocab=4096, lm_head_bf16=True)
        ref = ToyDecoderRef(w, quant=round_bf16)
        prompt = [int(t) for t in np.random.default_rng(seed).integers(0, w.vocab, size=24)]
        stream, margin = ref.greedy_ar(prompt, 16)
        if margin >= 1.0:
            return w, prompt, stream
    raise AssertionError("no seed with a wide enough margin")


@pytest.fixture(scope="module")
def bf16_toy():
    return _bf16_toy()


@pytest.mark.parametrize("kind", ["random", "replay", "corrupting"])
@pytest.mark.parametrize("topology", ["tree60", "chain4", "single"])
def test_greedy_losslessness_with_the_matrix_core_kernels_in_the_loop(bf16_toy, kind, topology):
    """The draft-verify-accept-compact loop on the bf16 path (MFMA attention; MFMA LM head; acceptance; compaction into bf16 pools) emits the plain greedy stream of
    the decoder's exact description.  "single" is plain autoregressive decoding through the same
    kernels (one node per step)."""
    from toy_gpu import ToyDecoderGpu
    w, prompt, stream = bf16_toy
    n_new = len(stream)
    drafter = {
        "random": W.random_drafter(1, w.vocab),
        "replay": W.replay_drafter(1, w.vocab, len(prompt), stream),
        "corrupting": W.replay_drafter(1, w.vocab, len(prompt), stream, wrong_after=(0, 4)),
    }[kind]
    tree = {"tree60": lambda s: W.seeded_tree(s), "chain4": lambda s: W.chain_tree(4),
            "single": lambda s: W.chain_tree(1)}[topology]
    table = np.random.default_rng(3).permutation(16)
    gpu = ToyDecoderGpu(w, n_blocks=16, dtype="bf16")
    out, lens = gpu.spec_decode(prompt, n_new, drafter, tree, table)
    assert out == stream
    if kind == "replay" and topology != "single":
        full = 6 if topology == "tree60" else 4
        assert all(l == full for l in lens[:-1])


def _bf16_all_toy():
    """As _bf16_toy, for the toy whose whole layers run on bf16 kernels: bf16-representable
    weights, and the exact description rounds at every hand-over between kernels."""
    from oracle.toy_decoder import round_bf16
    for seed in range(200):
        w = W.make_toy_weights(seed, d=256, n_layers=2, Hq=8, Hkv=2, Dh=128, ffn=512, vocab=4096, weights_bf16=True)
        ref = ToyDecoderRef(w, quant=round_bf16, quant_dense=round_bf16)
        prompt = [int(t) for t in np.random.default_rng(seed).integers(0, w.vocab, size=24)]
        stream, margin = ref.greedy_ar(prompt, 16)
        if margin >= 1.0:
            return w, prompt, stream
    raise AssertionError("no seed with a wide enough margin")


@pytest.fixture(scope="module")
def bf16_all_toy():
    return _bf16_all_toy()


@pytest.mark.parametrize("kind,topology", [("random", "tree60"), ("replay", "tree60"), ("corrupting", "chain4"),
                                           ("replay", "chain4"), ("random", "single")])
def test_greedy_losslessness_with_every_kernel_of_the_layer_in_the_loop(bf16_all_toy, kind, topology):
    """The same loop with the whole decoder on the library's kernels: RMSNorm, QKV projection +
    rotary embedding, attention, output projection with residual, RMSNorm, gated-SiLU projection,
    down projection with residual, final RMSNorm, LM head, acceptance, compaction (only the
    embedding lookup is torch's).  The emitted stream is the plain greedy stream of the decoder's
    exact description (float64 arithmetic, bf16 rounding at every hand-over between kernels)."""
    from toy_gpu import ToyDecoderGpu
    w, prompt, stream = bf16_all_toy
    n_new = len(stream)
    drafter = {
        "random": W.random_drafter(1, w.vocab),
        "replay": W.replay_drafter(1, w.vocab, len(prompt), stream),
        "corrupting": W.replay_drafter(1, w.vocab, len(prompt), stream, wrong_after=(0, 4)),
    }[kind]
    tree = {"tree60": lambda s: W.seeded_tree(s), "chain4": lambda s: W.chain_tree(4),
            "single": lambda s: W.chain_tree(1)}[topology]
    table = np.random.default_rng(3).permutation(16)
    gpu = ToyDecoderGpu(w, n_blocks=16, dtype="bf16_all")
    out, lens = gpu.spec_decode(prompt, n_new, drafter, tree, table)
    assert out == stream
    if kind == "replay":
        full = 6 if topology == "tree60" else 4
        assert all(l == full for l in lens[:-1])


@pytest.mark.parametrize("K,T,N", [(3, 4, 12), (4, 3, 20), (1, 5, 6)])
def test_greedy_losslessness_with_trees_built_on_the_device(bf16_toy, K, T, N):
    """Draft logits -> hb_topk_logprob -> hb_tree_grow per level -> hb_tree_finalize -> verification
    -> acceptance -> compaction, in a loop: whatever the draft proposes, the emitted stream is the
    plain greedy stream.  The 'draft model' is a seeded table of logits per token path that
    favours the true next token along the committed stream with a margin that shrinks with depth
    (so deeper levels branch and miss more), and anything otherwise."""
    import paper_2509_18824_amd.step as St
    from toy_gpu import ToyDecoderGpu
    w, prompt, stream = bf16_toy
    n_new = len(stream)
    full = list(prompt) + list(stream)
    V = w.vocab

    def draft_logits(paths):
        out = np.empty((len(paths), V), dtype=np.float32)
        for i, path in enumerate(paths):
            rng = np.random.default_rng([77, len(path)] + [int(t) for t in path[-6:]])
            row = rng.normal(0, 1.5, size=V).astype(np.float32)
            if len(path) < len(full) and list(path) == full[:len(path)]:
                row[full[len(path)]] += np.float32(6.0 - 1.2 * (len(path) - len(prompt)) % 5)
            out[i] = row
        return torch.from_numpy(out).cuda()

    lens_seen = []

    def tree_builder(step, toks):
        builder = St.DraftTreeBuilder(1, K, T)
        paths = [list(toks)]
        for level in range(T):
            ids, logp = St.topk_logprob(draft_logits(paths), K)
            frontier, slot = builder.grow(ids, logp)
            torch.cuda.synchronize()
            cand_tok = builder.cand_token[0].cpu().numpy()
            paths = [paths[s] + [int(cand_tok[c])] for c, s in zip(frontier[0].tolist(), slot[0].tolist())]
        out = builder.finalize(N, torch.tensor([toks[-1]], dtype=torch.int32, device="cuda"))
        torch.cuda.synchronize()
        parent = out["parent"].cpu().numpy()
        ids = out["draft_ids"].cpu().numpy()
        assert len(parent) == min(N, 1 + K + (T - 1) * K * K) and parent[0] == -1 and ids[0] == toks[-1]
        return parent, ids

    table = np.random.default_rng(5).permutation(16)
    gpu = ToyDecoderGpu(w, n_blocks=16, dtype="bf16")
    out, lens = gpu.spec_decode(prompt, n_new, None, None, table, tree_builder=tree_builder)
    assert out == stream
    assert max(lens) >= 2  # the draft was right often enough to accept something


def test_full_step_replays_from_a_hip_graph(S):
    """The four calls only enqueue kernels on the caller's stream (no allocation, no memset, no
    host synchronisation), so a step can be captured into a HIP graph.  The graph is replayed
    several times, with eager steps and synchronisations in between, on inputs that change
    between replays (the draft ids), and every replay must give what the eager step gives."""
    inp = W.make_config(4, scale_down=8)
    V = 8192
    _, weight = W.make_lmhead_inputs(45, 1, inp.Hq * inp.D, V, dtype="bf16")
    dev = S.to_device(inp)
    desc = S.desc_for(inp)
    wdev = weight.cuda()
    draft = torch.zeros(inp.total_nodes, dtype=torch.int32, device="cuda")
    stp = S.VerifyStep(desc, dev, wdev, draft, inp.max_path)
    stp.run(compact=False)
    torch.cuda.synchronize()
    target = stp.target_ids.cpu().numpy()

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        stp.run()  # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        stp.run()

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in (stp.out, stp.target_ids, stp.accept_len, stp.accept_path, stp.out_tokens,
                                    stp.bonus, stp.out_slots, stp.new_len, dev.k_pool, dev.v_pool)]

    for seed in (4, 5, 6):
        ids, planted = W.plant_draft_ids(seed, inp.trees(), target, V)
        stp.draft_ids.copy_(torch.from_numpy(ids))
        stp.run()
        eager = snapshot()
        assert list(stp.accept_len.cpu().numpy()) == [d + 1 for d in planted]
        for t in (stp.out, stp.target_ids, stp.accept_len, stp.accept_path, stp.out_tokens, stp.bonus,
                  stp.out_slots, stp.new_len):
            t.fill_(0) if t.dtype != torch.bfloat16 else t.zero_()
        graph.replay()
        replayed = snapshot()
        for a, b in zip(eager, replayed):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))


def _mlp_weights(mk, n_layers, K, F):
    return dict(norm1=[mk(K, std=0.2) + 1 for _ in range(n_layers)], norm2=[mk(K, std=0.2) + 1 for _ in range(n_layers)],
                w_gate_up=[mk(2 * F, K, std=K ** -0.5) for _ in range(n_layers)],
                w_down=[mk(K, F, std=0.3 * F ** -0.5) for _ in range(n_layers)], norm_f=mk(K, std=0.2) + 1, eps=1e-6)


@pytest.mark.parametrize("tree", ["tree", "chain8"])
def test_whole_decoder_layers_against_the_oracle(S, tree):
    """Two whole pre-norm layers (RMSNorm, QKV projection + rotary embedding, attention, output
    projection with residual, RMSNorm, gated-SiLU projection, down projection with residual) and
    the final RMSNorm, against the float64 oracle chained the same way and rounded to bf16 where
    the kernels hand a bf16 tensor on."""
    from oracle import (tree_positions_ref, qkv_rope_project_ref, tree_attn_ref, linear_ref, rmsnorm_ref, swiglu_ref)
    from oracle.toy_decoder import round_bf16
    inp = W.make_config(4, scale_down=8, tree=tree)
    n_layers, F = 2, 1024
    T, Hq, Hkv, D = inp.total_nodes, inp.Hq, inp.Hkv, inp.D
    K = Hq * D
    dev = S.to_device(inp)
    desc = S.desc_for(inp)
    g = torch.Generator(device="cuda").manual_seed(17)
    mk = lambda *shape, std: (torch.randn(shape, generator=g, device="cuda") * std).to(torch.bfloat16)
    w_qkv = [mk((Hq + 2 * Hkv) * D, K, std=K ** -0.5) for _ in range(n_layers)]
    w_o = [mk(K, K, std=0.3 * K ** -0.5) for _ in range(n_layers)]
    mlp = _mlp_weights(mk, n_layers, K, F)
    lm = mk(4096, K, std=0.02)
    hidden0 = mk(T, K, std=1.0)
    pools = [(dev.k_pool, dev.v_pool), (dev.k_pool.clone(), dev.v_pool.clone())]
    draft = torch.zeros(T, dtype=torch.int32, device="cuda")
    stack = S.VerifyLayerStack(desc, dev, pools, w_qkv, w_o, lm, draft, inp.max_path, hidden0, mlp=mlp)
    stack.run(compact=False)
    torch.cuda.synchronize()
    wd = W.widen
    pos = tree_positions_ref(inp.node_offset.numpy(), inp.parent.numpy(), inp.prefix_len.numpy())
    x = wd(hidden0.cpu())
    for l in range(n_layers):
        a = round_bf16(rmsnorm_ref(x, wd(mlp["norm1"][l].cpu()), 1e-6))
        q, k, v = (round_bf16(t) for t in qkv_rope_project_ref(a, wd(w_qkv[l].cpu()), None, pos, Hq, Hkv, D, 1e6))
        attn, _ = tree_attn_ref(q, k, v, wd(pools[l][0].cpu()), wd(pools[l][1].cpu()), inp.block_table.numpy(),
                                inp.prefix_len.numpy(), inp.node_offset.numpy(), inp.parent.numpy(), inp.softmax_scale)
        y = round_bf16(linear_ref(round_bf16(attn).reshape(T, -1), wd(w_o[l].cpu()), x))
        m = round_bf16(rmsnorm_ref(y, wd(mlp["norm2"][l].cpu()), 1e-6))
        act = round_bf16(swiglu_ref(m, wd(mlp["w_gate_up"][l].cpu())))
        x = round_bf16(linear_ref(act, wd(mlp["w_down"][l].cpu()), y))
    ref = rmsnorm_ref(x, wd(mlp["norm_f"].cpu()), 1e-6)
    got = wd(stack.final_hidden.cpu())
    rel = np.linalg.norm(got - ref) / np.linalg.norm(ref)
    assert rel <= 1e-2, rel                      # two layers of bf16 hand-overs
    assert np.abs(got - ref).max() <= 0.1 * (1 + np.abs(ref).max())


@pytest.mark.parametrize("tree,whole", [("tree", False), ("chain8", False), ("tree", True), ("chain8", True)])
def test_layer_stack_replays_from_a_hip_graph(S, tree, whole):
    """Three decoder layers (QKV projection + rotary embedding, attention over each layer's own
    pools, output projection; with 8-node chains the projections take the split-K path; with
    ``whole`` also the normalisations and the feed-forward block), LM head,
    acceptance and the compaction of all layers in one launch, captured once and replayed with
    eager steps in between on changing draft ids: every replay equals the eager step, bit for bit,
    pools of every layer included."""
    inp = W.make_config(4, scale_down=8, tree=tree)
    V, n_layers = 4096, 3
    T, Hq, Hkv, D = inp.total_nodes, inp.Hq, inp.Hkv, inp.D
    K = Hq * D
    dev = S.to_device(inp)
    desc = S.desc_for(inp)
    g = torch.Generator(device="cuda").manual_seed(11)
    mk = lambda *shape, std: (torch.randn(shape, generator=g, device="cuda") * std).to(torch.bfloat16)
    w_qkv = [mk((Hq + 2 * Hkv) * D, K, std=K ** -0.5) for _ in range(n_layers)]
    w_o = [mk(K, K, std=0.3 * K ** -0.5) for _ in range(n_layers)]
    lm = mk(V, K, std=0.02)
    hidden0 = mk(T, K, std=1.0)
    pools = [(dev.k_pool, dev.v_pool)] + [(dev.k_pool.clone(), dev.v_pool.clone()) for _ in range(n_layers - 1)]
    pristine = [(k.clone(), v.clone()) for k, v in pools]
    draft = torch.zeros(T, dtype=torch.int32, device="cuda")
    mlp = _mlp_weights(mk, n_layers, K, 1536) if whole else None
    stack = S.VerifyLayerStack(desc, dev, pools, w_qkv, w_o, lm, draft, inp.max_path, hidden0, mlp=mlp)
    assert stack.ws_proj is not None or T > 512
    stack.run(compact=False)
    torch.cuda.synchronize()
    target = stack.target_ids.cpu().numpy()

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        stack.run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        stack.run()

    def restore():
        for (k, v), (k0, v0) in zip(pools, pristine):
            k.copy_(k0); v.copy_(v0)

    def snapshot():
        torch.cuda.synchronize()
        outs = [stack.final_hidden, stack.target_ids, stack.accept_len, stack.accept_path, stack.out_tokens,
                stack.bonus, stack.out_slots, stack.new_len]
        return [t.clone() for t in outs] + [t.clone() for kv in pools for t in kv]

    for seed in (4, 5, 6):
        ids, planted = W.plant_draft_ids(seed, inp.trees(), target, V)
        stack.draft_ids.copy_(torch.from_numpy(ids))
        restore()
        stack.run()
        eager = snapshot()
        assert list(stack.accept_len.cpu().numpy()) == [d + 1 for d in planted]
        # the compaction wrote the accepted nodes into every layer's pools
        assert all(not torch.equal(k.view(torch.int16), k0.view(torch.int16)) for (k, _), (k0, _) in zip(pools, pristine))
        restore()
        for t in (stack.target_ids, stack.accept_len, stack.accept_path, stack.out_tokens, stack.bonus,
                  stack.out_slots, stack.new_len):
            t.fill_(0)
        graph.replay()
        replayed = snapshot()
        for a, b in zip(eager, replayed):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))
