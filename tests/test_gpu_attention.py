"""GPU parity: hb_tree_verify_attn against the CPU oracle, element by element on sizes the
oracle finishes in seconds, and on sampled nodes at the full workload sizes."""
import numpy as np
import pytest
import torch

import workloads as W
from parity import check_attn, oracle_attn

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hb():
    import paper_2509_18824_amd as m
    return m


@pytest.fixture(scope="module")
def step():
    import paper_2509_18824_amd.step as s
    return s


def _run(step, inp, **kw):
    dev = step.to_device(inp)
    desc = step.desc_for(inp, **kw)
    out, lse = step.tree_verify_attn(desc, dev)
    torch.cuda.synchronize()
    return out, lse, desc


def _algos(hb, inp):
    """Every kernel the library offers for this shape (a descriptor it cannot take plans 0 splits)."""
    import paper_2509_18824_amd.step as s
    algos = [hb.HB_ATTN_SCALAR]
    if hb.hb_tree_verify_attn_num_splits(s.desc_for(inp, algo=hb.HB_ATTN_MFMA)) > 0:
        algos.append(hb.HB_ATTN_MFMA)
    return algos


def test_matrix_core_kernel_takes_the_bf16_workloads(hb, step):
    """The workloads with bf16 KV, head_dim 128 and page 16 must run on the MFMA kernel, both when
    asked for explicitly and by default (so the parity tests below really cover it)."""
    for cfg in (1, 2, 3, 4):
        inp = W.make_config(cfg, scale_down=32)
        assert hb.HB_ATTN_MFMA in _algos(hb, inp)
    assert hb.HB_ATTN_MFMA not in _algos(hb, W.make_config(0))


def test_config0_fp32_chain(hb, step):
    for peaked in (False, True):
        inp = W.make_config(0, peaked=peaked)
        ref = oracle_attn(inp)
        for splits in (1, 2, 0):
            out, lse, _ = _run(step, inp, num_splits=splits)
            check_attn(inp, out, lse, ref=ref, label=f"cfg0 peaked={peaked} splits={splits}")


@pytest.mark.parametrize("peaked", [False, True])
def test_config1_single_sequence_bf16(hb, step, peaked):
    inp = W.make_config(1, peaked=peaked)
    ref = oracle_attn(inp)
    for algo in _algos(hb, inp):
        for splits in (1, 2, 7, 0):
            out, lse, _ = _run(step, inp, num_splits=splits, algo=algo)
            check_attn(inp, out, lse, ref=ref, label=f"cfg1 algo={algo} splits={splits} peaked={peaked}")


@pytest.mark.parametrize("cfg,scale_down", [(2, 8), (3, 16), (4, 8)])
@pytest.mark.parametrize("peaked", [False, True])
def test_scaled_copies_of_the_batched_workloads(hb, step, cfg, scale_down, peaked):
    """Same structure as the big workloads (ragged lengths, permuted pages, 60-node trees), with
    prefixes short enough for the oracle to cover every node."""
    inp = W.make_config(cfg, peaked=peaked, scale_down=scale_down)
    ref = oracle_attn(inp)
    for algo in _algos(hb, inp):
        for splits in (1, 3, 0):
            out, lse, _ = _run(step, inp, num_splits=splits, algo=algo)
            check_attn(inp, out, lse, ref=ref, label=f"cfg{cfg}/{scale_down} algo={algo} splits={splits}")


def test_ragged_edges_and_odd_shapes(hb, step):
    """Empty prefix, prefix shorter than a page, lengths around page and tile boundaries,
    single-node trees, a 64-node tree, group sizes 1 and 8, head dims 64 and 128."""
    trees = [W.chain_tree(1), W.chain_tree(8), W.seeded_tree(1), W.seeded_tree(2, n_nodes=64),
             W.seeded_tree(3, n_nodes=17, levels=4, root_fanout=4), W.chain_tree(3), W.seeded_tree(4)]
    lens = [0, 5, 16, 63, 64, 65, 1000]
    # (8, 8), (8, 4) and (28, 4) / (8, 1) give 64, 128 and 448 / 512 query rows per kv head: the
    # three workgroup shapes of the matrix-core kernel
    for dtype, Hq, Hkv, D in [("bf16", 28, 4, 128), ("bf16", 8, 8, 128), ("bf16", 8, 4, 128), ("bf16", 8, 1, 128),
                              ("f32", 6, 2, 64), ("bf16", 4, 2, 64), ("f32", 4, 4, 128)]:
        inp = W.make_verify_inputs(77, dtype, Hq, Hkv, D, lens, trees, kv_std=1.0, q_std=1.0)
        ref = oracle_attn(inp)
        for algo in _algos(hb, inp):
            for splits in (1, 4, 0):
                out, lse, _ = _run(step, inp, num_splits=splits, algo=algo)
                check_attn(inp, out, lse, ref=ref, label=f"edges {dtype} Hq={Hq} Hkv={Hkv} D={D} algo={algo} s={splits}")


def test_schedules_of_the_matrix_core_kernel(hb, step):
    """With num_splits = 0 the kernel cuts the KV itself, on the device, from the prefix lengths:
    work-proportionally when that finishes first (one long sequence among short ones: pieces of
    several sequences per workgroup, rows written directly next to rows that go through the
    merge), with equal pieces per sequence otherwise (equal lengths), and with host-planned
    chunks for more than 64 sequences."""
    cases = {
        "one long, many short": ([3000, 0, 70, 1, 130, 64, 17, 300], 8),
        "equal lengths": ([1536] * 4, 4),
        "more than 64 sequences": ([33 + 7 * i for i in range(66)], 66),
    }
    for name, (lens, B) in cases.items():
        trees = [W.seeded_tree(10 + i, n_nodes=15 + (i * 11) % 46) for i in range(B)]
        inp = W.make_verify_inputs(91, "bf16", 28, 4, 128, lens, trees, kv_std=1.0, q_std=1.0)
        ref = oracle_attn(inp)
        out, lse, desc = _run(step, inp, num_splits=0, algo=hb.HB_ATTN_MFMA, hint=max(lens))
        check_attn(inp, out, lse, ref=ref, label=f"schedule: {name}")
        out2, lse2, _ = _run(step, inp, num_splits=0, algo=hb.HB_ATTN_MFMA)  # no length hint
        check_attn(inp, out2, lse2, ref=ref, label=f"schedule, no hint: {name}")


def test_poisoned_tree_nodes_off_the_path_do_not_leak(hb, step):
    """Inputs already carry NaN in every slot past the prefix and in unmapped pages.  Here the
    tree K/V of one branch is additionally set to Inf/NaN: nodes outside that branch must be
    bitwise unchanged."""
    inp = W.make_config(1)
    par = inp.trees()[0]
    bad = 1  # first child of the root; poison it and all its descendants
    sub = [i for i in range(len(par)) if bad in _path(par, i)]
    clean = [i for i in range(len(par)) if i not in sub]
    for algo in _algos(hb, inp):
        base, lse0, _ = _run(step, inp, algo=algo)
        dirty = W.make_config(1)
        dirty.k_tree[sub] = float("inf")
        dirty.v_tree[sub] = float("nan")
        got, lse1, _ = _run(step, dirty, algo=algo)
        assert torch.equal(base[clean].view(torch.int16), got[clean].view(torch.int16))
        assert torch.equal(lse0[clean], lse1[clean])


def _path(par, i):
    out = []
    while i >= 0:
        out.append(i); i = int(par[i])
    return out


def test_results_are_deterministic(hb, step):
    inp = W.make_config(2, scale_down=8)
    for algo in _algos(hb, inp):
        a, la, _ = _run(step, inp, algo=algo)
        b, lb, _ = _run(step, inp, algo=algo)
        assert torch.equal(a.view(torch.int16), b.view(torch.int16)) and torch.equal(la, lb)


@pytest.mark.parametrize("cfg", [2, 3, 4])
def test_full_size_workloads_on_sampled_nodes(hb, step, cfg):
    """Full sizes, default launch configuration (the one the benchmark times); the oracle
    recomputes a seeded sample of nodes from every sequence."""
    inp = W.make_config(cfg)
    rng = np.random.default_rng(cfg)
    off = inp.node_offset.numpy()
    per_seq = 2 if cfg != 3 else 6
    nodes = sorted(int(off[b] + i) for b in range(inp.B)
                   for i in rng.choice(off[b + 1] - off[b], size=per_seq, replace=False))
    ref = oracle_attn(inp, nodes=nodes)
    hint = int(inp.prefix_len.max())
    for kw in (dict(), dict(hint=hint)):
        out, lse, desc = _run(step, inp, **kw)
        check_attn(inp, out, lse, nodes=nodes, ref=ref, label=f"cfg{cfg} full {kw}")
        assert torch.isfinite(out.float()).all()
    if cfg == 3 and hb.HB_ATTN_MFMA in _algos(hb, inp):
        # only 8 (sequence, kv head) pairs: the KV-sharing kernel must split the long context
        assert hb.hb_tree_verify_attn_num_splits(desc) > 1


def test_device_side_cut_on_random_batches(hb, step):
    """Seeded random batches (1..20 sequences, prefix lengths 0..2500 with a bias to short ones,
    trees of 15..60 nodes) through the matrix-core kernel with the library's own KV cut."""
    rng = np.random.default_rng(2024)
    for case in range(6):
        B = int(rng.integers(1, 21))
        lens = [int(x) for x in np.minimum(rng.geometric(1.0 / 400.0, size=B) - 1, 2500)]
        if case == 0:
            lens[0] = 2500
        trees = [W.seeded_tree(1000 * case + i, n_nodes=int(rng.integers(15, 61))) for i in range(B)]
        inp = W.make_verify_inputs(500 + case, "bf16", 8, 2, 128, lens, trees, kv_std=1.0, q_std=1.0)
        ref = oracle_attn(inp)
        out, lse, _ = _run(step, inp, num_splits=0, algo=hb.HB_ATTN_MFMA, hint=max(max(lens), 1))
        check_attn(inp, out, lse, ref=ref, label=f"random batch {case}: B={B} lens={lens}")
