"""GPU parity: hb_tree_verify_attn against the CPU oracle, element by element on sizes the
oracle finishes in seconds, and on every node at the full workload sizes."""
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


@pytest.mark.parametrize("cfg,tree", [(2, "tree"), (3, "tree"), (4, "tree"), (4, "chain8")])
def test_full_size_workloads_every_node(hb, step, cfg, tree):
    """Full sizes, default launch configuration (the one the benchmark times), with and without
    the length hint the benchmark passes; the oracle recomputes every node of every sequence.
    The 8-node-chain run of the full-step workload takes the four-wavefront kernel with the
    device-side KV cut over 16 ragged prefixes."""
    inp = W.make_config(cfg, tree=tree)
    ref = oracle_attn(inp)
    hint = int(inp.prefix_len.max())
    for kw in (dict(), dict(hint=hint)):
        out, lse, desc = _run(step, inp, **kw)
        check_attn(inp, out, lse, ref=ref, label=f"cfg{cfg} {tree} full {kw}")
        assert torch.isfinite(out.float()).all()
        # per-row check as well: a wrong row must not hide in the batch-wide norms
        got, want = W.widen(out), ref[0]
        rel_rows = np.linalg.norm(got - want, axis=2) / np.linalg.norm(want, axis=2)
        assert rel_rows.max() <= 3e-2, f"cfg{cfg} {tree}: worst row rel err {rel_rows.max():.3e}"
    if cfg == 3 and hb.HB_ATTN_MFMA in _algos(hb, inp):
        # only 8 (sequence, kv head) pairs: the KV-sharing kernel must split the long context
        assert hb.hb_tree_verify_attn_num_splits(desc) > 1


def _planted_scores(inp, log2_scores):
    """Overwrite sequence 0 so that the prefix key at position p scores log2_scores[p] (in log2
    units, i.e. score * log2(e)) against a query that is c_r * e_0, c_r = 1 for row 0 and
    slightly different for other rows; all other key components are 0, V stays random."""
    L = len(log2_scores)
    assert int(inp.prefix_len[0]) == L
    ln2 = float(np.log(2.0))
    q = torch.zeros_like(inp.q, dtype=torch.float32)
    T, Hq, _ = inp.q.shape
    # row-dependent gain: rows cross the rescale threshold at different blocks
    gain = 1.0 + 0.03125 * (torch.arange(T * Hq).reshape(T, Hq) % 5).float()
    q[:, :, 0] = gain / inp.softmax_scale
    inp.q.copy_(q.to(inp.q.dtype))
    kt = torch.zeros_like(inp.k_tree, dtype=torch.float32)
    kt[:, :, 0] = float(log2_scores[-1]) * ln2  # tree keys score like the last prefix key
    inp.k_tree.copy_(kt.to(inp.k_tree.dtype))
    for p in range(L):
        blk = int(inp.block_table[0, p // inp.page])
        row = torch.zeros(inp.D)
        row[0] = float(log2_scores[p]) * ln2
        inp.k_pool[blk, :, p % inp.page] = row.to(inp.k_pool.dtype)
    return inp


@pytest.mark.parametrize("shape", ["tree60_gqa7", "chain8_gqa7", "tree20_gqa1"])
def test_reference_exponent_of_the_online_softmax_under_climbing_scores(hb, step, shape):
    """The matrix-core kernel keeps a per-row reference exponent that moves only when a score
    outgrows it by a fixed slack (2^8).  Scores that climb by just under / just over that slack
    from one 32-key block to the next, by fractions of it, that ramp from 60 below to 60 above,
    that jump up once at the very end, and that fall all the way: each must still give the
    oracle's output and log-sum-exp."""
    Hq, Hkv, tree = {"tree60_gqa7": (28, 4, W.seeded_tree(5)), "chain8_gqa7": (28, 4, W.chain_tree(8)),
                     "tree20_gqa1": (2, 2, W.seeded_tree(6, n_nodes=20))}[shape]
    nblk = 40
    L = 32 * nblk
    blk = np.arange(L) // 32
    jitter = np.random.default_rng(0).uniform(-0.5, 0.0, size=L)
    patterns = {
        "step 7.9": 7.9 * blk, "step 8.1": 8.1 * blk, "step 3.9": 3.9 * blk, "step 16.3": 16.3 * blk,
        "ramp -60..60": np.linspace(-60.0, 60.0, L) / np.log(2.0),
        "late jump": np.where(np.arange(L) == L - 3, 90.0, 0.0) + jitter,
        "falling": -7.9 * blk + jitter,
        "sawtooth": 7.9 * (blk % 3) + 8.1 * (blk // 3) + jitter,
    }
    for name, sc in patterns.items():
        inp = W.make_verify_inputs(321, "bf16", Hq, Hkv, 128, [L], [tree], kv_std=1.0, q_std=1.0)
        inp = _planted_scores(inp, sc)
        ref = oracle_attn(inp)
        for splits in (1, 0, 3):
            out, lse, _ = _run(step, inp, num_splits=splits, algo=hb.HB_ATTN_MFMA)
            check_attn(inp, out, lse, ref=ref, label=f"{shape} {name} splits={splits}")


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
