#!/usr/bin/env python3
"""Benchmark of the full verification step on one MI355X.

A step = tree-verify attention (one layer) + LM head with fused argmax + greedy acceptance +
KV compaction over the batch-16 full-step workload (ragged prefixes in [1024, 4096], one 60-node
tree per sequence, hidden 3584 x vocab 152064, bf16).  All inputs are synthetic, seeded, and
resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--tree tree|chain8] [--no-attn-extra]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

FFN_WIDTH = 18944  # feed-forward width of the decoder28 blocks
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E, published
PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, published

# HBM traffic of one LM-head launch on this workload, from hardware counters (FETCH_SIZE and
# WRITE_SIZE, each scaled by what the same counter reads for a 1 GiB device copy in the same
# run: `--copy-probe`).  Valid only for the kernel source it was measured on: keyed by the
# first 16 hex digits of the SHA-256 over csrc/lmhead_mfma.hip followed by
# csrc/mfma_gemm_tile.inc (the tile loop the kernel includes); anything else reports null.
# "tree": the 960-row launch of the headline step; "chain8": the 128-row launch of the chain run.
LMHEAD_TRAFFIC = {
    "5590a872aae69250": {
        "tree": {"fetch_bytes": 1.8424e9, "write_bytes": 1.9e5, "bytes": 1.8426e9,
                 "algorithmic_bytes": 152064 * 3584 * 2 + 960 * 3584 * 2},
        "chain8": {"fetch_bytes": 1.1139e9, "write_bytes": 3.5e4, "bytes": 1.1140e9,
                   "algorithmic_bytes": 152064 * 3584 * 2 + 128 * 3584 * 2},
    },
}


def _lmhead_traffic(which="tree"):
    import hashlib
    h = hashlib.sha256()
    try:
        for name in ("lmhead_mfma.hip", "mfma_gemm_tile.inc"):
            h.update(open(os.path.join(ROOT, "paper_2509_18824_amd", "csrc", name), "rb").read())
    except OSError:
        return None
    return (LMHEAD_TRAFFIC.get(h.hexdigest()[:16]) or {}).get(which)


def _events(n):
    import torch
    return [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]


def _mean_ms(pairs):
    return sum(a.elapsed_time(b) for a, b in pairs) / max(len(pairs), 1)


def cpu_baseline(inp, weight, draft_ids, sample_per_seq=60, passes=3):
    """The CPU oracle, as it stands, on a bounded sample of the same workload: `sample_per_seq`
    nodes of every sequence (all 60 by default) go through attention and the LM head (weight
    widened to float64 every pass, as the oracle does), then acceptance and compaction run on
    the whole batch; `passes` such passes (about 10-20 s of CPU work in all)."""
    import numpy as np
    import workloads as W
    from oracle import tree_attn_ref, lmhead_argmax_ref, tree_accept_ref, kv_compact_ref

    rng = np.random.default_rng(0)
    off = inp.node_offset.numpy()
    nodes = sorted(int(off[b] + i) for b in range(inp.B)
                   for i in rng.choice(off[b + 1] - off[b], size=min(sample_per_seq, off[b + 1] - off[b]),
                                       replace=False))
    bits = lambda t: t.view(__import__("torch").int16).numpy()
    t_attn = t_lm = t_rest = 0.0
    for _ in range(passes):
        t0 = time.perf_counter()
        out, _ = tree_attn_ref(W.widen(inp.q), W.widen(inp.k_tree), W.widen(inp.v_tree), W.widen(inp.k_pool),
                               W.widen(inp.v_pool), inp.block_table.numpy(), inp.prefix_len.numpy(),
                               inp.node_offset.numpy(), inp.parent.numpy(), inp.softmax_scale, nodes=nodes)
        t1 = time.perf_counter()
        hidden = out.reshape(len(nodes), -1)
        ids, _ = lmhead_argmax_ref(hidden, W.widen(weight))
        t2 = time.perf_counter()
        target = np.zeros(inp.total_nodes, dtype=np.int64)
        target[nodes] = ids
        alen, apath, _, _ = tree_accept_ref(off, inp.parent.numpy(), draft_ids, target, inp.max_path)
        kv_compact_ref(bits(inp.k_tree), bits(inp.v_tree), bits(inp.k_pool), bits(inp.v_pool),
                       inp.block_table.numpy(), inp.prefix_len.numpy(), off, alen, apath)
        t3 = time.perf_counter()
        t_attn += t1 - t0
        t_lm += t2 - t1
        t_rest += t3 - t2
    cores = len(os.sched_getaffinity(0))
    for var in ("OMP_NUM_THREADS", "OPENBLAS_NUM_THREADS", "MKL_NUM_THREADS"):
        if os.environ.get(var, "").isdigit():
            cores = min(cores, int(os.environ[var]))
    total = t_attn + t_lm + t_rest
    return {
        "value": passes * len(nodes) / total, "unit": "tokens/s", "cores": cores, "kind": "oracle",
        "sample": f"{passes} passes over {len(nodes)} of {inp.total_nodes} tree nodes ({sample_per_seq} per "
                  f"sequence): attention ({t_attn:.1f} s), LM head over the full vocabulary ({t_lm:.1f} s, "
                  f"includes widening the weight to float64), acceptance and compaction on the whole "
                  f"batch ({t_rest:.2f} s); float64 numpy",
        "seconds": total,
    }


def bench_attention_only(cfg, steps, warmup, n_pools=4):
    """Attention kernel alone on workload `cfg`, rotating over `n_pools` distinct copies of the KV
    pools so that consecutive launches do not find their KV in the 256 MB last-level cache."""
    import torch
    import workloads as W
    import paper_2509_18824_amd as hb
    import paper_2509_18824_amd.step as S

    inp = W.make_config(cfg)
    dev = S.to_device(inp)
    hint = int(inp.prefix_len.max())
    desc = S.desc_for(inp, hint=hint)
    pools = [(dev.k_pool, dev.v_pool)] + [(dev.k_pool.clone(), dev.v_pool.clone()) for _ in range(n_pools - 1)]
    out = torch.empty_like(dev.q)
    ws = S.alloc_workspace(hb.hb_tree_verify_attn_workspace_bytes(desc))

    def launch(i):
        kp, vp = pools[i % n_pools]
        hb.hb_tree_verify_attn(desc, dev.q, dev.k_tree, dev.v_tree, kp, vp, dev.block_table, dev.prefix_len,
                               dev.node_offset, dev.parent, out, None, ws)

    for i in range(warmup):
        launch(i)
    torch.cuda.synchronize()
    ev = _events(steps)
    for i, (a, b) in enumerate(ev):
        a.record()
        launch(i)
        b.record()
    torch.cuda.synchronize()
    ms = _mean_ms(ev)
    kv_bytes = inp.kv_bytes()
    rows = inp.total_nodes * inp.Hq
    flops = 4.0 * inp.D * inp.Hq * sum(
        int(n) * (int(L) + 0) for n, L in zip((inp.node_offset[1:] - inp.node_offset[:-1]).tolist(),
                                              inp.prefix_len.tolist()))
    # vector-ALU estimate: per score about 6.5 lane operations (scale, exp2 at quarter rate counted
    # as 4, max, half a convert) against 256 CUs x 64 lanes x 2.4 GHz
    scores_per_s = flops / (4.0 * inp.D) / (ms * 1e-3)
    valu_frac = scores_per_s * 6.5 / (256 * 64 * 2.4e9)
    fracs = {"hbm": kv_bytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
             "mfma": flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, "valu": valu_frac}
    return {
        "valu_frac_estimate": valu_frac, "nearest_bound": max(fracs, key=fracs.get),
        "workload": inp.name, "ms": ms, "tree_tokens_per_s": inp.total_nodes / (ms * 1e-3),
        "kv_bytes": kv_bytes, "kv_GBps": kv_bytes / (ms * 1e-3) / 1e9,
        "kv_frac_of_hbm_peak": kv_bytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
        "attn_TFLOPs": flops / (ms * 1e-3) / 1e12,
        "attn_frac_of_bf16_mfma_peak": flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "splits": hb.hb_tree_verify_attn_num_splits(desc), "rows": rows,
    }


def run_full_step(tree, steps, warmup, weight, V, K):
    """Times `steps` full verification steps (attention of one layer, LM head with fused argmax,
    acceptance, compaction) on the full-step workload with `tree` = "tree" (60-node trees) or
    "chain8" (8-node chains).  Returns the measurements and what the parity check needs."""
    import torch
    import workloads as W
    import paper_2509_18824_amd as hb
    import paper_2509_18824_amd.step as S

    inp = W.make_config(4, tree=tree)
    dev = S.to_device(inp)
    wdev = weight if weight.is_cuda else weight.cuda()
    hint = int(inp.prefix_len.max())
    desc = S.desc_for(inp, hint=hint)
    draft = torch.zeros(inp.total_nodes, dtype=torch.int32, device="cuda")
    step = S.VerifyStep(desc, dev, wdev, draft, inp.max_path)

    # pass 1: target ids; the host then plants draft ids along a seeded path per sequence
    step.run(compact=False)
    torch.cuda.synchronize()
    target = step.target_ids.cpu().numpy()
    draft_np, planted = W.plant_draft_ids(4, inp.trees(), target, V)
    step.draft_ids.copy_(torch.from_numpy(draft_np))
    k_pool0, v_pool0 = dev.k_pool.clone(), dev.v_pool.clone()  # the cache before any compaction

    for _ in range(warmup):
        step.run()
    torch.cuda.synchronize()
    dv = step.dev

    def one_step(i, ev_attn=None, ev_lm=None, ev_acc=None, ev_cmp=None):
        if ev_attn: ev_attn[i][0].record()
        hb.hb_tree_verify_attn(desc, dv.q, dv.k_tree, dv.v_tree, dv.k_pool, dv.v_pool, dv.block_table,
                               dv.prefix_len, dv.node_offset, dv.parent, step.out, None, step.ws_attn)
        if ev_attn: ev_attn[i][1].record()
        if ev_lm: ev_lm[i][0].record()
        hb.hb_lmhead_argmax(step.out.view(inp.total_nodes, -1), wdev, step.target_ids, None, step.ws_lm)
        if ev_lm: ev_lm[i][1].record()
        if ev_acc: ev_acc[i][0].record()
        hb.hb_tree_accept(desc.batch, desc.max_nodes_per_tree, dv.node_offset, dv.parent, step.draft_ids,
                          step.target_ids, step.max_path, step.accept_len, step.accept_path, step.out_tokens,
                          step.bonus)
        if ev_acc: ev_acc[i][1].record()
        if ev_cmp: ev_cmp[i][0].record()
        hb.hb_kv_compact(desc, dv.k_tree, dv.v_tree, dv.k_pool, dv.v_pool, dv.block_table, dv.prefix_len,
                         dv.node_offset, step.accept_len, step.accept_path, step.max_path, step.out_slots,
                         step.new_len)
        if ev_cmp: ev_cmp[i][1].record()

    # Timed region: exactly `steps` full steps.  Inside it HIP events (on the launch stream)
    # bracket the LM-head call only, the dominant kernel whose duration the roofline needs: an
    # event pair costs the stream about 5 us, and eight of them per step would take 4 % off the
    # figure they are there to explain.
    ev_lm = _events(steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        one_step(i, ev_lm=ev_lm)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_step = (t1 - t0) * 1e3 / steps
    ms_lm = _mean_ms(ev_lm)
    # The other calls' durations come from a second pass of the same steps, outside the timed
    # region, with events around every call.
    ev_attn, ev_lm2, ev_acc, ev_cmp = (_events(steps) for _ in range(4))
    for i in range(steps):
        one_step(i, ev_attn, ev_lm2, ev_acc, ev_cmp)
    torch.cuda.synchronize()
    ms_attn, ms_acc, ms_cmp = map(_mean_ms, (ev_attn, ev_acc, ev_cmp))
    accept_len = step.accept_len.cpu().numpy()
    assert list(accept_len) == [d + 1 for d in planted], "accepted lengths differ from the planted paths"
    return dict(inp=inp, desc=desc, step=step, dev=dv, wdev=wdev, draft_np=draft_np, planted=planted,
                ms_step=ms_step, ms_lm=ms_lm, ms_attn=ms_attn, ms_acc=ms_acc, ms_cmp=ms_cmp,
                accept_len=accept_len, k_pool0=k_pool0, v_pool0=v_pool0)


def parity_check(run, weight):
    """GPU outputs of the last timed step against the CPU oracle on the same inputs, every node
    (outside the timed region): attention output of all tree nodes; LM-head ids of all rows by
    the margin rule (the oracle's logits are computed from the GPU's own bf16 hidden states, so
    that the comparison isolates the LM head); acceptance and compaction bit for bit."""
    import numpy as np
    import torch
    import workloads as W
    from oracle import tree_attn_ref, lmhead_logits_ref, tree_accept_ref, kv_compact_ref

    inp, step = run["inp"], run["step"]
    ref, _ = tree_attn_ref(W.widen(inp.q), W.widen(inp.k_tree), W.widen(inp.v_tree), W.widen(run["k_pool0"]),
                           W.widen(run["v_pool0"]), inp.block_table.numpy(), inp.prefix_len.numpy(),
                           inp.node_offset.numpy(), inp.parent.numpy(), inp.softmax_scale)
    got = W.widen(step.out)
    attn_abs = float(np.abs(got - ref).max())
    attn_rel = float(np.linalg.norm(got - ref) / np.linalg.norm(ref))
    hidden = got.reshape(inp.total_nodes, -1)
    w = W.widen(weight)
    w_rms = float(np.sqrt((w * w).sum(1).mean()))
    ids = step.target_ids.cpu().numpy()
    mism_clear = n_clear = mism_any = 0
    for r0 in range(0, hidden.shape[0], 192):
        h = hidden[r0:r0 + 192]
        logits = lmhead_logits_ref(h, w)
        r = np.arange(h.shape[0])
        top1 = np.argmax(logits, axis=1)
        best = logits[r, top1]
        logits[r, top1] = -np.inf
        top2 = np.argmax(logits, axis=1)
        margin = best - logits[r, top2]
        clear = margin > 1e-4 * np.linalg.norm(h, axis=1) * w_rms
        g = ids[r0:r0 + 192]
        mism_clear += int((g[clear] != top1[clear]).sum())
        mism_any += int(((g != top1) & (g != top2)).sum())
        n_clear += int(clear.sum())
    off = inp.node_offset.numpy()
    alen, apath, otoks, bonus = tree_accept_ref(off, inp.parent.numpy(), run["draft_np"], ids, inp.max_path)
    accept_exact = bool(np.array_equal(step.accept_len.cpu().numpy(), alen)
                        and np.array_equal(step.accept_path.cpu().numpy(), apath)
                        and np.array_equal(step.out_tokens.cpu().numpy(), otoks)
                        and np.array_equal(step.bonus.cpu().numpy(), bonus))
    bits = lambda t: t.detach().cpu().view(torch.int16).numpy()
    rk, rv, rslots, rlen = kv_compact_ref(bits(inp.k_tree), bits(inp.v_tree), bits(run["k_pool0"]), bits(run["v_pool0"]),
                                          inp.block_table.numpy(), inp.prefix_len.numpy(), off, alen, apath)
    compact_exact = bool(np.array_equal(bits(run["dev"].k_pool), rk) and np.array_equal(bits(run["dev"].v_pool), rv)
                         and np.array_equal(step.out_slots.cpu().numpy(), rslots)
                         and np.array_equal(step.new_len.cpu().numpy(), rlen))
    return {"nodes": int(inp.total_nodes), "attn_max_abs": attn_abs, "attn_rel_l2": attn_rel,
            "attn_tolerance": {"max_abs": 2e-2, "rel_l2": 1e-2},
            "argmax_rows_clear": n_clear, "argmax_mismatch_clear": mism_clear,
            "argmax_outside_top2": mism_any, "accept_exact": accept_exact, "compact_exact": compact_exact,
            "ok": bool(attn_abs <= 2e-2 and attn_rel <= 1e-2 and mism_clear == 0 and mism_any == 0
                       and accept_exact and compact_exact)}


def achievable_peaks():
    """What this machine delivers on plain library kernels, measured in this run: a 1 GiB device copy
    and a 1 GiB read (HBM), and bf16 GEMMs by the vendor library through torch.matmul (a square
    one and one of the LM head's shape, logits written out)."""
    import torch
    out = {}
    src = torch.ones(1 << 29, dtype=torch.bfloat16, device="cuda")  # 1 GiB
    dst = torch.empty_like(src)

    def timed(fn, n=5):
        fn(); torch.cuda.synchronize()
        ev = _events(n)
        for a, b in ev:
            a.record(); fn(); b.record()
        torch.cuda.synchronize()
        return min(a.elapsed_time(b) for a, b in ev)
    ms = timed(lambda: dst.copy_(src))
    out["hbm_copy_GBps"] = 2 * src.numel() * 2 / (ms * 1e-3) / 1e9  # bytes read + bytes written
    ms = timed(lambda: torch.max(src.view(torch.int16)))
    out["hbm_read_GBps"] = src.numel() * 2 / (ms * 1e-3) / 1e9
    del src, dst
    a = torch.randn(8192, 8192, device="cuda", dtype=torch.bfloat16)
    b = torch.randn(8192, 8192, device="cuda", dtype=torch.bfloat16)
    ms = timed(lambda: torch.matmul(a, b))
    out["bf16_gemm_8192_TFLOPs"] = 2 * 8192.0 ** 3 / (ms * 1e-3) / 1e12
    del a, b
    h = torch.randn(960, 3584, device="cuda", dtype=torch.bfloat16)
    w = (torch.randn(152064, 3584, device="cuda", dtype=torch.float32) * 0.02).to(torch.bfloat16)
    ms = timed(lambda: torch.matmul(h, w.t()))
    out["bf16_gemm_lmhead_shape_TFLOPs"] = 2.0 * 960 * 3584 * 152064 / (ms * 1e-3) / 1e12
    out["bf16_gemm_lmhead_shape_ms"] = ms
    del h, w
    torch.cuda.empty_cache()
    # the library's fused attention on the dense problem of the long-context workload's shape (per
    # (sequence, kv head): 420 query rows against 32768 keys, head size 128, bf16, no mask, contiguous
    # K/V): what a tuned library kernel reaches on this few-rows-many-keys shape, without paging,
    # tree mask or split-K merge
    try:
        q = torch.randn(8, 1, 420, 128, device="cuda", dtype=torch.bfloat16)
        kk = torch.randn(8, 1, 32768, 128, device="cuda", dtype=torch.bfloat16)
        vv = torch.randn(8, 1, 32768, 128, device="cuda", dtype=torch.bfloat16)
        ms = timed(lambda: torch.nn.functional.scaled_dot_product_attention(q, kk, vv))
        out["sdpa_long_context_shape_ms"] = ms
        out["sdpa_long_context_shape_TFLOPs"] = 4.0 * 8 * 420 * 32768 * 128 / (ms * 1e-3) / 1e12
        del q, kk, vv
        # the same flops with the keys cut into 32 chunks handed over as batch entries (the
        # parallelism a split-K plan gives, without the merge): the library kernel's own rate on
        # 420-row query tiles
        q = torch.randn(256, 1, 420, 128, device="cuda", dtype=torch.bfloat16)
        kk = torch.randn(256, 1, 1024, 128, device="cuda", dtype=torch.bfloat16)
        vv = torch.randn(256, 1, 1024, 128, device="cuda", dtype=torch.bfloat16)
        ms = timed(lambda: torch.nn.functional.scaled_dot_product_attention(q, kk, vv))
        out["sdpa_presplit_ms"] = ms
        out["sdpa_presplit_TFLOPs"] = 4.0 * 256 * 420 * 1024 * 128 / (ms * 1e-3) / 1e12
        del q, kk, vv
    except Exception as e:  # a build without a fused attention kernel for this shape
        out["sdpa_long_context_shape_TFLOPs"] = None
        out["sdpa_error"] = str(e)[:200]
    torch.cuda.empty_cache()
    out["note"] = "library kernels through torch on this box in this run; fractions of the published peaks: " \
                  f"copy {out['hbm_copy_GBps'] / PEAK_HBM_GBS:.2f}, read {out['hbm_read_GBps'] / PEAK_HBM_GBS:.2f}, " \
                  f"GEMM {out['bf16_gemm_8192_TFLOPs'] / PEAK_BF16_TFLOPS:.2f}"
    return out


def bench_draft_tree(steps, warmup, B=16, K=10, T=5, N=60, V=152064):
    """Construction of the 60-node draft trees of the batch-16 workload from synthetic draft
    logits: per level one top-k pass over the logits of the rows the draft model ran on (16 at the
    root level, then 160) and one hb_tree_grow; hb_tree_finalize at the end.  The draft model's
    own forward passes are not part of it.  The top-k pass is bound by HBM (it reads every logit
    once); three sets of logits rotate so that a pass does not find them in the last-level cache."""
    import torch
    import workloads as W
    import paper_2509_18824_amd as hb
    import paper_2509_18824_amd.step as S

    sets = [torch.from_numpy(W.make_draft_logits(70 + i, B * K, V)).cuda() for i in range(3)]
    roots = [x[:B].contiguous() for x in sets]
    ids0, lp0 = (torch.empty((B, K), dtype=t, device="cuda") for t in (torch.int32, torch.float32))
    ids1, lp1 = (torch.empty((B * K, K), dtype=t, device="cuda") for t in (torch.int32, torch.float32))
    ws = S.alloc_workspace(hb.hb_topk_logprob_workspace_bytes(B * K, V, K))
    builder = S.DraftTreeBuilder(B, K, T)
    root_token = torch.arange(B, dtype=torch.int32, device="cuda")
    n = B * N
    i32 = lambda m: torch.empty(m, dtype=torch.int32, device="cuda")
    outs = (i32(B + 1), i32(n), i32(n), i32(n), torch.empty(n, dtype=torch.int64, device="cuda"), i32(n),
            torch.empty(n, dtype=torch.float32, device="cuda"))

    def build(i):
        for level in range(T):
            x = roots[(i + level) % 3] if level == 0 else sets[(i + level) % 3]
            ids, lp = (ids0, lp0) if level == 0 else (ids1, lp1)
            hb.hb_topk_logprob(x, K, ids, lp, ws)
            hb.hb_tree_grow(B, K, T, level, ids, lp, builder.cand_score, builder.cand_token, builder.cand_parent,
                            builder.frontier, builder.frontier_slot)
        hb.hb_tree_finalize(B, K, T, N, builder.cand_score, builder.cand_token, builder.cand_parent, root_token, *outs)

    for i in range(warmup):
        build(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        build(i)
    torch.cuda.synchronize()
    ms_build = (time.perf_counter() - t0) * 1e3 / steps
    # the top-k pass of one level (160 rows) alone: back-to-back calls over the rotating logits,
    # one event pair around all of them (an event pair per call would add its own 10-20 us)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for i in range(steps):
        hb.hb_topk_logprob(sets[i % 3], K, ids1, lp1, ws)
    b.record()
    torch.cuda.synchronize()
    ms_topk = a.elapsed_time(b) / steps
    level_bytes = B * K * V * 4
    return {
        "what": f"{B} trees of {N} nodes from {K} children per node over {T} levels, vocabulary {V}, float32 logits; "
                "top-k + grow per level, finalize; the draft model's forward passes are not included",
        "ms_per_build": ms_build, "trees_per_s": B / (ms_build * 1e-3),
        "topk_level_ms": ms_topk, "topk_level_rows": B * K, "topk_level_bytes": level_bytes,
        "topk_GBps": level_bytes / (ms_topk * 1e-3) / 1e9,
        "topk_frac_of_hbm_peak": level_bytes / (ms_topk * 1e-3) / 1e9 / PEAK_HBM_GBS,
    }


def bench_meta_query(steps, warmup, n_tok=96, L=28, D=3584, H=28, Q=3):
    """The draft model's intermediate layer (meta-query cross-attention over the target's layer
    features, output projection with skip connection, fc1) on the tokens one step commits at most
    (16 sequences x 6), random weights.  Per call: value projection GEMM [n_tok * L, D] x [D, D],
    the score and softmax / mixing kernels, output projection, fc1."""
    import torch
    import workloads as W
    import paper_2509_18824_amd as hb
    import paper_2509_18824_amd.step as S

    x = {k: v.cuda() for k, v in W.make_meta_inputs(90, n_tok, L, D, H, Q).items()}
    layer = S.MetaQueryLayer(x["f_q"], x["w_q"], x["w_k"], x["w_v"], x["w_o"], x["w_fc1"], H, residual_layers=[2, L // 2, L - 1])
    feats = x["feats"]
    bf = lambda *shape: torch.empty(shape, dtype=torch.bfloat16, device="cuda")
    v_proj, pre, res, f_c, out = bf(n_tok * L, D), bf(n_tok * Q, D), bf(n_tok * Q, D), bf(n_tok * Q, D), bf(n_tok, D)
    names = ("value_projection", "meta_query_attn", "output_projection", "fc1")
    ws_fc1 = S.alloc_workspace(hb.hb_proj_workspace_bytes(n_tok, Q * D, D))  # split-K partials (few tokens only)
    ws_out = S.alloc_workspace(hb.hb_proj_workspace_bytes(n_tok * Q, D, D))
    ws_attn = S.alloc_workspace(hb.hb_meta_query_attn_workspace_bytes(n_tok, D, H, Q))  # partial scores

    def call(ev=None):
        marks = []
        def mark():
            if ev is not None:
                e = torch.cuda.Event(enable_timing=True)
                e.record()
                marks.append(e)
        mark()
        hb.hb_out_project(feats.view(n_tok * L, D), layer.w_v, None, v_proj)
        mark()
        hb.hb_meta_query_attn(H, Q, feats, v_proj.view(n_tok, L, D), layer.a_fold, layer.residual_layers,
                              pre.view(n_tok, Q, D), res.view(n_tok, Q, D), ws_attn)
        mark()
        hb.hb_out_project_ws(pre, layer.w_o, res, f_c, ws_out)
        mark()
        hb.hb_out_project_ws(f_c.view(n_tok, Q * D), layer.w_fc1, None, out, ws_fc1)
        mark()
        if ev is not None:
            ev.append(marks)

    for _ in range(warmup):
        call()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        call()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    ev = []
    for _ in range(steps):
        call(ev)
    torch.cuda.synchronize()
    parts = {n: sum(m[i].elapsed_time(m[i + 1]) for m in ev) / steps for i, n in enumerate(names)}
    attn_bytes = 2 * n_tok * L * D * 2 + 2 * n_tok * Q * D * 2
    return {
        "what": f"{n_tok} tokens x {L} layer features of size {D}, {H} heads, {Q} meta queries, bf16, random weights",
        "ms_per_call": ms, "tokens_per_s": n_tok / (ms * 1e-3), "ms_by_call": parts,
        "value_projection_TFLOPs": 2.0 * n_tok * L * D * D / (parts["value_projection"] * 1e-3) / 1e12,
        "meta_query_attn_bytes": attn_bytes,
        "meta_query_attn_GBps": attn_bytes / (parts["meta_query_attn"] * 1e-3) / 1e9,
    }


def bench_layer_stack(inp, desc, dv, lm_weight, draft_np, n_steps, n_layers=28, ffn=0):
    """The step at a realistic depth: 28 layers, each QKV projection + rotary embedding ->
    tree-verify attention over its own KV pools (2.3 GB in all, so every layer streams its KV from
    HBM) -> output projection with residual (random weights, hidden size 3584); then the LM head,
    acceptance, and 28 compactions.  With ``ffn`` > 0 the layers are whole pre-norm decoder layers:
    RMSNorm in front of both halves, a gated-SiLU feed-forward block of that width behind the
    attention half (0.41 GB of weights per layer at 18944), a final RMSNorm.  Captured once into a
    HIP graph and replayed; the eager run gives the share of each kind of call (events on the
    launch stream)."""
    import torch
    import paper_2509_18824_amd.step as S

    T, Hq, D = dv.q.shape
    Hkv = dv.k_tree.shape[1]
    K = Hq * D
    g = torch.Generator(device="cuda").manual_seed(28)
    mk = lambda *shape, std: (torch.randn(shape, generator=g, device="cuda", dtype=torch.float32) * std).to(torch.bfloat16)
    w_qkv = [mk((Hq + 2 * Hkv) * D, K, std=K ** -0.5) for _ in range(n_layers)]
    w_o = [mk(K, K, std=0.3 * K ** -0.5) for _ in range(n_layers)]
    hidden0 = mk(T, K, std=1.0)
    pools = [(dv.k_pool, dv.v_pool)] + [(dv.k_pool.clone(), dv.v_pool.clone()) for _ in range(n_layers - 1)]
    draft = torch.from_numpy(draft_np).to(torch.int32).cuda()
    mlp = None
    if ffn:
        ones = lambda: (1.0 + 0.1 * torch.randn(K, generator=g, device="cuda")).to(torch.bfloat16)
        mlp = dict(norm1=[ones() for _ in range(n_layers)], norm2=[ones() for _ in range(n_layers)],
                   w_gate_up=[mk(2 * ffn, K, std=K ** -0.5) for _ in range(n_layers)],
                   w_down=[mk(K, ffn, std=0.3 * ffn ** -0.5) for _ in range(n_layers)], norm_f=ones(), eps=1e-6)
    stack = S.VerifyLayerStack(desc, dv, pools, w_qkv, w_o, lm_weight, draft, inp.max_path, hidden0, mlp=mlp)

    for _ in range(2):
        stack.run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(n_steps):
        stack.run()
    torch.cuda.synchronize()
    ms_eager = (time.perf_counter() - t0) * 1e3 / n_steps
    # share of each kind of call: eager steps with an event before every call, the smallest of
    # three per kind (a single step now and then shows a stall of tens of milliseconds in one call)
    share = {}
    for _ in range(3):
        marks = []
        def on_call(name):
            ev = torch.cuda.Event(enable_timing=True)
            ev.record()
            marks.append((name, ev))
        stack.run(on_call=on_call)
        torch.cuda.synchronize()
        one = {}
        for (name, ev), (_, nxt) in zip(marks[:-1], marks[1:]):
            one[name] = one.get(name, 0.0) + ev.elapsed_time(nxt)
        share = {k: min(v, share.get(k, v)) for k, v in one.items()}
    # graph: capture on a side stream, replay on it
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        stack.run()
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            stack.run()
        for _ in range(2):
            graph.replay()
        side.synchronize()
        t0 = time.perf_counter()
        for _ in range(n_steps):
            graph.replay()
        side.synchronize()
        ms_graph = (time.perf_counter() - t0) * 1e3 / n_steps
    target_graph = stack.target_ids.clone()
    stack.run()
    torch.cuda.synchronize()
    same = bool(torch.equal(target_graph, stack.target_ids))
    kv_bytes = inp.kv_bytes()
    gemm_flops = 2.0 * T * K * ((Hq + 2 * Hkv) * D + K)
    extra = {}
    if ffn:
        ffn_ms = share.get("swiglu_project", 0.0) + share.get("down_project", 0.0)
        extra = {"ffn_width": ffn, "ffn_TFLOPs": 2.0 * T * K * 3 * ffn * n_layers / (ffn_ms * 1e-3) / 1e12,
                 "ffn_weight_GBps": 3.0 * ffn * K * 2 * n_layers / (ffn_ms * 1e-3) / 1e9,
                 "weights_GB": n_layers * (3.0 * ffn * K + ((Hq + 2 * Hkv) * D + K) * K) * 2 / 1e9}
    return {
        **extra,
        "layers": n_layers, "steps": n_steps, "ms_per_step": ms_graph, "ms_per_step_eager": ms_eager,
        "tree_tokens_per_s": T / (ms_graph * 1e-3), "graph_replay_equals_eager": same,
        "eager_ms_by_call": share,
        "attn_ms_per_layer": share.get("tree_verify_attn", 0.0) / n_layers,
        "kv_GBps": kv_bytes / (share.get("tree_verify_attn", 1e9) / n_layers * 1e-3) / 1e9,
        "projection_TFLOPs": gemm_flops * n_layers / ((share.get("qkv_rope_project", 0) + share.get("out_project", 1e9)) * 1e-3) / 1e12,
        "what": ("per layer: RMSNorm, QKV projection + rotary embedding, tree-verify attention, output projection with "
                 "residual, RMSNorm, gated-SiLU projection, down projection with residual; final RMSNorm" if ffn else
                 "per layer: QKV projection + rotary embedding, tree-verify attention, output projection with residual "
                 "(the attention half only)")
                + "; then LM head + argmax, acceptance, compaction of all layers; one HIP graph per step",
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--tree", choices=["tree", "chain8"], default="tree",
                    help="the draft of the headline run (the default run reports the other one as a block)")
    ap.add_argument("--no-attn-extra", action="store_true", help="skip the attention-only runs of the "
                    "ragged-batch and long-context workloads")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-stack", action="store_true", help="skip the 28-layer variant of the step")
    ap.add_argument("--no-draft-tree", action="store_true", help="skip the draft tree's construction")
    ap.add_argument("--no-meta-query", action="store_true", help="skip the draft's intermediate layer")
    ap.add_argument("--no-chain", action="store_true", help="skip the 8-node-chain run of the step")
    ap.add_argument("--no-achievable", action="store_true", help="skip the library-kernel yardsticks")
    ap.add_argument("--no-parity", action="store_true", help="skip the comparison with the CPU oracle")
    ap.add_argument("--copy-probe", action="store_true", help="also run three 1 GiB device-to-device "
                    "copies before the timed region: the known-size reference for scaling the "
                    "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs on one GPU; --gpus must be 1 (no multi-GPU path exists)",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import workloads as W
    import paper_2509_18824_amd as hb
    import paper_2509_18824_amd.step as S

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    V, K = 152064, 28 * 128
    _, weight = W.make_lmhead_inputs(4000, 1, K, V, dtype="bf16")
    wdev = weight.cuda()

    if args.copy_probe:
        src = torch.ones(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    run = run_full_step(args.tree, args.steps, args.warmup, wdev, V, K)
    inp, desc, step, dv = run["inp"], run["desc"], run["step"], run["dev"]
    ms_step, ms_lm, ms_attn, ms_acc, ms_cmp = (run[k] for k in ("ms_step", "ms_lm", "ms_attn", "ms_acc", "ms_cmp"))
    accept_len = run["accept_len"]

    M = inp.total_nodes
    lm_flops = 2.0 * M * K * V
    lm_tflops = lm_flops / (ms_lm * 1e-3) / 1e12
    lm_bytes = V * K * 2 + M * K * 2
    kv_bytes = inp.kv_bytes()
    result = {
        "metric": "verified tree-tokens/sec per verify step",
        "value": M / (ms_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": f"{inp.name}: batch 16, ragged prefixes in [1024, 4096] (sum {int(inp.prefix_len.sum())}), "
                        f"28 q / 4 kv heads, head_dim 128, paged bf16 KV (page 16, permuted), "
                        f"{'60-node depth-6 trees' if args.tree == 'tree' else '8-node chains'} "
                        f"({M} nodes), 1 attention layer, LM head 3584 x 152064 with fused argmax, "
                        f"greedy acceptance, KV compaction",
            "tree": args.tree, "tree_nodes": M, "layers": 1,
            "mean_accept_len": float(accept_len.mean()),
        },
        "roofline": {
            "kernel": "lmhead_argmax",
            "bound": "mfma" if M >= 512 else "hbm",
            "achieved": lm_tflops if M >= 512 else lm_bytes / (ms_lm * 1e-3) / 1e9,
            "peak": PEAK_BF16_TFLOPS if M >= 512 else PEAK_HBM_GBS,
            "unit": "TFLOP/s" if M >= 512 else "GB/s",
            "frac": (lm_tflops / PEAK_BF16_TFLOPS) if M >= 512 else lm_bytes / (ms_lm * 1e-3) / 1e9 / PEAK_HBM_GBS,
            "traffic": (_lmhead_traffic(args.tree) or {}).get("bytes"),
            "traffic_detail": _lmhead_traffic(args.tree),
            "ms": ms_lm,
        },
        "kernels_ms": {"tree_verify_attn": ms_attn, "lmhead_argmax": ms_lm, "tree_accept": ms_acc,
                       "kv_compact": ms_cmp},
        "kv_read": {
            "bytes": kv_bytes, "GBps": kv_bytes / (ms_attn * 1e-3) / 1e9,
            "frac_of_hbm_peak": kv_bytes / (ms_attn * 1e-3) / 1e9 / PEAK_HBM_GBS,
            "attn_splits": hb.hb_tree_verify_attn_num_splits(desc),
        },
    }
    if not args.no_parity:
        result["parity"] = parity_check(run, weight)
    draft_np = run["draft_np"]
    if not args.no_stack:
        result["stack28"] = bench_layer_stack(inp, desc, dv, wdev, run["draft_np"], max(5, args.steps // 5))
        torch.cuda.empty_cache()
        # whole decoder layers: the feed-forward width of the 7B decoder that the paper's base model builds on
        result["decoder28"] = bench_layer_stack(inp, desc, dv, wdev, run["draft_np"], max(3, args.steps // 10), ffn=FFN_WIDTH)
        torch.cuda.empty_cache()
    other = "chain8" if args.tree == "tree" else "tree"
    if not args.no_chain:
        # The same step with the other draft shape (the paper measures chain drafts: Section 1,
        # Section 4.2): 8-node chains make 128 rows, where both the attention and the LM head are
        # bound by HBM, not by the matrix cores.
        del step, run
        torch.cuda.empty_cache()
        r2 = run_full_step(other, args.steps, args.warmup, wdev, V, K)
        M2 = r2["inp"].total_nodes
        kv2 = r2["inp"].kv_bytes()
        lm_gbps = lm_bytes_for(M2, K, V) / (r2["ms_lm"] * 1e-3) / 1e9
        result[other] = {
            "tree_nodes": M2, "ms_per_step": r2["ms_step"], "tree_tokens_per_s": M2 / (r2["ms_step"] * 1e-3),
            "mean_accept_len": float(r2["accept_len"].mean()),
            "kernels_ms": {"tree_verify_attn": r2["ms_attn"], "lmhead_argmax": r2["ms_lm"],
                           "tree_accept": r2["ms_acc"], "kv_compact": r2["ms_cmp"]},
            "lmhead_bound": "hbm" if M2 < 512 else "mfma",
            "lmhead_GBps": lm_gbps, "lmhead_frac_of_hbm_peak": lm_gbps / PEAK_HBM_GBS,
            "lmhead_TFLOPs": 2.0 * M2 * K * V / (r2["ms_lm"] * 1e-3) / 1e12,
            "lmhead_traffic": (_lmhead_traffic(other) or {}).get("bytes"),
            "kv_bytes": kv2, "kv_GBps": kv2 / (r2["ms_attn"] * 1e-3) / 1e9,
            "kv_frac_of_hbm_peak": kv2 / (r2["ms_attn"] * 1e-3) / 1e9 / PEAK_HBM_GBS,
        }
        if not args.no_parity:
            result[other]["parity"] = parity_check(r2, weight)
        if not args.no_stack:
            # the 28-layer variant with this draft shape too: with 128 tokens the projections are
            # weight streams and take the split-K path
            result[other]["stack28"] = bench_layer_stack(r2["inp"], r2["desc"], r2["dev"], wdev, r2["draft_np"],
                                                         max(5, args.steps // 5))
            torch.cuda.empty_cache()
            result[other]["decoder28"] = bench_layer_stack(r2["inp"], r2["desc"], r2["dev"], wdev, r2["draft_np"],
                                                           max(3, args.steps // 10), ffn=FFN_WIDTH)
            torch.cuda.empty_cache()
        del r2
    if not args.no_attn_extra and args.tree == "tree":
        step = run = None
        del wdev
        torch.cuda.empty_cache()
        result["attention_only"] = [bench_attention_only(c, max(args.steps, 20), args.warmup) for c in (2, 3)]
    if not args.no_draft_tree:
        torch.cuda.empty_cache()
        result["draft_tree"] = bench_draft_tree(max(args.steps, 20), args.warmup)
    if not args.no_meta_query:
        torch.cuda.empty_cache()
        result["meta_query"] = bench_meta_query(max(args.steps, 20), args.warmup)
    if not args.no_achievable:
        torch.cuda.empty_cache()
        result["achievable"] = achievable_peaks()
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(inp, weight, draft_np)
    print(json.dumps(result))


def lm_bytes_for(M, K, V):
    return V * K * 2 + M * K * 2


if __name__ == "__main__":
    main()
