"""Shared comparison helpers for the GPU parity tests (GPU result vs CPU oracle)."""
import numpy as np
import torch

import workloads as W
from oracle import tree_attn_ref

# Tolerances: the absolute bounds are the ones stated for this work (1e-5 for fp32 inputs,
# 2e-2 for bf16 inputs with fp32 accumulation).  With a near-uniform softmax over thousands of
# keys the outputs are only ~1e-2 in magnitude, so an absolute bound alone would accept zeros;
# the relative L2 error and the log-sum-exp error are checked as well.
TOL = {
    "f32": dict(abs=1e-5, rel_l2=1e-5, lse=1e-5),
    "bf16": dict(abs=2e-2, rel_l2=1e-2, lse=1e-2),
}


def oracle_attn(inp, nodes=None):
    return tree_attn_ref(W.widen(inp.q), W.widen(inp.k_tree), W.widen(inp.v_tree), W.widen(inp.k_pool),
                         W.widen(inp.v_pool), inp.block_table.numpy(), inp.prefix_len.numpy(),
                         inp.node_offset.numpy(), inp.parent.numpy(), inp.softmax_scale, nodes=nodes)


def check_attn(inp, out_gpu, lse_gpu, nodes=None, ref=None, label=""):
    ref_out, ref_lse = ref if ref is not None else oracle_attn(inp, nodes)
    got = W.widen(out_gpu)
    got_lse = W.widen(lse_gpu) if lse_gpu is not None else None
    if nodes is not None:
        got = got[list(nodes)]
        got_lse = got_lse[list(nodes)] if got_lse is not None else None
    tol = TOL[inp.dtype]
    assert np.isfinite(got).all(), f"{label}: non-finite output"
    err = np.abs(got - ref_out).max()
    rel = np.linalg.norm(got - ref_out) / max(np.linalg.norm(ref_out), 1e-30)
    assert err <= tol["abs"], f"{label}: max abs err {err:.3e} > {tol['abs']}"
    assert rel <= tol["rel_l2"], f"{label}: rel L2 err {rel:.3e} > {tol['rel_l2']}"
    if got_lse is not None:
        lerr = np.abs(got_lse - ref_lse).max()
        assert lerr <= tol["lse"], f"{label}: lse err {lerr:.3e} > {tol['lse']}"
    return err, rel


def bits(t: torch.Tensor) -> np.ndarray:
    """Bit pattern of a tensor as numpy (bf16 as int16)."""
    t = t.detach().cpu()
    return t.view(torch.int16).numpy() if t.dtype == torch.bfloat16 else t.numpy()
