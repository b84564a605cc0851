"""ctypes binding of include/hb.h: same names, argument marshalling only.

There is no fallback: if libhb.so is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libhb.so")

HB_F32, HB_BF16 = 0, 1
HB_ATTN_AUTO, HB_ATTN_SCALAR, HB_ATTN_MFMA = 0, 1, 2
_STATUS = {0: "HB_OK", 1: "HB_ERR_INVALID_ARG", 2: "HB_ERR_UNSUPPORTED", 3: "HB_ERR_WORKSPACE",
           4: "HB_ERR_DEVICE"}


class HbError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"{_STATUS.get(code, code)}: {message}")
        self.code = code


class AttnDesc(C.Structure):
    """Mirror of hb_attn_desc."""

    _fields_ = [
        ("dtype", C.c_int32), ("batch", C.c_int32), ("num_q_heads", C.c_int32),
        ("num_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("page_size", C.c_int32),
        ("max_blocks_per_seq", C.c_int32), ("num_blocks", C.c_int32), ("total_nodes", C.c_int32),
        ("max_nodes_per_tree", C.c_int32), ("num_splits", C.c_int32),
        ("max_prefix_len_hint", C.c_int32), ("algo", C.c_int32), ("softmax_scale", C.c_float),
    ]


def _load():
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is not built; run `python -m paper_2509_18824_amd.build` "
            "(hipcc, gfx950).  There is no fallback path.")
    lib = C.CDLL(_LIB_PATH)
    p, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    lib.hb_last_error.restype = C.c_char_p
    lib.hb_last_error.argtypes = []
    lib.hb_version.restype = i32
    lib.hb_version.argtypes = []
    lib.hb_tree_validate_host.restype = i32
    lib.hb_tree_validate_host.argtypes = [p, i32]
    lib.hb_tree_verify_attn.restype = i32
    lib.hb_tree_verify_attn.argtypes = [C.POINTER(AttnDesc)] + [p] * 11 + [p, sz, p]
    lib.hb_tree_verify_attn_workspace_bytes.restype = sz
    lib.hb_tree_verify_attn_workspace_bytes.argtypes = [C.POINTER(AttnDesc)]
    lib.hb_tree_verify_attn_num_splits.restype = i32
    lib.hb_tree_verify_attn_num_splits.argtypes = [C.POINTER(AttnDesc)]
    lib.hb_lmhead_argmax.restype = i32
    lib.hb_lmhead_argmax.argtypes = [i32, i32, i32, i32, p, p, p, p, p, sz, p]
    lib.hb_lmhead_argmax_workspace_bytes.restype = sz
    lib.hb_lmhead_argmax_workspace_bytes.argtypes = [i32]
    lib.hb_lmhead_argmax_noalloc.restype = i32
    lib.hb_lmhead_argmax_noalloc.argtypes = [i32, i32, i32, i32, p, p, p, p, p]
    lib.hb_lmhead_argmax_noalloc_max_rows.restype = i32
    lib.hb_lmhead_argmax_noalloc_max_rows.argtypes = []
    lib.hb_tree_positions.restype = i32
    lib.hb_tree_positions.argtypes = [i32, i32, i32, p, p, p, p, p]
    lib.hb_rope_table.restype = i32
    lib.hb_rope_table.argtypes = [i32, i32, C.c_double, p, p, p, p]
    lib.hb_qkv_rope_project.restype = i32
    lib.hb_qkv_rope_project.argtypes = [i32] * 5 + [p] * 8 + [p]
    lib.hb_out_project.restype = i32
    lib.hb_out_project.argtypes = [i32, i32, i32, p, p, p, p, p]
    lib.hb_proj_workspace_bytes.restype = sz
    lib.hb_proj_workspace_bytes.argtypes = [i32, i32, i32]
    lib.hb_qkv_rope_project_ws.restype = i32
    lib.hb_qkv_rope_project_ws.argtypes = [i32] * 5 + [p] * 8 + [p, sz, p]
    lib.hb_out_project_ws.restype = i32
    lib.hb_out_project_ws.argtypes = [i32, i32, i32, p, p, p, p, p, sz, p]
    lib.hb_tree_accept.restype = i32
    lib.hb_tree_accept.argtypes = [i32, i32, p, p, p, p, p, i32, p, p, p, p, p]
    lib.hb_tree_accept_sample.restype = i32
    lib.hb_tree_accept_sample.argtypes = [i32, i32, i32] + [p] * 7 + [i32] + [p] * 4 + [p, sz, p]
    lib.hb_tree_accept_sample_workspace_bytes.restype = sz
    lib.hb_tree_accept_sample_workspace_bytes.argtypes = [i32, i32]
    lib.hb_topk_logprob.restype = i32
    lib.hb_topk_logprob.argtypes = [i32, i32, i32, i32, p, p, p, p, sz, p]
    lib.hb_topk_logprob_workspace_bytes.restype = sz
    lib.hb_topk_logprob_workspace_bytes.argtypes = [i32, i32, i32]
    lib.hb_draft_tree_candidates.restype = i32
    lib.hb_draft_tree_candidates.argtypes = [i32, i32]
    lib.hb_tree_grow.restype = i32
    lib.hb_tree_grow.argtypes = [i32, i32, i32, i32] + [p] * 7 + [p]
    lib.hb_tree_finalize.restype = i32
    lib.hb_tree_finalize.argtypes = [i32, i32, i32, i32] + [p] * 11 + [p]
    lib.hb_rmsnorm.restype = i32
    lib.hb_rmsnorm.argtypes = [i32, i32, p, p, C.c_float, p, p]
    lib.hb_swiglu_project.restype = i32
    lib.hb_swiglu_project.argtypes = [i32, i32, i32, p, p, p, p, sz, p]
    lib.hb_meta_query_fold_bytes.restype = sz
    lib.hb_meta_query_fold_bytes.argtypes = [i32, i32, i32]
    lib.hb_meta_query_fold.restype = i32
    lib.hb_meta_query_fold.argtypes = [i32, i32, i32, p, p, p, p, p, sz, p]
    lib.hb_meta_query_attn.restype = i32
    lib.hb_meta_query_attn.argtypes = [i32] * 5 + [p, p, p, C.POINTER(i32), p, p, p, sz, p]
    lib.hb_meta_query_attn_workspace_bytes.restype = sz
    lib.hb_meta_query_attn_workspace_bytes.argtypes = [i32, i32, i32, i32]
    lib.hb_kv_compact.restype = i32
    lib.hb_kv_compact.argtypes = [C.POINTER(AttnDesc)] + [p] * 9 + [i32, p, p, p]
    lib.hb_kv_compact_layers.restype = i32
    lib.hb_kv_compact_layers.argtypes = [C.POINTER(AttnDesc), i32] + [p] * 9 + [i32, p, p, p]
    return lib


lib = _load()


def _check(rc: int):
    if rc != 0:
        raise HbError(rc, lib.hb_last_error().decode())


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("tensors handed to libhb must be contiguous")
    return C.c_void_p(t.data_ptr())


def _stream(stream) -> C.c_void_p:
    if stream is None:
        if not torch.cuda.is_available():
            return C.c_void_p(0)  # only argument validation can succeed without a device
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return HB_F32
    if t.dtype == torch.bfloat16:
        return HB_BF16
    raise HbError(2, f"dtype {t.dtype} is not supported")


def hb_last_error() -> str:
    return lib.hb_last_error().decode()


def hb_version() -> int:
    return int(lib.hb_version())


def hb_tree_validate_host(parent) -> None:
    arr = (C.c_int32 * len(parent))(*[int(x) for x in parent])
    _check(lib.hb_tree_validate_host(arr, len(parent)))


def hb_tree_verify_attn_workspace_bytes(desc: AttnDesc) -> int:
    return int(lib.hb_tree_verify_attn_workspace_bytes(C.byref(desc)))


def hb_tree_verify_attn_num_splits(desc: AttnDesc) -> int:
    return int(lib.hb_tree_verify_attn_num_splits(C.byref(desc)))


def hb_tree_verify_attn(desc: AttnDesc, q, k_tree, v_tree, k_pool, v_pool, block_table, prefix_len,
                        node_offset, parent, out, lse=None, workspace=None, stream=None) -> None:
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib.hb_tree_verify_attn(C.byref(desc), _ptr(q), _ptr(k_tree), _ptr(v_tree), _ptr(k_pool),
                                   _ptr(v_pool), _ptr(block_table), _ptr(prefix_len), _ptr(node_offset),
                                   _ptr(parent), _ptr(out), _ptr(lse), _ptr(workspace), ws_bytes,
                                   _stream(stream)))


def hb_lmhead_argmax_workspace_bytes(M: int) -> int:
    return int(lib.hb_lmhead_argmax_workspace_bytes(M))


def hb_lmhead_argmax(hidden, weight, out_ids, out_max=None, workspace=None, stream=None) -> None:
    M, K = hidden.shape
    V = weight.shape[0]
    if weight.shape[1] != K or weight.dtype != hidden.dtype:
        raise ValueError("weight must be [V, K] in the dtype of hidden")
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib.hb_lmhead_argmax(_dtype_code(hidden), M, K, V, _ptr(hidden), _ptr(weight), _ptr(out_ids),
                                _ptr(out_max), _ptr(workspace), ws_bytes, _stream(stream)))


def hb_lmhead_argmax_noalloc_max_rows() -> int:
    return int(lib.hb_lmhead_argmax_noalloc_max_rows())


def hb_lmhead_argmax_noalloc(hidden, weight, out_ids, out_max=None, stream=None) -> None:
    M, K = hidden.shape
    V = weight.shape[0]
    if weight.shape[1] != K or weight.dtype != hidden.dtype:
        raise ValueError("weight must be [V, K] in the dtype of hidden")
    _check(lib.hb_lmhead_argmax_noalloc(_dtype_code(hidden), M, K, V, _ptr(hidden), _ptr(weight), _ptr(out_ids),
                                        _ptr(out_max), _stream(stream)))


def hb_tree_positions(B: int, max_nodes_per_tree: int, node_offset, parent, prefix_len, positions, stream=None) -> None:
    _check(lib.hb_tree_positions(B, max_nodes_per_tree, positions.numel(), _ptr(node_offset), _ptr(parent),
                                 _ptr(prefix_len), _ptr(positions), _stream(stream)))


def hb_rope_table(head_dim: int, theta: float, positions, cos_out, sin_out, stream=None) -> None:
    _check(lib.hb_rope_table(positions.numel(), head_dim, float(theta), _ptr(positions), _ptr(cos_out), _ptr(sin_out),
                             _stream(stream)))


def hb_qkv_rope_project(hidden, w_qkv, bias, cos, sin, q, k, v, stream=None) -> None:
    T, K = hidden.shape
    _, Hq, D = q.shape
    Hkv = k.shape[1]
    if w_qkv.shape != ((Hq + 2 * Hkv) * D, K) or hidden.dtype != torch.bfloat16 or w_qkv.dtype != torch.bfloat16:
        raise ValueError("w_qkv must be bf16 [(Hq + 2 Hkv) * D, K]")
    _check(lib.hb_qkv_rope_project(T, K, Hq, Hkv, D, _ptr(hidden), _ptr(w_qkv), _ptr(bias), _ptr(cos), _ptr(sin),
                                   _ptr(q), _ptr(k), _ptr(v), _stream(stream)))


def hb_out_project(x, w, residual, out, stream=None) -> None:
    T, K = x.shape
    N = w.shape[0]
    if w.shape[1] != K or x.dtype != torch.bfloat16 or w.dtype != torch.bfloat16 or out.shape != (T, N):
        raise ValueError("need bf16 x [T, K], w [N, K], out [T, N]")
    _check(lib.hb_out_project(T, K, N, _ptr(x), _ptr(w), _ptr(residual), _ptr(out), _stream(stream)))


def hb_proj_workspace_bytes(T: int, K: int, N: int) -> int:
    return int(lib.hb_proj_workspace_bytes(T, K, N))


def hb_qkv_rope_project_ws(hidden, w_qkv, bias, cos, sin, q, k, v, workspace, stream=None) -> None:
    T, K = hidden.shape
    _, Hq, D = q.shape
    Hkv = k.shape[1]
    if w_qkv.shape != ((Hq + 2 * Hkv) * D, K) or hidden.dtype != torch.bfloat16 or w_qkv.dtype != torch.bfloat16:
        raise ValueError("w_qkv must be bf16 [(Hq + 2 Hkv) * D, K]")
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib.hb_qkv_rope_project_ws(T, K, Hq, Hkv, D, _ptr(hidden), _ptr(w_qkv), _ptr(bias), _ptr(cos), _ptr(sin),
                                      _ptr(q), _ptr(k), _ptr(v), _ptr(workspace), ws_bytes, _stream(stream)))


def hb_out_project_ws(x, w, residual, out, workspace, stream=None) -> None:
    T, K = x.shape
    N = w.shape[0]
    if w.shape[1] != K or x.dtype != torch.bfloat16 or w.dtype != torch.bfloat16 or out.shape != (T, N):
        raise ValueError("need bf16 x [T, K], w [N, K], out [T, N]")
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib.hb_out_project_ws(T, K, N, _ptr(x), _ptr(w), _ptr(residual), _ptr(out), _ptr(workspace), ws_bytes,
                                 _stream(stream)))


def hb_rmsnorm(x, weight, eps: float, out, stream=None) -> None:
    T, K = x.shape
    if x.dtype != torch.bfloat16 or weight.dtype != torch.bfloat16 or weight.shape != (K,) or out.shape != (T, K):
        raise ValueError("need bf16 x [T, K], weight [K], out [T, K]")
    _check(lib.hb_rmsnorm(T, K, _ptr(x), _ptr(weight), eps, _ptr(out), _stream(stream)))


def hb_swiglu_project(x, w_gate_up, out, workspace=None, stream=None) -> None:
    T, K = x.shape
    F = w_gate_up.shape[0] // 2
    if (w_gate_up.shape != (2 * F, K) or x.dtype != torch.bfloat16 or w_gate_up.dtype != torch.bfloat16
            or out.shape != (T, F)):
        raise ValueError("need bf16 x [T, K], w_gate_up [2 F, K], out [T, F]")
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib.hb_swiglu_project(T, K, F, _ptr(x), _ptr(w_gate_up), _ptr(out), _ptr(workspace), ws_bytes,
                                 _stream(stream)))


def hb_tree_accept(B: int, max_nodes_per_tree: int, node_offset, parent, draft_ids, target_ids,
                   max_path: int, accept_len, accept_path, out_tokens, bonus_id, stream=None,
                   prev_target=None) -> None:
    _check(lib.hb_tree_accept(B, max_nodes_per_tree, _ptr(node_offset), _ptr(parent), _ptr(draft_ids),
                              _ptr(target_ids), _ptr(prev_target), max_path, _ptr(accept_len), _ptr(accept_path),
                              _ptr(out_tokens), _ptr(bonus_id), _stream(stream)))


def hb_tree_accept_sample_workspace_bytes(B: int, V: int) -> int:
    return int(lib.hb_tree_accept_sample_workspace_bytes(B, V))


def hb_tree_accept_sample(B: int, max_nodes_per_tree: int, node_offset, parent, draft_ids, p_target, q_draft,
                          u_accept, u_bonus, max_path: int, accept_len, accept_path, out_tokens, bonus_id,
                          workspace, stream=None) -> None:
    V = p_target.shape[1]
    if p_target.dtype != torch.float32 or q_draft.dtype != torch.float32 or q_draft.shape != p_target.shape:
        raise ValueError("p_target and q_draft must be float32 [total_nodes, V]")
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib.hb_tree_accept_sample(B, max_nodes_per_tree, V, _ptr(node_offset), _ptr(parent), _ptr(draft_ids),
                                     _ptr(p_target), _ptr(q_draft), _ptr(u_accept), _ptr(u_bonus), max_path,
                                     _ptr(accept_len), _ptr(accept_path), _ptr(out_tokens), _ptr(bonus_id),
                                     _ptr(workspace), ws_bytes, _stream(stream)))


def hb_topk_logprob_workspace_bytes(M: int, V: int, k: int) -> int:
    return int(lib.hb_topk_logprob_workspace_bytes(M, V, k))


def hb_topk_logprob(logits, k: int, out_ids, out_logp, workspace, stream=None) -> None:
    if logits.dtype not in (torch.float32, torch.bfloat16) or logits.dim() != 2 or not logits.is_contiguous():
        raise ValueError("logits must be a contiguous float32 or bfloat16 [M, V] tensor")
    M, V = logits.shape
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib.hb_topk_logprob(HB_BF16 if logits.dtype == torch.bfloat16 else HB_F32, M, V, k, _ptr(logits),
                               _ptr(out_ids), _ptr(out_logp), _ptr(workspace), ws_bytes, _stream(stream)))


def hb_draft_tree_candidates(K: int, T: int) -> int:
    return int(lib.hb_draft_tree_candidates(K, T))


def hb_tree_grow(B: int, K: int, T: int, level: int, child_ids, child_logp, cand_score, cand_token, cand_parent,
                 frontier, frontier_slot, stream=None) -> None:
    _check(lib.hb_tree_grow(B, K, T, level, _ptr(child_ids), _ptr(child_logp), _ptr(cand_score), _ptr(cand_token),
                            _ptr(cand_parent), _ptr(frontier), _ptr(frontier_slot), _stream(stream)))


def hb_tree_finalize(B: int, K: int, T: int, n_nodes: int, cand_score, cand_token, cand_parent, root_token,
                     node_offset, parent, draft_ids, depth, anc_mask, node_cand, node_score, stream=None) -> None:
    _check(lib.hb_tree_finalize(B, K, T, n_nodes, _ptr(cand_score), _ptr(cand_token), _ptr(cand_parent),
                                _ptr(root_token), _ptr(node_offset), _ptr(parent), _ptr(draft_ids), _ptr(depth),
                                _ptr(anc_mask), _ptr(node_cand), _ptr(node_score), _stream(stream)))


def hb_meta_query_fold_bytes(Q: int, D: int, H: int) -> int:
    return int(lib.hb_meta_query_fold_bytes(Q, D, H))


def hb_meta_query_fold(H: int, f_q, w_q, w_k, a_fold, workspace, stream=None) -> None:
    Q, D = f_q.shape
    for t in (f_q, w_q, w_k, a_fold):
        if t.dtype != torch.bfloat16 or not t.is_contiguous():
            raise ValueError("bf16 contiguous tensors expected")
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib.hb_meta_query_fold(Q, D, H, _ptr(f_q), _ptr(w_q), _ptr(w_k), _ptr(a_fold), _ptr(workspace), ws_bytes,
                                  _stream(stream)))


def hb_meta_query_attn_workspace_bytes(S: int, D: int, H: int, Q: int) -> int:
    return int(lib.hb_meta_query_attn_workspace_bytes(S, D, H, Q))


def hb_meta_query_attn(H: int, Q: int, feats, v_proj, a_fold, residual_layers, pre, residual_out, workspace,
                       stream=None) -> None:
    S, L, D = feats.shape
    for t in (feats, v_proj, a_fold, pre):
        if t.dtype != torch.bfloat16 or not t.is_contiguous():
            raise ValueError("bf16 contiguous tensors expected")
    layers = (C.c_int32 * Q)(*[int(x) for x in residual_layers]) if residual_layers is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib.hb_meta_query_attn(S, L, D, H, Q, _ptr(feats), _ptr(v_proj), _ptr(a_fold), layers, _ptr(pre),
                                  _ptr(residual_out), _ptr(workspace), ws_bytes, _stream(stream)))


def hb_kv_compact(desc: AttnDesc, k_tree, v_tree, k_pool, v_pool, block_table, prefix_len, node_offset,
                  accept_len, accept_path, max_path: int, out_slots=None, new_len=None, stream=None) -> None:
    _check(lib.hb_kv_compact(C.byref(desc), _ptr(k_tree), _ptr(v_tree), _ptr(k_pool), _ptr(v_pool),
                             _ptr(block_table), _ptr(prefix_len), _ptr(node_offset), _ptr(accept_len),
                             _ptr(accept_path), max_path, _ptr(out_slots), _ptr(new_len), _stream(stream)))


def hb_kv_compact_layers(desc: AttnDesc, n_layers: int, k_tree_ptrs, v_tree_ptrs, k_pool_ptrs, v_pool_ptrs,
                         block_table, prefix_len, node_offset, accept_len, accept_path, max_path: int,
                         out_slots=None, new_len=None, stream=None) -> None:
    """*_ptrs: int64 device tensors holding the data pointers of every layer's tensor."""
    for t in (k_tree_ptrs, v_tree_ptrs, k_pool_ptrs, v_pool_ptrs):
        if t.dtype != torch.int64 or t.numel() < n_layers:
            raise ValueError("pointer tables must be int64 tensors with one entry per layer")
    _check(lib.hb_kv_compact_layers(C.byref(desc), n_layers, _ptr(k_tree_ptrs), _ptr(v_tree_ptrs), _ptr(k_pool_ptrs),
                                    _ptr(v_pool_ptrs), _ptr(block_table), _ptr(prefix_len), _ptr(node_offset),
                                    _ptr(accept_len), _ptr(accept_path), max_path, _ptr(out_slots), _ptr(new_len),
                                    _stream(stream)))
