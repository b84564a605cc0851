"""The C-ABI library loads, exports every symbol the header declares, and rejects bad
arguments on the host without touching a device (runs without a GPU)."""
import ctypes as C
import os
import re

import pytest

import paper_2509_18824_amd as hb
from paper_2509_18824_amd.step import make_desc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "hb.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hb_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = _declared()
    assert {"hb_tree_verify_attn", "hb_lmhead_argmax", "hb_tree_accept", "hb_kv_compact"} <= set(names)
    for n in names:
        assert hasattr(hb.lib, n), n
        assert hasattr(hb, n), f"python binding lacks {n}"


def test_version_and_tree_validation():
    assert hb.hb_version() >= 1
    hb.hb_tree_validate_host([-1, 0, 0, 2])
    for bad in ([0, 0], [-1, 1], [-1, 0, 3], [-1, -1]):
        with pytest.raises(hb.HbError) as e:
            hb.hb_tree_validate_host(bad)
        assert e.value.code == 1
    with pytest.raises(hb.HbError) as e:
        hb.hb_tree_validate_host([-1] + list(range(64)))
    assert e.value.code == 2


def _desc(**kw):
    base = dict(dtype="bf16", B=2, Hq=28, Hkv=4, D=128, page=16, max_blocks=64, num_blocks=200,
                total_nodes=120, max_nodes=60, softmax_scale=0.1)
    base.update(kw)
    return make_desc(**base)


def _attn_rc(desc, ws_bytes=0, ptr=0x1000):
    p = C.c_void_p(ptr)
    return hb.lib.hb_tree_verify_attn(C.byref(desc), p, p, p, p, p, p, p, p, p, p, None,
                                      C.c_void_p(0x1000) if ws_bytes else None, ws_bytes, None)


def test_attention_argument_errors():
    assert _attn_rc(_desc(Hq=30)) == 1  # heads do not divide
    assert "num_q_heads" in hb.hb_last_error()
    assert _attn_rc(_desc(D=100)) == 2
    assert _attn_rc(_desc(D=512)) == 2
    assert _attn_rc(_desc(max_nodes=65)) == 2
    assert "64" in hb.hb_last_error()
    assert _attn_rc(_desc(page=0)) == 1
    d = _desc()
    d.dtype = 7
    assert _attn_rc(d) == 2
    assert _attn_rc(_desc(), ptr=0) == 1  # null pointers
    d = _desc(num_splits=4)
    need = hb.hb_tree_verify_attn_workspace_bytes(d)
    assert need > 0 and hb.hb_tree_verify_attn_num_splits(d) == 4
    assert _attn_rc(d, ws_bytes=0) == 3
    assert _attn_rc(d, ws_bytes=need - 1) == 3
    assert _attn_rc(_desc(dtype="f32", D=64, algo=hb.HB_ATTN_MFMA)) == 2
    # empty batches are a no-op that needs no pointers
    assert _attn_rc(_desc(B=0, total_nodes=0), ptr=0) == 0
    # tensors must start at a 16-byte aligned address
    assert _attn_rc(_desc(), ptr=0x1008) == 1
    assert "aligned" in hb.hb_last_error()


def test_split_plan_is_consistent():
    for splits in (1, 2, 3, 7, 16):
        d = _desc(num_splits=splits, max_blocks=513)
        got = hb.hb_tree_verify_attn_num_splits(d)
        assert 1 <= got <= splits
        ws = hb.hb_tree_verify_attn_workspace_bytes(d)
        assert (ws == 0) == (got == 1)
        if got > 1:
            assert ws >= 120 * 28 * got * (128 + 2) * 4
    auto = hb.hb_tree_verify_attn_num_splits(_desc(max_blocks=2049))
    assert auto >= 1


def test_lmhead_accept_compact_argument_errors():
    p = C.c_void_p(0x1000)
    L = hb.lib
    assert L.hb_lmhead_argmax(1, 4, 8, 0, p, p, p, None, p, 64, None) == 1
    assert L.hb_lmhead_argmax(5, 4, 8, 16, p, p, p, None, p, 64, None) == 2
    assert L.hb_lmhead_argmax(1, 4, 8, 16, p, p, p, None, p, 8, None) == 3
    assert L.hb_lmhead_argmax(1, 4, 8, 16, None, p, p, None, p, 64, None) == 1
    assert L.hb_lmhead_argmax(1, 0, 8, 16, None, None, None, None, None, 0, None) == 0
    assert L.hb_lmhead_argmax(1, 4, 8, 16, C.c_void_p(0x1004), p, p, None, p, 64, None) == 1
    assert "aligned" in hb.hb_last_error()
    assert hb.hb_lmhead_argmax_workspace_bytes(960) == 960 * 8
    assert L.hb_tree_accept(2, 65, p, p, p, p, None, 6, p, p, p, p, None) == 2
    assert L.hb_tree_accept(2, 60, p, p, p, p, None, 0, p, p, p, p, None) == 1
    assert L.hb_tree_accept(2, 60, None, p, p, p, p, 6, p, p, p, p, None) == 1
    assert L.hb_tree_accept(0, 60, None, None, None, None, None, 6, None, None, None, None, None) == 0
    d = _desc()
    assert L.hb_kv_compact(C.byref(d), p, p, p, p, p, p, p, p, p, 0, None, None, None) == 1
    assert L.hb_kv_compact(C.byref(d), None, p, p, p, p, p, p, p, p, 6, None, None, None) == 1
    assert L.hb_kv_compact(None, p, p, p, p, p, p, p, p, p, 6, None, None, None) == 1
    assert L.hb_kv_compact(C.byref(d), C.c_void_p(0x1002), p, p, p, p, p, p, p, p, 6, None, None, None) == 1
    assert "aligned" in hb.hb_last_error()


def test_all_layer_compaction_argument_errors():
    L, p = hb.lib, C.c_void_p(0x1000)
    d = _desc()
    assert L.hb_kv_compact_layers(C.byref(d), 28, p, p, p, p, p, p, p, p, p, 0, None, None, None) == 1
    assert L.hb_kv_compact_layers(C.byref(d), -1, p, p, p, p, p, p, p, p, p, 6, None, None, None) == 1
    assert L.hb_kv_compact_layers(C.byref(d), 28, None, p, p, p, p, p, p, p, p, 6, None, None, None) == 1
    assert L.hb_kv_compact_layers(C.byref(d), 28, C.c_void_p(0x1004), p, p, p, p, p, p, p, p, 6, None, None, None) == 1
    assert L.hb_kv_compact_layers(C.byref(d), 0, None, None, None, None, None, None, None, None, None, 6, None, None, None) == 0
    assert L.hb_kv_compact_layers(None, 28, p, p, p, p, p, p, p, p, p, 6, None, None, None) == 1


def test_draft_tree_argument_errors():
    L, p = hb.lib, C.c_void_p(0x1000)
    assert L.hb_draft_tree_candidates(10, 5) == 410 and L.hb_draft_tree_candidates(1, 5) == 5
    assert L.hb_draft_tree_candidates(33, 2) == 0
    assert L.hb_topk_logprob(hb.HB_F32, 4, 100, 0, p, p, p, p, 1 << 20, None) == 1
    assert L.hb_topk_logprob(hb.HB_F32, 4, 100, 101, p, p, p, p, 1 << 20, None) == 1
    assert L.hb_topk_logprob(hb.HB_F32, 4, 100, 33, p, p, p, p, 1 << 20, None) == 2
    assert L.hb_topk_logprob(7, 4, 100, 5, p, p, p, p, 1 << 20, None) == 1
    assert L.hb_topk_logprob(hb.HB_F32, 4, 100, 5, None, p, p, p, 1 << 20, None) == 1
    assert L.hb_topk_logprob(hb.HB_F32, 4, 100, 5, p, p, p, p, 8, None) == 3
    assert L.hb_topk_logprob(hb.HB_F32, 0, 100, 5, None, None, None, None, 0, None) == 0
    assert hb.hb_topk_logprob_workspace_bytes(160, 152064, 10) == 160 * 10 * (8 + 80)
    assert L.hb_tree_grow(2, 10, 5, 5, p, p, p, p, p, p, p, None) == 1  # level outside [0, T)
    assert L.hb_tree_grow(2, 33, 5, 0, p, p, p, p, p, p, p, None) == 2
    assert L.hb_tree_grow(2, 10, 5, 0, p, None, p, p, p, p, p, None) == 1
    assert L.hb_tree_grow(0, 10, 5, 0, None, None, None, None, None, None, None, None) == 0
    assert L.hb_tree_finalize(2, 10, 5, 65, p, p, p, p, p, p, p, p, p, p, p, None) == 2
    assert L.hb_tree_finalize(2, 2, 2, 8, p, p, p, p, p, p, p, p, p, p, p, None) == 1  # 7 > 6 candidates
    assert L.hb_tree_finalize(2, 32, 6, 60, p, p, p, p, p, p, p, p, p, p, p, None) == 2  # 5152 candidates
    assert L.hb_tree_finalize(2, 10, 5, 60, p, p, p, None, p, p, p, p, p, p, p, None) == 1


def test_meta_query_argument_errors():
    L, p = hb.lib, C.c_void_p(0x1000)
    assert hb.hb_meta_query_fold_bytes(3, 3584, 28) == 2 * 96 * 3584 * 2
    assert L.hb_meta_query_fold(3, 3584, 28, p, p, p, p, p, 16, None) == 3
    assert L.hb_meta_query_fold(3, 3584, 27, p, p, p, p, p, 1 << 20, None) == 1      # H does not divide D
    assert L.hb_meta_query_fold(3, 3200, 5, p, p, p, p, p, 1 << 20, None) == 2       # D % 256
    assert L.hb_meta_query_fold(5, 3584, 28, p, p, p, p, p, 1 << 20, None) == 2      # Q > 4
    assert L.hb_meta_query_fold(3, 3584, 28, None, p, p, p, p, 1 << 20, None) == 1
    assert L.hb_meta_query_fold(3, 3584, 28, C.c_void_p(0x1002), p, p, p, p, 1 << 20, None) == 1
    layers = (C.c_int32 * 3)(0, 14, 28)
    assert L.hb_meta_query_attn(4, 28, 3584, 28, 3, p, p, p, layers, p, p, p, 1 << 30, None) == 1  # layer 28 of 28
    ok_layers = (C.c_int32 * 3)(0, 14, 27)
    assert L.hb_meta_query_attn(4, 28, 3584, 28, 3, p, p, p, ok_layers, p, None, p, 1 << 30, None) == 1  # no residual_out
    assert L.hb_meta_query_attn(4, 33, 3584, 28, 3, p, p, p, None, p, None, p, 1 << 30, None) == 2       # L > 32
    assert L.hb_meta_query_attn(4, 28, 3584, 56, 3, p, p, p, None, p, None, p, 1 << 30, None) == 2       # 168 rows
    assert L.hb_meta_query_attn(-1, 28, 3584, 28, 3, p, p, p, None, p, None, p, 1 << 30, None) == 1
    assert L.hb_meta_query_attn(0, 28, 3584, 28, 3, None, None, None, None, None, None, None, 0, None) == 0
    assert L.hb_meta_query_attn(4, 28, 3584, 28, 3, None, p, p, None, p, None, p, 1 << 30, None) == 1
    need = hb.hb_meta_query_attn_workspace_bytes(4, 3584, 28, 3)
    assert need == 14 * 4 * 96 * 32 * 4                      # 14 slices of 256 features, one workgroup column each
    assert hb.hb_meta_query_attn_workspace_bytes(8192, 3584, 28, 3) == 8192 * 96 * 32 * 4
    assert hb.hb_meta_query_attn_workspace_bytes(4, 3584, 56, 3) == 0
    assert L.hb_meta_query_attn(4, 28, 3584, 28, 3, p, p, p, None, p, None, p, need - 1, None) == 3
    assert L.hb_meta_query_attn(4, 28, 3584, 28, 3, p, p, p, None, p, None, None, need, None) == 3


def test_layer_rest_argument_errors():
    L, p = hb.lib, C.c_void_p(0x1000)
    assert L.hb_rmsnorm(4, 3584, p, p, 1e-6, None, None) == 1
    assert L.hb_rmsnorm(4, 3580, p, p, 1e-6, p, None) == 2            # K % 8
    assert L.hb_rmsnorm(4, 3584, p, p, -1.0, p, None) == 1            # eps < 0
    assert L.hb_rmsnorm(4, 3584, p, p, float("nan"), p, None) == 1
    assert L.hb_rmsnorm(4, 3584, C.c_void_p(0x1004), p, 1e-6, p, None) == 1
    assert L.hb_rmsnorm(0, 3584, None, None, 1e-6, None, None) == 0
    assert L.hb_swiglu_project(4, 3584, 18944, p, p, None, None, 0, None) == 1
    assert L.hb_swiglu_project(4, 3580, 18944, p, p, p, None, 0, None) == 2   # K % 64
    assert L.hb_swiglu_project(4, 3584, 18942, p, p, p, None, 0, None) == 2   # F % 4
    assert L.hb_swiglu_project(-1, 3584, 18944, p, p, p, None, 0, None) == 1
    assert L.hb_swiglu_project(0, 3584, 18944, None, None, None, None, 0, None) == 0
