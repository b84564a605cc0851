"""GPU test of hb_lmhead_argmax_noalloc, the entry point that allocates nothing: through the raw
C ABI (ctypes), against hb_lmhead_argmax on the same inputs, two calls in a row on one GPU, the
second with a smaller input (the library's row keys keep the first call's contents)."""
import ctypes as C

import numpy as np
import pytest
import torch

import workloads as W

pytestmark = pytest.mark.gpu


def _both(hb, hidden, weight):
    M, K = hidden.shape
    V = weight.shape[0]
    dt = hb.HB_BF16 if hidden.dtype == torch.bfloat16 else hb.HB_F32
    p = lambda t: C.c_void_p(t.data_ptr())
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    ids_a = torch.full((M,), -7, dtype=torch.int32, device="cuda")
    ids_b = torch.full((M,), -9, dtype=torch.int32, device="cuda")
    mx_a = torch.zeros(M, dtype=torch.float32, device="cuda")
    mx_b = torch.ones(M, dtype=torch.float32, device="cuda")
    ws = torch.empty(max(8, hb.hb_lmhead_argmax_workspace_bytes(M)), dtype=torch.uint8, device="cuda")
    rc = hb.lib.hb_lmhead_argmax(dt, M, K, V, p(hidden), p(weight), p(ids_a), p(mx_a), p(ws), ws.numel(), stream)
    assert rc == 0, hb.hb_last_error()
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    rc = hb.lib.hb_lmhead_argmax_noalloc(dt, M, K, V, p(hidden), p(weight), p(ids_b), p(mx_b), stream)
    assert rc == 0, hb.hb_last_error()
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(ids_a, ids_b), "ids differ between the workspace and the no-alloc entry point"
    assert torch.equal(mx_a, mx_b)
    return ids_b


def test_noalloc_matches_workspace_entry_point_twice_in_a_row():
    import paper_2509_18824_amd as hb
    assert hb.hb_lmhead_argmax_noalloc_max_rows() >= 960
    # first call: 960 rows on the matrix-core kernel, winners planted in the upper rows so that
    # stale keys of those rows would be visible to a later, smaller call
    hidden, weight = W.make_lmhead_inputs(31, 960, 512, 5000, dtype="bf16", w_std=0.05)
    for m in range(100, 960, 7):
        weight[(m * 5) % 5000] = (hidden[m].float() * 0.5).to(weight.dtype)
    h, w = hidden.cuda(), weight.cuda()
    ids1 = _both(hb, h, w)
    assert (ids1 >= 0).all() and (ids1 < 5000).all()
    # second call, right behind it: fewer rows, another vocabulary, the scalar kernel (K % 64 != 0)
    hidden2, weight2 = W.make_lmhead_inputs(32, 77, 136, 901, dtype="f32", w_std=0.05)
    ids2 = _both(hb, hidden2.cuda(), weight2.cuda())
    assert (ids2 >= 0).all() and (ids2 < 901).all()
    # third: a smaller bf16 call on the matrix-core kernel, then the first again
    ids3 = _both(hb, h[:130].contiguous(), w[:3000].contiguous())
    assert (ids3 < 3000).all()
    assert torch.equal(_both(hb, h, w), ids1)


def test_noalloc_rejects_more_rows_than_it_holds():
    import paper_2509_18824_amd as hb
    cap = hb.hb_lmhead_argmax_noalloc_max_rows()
    p = C.c_void_p(0x1000)
    rc = hb.lib.hb_lmhead_argmax_noalloc(hb.HB_BF16, cap + 1, 64, 100, p, p, p, None, None)
    assert rc == 2 and "at most" in hb.hb_last_error()
    assert hb.lib.hb_lmhead_argmax_noalloc(hb.HB_BF16, 0, 64, 100, None, None, None, None, None) == 0
    assert hb.lib.hb_lmhead_argmax_noalloc(hb.HB_BF16, 5, 64, 100, None, p, p, None, None) == 1
