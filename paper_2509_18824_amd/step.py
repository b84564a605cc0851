"""Convenience wrappers that allocate outputs/workspaces as torch tensors and call the C ABI.

Nothing here computes: each function sizes buffers, fills an ``AttnDesc`` and forwards to the
library.  ``VerifyStep`` chains the four calls of one verification step on the current stream.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import torch

from . import binding as hb


def make_desc(dtype, B, Hq, Hkv, D, page, max_blocks, num_blocks, total_nodes, max_nodes,
              softmax_scale, num_splits=0, hint=0, algo=hb.HB_ATTN_AUTO) -> hb.AttnDesc:
    code = hb.HB_F32 if dtype in ("f32", torch.float32) else hb.HB_BF16
    return hb.AttnDesc(dtype=code, batch=B, num_q_heads=Hq, num_kv_heads=Hkv, head_dim=D,
                       page_size=page, max_blocks_per_seq=max_blocks, num_blocks=num_blocks,
                       total_nodes=total_nodes, max_nodes_per_tree=max_nodes, num_splits=num_splits,
                       max_prefix_len_hint=hint, algo=algo, softmax_scale=float(softmax_scale))


@dataclass
class DeviceInputs:
    """Device copies of one batch (field names as in the C ABI)."""

    q: torch.Tensor
    k_tree: torch.Tensor
    v_tree: torch.Tensor
    k_pool: torch.Tensor
    v_pool: torch.Tensor
    block_table: torch.Tensor
    prefix_len: torch.Tensor
    node_offset: torch.Tensor
    parent: torch.Tensor


def to_device(inp, device="cuda") -> DeviceInputs:
    f = lambda t: t.to(device).contiguous()
    return DeviceInputs(f(inp.q), f(inp.k_tree), f(inp.v_tree), f(inp.k_pool), f(inp.v_pool),
                        f(inp.block_table), f(inp.prefix_len), f(inp.node_offset), f(inp.parent))


def desc_for(inp, num_splits=0, hint=0, algo=hb.HB_ATTN_AUTO) -> hb.AttnDesc:
    max_nodes = int((inp.node_offset[1:] - inp.node_offset[:-1]).max()) if inp.B else 1
    return make_desc(inp.dtype, inp.B, inp.Hq, inp.Hkv, inp.D, inp.page, inp.max_blocks,
                     inp.num_blocks, inp.total_nodes, max_nodes, inp.softmax_scale, num_splits,
                     hint, algo)


def alloc_workspace(nbytes: int, device="cuda") -> Optional[torch.Tensor]:
    if nbytes == 0:
        return None
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def tree_verify_attn(desc: hb.AttnDesc, dev: DeviceInputs, want_lse=True, workspace=None, out=None):
    """Returns (out, lse).  Allocates what is not passed in."""
    if out is None:
        out = torch.empty_like(dev.q)
    lse = torch.empty(dev.q.shape[:2], dtype=torch.float32, device=dev.q.device) if want_lse else None
    if workspace is None:
        workspace = alloc_workspace(hb.hb_tree_verify_attn_workspace_bytes(desc), dev.q.device)
    hb.hb_tree_verify_attn(desc, dev.q, dev.k_tree, dev.v_tree, dev.k_pool, dev.v_pool, dev.block_table,
                           dev.prefix_len, dev.node_offset, dev.parent, out, lse, workspace)
    return out, lse


def lmhead_argmax(hidden, weight, want_max=True, workspace=None):
    M = hidden.shape[0]
    ids = torch.empty(M, dtype=torch.int32, device=hidden.device)
    mx = torch.empty(M, dtype=torch.float32, device=hidden.device) if want_max else None
    if workspace is None:
        workspace = alloc_workspace(max(8, hb.hb_lmhead_argmax_workspace_bytes(M)), hidden.device)
    hb.hb_lmhead_argmax(hidden, weight, ids, mx, workspace)
    return ids, mx


def tree_accept(node_offset, parent, draft_ids, target_ids, max_path, max_nodes, prev_target=None):
    B = node_offset.numel() - 1
    dev = node_offset.device
    accept_len = torch.empty(B, dtype=torch.int32, device=dev)
    accept_path = torch.empty((B, max_path), dtype=torch.int32, device=dev)
    out_tokens = torch.empty((B, max_path), dtype=torch.int32, device=dev)
    bonus = torch.empty(B, dtype=torch.int32, device=dev)
    hb.hb_tree_accept(B, max_nodes, node_offset, parent, draft_ids, target_ids, max_path, accept_len,
                      accept_path, out_tokens, bonus, prev_target=prev_target)
    return accept_len, accept_path, out_tokens, bonus


def tree_accept_sample(node_offset, parent, draft_ids, p_target, q_draft, u_accept, u_bonus, max_path, max_nodes):
    """u_accept / u_bonus: int32 tensors holding the bit patterns of the 32-bit uniforms."""
    B = node_offset.numel() - 1
    dev = node_offset.device
    accept_len = torch.empty(B, dtype=torch.int32, device=dev)
    accept_path = torch.empty((B, max_path), dtype=torch.int32, device=dev)
    out_tokens = torch.empty((B, max_path), dtype=torch.int32, device=dev)
    bonus = torch.empty(B, dtype=torch.int32, device=dev)
    ws = alloc_workspace(max(4, hb.hb_tree_accept_sample_workspace_bytes(B, p_target.shape[1])), dev)
    hb.hb_tree_accept_sample(B, max_nodes, node_offset, parent, draft_ids, p_target, q_draft, u_accept, u_bonus,
                             max_path, accept_len, accept_path, out_tokens, bonus, ws)
    return accept_len, accept_path, out_tokens, bonus


def topk_logprob(logits, k):
    """ids int32 [M, k], logp float32 [M, k] of the k best tokens of every row."""
    M, V = logits.shape
    dev = logits.device
    ids = torch.empty((M, k), dtype=torch.int32, device=dev)
    logp = torch.empty((M, k), dtype=torch.float32, device=dev)
    ws = alloc_workspace(max(8, hb.hb_topk_logprob_workspace_bytes(M, V, k)), dev)
    hb.hb_topk_logprob(logits, k, ids, logp, ws)
    return ids, logp


class DraftTreeBuilder:
    """Device state of the draft tree's construction for a batch: the candidate pool and the
    frontier.  ``grow`` takes the top-k outputs of the rows the draft model just ran on (the
    root at level 0, then the frontier nodes in order); ``finalize`` emits the tree in the
    verification calls' layout."""

    def __init__(self, B: int, K: int, T: int, device="cuda"):
        self.B, self.K, self.T, self.level = B, K, T, 0
        C = hb.hb_draft_tree_candidates(K, T)
        if C <= 0:
            raise ValueError("unsupported K / T")
        self.C = C
        self.cand_score = torch.zeros((B, C), dtype=torch.float32, device=device)
        self.cand_token = torch.zeros((B, C), dtype=torch.int32, device=device)
        self.cand_parent = torch.full((B, C), -1, dtype=torch.int32, device=device)
        self.frontier = torch.zeros((B, K), dtype=torch.int32, device=device)
        self.frontier_slot = torch.zeros((B, K), dtype=torch.int32, device=device)

    def grow(self, child_ids, child_logp):
        hb.hb_tree_grow(self.B, self.K, self.T, self.level, child_ids, child_logp, self.cand_score, self.cand_token,
                        self.cand_parent, self.frontier, self.frontier_slot)
        self.level += 1
        return self.frontier, self.frontier_slot

    def finalize(self, n_nodes: int, root_token):
        B, dev = self.B, self.cand_score.device
        i32 = lambda *shape: torch.empty(shape, dtype=torch.int32, device=dev)
        out = dict(node_offset=i32(B + 1), parent=i32(B * n_nodes), draft_ids=i32(B * n_nodes), depth=i32(B * n_nodes),
                   anc_mask=torch.empty(B * n_nodes, dtype=torch.int64, device=dev), node_cand=i32(B * n_nodes),
                   node_score=torch.empty(B * n_nodes, dtype=torch.float32, device=dev))
        hb.hb_tree_finalize(B, self.K, self.T, n_nodes, self.cand_score, self.cand_token, self.cand_parent, root_token,
                            out["node_offset"], out["parent"], out["draft_ids"], out["depth"], out["anc_mask"],
                            out["node_cand"], out["node_score"])
        return out


def linear(x, w, residual, out):
    """out = x w^T (+ residual); small token counts take the split-K path (its workspace is allocated here)."""
    nbytes = hb.hb_proj_workspace_bytes(x.shape[0], x.shape[1], w.shape[0])
    ws = alloc_workspace(nbytes, x.device) if nbytes else None
    hb.hb_out_project_ws(x, w, residual, out, ws)


class MetaQueryLayer:
    """The draft model's intermediate layer up to fc1: meta-query cross-attention over the layer
    features of every token, output projection with the skip connection, fc1.  Weights bf16 in
    the y = x W^T layout; the key projection is folded into the queries at construction."""

    def __init__(self, f_q, w_q, w_k, w_v, w_o, w_fc1, H: int, residual_layers=None):
        self.Q, self.D = f_q.shape
        self.H, self.residual_layers = H, residual_layers
        self.w_v, self.w_o, self.w_fc1 = w_v, w_o, w_fc1
        dev = f_q.device
        self.a_fold = torch.empty(hb.hb_meta_query_fold_bytes(self.Q, self.D, H) // 2, dtype=torch.bfloat16, device=dev)
        ws = torch.empty(self.Q * self.D, dtype=torch.float32, device=dev)
        hb.hb_meta_query_fold(H, f_q, w_q, w_k, self.a_fold, ws)

    def run(self, feats):
        """feats bf16 [S, L, D] -> (F_c [S, Q * D], fc1 output [S, N1])."""
        S, L, D = feats.shape
        Q, dev = self.Q, feats.device
        bf = lambda *shape: torch.empty(shape, dtype=torch.bfloat16, device=dev)
        v_proj, pre, f_c = bf(S * L, D), bf(S * Q, D), bf(S * Q, D)
        res = bf(S * Q, D) if self.residual_layers is not None else None
        hb.hb_out_project(feats.view(S * L, D), self.w_v, None, v_proj)
        ws = torch.empty(hb.hb_meta_query_attn_workspace_bytes(S, D, self.H, Q) // 4, dtype=torch.float32, device=dev)
        hb.hb_meta_query_attn(self.H, Q, feats, v_proj.view(S, L, D), self.a_fold, self.residual_layers,
                              pre.view(S, Q, D), None if res is None else res.view(S, Q, D), ws)
        linear(pre, self.w_o, res, f_c)
        f_c = f_c.view(S, Q * D)
        out = bf(S, self.w_fc1.shape[0])
        linear(f_c, self.w_fc1, None, out)
        return f_c, out


def fc_concat(a, b, w_a, w_b):
    """fc over the concatenation [a, b]: a w_a^T + b w_b^T (w_a, w_b: the two column blocks of the
    layer's weight, stored as separate matrices)."""
    T = a.shape[0]
    tmp = torch.empty((T, w_a.shape[0]), dtype=torch.bfloat16, device=a.device)
    out = torch.empty_like(tmp)
    linear(a, w_a, None, tmp)
    linear(b, w_b, tmp, out)
    return out


def kv_compact(desc, dev: DeviceInputs, accept_len, accept_path):
    B, max_path = accept_path.shape
    out_slots = torch.empty((B, max_path), dtype=torch.int32, device=accept_path.device)
    new_len = torch.empty(B, dtype=torch.int32, device=accept_path.device)
    hb.hb_kv_compact(desc, dev.k_tree, dev.v_tree, dev.k_pool, dev.v_pool, dev.block_table, dev.prefix_len,
                     dev.node_offset, accept_len, accept_path, max_path, out_slots, new_len)
    return out_slots, new_len


class VerifyStep:
    """Pre-allocated buffers for one full verification step (attention of one layer, LM head,
    acceptance, compaction); ``run`` only enqueues kernels."""

    def __init__(self, desc: hb.AttnDesc, dev: DeviceInputs, weight: torch.Tensor, draft_ids: torch.Tensor,
                 max_path: int):
        self.desc, self.dev, self.weight, self.draft_ids, self.max_path = desc, dev, weight, draft_ids, max_path
        d = dev.q.device
        T, Hq, D = dev.q.shape
        B = desc.batch
        self.out = torch.empty_like(dev.q)
        self.ws_attn = alloc_workspace(hb.hb_tree_verify_attn_workspace_bytes(desc), d)
        self.ws_lm = alloc_workspace(max(8, hb.hb_lmhead_argmax_workspace_bytes(T)), d)
        self.target_ids = torch.empty(T, dtype=torch.int32, device=d)
        self.accept_len = torch.empty(B, dtype=torch.int32, device=d)
        self.accept_path = torch.empty((B, max_path), dtype=torch.int32, device=d)
        self.out_tokens = torch.empty((B, max_path), dtype=torch.int32, device=d)
        self.bonus = torch.empty(B, dtype=torch.int32, device=d)
        self.out_slots = torch.empty((B, max_path), dtype=torch.int32, device=d)
        self.new_len = torch.empty(B, dtype=torch.int32, device=d)

    def run(self, compact=True):
        dev, desc = self.dev, self.desc
        hb.hb_tree_verify_attn(desc, dev.q, dev.k_tree, dev.v_tree, dev.k_pool, dev.v_pool, dev.block_table,
                               dev.prefix_len, dev.node_offset, dev.parent, self.out, None, self.ws_attn)
        hidden = self.out.view(self.out.shape[0], -1)  # [T, Hq*D]: attention output feeds the LM head
        hb.hb_lmhead_argmax(hidden, self.weight, self.target_ids, None, self.ws_lm)
        hb.hb_tree_accept(desc.batch, desc.max_nodes_per_tree, dev.node_offset, dev.parent, self.draft_ids,
                          self.target_ids, self.max_path, self.accept_len, self.accept_path, self.out_tokens,
                          self.bonus)
        if compact:
            hb.hb_kv_compact(desc, dev.k_tree, dev.v_tree, dev.k_pool, dev.v_pool, dev.block_table,
                             dev.prefix_len, dev.node_offset, self.accept_len, self.accept_path, self.max_path,
                             self.out_slots, self.new_len)


class VerifyLayerStack:
    """Buffers and call chain of one verification step through ``n_layers`` decoder layers, then
    LM head with argmax, acceptance, and the append of the accepted nodes' K/V to every layer's
    pools.  Without ``mlp`` a layer is its attention half (QKV projection + rotary embedding ->
    tree-verify attention over that layer's KV pools -> output projection with residual).  With
    ``mlp = dict(norm1=[..], norm2=[..], w_gate_up=[..], w_down=[..], norm_f=.., eps=..)`` it is the
    whole pre-norm layer: RMSNorm in front of the attention half, then RMSNorm -> gated-SiLU
    projection -> down projection with residual, and a final RMSNorm in front of the LM head.
    ``run`` only enqueues kernels on the current stream (no allocation, no host synchronisation),
    so a step can be captured into a HIP graph once and replayed."""

    def __init__(self, desc: hb.AttnDesc, dev: DeviceInputs, pools, w_qkv, w_o, lm_weight, draft_ids, max_path: int,
                 hidden0: torch.Tensor, theta: float = 1e6, mlp=None):
        self.desc, self.dev, self.pools, self.w_qkv, self.w_o = desc, dev, pools, w_qkv, w_o
        self.lm_weight, self.draft_ids, self.max_path, self.theta = lm_weight, draft_ids, max_path, theta
        d = hidden0.device
        T, Hq, D = dev.q.shape
        Hkv = dev.k_tree.shape[1]
        B = desc.batch
        self.n_layers = len(pools)
        self.hidden = [hidden0] + [torch.empty_like(hidden0) for _ in range(2)]  # input, ping, pong
        self.mlp = mlp
        self.positions = torch.empty(T, dtype=torch.int32, device=d)
        self.cos = torch.empty((T, D // 2), dtype=torch.float32, device=d)
        self.sin = torch.empty_like(self.cos)
        self.q = torch.empty_like(dev.q)
        self.k_tree = [torch.empty_like(dev.k_tree) for _ in range(self.n_layers)]  # kept for the compaction
        self.v_tree = [torch.empty_like(dev.v_tree) for _ in range(self.n_layers)]
        self.attn_out = torch.empty_like(dev.q)
        self.ws_attn = alloc_workspace(hb.hb_tree_verify_attn_workspace_bytes(desc), d)
        self.ws_lm = alloc_workspace(max(8, hb.hb_lmhead_argmax_workspace_bytes(T)), d)
        K = hidden0.shape[1]
        proj_bytes = max(hb.hb_proj_workspace_bytes(T, K, w_qkv[0].shape[0]), hb.hb_proj_workspace_bytes(T, K, w_o[0].shape[0]))
        if mlp is not None:
            F = mlp["w_down"][0].shape[1]
            proj_bytes = max(proj_bytes, hb.hb_proj_workspace_bytes(T, K, 2 * F), hb.hb_proj_workspace_bytes(T, F, K))
            self.normed = torch.empty_like(hidden0)
            self.mid = torch.empty_like(hidden0)      # the layer's hidden state between its two halves
            self.act = torch.empty((T, F), dtype=hidden0.dtype, device=d)
        self.ws_proj = alloc_workspace(proj_bytes, d) if proj_bytes else None  # small token counts: split-K partials
        self.target_ids = torch.empty(T, dtype=torch.int32, device=d)
        self.accept_len = torch.empty(B, dtype=torch.int32, device=d)
        self.accept_path = torch.empty((B, max_path), dtype=torch.int32, device=d)
        self.out_tokens = torch.empty((B, max_path), dtype=torch.int32, device=d)
        self.bonus = torch.empty(B, dtype=torch.int32, device=d)
        self.out_slots = torch.empty((B, max_path), dtype=torch.int32, device=d)
        self.new_len = torch.empty(B, dtype=torch.int32, device=d)
        # tables of every layer's tensor addresses, for the compaction of all layers in one launch
        table = lambda ts: torch.tensor([t.data_ptr() for t in ts], dtype=torch.int64, device=d)
        self.ptr_tables = (table(self.k_tree), table(self.v_tree), table([p[0] for p in pools]),
                           table([p[1] for p in pools]))

    def run(self, compact=True, on_call=None):
        """``on_call(name)`` (optional) is invoked before every library call, e.g. to record events."""
        dev, desc = self.dev, self.desc
        T = self.q.shape[0]
        mark = on_call or (lambda name: None)
        mark("positions")
        hb.hb_tree_positions(desc.batch, desc.max_nodes_per_tree, dev.node_offset, dev.parent, dev.prefix_len,
                             self.positions)
        hb.hb_rope_table(self.q.shape[2], self.theta, self.positions, self.cos, self.sin)
        x = self.hidden[0]
        mlp = self.mlp
        for l in range(self.n_layers):
            nxt = self.hidden[1 + (l & 1)]
            y = nxt if mlp is None else self.mid
            kp, vp = self.pools[l]
            a = x
            if mlp is not None:
                mark("rmsnorm")
                hb.hb_rmsnorm(x, mlp["norm1"][l], mlp["eps"], self.normed)
                a = self.normed
            mark("qkv_rope_project")
            hb.hb_qkv_rope_project_ws(a, self.w_qkv[l], None, self.cos, self.sin, self.q, self.k_tree[l],
                                      self.v_tree[l], self.ws_proj)
            mark("tree_verify_attn")
            hb.hb_tree_verify_attn(desc, self.q, self.k_tree[l], self.v_tree[l], kp, vp, dev.block_table,
                                   dev.prefix_len, dev.node_offset, dev.parent, self.attn_out, None, self.ws_attn)
            mark("out_project")
            hb.hb_out_project_ws(self.attn_out.view(T, -1), self.w_o[l], x, y, self.ws_proj)
            if mlp is not None:
                mark("rmsnorm")
                hb.hb_rmsnorm(y, mlp["norm2"][l], mlp["eps"], self.normed)
                mark("swiglu_project")
                hb.hb_swiglu_project(self.normed, mlp["w_gate_up"][l], self.act, self.ws_proj)
                mark("down_project")
                hb.hb_out_project_ws(self.act, mlp["w_down"][l], y, nxt, self.ws_proj)
            x = nxt
        if mlp is not None and mlp.get("norm_f") is not None:
            mark("rmsnorm")
            hb.hb_rmsnorm(x, mlp["norm_f"], mlp["eps"], self.normed)
            x = self.normed
        self.final_hidden = x
        mark("lmhead_argmax")
        hb.hb_lmhead_argmax(x, self.lm_weight, self.target_ids, None, self.ws_lm)
        mark("tree_accept")
        hb.hb_tree_accept(desc.batch, desc.max_nodes_per_tree, dev.node_offset, dev.parent, self.draft_ids,
                          self.target_ids, self.max_path, self.accept_len, self.accept_path, self.out_tokens,
                          self.bonus)
        if compact:
            mark("kv_compact")
            hb.hb_kv_compact_layers(desc, self.n_layers, *self.ptr_tables, dev.block_table, dev.prefix_len,
                                    dev.node_offset, self.accept_len, self.accept_path, self.max_path,
                                    self.out_slots, self.new_len)
        mark("end")
