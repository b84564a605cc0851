"""Greedy speculative decoding of the toy decoder with the verification step on the GPU.

The decoder's dense layers (embedding, RMSNorm, projections, rotary, MLP) run as ordinary
torch fp32 ops on the device; attention, LM-head argmax, acceptance and KV compaction go
through the C ABI.  With dtype "bf16_all" the dense layers go through the C ABI as well
(hb_rmsnorm, hb_rope_table + hb_qkv_rope_project, hb_out_project, hb_swiglu_project): only the
embedding lookup is left to torch.  Written independently of the oracle's decoder."""
import math

import numpy as np
import torch

import paper_2509_18824_amd as hb
import paper_2509_18824_amd.step as S


class ToyDecoderGpu:
    def __init__(self, w, page=16, n_blocks=16, device="cuda", dtype="f32"):
        """dtype "bf16": q, k, v, the KV pools, the attention output and the LM head's inputs are
        bf16 (the matrix-core kernels run); everything between the library calls stays fp32."""
        self.w, self.page, self.n_blocks, self.dev = w, page, n_blocks, device
        self.all_bf16 = dtype == "bf16_all"
        self.dtype = dtype = "bf16" if self.all_bf16 else dtype
        self.tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
        f = lambda a: torch.tensor(a, dtype=torch.float32, device=device)
        self.embed = f(w.embed)
        self.layers = [dict(wq=f(w.wq[i]), wk=f(w.wk[i]), wv=f(w.wv[i]), wo=f(w.wo[i]), wg=f(w.w_gate[i]),
                            wu=f(w.w_up[i]), wd=f(w.w_down[i]), n1=f(w.norm1[i]), n2=f(w.norm2[i]))
                       for i in range(w.n_layers)]
        self.norm_f = f(w.norm_f)
        self.lm_head = f(w.lm_head).to(self.tdt).contiguous()
        if self.all_bf16:
            b = lambda a: f(np.ascontiguousarray(a)).to(torch.bfloat16).contiguous()
            self.embed = b(w.embed)
            self.norm_f = b(w.norm_f)
            self.layers = [dict(wqkv=b(np.concatenate([w.wq[i].T, w.wk[i].T, w.wv[i].T], axis=0)), wo=b(w.wo[i].T),
                                wgu=b(np.concatenate([w.w_gate[i].T, w.w_up[i].T], axis=0)), wd=b(w.w_down[i].T),
                                n1=b(w.norm1[i]), n2=b(w.norm2[i])) for i in range(w.n_layers)]
        half = w.Dh // 2
        self.inv_freq = torch.tensor([w.rope_base ** (-i / half) for i in range(half)], dtype=torch.float64,
                                     device=device)

    @staticmethod
    def _rms(x, g):
        return x * torch.rsqrt((x * x).mean(-1, keepdim=True) + 1e-6) * g

    def _rope(self, x, pos):
        ang = pos.to(torch.float64)[:, None] * self.inv_freq[None, :]
        cos, sin = ang.cos().float()[:, None, :], ang.sin().float()[:, None, :]
        half = x.shape[-1] // 2
        a, b = x[..., :half], x[..., half:]
        return torch.cat([a * cos - b * sin, b * cos + a * sin], dim=-1)

    def _qkv(self, lw, x, pos):
        w = self.w
        if self.all_bf16:
            T = x.shape[0]
            bf = lambda *shape: torch.empty(shape, dtype=torch.bfloat16, device=x.device)
            h, q, k, v = bf(T, w.d), bf(T, w.Hq, w.Dh), bf(T, w.Hkv, w.Dh), bf(T, w.Hkv, w.Dh)
            cos = torch.empty((T, w.Dh // 2), dtype=torch.float32, device=x.device)
            sin = torch.empty_like(cos)
            hb.hb_rmsnorm(x, lw["n1"], 1e-6, h)
            hb.hb_rope_table(w.Dh, w.rope_base, pos.to(torch.int32).contiguous(), cos, sin)
            hb.hb_qkv_rope_project(h, lw["wqkv"], None, cos, sin, q, k, v)
            return q, k, v
        h = self._rms(x, lw["n1"])
        T = x.shape[0]
        q = self._rope((h @ lw["wq"]).view(T, w.Hq, w.Dh), pos)
        k = self._rope((h @ lw["wk"]).view(T, w.Hkv, w.Dh), pos)
        v = (h @ lw["wv"]).view(T, w.Hkv, w.Dh)
        return q.to(self.tdt).contiguous(), k.to(self.tdt).contiguous(), v.to(self.tdt).contiguous()

    def _mlp(self, lw, x, attn):
        if self.all_bf16:
            T = x.shape[0]
            y, h, out = torch.empty_like(x), torch.empty_like(x), torch.empty_like(x)
            act = torch.empty((T, self.w.ffn), dtype=torch.bfloat16, device=x.device)
            hb.hb_out_project(attn.reshape(T, -1).contiguous(), lw["wo"], x, y)
            hb.hb_rmsnorm(y, lw["n2"], 1e-6, h)
            hb.hb_swiglu_project(h, lw["wgu"], act)
            hb.hb_out_project(act, lw["wd"], y, out)
            return out
        x = x + attn.float().reshape(x.shape[0], -1) @ lw["wo"]
        h = self._rms(x, lw["n2"])
        return x + (torch.nn.functional.silu(h @ lw["wg"]) * (h @ lw["wu"])) @ lw["wd"]

    def spec_decode(self, prompt, n_new, drafter, tree_for_step, block_table, algo=0, tree_builder=None):
        """tree_builder(step, tokens) -> (parent, draft_ids), when given, replaces the pair
        (tree_for_step, drafter): the tree's shape then comes with its tokens."""
        w, dev, page = self.w, self.dev, self.page
        bt = torch.tensor(np.asarray(block_table).reshape(1, -1), dtype=torch.int32, device=dev)
        pools = [(torch.zeros((self.n_blocks, w.Hkv, page, w.Dh), device=dev, dtype=self.tdt),
                  torch.zeros((self.n_blocks, w.Hkv, page, w.Dh), device=dev, dtype=self.tdt)) for _ in self.layers]
        toks = [int(t) for t in prompt]
        L = 0  # cached positions
        prefix_len = torch.zeros(1, dtype=torch.int32, device=dev)
        scale = 1.0 / math.sqrt(w.Dh)
        out, lens, step = [], [], 0
        # The prompt (all but its last token) is prefilled through the same verify path as chains
        # of up to 32 nodes whose "drafts" are the known prompt tokens: all of them are accepted
        # by construction of the cache update below (no acceptance test involved in prefill).
        pending = toks[:-1]
        while pending:
            chunk, pending = pending[:32], pending[32:]
            n = len(chunk)
            parent = torch.arange(-1, n - 1, dtype=torch.int32, device=dev)
            node_offset = torch.tensor([0, n], dtype=torch.int32, device=dev)
            ids = torch.tensor(chunk, device=dev)
            x = self.embed[ids]
            pos = torch.arange(L, L + n, device=dev)
            alen = torch.tensor([n], dtype=torch.int32, device=dev)
            apath = torch.arange(n, dtype=torch.int32, device=dev).view(1, n).contiguous()
            for lw, (kp, vp) in zip(self.layers, pools):
                q, k, v = self._qkv(lw, x, pos)
                desc = S.make_desc(self.dtype, 1, w.Hq, w.Hkv, w.Dh, page, bt.shape[1], self.n_blocks, n, n, scale,
                                   algo=algo)
                d = S.DeviceInputs(q, k, v, kp, vp, bt, prefix_len, node_offset, parent)
                attn, _ = S.tree_verify_attn(desc, d, want_lse=False)
                S.kv_compact(desc, d, alen, apath)
                x = self._mlp(lw, x, attn)
            L += n
            prefix_len.fill_(L)
        while len(out) < n_new:
            built = tree_builder(step, list(toks)) if tree_builder is not None else None
            par_np = np.asarray(built[0] if built is not None else tree_for_step(step), dtype=np.int32)
            n = len(par_np)
            depth = np.zeros(n, dtype=np.int64)
            for i in range(1, n):
                depth[i] = depth[par_np[i]] + 1
            max_path = int(depth.max()) + 1
            draft = np.asarray(built[1] if built is not None else drafter(list(toks), par_np), dtype=np.int32).copy()
            draft[0] = toks[-1]
            parent = torch.from_numpy(par_np).to(dev)
            node_offset = torch.tensor([0, n], dtype=torch.int32, device=dev)
            draft_ids = torch.from_numpy(draft).to(dev)
            x = self.embed[draft_ids.long()]
            pos = torch.from_numpy(L + depth).to(dev)
            desc = S.make_desc(self.dtype, 1, w.Hq, w.Hkv, w.Dh, page, bt.shape[1], self.n_blocks, n, n, scale, algo=algo)
            tree_kv = []
            for lw, (kp, vp) in zip(self.layers, pools):
                q, k, v = self._qkv(lw, x, pos)
                d = S.DeviceInputs(q, k, v, kp, vp, bt, prefix_len, node_offset, parent)
                attn, _ = S.tree_verify_attn(desc, d, want_lse=False)
                tree_kv.append(d)
                x = self._mlp(lw, x, attn)
            if self.all_bf16:
                hidden = torch.empty_like(x)
                hb.hb_rmsnorm(x, self.norm_f, 1e-6, hidden)
            else:
                hidden = self._rms(x, self.norm_f).to(self.tdt).contiguous()
            target_ids, _ = S.lmhead_argmax(hidden, self.lm_head, want_max=False)
            alen, apath, otoks, _ = S.tree_accept(node_offset, parent, draft_ids, target_ids, max_path, n)
            new_len = None
            for d in tree_kv:
                _, new_len = S.kv_compact(desc, d, alen, apath)
            k = int(alen.item())
            emitted = otoks[0, :k].tolist()
            toks.extend(emitted)
            out.extend(emitted)
            lens.append(k)
            L = int(new_len.item())
            prefix_len.fill_(L)
            step += 1
        return out[:n_new], lens
