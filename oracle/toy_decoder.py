"""A small random-weight decoder and two ways of decoding it greedily (oracle, float64).

The paper's claim for the understanding side (Section 1; Section 4.1 "Setup") is that
verification by the target leaves its outputs untouched.  Under greedy decoding this means:
speculative decoding, whatever the drafts are, emits exactly the token stream of plain
autoregressive decoding.  ``greedy_ar`` is the plain stream; ``spec_decode`` is the
draft-verify-accept-compact loop assembled from the four oracle functions of this package.

Model: pre-norm decoder layers (RMSNorm, rotary grouped-query attention, gated-SiLU MLP), a
final RMSNorm and an untied LM head.  A tree node at depth d below the pending token sits at
position L + d, L being the number of cached positions.
"""
from __future__ import annotations

import numpy as np

from .tree_attention import tree_attn_ref
from .lm_head import lmhead_argmax_ref
from .acceptance import tree_accept_ref
from .kv_compaction import kv_compact_ref

_EPS = 1e-6


def _rms_norm(x, gain):
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + _EPS) * gain


def _rope(x, pos, base):
    """Rotary embedding, rotate-half convention.  x [..., T, H, Dh], pos [T]."""
    dh = x.shape[-1]
    half = dh // 2
    inv = base ** (-np.arange(half) / half)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * inv[None, :]  # [T, half]
    cos, sin = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * cos - x2 * sin, x2 * cos + x1 * sin], axis=-1)


def _silu(x):
    return x / (1.0 + np.exp(-x))


def round_bf16(x):
    """Round float64 values to the nearest bfloat16 (ties to even), returned as float64: the
    rounding a bf16 kernel interface applies to what it is handed."""
    f = np.asarray(x, dtype=np.float64).astype(np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(np.float64)


class ToyDecoderRef:
    def __init__(self, w, quant=None, quant_dense=None):
        """``quant`` (optional, default identity) is applied where a decoder that keeps its
        attention inputs, attention output and LM-head input in a narrower storage type rounds
        them: to q, k, v after the rotary embedding, to the attention output, and to the
        normalised hidden state that feeds the LM head.  With ``round_bf16`` the three decoding
        modes below describe such a bf16 decoder exactly, in float64 arithmetic.
        ``quant_dense`` (optional, default identity) is applied where a decoder whose dense
        layers hand narrower tensors on as well rounds: to both normalised hidden states of a
        layer, to the hidden state after each residual addition, and to the gated activation."""
        self.w = w
        self.quant = quant if quant is not None else (lambda a: a)
        self.qd = quant_dense if quant_dense is not None else (lambda a: a)

    # -- pieces shared by every decoding mode (plain per-token maths) ---------------------
    def _qkv(self, layer, x, pos):
        w = self.w
        h = self.qd(_rms_norm(x, w.norm1[layer]))
        T = x.shape[0]
        q = (h @ w.wq[layer]).reshape(T, w.Hq, w.Dh)
        k = (h @ w.wk[layer]).reshape(T, w.Hkv, w.Dh)
        v = (h @ w.wv[layer]).reshape(T, w.Hkv, w.Dh)
        qt = self.quant
        return qt(_rope(q, pos, w.rope_base)), qt(_rope(k, pos, w.rope_base)), qt(v)

    def _after_attn(self, layer, x, attn):
        w = self.w
        attn = self.quant(attn)
        qd = self.qd
        x = qd(x + attn.reshape(x.shape[0], -1) @ w.wo[layer])
        h = qd(_rms_norm(x, w.norm2[layer]))
        return qd(x + qd(_silu(h @ w.w_gate[layer]) * (h @ w.w_up[layer])) @ w.w_down[layer])

    def _logits(self, x):
        return self.quant(_rms_norm(x, self.w.norm_f)) @ self.w.lm_head.T

    # -- reference 1: whole-sequence causal forward, no cache ----------------------------
    def full_forward(self, tokens):
        """Logits at every position of ``tokens`` with ordinary causal attention."""
        w = self.w
        T = len(tokens)
        pos = np.arange(T)
        x = w.embed[np.asarray(tokens)]
        G = w.Hq // w.Hkv
        scale = 1.0 / np.sqrt(w.Dh)
        for layer in range(w.n_layers):
            q, k, v = self._qkv(layer, x, pos)
            attn = np.zeros((T, w.Hq, w.Dh))
            for t in range(T):
                for h in range(w.Hq):
                    s = scale * (k[: t + 1, h // G] @ q[t, h])
                    p = np.exp(s - s.max())
                    attn[t, h] = (p / p.sum()) @ v[: t + 1, h // G]
            x = self._after_attn(layer, x, attn)
        return self._logits(x)

    # -- reference 2: plain greedy autoregressive decoding with a KV cache ----------------
    def _decode_one(self, token, pos, cache):
        w = self.w
        G = w.Hq // w.Hkv
        scale = 1.0 / np.sqrt(w.Dh)
        x = w.embed[np.asarray([token])]
        for layer in range(w.n_layers):
            q, k, v = self._qkv(layer, x, [pos])
            cache[layer][0].append(k[0])
            cache[layer][1].append(v[0])
            ks, vs = np.stack(cache[layer][0]), np.stack(cache[layer][1])  # [pos+1, Hkv, Dh]
            attn = np.zeros((1, w.Hq, w.Dh))
            for h in range(w.Hq):
                s = scale * (ks[:, h // G] @ q[0, h])
                p = np.exp(s - s.max())
                attn[0, h] = (p / p.sum()) @ vs[:, h // G]
            x = self._after_attn(layer, x, attn)
        return self._logits(x)[0]

    def greedy_ar(self, prompt, n_new):
        """Returns (generated tokens, smallest top-1 minus top-2 logit margin met on the way)."""
        cache = [([], []) for _ in range(self.w.n_layers)]
        logits = None
        for p, tok in enumerate(prompt):
            logits = self._decode_one(int(tok), p, cache)
        out, min_margin = [], np.inf
        pos = len(prompt)
        for _ in range(n_new):
            top = np.sort(logits)[-2:]
            min_margin = min(min_margin, float(top[1] - top[0]))
            tok = int(np.argmax(logits))
            out.append(tok)
            logits = self._decode_one(tok, pos, cache)
            pos += 1
        return out, min_margin

    # -- greedy speculative decoding from the four verification functions -----------------
    def spec_decode(self, prompt, n_new, drafter, tree_for_step, block_table, page=16):
        """Draft-verify-accept-compact loop for one sequence.

        ``drafter(committed_tokens, parent)`` returns draft ids for every node (entry 0 is
        ignored: the root is the pending committed token).  ``tree_for_step(step)`` returns the
        parent array of that step.  ``block_table`` int32 [1, max_blocks] maps the sequence's
        pages into pools of ``block_table.max()+1`` pages.  Returns (tokens, accept_lens)."""
        w = self.w
        block_table = np.asarray(block_table, dtype=np.int32).reshape(1, -1)
        n_blocks = int(block_table.max()) + 1
        pools = [(np.zeros((n_blocks, w.Hkv, page, w.Dh)), np.zeros((n_blocks, w.Hkv, page, w.Dh)))
                 for _ in range(w.n_layers)]
        scale = 1.0 / np.sqrt(w.Dh)

        # prefill all prompt tokens but the last with ordinary decode steps, then page them in
        cache = [([], []) for _ in range(w.n_layers)]
        for p, tok in enumerate(prompt[:-1]):
            self._decode_one(int(tok), p, cache)
        L = len(prompt) - 1
        for layer in range(w.n_layers):
            for p in range(L):
                blk = block_table[0, p // page]
                pools[layer][0][blk, :, p % page] = cache[layer][0][p]
                pools[layer][1][blk, :, p % page] = cache[layer][1][p]

        toks = [int(t) for t in prompt]
        out, accept_lens, step = [], [], 0
        while len(out) < n_new:
            parent = np.asarray(tree_for_step(step), dtype=np.int32)
            n = parent.shape[0]
            depth = np.zeros(n, dtype=np.int64)
            for i in range(1, n):
                depth[i] = depth[parent[i]] + 1
            max_path = int(depth.max()) + 1
            draft_ids = np.asarray(drafter(list(toks), parent), dtype=np.int32).copy()
            draft_ids[0] = toks[-1]
            node_offset = np.array([0, n], dtype=np.int32)
            prefix_len = np.array([L], dtype=np.int32)
            x = w.embed[draft_ids]
            tree_kv = []
            for layer in range(w.n_layers):
                q, k, v = self._qkv(layer, x, L + depth)
                attn, _ = tree_attn_ref(q, k, v, pools[layer][0], pools[layer][1], block_table,
                                        prefix_len, node_offset, parent, scale)
                tree_kv.append((k, v))
                x = self._after_attn(layer, x, attn)
            hidden = self.quant(_rms_norm(x, w.norm_f))
            target_ids, _ = lmhead_argmax_ref(hidden, w.lm_head)
            alen, apath, otoks, _ = tree_accept_ref(node_offset, parent, draft_ids, target_ids, max_path)
            for layer in range(w.n_layers):
                kp, vp, _, new_len = kv_compact_ref(tree_kv[layer][0], tree_kv[layer][1],
                                                    pools[layer][0], pools[layer][1], block_table,
                                                    prefix_len, node_offset, alen, apath)
                pools[layer] = (kp, vp)
            emitted = [int(t) for t in otoks[0, : int(alen[0])]]
            toks.extend(emitted)
            out.extend(emitted)
            accept_lens.append(int(alen[0]))
            L = int(new_len[0])
            step += 1
        return out[:n_new], accept_lens
