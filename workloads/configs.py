"""Seeded input tensors for the five verification workloads and for the toy decoder.

Everything here is drawn from explicit seeds.  One generator stream serves each kind of
quantity (lengths, span map, page permutation, trees, Q, K, V, ids) so that changing one does
not shift the others.  The tensors are torch CPU tensors in the storage dtype of the workload
(fp32 or bf16); ``widen`` turns them into float64 / int64 numpy arrays without rounding.

Workload structure (stand-in for the paper's understanding workload, Section 3.1.1 and
Section 4.1 "Setup": a context in which text, ViT-image and prefilled clean-latent positions are
interleaved): every prefix carries a seeded map of image spans, and K/V drawn inside an image span
get a span-specific gain and offset, mimicking modality-dependent statistics.  The span map is
never an input of the verification step: every draft node is a text position that attends to the
whole prefix.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np
import torch

from .trees import chain_tree, seeded_tree, tree_depths

CONFIG_NAMES = (
    "cfg0_tiny_fp32_chain4",
    "cfg1_single_seq_bf16",
    "cfg2_ragged_batch16_bf16",
    "cfg3_long_context_32k_bf16",
    "cfg4_full_step_batch16_bf16",
)

_TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}


def widen(t):
    """Exact widening of a torch tensor to numpy (float64 for floating point, int64 for ints)."""
    if isinstance(t, np.ndarray):
        return t.astype(np.float64) if t.dtype.kind == "f" else t.astype(np.int64)
    t = t.detach().cpu()
    if t.is_floating_point():
        return t.to(torch.float64).numpy()
    return t.to(torch.int64).numpy()


@dataclass
class VerifyInputs:
    """One batch of inputs for a verification step (one attention layer)."""

    name: str
    dtype: str  # "f32" or "bf16"
    B: int
    Hq: int
    Hkv: int
    D: int
    page: int
    max_blocks: int
    num_blocks: int
    softmax_scale: float
    max_path: int  # longest root-to-leaf path (in nodes) over the batch
    q: torch.Tensor  # [total_nodes, Hq, D]
    k_tree: torch.Tensor  # [total_nodes, Hkv, D]
    v_tree: torch.Tensor  # [total_nodes, Hkv, D]
    k_pool: torch.Tensor  # [num_blocks, Hkv, page, D]
    v_pool: torch.Tensor  # [num_blocks, Hkv, page, D]
    block_table: torch.Tensor  # int32 [B, max_blocks]
    prefix_len: torch.Tensor  # int32 [B]
    node_offset: torch.Tensor  # int32 [B+1]
    parent: torch.Tensor  # int32 [total_nodes], tree-local
    poison_block: int
    spans: List[List[Tuple[int, int]]] = field(default_factory=list)  # image spans per sequence

    @property
    def total_nodes(self) -> int:
        return int(self.node_offset[-1])

    def trees(self) -> List[np.ndarray]:
        off = self.node_offset.numpy()
        par = self.parent.numpy()
        return [par[off[b]:off[b + 1]].copy() for b in range(self.B)]

    def kv_bytes(self) -> int:
        """Bytes of K and V the step must read once: every prefix position and tree node."""
        esz = 4 if self.dtype == "f32" else 2
        toks = int(self.prefix_len.sum()) + self.total_nodes
        return toks * self.Hkv * self.D * esz * 2


def _image_spans(rng: np.random.Generator, L: int, frac_lo: float, frac_hi: float,
                 n_spans: Optional[int] = None, interleave_equal: bool = False):
    """Seeded image spans covering a fraction of [0, L) (not page aligned)."""
    if L <= 0:
        return []
    if interleave_equal:
        # n_spans image spans of equal length separated by text of equal length
        n = n_spans or 1
        img = int(frac_lo * L) // n
        gap = (L - img * n) // n
        spans, pos = [], 0
        for _ in range(n):
            spans.append((pos, pos + img))
            pos += img + gap
        return spans
    frac = rng.uniform(frac_lo, frac_hi)
    n = n_spans or int(rng.integers(1, 5))
    total_img = int(frac * L)
    if total_img < n:
        return []
    cuts = np.sort(rng.choice(np.arange(1, total_img), size=n - 1, replace=False)) if n > 1 else []
    img_lens = np.diff(np.concatenate(([0], cuts, [total_img]))).astype(int)
    text_total = L - total_img
    tcuts = np.sort(rng.integers(0, text_total + 1, size=n))
    gaps = np.diff(np.concatenate(([0], tcuts))).astype(int)
    spans, pos = [], 0
    for g, ln in zip(gaps, img_lens):
        pos += int(g)
        spans.append((pos, pos + int(ln)))
        pos += int(ln)
    return spans


def make_verify_inputs(
    seed: int,
    dtype: str,
    Hq: int,
    Hkv: int,
    D: int,
    prefix_lens: Sequence[int],
    trees: Sequence[np.ndarray],
    page: int = 16,
    kv_std: float = 1.0,
    q_std: float = 1.0,
    softmax_scale: Optional[float] = None,
    image_frac: Tuple[float, float] = (0.3, 0.7),
    n_spans: Optional[int] = None,
    interleave_equal: bool = False,
    permute_blocks: bool = True,
    poison: bool = True,
    peaked: bool = False,
    spare_blocks: int = 3,
    name: str = "custom",
) -> VerifyInputs:
    """Build one batch.  ``prefix_lens[b]`` tokens of prefix KV and one tree per sequence.

    Pages: each sequence maps ``ceil((L_b + max_path) / page)`` pages (room for the accepted
    path to be appended); every other table entry points at one shared *poison* page.  With
    ``poison`` the poison page, the spare pages, and every slot at or beyond ``L_b`` hold NaN,
    so that any read of a position that must not influence the result shows up in the output.
    """
    tdt = _TORCH_DTYPE[dtype]
    B = len(prefix_lens)
    assert B == len(trees) and Hq % Hkv == 0
    rng_struct = np.random.default_rng(seed * 16 + 1)  # span maps
    rng_perm = np.random.default_rng(seed * 16 + 2)  # page permutation
    gq = torch.Generator().manual_seed(seed * 16 + 3)
    gk = torch.Generator().manual_seed(seed * 16 + 4)
    gv = torch.Generator().manual_seed(seed * 16 + 5)
    rng_peak = np.random.default_rng(seed * 16 + 6)

    node_offset = np.zeros(B + 1, dtype=np.int32)
    for b, t in enumerate(trees):
        node_offset[b + 1] = node_offset[b] + len(t)
    total_nodes = int(node_offset[-1])
    parent = (np.concatenate([np.asarray(t, dtype=np.int32) for t in trees]).astype(np.int32)
              if B else np.zeros(0, np.int32))
    max_path = max((int(tree_depths(t).max()) + 1 for t in trees if len(t)), default=1)

    pages_per_seq = [-(-(int(L) + max_path) // page) for L in prefix_lens]
    max_blocks = max(pages_per_seq, default=1) + 1  # at least one unmapped entry per row
    num_blocks = sum(pages_per_seq) + 1 + spare_blocks
    ids = rng_perm.permutation(num_blocks) if permute_blocks else np.arange(num_blocks)
    poison_block = int(ids[sum(pages_per_seq)])
    block_table = np.full((B, max_blocks), poison_block, dtype=np.int32)
    cursor = 0
    for b, n in enumerate(pages_per_seq):
        block_table[b, :n] = ids[cursor:cursor + n]
        cursor += n

    fill = float("nan") if poison else 0.0
    k_pool = torch.full((num_blocks, Hkv, page, D), fill, dtype=torch.float32)
    v_pool = torch.full((num_blocks, Hkv, page, D), fill, dtype=torch.float32)
    spans_all = []
    for b, L in enumerate(prefix_lens):
        L = int(L)
        spans = _image_spans(rng_struct, L, image_frac[0], image_frac[1], n_spans, interleave_equal)
        spans_all.append(spans)
        if L == 0:
            continue
        k = torch.randn((L, Hkv, D), generator=gk) * kv_std
        v = torch.randn((L, Hkv, D), generator=gv) * kv_std
        for (s, e) in spans:
            # image positions: span-specific gain/offset (modality-dependent statistics)
            gain = float(rng_struct.uniform(0.8, 1.25))
            shift = float(rng_struct.uniform(-0.1, 0.1)) * kv_std
            k[s:e] = k[s:e] * gain + shift
            v[s:e] = v[s:e] * gain - shift
        npg = -(-L // page)
        pad = npg * page - L
        if pad:
            padt = torch.full((pad, Hkv, D), fill)
            k = torch.cat([k, padt])
            v = torch.cat([v, padt])
        phys = torch.from_numpy(block_table[b, :npg].astype(np.int64))
        k_pool[phys] = k.view(npg, page, Hkv, D).permute(0, 2, 1, 3)
        v_pool[phys] = v.view(npg, page, Hkv, D).permute(0, 2, 1, 3)

    q = torch.randn((total_nodes, Hq, D), generator=gq) * q_std
    k_tree = torch.randn((total_nodes, Hkv, D), generator=gk) * kv_std
    v_tree = torch.randn((total_nodes, Hkv, D), generator=gv) * kv_std
    scale = float(softmax_scale) if softmax_scale is not None else 1.0 / float(np.sqrt(D))

    if peaked:
        # Plant a few anchor keys per (sequence, kv head) and steer every query towards one of
        # them, so the softmax is concentrated and |o| = O(1) instead of a near-uniform average.
        G = Hq // Hkv
        r_k = kv_std * float(np.sqrt(D))  # the norm of a typical key
        r_q = 12.0 / (scale * r_k)  # planted score = scale * r_q * r_k = 12
        for b, L in enumerate(prefix_lens):
            L = int(L)
            n0, n1 = int(node_offset[b]), int(node_offset[b + 1])
            if L == 0 or n1 == n0:
                continue
            n_anchor = min(8, L)
            for h in range(Hkv):
                pos = rng_peak.choice(L, size=n_anchor, replace=False)
                dirs = torch.from_numpy(rng_peak.standard_normal((n_anchor, D))).float()
                dirs = dirs / dirs.norm(dim=1, keepdim=True)
                for a, p in enumerate(pos):
                    blk = int(block_table[b, p // page])
                    k_pool[blk, h, p % page] = dirs[a] * r_k
                for i in range(n0, n1):
                    for g in range(G):
                        a = int(rng_peak.integers(0, n_anchor))
                        q[i, h * G + g] += dirs[a] * r_q

    return VerifyInputs(
        name=name, dtype=dtype, B=B, Hq=Hq, Hkv=Hkv, D=D, page=page, max_blocks=max_blocks,
        num_blocks=num_blocks, softmax_scale=scale, max_path=max_path,
        q=q.to(tdt), k_tree=k_tree.to(tdt), v_tree=v_tree.to(tdt),
        k_pool=k_pool.to(tdt), v_pool=v_pool.to(tdt),
        block_table=torch.from_numpy(block_table), prefix_len=torch.tensor(list(prefix_lens), dtype=torch.int32),
        node_offset=torch.from_numpy(node_offset), parent=torch.from_numpy(parent),
        poison_block=poison_block, spans=spans_all,
    )


def make_config(cfg: int, peaked: bool = False, seed_shift: int = 0, tree: str = "tree",
                scale_down: int = 1) -> VerifyInputs:
    """The attention inputs of workload ``cfg`` (0..4).

    ``tree="chain8"`` swaps every 60-node tree for an 8-node chain (the comparison run of the
    full-step workload).  ``scale_down`` divides the prefix lengths (for quick CPU-sized copies
    of the big workloads with the same structure)."""
    seed = 1000 * cfg + seed_shift
    rng_len = np.random.default_rng(seed * 16 + 7)

    def trees_for(B):
        if tree == "chain8":
            return [chain_tree(8) for _ in range(B)]
        return [seeded_tree(seed * 64 + b) for b in range(B)]

    if cfg == 0:
        return make_verify_inputs(seed, "f32", 4, 1, 64, [256 // scale_down], [chain_tree(4)],
                                  kv_std=1.0, q_std=1.0, peaked=peaked, name=CONFIG_NAMES[0])
    if cfg == 1:
        # 2048 = 1024 image positions + 1024 text positions
        return make_verify_inputs(seed, "bf16", 28, 4, 128, [2048 // scale_down], trees_for(1),
                                  kv_std=0.5, q_std=0.5, image_frac=(0.5, 0.5),
                                  peaked=peaked, name=CONFIG_NAMES[1])
    if cfg == 2:
        lens = [int(x) // scale_down for x in rng_len.integers(1024, 8193, size=16)]
        return make_verify_inputs(seed, "bf16", 28, 4, 128, lens, trees_for(16),
                                  kv_std=1.0, q_std=1.0 / np.sqrt(128.0), softmax_scale=1.0,
                                  image_frac=(0.3, 0.7), peaked=peaked, name=CONFIG_NAMES[2])
    if cfg == 3:
        # eight 4096-token image spans interleaved with text: 32768 positions in all
        L = 32768 // scale_down
        return make_verify_inputs(seed, "bf16", 28, 4, 128, [L, L], trees_for(2),
                                  kv_std=1.0, q_std=1.0, image_frac=(0.5, 0.5), n_spans=8,
                                  interleave_equal=True, peaked=peaked, name=CONFIG_NAMES[3])
    if cfg == 4:
        lens = [int(x) // scale_down for x in rng_len.integers(1024, 4097, size=16)]
        return make_verify_inputs(seed, "bf16", 28, 4, 128, lens, trees_for(16),
                                  kv_std=1.0, q_std=1.0, image_frac=(0.3, 0.7),
                                  peaked=peaked, name=CONFIG_NAMES[4])
    raise ValueError("cfg must be 0..4")


def make_lmhead_inputs(seed: int, M: int, K: int, V: int, dtype: str = "bf16",
                       w_std: float = 0.02, h_std: float = 1.0, hidden: Optional[torch.Tensor] = None):
    """Hidden states [M, K] (drawn here unless given) and LM-head weight [V, K] ~ N(0, w_std)."""
    tdt = _TORCH_DTYPE[dtype]
    gw = torch.Generator().manual_seed(seed * 16 + 8)
    gh = torch.Generator().manual_seed(seed * 16 + 9)
    weight = torch.empty((V, K), dtype=tdt)
    step = max(1, (1 << 26) // max(K, 1))
    for v0 in range(0, V, step):
        v1 = min(V, v0 + step)
        weight[v0:v1] = (torch.randn((v1 - v0, K), generator=gw) * w_std).to(tdt)
    if hidden is None:
        hidden = (torch.randn((M, K), generator=gh) * h_std).to(tdt)
    return hidden, weight


def plant_draft_ids(seed: int, trees: Sequence[np.ndarray], target_ids: np.ndarray, vocab: int,
                    want_depth: Optional[Sequence[int]] = None, root_ids: Optional[Sequence[int]] = None):
    """Draft token ids for a batch of trees such that, per sequence, the draft agrees with the
    given target ids along one seeded root-to-node path of a seeded depth and disagrees
    everywhere else; sibling ids are distinct.  Returns (draft_ids int32[total], planted_depths).

    ``target_ids[node_offset[b] + i]`` is the target's choice for the token after node i.  A
    non-root node agrees when its id equals the target's choice at its parent."""
    rng = np.random.default_rng(seed * 16 + 10)
    out, planted = [], []
    off = 0
    for b, par in enumerate(trees):
        n = len(par)
        depth = tree_depths(par)
        tgt = np.asarray(target_ids[off:off + n]).astype(np.int64)
        d_want = int(want_depth[b]) if want_depth is not None else int(rng.integers(0, depth.max() + 1))
        d_want = min(d_want, int(depth.max()))
        cands = np.flatnonzero(depth == d_want)
        end = int(rng.choice(cands))
        on_path = set()
        x = end
        while x >= 0:
            on_path.add(x)
            x = int(par[x])
        ids = np.zeros(n, dtype=np.int64)
        ids[0] = int(root_ids[b]) if root_ids is not None else int(rng.integers(0, vocab))
        children = {}
        for i in range(1, n):
            children.setdefault(int(par[i]), []).append(i)
        for p, ch in children.items():
            used = set()
            for c in ch:
                if c in on_path:
                    ids[c] = tgt[p]
                    used.add(int(tgt[p]))
            for c in ch:
                if c in on_path:
                    continue
                while True:
                    cand = int(rng.integers(0, vocab))
                    if cand != tgt[p] and cand not in used:
                        break
                ids[c] = cand
                used.add(cand)
        out.append(ids)
        planted.append(d_want)
        off += n
    return np.concatenate(out).astype(np.int32), planted


@dataclass
class ToyWeights:
    """Random weights of a small pre-norm decoder (RMSNorm, rotary GQA attention, gated-SiLU MLP,
    untied LM head) used only by the greedy-losslessness check.  float64 numpy arrays."""

    d: int
    n_layers: int
    Hq: int
    Hkv: int
    Dh: int
    ffn: int
    vocab: int
    rope_base: float
    embed: np.ndarray  # [vocab, d]
    wq: List[np.ndarray]  # [d, Hq*Dh]
    wk: List[np.ndarray]  # [d, Hkv*Dh]
    wv: List[np.ndarray]  # [d, Hkv*Dh]
    wo: List[np.ndarray]  # [Hq*Dh, d]
    w_gate: List[np.ndarray]  # [d, ffn]
    w_up: List[np.ndarray]  # [d, ffn]
    w_down: List[np.ndarray]  # [ffn, d]
    norm1: List[np.ndarray]  # [d]
    norm2: List[np.ndarray]  # [d]
    norm_f: np.ndarray  # [d]
    lm_head: np.ndarray  # [vocab, d]


def make_toy_weights(seed: int, d: int = 64, n_layers: int = 2, Hq: int = 4, Hkv: int = 1,
                     Dh: int = 64, ffn: int = 256, vocab: int = 1000, lm_head_bf16: bool = False,
                     weights_bf16: bool = False) -> ToyWeights:
    """``lm_head_bf16``: the LM-head matrix holds bf16-representable values (for the toy whose
    verification step runs in bf16).  ``weights_bf16``: so do the embedding and every layer's
    matrices (for the toy whose whole layers run in bf16); the norm gains are 1."""
    rng = np.random.default_rng(seed * 16 + 11)
    as_bf16 = lambda m: torch.from_numpy(np.ascontiguousarray(m)).to(torch.bfloat16).to(torch.float64).numpy()

    def mat(i, o, gain=1.0):
        # values rounded to fp32 so that an fp32 copy of the model holds exactly the same weights
        m = (rng.standard_normal((i, o)) * gain / np.sqrt(i)).astype(np.float32)
        return as_bf16(m) if weights_bf16 else m.astype(np.float64)

    return ToyWeights(
        d=d, n_layers=n_layers, Hq=Hq, Hkv=Hkv, Dh=Dh, ffn=ffn, vocab=vocab, rope_base=10000.0,
        embed=(lambda m: as_bf16(m) if weights_bf16 else m.astype(np.float64))(rng.standard_normal((vocab, d)).astype(np.float32)),
        wq=[mat(d, Hq * Dh, 2.0) for _ in range(n_layers)],
        wk=[mat(d, Hkv * Dh, 2.0) for _ in range(n_layers)],
        wv=[mat(d, Hkv * Dh) for _ in range(n_layers)],
        wo=[mat(Hq * Dh, d) for _ in range(n_layers)],
        w_gate=[mat(d, ffn) for _ in range(n_layers)],
        w_up=[mat(d, ffn) for _ in range(n_layers)],
        w_down=[mat(ffn, d) for _ in range(n_layers)],
        norm1=[np.ones(d) for _ in range(n_layers)],
        norm2=[np.ones(d) for _ in range(n_layers)],
        norm_f=np.ones(d),
        lm_head=(lambda m: as_bf16(m) if (lm_head_bf16 or weights_bf16)
                 else m.astype(np.float64))((rng.standard_normal((vocab, d)) * 2.0).astype(np.float32)),
    )
