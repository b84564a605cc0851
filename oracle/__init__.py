"""CPU oracle for the target model's batched verification of a draft token tree.

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain definition that the GPU library is
checked against: float64 numpy, no paging tricks, no splitting, no code shared with the GPU
path.  Only the tests, the smoke check and the benchmark's CPU-baseline leg may import it; the
product path never does.

What it defines (the paper, Section 1: a draft model proposes several consecutive tokens and
the target model validates them in one batched pass; Section 4.1 "Setup": because the target
verifies, understanding quality is unaffected, i.e. greedy speculative decoding must emit the
target's own greedy stream):

  tree_attention.tree_attn_ref     attention of every draft node over prefix KV + its ancestors
  lm_head.lmhead_argmax_ref        per-node target token = argmax of the LM-head logits
  acceptance.tree_accept_ref       greedy longest accepted root-to-node path, bonus token
  kv_compaction.kv_compact_ref     append the accepted nodes' K/V to the paged cache
  stochastic_acceptance.tree_accept_sample_ref   sampling acceptance (speculative sampling over a tree)
  projections.qkv_rope_project_ref / linear_ref / tree_positions_ref   the projections around the attention
  projections.rmsnorm_ref / swiglu_ref                                 the layer's normalisations and feed-forward gate
  draft_tree.topk_logprob_ref / DraftTreeRef / build_draft_tree_ref   the draft tree's construction
  meta_query.meta_query_attn_ref / fc_concat_ref   the draft's intermediate layer (Section 3.1.1, Eq. 1)
  toy_decoder.ToyDecoderRef        small random-weight decoder: greedy autoregressive stream and
                                   greedy speculative decoding built from the four functions above

The paper defines neither the tree mask nor the acceptance rule (its experiments use chain
drafts and cite EAGLE-3 for the rest); the readings taken here are listed in the design notes.
Every function is pinned by CPU tests against closed forms, brute force on tiny inputs and
library routines.  The paper's own acceptance-length and tokens-per-second figures (Table 1,
Section 1) need trained weights and data and stay "parity unpinned".
"""
from .tree_attention import tree_attn_ref, ancestors
from .lm_head import lmhead_logits_ref, lmhead_argmax_ref
from .acceptance import tree_accept_ref
from .kv_compaction import kv_compact_ref
from .toy_decoder import ToyDecoderRef
from .stochastic_acceptance import tree_accept_sample_ref
from .draft_tree import topk_logprob_ref, DraftTreeRef, build_draft_tree_ref
from .meta_query import meta_query_attn_ref, fc_concat_ref
from .projections import tree_positions_ref, rope_ref, qkv_rope_project_ref, linear_ref, rmsnorm_ref, swiglu_ref

__all__ = [
    "tree_attn_ref",
    "ancestors",
    "lmhead_logits_ref",
    "lmhead_argmax_ref",
    "tree_accept_ref",
    "kv_compact_ref",
    "ToyDecoderRef",
    "tree_accept_sample_ref",
    "tree_positions_ref",
    "rope_ref",
    "qkv_rope_project_ref",
    "linear_ref",
    "rmsnorm_ref",
    "swiglu_ref",
    "topk_logprob_ref",
    "DraftTreeRef",
    "build_draft_tree_ref",
    "meta_query_attn_ref",
    "fc_concat_ref",
]
