/*
 * hb.h - C ABI of the tree-verification step of speculative decoding on MI355X (gfx950).
 *
 * The step (paper, Section 1): a draft model proposes several tokens, here arranged as a token
 * tree, and the target model validates all of them in one batched pass.  Because the target
 * decides, its outputs are unchanged (Section 4.1 "Setup"): under greedy decoding the emitted
 * stream equals plain autoregressive decoding.  The core of this library is that target-side
 * pass: attention of every tree node over the paged prefix KV cache plus its own ancestors, LM
 * head with a fused argmax, greedy longest-accepted-path selection (or sampling acceptance), and
 * the append of the accepted nodes' K/V to the cache (the paper keeps committed context in the
 * KV cache, Section 4.1).  Around it: the rest of the target's decoder layer (positions, rotary
 * table, fused QKV projection, output projection, normalisation, feed-forward block), the
 * construction of the draft tree from the draft model's logits, and the draft model's
 * intermediate layer (aggregation of the target's layer features with meta queries, Section
 * 3.1.1).
 *
 * Conventions for every entry point
 *   - Returns an hb_status; on failure hb_last_error() gives a thread-local message.
 *   - "device" pointers are GPU memory owned by the caller (valid on the current HIP device).
 *     The library never allocates, frees or keeps them.  "host" pointers are ordinary memory.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the default stream)
 *     and the call returns without waiting for it.
 *   - Only host-visible arguments are validated.  Malformed device data (a parent index that
 *     is not smaller than its node, a page id outside the pool, a prefix longer than the page
 *     table covers) is clamped so that every access stays inside the caller's buffers; the
 *     result for such input is unspecified.
 *   - A tree is an int32 parent array local to its sequence: parent[0] = -1 (the root is the
 *     pending committed token), 0 <= parent[i] < i otherwise.  Trees of a batch are
 *     concatenated; node_offset[b] .. node_offset[b+1] are the nodes of sequence b.
 *   - Tensors are dense, row-major, in the layouts stated per function, and start at a 16-byte
 *     aligned address (kernels move 16-byte pieces; another address is HB_ERR_INVALID_ARG).
 *     bf16 is the upper half of an IEEE float32 (round to nearest even on output).
 */
#ifndef HB_H
#define HB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum hb_status {
  HB_OK = 0,
  HB_ERR_INVALID_ARG = 1, /* null pointer, negative size, inconsistent sizes           */
  HB_ERR_UNSUPPORTED = 2, /* a shape or dtype this library has no kernel for           */
  HB_ERR_WORKSPACE = 3,   /* workspace missing or smaller than the *_workspace_bytes   */
  HB_ERR_DEVICE = 4       /* a HIP call failed; the message carries hipGetErrorString  */
} hb_status;

typedef enum hb_dtype { HB_F32 = 0, HB_BF16 = 1 } hb_dtype;

/* Kernel choice for hb_tree_verify_attn. */
typedef enum hb_attn_algo {
  HB_ATTN_AUTO = 0,   /* MFMA kernel when the shape allows it, else the scalar kernel        */
  HB_ATTN_SCALAR = 1, /* one wavefront per (node, query head, split); any dtype, fp32 math  */
  HB_ATTN_MFMA = 2    /* bf16, head_dim 128, page 16: KV tile shared by all nodes and the   */
                      /* query heads of a kv group, bf16 MFMA with fp32 accumulation         */
} hb_attn_algo;

/* Shapes of one attention layer of one verification step. */
typedef struct hb_attn_desc {
  int32_t dtype;               /* hb_dtype of q, k/v (tree and pools) and out               */
  int32_t batch;               /* B, number of sequences                                    */
  int32_t num_q_heads;         /* Hq                                                        */
  int32_t num_kv_heads;        /* Hkv, divides Hq; query head h reads kv head h / (Hq/Hkv)  */
  int32_t head_dim;            /* D, multiple of 8, at most 256                             */
  int32_t page_size;           /* tokens per KV page                                        */
  int32_t max_blocks_per_seq;  /* row length of block_table                                 */
  int32_t num_blocks;          /* pages in each pool (page ids are clamped to this)         */
  int32_t total_nodes;         /* node_offset[B]                                            */
  int32_t max_nodes_per_tree;  /* upper bound on nodes per sequence, at most 64             */
  int32_t num_splits;          /* KV partitions per sequence; 0 = let the library choose    */
                               /* (the MFMA kernel then cuts the KV on the device, from the */
                               /* actual prefix lengths, evenly over the workgroups)        */
  int32_t max_prefix_len_hint; /* upper bound on prefix_len known to the host, 0 = unknown  */
                               /* (then max_blocks_per_seq * page_size is assumed); with a  */
                               /* prefix longer than a given bound the result is unspecified */
  int32_t algo;                /* hb_attn_algo                                              */
  float softmax_scale;         /* scores are softmax_scale * <q, k>                         */
} hb_attn_desc;

const char *hb_last_error(void);
int32_t hb_version(void);

/* Host-side check of one tree's parent array (host pointer): HB_OK iff parent[0] == -1 and
 * 0 <= parent[i] < i for 0 < i < n, and 1 <= n <= 64. */
int32_t hb_tree_validate_host(const int32_t *parent, int32_t n);

/*
 * Tree-masked attention (the batched validation pass of Section 1).
 * For node i of sequence b and query head h (kv head g = h / (Hq/Hkv)):
 *   keys   = prefix positions 0 .. prefix_len[b]-1  and the tree nodes on the path root .. i
 *   out    = sum_j softmax_j(softmax_scale * <q[i,h], k_j>) * v_j       over those keys
 *   lse    = log sum_j exp(softmax_scale * <q[i,h], k_j>)               (natural log)
 * Prefix position p is read at pool[block_table[b][p / page_size]][g][p % page_size][:].
 *
 *   q, out          device [total_nodes, Hq, D]        desc->dtype
 *   k_tree, v_tree  device [total_nodes, Hkv, D]       desc->dtype (K/V of the tree nodes)
 *   k_pool, v_pool  device [num_blocks, Hkv, page, D]  desc->dtype
 *   block_table     device int32 [B, max_blocks_per_seq]
 *   prefix_len      device int32 [B]
 *   node_offset     device int32 [B+1]
 *   parent          device int32 [total_nodes]
 *   lse             device float32 [total_nodes, Hq], or NULL
 *   workspace       device, at least hb_tree_verify_attn_workspace_bytes(desc) bytes, 256-byte
 *                   aligned; may be NULL when that size is 0.  Contents are scratch.
 * Accumulation is fp32; bf16 results are rounded once at the end.  Slots of a page at or beyond
 * prefix_len, unmapped pages and tree nodes off the path are never allowed to influence the
 * result, whatever bit patterns they hold.
 * Errors: INVALID_ARG (null pointers, sizes <= 0 where a positive size is needed, Hq % Hkv),
 * UNSUPPORTED (dtype, D, more than 64 nodes per tree, HB_ATTN_MFMA on a shape it cannot take),
 * WORKSPACE, DEVICE.  batch == 0 or total_nodes == 0 is a successful no-op.
 */
int32_t hb_tree_verify_attn(const hb_attn_desc *desc, const void *q, const void *k_tree,
                            const void *v_tree, const void *k_pool, const void *v_pool,
                            const int32_t *block_table, const int32_t *prefix_len,
                            const int32_t *node_offset, const int32_t *parent, void *out,
                            float *lse, void *workspace, size_t workspace_bytes, void *stream);

/* Bytes of workspace hb_tree_verify_attn needs for this descriptor (0 on a bad descriptor). */
size_t hb_tree_verify_attn_workspace_bytes(const hb_attn_desc *desc);

/* The number of KV partitions the library uses for this descriptor (resolves num_splits == 0):
 * the number of partial results per query row that the workspace has room for. */
int32_t hb_tree_verify_attn_num_splits(const hb_attn_desc *desc);

/*
 * LM head with fused argmax: the target's token after each node (greedy validation,
 * Section 1 / Section 4.1).  out_ids[m] = the lowest v maximising sum_k hidden[m,k]*weight[v,k];
 * logits are never written to memory.  A NaN logit never wins.
 *
 *   hidden    device [M, K]   dtype          weight   device [V, K]  dtype (nn.Linear layout)
 *   out_ids   device int32 [M]               out_max  device float32 [M] or NULL: the winning
 *                                                     logit as accumulated in fp32
 *   workspace device, hb_lmhead_argmax_workspace_bytes(M) bytes, 8-byte aligned
 * bf16 inputs with K % 64 == 0 take the MFMA kernel; everything else a scalar fp32 kernel.
 * Errors: INVALID_ARG, UNSUPPORTED (dtype), WORKSPACE, DEVICE.  M == 0 is a no-op; V >= 1.
 */
int32_t hb_lmhead_argmax(int32_t dtype, int32_t M, int32_t K, int32_t V, const void *hidden,
                         const void *weight, int32_t *out_ids, float *out_max, void *workspace,
                         size_t workspace_bytes, void *stream);

size_t hb_lmhead_argmax_workspace_bytes(int32_t M);

/*
 * hb_lmhead_argmax for callers that cannot allocate device memory or carry a workspace around
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same
 * arguments without the workspace, same kernels, same results.  The per-row keys live in a
 * device array that belongs to the library (8 bytes per row, 128 KiB on every GPU the library
 * runs on, held until the process ends); the call allocates and frees nothing.
 *   M <= hb_lmhead_argmax_noalloc_max_rows() (16384), else HB_ERR_UNSUPPORTED.
 * Every call on a GPU uses that GPU's one array (cleared by a kernel at the start of the
 * call): calls that overlap on one GPU (different streams, or graphs replayed concurrently)
 * race and give unspecified ids; calls ordered on one stream, or otherwise serialised, are fine.
 * Errors otherwise as hb_lmhead_argmax (DEVICE also when the array's address cannot be found).
 */
int32_t hb_lmhead_argmax_noalloc(int32_t dtype, int32_t M, int32_t K, int32_t V, const void *hidden,
                                 const void *weight, int32_t *out_ids, float *out_max, void *stream);

int32_t hb_lmhead_argmax_noalloc_max_rows(void);

/*
 * The target's projections around the attention of one decoder layer (the validation pass of
 * Section 1 runs the whole target model over the drafted tokens; the paper gives no model
 * dimensions, the shapes are those of the workloads here).  bf16 storage, fp32 accumulation.
 *
 * hb_tree_positions: positions[n] = prefix_len[b] + depth of node n in its tree: the position the
 * drafted token would have in sequential decoding.
 *   node_offset device int32 [B+1], parent device int32 [total], prefix_len device int32 [B],
 *   positions device int32 [total] (out).  Trees of at most 64 nodes.
 * hb_rope_table: cos_out[t, d] = cos(positions[t] * theta^(-d / half)), sin_out likewise,
 *   d < half = head_dim / 2; device float32 [T, half], computed in double precision.
 * hb_qkv_rope_project: y = hidden W^T (+ bias); rows of W are the Hq query heads, then the Hkv key
 *   heads, then the Hkv value heads, 128 features each; queries and keys get the rotary embedding
 *   (rotate-half convention: feature d < 64 of a head is paired with d + 64 and the pair rotated
 *   by the angle of the token's row of the table); results go to q [T, Hq, 128], k [T, Hkv, 128],
 *   v [T, Hkv, 128], the layouts hb_tree_verify_attn takes.
 *   hidden device bf16 [T, K]; w_qkv device bf16 [(Hq + 2 Hkv) * 128, K]; bias device bf16
 *   [(Hq + 2 Hkv) * 128] or NULL; cos, sin device float32 [T, 64].  K % 64 == 0, head_dim 128.
 * hb_out_project: out = x W^T (+ residual): x device bf16 [T, K], w device bf16 [N, K], residual
 *   device bf16 [T, N] or NULL, out device bf16 [T, N]; K % 64 == 0, N % 4 == 0.
 * All tensors 16-byte aligned.  Errors: INVALID_ARG, UNSUPPORTED (shape), DEVICE.  T == 0: no-op.
 */
int32_t hb_tree_positions(int32_t B, int32_t max_nodes_per_tree, int32_t total_nodes,
                          const int32_t *node_offset, const int32_t *parent, const int32_t *prefix_len,
                          int32_t *positions, void *stream);
int32_t hb_rope_table(int32_t T, int32_t head_dim, double theta, const int32_t *positions, float *cos_out,
                      float *sin_out, void *stream);
int32_t hb_qkv_rope_project(int32_t T, int32_t K, int32_t Hq, int32_t Hkv, int32_t head_dim, const void *hidden,
                            const void *w_qkv, const void *bias_or_null, const float *cos, const float *sin,
                            void *q, void *k, void *v, void *stream);
int32_t hb_out_project(int32_t T, int32_t K, int32_t N, const void *x, const void *w,
                       const void *residual_or_null, void *out, void *stream);

/*
 * The same two projections for small token counts (chain drafts, the draft model's batches), the
 * setting of the paper's own measurements (Section 4.2: chain decoding).  With a few hundred tokens
 * or fewer (and with up to a thousand when K is long) a projection is a stream of its weight
 * matrix from HBM, and one workgroup per 256-row weight tile and tile of tokens leaves most of
 * the chip idle; given a workspace these calls cut K into parts, one workgroup per (weight tile, K part, tile of tokens), keep the parts' fp32
 * partial results in the workspace and finish (sum in fixed order, bias, rotary embedding,
 * residual) in a second kernel.  Results are deterministic; they differ from the calls above in
 * fp32 summation order only.
 *   workspace   device, hb_proj_workspace_bytes(T, K, N) bytes (N = (Hq + 2 Hkv) * 128 for the
 *               QKV projection), 16-byte aligned.  That size is 0 when the split does not apply
 *               (more than 1024 tokens, K too short to cut, or more than 512 tokens and no gain
 *               expected: the split pays there for long K only); with a NULL, short or misaligned
 *               workspace the calls behave exactly as the ones above.
 * Errors as above.
 */
size_t hb_proj_workspace_bytes(int32_t T, int32_t K, int32_t N);
int32_t hb_qkv_rope_project_ws(int32_t T, int32_t K, int32_t Hq, int32_t Hkv, int32_t head_dim, const void *hidden,
                               const void *w_qkv, const void *bias_or_null, const float *cos, const float *sin,
                               void *q, void *k, void *v, void *workspace, size_t workspace_bytes, void *stream);
int32_t hb_out_project_ws(int32_t T, int32_t K, int32_t N, const void *x, const void *w,
                          const void *residual_or_null, void *out, void *workspace, size_t workspace_bytes,
                          void *stream);

/*
 * The rest of a decoder layer of the target around the attention block (Section 1: the target
 * validates the drafted tokens in one parallel pass over whole layers; pre-norm layers with
 * root-mean-square normalisation and a gated-SiLU feed-forward block, the decoder family that the
 * paper's base model builds on).  All tensors bf16, device, 16-byte aligned, row-major; fp32
 * accumulation, one rounding to bf16 at the end.
 *
 * hb_rmsnorm:  out[t, :] = x[t, :] / sqrt(mean_k x[t, k]^2 + eps) * weight.
 *   x, out [T, K] (out may be x);  weight [K];  eps >= 0.
 * hb_swiglu_project:  out[t, f] = silu(x[t] . w_gate[f]) * (x[t] . w_up[f]),  silu(z) = z / (1 + exp(-z)),
 *   both projections in one pass over x.
 *   x [T, K];  w_gate_up [2 F, K]: the gate projection's F rows, then the up projection's F rows
 *   (y = x W^T layout);  out [T, F].
 *   workspace_or_null   device, hb_proj_workspace_bytes(T, K, 2 * F) bytes, 16-byte aligned: with
 *               it, few tokens take the split over K of hb_out_project_ws; NULL, short or
 *               misaligned: the unsplit kernel.
 * The block's down projection with its residual is hb_out_project(T, F, K, act, w_down, residual, out).
 * Errors: INVALID_ARG (T < 0, sizes < 1, eps < 0, NULL or misaligned pointers), UNSUPPORTED
 * (hb_rmsnorm: K % 8 != 0; hb_swiglu_project: K % 64 != 0, F % 4 != 0), DEVICE.  T == 0 is a no-op.
 */
int32_t hb_rmsnorm(int32_t T, int32_t K, const void *x, const void *weight, float eps, void *out, void *stream);
int32_t hb_swiglu_project(int32_t T, int32_t K, int32_t F, const void *x, const void *w_gate_up, void *out,
                          void *workspace_or_null, size_t workspace_bytes, void *stream);

/*
 * Greedy longest accepted path per sequence.  Node 0 is always accepted; node i > 0 matches
 * when draft_ids[i] == target_ids[parent[i]] and is accepted when it and all its ancestors
 * match.  The deepest accepted node wins (lowest id among equals).  accept_len is the number
 * of tokens the step emits (accepted drafts below the root plus the bonus token), the quantity
 * whose mean the paper reports as average acceptance length (Table 1).
 * prev_target_or_null (device int32 [B], or NULL) switches to the reading in which the root too
 * is a guess: it matches only when draft_ids[root] == prev_target[b], the token the target chose
 * at the end of the previous step.  A rejected root voids the whole tree: accept_len = 0, path
 * and tokens all -1, bonus_id = prev_target[b].  A sequence without nodes gives accept_len = 0,
 * path and tokens -1 and bonus_id = prev_target[b] (-1 when NULL); hb_kv_compact then copies
 * nothing for it.
 *
 *   node_offset  device int32 [B+1]     parent, draft_ids, target_ids  device int32 [total]
 *   accept_len   device int32 [B]       bonus_id  device int32 [B] = target_ids[best node]
 *   accept_path  device int32 [B, max_path]  tree-local node ids root..best, then -1
 *   out_tokens   device int32 [B, max_path]  draft ids of path[1..], then the bonus id, then -1
 * Nodes deeper than max_path-1 are treated as not accepted.  Trees with more than
 * max_nodes_per_tree (<= 64) nodes are cut at that many nodes.
 * Errors: INVALID_ARG, UNSUPPORTED (max_nodes_per_tree > 64), DEVICE.  B == 0 is a no-op.
 */
int32_t hb_tree_accept(int32_t B, int32_t max_nodes_per_tree, const int32_t *node_offset,
                       const int32_t *parent, const int32_t *draft_ids, const int32_t *target_ids,
                       const int32_t *prev_target_or_null, int32_t max_path, int32_t *accept_len,
                       int32_t *accept_path, int32_t *out_tokens, int32_t *bonus_id, void *stream);

/*
 * Sampling acceptance (lossless under sampling: the emitted tokens are distributed as the
 * target's own samples; the paper, Section 1 and Section 4.1 "Setup", states the lossless
 * validation and defers the procedure to EAGLE-3).  The rule is speculative sampling with several
 * candidates per position: the children of the current node are tried in index order, child with
 * token x is accepted with probability min(1, p(x)/q(x)), p / q = the target's / the draft's
 * distribution of the token after the current node; a rejection replaces p by the renormalised
 * residual max(p - q, 0) and removes x from q (candidates are drawn without replacement).  When
 * no child is accepted, or the node has none, or the path holds max_path nodes, the step's last
 * token is drawn from the current p.  Node 0 is always on the path.  Outputs as hb_tree_accept.
 *
 * Every decision is taken in exact integers, reproducible bit for bit: fix(p) = floor(p * 2^30),
 * S = sum over the vocabulary,
 *   accept        iff  u * q_x * S(p) < 2^32 * p_x * S(q)
 *   residual      r_v = max(p_v * S(q) - q_v * S(p), 0),  p_v <- r_v / max(S(r) >> 30, 1)
 *                 (integer division; p unchanged when S(r) = 0),  q_x <- 0
 *   last token    the smallest v with p_0 + .. + p_v > (u_bonus * S(p)) >> 32  (-1 when S(p) = 0)
 *
 *   p_target, q_draft  device float32 [total_nodes, V]: distributions AFTER each node (entries in
 *                      [0, 1], each row summing to at most about 1: larger sums overflow the
 *                      integer products and give unspecified, though memory-safe, results)
 *   u_accept   device uint32 [total_nodes]: the uniform used when that node is tried as a child
 *   u_bonus    device uint32 [B]: the uniform of the step's last token
 *   workspace  device, hb_tree_accept_sample_workspace_bytes(B, V) bytes, 4-byte aligned
 * Errors: INVALID_ARG, UNSUPPORTED (max_nodes_per_tree > 64), WORKSPACE, DEVICE.  B == 0: no-op.
 */
int32_t hb_tree_accept_sample(int32_t B, int32_t max_nodes_per_tree, int32_t V, const int32_t *node_offset,
                              const int32_t *parent, const int32_t *draft_ids, const float *p_target,
                              const float *q_draft, const uint32_t *u_accept, const uint32_t *u_bonus,
                              int32_t max_path, int32_t *accept_len, int32_t *accept_path,
                              int32_t *out_tokens, int32_t *bonus_id, void *workspace,
                              size_t workspace_bytes, void *stream);

size_t hb_tree_accept_sample_workspace_bytes(int32_t B, int32_t V);

/*
 * Append the accepted path's K/V to the paged cache of one layer (Section 4.1: committed
 * context lives in the KV cache).  For j < accept_len[b]: position p = prefix_len[b] + j,
 * slot = block_table[b][p / page] * page + p % page; the K and V rows (all kv heads) of tree
 * node accept_path[b][j] are copied there bit for bit; out_slots[b][j] = slot, -1 for
 * j >= accept_len[b]; new_len[b] = prefix_len[b] + accept_len[b].  No other byte of the pools
 * changes.  The caller guarantees block_table maps the pages up to prefix_len + max_path;
 * positions beyond max_blocks_per_seq * page are skipped.
 * Uses desc->{dtype, batch, num_kv_heads, head_dim, page_size, max_blocks_per_seq, num_blocks,
 * total_nodes}.  out_slots and new_len may be NULL.
 * Errors: INVALID_ARG, UNSUPPORTED, DEVICE.
 */
int32_t hb_kv_compact(const hb_attn_desc *desc, const void *k_tree, const void *v_tree,
                      void *k_pool, void *v_pool, const int32_t *block_table,
                      const int32_t *prefix_len, const int32_t *node_offset,
                      const int32_t *accept_len, const int32_t *accept_path, int32_t max_path,
                      int32_t *out_slots, int32_t *new_len, void *stream);

/*
 * hb_kv_compact for every layer of the model in one launch (the same accepted path goes into
 * each layer's cache; Section 4.1: committed context lives in the KV cache).  k_tree, v_tree,
 * k_pool, v_pool are DEVICE arrays of n_layers device pointers (8-byte aligned tables; every
 * tensor as in hb_kv_compact, 16-byte aligned, which the call cannot check on the host).  The
 * page table, lengths and path are shared by the layers; out_slots and new_len (optional) are
 * written once.  Errors: INVALID_ARG, UNSUPPORTED, DEVICE.  n_layers == 0 is a no-op.
 */
int32_t hb_kv_compact_layers(const hb_attn_desc *desc, int32_t n_layers, const void *const *k_tree,
                             const void *const *v_tree, void *const *k_pool, void *const *v_pool,
                             const int32_t *block_table, const int32_t *prefix_len, const int32_t *node_offset,
                             const int32_t *accept_len, const int32_t *accept_path, int32_t max_path,
                             int32_t *out_slots, int32_t *new_len, void *stream);

/*
 * Construction of the draft tree from the draft model's outputs: the step before the
 * verification (the paper drafts in the EAGLE-3 manner, Section 3.1, and leaves the arrangement of
 * the drafted tokens open; its measurements use chains, Section 4.2).  This is the dynamic tree of
 * that line of work: the draft model runs level by level; a node's K most probable next tokens are
 * its candidate children, a candidate's score is the log-probability of its whole path; of each
 * level's candidates the K best are run again; after T levels all candidates are re-ranked and
 * the n - 1 best form, with the root, the tree that the target verifies.
 *
 * hb_topk_logprob: per row of logits the k best tokens, ordered by (logit descending, token id
 * ascending; -0 equals +0), and their log-probabilities logit - logsumexp(row) (float32, never
 * above 0).  The ids depend on comparisons only and are exact; NaN logits rank as -inf.
 *   dtype      HB_F32 or HB_BF16 (type of logits)
 *   logits     device [M, V] row-major
 *   out_ids    device int32 [M, k];  out_logp  device float32 [M, k]
 *   workspace  device, hb_topk_logprob_workspace_bytes(M, V, k) bytes, 8-byte aligned
 * Errors: INVALID_ARG (M < 0, V <= 0, k < 1, k > V, NULL pointers), UNSUPPORTED (k > 32),
 * WORKSPACE, DEVICE.  M == 0 is a no-op.
 */
int32_t hb_topk_logprob(int32_t dtype, int32_t M, int32_t V, int32_t k, const void *logits, int32_t *out_ids,
                        float *out_logp, void *workspace, size_t workspace_bytes, void *stream);

size_t hb_topk_logprob_workspace_bytes(int32_t M, int32_t V, int32_t k);

/* Candidates a pool holds per sequence after T levels: K + (T - 1) K^2. */
int32_t hb_draft_tree_candidates(int32_t K, int32_t T);

/*
 * One level of the draft tree.  Level 0 takes the root's K children (F = 1 row per sequence):
 * candidates 0 .. K-1, all of them form the frontier.  Level l >= 1 takes the K children of each
 * of the K frontier nodes (F = K rows per sequence, in frontier order): candidate
 * K + (l - 1) K^2 + f K + j for frontier slot f and child rank j, with
 *   score = score(parent) + child_logp      (ONE float32 addition, round to nearest; NaN -> -inf)
 * and the K best of them (higher score first, equal scores: lower candidate index) become the
 * new frontier, best first.
 *   child_ids, child_logp   device int32 / float32 [B, F, K] (hb_topk_logprob's outputs for the
 *                           B * F rows the draft model just ran on; log-probabilities <= 0)
 *   cand_score, cand_token, cand_parent   device float32 / int32 / int32 [B, C], C =
 *                           hb_draft_tree_candidates(K, T): the pool, owned by the caller, appended
 *                           to by every level (cand_parent = candidate index of the parent, -1 = root)
 *   frontier       device int32 [B, K]: in (level >= 1) the candidate indices the rows belong to,
 *                  out the new frontier; frontier_slot device int32 [B, K]: out, the slot f of
 *                  each new frontier node's parent (which row of this level it descends from)
 * Errors: INVALID_ARG (B < 0, K < 1, T < 1, level outside [0, T), NULL pointers), UNSUPPORTED
 * (K > 32), DEVICE.  B == 0 is a no-op.
 */
int32_t hb_tree_grow(int32_t B, int32_t K, int32_t T, int32_t level, const int32_t *child_ids,
                     const float *child_logp, float *cand_score, int32_t *cand_token, int32_t *cand_parent,
                     int32_t *frontier, int32_t *frontier_slot, void *stream);

/*
 * Re-ranking: of the C = hb_draft_tree_candidates(K, T) candidates of each sequence the
 * n_nodes - 1 best are kept (order as in hb_tree_grow) and numbered 1 .. n_nodes-1 in candidate
 * order, which puts every parent before its children; node 0 is the root.  Log-probabilities
 * <= 0 make scores fall along a path, so a kept node's parent is kept; otherwise (malformed
 * input) the node is hung under the root.  Outputs are in the verification calls' layout:
 *   root_token   device int32 [B]: the pending committed token of each sequence
 *   node_offset  device int32 [B + 1] = b * n_nodes
 *   parent, draft_ids, depth   device int32 [B * n_nodes] (tree-local parents, -1 for the root)
 *   anc_mask     device uint64 [B * n_nodes]: bit j of entry i set iff node j is i or an ancestor of i
 *   node_cand    device int32 [B * n_nodes]: the node's candidate index (-1 for the root)
 *   node_score   device float32 [B * n_nodes]: the node's path log-probability (0 for the root)
 * Errors: INVALID_ARG (n_nodes < 1 or n_nodes - 1 > C, NULL pointers), UNSUPPORTED (n_nodes > 64,
 * K > 32, C > 4096), DEVICE.  B == 0 is a no-op.
 */
int32_t hb_tree_finalize(int32_t B, int32_t K, int32_t T, int32_t n_nodes, const float *cand_score,
                         const int32_t *cand_token, const int32_t *cand_parent, const int32_t *root_token,
                         int32_t *node_offset, int32_t *parent, int32_t *draft_ids, int32_t *depth,
                         uint64_t *anc_mask, int32_t *node_cand, float *node_score, void *stream);

/*
 * Target-feature aggregation with meta queries, the draft model's intermediate layer (Section
 * 3.1.1, Eq. 1; skip connection and the fully connected layers around it: Section 3.1.2).  Read
 * as multi-head cross-attention (H heads of size d = D / H, no biases, weights in the y = x W^T
 * layout, scores scaled by 1 / sqrt(d)) of Q token-independent queries f_q over the L layer
 * features f_i of every token:
 *   f_c^i = flatten( concat_h( softmax(q_h k_{i,h}^T / sqrt(d)) v_{i,h} ) W_o^T + f_i[residual layers] ),
 *   q = f_q W_q^T,  k_i = f_i W_k^T,  v_i = f_i W_v^T.
 * The calls split it so that every dense product runs on the matrix cores and the key projection
 * disappears: (1) once per set of weights, hb_meta_query_fold builds A[h Q + q] =
 * (f_q W_q^T)_{q,h} W_k[h d .. (h+1) d, :] / sqrt(d), so that score(q, h, l) = A[h Q + q] . f_i[l];
 * (2) per batch of tokens, v_proj = feats W_v^T by hb_out_project(S * L, D, D, feats, w_v, NULL,
 * v_proj); (3) hb_meta_query_attn computes the scores, the softmax over the layers and
 * pre[i, q, c] = sum_l P[i, head(c), q, l] v_proj[i, l, c], and copies the residual rows; (4)
 * f_c = hb_out_project(S * Q, D, D, pre, w_o, residual, f_c), read as [S, Q * D]; fc1 and fc2 are
 * further hb_out_project calls (fc2 over a concatenation [a, b] as two calls, the second with the
 * first's output as residual).  All tensors bf16, 16-byte aligned, row-major.
 *
 * hb_meta_query_fold:
 *   f_q [Q, D], w_q [D, D], w_k [D, D]   device
 *   a_fold      device, hb_meta_query_fold_bytes(Q, D, H) bytes: two bf16 matrices
 *               [rows_pad, D] (value rounded to bf16, and the rounded remainder), rows_pad =
 *               H * Q rounded up to a multiple of 16
 *   workspace   device, Q * D floats
 * hb_meta_query_attn:
 *   feats, v_proj [S, L, D] device;  a_fold from hb_meta_query_fold
 *   residual_layers_or_null   HOST int32 [Q]: the layer whose feature is each query's residual
 *   pre [S, Q, D] device;  residual_out_or_null [S, Q, D] device (written iff residual layers given)
 *   workspace   device, hb_meta_query_attn_workspace_bytes(S, D, H, Q) bytes (0 for an unsupported
 *               shape), 4-byte aligned, overwritten: partial scores of the tokens, about 12 KB per
 *               token and per share of D that a workgroup column takes (14 shares of D = 3584
 *               for up to about 300 tokens, one from 4096 tokens on)
 * Errors: INVALID_ARG (sizes < 1, H not dividing D, residual layer outside [0, L), NULL or
 * misaligned pointers), UNSUPPORTED (D % 256 != 0, (D / H) % 8 != 0, H * Q > 96, Q > 4, L > 32),
 * WORKSPACE, DEVICE.  S == 0 is a no-op.
 */
size_t hb_meta_query_fold_bytes(int32_t Q, int32_t D, int32_t H);

int32_t hb_meta_query_fold(int32_t Q, int32_t D, int32_t H, const void *f_q, const void *w_q, const void *w_k,
                           void *a_fold, void *workspace, size_t workspace_bytes, void *stream);

size_t hb_meta_query_attn_workspace_bytes(int32_t S, int32_t D, int32_t H, int32_t Q);

int32_t hb_meta_query_attn(int32_t S, int32_t L, int32_t D, int32_t H, int32_t Q, const void *feats,
                           const void *v_proj, const void *a_fold, const int32_t *residual_layers_or_null,
                           void *pre, void *residual_out_or_null, void *workspace, size_t workspace_bytes,
                           void *stream);

#ifdef __cplusplus
}
#endif
#endif /* HB_H */
