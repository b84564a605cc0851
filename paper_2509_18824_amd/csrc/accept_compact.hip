// Greedy longest-accepted-path selection and KV compaction.
//
// Acceptance: one wavefront per sequence, one lane per tree node (at most 64 nodes).  Each lane
// walks to the root once to collect its ancestor set as a 64-bit mask; a wave ballot of the
// per-node match flags then tells every lane at once whether its whole path matches.
// Compaction: one workgroup per (path slot, sequence) copies that node's K and V rows into the
// page slot that follows the prefix, in 16-byte pieces.
#include "hb_internal.h"

namespace hb {

namespace {

__global__ __launch_bounds__(64) void tree_accept_kernel(
    int max_nodes, const int32_t *__restrict__ node_offset, const int32_t *__restrict__ parent,
    const int32_t *__restrict__ draft_ids, const int32_t *__restrict__ target_ids,
    const int32_t *__restrict__ prev_target, int max_path, int32_t *__restrict__ accept_len, int32_t *__restrict__ accept_path, int32_t *__restrict__ out_tokens,
    int32_t *__restrict__ bonus_id) {
  __shared__ int32_t spar[64];
  const int b = blockIdx.x;
  const int lane = threadIdx.x;
  const int n0 = node_offset[b];
  int n = node_offset[b + 1] - n0;
  n = n < 0 ? 0 : (n > max_nodes ? max_nodes : n);
  const bool live = lane < n;

  int par = -1, did = 0, tid_ = 0;
  if (live) {
    par = parent[n0 + lane];
    if (par >= lane || par < -1) par = -1;  // malformed: treat as a root-like node
    if (lane == 0) par = -1;
    did = draft_ids[n0 + lane];
    tid_ = target_ids[n0 + lane];
  }
  spar[lane] = par;
  __syncthreads();

  // ancestor set (self included) and whether this node's own id matches its parent's target
  unsigned long long anc = live ? (1ull << lane) : 0ull;
  int x = par;
  for (int guard = 0; x >= 0 && guard < 64; ++guard) {
    anc |= 1ull << x;
    x = spar[x];
  }
  bool rooted = live && (anc & 1ull);  // a path that does not reach node 0 is never accepted
  int par_target = __shfl(tid_, par < 0 ? 0 : par, 64);
  // the root is the pending committed token (always a match) unless the caller names the token
  // the target chose last step: then the root is a guess like any other node
  const int prev = prev_target ? prev_target[b] : 0;
  bool match = live && (lane == 0 ? (!prev_target || did == prev) : did == par_target);
  unsigned long long match_mask = __ballot(match);
  int depth = __popcll(anc) - 1;
  bool accepted = rooted && ((anc & ~match_mask) == 0ull) && depth < max_path;

  // deepest accepted node, lowest id among equals: maximise depth * 64 + (63 - lane)
  int key = accepted ? depth * 64 + (63 - lane) : -1;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) key = max(key, __shfl_xor(key, off, 64));
  // no node accepted (no nodes at all, or a rejected root): nothing is emitted, the pending
  // token stays what it was
  if (key < 0) {
    for (int j = lane; j < max_path; j += 64) {
      accept_path[(size_t)b * max_path + j] = -1;
      out_tokens[(size_t)b * max_path + j] = -1;
    }
    if (lane == 0) {
      accept_len[b] = 0;
      bonus_id[b] = prev_target ? prev : -1;
    }
    return;
  }
  const int best = 63 - (key & 63);
  const int len = (key >> 6) + 1;
  const unsigned long long best_anc = __shfl((long long)anc, best, 64);
  const int best_target = __shfl(tid_, best, 64);

  if (live && ((best_anc >> lane) & 1ull)) {
    int rank = __popcll(best_anc & ((1ull << lane) - 1ull));
    accept_path[(size_t)b * max_path + rank] = lane;
    if (rank >= 1) out_tokens[(size_t)b * max_path + rank - 1] = did;
  }
  for (int j = len + lane; j < max_path; j += 64) {
    accept_path[(size_t)b * max_path + j] = -1;
    out_tokens[(size_t)b * max_path + j] = -1;
  }
  if (lane == 0) {
    out_tokens[(size_t)b * max_path + len - 1] = best_target;
    accept_len[b] = len;
    bonus_id[b] = best_target;
  }
}

// one (path slot j, sequence b) of one layer; out_slots / new_len are written when given
__device__ __forceinline__ void compact_one(
    const hb_attn_desc &d, int row_bytes, const uint4 *__restrict__ k_tree, const uint4 *__restrict__ v_tree,
    uint4 *__restrict__ k_pool, uint4 *__restrict__ v_pool, const int32_t *__restrict__ block_table,
    const int32_t *__restrict__ prefix_len, const int32_t *__restrict__ node_offset,
    const int32_t *__restrict__ accept_len, const int32_t *__restrict__ accept_path, int max_path,
    int32_t *__restrict__ out_slots, int32_t *__restrict__ new_len) {
  const int j = blockIdx.x;
  const int b = blockIdx.y;
  int len = accept_len[b];
  len = len < 0 ? 0 : (len > max_path ? max_path : len);
  int L = prefix_len[b];
  L = L < 0 ? 0 : L;
  if (j == 0 && threadIdx.x == 0 && new_len) new_len[b] = L + len;
  const long long p = (long long)L + j;
  const bool in_table = p < (long long)d.max_blocks_per_seq * d.page_size;
  if (j >= len || !in_table) {
    if (threadIdx.x == 0 && out_slots) out_slots[(size_t)b * max_path + j] = -1;
    return;
  }
  const int n0 = node_offset[b];
  int n = node_offset[b + 1] - n0;
  int node = accept_path[(size_t)b * max_path + j];
  node = node < 0 ? 0 : (node >= n ? n - 1 : node);
  int src = n0 + node;
  src = src < 0 ? 0 : (src >= d.total_nodes ? d.total_nodes - 1 : src);
  int blk = block_table[(size_t)b * d.max_blocks_per_seq + (int)(p / d.page_size)];
  blk = blk < 0 ? 0 : (blk >= d.num_blocks ? d.num_blocks - 1 : blk);
  const int off = (int)(p % d.page_size);
  if (threadIdx.x == 0 && out_slots) out_slots[(size_t)b * max_path + j] = blk * d.page_size + off;
  const int vec_per_row = row_bytes / 16;  // 16-byte pieces of one head's row
  for (int t = threadIdx.x; t < d.num_kv_heads * vec_per_row; t += blockDim.x) {
    int h = t / vec_per_row, w = t - h * vec_per_row;
    size_t s_idx = ((size_t)src * d.num_kv_heads + h) * vec_per_row + w;
    size_t d_idx = (((size_t)blk * d.num_kv_heads + h) * d.page_size + off) * vec_per_row + w;
    k_pool[d_idx] = k_tree[s_idx];
    v_pool[d_idx] = v_tree[s_idx];
  }
}

__global__ __launch_bounds__(256) void kv_compact_kernel(
    hb_attn_desc d, int row_bytes, const uint4 *__restrict__ k_tree, const uint4 *__restrict__ v_tree,
    uint4 *__restrict__ k_pool, uint4 *__restrict__ v_pool, const int32_t *__restrict__ block_table,
    const int32_t *__restrict__ prefix_len, const int32_t *__restrict__ node_offset,
    const int32_t *__restrict__ accept_len, const int32_t *__restrict__ accept_path, int max_path,
    int32_t *__restrict__ out_slots, int32_t *__restrict__ new_len) {
  compact_one(d, row_bytes, k_tree, v_tree, k_pool, v_pool, block_table, prefix_len, node_offset, accept_len,
              accept_path, max_path, out_slots, new_len);
}

// all layers in one launch: blockIdx.z = layer, its tensors from tables of device pointers
__global__ __launch_bounds__(256) void kv_compact_layers_kernel(
    hb_attn_desc d, int row_bytes, const uint4 *const *__restrict__ k_tree, const uint4 *const *__restrict__ v_tree,
    uint4 *const *__restrict__ k_pool, uint4 *const *__restrict__ v_pool, const int32_t *__restrict__ block_table,
    const int32_t *__restrict__ prefix_len, const int32_t *__restrict__ node_offset,
    const int32_t *__restrict__ accept_len, const int32_t *__restrict__ accept_path, int max_path,
    int32_t *__restrict__ out_slots, int32_t *__restrict__ new_len) {
  const int l = blockIdx.z;
  compact_one(d, row_bytes, k_tree[l], v_tree[l], k_pool[l], v_pool[l], block_table, prefix_len, node_offset,
              accept_len, accept_path, max_path, l == 0 ? out_slots : nullptr, l == 0 ? new_len : nullptr);
}

}  // namespace

hipError_t launch_tree_accept(int32_t B, int32_t max_nodes, const int32_t *node_offset,
                              const int32_t *parent, const int32_t *draft_ids,
                              const int32_t *target_ids, const int32_t *prev_target, int32_t max_path,
                              int32_t *accept_len, int32_t *accept_path, int32_t *out_tokens,
                              int32_t *bonus_id, hipStream_t s) {
  tree_accept_kernel<<<B, 64, 0, s>>>(max_nodes, node_offset, parent, draft_ids, target_ids, prev_target, max_path,
                                      accept_len, accept_path, out_tokens, bonus_id);
  return hipGetLastError();
}

hipError_t launch_kv_compact(const hb_attn_desc &d, const void *k_tree, const void *v_tree,
                             void *k_pool, void *v_pool, const int32_t *block_table,
                             const int32_t *prefix_len, const int32_t *node_offset,
                             const int32_t *accept_len, const int32_t *accept_path,
                             int32_t max_path, int32_t *out_slots, int32_t *new_len, hipStream_t s) {
  int row_bytes = d.head_dim * (d.dtype == HB_F32 ? 4 : 2);  // head_dim % 8 == 0, so % 16 == 0
  dim3 grid((unsigned)max_path, (unsigned)d.batch);
  kv_compact_kernel<<<grid, 256, 0, s>>>(d, row_bytes, (const uint4 *)k_tree, (const uint4 *)v_tree,
                                         (uint4 *)k_pool, (uint4 *)v_pool, block_table, prefix_len,
                                         node_offset, accept_len, accept_path, max_path, out_slots, new_len);
  return hipGetLastError();
}

hipError_t launch_kv_compact_layers(const hb_attn_desc &d, int32_t n_layers, const void *const *k_tree,
                                    const void *const *v_tree, void *const *k_pool, void *const *v_pool,
                                    const int32_t *block_table, const int32_t *prefix_len,
                                    const int32_t *node_offset, const int32_t *accept_len,
                                    const int32_t *accept_path, int32_t max_path, int32_t *out_slots,
                                    int32_t *new_len, hipStream_t s) {
  int row_bytes = d.head_dim * (d.dtype == HB_F32 ? 4 : 2);
  dim3 grid((unsigned)max_path, (unsigned)d.batch, (unsigned)n_layers);
  kv_compact_layers_kernel<<<grid, 256, 0, s>>>(d, row_bytes, (const uint4 *const *)k_tree, (const uint4 *const *)v_tree,
                                                (uint4 *const *)k_pool, (uint4 *const *)v_pool, block_table,
                                                prefix_len, node_offset, accept_len, accept_path, max_path,
                                                out_slots, new_len);
  return hipGetLastError();
}

}  // namespace hb
