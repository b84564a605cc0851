// Scalar tree-verify attention: one wavefront per (node, query head, KV chunk), lanes spread
// over the head dimension, fp32 arithmetic whatever the storage type.  It is the kernel for
// fp32 inputs and for shapes the MFMA kernel does not take, and it defines the semantics the
// fast kernel must match: keys are the prefix positions of the chunk, plus (chunk 0 only) the
// tree nodes on the node's own root path.  Also holds the split-K merge kernel.
#include "hb_internal.h"

namespace hb {

namespace {

constexpr int kMaxPerLane = 4;  // head_dim <= 256 = 64 lanes * 4

__device__ inline float wave_sum(float x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
  return x;
}

struct OnlineSoftmax {
  float m, l;
  float acc[kMaxPerLane];
};

template <typename T>
__device__ inline void absorb_key(OnlineSoftmax &st, const float (&qv)[kMaxPerLane], const T *krow,
                                  const T *vrow, int D, int lane, float scale) {
  float part = 0.f;
  float vv[kMaxPerLane];
#pragma unroll
  for (int e = 0; e < kMaxPerLane; ++e) {
    int d = lane + 64 * e;
    float kd = 0.f;
    vv[e] = 0.f;
    if (d < D) {
      kd = load_f32(krow + d);
      vv[e] = load_f32(vrow + d);
    }
    // select, not multiply: a lane past D contributes exactly zero
    part += (d < D) ? qv[e] * kd : 0.f;
  }
  float s = wave_sum(part) * scale;
  float m_new = fmaxf(st.m, s);
  float corr = expf(st.m - m_new);  // exp(-inf) = 0 on the first key
  float p = expf(s - m_new);
  st.l = st.l * corr + p;
#pragma unroll
  for (int e = 0; e < kMaxPerLane; ++e) st.acc[e] = st.acc[e] * corr + p * vv[e];
  st.m = m_new;
}

template <typename T>
__global__ __launch_bounds__(64) void attn_scalar_kernel(
    hb_attn_desc d, int splits, int chunk_tokens, const T *__restrict__ q, const T *__restrict__ k_tree,
    const T *__restrict__ v_tree, const T *__restrict__ k_pool, const T *__restrict__ v_pool,
    const int32_t *__restrict__ block_table, const int32_t *__restrict__ prefix_len,
    const int32_t *__restrict__ node_offset, const int32_t *__restrict__ parent, T *__restrict__ out,
    float *__restrict__ lse, float *__restrict__ part_o, float *__restrict__ part_ml) {
  const int lane = threadIdx.x;
  const int row = blockIdx.x;  // node * Hq + head
  const int c = blockIdx.y;
  const int node = row / d.num_q_heads;
  const int h = row - node * d.num_q_heads;
  const int g = h / (d.num_q_heads / d.num_kv_heads);
  const int D = d.head_dim;

  // sequence of this node: largest b with node_offset[b] <= node
  int lo = 0, hi = d.batch;  // invariant: node_offset[lo] <= node < node_offset[hi] (if well formed)
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (node_offset[mid] <= node) lo = mid; else hi = mid;
  }
  const int b = lo;
  const int n0 = node_offset[b];
  int n_nodes = node_offset[b + 1] - n0;
  if (n_nodes > d.max_nodes_per_tree) n_nodes = d.max_nodes_per_tree;
  int L = prefix_len[b];
  const int cap = d.max_blocks_per_seq * d.page_size;
  L = L < 0 ? 0 : (L > cap ? cap : L);

  float qv[kMaxPerLane];
#pragma unroll
  for (int e = 0; e < kMaxPerLane; ++e) {
    int dd = lane + 64 * e;
    qv[e] = dd < D ? load_f32(q + (size_t)row * D + dd) : 0.f;
  }
  OnlineSoftmax st;
  st.m = -__builtin_huge_valf();
  st.l = 0.f;
#pragma unroll
  for (int e = 0; e < kMaxPerLane; ++e) st.acc[e] = 0.f;

  int begin = c * chunk_tokens;
  int end = (c == splits - 1) ? L : min(L, begin + chunk_tokens);
  const size_t page_stride = (size_t)d.num_kv_heads * d.page_size * D;
  for (int p = begin; p < end; ++p) {
    int blk = block_table[(size_t)b * d.max_blocks_per_seq + p / d.page_size];
    blk = blk < 0 ? 0 : (blk >= d.num_blocks ? d.num_blocks - 1 : blk);
    size_t off = (size_t)blk * page_stride + ((size_t)g * d.page_size + p % d.page_size) * D;
    absorb_key(st, qv, k_pool + off, v_pool + off, D, lane, d.softmax_scale);
  }
  if (c == 0) {
    // walk up from the node to the root; every visited node is on the node's own path
    int x = node - n0;
    if (x >= n_nodes) x = -1;
    for (int guard = 0; x >= 0 && guard < 64; ++guard) {
      size_t off = ((size_t)(n0 + x) * d.num_kv_heads + g) * D;
      absorb_key(st, qv, k_tree + off, v_tree + off, D, lane, d.softmax_scale);
      int px = parent[n0 + x];
      x = (px < x) ? px : -1;  // a malformed parent ends the walk
    }
  }

  if (splits == 1) {
    float inv = st.l > 0.f ? 1.f / st.l : 0.f;
#pragma unroll
    for (int e = 0; e < kMaxPerLane; ++e) {
      int dd = lane + 64 * e;
      if (dd < D) store_f32(out + (size_t)row * D + dd, st.acc[e] * inv);
    }
    if (lse && lane == 0) lse[row] = st.m + logf(st.l);
  } else {
    size_t slot = (size_t)row * splits + c;
#pragma unroll
    for (int e = 0; e < kMaxPerLane; ++e) {
      int dd = lane + 64 * e;
      if (dd < D) part_o[slot * D + dd] = st.acc[e];
    }
    if (lane == 0) {
      part_ml[slot * 2 + 0] = st.m;
      part_ml[slot * 2 + 1] = st.l;
    }
  }
}

// out[row] = sum_c O_c e^{m_c - m} / sum_c l_c e^{m_c - m}; chunks with l_c == 0 are empty and
// their O_c was never written.  One thread per four consecutive d of a row (D / 4 threads per
// row, 16-byte loads and stores); every thread reads its row's (m_c, l_c) pairs itself (they are
// a few cached bytes), and the loads of up to kMergeBatch chunks are issued together before any
// arithmetic, so the kernel runs at memory rate instead of one chunk latency at a time.
constexpr int kMergeBatch = 8;
typedef float merge_f32x4 __attribute__((ext_vector_type(4)));
typedef float merge_f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t merge_u32x2 __attribute__((ext_vector_type(2)));

__device__ inline void store_row4(float *p, merge_f32x4 v) { *reinterpret_cast<merge_f32x4 *>(p) = v; }
__device__ inline void store_row4(bf16_t *p, merge_f32x4 v) {
  merge_u32x2 w;
  w.x = (uint32_t)f32_to_bf16(v.x) | ((uint32_t)f32_to_bf16(v.y) << 16);
  w.y = (uint32_t)f32_to_bf16(v.z) | ((uint32_t)f32_to_bf16(v.w) << 16);
  *reinterpret_cast<merge_u32x2 *>(p) = w;
}

template <typename T>
__global__ __launch_bounds__(256) void attn_merge_kernel(int rows, int D, int splits,
                                                         const float *__restrict__ part_o,
                                                         const float *__restrict__ part_ml,
                                                         T *__restrict__ out, float *__restrict__ lse) {
  const int tpr = D >> 2;  // threads per row (D % 4 == 0)
  const long gid = (long)blockIdx.x * 256 + threadIdx.x;
  const int row = (int)(gid / tpr);
  const int piece = (int)(gid - (long)row * tpr);
  if (row >= rows) return;
  const merge_f32x2 *ml = reinterpret_cast<const merge_f32x2 *>(part_ml) + (size_t)row * splits;
  // Chunks are filled from slot 0 on and empty ones only follow non-empty ones (a chunk that
  // holds any key has l > 0), so the first empty slot ends the list; producers need to mark
  // only that one.
  // Slots are read kMergeBatch at a time (independent loads: one round trip per batch instead
  // of one per slot).
  float m = -__builtin_huge_valf();
  int live = 0;
  bool open = true;
  for (int c0 = 0; c0 < splits && open; c0 += kMergeBatch) {
    merge_f32x2 x[kMergeBatch];
#pragma unroll
    for (int i = 0; i < kMergeBatch; ++i) {
      x[i] = (merge_f32x2){0.f, 0.f};
      if (c0 + i < splits) x[i] = ml[c0 + i];
    }
    if (c0 == 0 && x[0].y < 0.f) return;  // the attention kernel wrote this row out itself (row sums are never negative)
#pragma unroll
    for (int i = 0; i < kMergeBatch; ++i) {
      open = open && x[i].y > 0.f;
      m = open ? fmaxf(m, x[i].x) : m;
      live += open ? 1 : 0;
    }
  }
  const merge_f32x4 *po = reinterpret_cast<const merge_f32x4 *>(part_o) + (size_t)row * splits * tpr + piece;
  float l = 0.f;
  merge_f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int c0 = 0; c0 < live; c0 += kMergeBatch) {
    float w[kMergeBatch];
    merge_f32x4 o[kMergeBatch];
#pragma unroll
    for (int i = 0; i < kMergeBatch; ++i) {
      const int c = c0 + i;
      merge_f32x2 x = {0.f, 0.f};
      if (c < live) x = ml[c];
      const bool ok = c < live;
      w[i] = ok ? expf(x.x - m) : 0.f;
      l += ok ? x.y * w[i] : 0.f;
      merge_f32x4 v = {0.f, 0.f, 0.f, 0.f};
      if (ok) v = po[(size_t)c * tpr];  // an empty chunk's slot is never read
      o[i] = v;
    }
#pragma unroll
    for (int i = 0; i < kMergeBatch; ++i) acc += o[i] * w[i];
  }
  const float inv = l > 0.f ? 1.f / l : 0.f;
  store_row4(out + (size_t)row * D + piece * 4, acc * inv);
  if (lse && piece == 0) lse[row] = m + logf(l);
}

}  // namespace

hipError_t launch_attn_scalar(const hb_attn_desc &d, const AttnPlan &plan, const void *q,
                              const void *k_tree, const void *v_tree, const void *k_pool,
                              const void *v_pool, const int32_t *block_table,
                              const int32_t *prefix_len, const int32_t *node_offset,
                              const int32_t *parent, void *out, float *lse, float *part_o,
                              float *part_ml, hipStream_t s) {
  dim3 grid((unsigned)(d.total_nodes * d.num_q_heads), (unsigned)plan.splits);
  if (d.dtype == HB_F32)
    attn_scalar_kernel<float><<<grid, 64, 0, s>>>(d, plan.splits, plan.chunk_tokens, (const float *)q,
        (const float *)k_tree, (const float *)v_tree, (const float *)k_pool, (const float *)v_pool,
        block_table, prefix_len, node_offset, parent, (float *)out, lse, part_o, part_ml);
  else
    attn_scalar_kernel<bf16_t><<<grid, 64, 0, s>>>(d, plan.splits, plan.chunk_tokens, (const bf16_t *)q,
        (const bf16_t *)k_tree, (const bf16_t *)v_tree, (const bf16_t *)k_pool, (const bf16_t *)v_pool,
        block_table, prefix_len, node_offset, parent, (bf16_t *)out, lse, part_o, part_ml);
  return hipGetLastError();
}

hipError_t launch_attn_merge(const hb_attn_desc &d, const AttnPlan &plan, const float *part_o,
                             const float *part_ml, void *out, float *lse, hipStream_t s) {
  int rows = d.total_nodes * d.num_q_heads;
  long threads = (long)rows * (d.head_dim / 4);
  dim3 grid((unsigned)((threads + 255) / 256));
  if (d.dtype == HB_F32)
    attn_merge_kernel<float><<<grid, 256, 0, s>>>(rows, d.head_dim, plan.splits, part_o, part_ml, (float *)out, lse);
  else
    attn_merge_kernel<bf16_t><<<grid, 256, 0, s>>>(rows, d.head_dim, plan.splits, part_o, part_ml, (bf16_t *)out, lse);
  return hipGetLastError();
}

}  // namespace hb
