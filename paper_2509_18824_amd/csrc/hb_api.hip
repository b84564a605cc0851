// Host side of libhb: argument validation, split-K planning, dispatch, error text.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>
#include <mutex>
#include "hb_internal.h"

// Row keys of hb_lmhead_argmax_noalloc: device memory that belongs to the library, one copy per
// GPU, held until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; the address kernels get is looked up once per device (scratch_on_device).
#define HB_NOALLOC_MAX_ROWS 16384
static __device__ __align__(256) unsigned long long scratch[HB_NOALLOC_MAX_ROWS];

namespace hb {

static thread_local char g_err[512] = "";

int32_t fail(int32_t code, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

int32_t fail_hip(hipError_t e, const char *what) {
  return fail(HB_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
}

// Device address of `scratch` on the current device; looked up at the first call per device.
static hipError_t scratch_on_device(unsigned long long **out) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static unsigned long long *ptrs[kMaxDevices] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptrs[dev]) {
    unsigned long long *p = nullptr;
    e = hipGetSymbolAddress((void **)&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    ptrs[dev] = p;
  }
  *out = ptrs[dev];
  return hipSuccess;
}

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
// tensors start at a 16-byte aligned address (the kernels move 16-byte pieces)
static bool misaligned(const void *p) { return ((uintptr_t)p & 15) != 0; }
static int32_t gcd32(int32_t a, int32_t b) { while (b) { int32_t t = a % b; a = b; b = t; } return a; }

static int32_t check_shape(const hb_attn_desc *d) {
  if (!d) return fail(HB_ERR_INVALID_ARG, "desc is NULL");
  if (d->dtype != HB_F32 && d->dtype != HB_BF16)
    return fail(HB_ERR_UNSUPPORTED, "dtype %d: only HB_F32 and HB_BF16 are supported", d->dtype);
  if (d->batch < 0 || d->total_nodes < 0) return fail(HB_ERR_INVALID_ARG, "negative batch or total_nodes");
  if (d->num_q_heads <= 0 || d->num_kv_heads <= 0 || d->num_q_heads % d->num_kv_heads)
    return fail(HB_ERR_INVALID_ARG, "num_q_heads %d must be a positive multiple of num_kv_heads %d",
                d->num_q_heads, d->num_kv_heads);
  if (d->head_dim <= 0 || d->head_dim % 8 || d->head_dim > 256)
    return fail(HB_ERR_UNSUPPORTED, "head_dim %d: must be a multiple of 8, at most 256", d->head_dim);
  if (d->page_size <= 0 || d->max_blocks_per_seq <= 0 || d->num_blocks <= 0)
    return fail(HB_ERR_INVALID_ARG, "page_size, max_blocks_per_seq and num_blocks must be positive");
  if ((int64_t)d->page_size * d->max_blocks_per_seq > (int64_t)1 << 30)
    return fail(HB_ERR_UNSUPPORTED, "page table covers more than 2^30 positions");
  if (d->max_nodes_per_tree <= 0) return fail(HB_ERR_INVALID_ARG, "max_nodes_per_tree must be positive");
  if (d->max_nodes_per_tree > 64)
    return fail(HB_ERR_UNSUPPORTED, "max_nodes_per_tree %d: trees of more than 64 nodes are not supported",
                d->max_nodes_per_tree);
  if (d->num_splits < 0 || d->max_prefix_len_hint < 0)
    return fail(HB_ERR_INVALID_ARG, "num_splits and max_prefix_len_hint must be >= 0");
  if (d->algo < HB_ATTN_AUTO || d->algo > HB_ATTN_MFMA) return fail(HB_ERR_INVALID_ARG, "algo %d", d->algo);
  return HB_OK;
}

int32_t make_attn_plan(const hb_attn_desc *d, AttnPlan *plan) {
  int32_t rc = check_shape(d);
  if (rc) return rc;
  bool can_mfma = attn_mfma_supports(*d);
  if (d->algo == HB_ATTN_MFMA && !can_mfma)
    return fail(HB_ERR_UNSUPPORTED,
                "HB_ATTN_MFMA needs bf16, head_dim 128, page_size 16 and (Hq/Hkv)*max_nodes_per_tree <= 512");
  plan->mfma = (d->algo == HB_ATTN_MFMA) || (d->algo == HB_ATTN_AUTO && can_mfma);
  plan->row_groups = plan->mfma ? attn_mfma_row_groups(*d) : 1;
  int64_t span = (int64_t)d->page_size * d->max_blocks_per_seq;
  if (d->max_prefix_len_hint > 0 && d->max_prefix_len_hint < span) span = d->max_prefix_len_hint;
  if (span < 1) span = 1;
  int32_t gran = d->page_size * (64 / gcd32(d->page_size, 64));  // multiple of the page and of 64
  int64_t splits = d->num_splits;
  plan->workers = 0;
  if (splits == 0) {
    if (plan->mfma) {
      // Parallelism comes first from row groups (they cost no partials), then from cutting the
      // KV: aim at eight wavefronts on each of the 256 CUs.
      const int waves = attn_mfma_waves(*d);
      const int64_t want = 256 * 8 / waves;
      if (d->batch <= 64) {
        // Work-proportional schedule, resolved on the device from prefix_len (see the kernel): a
        // fixed number of workers per kv head share the tiles of all sequences evenly.  What the
        // host fixes is the number of partial slots per row: a sequence of t tiles is cut into at
        // most ceil((t - 1) / per) + 1 pieces, per >= kMinPer tiles, and never more than there
        // are workers.
        int64_t workers = want / ((int64_t)d->num_kv_heads * plan->row_groups);
        if (workers < 1) workers = 1;
        if (workers > 4096) workers = 4096;
        const int64_t min_per = waves == 8 ? 16 : 8;  // kMinPer of the kernel
        const int64_t prefix_tiles = (span + 63) / 64;
        int64_t slots = (prefix_tiles + min_per - 1) / min_per + 1;
        if (slots > workers) slots = workers;
        plan->workers = (int32_t)workers;
        plan->splits = (int32_t)slots;
        plan->chunk_tokens = 64;  // unused by this schedule
        size_t rows = (size_t)d->total_nodes * d->num_q_heads;
        if (slots > 1) {
          plan->ml_offset = align_up(rows * slots * d->head_dim * sizeof(float), 256);
          plan->bytes = plan->ml_offset + align_up(rows * slots * 2 * sizeof(float), 256);
        } else {
          plan->ml_offset = 0;
          plan->bytes = 0;
        }
        return HB_OK;
      }
      // more sequences than one wavefront can schedule: chunks of equal length per sequence; a
      // chunk stays at 1024 tokens or more when many rows share it, 512 with few rows
      int64_t items = (int64_t)d->batch * d->num_kv_heads * plan->row_groups;
      splits = items > 0 ? (want + items - 1) / items : 1;
      const int64_t min_chunk = waves == 8 ? 1024 : 512;
      int64_t cap = (span + min_chunk - 1) / min_chunk;
      if (splits > cap) splits = cap;
    } else {
      int64_t rows = (int64_t)d->total_nodes * d->num_q_heads;
      splits = rows > 0 ? (2048 + rows - 1) / rows : 1;
      int64_t cap = (span + 255) / 256;
      if (splits > cap) splits = cap;
    }
    if (splits < 1) splits = 1;
  }
  if (splits > 1024) splits = 1024;
  int64_t chunk = (span + splits - 1) / splits;
  chunk = (chunk + gran - 1) / gran * gran;
  splits = (span + chunk - 1) / chunk;
  if (splits < 1) splits = 1;
  plan->splits = (int32_t)splits;
  plan->chunk_tokens = (int32_t)chunk;
  size_t rows = (size_t)d->total_nodes * d->num_q_heads;
  if (splits > 1) {
    plan->ml_offset = align_up(rows * splits * d->head_dim * sizeof(float), 256);
    plan->bytes = plan->ml_offset + align_up(rows * splits * 2 * sizeof(float), 256);
  } else {
    plan->ml_offset = 0;
    plan->bytes = 0;
  }
  return HB_OK;
}

}  // namespace hb

using namespace hb;

extern "C" {

const char *hb_last_error(void) { return g_err; }
int32_t hb_version(void) { return 1; }

int32_t hb_tree_validate_host(const int32_t *parent, int32_t n) {
  if (!parent) return fail(HB_ERR_INVALID_ARG, "parent is NULL");
  if (n < 1 || n > 64) return fail(HB_ERR_UNSUPPORTED, "a tree has 1..64 nodes, got %d", n);
  if (parent[0] != -1) return fail(HB_ERR_INVALID_ARG, "parent[0] must be -1, got %d", parent[0]);
  for (int32_t i = 1; i < n; ++i)
    if (parent[i] < 0 || parent[i] >= i)
      return fail(HB_ERR_INVALID_ARG, "parent[%d] = %d must lie in [0, %d)", i, parent[i], i);
  return HB_OK;
}

size_t hb_tree_verify_attn_workspace_bytes(const hb_attn_desc *desc) {
  AttnPlan plan;
  if (make_attn_plan(desc, &plan)) return 0;
  return plan.bytes;
}

int32_t hb_tree_verify_attn_num_splits(const hb_attn_desc *desc) {
  AttnPlan plan;
  if (make_attn_plan(desc, &plan)) return 0;
  return plan.splits;
}

int32_t hb_tree_verify_attn(const hb_attn_desc *desc, const void *q, const void *k_tree,
                            const void *v_tree, const void *k_pool, const void *v_pool,
                            const int32_t *block_table, const int32_t *prefix_len,
                            const int32_t *node_offset, const int32_t *parent, void *out,
                            float *lse, void *workspace, size_t workspace_bytes, void *stream) {
  AttnPlan plan;
  int32_t rc = make_attn_plan(desc, &plan);
  if (rc) return rc;
  if (desc->batch == 0 || desc->total_nodes == 0) return HB_OK;
  if (!q || !k_tree || !v_tree || !k_pool || !v_pool || !block_table || !prefix_len || !node_offset ||
      !parent || !out)
    return fail(HB_ERR_INVALID_ARG, "a required device pointer is NULL");
  if (misaligned(q) || misaligned(k_tree) || misaligned(v_tree) || misaligned(k_pool) || misaligned(v_pool) ||
      misaligned(out))
    return fail(HB_ERR_INVALID_ARG, "q, k_tree, v_tree, k_pool, v_pool and out must be 16-byte aligned");
  float *part_o = nullptr, *part_ml = nullptr;
  if (plan.splits > 1) {
    if (!workspace || workspace_bytes < plan.bytes)
      return fail(HB_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", plan.bytes,
                  workspace ? workspace_bytes : (size_t)0);
    if ((uintptr_t)workspace % 256) return fail(HB_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    part_o = (float *)workspace;
    part_ml = (float *)((char *)workspace + plan.ml_offset);
  }
  hipStream_t s = (hipStream_t)stream;
  if (plan.mfma)
    HB_HIP_TRY(launch_attn_mfma(*desc, plan, q, k_tree, v_tree, k_pool, v_pool, block_table, prefix_len,
                                node_offset, parent, out, lse, part_o, part_ml, s));
  else
    HB_HIP_TRY(launch_attn_scalar(*desc, plan, q, k_tree, v_tree, k_pool, v_pool, block_table, prefix_len,
                                  node_offset, parent, out, lse, part_o, part_ml, s));
  if (plan.splits > 1) HB_HIP_TRY(launch_attn_merge(*desc, plan, part_o, part_ml, out, lse, s));
  return HB_OK;
}

size_t hb_lmhead_argmax_workspace_bytes(int32_t M) { return M > 0 ? (size_t)M * 8 : 0; }

static int32_t check_lmhead_args(int32_t dtype, int32_t M, int32_t K, int32_t V, const void *hidden,
                                 const void *weight, const int32_t *out_ids) {
  if (dtype != HB_F32 && dtype != HB_BF16)
    return fail(HB_ERR_UNSUPPORTED, "dtype %d: only HB_F32 and HB_BF16 are supported", dtype);
  if (M < 0 || K <= 0 || V <= 0) return fail(HB_ERR_INVALID_ARG, "need M >= 0, K > 0, V > 0 (got %d, %d, %d)", M, K, V);
  if (M == 0) return HB_OK;
  if (!hidden || !weight || !out_ids) return fail(HB_ERR_INVALID_ARG, "a required device pointer is NULL");
  if (misaligned(hidden) || misaligned(weight))
    return fail(HB_ERR_INVALID_ARG, "hidden and weight must be 16-byte aligned");
  return HB_OK;
}

// init (every key starts at zero, by a fill kernel), GEMM + argmax into the keys, keys -> ids
static int32_t lmhead_enqueue(int32_t dtype, int32_t M, int32_t K, int32_t V, const void *hidden,
                              const void *weight, int32_t *out_ids, float *out_max,
                              unsigned long long *keys, hipStream_t s) {
  HB_HIP_TRY(launch_lmhead_init(keys, M, s));
  if (lmhead_mfma_supports(dtype, M, K, V))
    HB_HIP_TRY(launch_lmhead_mfma(M, K, V, hidden, weight, keys, s));
  else
    HB_HIP_TRY(launch_lmhead_scalar(dtype, M, K, V, hidden, weight, keys, s));
  HB_HIP_TRY(launch_lmhead_finish(keys, M, V, out_ids, out_max, s));
  return HB_OK;
}

int32_t hb_lmhead_argmax_noalloc_max_rows(void) { return HB_NOALLOC_MAX_ROWS; }

int32_t hb_lmhead_argmax_noalloc(int32_t dtype, int32_t M, int32_t K, int32_t V, const void *hidden,
                                 const void *weight, int32_t *out_ids, float *out_max, void *stream) {
  int32_t rc = check_lmhead_args(dtype, M, K, V, hidden, weight, out_ids);
  if (rc || M == 0) return rc;
  if (M > HB_NOALLOC_MAX_ROWS)
    return fail(HB_ERR_UNSUPPORTED, "hb_lmhead_argmax_noalloc takes at most %d rows, got %d; use hb_lmhead_argmax "
                "with a caller-provided workspace", HB_NOALLOC_MAX_ROWS, M);
  unsigned long long *keys = nullptr;
  HB_HIP_TRY(scratch_on_device(&keys));
  return lmhead_enqueue(dtype, M, K, V, hidden, weight, out_ids, out_max, keys, (hipStream_t)stream);
}

int32_t hb_lmhead_argmax(int32_t dtype, int32_t M, int32_t K, int32_t V, const void *hidden,
                         const void *weight, int32_t *out_ids, float *out_max, void *workspace,
                         size_t workspace_bytes, void *stream) {
  int32_t rc = check_lmhead_args(dtype, M, K, V, hidden, weight, out_ids);
  if (rc || M == 0) return rc;
  size_t need = hb_lmhead_argmax_workspace_bytes(M);
  if (!workspace || workspace_bytes < need)
    return fail(HB_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", need,
                workspace ? workspace_bytes : (size_t)0);
  if ((uintptr_t)workspace % 8) return fail(HB_ERR_WORKSPACE, "workspace must be 8-byte aligned");
  hipStream_t s = (hipStream_t)stream;
  unsigned long long *keys = (unsigned long long *)workspace;
  return lmhead_enqueue(dtype, M, K, V, hidden, weight, out_ids, out_max, keys, s);
}

int32_t hb_tree_positions(int32_t B, int32_t max_nodes_per_tree, int32_t total_nodes,
                          const int32_t *node_offset, const int32_t *parent, const int32_t *prefix_len,
                          int32_t *positions, void *stream) {
  if (B < 0 || total_nodes < 0 || max_nodes_per_tree <= 0)
    return fail(HB_ERR_INVALID_ARG, "need B >= 0, total_nodes >= 0, max_nodes_per_tree > 0");
  if (max_nodes_per_tree > 64)
    return fail(HB_ERR_UNSUPPORTED, "max_nodes_per_tree %d: trees of more than 64 nodes are not supported",
                max_nodes_per_tree);
  if (B == 0 || total_nodes == 0) return HB_OK;
  if (!node_offset || !parent || !prefix_len || !positions)
    return fail(HB_ERR_INVALID_ARG, "a required device pointer is NULL");
  HB_HIP_TRY(launch_tree_positions(B, max_nodes_per_tree, total_nodes, node_offset, parent, prefix_len, positions,
                                   (hipStream_t)stream));
  return HB_OK;
}

int32_t hb_rope_table(int32_t T, int32_t head_dim, double theta, const int32_t *positions, float *cos_out,
                      float *sin_out, void *stream) {
  if (T < 0 || head_dim <= 0 || head_dim % 2 || !(theta > 0.0))
    return fail(HB_ERR_INVALID_ARG, "need T >= 0, an even head_dim > 0 and theta > 0");
  if (T == 0) return HB_OK;
  if (!positions || !cos_out || !sin_out) return fail(HB_ERR_INVALID_ARG, "a required device pointer is NULL");
  HB_HIP_TRY(launch_rope_table(T, head_dim / 2, theta, positions, cos_out, sin_out, (hipStream_t)stream));
  return HB_OK;
}

// Workspace of the split-K path: usable when present, large enough and 16-byte aligned; the
// calls fall back to one workgroup per tile otherwise.
static float *proj_part(int32_t T, int32_t K, int32_t N, void *workspace, size_t workspace_bytes) {
  const size_t need = proj_workspace_bytes(T, K, N);
  if (need == 0 || !workspace || workspace_bytes < need || misaligned(workspace)) return nullptr;
  return (float *)workspace;
}

size_t hb_proj_workspace_bytes(int32_t T, int32_t K, int32_t N) {
  return (T > 0 && K > 0 && N > 0) ? proj_workspace_bytes(T, K, N) : 0;
}

static int32_t qkv_rope_project(int32_t T, int32_t K, int32_t Hq, int32_t Hkv, int32_t head_dim, const void *hidden,
                                const void *w_qkv, const void *bias_or_null, const float *cos, const float *sin,
                                void *q, void *k, void *v, void *workspace, size_t workspace_bytes, void *stream) {
  if (T < 0 || K <= 0 || Hq <= 0 || Hkv <= 0) return fail(HB_ERR_INVALID_ARG, "need T >= 0 and K, Hq, Hkv > 0");
  if (head_dim != 128) return fail(HB_ERR_UNSUPPORTED, "head_dim %d: the fused projection takes head_dim 128", head_dim);
  if (K % 64) return fail(HB_ERR_UNSUPPORTED, "K %d: must be a multiple of 64", K);
  if ((int64_t)(Hq + 2 * Hkv) * 128 > (int64_t)1 << 24) return fail(HB_ERR_UNSUPPORTED, "too many heads");
  if (T == 0) return HB_OK;
  if (!hidden || !w_qkv || !cos || !sin || !q || !k || !v)
    return fail(HB_ERR_INVALID_ARG, "a required device pointer is NULL");
  if (misaligned(hidden) || misaligned(w_qkv) || misaligned(cos) || misaligned(sin) || misaligned(q) || misaligned(k) ||
      misaligned(v) || (bias_or_null && misaligned(bias_or_null)))
    return fail(HB_ERR_INVALID_ARG, "tensors must be 16-byte aligned");
  HB_HIP_TRY(launch_qkv_rope(T, K, Hq, Hkv, hidden, w_qkv, bias_or_null, cos, sin, q, k, v,
                             proj_part(T, K, (Hq + 2 * Hkv) * 128, workspace, workspace_bytes), (hipStream_t)stream));
  return HB_OK;
}

static int32_t out_project(int32_t T, int32_t K, int32_t N, const void *x, const void *w, const void *residual_or_null,
                           void *out, void *workspace, size_t workspace_bytes, void *stream) {
  if (T < 0 || K <= 0 || N <= 0) return fail(HB_ERR_INVALID_ARG, "need T >= 0 and K, N > 0");
  if (K % 64 || N % 4) return fail(HB_ERR_UNSUPPORTED, "K %d must be a multiple of 64 and N %d of 4", K, N);
  if (T == 0) return HB_OK;
  if (!x || !w || !out) return fail(HB_ERR_INVALID_ARG, "a required device pointer is NULL");
  if (misaligned(x) || misaligned(w) || misaligned(out) || (residual_or_null && misaligned(residual_or_null)))
    return fail(HB_ERR_INVALID_ARG, "tensors must be 16-byte aligned");
  HB_HIP_TRY(launch_linear(T, K, N, x, w, residual_or_null, out, proj_part(T, K, N, workspace, workspace_bytes),
                           (hipStream_t)stream));
  return HB_OK;
}

int32_t hb_qkv_rope_project(int32_t T, int32_t K, int32_t Hq, int32_t Hkv, int32_t head_dim, const void *hidden,
                            const void *w_qkv, const void *bias_or_null, const float *cos, const float *sin,
                            void *q, void *k, void *v, void *stream) {
  return qkv_rope_project(T, K, Hq, Hkv, head_dim, hidden, w_qkv, bias_or_null, cos, sin, q, k, v, nullptr, 0, stream);
}

int32_t hb_qkv_rope_project_ws(int32_t T, int32_t K, int32_t Hq, int32_t Hkv, int32_t head_dim, const void *hidden,
                               const void *w_qkv, const void *bias_or_null, const float *cos, const float *sin,
                               void *q, void *k, void *v, void *workspace, size_t workspace_bytes, void *stream) {
  return qkv_rope_project(T, K, Hq, Hkv, head_dim, hidden, w_qkv, bias_or_null, cos, sin, q, k, v, workspace,
                          workspace_bytes, stream);
}

int32_t hb_out_project(int32_t T, int32_t K, int32_t N, const void *x, const void *w,
                       const void *residual_or_null, void *out, void *stream) {
  return out_project(T, K, N, x, w, residual_or_null, out, nullptr, 0, stream);
}

int32_t hb_out_project_ws(int32_t T, int32_t K, int32_t N, const void *x, const void *w,
                          const void *residual_or_null, void *out, void *workspace, size_t workspace_bytes,
                          void *stream) {
  return out_project(T, K, N, x, w, residual_or_null, out, workspace, workspace_bytes, stream);
}

int32_t hb_swiglu_project(int32_t T, int32_t K, int32_t F, const void *x, const void *w_gate_up, void *out,
                          void *workspace_or_null, size_t workspace_bytes, void *stream) {
  if (T < 0 || K <= 0 || F <= 0) return fail(HB_ERR_INVALID_ARG, "need T >= 0 and K, F > 0");
  if (K % 64 || F % 4) return fail(HB_ERR_UNSUPPORTED, "K %d must be a multiple of 64 and F %d of 4", K, F);
  if ((int64_t)F > (int64_t)1 << 24) return fail(HB_ERR_UNSUPPORTED, "F %d: too many features", F);
  if (T == 0) return HB_OK;
  if (!x || !w_gate_up || !out) return fail(HB_ERR_INVALID_ARG, "a required device pointer is NULL");
  if (misaligned(x) || misaligned(w_gate_up) || misaligned(out))
    return fail(HB_ERR_INVALID_ARG, "tensors must be 16-byte aligned");
  HB_HIP_TRY(launch_swiglu(T, K, F, x, w_gate_up, out, proj_part(T, K, 2 * F, workspace_or_null, workspace_bytes),
                           (hipStream_t)stream));
  return HB_OK;
}

int32_t hb_rmsnorm(int32_t T, int32_t K, const void *x, const void *weight, float eps, void *out, void *stream) {
  if (T < 0 || K <= 0) return fail(HB_ERR_INVALID_ARG, "need T >= 0 and K > 0");
  if (!(eps >= 0.f)) return fail(HB_ERR_INVALID_ARG, "eps must be >= 0");
  if (K % 8) return fail(HB_ERR_UNSUPPORTED, "K %d must be a multiple of 8", K);
  if (T == 0) return HB_OK;
  if (!x || !weight || !out) return fail(HB_ERR_INVALID_ARG, "a required device pointer is NULL");
  if (misaligned(x) || misaligned(weight) || misaligned(out))
    return fail(HB_ERR_INVALID_ARG, "tensors must be 16-byte aligned");
  HB_HIP_TRY(launch_rmsnorm(T, K, x, weight, eps, out, (hipStream_t)stream));
  return HB_OK;
}

int32_t hb_tree_accept(int32_t B, int32_t max_nodes_per_tree, const int32_t *node_offset,
                       const int32_t *parent, const int32_t *draft_ids, const int32_t *target_ids,
                       const int32_t *prev_target_or_null, int32_t max_path, int32_t *accept_len,
                       int32_t *accept_path, int32_t *out_tokens, int32_t *bonus_id, void *stream) {
  if (B < 0 || max_path <= 0 || max_nodes_per_tree <= 0)
    return fail(HB_ERR_INVALID_ARG, "need B >= 0, max_path > 0, max_nodes_per_tree > 0");
  if (max_nodes_per_tree > 64)
    return fail(HB_ERR_UNSUPPORTED, "max_nodes_per_tree %d: trees of more than 64 nodes are not supported",
                max_nodes_per_tree);
  if (B == 0) return HB_OK;
  if (!node_offset || !parent || !draft_ids || !target_ids || !accept_len || !accept_path || !out_tokens ||
      !bonus_id)
    return fail(HB_ERR_INVALID_ARG, "a required device pointer is NULL");
  HB_HIP_TRY(launch_tree_accept(B, max_nodes_per_tree, node_offset, parent, draft_ids, target_ids,
                                prev_target_or_null, max_path,
                                accept_len, accept_path, out_tokens, bonus_id, (hipStream_t)stream));
  return HB_OK;
}

size_t hb_tree_accept_sample_workspace_bytes(int32_t B, int32_t V) {
  return (B > 0 && V > 0) ? (size_t)B * (size_t)V * sizeof(uint32_t) : 0;
}

int32_t hb_tree_accept_sample(int32_t B, int32_t max_nodes_per_tree, int32_t V, const int32_t *node_offset,
                              const int32_t *parent, const int32_t *draft_ids, const float *p_target,
                              const float *q_draft, const uint32_t *u_accept, const uint32_t *u_bonus,
                              int32_t max_path, int32_t *accept_len, int32_t *accept_path,
                              int32_t *out_tokens, int32_t *bonus_id, void *workspace,
                              size_t workspace_bytes, void *stream) {
  if (B < 0 || max_path <= 0 || max_nodes_per_tree <= 0 || V <= 0)
    return fail(HB_ERR_INVALID_ARG, "need B >= 0, max_path > 0, max_nodes_per_tree > 0, V > 0");
  if (max_nodes_per_tree > 64)
    return fail(HB_ERR_UNSUPPORTED, "max_nodes_per_tree %d: trees of more than 64 nodes are not supported",
                max_nodes_per_tree);
  if (B == 0) return HB_OK;
  if (!node_offset || !parent || !draft_ids || !p_target || !q_draft || !u_accept || !u_bonus || !accept_len ||
      !accept_path || !out_tokens || !bonus_id)
    return fail(HB_ERR_INVALID_ARG, "a required device pointer is NULL");
  const size_t need = hb_tree_accept_sample_workspace_bytes(B, V);
  if (!workspace || workspace_bytes < need)
    return fail(HB_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", need,
                workspace ? workspace_bytes : (size_t)0);
  if ((uintptr_t)workspace % 4) return fail(HB_ERR_WORKSPACE, "workspace must be 4-byte aligned");
  HB_HIP_TRY(launch_tree_accept_sample(B, max_nodes_per_tree, V, node_offset, parent, draft_ids, p_target, q_draft,
                                       u_accept, u_bonus, max_path, accept_len, accept_path, out_tokens, bonus_id,
                                       (uint32_t *)workspace, (hipStream_t)stream));
  return HB_OK;
}

size_t hb_topk_logprob_workspace_bytes(int32_t M, int32_t V, int32_t k) {
  return (M > 0 && V > 0 && k > 0) ? topk_workspace_bytes(M, V, k) : 0;
}

int32_t hb_topk_logprob(int32_t dtype, int32_t M, int32_t V, int32_t k, const void *logits, int32_t *out_ids,
                        float *out_logp, void *workspace, size_t workspace_bytes, void *stream) {
  if (dtype != HB_F32 && dtype != HB_BF16) return fail(HB_ERR_INVALID_ARG, "dtype %d", dtype);
  if (M < 0 || V <= 0 || k < 1 || k > V) return fail(HB_ERR_INVALID_ARG, "need M >= 0, V > 0, 1 <= k <= V");
  if (k > 32) return fail(HB_ERR_UNSUPPORTED, "k %d: at most 32 tokens per row", k);
  if (M > 65535) return fail(HB_ERR_UNSUPPORTED, "M %d: at most 65535 rows per call", M);
  if (M == 0) return HB_OK;
  if (!logits || !out_ids || !out_logp) return fail(HB_ERR_INVALID_ARG, "a required device pointer is NULL");
  if ((uintptr_t)logits % (dtype == HB_BF16 ? 2 : 4)) return fail(HB_ERR_INVALID_ARG, "logits are not aligned to their type");
  const size_t need = hb_topk_logprob_workspace_bytes(M, V, k);
  if (!workspace || workspace_bytes < need)
    return fail(HB_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", need,
                workspace ? workspace_bytes : (size_t)0);
  if ((uintptr_t)workspace % 8) return fail(HB_ERR_WORKSPACE, "workspace must be 8-byte aligned");
  HB_HIP_TRY(launch_topk_logprob(dtype, M, V, k, logits, out_ids, out_logp, workspace, (hipStream_t)stream));
  return HB_OK;
}

int32_t hb_draft_tree_candidates(int32_t K, int32_t T) {
  if (K < 1 || T < 1 || K > 32 || T > 64) return 0;
  return K + (T - 1) * K * K;
}

int32_t hb_tree_grow(int32_t B, int32_t K, int32_t T, int32_t level, const int32_t *child_ids,
                     const float *child_logp, float *cand_score, int32_t *cand_token, int32_t *cand_parent,
                     int32_t *frontier, int32_t *frontier_slot, void *stream) {
  if (B < 0 || K < 1 || T < 1 || level < 0 || level >= T)
    return fail(HB_ERR_INVALID_ARG, "need B >= 0, K >= 1, T >= 1, 0 <= level < T");
  if (K > 32 || T > 64) return fail(HB_ERR_UNSUPPORTED, "K %d, T %d: at most 32 children per node and 64 levels", K, T);
  if (B == 0) return HB_OK;
  if (!child_ids || !child_logp || !cand_score || !cand_token || !cand_parent || !frontier || !frontier_slot)
    return fail(HB_ERR_INVALID_ARG, "a required device pointer is NULL");
  HB_HIP_TRY(launch_tree_grow(B, K, level, hb_draft_tree_candidates(K, T), child_ids, child_logp, cand_score,
                              cand_token, cand_parent, frontier, frontier_slot, (hipStream_t)stream));
  return HB_OK;
}

int32_t hb_tree_finalize(int32_t B, int32_t K, int32_t T, int32_t n_nodes, const float *cand_score,
                         const int32_t *cand_token, const int32_t *cand_parent, const int32_t *root_token,
                         int32_t *node_offset, int32_t *parent, int32_t *draft_ids, int32_t *depth,
                         uint64_t *anc_mask, int32_t *node_cand, float *node_score, void *stream) {
  if (B < 0 || K < 1 || T < 1) return fail(HB_ERR_INVALID_ARG, "need B >= 0, K >= 1, T >= 1");
  if (K > 32 || T > 64) return fail(HB_ERR_UNSUPPORTED, "K %d, T %d: at most 32 children per node and 64 levels", K, T);
  const int32_t C = hb_draft_tree_candidates(K, T);
  if (C > 4096) return fail(HB_ERR_UNSUPPORTED, "%d candidates per sequence: at most 4096", C);
  if (n_nodes < 1 || n_nodes - 1 > C) return fail(HB_ERR_INVALID_ARG, "n_nodes %d with %d candidates", n_nodes, C);
  if (n_nodes > 64) return fail(HB_ERR_UNSUPPORTED, "n_nodes %d: trees of more than 64 nodes are not supported", n_nodes);
  if ((int64_t)B * n_nodes > INT32_MAX) return fail(HB_ERR_INVALID_ARG, "B * n_nodes overflows int32");
  if (B == 0) return HB_OK;
  if (!cand_score || !cand_token || !cand_parent || !root_token || !node_offset || !parent || !draft_ids || !depth ||
      !anc_mask || !node_cand || !node_score)
    return fail(HB_ERR_INVALID_ARG, "a required device pointer is NULL");
  HB_HIP_TRY(launch_tree_finalize(B, C, n_nodes, cand_score, cand_token, cand_parent, root_token, node_offset, parent,
                                  draft_ids, depth, (unsigned long long *)anc_mask, node_cand, node_score,
                                  (hipStream_t)stream));
  return HB_OK;
}

static int32_t check_meta_shape(int32_t L, int32_t D, int32_t H, int32_t Q) {
  if (L < 1 || D < 1 || H < 1 || Q < 1) return fail(HB_ERR_INVALID_ARG, "need L, D, H, Q >= 1");
  if (D % H) return fail(HB_ERR_INVALID_ARG, "H %d does not divide D %d", H, D);
  if (D % 256 || (D / H) % 8)
    return fail(HB_ERR_UNSUPPORTED, "D %d must be a multiple of 256 and the head size %d of 8", D, D / H);
  if (Q > 4 || (int64_t)H * Q > 96 || L > 32)
    return fail(HB_ERR_UNSUPPORTED, "at most 4 queries, 96 (head, query) rows and 32 layers (Q %d, H %d, L %d)", Q, H, L);
  return HB_OK;
}

size_t hb_meta_query_fold_bytes(int32_t Q, int32_t D, int32_t H) {
  if (Q < 1 || D < 1 || H < 1) return 0;
  return (size_t)2 * meta_rows_pad(H, Q) * (size_t)D * sizeof(bf16_t);
}

int32_t hb_meta_query_fold(int32_t Q, int32_t D, int32_t H, const void *f_q, const void *w_q, const void *w_k,
                           void *a_fold, void *workspace, size_t workspace_bytes, void *stream) {
  int32_t rc = check_meta_shape(1, D, H, Q);
  if (rc) return rc;
  if (!f_q || !w_q || !w_k || !a_fold) return fail(HB_ERR_INVALID_ARG, "a required device pointer is NULL");
  if (misaligned(f_q) || misaligned(w_q) || misaligned(w_k) || misaligned(a_fold))
    return fail(HB_ERR_INVALID_ARG, "tensors must be 16-byte aligned");
  const size_t need = (size_t)Q * D * sizeof(float);
  if (!workspace || workspace_bytes < need)
    return fail(HB_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", need,
                workspace ? workspace_bytes : (size_t)0);
  if ((uintptr_t)workspace % 4) return fail(HB_ERR_WORKSPACE, "workspace must be 4-byte aligned");
  HB_HIP_TRY(launch_meta_fold(Q, D, H, f_q, w_q, w_k, a_fold, (float *)workspace, (hipStream_t)stream));
  return HB_OK;
}

size_t hb_meta_query_attn_workspace_bytes(int32_t S, int32_t D, int32_t H, int32_t Q) {
  if (S < 1 || check_meta_shape(1, D, H, Q)) return 0;
  return meta_attn_workspace_bytes(S, D, H, Q);
}

int32_t hb_meta_query_attn(int32_t S, int32_t L, int32_t D, int32_t H, int32_t Q, const void *feats,
                           const void *v_proj, const void *a_fold, const int32_t *residual_layers_or_null,
                           void *pre, void *residual_out_or_null, void *workspace, size_t workspace_bytes,
                           void *stream) {
  if (S < 0) return fail(HB_ERR_INVALID_ARG, "S must be >= 0");
  int32_t rc = check_meta_shape(L, D, H, Q);
  if (rc) return rc;
  if (residual_layers_or_null) {
    for (int q = 0; q < Q; ++q)
      if (residual_layers_or_null[q] < 0 || residual_layers_or_null[q] >= L)
        return fail(HB_ERR_INVALID_ARG, "residual layer %d of query %d outside [0, %d)", residual_layers_or_null[q], q, L);
    if (!residual_out_or_null) return fail(HB_ERR_INVALID_ARG, "residual layers given without residual_out");
  }
  if (S == 0) return HB_OK;
  if (!feats || !v_proj || !a_fold || !pre) return fail(HB_ERR_INVALID_ARG, "a required device pointer is NULL");
  if (misaligned(feats) || misaligned(v_proj) || misaligned(a_fold) || misaligned(pre) ||
      (residual_out_or_null && misaligned(residual_out_or_null)))
    return fail(HB_ERR_INVALID_ARG, "tensors must be 16-byte aligned");
  const size_t need = meta_attn_workspace_bytes(S, D, H, Q);
  if (!workspace || workspace_bytes < need)
    return fail(HB_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", need,
                workspace ? workspace_bytes : (size_t)0);
  if ((uintptr_t)workspace % 4) return fail(HB_ERR_WORKSPACE, "workspace must be 4-byte aligned");
  HB_HIP_TRY(launch_meta_attn(S, L, D, H, Q, feats, v_proj, a_fold, residual_layers_or_null, pre,
                              residual_layers_or_null ? residual_out_or_null : nullptr, (float *)workspace,
                              (hipStream_t)stream));
  return HB_OK;
}

int32_t hb_kv_compact(const hb_attn_desc *desc, const void *k_tree, const void *v_tree,
                      void *k_pool, void *v_pool, const int32_t *block_table,
                      const int32_t *prefix_len, const int32_t *node_offset,
                      const int32_t *accept_len, const int32_t *accept_path, int32_t max_path,
                      int32_t *out_slots, int32_t *new_len, void *stream) {
  int32_t rc = check_shape(desc);
  if (rc) return rc;
  if (max_path <= 0) return fail(HB_ERR_INVALID_ARG, "max_path must be positive");
  if (desc->batch == 0) return HB_OK;
  if (!k_tree || !v_tree || !k_pool || !v_pool || !block_table || !prefix_len || !node_offset ||
      !accept_len || !accept_path)
    return fail(HB_ERR_INVALID_ARG, "a required device pointer is NULL");
  if (misaligned(k_tree) || misaligned(v_tree) || misaligned(k_pool) || misaligned(v_pool))
    return fail(HB_ERR_INVALID_ARG, "k_tree, v_tree, k_pool and v_pool must be 16-byte aligned");
  HB_HIP_TRY(launch_kv_compact(*desc, k_tree, v_tree, k_pool, v_pool, block_table, prefix_len, node_offset,
                               accept_len, accept_path, max_path, out_slots, new_len, (hipStream_t)stream));
  return HB_OK;
}

int32_t hb_kv_compact_layers(const hb_attn_desc *desc, int32_t n_layers, const void *const *k_tree,
                             const void *const *v_tree, void *const *k_pool, void *const *v_pool,
                             const int32_t *block_table, const int32_t *prefix_len, const int32_t *node_offset,
                             const int32_t *accept_len, const int32_t *accept_path, int32_t max_path,
                             int32_t *out_slots, int32_t *new_len, void *stream) {
  int32_t rc = check_shape(desc);
  if (rc) return rc;
  if (max_path <= 0 || n_layers < 0) return fail(HB_ERR_INVALID_ARG, "need max_path > 0 and n_layers >= 0");
  if (n_layers > 65535) return fail(HB_ERR_UNSUPPORTED, "n_layers %d: at most 65535 layers per call", n_layers);
  if (desc->batch == 0 || n_layers == 0) return HB_OK;
  if (!k_tree || !v_tree || !k_pool || !v_pool || !block_table || !prefix_len || !node_offset || !accept_len ||
      !accept_path)
    return fail(HB_ERR_INVALID_ARG, "a required device pointer is NULL");
  if (((uintptr_t)k_tree | (uintptr_t)v_tree | (uintptr_t)k_pool | (uintptr_t)v_pool) & 7)
    return fail(HB_ERR_INVALID_ARG, "the pointer tables must be 8-byte aligned");
  HB_HIP_TRY(launch_kv_compact_layers(*desc, n_layers, k_tree, v_tree, k_pool, v_pool, block_table, prefix_len,
                                      node_offset, accept_len, accept_path, max_path, out_slots, new_len,
                                      (hipStream_t)stream));
  return HB_OK;
}

}  // extern "C"
