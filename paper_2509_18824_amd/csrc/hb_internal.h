// Internal declarations shared by the translation units of libhb (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "hb.h"

namespace hb {

// thread-local error text behind hb_last_error()
int32_t fail(int32_t code, const char *fmt, ...);
int32_t fail_hip(hipError_t e, const char *what);

#define HB_HIP_TRY(expr)                                  \
  do {                                                    \
    hipError_t e__ = (expr);                              \
    if (e__ != hipSuccess) return ::hb::fail_hip(e__, #expr); \
  } while (0)

// ---- storage helpers --------------------------------------------------------------------
typedef uint16_t bf16_t;  // upper half of an IEEE float32

__host__ __device__ inline float bf16_to_f32(bf16_t x) {
  union { uint32_t u; float f; } c;
  c.u = (uint32_t)x << 16;
  return c.f;
}

// round to nearest even; NaN stays NaN (quiet)
__host__ __device__ inline bf16_t f32_to_bf16(float f) {
  union { uint32_t u; float f; } c;
  c.f = f;
  uint32_t u = c.u;
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x0040u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

template <typename T> __device__ inline float load_f32(const T *p);
template <> __device__ inline float load_f32<float>(const float *p) { return *p; }
template <> __device__ inline float load_f32<bf16_t>(const bf16_t *p) { return bf16_to_f32(*p); }
template <typename T> __device__ inline void store_f32(T *p, float v);
template <> __device__ inline void store_f32<float>(float *p, float v) { *p = v; }
template <> __device__ inline void store_f32<bf16_t>(bf16_t *p, float v) { *p = f32_to_bf16(v); }

// ---- split-K plan -----------------------------------------------------------------------
// A sequence's prefix is cut into `splits` chunks of `chunk_tokens` tokens (a multiple of the
// page size and of the kernels' key tile).  Chunk 0 also takes the tree keys.  Partials of
// row R = node * Hq + head and chunk c live at  part_o[(R * splits + c) * D .. +D)  (fp32,
// un-normalised) and part_ml[(R * splits + c) * 2 .. +2) = (running max, running sum).
struct AttnPlan {
  int32_t splits;
  int32_t chunk_tokens;
  int32_t row_groups;  // MFMA kernel: workgroups that split the query rows of one (sequence, kv head, chunk)
  int32_t workers;     // MFMA kernel: > 0 = work-proportional schedule with this many workers per kv head
  bool mfma;
  size_t ml_offset;  // byte offset of part_ml in the workspace
  size_t bytes;      // workspace size (0 when splits == 1)
};
int32_t make_attn_plan(const hb_attn_desc *d, AttnPlan *plan);  // validates shape fields

// ---- kernel launchers (each enqueues on `s`, returns a hipError_t from the launch) -------
hipError_t launch_attn_scalar(const hb_attn_desc &d, const AttnPlan &plan, const void *q,
                              const void *k_tree, const void *v_tree, const void *k_pool,
                              const void *v_pool, const int32_t *block_table,
                              const int32_t *prefix_len, const int32_t *node_offset,
                              const int32_t *parent, void *out, float *lse, float *part_o,
                              float *part_ml, hipStream_t s);
hipError_t launch_attn_mfma(const hb_attn_desc &d, const AttnPlan &plan, const void *q,
                            const void *k_tree, const void *v_tree, const void *k_pool,
                            const void *v_pool, const int32_t *block_table,
                            const int32_t *prefix_len, const int32_t *node_offset,
                            const int32_t *parent, void *out, float *lse, float *part_o,
                            float *part_ml, hipStream_t s);
bool attn_mfma_supports(const hb_attn_desc &d);
int32_t attn_mfma_row_groups(const hb_attn_desc &d);
int32_t attn_mfma_waves(const hb_attn_desc &d);  // wavefronts per workgroup (4 or 8)
hipError_t launch_attn_merge(const hb_attn_desc &d, const AttnPlan &plan, const float *part_o,
                             const float *part_ml, void *out, float *lse, hipStream_t s);

hipError_t launch_lmhead_scalar(int32_t dtype, int32_t M, int32_t K, int32_t V, const void *hidden,
                                const void *weight, unsigned long long *keys, hipStream_t s);
hipError_t launch_lmhead_mfma(int32_t M, int32_t K, int32_t V, const void *hidden,
                              const void *weight, unsigned long long *keys, hipStream_t s);
bool lmhead_mfma_supports(int32_t dtype, int32_t M, int32_t K, int32_t V);
hipError_t launch_lmhead_init(unsigned long long *keys, int32_t M, hipStream_t s);
hipError_t launch_lmhead_finish(const unsigned long long *keys, int32_t M, int32_t V,
                                int32_t *out_ids, float *out_max, hipStream_t s);

bool proj_mfma_supports(int32_t M, int32_t K, int32_t N);
// part: fp32 scratch of proj_workspace_bytes(M, K, N) bytes for the split-K path, or null (then: one workgroup per tile)
size_t proj_workspace_bytes(int32_t M, int32_t K, int32_t N);
hipError_t launch_qkv_rope(int32_t M, int32_t K, int32_t Hq, int32_t Hkv, const void *hidden, const void *w_qkv,
                           const void *bias, const float *cos, const float *sin, void *q, void *k, void *v,
                           float *part, hipStream_t s);
hipError_t launch_linear(int32_t M, int32_t K, int32_t N, const void *x, const void *w, const void *residual,
                         void *out, float *part, hipStream_t s);
hipError_t launch_swiglu(int32_t M, int32_t K, int32_t F, const void *x, const void *w_gate_up, void *out, float *part,
                         hipStream_t s);
hipError_t launch_rmsnorm(int32_t T, int32_t K, const void *x, const void *weight, float eps, void *out, hipStream_t s);
hipError_t launch_tree_positions(int32_t B, int32_t max_nodes, int32_t total_nodes, const int32_t *node_offset,
                                 const int32_t *parent, const int32_t *prefix_len, int32_t *positions, hipStream_t s);
hipError_t launch_rope_table(int32_t T, int32_t half, double theta, const int32_t *positions, float *cos, float *sin,
                             hipStream_t s);

hipError_t launch_tree_accept(int32_t B, int32_t max_nodes, const int32_t *node_offset,
                              const int32_t *parent, const int32_t *draft_ids,
                              const int32_t *target_ids, const int32_t *prev_target, int32_t max_path,
                              int32_t *accept_len, int32_t *accept_path, int32_t *out_tokens,
                              int32_t *bonus_id, hipStream_t s);
hipError_t launch_tree_accept_sample(int32_t B, int32_t max_nodes, int32_t V, const int32_t *node_offset,
                                     const int32_t *parent, const int32_t *draft_ids, const float *p_target,
                                     const float *q_draft, const uint32_t *u_accept, const uint32_t *u_bonus,
                                     int32_t max_path, int32_t *accept_len, int32_t *accept_path,
                                     int32_t *out_tokens, int32_t *bonus_id, uint32_t *work, hipStream_t s);
size_t topk_workspace_bytes(int32_t M, int32_t V, int32_t k);
hipError_t launch_topk_logprob(int32_t dtype, int32_t M, int32_t V, int32_t k, const void *logits, int32_t *out_ids,
                               float *out_logp, void *work, hipStream_t s);
hipError_t launch_tree_grow(int32_t B, int32_t K, int32_t level, int32_t C, const int32_t *child_ids,
                            const float *child_logp, float *cand_score, int32_t *cand_token, int32_t *cand_parent,
                            int32_t *frontier, int32_t *frontier_slot, hipStream_t s);
hipError_t launch_tree_finalize(int32_t B, int32_t C, int32_t n, const float *cand_score, const int32_t *cand_token,
                                const int32_t *cand_parent, const int32_t *root_token, int32_t *node_offset,
                                int32_t *parent, int32_t *draft_ids, int32_t *depth, unsigned long long *anc,
                                int32_t *node_cand, float *node_score, hipStream_t s);
int32_t meta_rows_pad(int32_t H, int32_t Q);
hipError_t launch_meta_fold(int32_t Q, int32_t D, int32_t H, const void *f_q, const void *w_q, const void *w_k,
                            void *a_fold, float *qproj, hipStream_t s);
hipError_t launch_meta_attn(int32_t S, int32_t L, int32_t D, int32_t H, int32_t Q, const void *feats, const void *v_proj,
                            const void *a_fold, const int32_t *residual_layers, void *pre, void *res_out,
                            float *part, hipStream_t s);
size_t meta_attn_workspace_bytes(int32_t S, int32_t D, int32_t H, int32_t Q);
hipError_t launch_kv_compact(const hb_attn_desc &d, const void *k_tree, const void *v_tree,
                             void *k_pool, void *v_pool, const int32_t *block_table,
                             const int32_t *prefix_len, const int32_t *node_offset,
                             const int32_t *accept_len, const int32_t *accept_path,
                             int32_t max_path, int32_t *out_slots, int32_t *new_len, hipStream_t s);

hipError_t launch_kv_compact_layers(const hb_attn_desc &d, int32_t n_layers, const void *const *k_tree,
                                    const void *const *v_tree, void *const *k_pool, void *const *v_pool,
                                    const int32_t *block_table, const int32_t *prefix_len,
                                    const int32_t *node_offset, const int32_t *accept_len,
                                    const int32_t *accept_path, int32_t max_path, int32_t *out_slots,
                                    int32_t *new_len, hipStream_t s);

// ---- argmax key: (order-preserving float bits << 32) | (0xffffffff - index) ---------------
// max over keys = largest value, lowest index among equal values.  NaN is mapped to -inf.
__device__ inline unsigned long long argmax_key(float v, uint32_t idx) {
  if (!(v == v)) v = -__builtin_huge_valf();
  uint32_t u = __float_as_uint(v);
  u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  return ((unsigned long long)u << 32) | (unsigned long long)(0xffffffffu - idx);
}
__device__ inline float argmax_key_value(unsigned long long key) {
  uint32_t u = (uint32_t)(key >> 32);
  u = (u & 0x80000000u) ? (u & 0x7fffffffu) : ~u;
  return __uint_as_float(u);
}
__device__ inline uint32_t argmax_key_index(unsigned long long key) {
  return 0xffffffffu - (uint32_t)(key & 0xffffffffull);
}

}  // namespace hb
