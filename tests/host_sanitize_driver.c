/* Host-side checks of the C ABI's argument validation, planning and error text, built with
 * AddressSanitizer and UndefinedBehaviorSanitizer on the host code of the library (see
 * tests/test_host_sanitizers.py).  No call here reaches a kernel launch: every one fails, or
 * succeeds as a no-op, on host-visible arguments alone, so it runs without a GPU. */
#include <stdio.h>
#include <string.h>
#include "hb.h"

#define CHECK(cond)                                                        \
  do {                                                                     \
    if (!(cond)) {                                                         \
      printf("FAILED line %d: %s (last error: %s)\n", __LINE__, #cond, hb_last_error()); \
      return 1;                                                            \
    }                                                                      \
  } while (0)

static hb_attn_desc base_desc(void) {
  hb_attn_desc d;
  memset(&d, 0, sizeof d);
  d.dtype = HB_BF16; d.batch = 2; d.num_q_heads = 28; d.num_kv_heads = 4; d.head_dim = 128;
  d.page_size = 16; d.max_blocks_per_seq = 64; d.num_blocks = 200; d.total_nodes = 120;
  d.max_nodes_per_tree = 60; d.softmax_scale = 0.1f;
  return d;
}

int main(void) {
  static int32_t buf[4096] __attribute__((aligned(256)));
  void *p = buf;
  CHECK(hb_version() >= 1);

  int32_t par[65];
  par[0] = -1;
  for (int i = 1; i < 65; ++i) par[i] = i - 1;
  CHECK(hb_tree_validate_host(par, 64) == HB_OK);
  CHECK(hb_tree_validate_host(par, 65) == HB_ERR_UNSUPPORTED);
  CHECK(hb_tree_validate_host(par, 0) == HB_ERR_UNSUPPORTED);
  CHECK(hb_tree_validate_host(NULL, 4) == HB_ERR_INVALID_ARG);
  par[3] = 3;
  CHECK(hb_tree_validate_host(par, 8) == HB_ERR_INVALID_ARG);
  CHECK(strstr(hb_last_error(), "parent[3]") != NULL);

  /* planning over a range of shapes: sizes must be consistent and never overflow */
  for (int batch = 1; batch <= 130; batch += 43)
    for (int nodes = 1; nodes <= 64; nodes += 21)
      for (int blocks = 1; blocks <= 4096; blocks *= 8)
        for (int dtype = 0; dtype < 2; ++dtype)
          for (int splits = 0; splits <= 7; splits += 7)
            for (int algo = 0; algo <= 2; ++algo) {
              hb_attn_desc d = base_desc();
              d.batch = batch; d.max_nodes_per_tree = nodes; d.total_nodes = batch * nodes;
              d.max_blocks_per_seq = blocks; d.num_blocks = blocks * batch + 4; d.dtype = dtype;
              d.num_splits = splits; d.algo = algo; d.max_prefix_len_hint = blocks > 8 ? blocks * 8 : 0;
              size_t ws = hb_tree_verify_attn_workspace_bytes(&d);
              int32_t ns = hb_tree_verify_attn_num_splits(&d);
              if (algo == HB_ATTN_MFMA && dtype == HB_F32) { CHECK(ns == 0 && ws == 0); continue; }
              CHECK(ns >= 1 && ns <= 4096);
              CHECK((ns == 1) == (ws == 0));
              if (ns > 1) CHECK(ws >= (size_t)d.total_nodes * d.num_q_heads * ns * (d.head_dim + 2) * 4);
            }

  hb_attn_desc d = base_desc();
  d.num_q_heads = 30;
  CHECK(hb_tree_verify_attn(&d, p, p, p, p, p, p, p, p, p, p, NULL, NULL, 0, NULL) == HB_ERR_INVALID_ARG);
  d = base_desc(); d.head_dim = 100;
  CHECK(hb_tree_verify_attn(&d, p, p, p, p, p, p, p, p, p, p, NULL, NULL, 0, NULL) == HB_ERR_UNSUPPORTED);
  d = base_desc(); d.max_nodes_per_tree = 65;
  CHECK(hb_tree_verify_attn(&d, p, p, p, p, p, p, p, p, p, p, NULL, NULL, 0, NULL) == HB_ERR_UNSUPPORTED);
  d = base_desc(); d.dtype = 7;
  CHECK(hb_tree_verify_attn(&d, p, p, p, p, p, p, p, p, p, p, NULL, NULL, 0, NULL) == HB_ERR_UNSUPPORTED);
  d = base_desc(); d.algo = 9;
  CHECK(hb_tree_verify_attn(&d, p, p, p, p, p, p, p, p, p, p, NULL, NULL, 0, NULL) == HB_ERR_INVALID_ARG);
  d = base_desc();
  CHECK(hb_tree_verify_attn(&d, NULL, p, p, p, p, p, p, p, p, p, NULL, NULL, 0, NULL) == HB_ERR_INVALID_ARG);
  CHECK(hb_tree_verify_attn(&d, (char *)p + 4, p, p, p, p, p, p, p, p, p, NULL, NULL, 0, NULL) == HB_ERR_INVALID_ARG);
  CHECK(hb_tree_verify_attn(&d, p, p, p, p, p, p, p, p, p, p, NULL, NULL, 0, NULL) == HB_ERR_WORKSPACE);
  CHECK(hb_tree_verify_attn(&d, p, p, p, p, p, p, p, p, p, p, NULL, (char *)p + 8, (size_t)1 << 40, NULL) == HB_ERR_WORKSPACE);
  CHECK(hb_tree_verify_attn(NULL, p, p, p, p, p, p, p, p, p, p, NULL, NULL, 0, NULL) == HB_ERR_INVALID_ARG);
  d = base_desc(); d.batch = 0; d.total_nodes = 0;
  CHECK(hb_tree_verify_attn(&d, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, 0, NULL) == HB_OK);

  CHECK(hb_lmhead_argmax(HB_BF16, 0, 64, 100, NULL, NULL, NULL, NULL, NULL, 0, NULL) == HB_OK);
  CHECK(hb_lmhead_argmax(HB_BF16, 5, 0, 100, p, p, p, NULL, p, 64, NULL) == HB_ERR_INVALID_ARG);
  CHECK(hb_lmhead_argmax(3, 5, 64, 100, p, p, p, NULL, p, 64, NULL) == HB_ERR_UNSUPPORTED);
  CHECK(hb_lmhead_argmax(HB_BF16, 5, 64, 100, p, NULL, p, NULL, p, 64, NULL) == HB_ERR_INVALID_ARG);
  CHECK(hb_lmhead_argmax(HB_BF16, 5, 64, 100, p, p, p, NULL, p, 8, NULL) == HB_ERR_WORKSPACE);
  CHECK(hb_lmhead_argmax(HB_BF16, 5, 64, 100, p, p, p, NULL, (char *)p + 4, 64, NULL) == HB_ERR_WORKSPACE);
  CHECK(hb_lmhead_argmax_workspace_bytes(960) == 960 * 8 && hb_lmhead_argmax_workspace_bytes(-3) == 0);
  CHECK(hb_lmhead_argmax_noalloc(HB_BF16, hb_lmhead_argmax_noalloc_max_rows() + 1, 64, 100, p, p, p, NULL, NULL) == HB_ERR_UNSUPPORTED);
  CHECK(hb_lmhead_argmax_noalloc(HB_BF16, 0, 64, 100, NULL, NULL, NULL, NULL, NULL) == HB_OK);
  CHECK(hb_lmhead_argmax_noalloc(HB_BF16, 5, 64, 100, NULL, p, p, NULL, NULL) == HB_ERR_INVALID_ARG);

  CHECK(hb_tree_accept(2, 65, p, p, p, p, NULL, 6, p, p, p, p, NULL) == HB_ERR_UNSUPPORTED);
  CHECK(hb_tree_accept(2, 60, p, p, p, p, NULL, 0, p, p, p, p, NULL) == HB_ERR_INVALID_ARG);
  CHECK(hb_tree_accept(2, 60, NULL, p, p, p, p, 6, p, p, p, p, NULL) == HB_ERR_INVALID_ARG);
  CHECK(hb_tree_accept(0, 60, NULL, NULL, NULL, NULL, NULL, 6, NULL, NULL, NULL, NULL, NULL) == HB_OK);

  d = base_desc();
  CHECK(hb_kv_compact(&d, p, p, p, p, p, p, p, p, p, 0, NULL, NULL, NULL) == HB_ERR_INVALID_ARG);
  CHECK(hb_kv_compact(&d, p, p, NULL, p, p, p, p, p, p, 6, NULL, NULL, NULL) == HB_ERR_INVALID_ARG);
  CHECK(hb_kv_compact(&d, (char *)p + 2, p, p, p, p, p, p, p, p, 6, NULL, NULL, NULL) == HB_ERR_INVALID_ARG);
  d.batch = 0;
  CHECK(hb_kv_compact(&d, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, 6, NULL, NULL, NULL) == HB_OK);

  /* sampling acceptance, projections, draft tree, meta queries: every call below fails or is a
   * no-op on host-visible arguments */
  CHECK(hb_tree_accept_sample(2, 65, 100, p, p, p, p, p, p, p, 6, p, p, p, p, p, 1 << 20, NULL) == HB_ERR_UNSUPPORTED);
  CHECK(hb_tree_accept_sample(2, 60, 100, p, p, p, p, p, p, p, 6, p, p, p, p, p, 8, NULL) == HB_ERR_WORKSPACE);
  CHECK(hb_tree_accept_sample(0, 60, 100, NULL, NULL, NULL, NULL, NULL, NULL, NULL, 6, NULL, NULL, NULL, NULL, NULL, 0, NULL) == HB_OK);
  CHECK(hb_tree_accept_sample_workspace_bytes(16, 152064) == (size_t)16 * 152064 * 4);
  CHECK(hb_tree_positions(2, 65, 120, p, p, p, p, NULL) == HB_ERR_UNSUPPORTED);
  CHECK(hb_rope_table(4, 127, 1e6, p, p, p, NULL) == HB_ERR_INVALID_ARG);
  CHECK(hb_rope_table(0, 128, 1e6, NULL, NULL, NULL, NULL) == HB_OK);
  CHECK(hb_qkv_rope_project(4, 3584, 28, 4, 64, p, p, NULL, p, p, p, p, p, NULL) == HB_ERR_UNSUPPORTED);
  CHECK(hb_qkv_rope_project(4, 100, 28, 4, 128, p, p, NULL, p, p, p, p, p, NULL) == HB_ERR_UNSUPPORTED);
  CHECK(hb_qkv_rope_project(4, 3584, 28, 4, 128, p, NULL, NULL, p, p, p, p, p, NULL) == HB_ERR_INVALID_ARG);
  CHECK(hb_qkv_rope_project_ws(4, 3584, 28, 4, 128, (char *)p + 2, p, NULL, p, p, p, p, p, p, 64, NULL) == HB_ERR_INVALID_ARG);
  CHECK(hb_out_project(4, 64, 6, p, p, NULL, p, NULL) == HB_ERR_UNSUPPORTED);
  CHECK(hb_out_project_ws(4, 64, 8, p, p, NULL, NULL, p, 64, NULL) == HB_ERR_INVALID_ARG);
  CHECK(hb_out_project_ws(0, 64, 8, NULL, NULL, NULL, NULL, NULL, 0, NULL) == HB_OK);
  for (int t = 1; t <= 1400; t += 33)
    for (int k = 64; k <= 16384; k *= 2)
      for (int n = 4; n <= 200000; n *= 7) {
        size_t ws = hb_proj_workspace_bytes(t, k, n);
        CHECK(t <= 1024 || ws == 0);
        /* at most 256 workgroups, each with a tile of 256 x 256 fp32 partials at most */
        CHECK(ws % 4 == 0 && ws <= (size_t)256 * 256 * 256 * 4);
      }
  CHECK(hb_rmsnorm(4, 3580, p, p, 1e-6f, p, NULL) == HB_ERR_UNSUPPORTED);
  CHECK(hb_rmsnorm(4, 3584, p, p, -1.f, p, NULL) == HB_ERR_INVALID_ARG);
  CHECK(hb_rmsnorm(0, 3584, NULL, NULL, 1e-6f, NULL, NULL) == HB_OK);
  CHECK(hb_swiglu_project(4, 3584, 18942, p, p, p, NULL, 0, NULL) == HB_ERR_UNSUPPORTED);
  CHECK(hb_swiglu_project(4, 3584, 18944, p, NULL, p, NULL, 0, NULL) == HB_ERR_INVALID_ARG);
  CHECK(hb_swiglu_project(0, 3584, 18944, NULL, NULL, NULL, NULL, 0, NULL) == HB_OK);
  CHECK(hb_topk_logprob(HB_F32, 4, 100, 0, p, p, (float *)p, p, 1 << 20, NULL) == HB_ERR_INVALID_ARG);
  CHECK(hb_topk_logprob(HB_F32, 4, 100, 33, p, p, (float *)p, p, 1 << 20, NULL) == HB_ERR_UNSUPPORTED);
  CHECK(hb_topk_logprob(HB_F32, 4, 100, 5, p, p, (float *)p, p, 8, NULL) == HB_ERR_WORKSPACE);
  CHECK(hb_topk_logprob(HB_BF16, 0, 100, 5, NULL, NULL, NULL, NULL, 0, NULL) == HB_OK);
  for (int m = 1; m <= 3000; m = m * 5 + 1)
    for (int v = 1; v <= 2000000; v = v * 11 + 3) {
      size_t ws = hb_topk_logprob_workspace_bytes(m, v, 10);
      CHECK(ws >= (size_t)m * 88 && ws <= (size_t)m * 88 * (size_t)(v / 2048 + 1));
    }
  CHECK(hb_draft_tree_candidates(10, 5) == 410 && hb_draft_tree_candidates(0, 5) == 0);
  CHECK(hb_tree_grow(2, 10, 5, 5, p, (float *)p, (float *)p, p, p, p, p, NULL) == HB_ERR_INVALID_ARG);
  CHECK(hb_tree_grow(2, 40, 5, 0, p, (float *)p, (float *)p, p, p, p, p, NULL) == HB_ERR_UNSUPPORTED);
  CHECK(hb_tree_grow(0, 10, 5, 0, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL) == HB_OK);
  CHECK(hb_tree_finalize(2, 10, 5, 65, (float *)p, p, p, p, p, p, p, p, (uint64_t *)p, p, (float *)p, NULL) == HB_ERR_UNSUPPORTED);
  CHECK(hb_tree_finalize(2, 2, 2, 8, (float *)p, p, p, p, p, p, p, p, (uint64_t *)p, p, (float *)p, NULL) == HB_ERR_INVALID_ARG);
  CHECK(hb_tree_finalize(0, 10, 5, 60, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL) == HB_OK);
  CHECK(hb_meta_query_fold_bytes(3, 3584, 28) == (size_t)2 * 96 * 3584 * 2);
  CHECK(hb_meta_query_fold(3, 3584, 27, p, p, p, p, p, 1 << 20, NULL) == HB_ERR_INVALID_ARG);
  CHECK(hb_meta_query_fold(3, 3584, 28, p, p, p, p, p, 16, NULL) == HB_ERR_WORKSPACE);
  {
    int32_t layers_bad[3] = {0, 14, 28}, layers_ok[3] = {0, 14, 27};
    CHECK(hb_meta_query_attn(4, 28, 3584, 28, 3, p, p, p, layers_bad, p, p, p, (size_t)1 << 30, NULL) == HB_ERR_INVALID_ARG);
    CHECK(hb_meta_query_attn(4, 28, 3584, 28, 3, p, p, p, layers_ok, p, NULL, p, (size_t)1 << 30, NULL) == HB_ERR_INVALID_ARG);
    CHECK(hb_meta_query_attn(4, 33, 3584, 28, 3, p, p, p, NULL, p, NULL, p, (size_t)1 << 30, NULL) == HB_ERR_UNSUPPORTED);
    CHECK(hb_meta_query_attn(0, 28, 3584, 28, 3, NULL, NULL, NULL, layers_ok, NULL, p, NULL, 0, NULL) == HB_OK);
    CHECK(hb_meta_query_attn(4, 28, 3584, 28, 3, p, p, p, NULL, p, NULL, p, 16, NULL) == HB_ERR_WORKSPACE);
    for (int32_t S = 1; S <= 20000; S = S * 3 + 1) {
      size_t nb = hb_meta_query_attn_workspace_bytes(S, 3584, 28, 3);
      CHECK(nb >= (size_t)S * 96 * 32 * 4 && nb <= (size_t)14 * S * 96 * 32 * 4);
    }
  }
  printf("host shim checks passed\n");
  return 0;
}
