// Target-feature aggregation with meta queries (the paper, Section 3.1.1, Eq. 1): for every token,
// Q learnable queries attend over the L layer features of that token (multi-head, H heads of size
// d = D / H) and the Q outputs are flattened.
//
// The queries do not depend on the token, so the key projection is folded into them once:
//   score(q, h, l) = (f_q W_q^T)_{q,h} . (f_i[l] W_k^T)_h / sqrt(d) = A[h Q + q] . f_i[l],
//   A[h Q + q] = (f_q W_q^T)_{q,h} W_k[h d .. (h + 1) d, :] / sqrt(d)          (a D-vector)
// which removes the L x D x D key projection per token: the scores are one small dense product
// [H Q, D] x [D, L] per token, on the matrix cores.  A is kept as the sum of two bf16 matrices
// (value rounded to bf16 plus the rounded remainder), so that folding costs the scores no
// accuracy against projecting keys in fp32.
//
// meta_scores_kernel: the scores of all tokens are one dense product A [H Q, D] x feats^T
// [D, S L].  A workgroup takes eight tokens and a range of 256-feature slices of D; it stages the
// slice of A (both halves) in LDS once and its four wavefronts, two tokens each, run MFMA
// 16x16x32 with the A fragments from LDS and the tokens' features straight from memory in
// fragment layout, so A crosses the vector memory path once per eight tokens.  With few tokens
// the slices are spread over several workgroups, which write partial scores (fp32) to a workspace.
// meta_mix_kernel, one workgroup per token (and per 4096 features): sums the partial scores, one thread per (head, query)
// row does the softmax over the L layers, and every thread then mixes the token's projected values
// (v_proj = f_i W_v^T, a plain linear layer run beforehand) for eight feature columns of all Q
// queries:  pre[q, c] = sum_l P[head(c) Q + q, l] v_proj[l, c].
// The output projection and the skip connection (Section 3.1.2) are a linear layer with residual
// run afterwards on pre; the mixing kernel also copies the residual rows f_i[residual_layers[q]].
#include "hb_internal.h"

namespace hb {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;       // the two set-up kernels
constexpr int kWaves = 4;
constexpr int kScoreWaves = 4;      // wavefronts of meta_scores_kernel
constexpr int kScoreThreads = 64 * kScoreWaves;
constexpr int kTokPerWave = 2;      // tokens whose scores one wavefront accumulates
constexpr int kTokPerGroup = kScoreWaves * kTokPerWave;
constexpr int kSlice = 256;         // features of A staged in LDS at a time
constexpr int kSlicePieces = kSlice / 8;       // 16-byte pieces per row of a slice
constexpr int kSliceSteps = kSlice / 32;       // MFMA steps per slice
constexpr int kRowPieces = kSlicePieces + 1;   // LDS row stride in pieces: fragment reads of 16 rows hit distinct banks
constexpr int kMixThreads = 512;      // meta_mix_kernel: one thread per eight feature columns
constexpr int kMaxParts = 16;         // workgroup columns of the score kernel
constexpr int kMaxRowTiles = 6;   // H * Q <= 96
constexpr int kMaxRows = 16 * kMaxRowTiles;
constexpr int kMaxL = 32;
constexpr int kLdsL = kMaxL + 1;    // row stride of the score tables in LDS: one thread per row reads without bank conflicts
constexpr int kMaxQ = 4;

// qproj[q, n] = sum_c f_q[q, c] w_q[n, c]: one wavefront per output
__global__ __launch_bounds__(kThreads) void meta_qproj_kernel(int Q, int D, const bf16_t *__restrict__ f_q,
                                                              const bf16_t *__restrict__ w_q,
                                                              float *__restrict__ qproj) {
  const int out = blockIdx.x * kWaves + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (out >= Q * D) return;
  const int q = out / D, n = out - q * D;
  float acc = 0.f;
  for (int c = lane; c < D; c += 64) acc += bf16_to_f32(f_q[(size_t)q * D + c]) * bf16_to_f32(w_q[(size_t)n * D + c]);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
  if (lane == 0) qproj[out] = acc;
}

// A[h Q + q, c] = scale * sum_j qproj[q, h d + j] w_k[h d + j, c], split into two bf16 matrices;
// rows from H * Q up to rows_pad are zero
__global__ __launch_bounds__(kThreads) void meta_fold_kernel(int Q, int D, int H, int rows_pad, float scale,
                                                             const float *__restrict__ qproj,
                                                             const bf16_t *__restrict__ w_k,
                                                             bf16_t *__restrict__ a_hi, bf16_t *__restrict__ a_lo) {
  const int c = blockIdx.x * kThreads + threadIdx.x;
  const int r = blockIdx.y;
  if (c >= D) return;
  float acc = 0.f;
  if (r < H * Q) {
    const int h = r / Q, q = r - h * Q, d = D / H;
    for (int j = 0; j < d; ++j) acc += qproj[(size_t)q * D + h * d + j] * bf16_to_f32(w_k[(size_t)(h * d + j) * D + c]);
    acc *= scale;
  }
  const bf16_t hi = f32_to_bf16(acc);
  a_hi[(size_t)r * D + c] = hi;
  a_lo[(size_t)r * D + c] = f32_to_bf16(acc - bf16_to_f32(hi));
}

struct ResidualLayers {
  int32_t layer[kMaxQ];
  int32_t on;
};

// part[p][s][row][l] (row stride 32): the scores of token s summed over the slices that
// workgroup column p covers
__global__ __launch_bounds__(kScoreThreads) void meta_scores_kernel(int S, int L, int D, int row_tiles,
                                                                    int slices_per_wg,
                                                                    const u32x4 *__restrict__ feats,
                                                                    const u32x4 *__restrict__ a_hi,
                                                                    const u32x4 *__restrict__ a_lo,
                                                                    float *__restrict__ part) {
  extern __shared__ u32x4 meta_a_lds[];  // [2][rows_pad][kRowPieces]
  const int rows_pad = 16 * row_tiles;
  u32x4 *lds_hi = meta_a_lds, *lds_lo = meta_a_lds + rows_pad * kRowPieces;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j16 = lane & 15, kq = lane >> 4;
  const int dp = D / 8;                       // 16-byte pieces per feature row
  const int tok0 = blockIdx.x * kTokPerGroup + wave * kTokPerWave;
  const int slices = D / kSlice;
  const int sl_begin = blockIdx.y * slices_per_wg;
  const int sl_end = sl_begin + slices_per_wg < slices ? sl_begin + slices_per_wg : slices;

  // B operand: lane (j16, kq) feeds layer 16 ct + j16, features 8 kq .. 8 kq + 7 of the step.
  // Tokens past the end and layers past L read a valid row and are zeroed or dropped later.
  const u32x4 *bp[kTokPerWave][2];
  bool live[2];
#pragma unroll
  for (int ct = 0; ct < 2; ++ct) live[ct] = 16 * ct + j16 < L;
#pragma unroll
  for (int t = 0; t < kTokPerWave; ++t) {
    const int tk = tok0 + t < S ? tok0 + t : S - 1;
#pragma unroll
    for (int ct = 0; ct < 2; ++ct) bp[t][ct] = feats + ((size_t)tk * L + (live[ct] ? 16 * ct + j16 : 0)) * dp + kq;
  }
  f32x4 acc[kMaxRowTiles][kTokPerWave][2];
#pragma unroll
  for (int mt = 0; mt < kMaxRowTiles; ++mt)
#pragma unroll
    for (int t = 0; t < kTokPerWave; ++t)
#pragma unroll
      for (int ct = 0; ct < 2; ++ct) acc[mt][t][ct] = (f32x4){0.f, 0.f, 0.f, 0.f};
  const u32x4 zero = {0u, 0u, 0u, 0u};

  for (int sl = sl_begin; sl < sl_end; ++sl) {
    const int piece0 = sl * kSlicePieces;
    // the tokens' fragments of the whole slice are requested before A is staged
    u32x4 fb[kSliceSteps][kTokPerWave][2];
#pragma unroll
    for (int st = 0; st < kSliceSteps; ++st)
#pragma unroll
      for (int t = 0; t < kTokPerWave; ++t)
#pragma unroll
        for (int ct = 0; ct < 2; ++ct) fb[st][t][ct] = bp[t][ct][piece0 + 4 * st];
    __syncthreads();  // the previous slice's fragment reads are done
    // all of the slice's loads are issued before the first LDS write
    constexpr int kStage = kMaxRows * kSlicePieces / kScoreThreads;
    u32x4 sh[kStage], sl_[kStage];
#pragma unroll
    for (int i = 0; i < kStage; ++i) {
      const int idx = tid + i * kScoreThreads;
      if (idx < rows_pad * kSlicePieces) {
        const int row = idx / kSlicePieces, pc = idx % kSlicePieces;
        sh[i] = a_hi[(size_t)row * dp + piece0 + pc];
        sl_[i] = a_lo[(size_t)row * dp + piece0 + pc];
      }
    }
#pragma unroll
    for (int i = 0; i < kStage; ++i) {
      const int idx = tid + i * kScoreThreads;
      if (idx < rows_pad * kSlicePieces) {
        const int row = idx / kSlicePieces, pc = idx % kSlicePieces;
        lds_hi[row * kRowPieces + pc] = sh[i];
        lds_lo[row * kRowPieces + pc] = sl_[i];
      }
    }
    __syncthreads();
#pragma unroll
    for (int st = 0; st < kSliceSteps; ++st) {
      bf16x8 x[kTokPerWave][2];
#pragma unroll
      for (int t = 0; t < kTokPerWave; ++t)
#pragma unroll
        for (int ct = 0; ct < 2; ++ct) x[t][ct] = __builtin_bit_cast(bf16x8, live[ct] ? fb[st][t][ct] : zero);
#pragma unroll
      for (int mt = 0; mt < kMaxRowTiles; ++mt) {
        if (mt < row_tiles) {
          const int at = (16 * mt + j16) * kRowPieces + 4 * st + kq;
          const bf16x8 h8 = __builtin_bit_cast(bf16x8, lds_hi[at]);
          const bf16x8 l8 = __builtin_bit_cast(bf16x8, lds_lo[at]);
#pragma unroll
          for (int t = 0; t < kTokPerWave; ++t)
#pragma unroll
            for (int ct = 0; ct < 2; ++ct) {
              acc[mt][t][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(h8, x[t][ct], acc[mt][t][ct], 0, 0, 0);
              acc[mt][t][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(l8, x[t][ct], acc[mt][t][ct], 0, 0, 0);
            }
        }
      }
    }
  }
  // lane (j16, kq) holds rows 16 mt + 4 kq + r of layer 16 ct + j16
#pragma unroll
  for (int t = 0; t < kTokPerWave; ++t) {
    if (tok0 + t < S) {
      float *dst = part + ((size_t)blockIdx.y * S + tok0 + t) * rows_pad * kMaxL;
#pragma unroll
      for (int mt = 0; mt < kMaxRowTiles; ++mt) {
        if (mt < row_tiles) {
#pragma unroll
          for (int ct = 0; ct < 2; ++ct)
#pragma unroll
            for (int r = 0; r < 4; ++r) dst[(16 * mt + 4 * kq + r) * kMaxL + 16 * ct + j16] = acc[mt][t][ct][r];
        }
      }
    }
  }
}

__global__ __launch_bounds__(kMixThreads) void meta_mix_kernel(int S, int L, int D, int H, int Q, int rows_pad,
                                                               int parts, const float *__restrict__ part,
                                                               const u32x4 *__restrict__ feats,
                                                               const u32x4 *__restrict__ v_proj, ResidualLayers res,
                                                               u32x4 *__restrict__ pre, u32x4 *__restrict__ res_out) {
  __shared__ float prob[kMaxRows][kLdsL];
  const int s = blockIdx.x;
  const int tid = threadIdx.x;
  const int dp = D / 8;                       // 16-byte pieces per feature row
  const u32x4 *f_tok = feats + (size_t)s * L * dp;
  const u32x4 *g_tok = v_proj + (size_t)s * L * dp;
  const int rows = H * Q;

  // Everything the token needs from memory is requested up front, in one round: the projected
  // values of this thread's eight columns for all layers, the residual rows, the partial scores.
  const int d8 = (D / H) / 8;  // 16-byte pieces per head
  const int cg = blockIdx.y * kMixThreads + tid;  // this thread's 16-byte column group
  const bool mixer = cg < dp;
  u32x4 g[kMaxL], rr[kMaxQ];
#pragma unroll
  for (int l = 0; l < kMaxL; ++l)
    if (mixer && l < L) g[l] = g_tok[(size_t)l * dp + cg];
#pragma unroll
  for (int q = 0; q < kMaxQ; ++q)
    if (mixer && res.on && q < Q) rr[q] = f_tok[(size_t)res.layer[q] * dp + cg];

  // ---- the token's scores: sum over the workgroup columns of the score kernel ----------------
  const int n4 = rows_pad * kMaxL / 4;  // float4 pieces of one partial table
  const f32x4 *part4 = reinterpret_cast<const f32x4 *>(part);
#pragma unroll
  for (int it = 0; it < (kMaxRows * kMaxL / 4 + kMixThreads - 1) / kMixThreads; ++it) {
    const int i = tid + it * kMixThreads;
    if (i < n4) {
      f32x4 v[kMaxParts];
#pragma unroll
      for (int p = 0; p < kMaxParts; ++p)
        if (p < parts) v[p] = part4[((size_t)p * S + s) * n4 + i];
      f32x4 t = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int p = 0; p < kMaxParts; ++p)
        if (p < parts) t += v[p];
      const int row = i / (kMaxL / 4), c4 = i % (kMaxL / 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) prob[row][4 * c4 + e] = t[e];
    }
  }
  __syncthreads();

  // ---- softmax over the layers, one thread per (head, query) row -----------------------------
  if (tid < rows) {
    float sc[kMaxL];
    float mx = -__builtin_huge_valf();
#pragma unroll
    for (int l = 0; l < kMaxL; ++l) {
      sc[l] = prob[tid][l];
      if (l < L) mx = fmaxf(mx, sc[l]);
    }
    float sum = 0.f;
#pragma unroll
    for (int l = 0; l < kMaxL; ++l) {
      sc[l] = l < L ? __expf(sc[l] - mx) : 0.f;
      sum += sc[l];
    }
    const float inv = 1.f / sum;
#pragma unroll
    for (int l = 0; l < kMaxL; ++l) prob[tid][l] = sc[l] * inv;
  }
  __syncthreads();

  // ---- mix the projected values: eight feature columns per thread, all queries ---------------
  if (!mixer) return;
  const int h = cg / d8;
  float o[kMaxQ][8];
#pragma unroll
  for (int q = 0; q < kMaxQ; ++q)
#pragma unroll
    for (int e = 0; e < 8; ++e) o[q][e] = 0.f;
#pragma unroll
  for (int l = 0; l < kMaxL; ++l) {
    if (l < L) {
      float gv[8];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        gv[2 * e] = __uint_as_float(g[l][e] << 16);
        gv[2 * e + 1] = __uint_as_float(g[l][e] & 0xffff0000u);
      }
#pragma unroll
      for (int q = 0; q < kMaxQ; ++q) {
        if (q < Q) {
          const float p = prob[h * Q + q][l];
#pragma unroll
          for (int e = 0; e < 8; ++e) o[q][e] += p * gv[e];
        }
      }
    }
  }
#pragma unroll
  for (int q = 0; q < kMaxQ; ++q) {
    if (q < Q) {
      u32x4 w;
#pragma unroll
      for (int e = 0; e < 4; ++e)
        w[e] = (uint32_t)f32_to_bf16(o[q][2 * e]) | ((uint32_t)f32_to_bf16(o[q][2 * e + 1]) << 16);
      pre[((size_t)s * Q + q) * dp + cg] = w;
      if (res.on) res_out[((size_t)s * Q + q) * dp + cg] = rr[q];
    }
  }
}

}  // namespace

int32_t meta_rows_pad(int32_t H, int32_t Q) { return (H * Q + 15) / 16 * 16; }

hipError_t launch_meta_fold(int32_t Q, int32_t D, int32_t H, const void *f_q, const void *w_q, const void *w_k,
                            void *a_fold, float *qproj, hipStream_t s) {
  const int rows_pad = meta_rows_pad(H, Q);
  meta_qproj_kernel<<<(Q * D + kWaves - 1) / kWaves, kThreads, 0, s>>>(Q, D, (const bf16_t *)f_q, (const bf16_t *)w_q,
                                                                      qproj);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  bf16_t *a_hi = (bf16_t *)a_fold, *a_lo = a_hi + (size_t)rows_pad * D;
  const float scale = 1.f / sqrtf((float)(D / H));
  meta_fold_kernel<<<dim3((D + kThreads - 1) / kThreads, rows_pad), kThreads, 0, s>>>(Q, D, H, rows_pad, scale, qproj,
                                                                                      (const bf16_t *)w_k, a_hi, a_lo);
  return hipGetLastError();
}

// Workgroup columns of the score kernel: enough of them that a few tokens still fill the chip
static void score_split(int32_t S, int32_t D, int *slices_per_wg, int *parts) {
  const int slices = D / kSlice;
  const int groups = (S + kTokPerGroup - 1) / kTokPerGroup;
  int p = (512 + groups - 1) / groups;
  if (p > slices) p = slices;
  if (p > kMaxParts) p = kMaxParts;
  if (p < 1) p = 1;
  *slices_per_wg = (slices + p - 1) / p;
  *parts = (slices + *slices_per_wg - 1) / *slices_per_wg;
}

size_t meta_attn_workspace_bytes(int32_t S, int32_t D, int32_t H, int32_t Q) {
  int spw, parts;
  score_split(S, D, &spw, &parts);
  return (size_t)parts * S * meta_rows_pad(H, Q) * kMaxL * sizeof(float);
}

hipError_t launch_meta_attn(int32_t S, int32_t L, int32_t D, int32_t H, int32_t Q, const void *feats, const void *v_proj,
                            const void *a_fold, const int32_t *residual_layers, void *pre, void *res_out,
                            float *part, hipStream_t s) {
  const int rows_pad = meta_rows_pad(H, Q);
  ResidualLayers res = {};
  if (residual_layers && res_out) {
    res.on = 1;
    for (int q = 0; q < Q; ++q) res.layer[q] = residual_layers[q];
  }
  const bf16_t *a_hi = (const bf16_t *)a_fold, *a_lo = a_hi + (size_t)rows_pad * D;
  int spw, parts;
  score_split(S, D, &spw, &parts);
  const size_t lds = (size_t)2 * rows_pad * kRowPieces * sizeof(u32x4);
  hipError_t e = hipFuncSetAttribute((const void *)meta_scores_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                     (int)((size_t)2 * kMaxRows * kRowPieces * sizeof(u32x4)));
  if (e != hipSuccess) return e;
  meta_scores_kernel<<<dim3((S + kTokPerGroup - 1) / kTokPerGroup, parts), kScoreThreads, lds, s>>>(
      S, L, D, rows_pad / 16, spw, (const u32x4 *)feats, (const u32x4 *)a_hi, (const u32x4 *)a_lo, part);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  meta_mix_kernel<<<dim3(S, (D / 8 + kMixThreads - 1) / kMixThreads), kMixThreads, 0, s>>>(S, L, D, H, Q, rows_pad, parts, part, (const u32x4 *)feats,
                                            (const u32x4 *)v_proj, res, (u32x4 *)pre, (u32x4 *)res_out);
  return hipGetLastError();
}

}  // namespace hb
