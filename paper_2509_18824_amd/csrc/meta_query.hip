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
// meta_attn_kernel, one workgroup per token: the eight wavefronts split D, each accumulates its
// share of the [H Q, L] scores with MFMA 16x16x32 (operands straight from memory in fragment
// layout: the A rows come from L2, the token's features from HBM), the partial scores meet in
// LDS, one thread per (head, query) row does the softmax over the L layers, and every thread then
// mixes the token's projected values (v_proj = f_i W_v^T, a plain linear layer run beforehand)
// for eight feature columns of all Q queries:  pre[q, c] = sum_l P[head(c) Q + q, l] v_proj[l, c].
// The output projection and the skip connection (Section 3.1.2) are a linear layer with residual
// run afterwards on pre; this kernel also copies the residual rows f_i[residual_layers[q]].
#include "hb_internal.h"

namespace hb {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;       // the two set-up kernels
constexpr int kWaves = 4;
constexpr int kAttnWaves = 8;       // wavefronts of meta_attn_kernel: each takes an eighth of D
constexpr int kAttnThreads = 64 * kAttnWaves;
constexpr int kBRing = 4;           // steps that the token's feature fragments are loaded ahead
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

__global__ __launch_bounds__(kAttnThreads) void meta_attn_kernel(int L, int D, int H, int Q, int row_tiles,
                                                                 const u32x4 *__restrict__ feats,
                                                                 const u32x4 *__restrict__ v_proj,
                                                                 const u32x4 *__restrict__ a_hi,
                                                                 const u32x4 *__restrict__ a_lo, ResidualLayers res,
                                                                 u32x4 *__restrict__ pre, u32x4 *__restrict__ res_out) {
  extern __shared__ float meta_lds[];
  float (*part)[kMaxRows][kLdsL] = reinterpret_cast<float (*)[kMaxRows][kLdsL]>(meta_lds);  // [kAttnWaves]
  float (*prob)[kLdsL] = reinterpret_cast<float (*)[kLdsL]>(meta_lds + kAttnWaves * kMaxRows * kLdsL);
  const int s = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j16 = lane & 15, kq = lane >> 4;
  const int dp = D / 8;                       // 16-byte pieces per feature row
  const u32x4 *f_tok = feats + (size_t)s * L * dp;
  const u32x4 *g_tok = v_proj + (size_t)s * L * dp;
  const int rows = H * Q;

  // ---- scores: this wavefront's eighth of D ------------------------------------------------
  // The A rows come from L2 (every token re-reads them), one step ahead; the token's own
  // features come from HBM and are requested kBRing - 1 steps ahead.
  f32x4 acc[kMaxRowTiles][2];
#pragma unroll
  for (int mt = 0; mt < kMaxRowTiles; ++mt) {
    acc[mt][0] = (f32x4){0.f, 0.f, 0.f, 0.f};
    acc[mt][1] = (f32x4){0.f, 0.f, 0.f, 0.f};
  }
  const int steps = D / (32 * kAttnWaves);    // 32 features per MFMA step
  const int piece0 = wave * steps * 4 + kq;   // 16-byte piece of the lane's fragment at step 0
  const u32x4 zero = {0u, 0u, 0u, 0u};
  const int l0 = j16, l1 = 16 + j16;          // the lane's layers (B operand columns)
  const u32x4 *b0 = f_tok + (size_t)(l0 < L ? l0 : 0) * dp + piece0;
  const u32x4 *b1 = f_tok + (size_t)(l1 < L ? l1 : 0) * dp + piece0;
  const u32x4 *ah = a_hi + (size_t)j16 * dp + piece0;
  const u32x4 *al = a_lo + (size_t)j16 * dp + piece0;
  u32x4 fb[kBRing][2], fh[2][kMaxRowTiles], fl[2][kMaxRowTiles];
#define HB_META_LOAD_B(buf_, step_)                                            \
  {                                                                            \
    fb[buf_][0] = b0[(step_) * 4];                                             \
    fb[buf_][1] = b1[(step_) * 4];                                             \
  }
#define HB_META_LOAD_A(buf_, step_)                                            \
  {                                                                            \
    _Pragma("unroll") for (int mt = 0; mt < kMaxRowTiles; ++mt) {               \
      if (mt < row_tiles) {                                                    \
        fh[buf_][mt] = ah[(size_t)mt * 16 * dp + (step_) * 4];                 \
        fl[buf_][mt] = al[(size_t)mt * 16 * dp + (step_) * 4];                 \
      }                                                                        \
    }                                                                          \
  }
#define HB_META_MMA(abuf_, bbuf_)                                                                                \
  {                                                                                                              \
    const bf16x8 x0 = __builtin_bit_cast(bf16x8, l0 < L ? fb[bbuf_][0] : zero);                                  \
    const bf16x8 x1 = __builtin_bit_cast(bf16x8, l1 < L ? fb[bbuf_][1] : zero);                                  \
    _Pragma("unroll") for (int mt = 0; mt < kMaxRowTiles; ++mt) {                                                 \
      if (mt < row_tiles) {                                                                                      \
        const bf16x8 h8 = __builtin_bit_cast(bf16x8, fh[abuf_][mt]);                                             \
        const bf16x8 l8 = __builtin_bit_cast(bf16x8, fl[abuf_][mt]);                                             \
        acc[mt][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(h8, x0, acc[mt][0], 0, 0, 0);                       \
        acc[mt][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(h8, x1, acc[mt][1], 0, 0, 0);                       \
        acc[mt][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(l8, x0, acc[mt][0], 0, 0, 0);                       \
        acc[mt][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(l8, x1, acc[mt][1], 0, 0, 0);                       \
      }                                                                                                          \
    }                                                                                                            \
  }
#pragma unroll
  for (int u = 0; u < kBRing - 1; ++u)
    if (u < steps) HB_META_LOAD_B(u, u);
  HB_META_LOAD_A(0, 0);
  for (int st = 0; st < steps; st += kBRing) {
#pragma unroll
    for (int u = 0; u < kBRing; ++u) {
      const int cur = st + u;
      if (cur < steps) {
        if (cur + kBRing - 1 < steps) HB_META_LOAD_B((u + kBRing - 1) % kBRing, cur + kBRing - 1);
        if (cur + 1 < steps) HB_META_LOAD_A((u + 1) & 1, cur + 1);
        HB_META_MMA(u & 1, u);
      }
    }
  }
#undef HB_META_LOAD_A
#undef HB_META_LOAD_B
#undef HB_META_MMA
  // lane (j16, kq) holds rows 16 mt + 4 kq + r of layer 16 ct + j16
#pragma unroll
  for (int mt = 0; mt < kMaxRowTiles; ++mt) {
    if (mt < row_tiles) {
#pragma unroll
      for (int ct = 0; ct < 2; ++ct)
#pragma unroll
        for (int r = 0; r < 4; ++r) part[wave][16 * mt + 4 * kq + r][16 * ct + j16] = acc[mt][ct][r];
    }
  }
  __syncthreads();

  // ---- softmax over the layers, one thread per (head, query) row -----------------------------
  if (tid < rows) {
    float sc[kMaxL];
    float mx = -__builtin_huge_valf();
#pragma unroll
    for (int l = 0; l < kMaxL; ++l) {
      float t = 0.f;
#pragma unroll
      for (int w = 0; w < kAttnWaves; ++w) t += part[w][tid][l];
      sc[l] = t;
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
  const int d8 = (D / H) / 8;  // 16-byte pieces per head
  for (int cg = tid; cg < dp; cg += kAttnThreads) {
    const int h = cg / d8;
    float o[kMaxQ][8];
#pragma unroll
    for (int q = 0; q < kMaxQ; ++q)
#pragma unroll
      for (int e = 0; e < 8; ++e) o[q][e] = 0.f;
#pragma unroll 8
    for (int l = 0; l < L; ++l) {
      const u32x4 g = g_tok[(size_t)l * dp + cg];
      float gv[8];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        gv[2 * e] = __uint_as_float(g[e] << 16);
        gv[2 * e + 1] = __uint_as_float(g[e] & 0xffff0000u);
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
#pragma unroll
    for (int q = 0; q < kMaxQ; ++q) {
      if (q < Q) {
        u32x4 w;
#pragma unroll
        for (int e = 0; e < 4; ++e)
          w[e] = (uint32_t)f32_to_bf16(o[q][2 * e]) | ((uint32_t)f32_to_bf16(o[q][2 * e + 1]) << 16);
        pre[((size_t)s * Q + q) * dp + cg] = w;
        if (res.on) res_out[((size_t)s * Q + q) * dp + cg] = f_tok[(size_t)res.layer[q] * dp + cg];
      }
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

hipError_t launch_meta_attn(int32_t S, int32_t L, int32_t D, int32_t H, int32_t Q, const void *feats, const void *v_proj,
                            const void *a_fold, const int32_t *residual_layers, void *pre, void *res_out,
                            hipStream_t s) {
  const int rows_pad = meta_rows_pad(H, Q);
  ResidualLayers res = {};
  if (residual_layers && res_out) {
    res.on = 1;
    for (int q = 0; q < Q; ++q) res.layer[q] = residual_layers[q];
  }
  const bf16_t *a_hi = (const bf16_t *)a_fold, *a_lo = a_hi + (size_t)rows_pad * D;
  constexpr size_t kLds = (size_t)(kAttnWaves + 1) * kMaxRows * kLdsL * sizeof(float);
  hipError_t e = hipFuncSetAttribute((const void *)meta_attn_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLds);
  if (e != hipSuccess) return e;
  meta_attn_kernel<<<S, kAttnThreads, kLds, s>>>(L, D, H, Q, rows_pad / 16, (const u32x4 *)feats, (const u32x4 *)v_proj,
                                          (const u32x4 *)a_hi, (const u32x4 *)a_lo, res, (u32x4 *)pre, (u32x4 *)res_out);
  return hipGetLastError();
}

}  // namespace hb
