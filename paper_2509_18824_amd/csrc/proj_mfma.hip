// The target's projections around the tree-verify attention, on the bf16 matrix cores:
//   * fused query/key/value projection + bias + rotary embedding, written straight into the
//     layouts hb_tree_verify_attn reads (q [T, Hq, D], k_tree / v_tree [T, Hkv, D]);
//   * output projection (a plain  out = x W^T (+ residual)  in bf16 with fp32 accumulation);
//   * the gated-SiLU half of the feed-forward block, out = silu(x Wg^T) * (x Wu^T), gate and up
//     projection in one pass (the down projection is the plain one with the residual);
//   * root-mean-square normalisation of the rows;
//   * the two small kernels that give every tree node its position (prefix length + depth) and
//     the cosine / sine table of those positions.
// The matrix work is the tile loop of the LM head (mfma_gemm_tile.inc: C^T = W H^T, weight rows
// as the MFMA "A" operand, so a lane's accumulators of a 32x32 tile are 16 output features of ONE
// token).  For the rotary embedding the 256 weight rows of a tile are not taken in memory order:
// a tile holds two heads, and the rows are arranged so that the two accumulators a lane holds at
// the same position of its two 32-row sub-tiles are the pair (d, d + 64) of one head, which is
// what the rotate-half convention rotates together: the rotation costs no exchange at all.  The
// gated projection uses the same device: a tile holds 128 features, the gate rows in the first
// 32-row sub-tile of every wavefront row and the matching up rows in the second, so silu(gate) * up
// is one lane's own two accumulators.
#include "hb_internal.h"

namespace hb {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int BK = 64;
constexpr int TV = 256;
constexpr int CH = BK / 8;
constexpr int kXcds = 8;
constexpr int kHeadDim = 128;

__device__ inline int swz(int r, int c) { return r * CH + (c ^ ((r & 7) ^ ((r >> 3) & 1))); }

__device__ inline uint32_t pack_bf16(float a, float b) { return (uint32_t)f32_to_bf16(a) | ((uint32_t)f32_to_bf16(b) << 16); }

struct QkvArgs {
  const bf16_t *bias;      // [(Hq + 2 Hkv) * 128] or null
  const float *cos, *sin;  // [M, 64]
  bf16_t *q, *k, *v;       // [M, Hq, 128], [M, Hkv, 128], [M, Hkv, 128]
  int Hq, Hkv;
};
struct StoreArgs {
  const bf16_t *residual;  // [M, N] or null
  bf16_t *out;             // [M, N]
};

// ROPE: query/key/value projection with rotary embedding (V = (Hq + 2 Hkv) * 128 weight rows),
// else plain projection.  One workgroup per (weight tile, hidden tile); the workgroups that share
// a weight tile get neighbouring slots of one XCD (ids 8 apart) and find it in that XCD's L2.
template <int MT, bool ROPE, bool GLU>
__global__ __launch_bounds__(512) void proj_mfma_kernel(int M, int K, int V, int m_tiles, int v_tiles,
                                                        const u32x4 *__restrict__ hidden,
                                                        const u32x4 *__restrict__ weight, QkvArgs qa, StoreArgs sa) {
  constexpr int WV = 4;
  constexpr bool WNT = false;
  constexpr int TM = 64 * MT;
  constexpr int VT = 8 / WV;
  extern __shared__ u32x4 lds[];
  u32x4 *lw = lds;
  u32x4 *lh = lds + 3 * TV * CH;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wv = wave >> 1;
  const int wm = wave & 1;
  const int id = blockIdx.x;
  const int xcd = id % kXcds, slot = id / kXcds;
  const int v_tile = (slot / m_tiles) * kXcds + xcd;
  const int m_tile = slot % m_tiles;
  if (v_tile >= v_tiles) return;
  const int m0 = m_tile * TM;
  const int v0 = v_tile * TV;
  const int kp = K / 8;

  // Tile row t (wavefront row wv = t / 64, sub-tile i = (t % 64) / 32, rr = t % 32) holds, for the
  // rotary variant, feature  (wv / 2) * 128 + (wv % 2) * 32 + 64 i + rr  of the tile's two heads.
  // ... and for the gated projection (V = 2 F weight rows: F gate rows, then F up rows) feature
  // v0 / 2 + 32 wv + rr of the gate (i = 0) or of the up projection (i = 1).
#define HB_GEMM_W_ROW(t_) (ROPE ? v0 + (((t_) >> 7) << 7) + ((((t_) >> 6) & 1) << 5) + ((((t_) >> 5) & 1) << 6) + ((t_) & 31) \
                           : GLU ? (((t_) >> 5) & 1) * (V >> 1) + (v0 >> 1) + (((t_) >> 6) << 5) + ((t_) & 31)                  \
                                 : v0 + (t_))
#include "mfma_gemm_tile.inc"
#undef HB_GEMM_W_ROW

  // Epilogue.  Accumulator r = 4 c + e of lane l in tile (i, j): tile row wv*64 + i*32 + 8 c +
  // 4 (l / 32) + e, token m0 + wm*32*MT + j*32 + l % 32.
#pragma unroll
  for (int j = 0; j < MT; ++j) {
    const int m = m0 + wm * 32 * MT + j * 32 + frag_row;
    if (m >= M) continue;
    if (ROPE) {
      const int head = (v0 >> 7) + (wv >> 1);
      if (head >= qa.Hq + 2 * qa.Hkv) continue;  // second half of the last tile when the heads are odd in number
      const bool rotate = head < qa.Hq + qa.Hkv;
      bf16_t *dst = head < qa.Hq ? qa.q + ((size_t)m * qa.Hq + head) * kHeadDim
                    : head < qa.Hq + qa.Hkv ? qa.k + ((size_t)m * qa.Hkv + (head - qa.Hq)) * kHeadDim
                                            : qa.v + ((size_t)m * qa.Hkv + (head - qa.Hq - qa.Hkv)) * kHeadDim;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int d = (wv & 1) * 32 + 8 * c + 4 * frag_half;  // d .. d + 3 and d + 64 .. d + 67
        float x1[4], x2[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          x1[e] = acc[0][j][4 * c + e];
          x2[e] = acc[1][j][4 * c + e];
        }
        if (qa.bias) {
          const u32x2 b1 = *(const u32x2 *)(qa.bias + head * kHeadDim + d);
          const u32x2 b2 = *(const u32x2 *)(qa.bias + head * kHeadDim + d + 64);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            x1[e] += __uint_as_float((e & 1) ? (b1[e >> 1] & 0xffff0000u) : (b1[e >> 1] << 16));
            x2[e] += __uint_as_float((e & 1) ? (b2[e >> 1] & 0xffff0000u) : (b2[e >> 1] << 16));
          }
        }
        if (rotate) {
          const f32x4 cs = *(const f32x4 *)(qa.cos + (size_t)m * 64 + d);
          const f32x4 sn = *(const f32x4 *)(qa.sin + (size_t)m * 64 + d);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float a = x1[e] * cs[e] - x2[e] * sn[e];
            const float b = x2[e] * cs[e] + x1[e] * sn[e];
            x1[e] = a;
            x2[e] = b;
          }
        }
        *(u32x2 *)(dst + d) = (u32x2){pack_bf16(x1[0], x1[1]), pack_bf16(x1[2], x1[3])};
        *(u32x2 *)(dst + d + 64) = (u32x2){pack_bf16(x2[0], x2[1]), pack_bf16(x2[2], x2[3])};
      }
    } else if (GLU) {
      const int F = V >> 1;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int f = (v0 >> 1) + wv * 32 + 8 * c + 4 * frag_half;  // f .. f + 3, F % 4 == 0
        if (f >= F) continue;
        float y[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float g = acc[0][j][4 * c + e];
          y[e] = g / (1.f + __expf(-g)) * acc[1][j][4 * c + e];
        }
        *(u32x2 *)(sa.out + (size_t)m * F + f) = (u32x2){pack_bf16(y[0], y[1]), pack_bf16(y[2], y[3])};
      }
    } else {
#pragma unroll
      for (int i = 0; i < VT; ++i)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int n = v0 + wv * 32 * VT + i * 32 + 8 * c + 4 * frag_half;  // n .. n + 3, V % 4 == 0
          if (n >= V) continue;
          float x[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) x[e] = acc[i][j][4 * c + e];
          if (sa.residual) {
            const u32x2 r = *(const u32x2 *)(sa.residual + (size_t)m * V + n);
#pragma unroll
            for (int e = 0; e < 4; ++e) x[e] += __uint_as_float((e & 1) ? (r[e >> 1] & 0xffff0000u) : (r[e >> 1] << 16));
          }
          *(u32x2 *)(sa.out + (size_t)m * V + n) = (u32x2){pack_bf16(x[0], x[1]), pack_bf16(x[2], x[3])};
        }
    }
  }
}

template <int MT, bool ROPE, bool GLU>
hipError_t launch(int M, int K, int V, const void *hidden, const void *weight, const QkvArgs &qa, const StoreArgs &sa,
                  hipStream_t s) {
  constexpr int TM = 64 * MT;
  const int m_tiles = (M + TM - 1) / TM;
  const int v_tiles = (V + TV - 1) / TV;
  const size_t lds_bytes = (size_t)(3 * TV + 2 * TM) * CH * sizeof(u32x4);
  auto kern = proj_mfma_kernel<MT, ROPE, GLU>;
  hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
  if (e != hipSuccess) return e;
  dim3 grid((unsigned)((v_tiles + kXcds - 1) / kXcds * kXcds * m_tiles));
  kern<<<grid, 512, lds_bytes, s>>>(M, K, V, m_tiles, v_tiles, (const u32x4 *)hidden, (const u32x4 *)weight, qa, sa);
  return hipGetLastError();
}

// ---- few tokens: split K ---------------------------------------------------------------------
// With few tokens a projection is a stream of its weight matrix from HBM, and one workgroup per
// 256-row weight tile and hidden tile would give work to a few dozen CUs only.  Here the K range
// of every tile is cut into `ks` parts, one workgroup per (weight tile, K part, hidden tile); the
// workgroups that differ in the hidden tile only, which read the same weights, get neighbouring
// slots of one XCD.  A workgroup runs the same tile loop over its part and stores its fp32
// accumulators to the caller's workspace as part[kpart][weight row][token] (tokens contiguous: a
// lane's 32 neighbours hold consecutive tokens of one weight row).  proj_reduce_kernel then sums
// the parts in order and applies the epilogue (bias, rotary embedding, residual), one thread per
// token and group of four features (for the rotary variant: four (d, d + 64) pairs).
template <int MT>
__global__ __launch_bounds__(512) void proj_splitk_kernel(int M, int Kfull, int V, int ks, int v_pad, int m_tiles,
                                                          int m_pad, int units,
                                                          const u32x4 *__restrict__ hidden_full,
                                                          const u32x4 *__restrict__ weight_full,
                                                          float *__restrict__ part) {
  constexpr int WV = 4;
  constexpr bool WNT = false;  // measured: the non-temporal hint costs 10-25 % here, also with a single hidden tile
  constexpr int TM = 64 * MT;
  constexpr int VT = 8 / WV;
  extern __shared__ u32x4 lds[];
  u32x4 *lw = lds;
  u32x4 *lh = lds + 3 * TV * CH;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wv = wave >> 1;
  const int wm = wave & 1;
  const int xcd = blockIdx.x % kXcds, slot = blockIdx.x / kXcds;
  const int unit = (slot / m_tiles) * kXcds + xcd;  // (weight tile, K part)
  if (unit >= units) return;
  const int v_tile = unit / ks, kpart = unit % ks;
  const int m0 = (slot % m_tiles) * TM;
  const int v0 = v_tile * TV;
  const int K = Kfull / ks;          // this workgroup's share
  const int kp = Kfull / 8;          // row stride in 16-byte pieces
  const u32x4 *hidden = hidden_full + (size_t)kpart * (K / 8);
  const u32x4 *weight = weight_full + (size_t)kpart * (K / 8);
#define HB_GEMM_W_ROW(t_) (v0 + (t_))
#include "mfma_gemm_tile.inc"
#undef HB_GEMM_W_ROW
  float *dst = part + ((size_t)kpart * v_pad + v0) * m_pad + m0;
#pragma unroll
  for (int i = 0; i < VT; ++i)
#pragma unroll
    for (int j = 0; j < MT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = wv * 32 * VT + i * 32 + 8 * (r >> 2) + 4 * frag_half + (r & 3);
        dst[(size_t)row * m_pad + wm * 32 * MT + j * 32 + frag_row] = acc[i][j][r];
      }
}

template <bool ROPE, bool GLU>
__global__ __launch_bounds__(256) void proj_reduce_kernel(int M, int V, int ks, int v_pad, int tm,
                                                          const float *__restrict__ part, QkvArgs qa, StoreArgs sa) {
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  const int m = (int)(idx % tm);
  const int g = (int)(idx / tm);
  if (m >= M) return;
  if (ROPE) {
    const int head = g >> 4, d = (g & 15) * 4;
    if (head >= qa.Hq + 2 * qa.Hkv) return;
    float x1[4] = {0.f, 0.f, 0.f, 0.f}, x2[4] = {0.f, 0.f, 0.f, 0.f};
    for (int kpart = 0; kpart < ks; ++kpart) {
      const float *src = part + ((size_t)kpart * v_pad + head * kHeadDim + d) * tm + m;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        x1[e] += src[(size_t)e * tm];
        x2[e] += src[(size_t)(64 + e) * tm];
      }
    }
    if (qa.bias) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        x1[e] += bf16_to_f32(qa.bias[head * kHeadDim + d + e]);
        x2[e] += bf16_to_f32(qa.bias[head * kHeadDim + 64 + d + e]);
      }
    }
    const bool rotate = head < qa.Hq + qa.Hkv;
    bf16_t *dst = head < qa.Hq ? qa.q + ((size_t)m * qa.Hq + head) * kHeadDim
                  : head < qa.Hq + qa.Hkv ? qa.k + ((size_t)m * qa.Hkv + (head - qa.Hq)) * kHeadDim
                                          : qa.v + ((size_t)m * qa.Hkv + (head - qa.Hq - qa.Hkv)) * kHeadDim;
    if (rotate) {
      const f32x4 cs = *(const f32x4 *)(qa.cos + (size_t)m * 64 + d);
      const f32x4 sn = *(const f32x4 *)(qa.sin + (size_t)m * 64 + d);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float a = x1[e] * cs[e] - x2[e] * sn[e];
        const float b = x2[e] * cs[e] + x1[e] * sn[e];
        x1[e] = a;
        x2[e] = b;
      }
    }
    *(u32x2 *)(dst + d) = (u32x2){pack_bf16(x1[0], x1[1]), pack_bf16(x1[2], x1[3])};
    *(u32x2 *)(dst + d + 64) = (u32x2){pack_bf16(x2[0], x2[1]), pack_bf16(x2[2], x2[3])};
  } else if (GLU) {
    const int F = V >> 1, f = g * 4;
    if (f >= F) return;
    float xg[4] = {0.f, 0.f, 0.f, 0.f}, xu[4] = {0.f, 0.f, 0.f, 0.f};
    for (int kpart = 0; kpart < ks; ++kpart) {
      const float *src = part + ((size_t)kpart * v_pad + f) * tm + m;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        xg[e] += src[(size_t)e * tm];
        xu[e] += src[(size_t)(F + e) * tm];
      }
    }
    float y[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) y[e] = xg[e] / (1.f + __expf(-xg[e])) * xu[e];
    *(u32x2 *)(sa.out + (size_t)m * F + f) = (u32x2){pack_bf16(y[0], y[1]), pack_bf16(y[2], y[3])};
  } else {
    const int n = g * 4;
    if (n >= V) return;
    float x[4] = {0.f, 0.f, 0.f, 0.f};
    for (int kpart = 0; kpart < ks; ++kpart) {
      const float *src = part + ((size_t)kpart * v_pad + n) * tm + m;
#pragma unroll
      for (int e = 0; e < 4; ++e) x[e] += src[(size_t)e * tm];
    }
    if (sa.residual) {
      const u32x2 r = *(const u32x2 *)(sa.residual + (size_t)m * V + n);
#pragma unroll
      for (int e = 0; e < 4; ++e) x[e] += __uint_as_float((e & 1) ? (r[e >> 1] & 0xffff0000u) : (r[e >> 1] << 16));
    }
    *(u32x2 *)(sa.out + (size_t)m * V + n) = (u32x2){pack_bf16(x[0], x[1]), pack_bf16(x[2], x[3])};
  }
}

// Hidden tile height (64 mt rows) of the unsplit kernel by a small cost model: a workgroup's time
// per K step is about 1 + 0.55 mt units (staging of the 256-row weight tile + mt x the matrix work
// of 64 rows, from the LM head's measured 2100 clocks at mt = 3); one workgroup per CU at a time,
// so the launch takes ceil(units / 256) rounds of that.  960 x 4608: mt = 2 (144 units, one round)
// beats mt = 1 (270 units: a second round for 14 of them) and mt = 3 (90 units).
int plain_tile_height(int M, int v_tiles) {
  int mt = 1;
  double best = 1e30;
  for (int t = 1; t <= 4; ++t) {
    const long units = (long)v_tiles * ((M + 64 * t - 1) / (64 * t));
    const double cost = (double)((units + 255) / 256) * (1.0 + 0.55 * t);
    if (cost < best - 1e-9) { best = cost; mt = t; }
  }
  return mt;
}

// The split over K: hidden tile height (64 mt rows) and K parts (a divisor of the K steps, at
// least kMinSteps steps per part, all workgroups resident at once), by a cost model fitted to
// measurements on weights too many to stay in the last-level cache (microseconds):
//   split:  6 + steps / ks * (0.70 | 0.86 | 1.15 | 1.45 for mt = 1 .. 4) + partial bytes written and read / 4 TB/s
//   plain:  3 + steps * 0.75 per round of 256 workgroups (at most 512 tokens)
//           3 + steps * (0.72 | 0.95 | 1.15 | 1.4 for the unsplit kernel's mt) per round (more tokens)
// Up to 512 tokens the tile is 64 or 128 rows high; from there to kSplitMaxM tokens 128 to 256 rows,
// and the split must win by 10 % (it does for long K: the feed-forward block's down projection,
// 960 x 18944 -> 3584, takes 145 us in 4 parts of 256-row tiles against 209 us unsplit; with K =
// 3584 the unsplit kernel stays).  ks = 1 means: do not split.
constexpr int kSplitMaxM = 1024;
constexpr int kMinSteps = 4;
struct SplitPlan {
  int ks, mt;
};
SplitPlan split_plan(int M, int K, int V) {
  SplitPlan best = {1, 1};
  if (M > kSplitMaxM || K % BK) return best;
  const int steps = K / BK, v_tiles = (V + TV - 1) / TV;
  const bool few = M <= 512;
  static const double kStepSplit[5] = {0, 0.70, 0.86, 1.15, 1.45}, kStepPlain[5] = {0, 0.72, 0.95, 1.15, 1.4};
  double best_cost;
  if (few) {
    const long plain_units = (long)v_tiles * ((M + 63) / 64);
    best_cost = 3.0 + steps * 0.75 * (double)((plain_units + 255) / 256);
  } else {
    const int pm = plain_tile_height(M, v_tiles);
    const long plain_units = (long)v_tiles * ((M + 64 * pm - 1) / (64 * pm));
    best_cost = 0.9 * (3.0 + steps * kStepPlain[pm] * (double)((plain_units + 255) / 256));
  }
  for (int mt = few ? 1 : 2; mt <= (few ? 2 : 4); ++mt) {
    const int m_tiles = (M + 64 * mt - 1) / (64 * mt);
    for (int d = 2; d <= steps; ++d) {
      if (steps % d || steps / d < kMinSteps || (long)v_tiles * m_tiles * d > 256) continue;
      const double bytes = 8.0 * d * v_tiles * TV * m_tiles * 64 * mt;
      const double cost = 6.0 + (double)(steps / d) * kStepSplit[mt] + bytes / 4e6;
      if (cost < best_cost - 1e-9) {
        best_cost = cost;
        best = {d, mt};
      }
    }
  }
  return best;
}

template <bool ROPE, bool GLU>
hipError_t launch_splitk(int M, int K, int V, SplitPlan plan, const void *hidden, const void *weight, const QkvArgs &qa,
                         const StoreArgs &sa, float *part, hipStream_t s) {
  const int ks = plan.ks, tm = 64 * plan.mt;
  const int m_tiles = (M + tm - 1) / tm, m_pad = m_tiles * tm;
  const int v_tiles = (V + TV - 1) / TV, v_pad = v_tiles * TV;
  const int units = v_tiles * ks;
  const unsigned grid = (unsigned)((units + kXcds - 1) / kXcds * kXcds * m_tiles);
  const size_t lds_bytes = (size_t)(3 * TV + 2 * tm) * CH * sizeof(u32x4);
  hipError_t e;
  switch (plan.mt) {
#define HB_SPLITK_CASE(MT_)                                                                                       \
  case MT_: {                                                                                                     \
    auto kern = proj_splitk_kernel<MT_>;                                                                          \
    e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);      \
    if (e != hipSuccess) return e;                                                                                \
    kern<<<grid, 512, lds_bytes, s>>>(M, K, V, ks, v_pad, m_tiles, m_pad, units, (const u32x4 *)hidden,           \
                                      (const u32x4 *)weight, part);                                               \
  } break;
    HB_SPLITK_CASE(1)
    HB_SPLITK_CASE(2)
    HB_SPLITK_CASE(3)
    HB_SPLITK_CASE(4)
#undef HB_SPLITK_CASE
    default: return hipErrorInvalidValue;
  }
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  const long groups = ROPE ? (long)(V / kHeadDim) * 16 : GLU ? (V / 2 + 3) / 4 : (V + 3) / 4;
  const long threads = groups * m_pad;
  proj_reduce_kernel<ROPE, GLU><<<(unsigned)((threads + 255) / 256), 256, 0, s>>>(M, V, ks, v_pad, m_pad, part, qa, sa);
  return hipGetLastError();
}

template <bool ROPE, bool GLU>
hipError_t dispatch(int M, int K, int V, const void *hidden, const void *weight, const QkvArgs &qa, const StoreArgs &sa,
                    hipStream_t s) {
  const int mt = plain_tile_height(M, (V + TV - 1) / TV);
  switch (mt) {
    case 4: return launch<4, ROPE, GLU>(M, K, V, hidden, weight, qa, sa, s);
    case 3: return launch<3, ROPE, GLU>(M, K, V, hidden, weight, qa, sa, s);
    case 2: return launch<2, ROPE, GLU>(M, K, V, hidden, weight, qa, sa, s);
    default: return launch<1, ROPE, GLU>(M, K, V, hidden, weight, qa, sa, s);
  }
}

// positions[n] = prefix_len[b] + depth(n); one wavefront per sequence, one lane per node
__global__ __launch_bounds__(64) void tree_positions_kernel(int max_nodes, int total_nodes,
                                                           const int32_t *__restrict__ node_offset,
                                                           const int32_t *__restrict__ parent,
                                                           const int32_t *__restrict__ prefix_len,
                                                           int32_t *__restrict__ positions) {
  __shared__ int32_t spar[64];
  const int b = blockIdx.x, lane = threadIdx.x;
  const int n0 = node_offset[b];
  int n = node_offset[b + 1] - n0;
  n = n < 0 ? 0 : (n > max_nodes ? max_nodes : n);
  if (n0 < 0 || n0 + n > total_nodes) n = 0;
  int par = -1;
  if (lane < n) {
    par = parent[n0 + lane];
    if (par >= lane || par < -1) par = -1;  // malformed: a root
  }
  spar[lane] = par;
  __syncthreads();
  int depth = 0;
  for (int x = par, guard = 0; x >= 0 && guard < 64; ++guard) {
    ++depth;
    x = spar[x];
  }
  if (lane < n) positions[n0 + lane] = prefix_len[b] + depth;
}

// cos / sin of positions[t] * theta^(-d / half), d < half, in double precision (the angle reaches
// tens of thousands of radians), stored as float
__global__ __launch_bounds__(256) void rope_table_kernel(int T, int half, double log2_theta,
                                                        const int32_t *__restrict__ positions,
                                                        float *__restrict__ cos_out, float *__restrict__ sin_out) {
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long)T * half) return;
  const int t = (int)(idx / half), d = (int)(idx - (long)t * half);
  const double inv_freq = exp2(-log2_theta * (double)d / (double)half);
  const double ang = (double)positions[t] * inv_freq;
  double sv, cv;
  sincos(ang, &sv, &cv);
  cos_out[idx] = (float)cv;
  sin_out[idx] = (float)sv;
}

// out[t, :] = x[t, :] / sqrt(mean(x[t, :]^2) + eps) * weight: one workgroup per row, the row is
// read once (16-byte loads, K % 8 == 0) and kept in registers between the two passes when it
// fits (K <= 8192), otherwise read again
__global__ __launch_bounds__(256) void rmsnorm_kernel(int K, const bf16_t *__restrict__ x,
                                                      const bf16_t *__restrict__ weight, float eps,
                                                      bf16_t *__restrict__ out) {
  __shared__ float red[4];
  constexpr int kKeep = 4;  // 16-byte pieces a thread keeps: 4 * 256 * 8 = 8192 values
  const int t = blockIdx.x, tid = threadIdx.x;
  const int pieces = K / 8;
  const u32x4 *row = (const u32x4 *)(x + (size_t)t * K);
  const u32x4 *wv = (const u32x4 *)weight;
  u32x4 *dst = (u32x4 *)(out + (size_t)t * K);
  u32x4 keep[kKeep];
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < kKeep; ++i) {
    const int p = tid + i * 256;
    keep[i] = row[p < pieces ? p : pieces - 1];
  }
#pragma unroll
  for (int i = 0; i < kKeep; ++i) {
    if (tid + i * 256 < pieces) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float a = __uint_as_float(keep[i][e] << 16), b = __uint_as_float(keep[i][e] & 0xffff0000u);
        ss += a * a + b * b;
      }
    }
  }
  for (int p = tid + kKeep * 256; p < pieces; p += 256) {
    const u32x4 v = row[p];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float a = __uint_as_float(v[e] << 16), b = __uint_as_float(v[e] & 0xffff0000u);
      ss += a * a + b * b;
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
  if ((tid & 63) == 0) red[tid >> 6] = ss;
  __syncthreads();
  const float scale = rsqrtf(((red[0] + red[1]) + (red[2] + red[3])) / (float)K + eps);
  auto emit = [&](int p, u32x4 v) {
    const u32x4 w = wv[p];
    u32x4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float a = __uint_as_float(v[e] << 16) * scale * __uint_as_float(w[e] << 16);
      const float b = __uint_as_float(v[e] & 0xffff0000u) * scale * __uint_as_float(w[e] & 0xffff0000u);
      o[e] = pack_bf16(a, b);
    }
    dst[p] = o;
  };
#pragma unroll
  for (int i = 0; i < kKeep; ++i)
    if (tid + i * 256 < pieces) emit(tid + i * 256, keep[i]);
  for (int p = tid + kKeep * 256; p < pieces; p += 256) emit(p, row[p]);
}

}  // namespace

bool proj_mfma_supports(int32_t M, int32_t K, int32_t N) { return M >= 1 && K >= BK && K % BK == 0 && N >= 4 && N % 4 == 0; }

size_t proj_workspace_bytes(int32_t M, int32_t K, int32_t N) {
  const SplitPlan plan = split_plan(M, K, N);
  if (plan.ks <= 1) return 0;
  const size_t v_pad = (size_t)((N + TV - 1) / TV) * TV;
  const size_t tm = 64 * plan.mt, m_pad = (M + tm - 1) / tm * tm;
  return (size_t)plan.ks * v_pad * m_pad * sizeof(float);
}

hipError_t launch_qkv_rope(int32_t M, int32_t K, int32_t Hq, int32_t Hkv, const void *hidden, const void *w_qkv,
                           const void *bias, const float *cos, const float *sin, void *q, void *k, void *v,
                           float *part, hipStream_t s) {
  QkvArgs qa = {(const bf16_t *)bias, cos, sin, (bf16_t *)q, (bf16_t *)k, (bf16_t *)v, Hq, Hkv};
  StoreArgs sa = {nullptr, nullptr};
  const int V = (Hq + 2 * Hkv) * kHeadDim;
  const SplitPlan plan = part ? split_plan(M, K, V) : SplitPlan{1, 1};
  if (plan.ks > 1) return launch_splitk<true, false>(M, K, V, plan, hidden, w_qkv, qa, sa, part, s);
  return dispatch<true, false>(M, K, V, hidden, w_qkv, qa, sa, s);
}

hipError_t launch_linear(int32_t M, int32_t K, int32_t N, const void *x, const void *w, const void *residual, void *out,
                         float *part, hipStream_t s) {
  QkvArgs qa = {};
  StoreArgs sa = {(const bf16_t *)residual, (bf16_t *)out};
  const SplitPlan plan = part ? split_plan(M, K, N) : SplitPlan{1, 1};
  if (plan.ks > 1) return launch_splitk<false, false>(M, K, N, plan, x, w, qa, sa, part, s);
  return dispatch<false, false>(M, K, N, x, w, qa, sa, s);
}

hipError_t launch_swiglu(int32_t M, int32_t K, int32_t F, const void *x, const void *w_gate_up, void *out, float *part,
                         hipStream_t s) {
  QkvArgs qa = {};
  StoreArgs sa = {nullptr, (bf16_t *)out};
  const SplitPlan plan = part ? split_plan(M, K, 2 * F) : SplitPlan{1, 1};
  if (plan.ks > 1) return launch_splitk<false, true>(M, K, 2 * F, plan, x, w_gate_up, qa, sa, part, s);
  return dispatch<false, true>(M, K, 2 * F, x, w_gate_up, qa, sa, s);
}

hipError_t launch_rmsnorm(int32_t T, int32_t K, const void *x, const void *weight, float eps, void *out, hipStream_t s) {
  rmsnorm_kernel<<<T, 256, 0, s>>>(K, (const bf16_t *)x, (const bf16_t *)weight, eps, (bf16_t *)out);
  return hipGetLastError();
}

hipError_t launch_tree_positions(int32_t B, int32_t max_nodes, int32_t total_nodes, const int32_t *node_offset,
                                 const int32_t *parent, const int32_t *prefix_len, int32_t *positions, hipStream_t s) {
  tree_positions_kernel<<<B, 64, 0, s>>>(max_nodes, total_nodes, node_offset, parent, prefix_len, positions);
  return hipGetLastError();
}

hipError_t launch_rope_table(int32_t T, int32_t half, double theta, const int32_t *positions, float *cos, float *sin,
                             hipStream_t s) {
  const long n = (long)T * half;
  rope_table_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(T, half, log2(theta), positions, cos, sin);
  return hipGetLastError();
}

}  // namespace hb
