// LM head with fused argmax on the bf16 matrix cores of gfx950.
//
// Computes C^T[v, m] = sum_k W[v, k] * H[m, k] tile by tile and never stores it: the weight
// rows are the MFMA "A" operand and the hidden rows the "B" operand, so that one lane's
// accumulators of a 32x32 tile all belong to ONE hidden row m and 16 different vocabulary
// entries v.  The row-wise argmax is then an in-register scan, one exchange between the two
// lane halves, and one 64-bit atomic max per (row, workgroup).
//
// Workgroup: 512 threads = 8 wavefronts (two per SIMD) in a 4 (v) x 2 (m) arrangement; workgroup
// tile TV = 256 vocabulary rows x TM = 64 * MT hidden rows, K step 64.  Both operands are
// K-contiguous in memory ([V, K] and [M, K] row-major), which is exactly what the MFMA operand
// layout wants (8 consecutive k per lane), so tiles go global -> LDS directly as 16-byte pieces
// (global_load_lds), XOR-swizzled so that the 16-byte operand reads of 8 consecutive rows hit
// all banks.  Weight tiles sit in a ring of three LDS stages and are fetched two K steps ahead,
// hidden tiles in two stages one step ahead; one barrier per K step, placed before the step's
// last MFMAs (see the pipeline comment in the kernel).
//
// What bounds the kernel is the path L2 -> LDS: a 256 x 192 tile needs one operand byte per 110
// flop, and all CUs together draw about 10 KB per clock from the L2s at best, so operand
// delivery and the matrix cores are busy for about the same number of cycles.  Everything here
// serves to keep both going at once: loads in flight across barriers, no burst at a step start,
// workgroups in lockstep so that shared tiles are fetched from HBM once.
//
// Grid: persistent workgroups, one per CU, in groups that walk the vocabulary tiles in lockstep
// (one hidden tile per member) on one XCD.
#include "hb_internal.h"

namespace hb {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int BK = 64;           // k per step
constexpr int TV = 256;          // vocabulary rows per workgroup
constexpr int CH = BK / 8;       // 16-byte pieces per row per step (8)
constexpr int kXcds = 8;

// Offset (in 16-byte pieces) of piece `c` of row `r` in a swizzled [rows][8] tile.  Rows are
// 128 bytes; the XOR spreads the same logical piece of 8 consecutive rows, and of 8 consecutive
// rows of equal parity, over distinct 16-byte bank groups, which keeps the operand reads
// (lanes = consecutive rows, one piece each) conflict free for 128- and 256-byte wide LDS.
__device__ inline int swz(int r, int c) { return r * CH + (c ^ ((r & 7) ^ ((r >> 3) & 1))); }

// MT: 32-row hidden tiles per wavefront (the workgroup covers TM = 64 * MT hidden rows).
// WV: wavefront rows along the vocabulary (2 or 4); the workgroup has 2 * WV wavefronts, each
// with VT = 8 / WV vocabulary tiles of 32 rows.  WV = 4 (eight wavefronts, two per SIMD, at most
// 256 registers each) lets one wavefront's matrix work cover the other's LDS, barrier and
// memory waits.
// WNT: weight loads carry the non-temporal hint.  With one hidden tile nobody shares a weight
// tile, and streaming it through L2 without displacing the hidden rows is worth 5 %; with several
// hidden tiles the hint evicts weight lines before all sharers have read them.
template <int MT, int WV, bool WNT>
__global__ __launch_bounds__(128 * WV) void lmhead_mfma_kernel(int M, int K, int V, int m_tiles, int v_tiles, int groups, int spare, int spare_tiles,
                                                          const u32x4 *__restrict__ hidden,
                                                          const u32x4 *__restrict__ weight,
                                                          unsigned long long *__restrict__ keys) {
  constexpr int TM = 64 * MT;
  constexpr int NT = 128 * WV;             // threads
  constexpr int VT = 8 / WV;               // 32-row vocabulary tiles per wavefront
  extern __shared__ u32x4 lds[];           // [3][TV*CH] weight, then [2][TM*CH] hidden
  u32x4 *lw = lds;
  u32x4 *lh = lds + 3 * TV * CH;
  // per-row candidates of the epilogue; reuses the weight stages once the K loop is over
  unsigned long long (*row_key)[TM] = reinterpret_cast<unsigned long long (*)[TM]>(lds);
  static_assert(WV * TM * 8 <= 3 * TV * CH * 16, "row_key fits in the weight stages");

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wv = wave >> 1;  // which 32*VT vocabulary rows of the tile
  const int wm = wave & 1;   // which 32*MT hidden rows of the tile

  // Persistent workgroups in lockstep groups.  Workgroup ids go round-robin to the XCDs
  // (id % 8); on each XCD the grid places `groups` groups of m_tiles workgroups, one workgroup
  // per CU.  The workgroups of a group take the same sequence of vocabulary tiles, one hidden
  // tile each; having identical work they advance together, so the weight tile they share is
  // fetched from HBM once and found in the XCD's L2 by the others, and the groups of an XCD read
  // the same K range of the hidden rows at about the same time.
  // When the groups do not fill the XCD's CUs, the `spare` remaining workgroups of each XCD take
  // the XCD's first `spare_tiles` vocabulary tiles off the groups' hands, as units of one
  // (vocabulary tile, hidden tile) pair dealt round-robin, so that the groups need one round
  // fewer; consecutive units share the weight tile, which the spare workgroups therefore read at
  // about the same time.
  const int id = blockIdx.x;
  const int xcd = id % kXcds;
  const int slot = id / kXcds;
  const int in_group = groups * m_tiles;
  const bool is_spare = slot >= in_group;
  const int kp = K / 8;  // 16-byte pieces per matrix row (K % 8 == 0)
#pragma unroll 1
  for (int it = 0;; ++it) {
  int nth, m_tile;  // the XCD's nth vocabulary tile against hidden tile m_tile
  if (!is_spare) {
    nth = spare_tiles + slot / m_tiles + it * groups;
    m_tile = slot % m_tiles;
  } else {
    const int unit = slot - in_group + it * spare;
    if (unit >= spare_tiles * m_tiles) break;
    nth = unit / m_tiles;
    m_tile = unit - nth * m_tiles;
  }
  const int v_tile = nth * kXcds + xcd;
  if (v_tile >= v_tiles) break;
  const int m0 = m_tile * TM;
  const int v0 = v_tile * TV;

#define HB_GEMM_W_ROW(t_) (v0 + (t_))
#include "mfma_gemm_tile.inc"
#undef HB_GEMM_W_ROW

  // Epilogue.  Accumulator r of lane l in tile (i, j) is C^T[v, m] with
  //   v = v0 + wv*32*VT + i*32 + 8*(r/4) + 4*(l/32) + r%4,   m = m0 + wm*32*MT + j*32 + l%32.
  // Scanning (i, r) in order visits v in increasing order, so a strict '>' keeps the lowest v
  // among equal values; NaN compares false and never wins.
#pragma unroll
  for (int j = 0; j < MT; ++j) {
    float best = -__builtin_huge_valf();
    int best_v = -1;
#pragma unroll
    for (int i = 0; i < VT; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        int v = v0 + wv * 32 * VT + i * 32 + 8 * (r >> 2) + 4 * frag_half + (r & 3);
        float x = acc[i][j][r];
        bool take = (v < V) && (x > best);
        best = take ? x : best;
        best_v = take ? v : best_v;
      }
    // a lane that saw nothing above -inf offers no candidate (key 0 loses to every real key)
    unsigned long long key = best_v >= 0 ? argmax_key(best, (uint32_t)best_v) : 0ull;
    unsigned long long other = __shfl_xor(key, 32, 64);
    key = other > key ? other : key;
    if (lane < 32) row_key[wv][wm * 32 * MT + j * 32 + lane] = key;
  }
  __syncthreads();
  for (int r = tid; r < TM; r += NT) {
    int m = m0 + r;
    if (m >= M) continue;
    unsigned long long key = row_key[0][r];
#pragma unroll
    for (int w = 1; w < WV; ++w) key = row_key[w][r] > key ? row_key[w][r] : key;
    // skip the atomic when the row already holds something at least as good
    if (key > __atomic_load_n(&keys[m], __ATOMIC_RELAXED)) atomicMax(&keys[m], key);
  }
  __syncthreads();  // row_key shares LDS with the stages the next vocabulary tile fills
  }  // vocabulary tiles of this workgroup
}

template <int MT, int WV, bool WNT>
hipError_t launch(int M, int K, int V, const void *hidden, const void *weight, unsigned long long *keys,
                  hipStream_t s) {
  constexpr int TM = 64 * MT;
  int m_tiles = (M + TM - 1) / TM;
  int v_tiles = (V + TV - 1) / TV;
  // groups per XCD: at most as many as its 32 CUs hold with one workgroup per CU; then the
  // fewest that still need the same number of rounds, so that every group gets the same number
  // of vocabulary tiles (594 tiles of one hidden tile: 25 groups x 3 rounds per XCD instead of 32
  // groups of which a third work a round longer)
  int max_groups = 32 / m_tiles;
  if (max_groups < 1) max_groups = 1;
  int need = (v_tiles + kXcds - 1) / kXcds;
  int rounds = (need + max_groups - 1) / max_groups;
  int groups = (need + rounds - 1) / rounds;
  // CUs of an XCD that no group occupies: if handing them a few vocabulary tiles (every XCD has
  // at least v_tiles / 8) saves the groups a round, do so (960 rows = 5 hidden tiles: 6 groups
  // on 30 CUs would need 13 rounds for 75 tiles; with 3 tiles on the 2 other CUs, 15 units in 8
  // rounds, they need 12).  The fewest tiles that reach the best round count are handed over.
  int spare = 0, spare_tiles = 0;
  if (m_tiles <= 32) {
    const int left = 32 - max_groups * m_tiles;
    int best = rounds;
    for (int y = 1; left > 0 && y <= v_tiles / kXcds; ++y) {
      const int full = (need - y + max_groups - 1) / max_groups;
      const int mine = (y * m_tiles + left - 1) / left;
      const int cost = full > mine ? full : mine;
      if (cost < best) {
        best = cost;
        spare = left;
        spare_tiles = y;
      }
    }
    if (spare) groups = max_groups;
  }
  size_t lds_bytes = (size_t)(3 * TV + 2 * TM) * CH * sizeof(u32x4);
  auto kern = lmhead_mfma_kernel<MT, WV, WNT>;
  hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
  if (e != hipSuccess) return e;
  dim3 grid((unsigned)((groups * m_tiles + spare) * kXcds));
  kern<<<grid, 128 * WV, lds_bytes, s>>>(M, K, V, m_tiles, v_tiles, groups, spare, spare_tiles, (const u32x4 *)hidden, (const u32x4 *)weight, keys);
  return hipGetLastError();
}

}  // namespace

bool lmhead_mfma_supports(int32_t dtype, int32_t M, int32_t K, int32_t V) {
  return dtype == HB_BF16 && K % BK == 0 && M >= 1 && V >= 1;  // other K: the scalar kernel
}

hipError_t launch_lmhead_mfma(int32_t M, int32_t K, int32_t V, const void *hidden, const void *weight,
                              unsigned long long *keys, hipStream_t s) {
  // hidden tile height: the multiple of 64 (up to 256) that wastes the fewest padded rows,
  // preferring the taller tile on ties (fewer re-reads of the weight tile)
  int best_mt = 4;
  long best_rows = -1;
  for (int mt = 4; mt >= 1; --mt) {
    int tm = 64 * mt;
    long rows = (long)((M + tm - 1) / tm) * tm;
    if (best_rows < 0 || rows < best_rows) { best_rows = rows; best_mt = mt; }
  }
  switch (best_mt) {
    case 1: return M <= 64 * 1 ? launch<1, 4, true>(M, K, V, hidden, weight, keys, s)
                            : launch<1, 4, false>(M, K, V, hidden, weight, keys, s);
    case 2: return M <= 64 * 2 ? launch<2, 4, true>(M, K, V, hidden, weight, keys, s)
                            : launch<2, 4, false>(M, K, V, hidden, weight, keys, s);
    case 3: return M <= 64 * 3 ? launch<3, 4, true>(M, K, V, hidden, weight, keys, s)
                            : launch<3, 4, false>(M, K, V, hidden, weight, keys, s);
    default: return M <= 64 * 4 ? launch<4, 4, true>(M, K, V, hidden, weight, keys, s)
                            : launch<4, 4, false>(M, K, V, hidden, weight, keys, s);
  }
}

}  // namespace hb
