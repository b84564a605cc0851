// Tree-verify attention on the bf16 matrix cores of gfx950 (head_dim 128, page size 16).
//
// One workgroup owns one (sequence, kv head, KV chunk, row group).  Every KV tile it streams is
// staged once in LDS and used by all query rows of the group: rows of many tree nodes and of
// every query head of the kv group (N * G rows in all, 420 for 60 nodes and GQA 7:1), which is
// what turns the memory-bound decode step into a compute-dense one.  Up to 128 rows: four
// wavefronts, two workgroups per CU.  More: eight wavefronts and up to 256 rows per workgroup
// (staging a tile costs as much as the matrix work on 128 rows, so sharing it among twice the
// rows pays), row groups of one item on one XCD so that they share the KV stream in its L2.
//
// Formulation (transposed, so no score ever crosses lanes on its way into the second GEMM):
//   S^T = K Q^T     MFMA 16x16x32: A = K tile (16 keys x 32 d), B = Q^T (32 d x 16 rows)
//   O^T = V^T P^T   MFMA 16x16x32: A = V^T (16 d x 32 keys),    B = P^T (32 keys x 16 rows)
// The S^T accumulator of lane l holds, for query row l%16, the four keys 4*(l/16)+r of a 16-key
// tile; two such tiles give the eight k-slots that the same lane must supply as the B operand
// of the second MFMA, provided the V^T operand is read with the matching key order (the
// transposing LDS reads of the PV step fetch keys 16h + 4*(l/16) + 0..3 for h = 0, 1).
// Softmax is online per row in base 2 (scores scaled by softmax_scale*log2 e) against a
// reference exponent per row that is shared by the four lane groups of the row (two cross-lane
// exchanges per 32 keys).  The reference is the first block maximum the row sees and moves
// only when a later maximum exceeds it by more than 8 (a factor 256): row maxima of real score
// distributions creep up by small steps all the time, and rescaling the whole accumulator at
// every step would cost more vector work than the attention itself.  Row sums are taken on the
// matrix cores (an all-ones operand against the probabilities).
//
// Rows: row r = node * G + head_in_group, tiles of 16 rows dealt round-robin to the
// wavefronts; Q fragments and the fp32 O^T accumulators of a wavefront's (at most TPW = 2) tiles
// live in vector registers for the whole kernel, within 256 registers so that a CU holds eight
// wavefronts and one's matrix work overlaps another's vector work and waits.
//
// Keys: chunk 0 starts with one 64-key tile holding the tree nodes (masked per row by the
// node's ancestor bitmask), then every chunk streams its share of the prefix through the page
// table in 64-key tiles.  Prefix tiles go global -> LDS directly (no staging registers, no
// transposition in the vector unit) into a ring of LDS stages, several tiles ahead of the one
// being computed; V stays in memory order in LDS and is transposed by the LDS read itself.
#include "hb_internal.h"

namespace hb {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) bf16x4 *lds_bf16x4_ptr;
typedef __attribute__((address_space(1))) const void *gptr_t;
typedef __attribute__((address_space(3))) void *lptr_t;
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int D = 128;
constexpr int PAGE = 16;
constexpr int KT = 64;                 // keys per tile
constexpr int K_PIECES = KT * 16;      // 16-byte pieces of a K tile (16 per key row)
constexpr int V_BYTES = KT * 256;      // V tile: 64 keys x 256 bytes
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kSlack = 8.f;  // log2 units a row maximum may exceed its reference exponent
#define HB_NEG_INF (-__builtin_huge_valf())

__device__ __forceinline__ uint32_t finite_or_zero_bf16x2(uint32_t w) {
  // a bf16 is non-finite iff its exponent field is all ones
  uint32_t lo = ((w & 0x7f80u) == 0x7f80u) ? 0u : (w & 0xffffu);
  uint32_t hi = ((w & 0x7f800000u) == 0x7f800000u) ? 0u : (w & 0xffff0000u);
  return lo | hi;
}

// Where one thread's pieces of a 64-key tile come from.  A tile holds either tree nodes (keys =
// node ids < n_nodes, read from k_tree/v_tree) or prefix positions tile_start + key < end (read
// through the page table).  Slots that are not valid keys are masked in the scores; their V is
// staged as zeros, which keeps 0 * V finite.
struct TileSrc {
  const u32x4 *k_tree, *v_tree, *k_pool, *v_pool;
  const int32_t *bt;  // page table row of the sequence
  int g, n0, n_nodes, hkv, num_blocks;
};

// K: piece (tid % 16) of key tid/16 + 16*i
__device__ __forceinline__ u32x4 load_k_piece(const TileSrc &s, bool tree_tile, int tile_start, int end,
                                              int tid, int i) {
  const int piece = tid & 15;
  const int key = (tid >> 4) + 16 * i;
  u32x4 x = {0u, 0u, 0u, 0u};
  if (tree_tile) {
    if (key < s.n_nodes) x = s.k_tree[((size_t)(s.n0 + key) * s.hkv + s.g) * 16 + piece];
  } else {
    int pos = tile_start + key;
    if (pos < end) {
      int blk = s.bt[pos / PAGE];
      blk = blk < 0 ? 0 : (blk >= s.num_blocks ? s.num_blocks - 1 : blk);
      x = s.k_pool[(((size_t)blk * s.hkv + s.g) * PAGE + (pos % PAGE)) * 16 + piece];
    }
  }
  return x;
}

// V: d-piece (tid % 16) of key 4*(tid/16) + i
__device__ __forceinline__ u32x4 load_v_piece(const TileSrc &s, bool tree_tile, int tile_start, int end,
                                              int tid, int i) {
  const int piece = tid & 15;
  const int key = 4 * (tid >> 4) + i;
  u32x4 x = {0u, 0u, 0u, 0u};
  if (tree_tile) {
    if (key < s.n_nodes) {
      x = s.v_tree[((size_t)(s.n0 + key) * s.hkv + s.g) * 16 + piece];
      // tree nodes off a row's path get probability 0; their V must not turn 0 * V into NaN
      x[0] = finite_or_zero_bf16x2(x[0]);
      x[1] = finite_or_zero_bf16x2(x[1]);
      x[2] = finite_or_zero_bf16x2(x[2]);
      x[3] = finite_or_zero_bf16x2(x[3]);
    }
  } else {
    int pos = tile_start + key;
    if (pos < end) {
      int blk = s.bt[pos / PAGE];
      blk = blk < 0 ? 0 : (blk >= s.num_blocks ? s.num_blocks - 1 : blk);
      x = s.v_pool[(((size_t)blk * s.hkv + s.g) * PAGE + (pos % PAGE)) * 16 + piece];
    }
  }
  return x;
}

// Registers -> LDS, K.  Rows keep their layout ([key][16 pieces]); the piece index is XORed with
// the key so that the operand reads of 16 consecutive keys are conflict free.
__device__ __forceinline__ void store_k(u32x4 *__restrict__ lk, int tid, u32x4 k0, u32x4 k1, u32x4 k2, u32x4 k3) {
  const int piece = tid & 15;
  const int krow = tid >> 4;
  lk[(krow + 0) * 16 + (piece ^ krow)] = k0;   // (krow + 16 i) & 15 == krow
  lk[(krow + 16) * 16 + (piece ^ krow)] = k1;
  lk[(krow + 32) * 16 + (piece ^ krow)] = k2;
  lk[(krow + 48) * 16 + (piece ^ krow)] = k3;
}

// V tile in LDS: rows = keys, 256 bytes each, in memory order ([key][d]); the 16-byte piece index is
// XORed with v_swz(key).  The MFMA wants V^T (8 consecutive keys per lane at one d); the
// transposing LDS read (ds_read_b64_tr_b16) delivers exactly that from this layout: within 16
// lanes, lane i receives element i%4 of the 8 bytes addressed by lanes i/4, i/4+4, i/4+8, i/4+12.
// The swizzle was chosen by timing all XOR patterns of this family on gfx950: with it the
// transposed reads run conflict free (4x faster than unswizzled).
__device__ __forceinline__ int v_swz(int key) { return (key & 7) << 1; }

// Registers -> LDS, V rows of the tree tile: d-piece (tid % 16) of keys 4*(tid/16) .. +3.
__device__ __forceinline__ void store_v(u32x4 *__restrict__ lv, int tid, u32x4 v0, u32x4 v1, u32x4 v2, u32x4 v3) {
  const int piece = tid & 15;
  const int key = 4 * (tid >> 4);
  lv[(key + 0) * 16 + (piece ^ v_swz(key + 0))] = v0;
  lv[(key + 1) * 16 + (piece ^ v_swz(key + 1))] = v1;
  lv[(key + 2) * 16 + (piece ^ v_swz(key + 2))] = v2;
  lv[(key + 3) * 16 + (piece ^ v_swz(key + 3))] = v3;
}

// 2^x by the hardware instruction: arguments here are <= 0 and results below the normal range
// may flush to zero, which is what a vanishing softmax weight should do.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Maximum over the four lanes l, l^16, l^32, l^48 that hold the four key groups of one query
// row.  v_permlane16_swap exchanges rows 1<->0 and 3<->2 (rows of 16 lanes) between its two
// operands, v_permlane32_swap the upper half of one with the lower half of the other: fed the
// same value twice they hand every lane its partner's value next to its own, without the LDS
// round trip of a bpermute.
typedef unsigned int swap2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float group_max(float x) {
  swap2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  x = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
  r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// One 32-key block of the current tile against all row tiles of the wavefront.
//   partial (uniform): some keys of the block do not exist or are masked (chunk tail, tree tile).
// Row tiles are taken in groups of at most four: scores and softmax for the group (VALU work,
// QK^T on the matrix cores), then the group's O^T += V^T P^T.  This file is compiled with the
// matrix instructions in their vector-register form (scores are read by vector instructions
// right away, so accumulation registers would only add copies); after every instruction that
// defines an O^T accumulator an empty asm statement with a "v" constraint keeps the value where
// it is instead of letting it be shuffled around every iteration.
template <int TPW, int NW>
__device__ __forceinline__ void attend_block(bool partial, const u32x4 *__restrict__ lk, const unsigned char *__restrict__ lv,
                                             int blk32, int j, int kg, const bf16x8 (&qf)[TPW][4],
                                             f32x4 (&o)[TPW][8], float (&m_run)[TPW], f32x4 (&l_run)[TPW],
                                             float c1, int n_valid, bool is_tree, const unsigned long long *anc_lds,
                                             int wave, int R, int G) {
  // K fragments of the block's two 16-key halves, shared by all row tiles of the wavefront
  bf16x8 ak[2][4];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      int key = 32 * blk32 + 16 * a + j;
      ak[a][ks] = __builtin_bit_cast(bf16x8, lk[key * 16 + ((4 * ks + kg) ^ j)]);
    }
#pragma unroll
  for (int t0 = 0; t0 < TPW; t0 += 4) {
    constexpr int kGroup = 4;
    // -- scores of the group's tiles, masks, new running maxima (no branches: the matrix and
    //    vector work of different tiles can be interleaved by the scheduler)
    float sc[kGroup][8];
    float lmax[kGroup];
    bool need = false;
#pragma unroll
    for (int u = 0; u < kGroup; ++u) {
      const int t = t0 + u;
      if (t >= TPW) break;
      f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ak[0][ks], qf[t][ks], s0, 0, 0, 0);
        s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ak[1][ks], qf[t][ks], s1, 0, 0, 0);
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        sc[u][r] = s0[r];
        sc[u][4 + r] = s1[r];
      }
      if (partial) {
        // bit k of `allow`: key 32*blk32 + k exists and may be seen by this lane's row.  A select
        // (not arithmetic) removes forbidden scores, so NaN/Inf there cannot leak.
        uint32_t allow = ~0u;
        if (is_tree) {
          int row = (wave + NW * t) * 16 + j;  // `wave` here: the wavefront's first tile
          int node = row < R ? row / G : 0;
          allow = (uint32_t)(anc_lds[node] >> (32 * blk32));
        }
        int left = n_valid - 32 * blk32;
        allow &= left >= 32 ? ~0u : ((1u << (left < 0 ? 0 : left)) - 1u);
        allow >>= 4 * kg;
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
          for (int r = 0; r < 4; ++r)
            sc[u][4 * a + r] = ((allow >> (16 * a + r)) & 1u) ? sc[u][4 * a + r] : HB_NEG_INF;
      }
      // Largest of the lane's own eight scores.  The row's reference exponent stays as it is
      // unless one of the row's scores exceeds it by more than kSlack (then exp2(score -
      // reference) <= 2^kSlack stays far from overflow and nothing needs rescaling); the four
      // lanes that share a row see all of its scores between them, so a per-lane test decides
      // and the common case needs no maximum across lanes.  A row without reference yet (-inf:
      // first block) fails the test in every lane that holds an allowed key.
      float lm = fmaxf(fmaxf(fmaxf(fmaxf(fmaxf(fmaxf(fmaxf(sc[u][0], sc[u][1]), sc[u][2]), sc[u][3]), sc[u][4]), sc[u][5]), sc[u][6]), sc[u][7]);
      lmax[u] = lm;
      need |= !(lm * c1 <= m_run[t] + kSlack);
    }
    // -- all V^T fragments of the block, issued now so that they arrive during the vector work
    //    below (they take over the registers of the K fragments, which are done).  Lane (s, kg)
    //    of a 16-lane group addresses 8 bytes of key 16h + 4kg + s/4 at d = 16dt + 4(s%4); the
    //    transposing read hands lane j the four keys 16h + 4kg + 0..3 at d = 16dt + j, i.e. the
    //    k-slots 4h .. 4h+3 of the lane group in the order the score accumulators have.
    bf16x8 av[8];
    {
      const int vkey = 4 * kg + (j >> 2);                       // + 16h + 32 blk32
      const int vrow = (32 * blk32 + vkey) * 256 + 16 * ((j >> 1) & 1) + 8 * (j & 1);
      const int vx = v_swz(vkey) * 16;                          // XOR on the piece index, in bytes
#pragma unroll
      for (int dt = 0; dt < 8; ++dt) {
        const unsigned char *p0 = lv + vrow + ((32 * dt) ^ vx);
        bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(p0));
        bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(p0 + 16 * 256));
        av[dt] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    // -- rare: a row needs its first reference or has outgrown it.  The reference becomes the
    //    row's maximum over the block and what has been accumulated is rescaled (rows that stay
    //    get alpha = 1).  Uniform branches; the asm statement keeps the outer one a real branch,
    //    otherwise the multiply of the whole accumulator is speculated into every pass.
    if (__any(need)) {
      asm volatile("" ::: "memory");
#pragma unroll
      for (int u = 0; u < kGroup; ++u) {
        const int t = t0 + u;
        if (t >= TPW) break;
        const float mx = group_max(lmax[u]) * c1;  // c1 > 0: scaling commutes with the maximum
        const float m_old = m_run[t];
        const float m_ref = (m_old == HB_NEG_INF) ? mx : m_old;  // nothing accumulated yet: adopt, no rescale
        const bool grow = mx > m_ref + kSlack;
        m_run[t] = grow ? mx : m_ref;
        if (__any(grow)) {
          const float alpha = grow ? fast_exp2(m_ref - mx) : 1.f;
          l_run[t] *= alpha;
#pragma unroll
          for (int dt = 0; dt < 8; ++dt) {
            asm volatile("" : "+v"(o[t][dt]));
            o[t][dt] *= alpha;
            asm volatile("" : "+v"(o[t][dt]));
          }
        }
      }
    }
    // -- probabilities.  Every row has seen at least one allowed key by now (the first key of a
    //    prefix chunk, the root of the tree), so its reference is finite.
    bf16x8 pb[kGroup];
#pragma unroll
    for (int u = 0; u < kGroup; ++u) {
      const int t = t0 + u;
      if (t >= TPW) break;
      f32x8 p;
#pragma unroll
      for (int r = 0; r < 8; ++r) p[r] = fast_exp2(fmaf(sc[u][r], c1, -m_run[t]));
      pb[u] = __builtin_convertvector(p, bf16x8);
    }
    // -- row sums on the matrix cores: an all-ones A operand makes every row of the product the
    //    sum over the block's 32 keys of the (bf16) probabilities, summed across the lane groups
    //    too; eight vector additions per tile and the final cross-lane sum are saved
    {
      const bf16x8 ones = {(__bf16)1.f, (__bf16)1.f, (__bf16)1.f, (__bf16)1.f, (__bf16)1.f, (__bf16)1.f, (__bf16)1.f, (__bf16)1.f};
#pragma unroll
      for (int u = 0; u < kGroup; ++u) {
        const int t = t0 + u;
        if (t >= TPW) break;
        l_run[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pb[u], l_run[t], 0, 0, 0);
        asm volatile("" : "+v"(l_run[t]));
      }
    }
    // -- O^T += V^T P^T for the group, one 16-d slab of V^T at a time
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) {
#pragma unroll
      for (int u = 0; u < kGroup; ++u) {
        const int t = t0 + u;
        if (t >= TPW) break;
        o[t][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[dt], pb[u], o[t][dt], 0, 0, 0);
        asm volatile("" : "+v"(o[t][dt]));
      }
    }
  }
}

// TPW: 16-row tiles per wavefront (1 or 2).  NW: wavefronts per workgroup: 4 (two workgroups per
// CU) or 8 (one per CU, twice the rows sharing each staged tile).  NS: LDS stages of the KV ring.
// The tree tile, which goes through registers, is staged by all threads (NW = 4) or K by
// wavefronts 0-3 and V by wavefronts 4-7 (NW = 8).
template <int TPW, int NW, int NS>
__global__ __launch_bounds__(64 * NW, NW == 4 ? 2 : 1) void attn_mfma_kernel(
    hb_attn_desc d, int splits, int chunk_tokens, int workers, int row_groups, const u32x4 *__restrict__ q, const u32x4 *__restrict__ k_tree,
    const u32x4 *__restrict__ v_tree, const u32x4 *__restrict__ k_pool, const u32x4 *__restrict__ v_pool,
    const int32_t *__restrict__ block_table, const int32_t *__restrict__ prefix_len,
    const int32_t *__restrict__ node_offset, const int32_t *__restrict__ parent, bf16_t *__restrict__ out,
    float *__restrict__ lse, float *__restrict__ part_o, float *__restrict__ part_ml) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  // [NS stages][K tile 16 KiB | V tile 16 KiB] [64 ancestor masks]
  constexpr int kStageBytes = K_PIECES * 16 + V_BYTES;
  unsigned long long *anc_lds = (unsigned long long *)(smem + NS * kStageBytes);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // Consecutive workgroup ids land on different XCDs (id % 8); the row groups of one unit of work
  // get ids 8 apart, i.e. neighbouring slots of the same XCD, so the KV tiles they both read are
  // shared in that XCD's L2.
  const int id = blockIdx.x;
  const int xcd = id & 7, slot = id >> 3;
  const int rgi = slot % row_groups;
  const int unit = (slot / row_groups) * 8 + xcd;
  const int G = d.num_q_heads / d.num_kv_heads;
  const int cap = d.max_blocks_per_seq * PAGE;
  const int j = lane & 15;    // query row within a tile
  const int kg = lane >> 4;   // key group / k-slot group of this lane

  // What this workgroup does is a list of segments (sequence b, prefix tokens [begin, end), with
  // or without the tree tile, partial slot c).
  //  * workers == 0: one segment, chunk c of sequence b, chunks of equal length within a
  //    sequence (unit = (b, g, c)).
  //  * workers > 0 (batch <= 64): work-proportional.  The 64-key tiles of all sequences (tree
  //    tile first, then the prefix tiles) form one line; worker w of kv head g (unit = (w, g))
  //    takes tiles [w * per, (w + 1) * per) of it, per = max(kMinPer, ceil(total / workers)),
  //    whatever sequences they belong to.  Every workgroup finds the line by itself: lane b reads
  //    prefix_len[b], a prefix sum over the lanes gives each sequence's place.  A sequence cut
  //    by worker boundaries gets one partial slot per piece (consecutive workers, consecutive
  //    slots); the piece that ends it announces the unused slots as empty; a sequence that lies
  //    inside one worker's range is written out directly and slot 0 tells the merge so.
  constexpr int kMinPer = NW == 8 ? 16 : 8;
  constexpr int kRestart = 4;
  int g, seg_b = 0, lo = 0, hi = 0, per = 1, w_id = 0, al_k = 0, al_n = 0;
  bool aligned = false;
  int Lb = 0, tb = 0, cum = 0;  // lane b: prefix length, tiles and end of sequence b on the line
  if (workers == 0) {
    if (unit >= d.batch * d.num_kv_heads * splits) return;
    g = (unit / splits) % d.num_kv_heads;
  } else {
    if (unit >= d.num_kv_heads * workers) return;
    g = unit % d.num_kv_heads;
    w_id = unit / d.num_kv_heads;
    if (lane < d.batch) {
      Lb = prefix_len[lane];
      Lb = Lb < 0 ? 0 : (Lb > cap ? cap : Lb);
      tb = (Lb + KT - 1) / KT + 1;
    }
    cum = tb;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int y = __shfl_up(cum, off, 64);
      if (lane >= off) cum += y;
    }
    const int total = __builtin_amdgcn_readfirstlane(__shfl(cum, 63, 64));
    per = (total + workers - 1) / workers;
    per = per < kMinPer ? kMinPer : per;
    // The alternative: the same number of workers for every sequence, each sequence cut into
    // pieces of equal length.  No worker then has to start over on a second sequence (which
    // costs about kRestart tiles' time), but the longest sequence sets the pace.  Both plans
    // are known here; take the one that finishes first.
    al_k = workers / d.batch;
    if (al_k >= 1) {
      int nb = (tb + kMinPer - 1) / kMinPer;
      nb = nb < 1 ? 1 : (nb > al_k ? al_k : nb);
      nb = nb > splits ? splits : nb;
      al_n = nb;                                   // pieces of sequence `lane`
      int len = lane < d.batch ? (tb + nb - 1) / nb : 0;
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) len = max(len, __shfl_xor(len, off, 64));
      aligned = __builtin_amdgcn_readfirstlane(len) <= per + kRestart;
    }
    if (aligned) {
      seg_b = w_id / al_k;
      if (seg_b >= d.batch) return;
    } else {
      lo = w_id * per;
      hi = lo + per < total ? lo + per : total;
      if (lo >= total) return;
      const unsigned long long after = __ballot(cum > lo);  // sequences that end behind lo
      seg_b = after ? __builtin_ctzll(after) : d.batch;
    }
  }

#pragma unroll 1
  for (int seg = 0;; ++seg) {
  int b, c, L, begin, end;
  bool tree_chunk, direct_out, ends_seq;
  if (workers == 0) {
    if (seg > 0) break;
    c = unit % splits;
    b = unit / (splits * d.num_kv_heads);
    L = prefix_len[b];
    L = L < 0 ? 0 : (L > cap ? cap : L);
    // chunks of this sequence: as many as the plan allows, but never shorter than needed
    int n_chunks = (L + chunk_tokens - 1) / chunk_tokens;
    n_chunks = n_chunks < 1 ? 1 : (n_chunks > splits ? splits : n_chunks);
    int chunk = ((L + n_chunks - 1) / n_chunks + KT - 1) / KT * KT;
    chunk = chunk < KT ? KT : chunk;
    begin = c * chunk;
    end = min(L, begin + chunk);
    tree_chunk = (c == 0);
    direct_out = splits == 1;
    ends_seq = false;  // here every chunk, also an empty one, has a workgroup that announces it
  } else if (aligned) {
    if (seg > 0) break;
    b = seg_b;
    const int piece = w_id - b * al_k;
    const int t_b = __builtin_amdgcn_readfirstlane(__shfl(tb, b, 64));
    const int n_b = __builtin_amdgcn_readfirstlane(__shfl(al_n, b, 64));
    L = __builtin_amdgcn_readfirstlane(__shfl(Lb, b, 64));
    if (piece >= n_b) break;
    const int len = (t_b + n_b - 1) / n_b;
    const int rel_lo = piece * len;
    const int rel_hi = min(t_b, rel_lo + len);
    if (rel_lo >= rel_hi && piece > 0) {
      // pieces of equal length can leave the last ones without tiles: announce them as empty
      c = piece;
      begin = end = L;
      tree_chunk = false;
      direct_out = false;
      ends_seq = piece == n_b - 1;
    } else {
      tree_chunk = rel_lo == 0;
      begin = ((rel_lo > 1 ? rel_lo : 1) - 1) * KT;
      end = min(L, (rel_hi - 1) * KT);
      c = piece;
      ends_seq = piece == n_b - 1;
      direct_out = n_b == 1 || splits == 1;
    }
  } else {
    if (seg_b >= d.batch) break;
    b = seg_b++;
    const int t_b = __builtin_amdgcn_readfirstlane(__shfl(tb, b, 64));
    const int e_b = __builtin_amdgcn_readfirstlane(__shfl(cum, b, 64));
    L = __builtin_amdgcn_readfirstlane(__shfl(Lb, b, 64));
    const int s_b = e_b - t_b;                 // the sequence's tiles are [s_b, e_b) of the line
    if (s_b >= hi) break;
    const int rel_lo = (lo > s_b ? lo : s_b) - s_b;
    const int rel_hi = (hi < e_b ? hi : e_b) - s_b;
    tree_chunk = rel_lo == 0;                  // tile 0 of a sequence is its tree tile
    begin = ((rel_lo > 1 ? rel_lo : 1) - 1) * KT;
    end = min(L, (rel_hi - 1) * KT);
    c = w_id - s_b / per;
    ends_seq = e_b <= hi;
    direct_out = (tree_chunk && ends_seq) || splits == 1;
  }
  const int n0 = node_offset[b];
  int n_nodes = node_offset[b + 1] - n0;
  n_nodes = n_nodes < 0 ? 0 : (n_nodes > d.max_nodes_per_tree ? d.max_nodes_per_tree : n_nodes);
  if (n0 < 0 || n0 + n_nodes > d.total_nodes) n_nodes = 0;  // malformed offsets: touch nothing
  const int R = n_nodes * G;           // query rows of this (sequence, kv head)
  const int NT = (R + 15) >> 4;        // 16-row tiles
  const int tiles_per_group = (NT + row_groups - 1) / row_groups;
  const int tile_lo = rgi * tiles_per_group;                     // this workgroup's tiles
  const int tile_hi = min(NT, tile_lo + tiles_per_group);
  const int wtile = tile_lo + wave;    // the wavefront's tiles: wtile + NW*t < tile_hi
  if (tile_lo >= tile_hi) continue;
  if (c >= splits) continue;           // cannot happen with the planned slot count; never write past it

  const size_t row_base = (size_t)n0 * d.num_q_heads + (size_t)g * G;  // + node*Hq + head_in_group

  if (!tree_chunk && begin >= L) {
    // an empty chunk only announces itself to the merge (which stops at the first empty slot)
    for (int r = tile_lo * 16 + tid; r < min(R, tile_hi * 16); r += 64 * NW) {
      size_t rg = row_base + (size_t)(r / G) * d.num_q_heads + (r % G);
      part_ml[(rg * splits + c) * 2 + 0] = HB_NEG_INF;
      part_ml[(rg * splits + c) * 2 + 1] = 0.f;
    }
    continue;
  }

  if (tree_chunk && tid < 64) {
    // Ancestor masks: lane i walks from node i to the root.  The parent array is read once (one
    // value per lane) and the walk fetches parents from the other lanes' registers, so its length
    // costs register exchanges, not a chain of dependent memory loads.
    const int par = tid < n_nodes ? parent[n0 + tid] : -1;
    unsigned long long anc = tid < n_nodes ? 1ull << tid : 0ull;
    int x = tid < n_nodes ? tid : -1;
    for (int guard = 0; guard < 64; ++guard) {
      const int px = __shfl(par, x < 0 ? 0 : x, 64);
      const bool up = x >= 0 && px >= 0 && px < x;  // else: root reached (or malformed parent: stop)
      if (!__any(up)) break;
      if (up) anc |= 1ull << px;
      x = up ? px : -1;
    }
    anc_lds[tid] = anc;
  }

  // ---- Q fragments (B operand of S^T = K Q^T), kept for the whole kernel -------------------
  bf16x8 qf[TPW][4];
#pragma unroll
  for (int t = 0; t < TPW; ++t) {
    int row = (wtile + NW * t) * 16 + j;
    bool ok = row < R && (wtile + NW * t) < tile_hi;
    int node = ok ? row / G : 0;
    int hg = ok ? row - node * G : 0;
    const u32x4 *src = q + (row_base + (size_t)node * d.num_q_heads + hg) * 16;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      u32x4 x = {0u, 0u, 0u, 0u};
      if (ok) x = src[4 * ks + kg];
      qf[t][ks] = __builtin_bit_cast(bf16x8, x);
    }
  }

  // fp32 O^T accumulators, kept in place in vector registers
  f32x4 o[TPW][8];
  float m_run[TPW];
  f32x4 l_run[TPW];  // row sums of the probabilities (every element holds the row's sum)
#pragma unroll
  for (int t = 0; t < TPW; ++t) {
    m_run[t] = HB_NEG_INF;
    l_run[t] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) {
      o[t][dt] = (f32x4){0.f, 0.f, 0.f, 0.f};
      asm volatile("" : "+v"(o[t][dt]));
    }
  }
  const float c1 = d.softmax_scale * kLog2e;

  // ---- KV staging ---------------------------------------------------------------------------
  // Prefix tiles go global -> LDS directly (global_load_lds_dwordx4, no staging registers): one
  // instruction moves 64 lanes x 16 bytes = four consecutive keys x 256 bytes of K or of V into
  // 1 KiB of a stage; the XOR swizzle of the LDS layouts is applied on the source side (the lane
  // that fills physical piece p of a row fetches logical piece p ^ swizzle(row)).  A tile is 16
  // such row groups of K and 16 of V; wavefront w issues groups w, w + NW, ... of both, which all
  // have the same position inside their page, so one offset register each serves.  The page ids
  // of a tile (wave-uniform scalar loads, clamped into the pool so every address is valid) are
  // fetched one tile before they are needed.
  // Tiles are loaded NS - 1 ahead of the one being computed.  Every pipeline step issues one
  // batch of PER loads per wavefront, also past the end (then it re-fetches the last tile into a
  // free stage), so that the wait "all but the newest PER * (NS - 2) loads" always means "the
  // next tile has landed".
  // Slots of a tile at or past `end`: K keeps whatever the (valid) address held, the scores are
  // replaced by a select before anything is computed from them; the V rows are overwritten with
  // zeros once they have landed (0 * V must stay finite).
  constexpr int PER = 32 / NW;
  const int stid = tid & 255;               // thread index inside a staging role (tree tile)
  const bool do_k = NW == 4 || wave < 4;    // tree tile: who stages K, who stages V
  const bool do_v = NW == 4 || wave >= 4;
  const int lrow = lane >> 4;               // key inside a 4-key row group
  const bool whi = wave >= 4;               // eight wavefronts: which pair of the tile's pages
  const int gcls = wave & 3;                // row groups w + NW*i sit at keys 4*gcls .. +3 of their page
  const int pkey = 4 * gcls + lrow;         // key inside the page
  const size_t page_stride = (size_t)d.num_kv_heads * PAGE * 16;  // u32x4 units per page
  const u32x4 *k_lane = k_pool + (size_t)g * PAGE * 16 + pkey * 16 + ((lane & 15) ^ pkey);
  const u32x4 *v_lane = v_pool + (size_t)g * PAGE * 16 + pkey * 16 + ((lane & 15) ^ v_swz(pkey));
  const int last_page = d.max_blocks_per_seq - 1;
  const int n_prefix_tiles = end > begin ? (end - begin + KT - 1) / KT : 0;
  const int tree_off = tree_chunk ? 1 : 0;
  const int n_tiles = n_prefix_tiles + tree_off;
  int pg0 = 0, pg1 = 0, pg2 = 0, pg3 = 0;  // page ids of the batch issued next
#define HB_PAGE(idx_)                                                        \
  ({                                                                         \
    int pg__ = (idx_) < last_page ? (idx_) : last_page;                      \
    pg__ = pg__ < 0 ? 0 : pg__;                                              \
    int blk__ = bt_row[pg__];                                                \
    blk__ = blk__ < 0 ? 0 : (blk__ >= d.num_blocks ? d.num_blocks - 1 : blk__); \
    blk__;                                                                   \
  })
  // prefix tile (clamped to the chunk's last one) that pipeline step k_ loads
#define HB_TILE_OF(k_)                                                       \
  ({                                                                         \
    int pt__ = ((k_) < tree_off ? tree_off : (k_)) - tree_off;               \
    pt__ = pt__ < n_prefix_tiles - 1 ? pt__ : n_prefix_tiles - 1;            \
    pt__ < 0 ? 0 : pt__;                                                     \
  })
#define HB_FETCH_PAGES(k_)                                                  \
  {                                                                         \
    const int p0__ = (begin + HB_TILE_OF(k_) * KT) / PAGE;                  \
    pg0 = HB_PAGE(p0__ + 0);                                                \
    pg1 = HB_PAGE(p0__ + 1);                                                \
    pg2 = HB_PAGE(p0__ + 2);                                                \
    pg3 = HB_PAGE(p0__ + 3);                                                \
  }
  // batch k_: the tile of pipeline step max(k_, tree_off) into stage max(k_, tree_off) % NS
  // (in a tree chunk batch 0 loads the same as batch 1: stage 0 belongs to the tree tile)
#define HB_ISSUE_BATCH(k_)                                                                     \
  {                                                                                            \
    const int t__ = (k_) < tree_off ? tree_off : (k_);                                         \
    unsigned char *st__ = smem + (t__ % NS) * kStageBytes;                                     \
    _Pragma("unroll") for (int i__ = 0; i__ < PER; ++i__) {                                     \
      const int n__ = wave + NW * i__;          /* 0..15: K row group, 16..31: V row group */  \
      /* page (n__ >> 2) & 3 of the tile: i__ & 3 for four wavefronts, else wave / 4 + 2 * (i__ & 1) */ \
      const int pg__ = NW == 4 ? ((i__ & 3) == 0 ? pg0 : ((i__ & 3) == 1 ? pg1 : ((i__ & 3) == 2 ? pg2 : pg3))) \
                               : ((i__ & 1) ? (whi ? pg3 : pg2) : (whi ? pg1 : pg0));                         \
      const u32x4 *src__ = (n__ < 16 ? k_lane : v_lane) + (size_t)pg__ * page_stride;          \
      __builtin_amdgcn_global_load_lds((gptr_t)src__, (lptr_t)(st__ + n__ * 1024), 16, 0, 0); \
    }                                                                                          \
  }
  const int32_t *bt_row = block_table + (size_t)b * d.max_blocks_per_seq;

  // the next tile has landed as far as this wavefront's loads go
  constexpr int kKeep = PER * (NS - 2);
  constexpr int kWaitImm = (kKeep & 15) | ((kKeep >> 4) << 14) | (7 << 4) | (15 << 8);  // vmcnt only
#define HB_NEXT_LANDED() __builtin_amdgcn_s_waitcnt(kWaitImm)

  TileSrc src;
  src.k_tree = k_tree; src.v_tree = v_tree; src.k_pool = k_pool; src.v_pool = v_pool;
  src.bt = bt_row;
  src.g = g; src.n0 = n0; src.n_nodes = n_nodes; src.hkv = d.num_kv_heads; src.num_blocks = d.num_blocks;

  // prologue: the tree tile (keys = node ids, read straight from k_tree / v_tree, non-finite V
  // zeroed) goes through registers into stage 0; batches 0 .. NS-2 are issued behind its loads
  u32x4 tk0, tk1, tk2, tk3, tv0, tv1, tv2, tv3;
  if (tree_chunk) {
    if (do_k) {
      tk0 = load_k_piece(src, true, 0, 0, stid, 0);
      tk1 = load_k_piece(src, true, 0, 0, stid, 1);
      tk2 = load_k_piece(src, true, 0, 0, stid, 2);
      tk3 = load_k_piece(src, true, 0, 0, stid, 3);
    }
    if (do_v) {
      tv0 = load_v_piece(src, true, 0, 0, stid, 0);
      tv1 = load_v_piece(src, true, 0, 0, stid, 1);
      tv2 = load_v_piece(src, true, 0, 0, stid, 2);
      tv3 = load_v_piece(src, true, 0, 0, stid, 3);
    }
  }
  HB_FETCH_PAGES(0);
#pragma unroll
  for (int k = 0; k < NS - 1; ++k) {
    HB_ISSUE_BATCH(k);
    HB_FETCH_PAGES(k + 1);
  }
  if (tree_chunk) {
    if (do_k) store_k((u32x4 *)smem, stid, tk0, tk1, tk2, tk3);
    if (do_v) store_v((u32x4 *)(smem + K_PIECES * 16), stid, tv0, tv1, tv2, tv3);
  }
  // V rows past the end of the tile pipeline step t_ holds, zeroed by the wavefront that loaded
  // them (uniform condition; only a chunk's last prefix tile can be short)
#define HB_ZERO_V_TAIL(t_)                                                                     \
  {                                                                                            \
    const int pt__ = (t_) - tree_off;                                                          \
    const int nv__ = end - (begin + pt__ * KT);                                                \
    if (pt__ >= 0 && pt__ == n_prefix_tiles - 1 && nv__ < KT) {                                \
      unsigned char *st__ = smem + ((t_) % NS) * kStageBytes;                                  \
      _Pragma("unroll") for (int i__ = 0; i__ < PER; ++i__) {                                   \
        const int n__ = wave + NW * i__;                                                       \
        if (n__ >= 16 && 4 * (n__ - 16) + lrow >= nv__)                                        \
          *(u32x4 *)(st__ + n__ * 1024 + lane * 16) = (u32x4){0u, 0u, 0u, 0u};                 \
      }                                                                                        \
      __builtin_amdgcn_s_waitcnt(0xC07F); /* lgkmcnt(0): the zeros are in LDS */               \
    }                                                                                          \
  }
  // Workgroup barrier without the memory fence of __syncthreads(), which would wait for every
  // load in flight; LDS reads of the finished tile have all been consumed by MFMAs, and what
  // must be visible behind the barrier has been waited for explicitly.
#define HB_BARRIER() asm volatile("s_barrier" ::: "memory")
  // tile 0 is ready: everything but the newest NS - 2 batches has landed
  HB_NEXT_LANDED();
  HB_ZERO_V_TAIL(0);
  __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): the tree tile's LDS writes
  HB_BARRIER();

#pragma unroll 1  // also keeps the compiler from peeling the tree tile's iteration into a second copy
  for (int i = 0; i < n_tiles; ++i) {
    const bool is_tree = tree_chunk && i == 0;
    const int tile_start = begin + (i - tree_off) * KT;                 // prefix position of key 0
    const int n_valid = is_tree ? n_nodes : min(KT, end - tile_start);  // keys of this tile that exist
    const unsigned char *stage = smem + (i % NS) * kStageBytes;
    const u32x4 *lk = (const u32x4 *)stage;
    const unsigned char *lv = stage + K_PIECES * 16;
    const bool partial = is_tree || n_valid < KT;  // uniform

    // the stage of tile i - 1 is free (barrier below): fill it with tile i + NS - 1
    HB_ISSUE_BATCH(i + NS - 1);
    HB_FETCH_PAGES(i + NS);  // for the batch of the next iteration

#pragma unroll 1
    for (int blk32 = 0; blk32 < 2; ++blk32) {
      if (32 * blk32 < n_valid)
        attend_block<TPW, NW>(partial, lk, lv, blk32, j, kg, qf, o, m_run, l_run, c1, n_valid, is_tree, anc_lds, wtile,
                              R, G);
    }
    HB_NEXT_LANDED();
    HB_ZERO_V_TAIL(i + 1);
    HB_BARRIER();
  }
  // loads past the end are still in flight: let them land before the workgroup gives up its LDS
  __builtin_amdgcn_s_waitcnt((0 & 15) | (7 << 4) | (15 << 8));
#undef HB_PAGE
#undef HB_TILE_OF
#undef HB_FETCH_PAGES
#undef HB_ISSUE_BATCH
#undef HB_NEXT_LANDED
#undef HB_ZERO_V_TAIL
#undef HB_BARRIER

  // ---- write out: lane (j, kg) holds O[row j][16*dt + 4*kg + r] ---------------------------
#pragma unroll
  for (int t = 0; t < TPW; ++t) {
    int row = (wtile + NW * t) * 16 + j;
    if ((wtile + NW * t) >= tile_hi) continue;
    float l_tot = l_run[t][0];
    if (row >= R) continue;
    int node = row / G, hg = row - node * G;
    size_t rg = row_base + (size_t)node * d.num_q_heads + hg;
    if (direct_out) {
      float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
#pragma unroll
      for (int dt = 0; dt < 8; ++dt) {
        f32x4 v = o[t][dt];
        u32x2 w;
        w[0] = (uint32_t)f32_to_bf16(v[0] * inv) | ((uint32_t)f32_to_bf16(v[1] * inv) << 16);
        w[1] = (uint32_t)f32_to_bf16(v[2] * inv) | ((uint32_t)f32_to_bf16(v[3] * inv) << 16);
        *(u32x2 *)(out + rg * D + 16 * dt + 4 * kg) = w;
      }
      if (lse && kg == 0) lse[rg] = (m_run[t] + log2f(l_tot)) * kLn2;
      if (splits > 1 && kg == 0) {  // tell the merge that this row is final
        part_ml[(rg * splits) * 2 + 0] = 0.f;
        part_ml[(rg * splits) * 2 + 1] = -1.f;
      }
    } else {
      float *po = part_o + (rg * splits + c) * D;
#pragma unroll
      for (int dt = 0; dt < 8; ++dt) *(f32x4 *)(po + 16 * dt + 4 * kg) = o[t][dt];
      if (kg == 0) {
        part_ml[(rg * splits + c) * 2 + 0] = m_run[t] * kLn2;  // natural-log units for the merge
        part_ml[(rg * splits + c) * 2 + 1] = l_tot;
        if (ends_seq && c + 1 < splits) {  // the first empty slot ends the list for the merge
          part_ml[(rg * splits + c + 1) * 2 + 0] = HB_NEG_INF;
          part_ml[(rg * splits + c + 1) * 2 + 1] = 0.f;
        }
      }
    }
  }
  // the next segment reuses the LDS stages and the ancestor masks
  asm volatile("s_barrier" ::: "memory");
  }  // segments
}


template <int TPW, int NW, int NS>
hipError_t launch(int row_groups, const hb_attn_desc &d, const AttnPlan &plan, const void *q, const void *k_tree,
                  const void *v_tree, const void *k_pool, const void *v_pool, const int32_t *block_table,
                  const int32_t *prefix_len, const int32_t *node_offset, const int32_t *parent, void *out,
                  float *lse, float *part_o, float *part_ml, hipStream_t s) {
  const int items = plan.workers > 0 ? d.num_kv_heads * plan.workers : d.batch * d.num_kv_heads * plan.splits;
  dim3 grid((unsigned)((items + 7) / 8 * 8 * row_groups));
  constexpr size_t kLdsBytes = (size_t)NS * (K_PIECES * 16 + V_BYTES) + 64 * 8;
  auto kern = attn_mfma_kernel<TPW, NW, NS>;
  hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes);
  if (e != hipSuccess) return e;
  kern<<<grid, 64 * NW, kLdsBytes, s>>>(d, plan.splits, plan.chunk_tokens, plan.workers, row_groups, (const u32x4 *)q, (const u32x4 *)k_tree,
                                    (const u32x4 *)v_tree, (const u32x4 *)k_pool, (const u32x4 *)v_pool,
                                    block_table, prefix_len, node_offset, parent, (bf16_t *)out, lse, part_o,
                                    part_ml);
  return hipGetLastError();
}

}  // namespace

bool attn_mfma_supports(const hb_attn_desc &d) {
  if (d.dtype != HB_BF16 || d.head_dim != D || d.page_size != PAGE) return false;
  if (d.num_kv_heads <= 0 || d.num_q_heads % d.num_kv_heads) return false;
  int rows = (d.num_q_heads / d.num_kv_heads) * d.max_nodes_per_tree;
  if (d.max_nodes_per_tree > 64 || rows > 512) return false;  // at most 2 row groups of 16 tiles
  if (!(d.softmax_scale > 0.f) || !(d.softmax_scale < 1e30f)) return false;  // base-2 max tracking needs scale > 0
  if (d.batch > 65535 || d.num_kv_heads > 65535) return false;
  return true;
}

// Workgroup shape.  Up to eight 16-row tiles: four wavefronts (one or two tiles each), two
// workgroups per CU.  More: eight wavefronts with two tiles each (256 rows share every staged KV
// tile, which halves the staging work and the L2 -> LDS traffic per row), one workgroup per CU,
// and as many row groups as that takes; the row groups of one (sequence, kv head, chunk) stream
// the same KV and share it through their XCD's L2.
static int tiles_of(const hb_attn_desc &d) {
  int rows = (d.num_q_heads / d.num_kv_heads) * d.max_nodes_per_tree;
  return (rows + 15) / 16;
}

int32_t attn_mfma_waves(const hb_attn_desc &d) { return tiles_of(d) > 8 ? 8 : 4; }

int32_t attn_mfma_row_groups(const hb_attn_desc &d) {
  int tiles = tiles_of(d);
  return tiles > 8 ? (tiles + 15) / 16 : 1;
}

hipError_t launch_attn_mfma(const hb_attn_desc &d, const AttnPlan &plan, const void *q, const void *k_tree,
                            const void *v_tree, const void *k_pool, const void *v_pool,
                            const int32_t *block_table, const int32_t *prefix_len,
                            const int32_t *node_offset, const int32_t *parent, void *out, float *lse,
                            float *part_o, float *part_ml, hipStream_t s) {
  const int tiles = tiles_of(d);
  const int row_groups = plan.row_groups;
#define HB_GO(N, W) \
  return launch<N, W, (W == 8 ? 4 : 2)>(row_groups, d, plan, q, k_tree, v_tree, k_pool, v_pool, block_table, prefix_len, node_offset, parent, out, lse, part_o, part_ml, s)
  if (tiles <= 4) HB_GO(1, 4);
  if (tiles <= 8) HB_GO(2, 4);
  HB_GO(2, 8);  // attn_mfma_row_groups keeps a workgroup at sixteen tiles or fewer
#undef HB_GO
}

}  // namespace hb
