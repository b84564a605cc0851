// Construction of the draft token tree from the draft model's outputs (the step before the
// verification; the paper drafts in the EAGLE-3 manner, Section 3.1, and leaves the arrangement of
// the drafted tokens open: this is the dynamic tree of that line of work).
//
//   topk_logprob   per row of draft logits: the k best tokens (ties: lower id) and their
//                  log-probabilities.  Pass 1, one workgroup per (row, chunk of the vocabulary):
//                  the chunk is read from memory once, reduced to its maximum and its sum of
//                  exponentials, and its k best entries are picked as order-preserving integer
//                  keys.  Pass 2, one workgroup per row: the k best of the chunks' winners and
//                  the row's logsumexp from the chunks' partials.
//   tree_grow      one level: scores of the new candidates (ONE float32 addition each,
//                  parent's score + log-probability), the K best of them become the frontier.
//   tree_finalize  re-ranking of all candidates, the N - 1 best are kept and numbered in
//                  candidate order (parents first); parent, token, depth, ancestor mask per node.
// Ranking is by counting: rank(c) = number of candidates that beat c, where a beats c iff its
// score is higher, or equal with a lower candidate index: a strict total order, so the ranks are
// a permutation and every output slot is written exactly once.
#include "hb_internal.h"

namespace hb {

namespace {

constexpr int kThreads = 256;
constexpr int kMaxTopK = 32;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ unsigned long long wg_max_key(unsigned long long x, unsigned long long *red) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const unsigned long long y = __shfl_xor(x, off, 64);
    x = y > x ? y : x;
  }
  __syncthreads();  // red may still be read from the previous call
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
  __syncthreads();
  unsigned long long r = red[0];
#pragma unroll
  for (int w = 1; w < kThreads / 64; ++w) r = red[w] > r ? red[w] : r;
  return r;
}

__device__ __forceinline__ float wg_max_f(float x, float *red) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x = fmaxf(x, __shfl_xor(x, off, 64));
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
  __syncthreads();
  return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

__device__ __forceinline__ float wg_sum_f(float x, float *red) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}

// key of (value, index): larger value first, then lower index; -0 counts as +0
__device__ __forceinline__ unsigned long long sel_key(float v, uint32_t idx) { return argmax_key(v + 0.f, idx); }

// The k largest of the distinct keys[0 .. cnt) into win[0 .. k), largest first, by counting: the
// rank of a key is the number of keys above it.  Slots without a key (cnt < k) are 0.  The caller
// has made keys[] visible; win[] is visible to every thread on return.
__device__ __forceinline__ void rank_select(const unsigned long long *keys, int cnt, int k, unsigned long long *win) {
  if (threadIdx.x < k) win[threadIdx.x] = 0ull;
  __syncthreads();
  for (int i = threadIdx.x; i < cnt; i += kThreads) {
    const unsigned long long mine = keys[i];
    int rank = 0;
#pragma unroll 8
    for (int j = 0; j < cnt; ++j) rank += keys[j] > mine ? 1 : 0;
    if (rank < k) win[rank] = mine;
  }
  __syncthreads();
}

struct Partial {  // one per (row, chunk), followed in memory by k keys
  float max, sum;
};

constexpr int kChunkMax = 16384;            // logits per chunk: 64 per thread, held in registers
constexpr int kPerThread = kChunkMax / kThreads;
constexpr int kListCap = 2048;              // candidates that pass the threshold

// Position inside the chunk of a thread's j-th value, or n when the thread has no such value.
// Vector layout (rows whose chunk starts 16-byte aligned; loads of PER values, consecutive lanes
// consecutive loads): value e of load q sits at (q * 256 + tid) * PER + e while that load lies
// inside the n_full full vectors of the chunk; value kPerThread is the thread's share of the up
// to PER - 1 values behind them.  Scalar layout: value j sits at j * 256 + tid.
template <int PER>
__device__ __forceinline__ int pos_of(bool vec, int j, int n, int n_full) {
  const int tid = (int)threadIdx.x;
  if (!vec) return j < kPerThread ? min(n, j * kThreads + tid) : n;
  if (j == kPerThread) return min(n, n_full * PER + tid);
  return (j / PER) * kThreads + tid < n_full ? ((j / PER) * kThreads + tid) * PER + (j % PER) : n;
}

// Pass 1 of the top-k: one workgroup per (chunk, row).  The chunk goes from memory straight into
// registers (every load is in flight before the first value is used).  The k best entries are
// found without sorting: a threshold T that at least k values of the chunk reach (from the
// per-thread maxima, see below) is a lower bound of the chunk's k-th largest value, so only values
// >= T can be among the k best; those few are collected in LDS (as order-preserving keys) and
// the k best picked there by counting ranks.
// Many equal values can let more pass than the list holds; then k rounds of a workgroup-wide
// maximum run over the registers instead (same result, slower).
template <typename T>
__global__ __launch_bounds__(kThreads) void topk_chunk_kernel(int V, int k, int chunk, int n_chunks,
                                                              const T *__restrict__ logits,
                                                              unsigned char *__restrict__ work) {
  __shared__ unsigned long long red[kThreads / 64];
  __shared__ float fred[kThreads / 64];
  __shared__ unsigned long long win[kMaxTopK];
  __shared__ unsigned long long list[kListCap];
  __shared__ int list_n;
  __shared__ float thr_w[kThreads / 64];
  constexpr int PER = 16 / (int)sizeof(T);
  const int c = blockIdx.x, m = blockIdx.y;
  const int tid = threadIdx.x;
  const int v0 = c * chunk;
  const int n = min(chunk, V - v0);
  const T *row = logits + (size_t)m * V + v0;
  const int n_full = n / PER;
  const bool vec = (((size_t)row) & 15) == 0 && n_full > 0;
  const float ninf = -__builtin_huge_valf();
  // every load is unconditional (addresses clamped into the chunk) so that all of them are in
  // flight together; what a thread does not own is replaced by -inf afterwards
  float x[kPerThread + 1];
  if (vec) {
    u32x4 w[kPerThread / PER];
#pragma unroll
    for (int q = 0; q < kPerThread / PER; ++q) w[q] = ((const u32x4 *)row)[min(q * kThreads + tid, n_full - 1)];
    const float tail = load_f32<T>(row + min(n_full * PER + tid, n - 1));
#pragma unroll
    for (int q = 0; q < kPerThread / PER; ++q) {
      const bool own = q * kThreads + tid < n_full;
#pragma unroll
      for (int e = 0; e < PER; ++e) {
        float f;
        if (sizeof(T) == 4) f = __uint_as_float(w[q][e]);
        else f = __uint_as_float((e & 1) ? (w[q][e >> 1] & 0xffff0000u) : (w[q][e >> 1] << 16));
        x[q * PER + e] = (own && f == f) ? f : ninf;
      }
    }
    x[kPerThread] = (n_full * PER + tid < n && tail == tail) ? tail : ninf;
  } else {
#pragma unroll
    for (int j = 0; j < kPerThread; ++j) {
      const int p = j * kThreads + tid;
      const float f = load_f32<T>(row + min(p, n - 1));
      x[j] = (p < n && f == f) ? f : ninf;
    }
    x[kPerThread] = ninf;
  }
  if (tid == 0) list_n = 0;
  float mt = ninf;
#pragma unroll
  for (int j = 0; j <= kPerThread; ++j) mt = fmaxf(mt, x[j]);
  const float mx = wg_max_f(mt, fred);
  // Threshold T with at least k values >= T in the chunk: every wavefront takes the k-th largest
  // of its 64 lane maxima (a lane counts the maxima strictly above its own, lane by lane through
  // readlane; the smallest maximum with fewer than k above it is the k-th largest), which k of its
  // own values reach; T is the largest of the wavefronts' thresholds.  A wavefront with fewer
  // than k lanes holding values sets no threshold; if none does, everything passes.
  const bool has = pos_of<PER>(vec, 0, n, n_full) < n || pos_of<PER>(vec, kPerThread, n, n_full) < n;
  int above = 0;
#pragma unroll
  for (int l = 0; l < 64; ++l) {
    const float other = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(mt), l));
    above += other > mt ? 1 : 0;
  }
  const int holders = __popcll(__ballot(has));
  float tw = (has && above < k) ? mt : __builtin_huge_valf();
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) tw = fminf(tw, __shfl_xor(tw, off, 64));
  if (holders < k) tw = ninf;
  if ((tid & 63) == 0) thr_w[tid >> 6] = tw;
  __syncthreads();
  const float thr = fmaxf(fmaxf(thr_w[0], thr_w[1]), fmaxf(thr_w[2], thr_w[3]));
  float sum = 0.f;
  if (thr > ninf) {
    // the common case: values the thread does not own are -inf, fail the test and add exp(-inf) = 0
    const float c1 = 1.4426950408889634f, c0 = -mx * 1.4426950408889634f;
#pragma unroll
    for (int j = 0; j <= kPerThread; ++j) {
      sum += __builtin_amdgcn_exp2f(fmaf(x[j], c1, c0));
      if (x[j] >= thr) {
        const int at = atomicAdd(&list_n, 1);
        if (at < kListCap) list[at] = sel_key(x[j], (uint32_t)(v0 + pos_of<PER>(vec, j, n, n_full)));
      }
    }
  } else {
    const bool any = mx > ninf;
#pragma unroll
    for (int j = 0; j <= kPerThread; ++j) {
      const int p = pos_of<PER>(vec, j, n, n_full);
      if (any) sum += __expf(x[j] - mx);
      if (p < n) {
        const int at = atomicAdd(&list_n, 1);
        if (at < kListCap) list[at] = sel_key(x[j], (uint32_t)(v0 + p));
      }
    }
  }
  sum = wg_sum_f(sum, fred);  // its barriers also publish list and list_n
  const int cnt = list_n;
  if (cnt <= kListCap) {
    rank_select(list, cnt, k, win);
  } else {
    unsigned long long last = ~0ull;
    for (int r = 0; r < k; ++r) {
      unsigned long long best = 0ull;
#pragma unroll
      for (int j = 0; j <= kPerThread; ++j) {
        const int p = pos_of<PER>(vec, j, n, n_full);
        const unsigned long long key = p < n ? sel_key(x[j], (uint32_t)(v0 + p)) : 0ull;
        best = (key < last && key > best) ? key : best;
      }
      best = wg_max_key(best, red);
      if (tid == 0) win[r] = best;
      last = best;
    }
  }
  __syncthreads();
  unsigned char *slot = work + ((size_t)m * n_chunks + c) * (sizeof(Partial) + (size_t)k * 8);
  if (tid == 0) {
    Partial p;
    p.max = mx;
    p.sum = sum;
    *(Partial *)slot = p;
  }
  if (tid < k) ((unsigned long long *)(slot + sizeof(Partial)))[tid] = win[tid];
}

__global__ __launch_bounds__(kThreads) void topk_merge_kernel(int V, int k, int n_chunks,
                                                              const unsigned char *__restrict__ work,
                                                              int32_t *__restrict__ out_ids,
                                                              float *__restrict__ out_logp) {
  __shared__ unsigned long long red[kThreads / 64];
  __shared__ float fred[kThreads / 64];
  __shared__ unsigned long long win[kMaxTopK];
  __shared__ unsigned long long list[kListCap];
  const int m = blockIdx.x;
  const size_t stride = sizeof(Partial) + (size_t)k * 8;
  const unsigned char *base = work + (size_t)m * n_chunks * stride;
  float mx = -__builtin_huge_valf();
  for (int c = threadIdx.x; c < n_chunks; c += kThreads) mx = fmaxf(mx, ((const Partial *)(base + c * stride))->max);
  mx = wg_max_f(mx, fred);
  float sum = 0.f;
  for (int c = threadIdx.x; c < n_chunks; c += kThreads) {
    const Partial p = *(const Partial *)(base + c * stride);
    if (p.max > -__builtin_huge_valf()) sum += p.sum * __expf(p.max - mx);
  }
  sum = wg_sum_f(sum, fred);
  const float lse = mx + __logf(sum);
  // the chunks' winners are keys already
  const int n = n_chunks * k;
  if (n <= kListCap) {
    for (int i = threadIdx.x; i < n; i += kThreads)
      list[i] = ((const unsigned long long *)(base + (i / k) * stride + sizeof(Partial)))[i % k];
    __syncthreads();
    rank_select(list, n, k, win);
  } else {  // k rounds of the maximum below the last one
    unsigned long long last = ~0ull;
    for (int r = 0; r < k; ++r) {
      unsigned long long best = 0ull;
      for (int i = threadIdx.x; i < n; i += kThreads) {
        const unsigned long long key = ((const unsigned long long *)(base + (i / k) * stride + sizeof(Partial)))[i % k];
        best = (key < last && key > best) ? key : best;
      }
      best = wg_max_key(best, red);
      if (threadIdx.x == 0) win[r] = best;
      last = best;
    }
    __syncthreads();
  }
  if (threadIdx.x < k) {
    const unsigned long long key = win[threadIdx.x];
    const bool ok = key != 0ull;
    out_ids[(size_t)m * k + threadIdx.x] = ok ? (int32_t)argmax_key_index(key) : -1;
    out_logp[(size_t)m * k + threadIdx.x] = ok ? fminf(argmax_key_value(key) - lse, 0.f) : -__builtin_huge_valf();
  }
}

// score order: a beats b iff higher score, or equal score and lower index (no NaN in s[])
__device__ __forceinline__ bool beats(float sa, int a, float sb, int b) { return sa > sb || (sa == sb && a < b); }

__global__ __launch_bounds__(kThreads) void tree_grow_kernel(int K, int level, int C,
                                                             const int32_t *__restrict__ child_ids,
                                                             const float *__restrict__ child_logp,
                                                             float *__restrict__ cand_score,
                                                             int32_t *__restrict__ cand_token,
                                                             int32_t *__restrict__ cand_parent,
                                                             int32_t *__restrict__ frontier,
                                                             int32_t *__restrict__ frontier_slot) {
  __shared__ float s_new[kMaxTopK * kMaxTopK];
  const int b = blockIdx.x;
  const int F = level == 0 ? 1 : K;
  const int n_new = F * K;
  const int first = level == 0 ? 0 : K + (level - 1) * K * K;
  for (int t = threadIdx.x; t < n_new; t += kThreads) {
    const int f = t / K;
    int par = level == 0 ? -1 : frontier[(size_t)b * K + f];
    par = par < -1 ? -1 : (par >= first ? first - 1 : par);  // stay inside the pool whatever the caller left there
    const float base = par < 0 ? 0.f : cand_score[(size_t)b * C + par];
    float s = base + child_logp[((size_t)b * F) * K + t];
    if (!(s == s)) s = -__builtin_huge_valf();
    s_new[t] = s;
    cand_score[(size_t)b * C + first + t] = s;
    cand_token[(size_t)b * C + first + t] = child_ids[((size_t)b * F) * K + t];
    cand_parent[(size_t)b * C + first + t] = par;
  }
  __syncthreads();  // all reads of the old frontier are done
  for (int t = threadIdx.x; t < n_new; t += kThreads) {
    int rank = t;
    if (level > 0) {
      const float s = s_new[t];
      rank = 0;
#pragma unroll 8
      for (int u = 0; u < n_new; ++u) rank += beats(s_new[u], u, s, t) ? 1 : 0;
    }
    if (rank < K) {
      frontier[(size_t)b * K + rank] = first + t;
      frontier_slot[(size_t)b * K + rank] = t / K;
    }
  }
}

constexpr int kFinalThreads = 1024;  // one workgroup per sequence: sixteen wavefronts share the C^2 / 2 comparisons

__global__ __launch_bounds__(kFinalThreads) void tree_finalize_kernel(
    int B, int C, int n, const float *__restrict__ cand_score, const int32_t *__restrict__ cand_token,
    const int32_t *__restrict__ cand_parent, const int32_t *__restrict__ root_token, int32_t *__restrict__ node_offset,
    int32_t *__restrict__ parent, int32_t *__restrict__ draft_ids, int32_t *__restrict__ depth,
    unsigned long long *__restrict__ anc, int32_t *__restrict__ node_cand, float *__restrict__ node_score) {
  extern __shared__ unsigned char dyn[];
  float *s = (float *)dyn;                 // C scores
  int16_t *node_of = (int16_t *)(s + C);   // C: node index of a kept candidate, 0 otherwise
  unsigned char *kept = (unsigned char *)(node_of + C);  // C: the candidate is among the n - 1 best
  __shared__ int wave_kept[kFinalThreads / 64];
  __shared__ int spar[64];
  const int b = blockIdx.x, tid = threadIdx.x;
  const int keep = n - 1;
  for (int c = tid; c < C; c += kFinalThreads) {
    float x = cand_score[(size_t)b * C + c];
    s[c] = (x == x) ? x : -__builtin_huge_valf();
  }
  __syncthreads();
  // ranks: four neighbouring lanes share a candidate, each counts a quarter of the others
  const int sub = tid & 3;
  constexpr int kPerPass = kFinalThreads / 4;
  const int c_end = (C + kPerPass - 1) / kPerPass * kPerPass;  // the same trip count for every lane
  for (int c = tid >> 2; c < c_end; c += kPerPass) {
    const bool live = c < C;
    const float sc = live ? s[c] : 0.f;
    int rank = 0;
    if (live) {
#pragma unroll 8
      for (int u = sub; u < C; u += 4) rank += beats(s[u], u, sc, c) ? 1 : 0;
    }
    rank += __shfl_xor(rank, 1, 64);
    rank += __shfl_xor(rank, 2, 64);
    if (live && sub == 0) kept[c] = rank < keep ? 1 : 0;
  }
  __syncthreads();
  // each thread owns a contiguous run of candidates, so that kept candidates are counted in order
  const int per = (C + kFinalThreads - 1) / kFinalThreads;
  const int c0 = min(C, tid * per), c1 = min(C, c0 + per);
  int cnt = 0;
  for (int c = c0; c < c1; ++c) cnt += kept[c];
  // exclusive prefix count over the threads: inside the wavefront by shifts, then the wavefronts before
  int incl = cnt;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int y = __shfl_up(incl, off, 64);
    if ((tid & 63) >= off) incl += y;
  }
  if ((tid & 63) == 63) wave_kept[tid >> 6] = incl;
  __syncthreads();
  int before = incl - cnt;
  for (int w = 0; w < (tid >> 6); ++w) before += wave_kept[w];
  for (int c = c0; c < c1; ++c) {
    const bool k = kept[c] != 0;
    node_of[c] = k ? (int16_t)(1 + before) : (int16_t)0;
    before += k ? 1 : 0;
  }
  __syncthreads();
  const size_t o = (size_t)b * n;
  for (int c = c0; c < c1; ++c) {
    const int i = node_of[c];
    if (i == 0) continue;
    int pc = cand_parent[(size_t)b * C + c];
    pc = pc < 0 ? -1 : (pc >= c ? -1 : pc);  // a parent comes before its children, else: the root
    const int p = pc < 0 ? 0 : node_of[pc];  // a dropped parent (malformed scores) also maps to the root
    spar[i] = p;
    parent[o + i] = p;
    draft_ids[o + i] = cand_token[(size_t)b * C + c];
    node_cand[o + i] = c;
    node_score[o + i] = s[c];
  }
  if (tid == 0) {
    spar[0] = -1;
    parent[o] = -1;
    draft_ids[o] = root_token[b];
    node_cand[o] = -1;
    node_score[o] = 0.f;
    node_offset[b] = b * n;
    if (b == B - 1) node_offset[B] = B * n;
  }
  __syncthreads();
  if (tid < n) {
    unsigned long long a = 1ull << tid;
    int d = 0, x = tid;
    for (int guard = 0; guard < 64; ++guard) {
      const int p = spar[x];
      if (p < 0 || p >= x) break;
      a |= 1ull << p;
      ++d;
      x = p;
    }
    depth[o + tid] = d;
    anc[o + tid] = a;
  }
}

}  // namespace

int32_t topk_chunk_elems(int32_t M, int32_t V) {
  // at least about four workgroups per CU in pass 1, chunks of 2048 .. 16384 logits
  int64_t want = (1024 + M - 1) / (M > 0 ? M : 1);
  if (want < 1) want = 1;
  int64_t chunk = ((int64_t)V + want - 1) / want;
  chunk = (chunk + 1023) / 1024 * 1024;  // 16-byte alignment of a chunk's start follows the row's
  if (chunk < 2048) chunk = 2048;
  if (chunk > 16384) chunk = 16384;
  return (int32_t)chunk;
}

size_t topk_workspace_bytes(int32_t M, int32_t V, int32_t k) {
  const int chunk = topk_chunk_elems(M, V);
  const size_t n_chunks = ((size_t)V + chunk - 1) / chunk;
  return (size_t)M * n_chunks * (sizeof(Partial) + (size_t)k * 8);
}

hipError_t launch_topk_logprob(int32_t dtype, int32_t M, int32_t V, int32_t k, const void *logits, int32_t *out_ids,
                               float *out_logp, void *work, hipStream_t s) {
  const int chunk = topk_chunk_elems(M, V);
  const int n_chunks = (V + chunk - 1) / chunk;
  dim3 grid((unsigned)n_chunks, (unsigned)M);
  if (dtype == HB_BF16)
    topk_chunk_kernel<bf16_t><<<grid, kThreads, 0, s>>>(V, k, chunk, n_chunks, (const bf16_t *)logits,
                                                        (unsigned char *)work);
  else
    topk_chunk_kernel<float><<<grid, kThreads, 0, s>>>(V, k, chunk, n_chunks, (const float *)logits,
                                                       (unsigned char *)work);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  topk_merge_kernel<<<M, kThreads, 0, s>>>(V, k, n_chunks, (const unsigned char *)work, out_ids, out_logp);
  return hipGetLastError();
}

hipError_t launch_tree_grow(int32_t B, int32_t K, int32_t level, int32_t C, const int32_t *child_ids,
                            const float *child_logp, float *cand_score, int32_t *cand_token, int32_t *cand_parent,
                            int32_t *frontier, int32_t *frontier_slot, hipStream_t s) {
  tree_grow_kernel<<<B, kThreads, 0, s>>>(K, level, C, child_ids, child_logp, cand_score, cand_token, cand_parent,
                                          frontier, frontier_slot);
  return hipGetLastError();
}

hipError_t launch_tree_finalize(int32_t B, int32_t C, int32_t n, const float *cand_score, const int32_t *cand_token,
                                const int32_t *cand_parent, const int32_t *root_token, int32_t *node_offset,
                                int32_t *parent, int32_t *draft_ids, int32_t *depth, unsigned long long *anc,
                                int32_t *node_cand, float *node_score, hipStream_t s) {
  const size_t lds = (size_t)C * (sizeof(float) + sizeof(int16_t) + 1) + 16;
  tree_finalize_kernel<<<B, kFinalThreads, lds, s>>>(B, C, n, cand_score, cand_token, cand_parent, root_token, node_offset,
                                                parent, draft_ids, depth, anc, node_cand, node_score);
  return hipGetLastError();
}

}  // namespace hb
