// Sampling acceptance of a verified draft tree (speculative sampling with several candidates
// per position), in exact fixed-point integers so that every decision is reproducible.
//
// One workgroup per sequence walks the tree from the root.  At a node, the children are tried in
// index order: child with token x is accepted iff  u * q_x * S(p) < 2^32 * p_x * S(q)  (p, q:
// fix(.) = floor(. * 2^30) of the target's / the draft's distribution after the node, S = sum);
// a rejection replaces p by the residual  r_v = max(p_v S(q) - q_v S(p), 0)  rescaled to 2^30
// (r_v / max(S(r) >> 30, 1), kept in the caller's workspace) and removes x from q.  When no child
// is accepted the step's last token is the smallest v with p_0 + .. + p_v > (u_bonus S(p)) >> 32.
// Sums are integer sums, so they do not depend on the order in which the lanes add them up.
//
// Rejected tokens need no mask over q in the vocabulary passes: after its rejection round a token
// has p_x = 0 (rejection means q_x S(p) > p_x S(q)), so its residual is 0 whatever q_x is; only
// S(q) and the single look-ups of q_x honour the removals.
#include "hb_internal.h"

namespace hb {

namespace {

constexpr int kThreads = 256;
constexpr int kFixBits = 30;

__device__ __forceinline__ uint32_t fix_prob(float p) {
  if (!(p > 0.f)) return 0u;            // negative, zero, NaN
  if (p >= 2.f) return 0x7fffffffu;     // clamp (also +inf)
  return (uint32_t)(p * 1073741824.f);  // exact scaling by 2^30, truncation
}

// a * b < c * d in 128 bits (all operands < 2^64)
__device__ __forceinline__ bool mul_less(unsigned long long a, unsigned long long b, unsigned long long c,
                                         unsigned long long d) {
  const unsigned long long lh = __umul64hi(a, b), ll = a * b;
  const unsigned long long rh = __umul64hi(c, d), rl = c * d;
  return lh < rh || (lh == rh && ll < rl);
}

__device__ __forceinline__ unsigned long long block_sum(unsigned long long x, unsigned long long *red) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
  __syncthreads();  // red may still be read from the previous call
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}

__global__ __launch_bounds__(kThreads) void tree_accept_sample_kernel(
    int max_nodes, int V, const int32_t *__restrict__ node_offset, const int32_t *__restrict__ parent,
    const int32_t *__restrict__ draft_ids, const float *__restrict__ p_target, const float *__restrict__ q_draft,
    const uint32_t *__restrict__ u_accept, const uint32_t *__restrict__ u_bonus, int max_path,
    int32_t *__restrict__ accept_len, int32_t *__restrict__ accept_path, int32_t *__restrict__ out_tokens,
    int32_t *__restrict__ bonus_id, uint32_t *__restrict__ work_all) {
  __shared__ int32_t spar[64], sdraft[64], spath[64], sremoved[64];
  __shared__ unsigned long long red[4];
  __shared__ unsigned long long chunk_sum[kThreads];
  __shared__ int s_decision;
  const int b = blockIdx.x;
  const int tid = threadIdx.x;
  const int n0 = node_offset[b];
  int n = node_offset[b + 1] - n0;
  n = n < 0 ? 0 : (n > max_nodes ? max_nodes : n);
  int32_t *path_out = accept_path + (size_t)b * max_path;
  int32_t *tok_out = out_tokens + (size_t)b * max_path;
  if (n == 0) {  // nothing to verify: nothing is emitted
    for (int j = tid; j < max_path; j += kThreads) { path_out[j] = -1; tok_out[j] = -1; }
    if (tid == 0) { accept_len[b] = 0; bonus_id[b] = -1; }
    return;
  }
  if (tid < 64) {
    int par = -1, did = 0;
    if (tid < n) {
      par = parent[n0 + tid];
      if (par >= tid || par < -1 || tid == 0) par = -1;  // malformed: never anybody's child
      did = draft_ids[n0 + tid];
    }
    spar[tid] = par;
    sdraft[tid] = did;
  }
  __syncthreads();
  uint32_t *work = work_all + (size_t)b * V;

  int cur = 0, len = 1, bonus = -1;
  if (tid == 0) spath[0] = 0;
#pragma unroll 1
  for (;;) {
    const float *prow = p_target + (size_t)(n0 + cur) * V;
    const float *qrow = q_draft + (size_t)(n0 + cur) * V;
    bool in_work = false;  // current p: the target's row (false) or the residual in the workspace
    int n_removed = 0;
    unsigned long long sp = 0, sq = 0;
    for (int v = tid; v < V; v += kThreads) { sp += fix_prob(prow[v]); sq += fix_prob(qrow[v]); }
    sp = block_sum(sp, red);
    sq = block_sum(sq, red);
    int taken = -1;
    if (len < max_path) {
#pragma unroll 1
      for (int c = cur + 1; c < n; ++c) {
        if (spar[c] != cur) continue;  // uniform
        int x = sdraft[c];
        const bool x_ok = x >= 0 && x < V;
        x = x_ok ? x : 0;
        if (tid == 0) {
          unsigned long long px = x_ok ? (in_work ? work[x] : fix_prob(prow[x])) : 0ull;
          unsigned long long qx = x_ok ? fix_prob(qrow[x]) : 0ull;
          for (int i = 0; i < n_removed; ++i) qx = sremoved[i] == x ? 0ull : qx;
          const unsigned long long u = u_accept[n0 + c];
          // u q_x S(p) < 2^32 p_x S(q); u q_x < 2^63 and p_x S(q) < 2^62 fit 64 bits
          s_decision = mul_less(u * qx, sp, px * sq, 1ull << 32) ? 1 : 0;
          chunk_sum[0] = qx;
        }
        __syncthreads();
        const bool accept = s_decision != 0;
        const unsigned long long qx = chunk_sum[0];
        __syncthreads();
        if (accept) { taken = c; break; }
        // residual: first its sum, then the rescaled values (and their sum) into the workspace
        unsigned long long sr = 0;
        for (int v = tid; v < V; v += kThreads) {
          const unsigned long long pv = in_work ? work[v] : fix_prob(prow[v]);
          const unsigned long long a = pv * sq, bq = (unsigned long long)fix_prob(qrow[v]) * sp;
          sr += a > bq ? a - bq : 0ull;
        }
        sr = block_sum(sr, red);
        if (sr != 0) {
          unsigned long long div = sr >> kFixBits;
          div = div ? div : 1ull;
          unsigned long long snew = 0;
          for (int v = tid; v < V; v += kThreads) {
            const unsigned long long pv = in_work ? work[v] : fix_prob(prow[v]);
            const unsigned long long a = pv * sq, bq = (unsigned long long)fix_prob(qrow[v]) * sp;
            const unsigned long long r = (a > bq ? a - bq : 0ull) / div;
            work[v] = (uint32_t)r;
            snew += r;
          }
          sp = block_sum(snew, red);
          in_work = true;
        }
        if (tid == 0 && x_ok) sremoved[n_removed] = x;
        n_removed += x_ok ? 1 : 0;
        sq -= qx;
        __syncthreads();
      }
    }
    if (taken < 0) {
      // last token: inverse CDF of the current p over contiguous chunks, one per thread
      if (sp != 0) {
        const unsigned long long t = ((unsigned long long)u_bonus[b] * sp) >> 32;  // S(p) < 2^32
        const int chunk = (V + kThreads - 1) / kThreads;
        const int v0 = tid * chunk, v1 = min(V, v0 + chunk);
        unsigned long long cs = 0;
        for (int v = v0; v < v1; ++v) cs += in_work ? work[v] : fix_prob(prow[v]);
        __syncthreads();
        chunk_sum[tid] = cs;
        __syncthreads();
        unsigned long long before = 0;
        for (int i = 0; i < tid; ++i) before += chunk_sum[i];
        if (before <= t && t < before + cs) {  // exactly one thread
          unsigned long long acc = before;
          for (int v = v0; v < v1; ++v) {
            acc += in_work ? work[v] : fix_prob(prow[v]);
            if (acc > t) { s_decision = v; break; }
          }
        }
        __syncthreads();
        bonus = s_decision;
      }
      break;
    }
    if (tid == 0) spath[len] = taken;
    ++len;
    cur = taken;
    __syncthreads();
  }
  __syncthreads();
  for (int j = tid; j < max_path; j += kThreads) {
    path_out[j] = j < len ? spath[j] : -1;
    tok_out[j] = j + 1 < len ? sdraft[spath[j + 1]] : (j + 1 == len ? bonus : -1);
  }
  if (tid == 0) { accept_len[b] = len; bonus_id[b] = bonus; }
}

}  // namespace

hipError_t launch_tree_accept_sample(int32_t B, int32_t max_nodes, int32_t V, const int32_t *node_offset,
                                     const int32_t *parent, const int32_t *draft_ids, const float *p_target,
                                     const float *q_draft, const uint32_t *u_accept, const uint32_t *u_bonus,
                                     int32_t max_path, int32_t *accept_len, int32_t *accept_path,
                                     int32_t *out_tokens, int32_t *bonus_id, uint32_t *work, hipStream_t s) {
  tree_accept_sample_kernel<<<B, kThreads, 0, s>>>(max_nodes, V, node_offset, parent, draft_ids, p_target, q_draft,
                                                   u_accept, u_bonus, max_path, accept_len, accept_path, out_tokens,
                                                   bonus_id, work);
  return hipGetLastError();
}

}  // namespace hb
