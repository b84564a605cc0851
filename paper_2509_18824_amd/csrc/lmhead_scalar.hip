// LM head with fused argmax, scalar fp32 kernel (any dtype, any sizes), plus the two tiny
// kernels every LM-head path shares: key initialisation and the final unpack.
//
// Each workgroup computes a 64 x 64 tile of logits (rows of `hidden` x rows of `weight`) in
// registers, reduces each row of the tile to one (value, index) key and folds it into the
// row's global key with a 64-bit atomic max.  max over keys is order independent, so the
// result does not depend on scheduling.
#include "hb_internal.h"

namespace hb {

namespace {

constexpr int TM = 64, TN = 64, TK = 16;

template <typename T>
__global__ __launch_bounds__(256) void lmhead_scalar_kernel(int M, int K, int V, const T *__restrict__ hidden,
                                                            const T *__restrict__ weight,
                                                            unsigned long long *__restrict__ keys) {
  __shared__ float sh[TK][TM + 1];
  __shared__ float sw[TK][TN + 1];
  __shared__ unsigned long long srow[TM];
  const int tid = threadIdx.x;
  const int tx = tid & 15;   // column group: columns tx*4 .. tx*4+3
  const int ty = tid >> 4;   // row group: rows ty*4 .. ty*4+3
  const int m0 = blockIdx.y * TM;
  const int v0 = blockIdx.x * TN;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
  if (tid < TM) srow[tid] = 0ull;

  for (int k0 = 0; k0 < K; k0 += TK) {
    // 64 rows x 16 k for each operand: 1024 elements, 4 per thread
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      int e = tid + 256 * r;
      int rr = e >> 4, kk = e & 15;
      int m = m0 + rr, v = v0 + rr, k = k0 + kk;
      sh[kk][rr] = (m < M && k < K) ? load_f32(hidden + (size_t)m * K + k) : 0.f;
      sw[kk][rr] = (v < V && k < K) ? load_f32(weight + (size_t)v * K + k) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < TK; ++kk) {
      float a[4], bcol[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = sh[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) bcol[j] = sw[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], bcol[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    unsigned long long best = 0ull;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int v = v0 + tx * 4 + j;
      if (v < V) {
        unsigned long long key = argmax_key(acc[i][j], (uint32_t)v);
        best = key > best ? key : best;
      }
    }
    if (best) atomicMax(&srow[ty * 4 + i], best);
  }
  __syncthreads();
  if (tid < TM && m0 + tid < M && srow[tid]) atomicMax(&keys[m0 + tid], srow[tid]);
}

__global__ void lmhead_init_kernel(unsigned long long *keys, int M) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < M) keys[i] = 0ull;
}

__global__ void lmhead_finish_kernel(const unsigned long long *keys, int M, int V, int32_t *out_ids,
                                     float *out_max) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= M) return;
  unsigned long long key = keys[i];
  uint32_t idx = key ? argmax_key_index(key) : 0u;
  if (idx >= (uint32_t)V) idx = 0;
  out_ids[i] = (int32_t)idx;
  if (out_max) out_max[i] = key ? argmax_key_value(key) : -__builtin_huge_valf();
}

}  // namespace

hipError_t launch_lmhead_scalar(int32_t dtype, int32_t M, int32_t K, int32_t V, const void *hidden,
                                const void *weight, unsigned long long *keys, hipStream_t s) {
  dim3 grid((unsigned)((V + TN - 1) / TN), (unsigned)((M + TM - 1) / TM));
  if (dtype == HB_F32)
    lmhead_scalar_kernel<float><<<grid, 256, 0, s>>>(M, K, V, (const float *)hidden, (const float *)weight, keys);
  else
    lmhead_scalar_kernel<bf16_t><<<grid, 256, 0, s>>>(M, K, V, (const bf16_t *)hidden, (const bf16_t *)weight, keys);
  return hipGetLastError();
}

hipError_t launch_lmhead_init(unsigned long long *keys, int32_t M, hipStream_t s) {
  lmhead_init_kernel<<<(M + 255) / 256, 256, 0, s>>>(keys, M);
  return hipGetLastError();
}

hipError_t launch_lmhead_finish(const unsigned long long *keys, int32_t M, int32_t V, int32_t *out_ids,
                                float *out_max, hipStream_t s) {
  lmhead_finish_kernel<<<(M + 255) / 256, 256, 0, s>>>(keys, M, V, out_ids, out_max);
  return hipGetLastError();
}

}  // namespace hb
