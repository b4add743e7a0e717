// Device-side body of the stable bucketing (shared by the stand-alone bucket kernel and the
// fused router tail).  Must be called by all 256 threads of a work-group.
#pragma once

#include "moqe_internal.h"

namespace moqe {

// counts[k] = #{s : e[s] = k} (the n_i of MoQE Eq. 2); offsets = exclusive prefix sum;
// inv_perm[s] = offsets[e[s]] + #{s' < s : e[s'] = e[s]}; perm[inv_perm[s]] = s.
// The histogram uses LDS atomics; ranks use wave ballots so that the order inside a bucket is
// the sample order, which makes the permutation unique and reproducible.
static __device__ __forceinline__ void bucket_body(const int32_t* expert_idx, int S, int K,
                                                   int32_t* __restrict__ counts, int32_t* __restrict__ offsets,
                                                   int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm) {
  __shared__ int cnt[MOQE_MAX_EXPERTS];
  __shared__ int base[MOQE_MAX_EXPERTS + 1];
  __shared__ int run[MOQE_MAX_EXPERTS];
  __shared__ int wcnt[4][MOQE_MAX_EXPERTS];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid < MOQE_MAX_EXPERTS) { cnt[tid] = 0; run[tid] = 0; }
  __syncthreads();
  for (int s = tid; s < S; s += 256) {
    int e = expert_idx[s];
    if (e >= 0 && e < K) atomicAdd(&cnt[e], 1);
  }
  __syncthreads();
  if (tid == 0) {
    int acc = 0;
    for (int k = 0; k < K; ++k) { base[k] = acc; acc += cnt[k]; }
    base[K] = acc;
  }
  __syncthreads();
  if (tid <= K) offsets[tid] = base[tid];
  if (counts && tid < K) counts[tid] = cnt[tid];
  if (!perm && !inv_perm) return;

  const unsigned long long lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  for (int c0 = 0; c0 < S; c0 += 256) {
    const int s = c0 + tid;
    int e = (s < S) ? expert_idx[s] : -1;
    if (e >= K) e = -1;
    int my_rank = 0;
    for (int k = 0; k < K; ++k) {
      unsigned long long b = __ballot(e == k);
      if (e == k) my_rank = __popcll(b & lt_mask);
      if (lane == 0) wcnt[wave][k] = __popcll(b);
    }
    __syncthreads();
    if (e >= 0) {
      int pos = base[e] + run[e] + my_rank;
      for (int w = 0; w < wave; ++w) pos += wcnt[w][e];
      if (perm) perm[pos] = s;
      if (inv_perm) inv_perm[s] = pos;
    }
    __syncthreads();
    if (tid < K) run[tid] += wcnt[0][tid] + wcnt[1][tid] + wcnt[2][tid] + wcnt[3][tid];
    __syncthreads();
  }
}

}  // namespace moqe
