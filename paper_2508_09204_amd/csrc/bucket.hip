// Dispatch counts (the n_i of MoQE Eq. 2), their exclusive prefix sum, and the STABLE
// permutation that makes each expert's samples contiguous.  One work-group; the histogram
// uses LDS atomics, the ranks use wave ballots so that the order inside a bucket is the
// sample order (which makes the permutation unique and reproducible).
#include "moqe_internal.h"

namespace moqe {

__global__ __launch_bounds__(256) void k_bucket(const int32_t* __restrict__ expert_idx, int S, int K,
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

int32_t launch_bucket(const int32_t* idx, int S, int K, int32_t* counts, int32_t* offsets,
                      int32_t* perm, int32_t* inv_perm, hipStream_t st) {
  ProfileScope ps(MOQE_PK_BUCKET, st);
  hipLaunchKernelGGL(k_bucket, dim3(1), dim3(256), 0, st, idx, S, K, counts, offsets, perm, inv_perm);
  return check_launch("bucket");
}

}  // namespace moqe
