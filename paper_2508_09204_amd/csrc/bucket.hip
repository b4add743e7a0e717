// Dispatch counts (the n_i of MoQE Eq. 2), their exclusive prefix sum, and the STABLE
// permutation that makes each expert's samples contiguous.  One work-group.
#include "bucket_device.h"

namespace moqe {

__global__ __launch_bounds__(256) void k_bucket(const int32_t* __restrict__ expert_idx, int S, int K,
                                                 int32_t* __restrict__ counts, int32_t* __restrict__ offsets,
                                                 int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm) {
  bucket_body(expert_idx, S, K, counts, offsets, perm, inv_perm);
}

int32_t launch_bucket(const int32_t* idx, int S, int K, int32_t* counts, int32_t* offsets,
                      int32_t* perm, int32_t* inv_perm, hipStream_t st) {
  ProfileScope ps(MOQE_PK_BUCKET, st);
  hipLaunchKernelGGL(k_bucket, dim3(1), dim3(256), 0, st, idx, S, K, counts, offsets, perm, inv_perm);
  return check_launch("bucket");
}

// Load-balance statistics (MoQE Section 3.2, Eq. 1-2) of one batch.  One work-group: thread t adds
// the softmax probabilities of samples t, t + 256, ... in that order, the 256 partial sums per
// expert are added by a fixed tree in LDS, thread 0 finishes.  fp32 throughout.
__global__ __launch_bounds__(256) void k_balance_stats(const float* __restrict__ logits, const int32_t* __restrict__ counts,
                                                        int S, int K, float alpha, float* __restrict__ out) {
  __shared__ float red[MOQE_MAX_EXPERTS][256];
  const int tid = threadIdx.x;
  float psum[MOQE_MAX_EXPERTS];
#pragma unroll
  for (int k = 0; k < MOQE_MAX_EXPERTS; ++k) psum[k] = 0.f;
  for (int s = tid; s < S; s += 256) {
    const float* z = logits + size_t(s) * K;
    float zmax = z[0];
    for (int k = 1; k < K; ++k) zmax = fmaxf(zmax, z[k]);
    float e[MOQE_MAX_EXPERTS], den = 0.f;
#pragma unroll
    for (int k = 0; k < MOQE_MAX_EXPERTS; ++k) {
      e[k] = k < K ? expf(z[k] - zmax) : 0.f;
      den += e[k];
    }
    const float inv = 1.f / den;
#pragma unroll
    for (int k = 0; k < MOQE_MAX_EXPERTS; ++k) psum[k] += e[k] * inv;
  }
#pragma unroll
  for (int k = 0; k < MOQE_MAX_EXPERTS; ++k) red[k][tid] = psum[k];
  __syncthreads();
  for (int w = 128; w >= 1; w >>= 1) {
    if (tid < w) {
#pragma unroll
      for (int k = 0; k < MOQE_MAX_EXPERTS; ++k) red[k][tid] += red[k][tid + w];
    }
    __syncthreads();
  }
  if (tid == 0) {
    const float mean = float(S) / float(K);
    float lbal = 0.f, var = 0.f;
    for (int k = 0; k < K; ++k) {
      const float P = red[k][0] / float(S), n = float(counts[k]), F = n / float(S);
      out[k] = P;
      out[K + k] = F;
      lbal += P * F;
      var += (n - mean) * (n - mean);
    }
    const float sigma = sqrtf(var / float(K)) / mean;
    out[2 * K] = float(K) * lbal;
    out[2 * K + 1] = sigma;
    out[2 * K + 2] = alpha * (1.f + sigma);
  }
}

int32_t launch_balance_stats(const float* logits, const int32_t* counts, int S, int K, float alpha, float* out,
                             hipStream_t st) {
  ProfileScope ps(MOQE_PK_OTHER, st);
  hipLaunchKernelGGL(k_balance_stats, dim3(1), dim3(256), 0, st, logits, counts, S, K, alpha, out);
  return check_launch("balance_stats");
}

}  // namespace moqe
