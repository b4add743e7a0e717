// Dispatch counts (the n_i of MoQE Eq. 2), their exclusive prefix sum, and the STABLE
// permutation that makes each expert's samples contiguous.  One work-group.
#include "bucket_device.h"

namespace moqe {

__global__ __launch_bounds__(256) void k_bucket(const int32_t* __restrict__ expert_idx, int S, int K,
                                                 int32_t* __restrict__ counts, int32_t* __restrict__ offsets,
                                                 int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm) {
  bucket_body(expert_idx, S, K, counts, offsets, perm, inv_perm);
}

// Up to 64 samples: one wave, a sample per lane.  The count of expert k is the population of the
// ballot "my sample goes to k", a sample's rank inside its bucket the population of that ballot
// below its lane: no LDS, no barriers, same result as the general kernel.
__global__ __launch_bounds__(64) void k_bucket_wave(const int32_t* __restrict__ expert_idx, int S, int K,
                                                     int32_t* __restrict__ counts, int32_t* __restrict__ offsets,
                                                     int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm) {
  const int lane = threadIdx.x;
  int e = lane < S ? expert_idx[lane] : -1;
  if (e >= K) e = -1;
  const unsigned long long lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  int base = 0, my_pos = 0;
  for (int k = 0; k < K; ++k) {
    const unsigned long long b = __ballot(e == k);
    const int c = __popcll(b);
    if (e == k) my_pos = base + __popcll(b & lt_mask);
    if (lane == 0) {
      offsets[k] = base;
      if (counts) counts[k] = c;
    }
    base += c;
  }
  if (lane == 0) offsets[K] = base;
  if (e >= 0) {
    if (perm) perm[my_pos] = lane;
    if (inv_perm) inv_perm[lane] = my_pos;
  }
}

int32_t launch_bucket(const int32_t* idx, int S, int K, int32_t* counts, int32_t* offsets,
                      int32_t* perm, int32_t* inv_perm, hipStream_t st) {
  ProfileScope ps(MOQE_PK_BUCKET, st);
  if (S <= 64) hipLaunchKernelGGL(k_bucket_wave, dim3(1), dim3(64), 0, st, idx, S, K, counts, offsets, perm, inv_perm);
  else hipLaunchKernelGGL(k_bucket, dim3(1), dim3(256), 0, st, idx, S, K, counts, offsets, perm, inv_perm);
  return check_launch("bucket");
}

// Samples of different lengths.  After the samples are grouped by expert, their rows are: slot j of the
// bucket order holds sample perm[j] with the rows cu_rows[perm[j]] .. cu_rows[perm[j] + 1).
//   slot_rows[j]   = first bucket-order row of slot j (exclusive prefix sum of the lengths), slot_rows[S] = M
//   row_offsets[e] = slot_rows[offsets[e]]: first bucket-order row of expert e, row_offsets[K] = M
// One work-group; the scan over the slots runs in blocks of 256 with a fixed order.
__global__ __launch_bounds__(256) void k_slot_rows(const int32_t* __restrict__ cu_rows, const int32_t* __restrict__ offsets,
                                                    const int32_t* __restrict__ perm, int S, int K,
                                                    int32_t* __restrict__ slot_rows, int32_t* __restrict__ row_offsets) {
  __shared__ int part[256];
  __shared__ int carry;
  const int tid = threadIdx.x;
  if (tid == 0) carry = 0;
  __syncthreads();
  for (int j0 = 0; j0 < S; j0 += 256) {
    const int j = j0 + tid;
    int len = 0;
    if (j < S) { const int s = perm[j]; len = cu_rows[s + 1] - cu_rows[s]; }
    part[tid] = len;
    __syncthreads();
    for (int d = 1; d < 256; d <<= 1) {                 // inclusive scan (Hillis-Steele)
      const int v = tid >= d ? part[tid - d] : 0;
      __syncthreads();
      part[tid] += v;
      __syncthreads();
    }
    if (j < S) slot_rows[j] = carry + part[tid] - len;
    __syncthreads();
    if (tid == 255) carry += part[255];
    __syncthreads();
  }
  if (tid == 0) slot_rows[S] = carry;
  __syncthreads();
  if (tid <= K) {
    const int j = offsets[tid];
    row_offsets[tid] = j < S ? slot_rows[j] : carry;     // written by this work-group: visible after the barrier
  }
}

// row_perm[slot_rows[j] + t] = cu_rows[perm[j]] + t: source row of every bucket-order row.  A wave per slot.
__global__ __launch_bounds__(256) void k_row_perm(const int32_t* __restrict__ cu_rows, const int32_t* __restrict__ perm,
                                                   const int32_t* __restrict__ slot_rows, int S, int32_t* __restrict__ row_perm) {
  const int j = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (j >= S) return;
  const int s = perm[j], src0 = cu_rows[s], len = cu_rows[s + 1] - src0, dst0 = slot_rows[j];
  for (int t = threadIdx.x & 63; t < len; t += 64) row_perm[dst0 + t] = src0 + t;
}

int32_t launch_expand_rows(const int32_t* cu_rows, const int32_t* offsets, const int32_t* perm, int S, int K,
                           int32_t* slot_rows, int32_t* row_offsets, int32_t* row_perm, hipStream_t st) {
  ProfileScope ps(MOQE_PK_BUCKET, st);
  hipLaunchKernelGGL(k_slot_rows, dim3(1), dim3(256), 0, st, cu_rows, offsets, perm, S, K, slot_rows, row_offsets);
  hipLaunchKernelGGL(k_row_perm, dim3((S + 3) / 4), dim3(256), 0, st, cu_rows, perm, slot_rows, S, row_perm);
  return check_launch("expand_rows");
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
