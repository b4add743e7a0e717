// The router's training labels (MoQE Section 3.3, first paragraph): every sample runs through ALL experts,
// the prediction loss of each expert on the sample is taken, and the expert of lowest loss is the label.
// The K full forward passes are ONE grouped launch over K*S virtual samples (virtual sample j*S + s is
// sample s in expert j's bucket); the kernels here build that dispatch, reduce the logits to one
// cross-entropy per (sample, expert) and pick the arg-min.
#include "moqe_internal.h"

namespace moqe {

// offsets[j] = j*S (j <= K), perm[j*S + s] = s: every expert's bucket holds every sample, in order.
__global__ __launch_bounds__(256) void k_label_dispatch(int S, int K, int32_t* __restrict__ offsets, int32_t* __restrict__ perm) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i <= K) offsets[i] = i * S;
  if (i < K * S) perm[i] = i % S;
}

// All 64 lanes get the same value: xor-butterfly with a fixed order.
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v = fmaxf(v, __shfl_xor(v, d));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d);
  return v;
}

// One work-group per (expert j, sample s); wave w takes rows w, w + 4, ... of the sample's T rows.
// Row loss = max + log(sum exp(y - max)) - y[target], fp32; a wave adds its rows in order, the four
// waves' sums are added in order: the result does not depend on timing.
// y: [K*S*T, n] fp32, row (j*S + s)*T + t; targets [S, T] (clamped into [0, n)); losses [S, K].
__global__ __launch_bounds__(256) void k_label_loss(const float* __restrict__ y, const int32_t* __restrict__ targets, int S,
                                                     int T, int n, int K, float* __restrict__ losses) {
  __shared__ float part[4];
  const int j = blockIdx.x / S, s = blockIdx.x % S;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  float acc = 0.f;
  for (int t = wave; t < T; t += 4) {
    const float* row = y + (size_t(j) * S + s) * size_t(T) * n + size_t(t) * n;
    float mx = -INFINITY;
    for (int c = lane; c < n; c += 64) mx = fmaxf(mx, row[c]);
    mx = wave_max(mx);
    float sum = 0.f;
    for (int c = lane; c < n; c += 64) sum += expf(row[c] - mx);
    sum = wave_sum(sum);
    int tg = targets[size_t(s) * T + t];
    tg = tg < 0 ? 0 : (tg >= n ? n - 1 : tg);
    acc += mx + logf(sum) - row[tg];
  }
  if (lane == 0) part[wave] = acc;
  __syncthreads();
  if (threadIdx.x == 0) losses[size_t(s) * K + j] = (((part[0] + part[1]) + part[2]) + part[3]) / float(T);
}

// labels[s] = the first expert whose loss is the lowest.
__global__ __launch_bounds__(256) void k_label_argmin(const float* __restrict__ losses, int S, int K, int32_t* __restrict__ labels) {
  const int s = blockIdx.x * 256 + threadIdx.x;
  if (s >= S) return;
  int best = 0;
  float lb = losses[size_t(s) * K];
  for (int j = 1; j < K; ++j) {
    const float l = losses[size_t(s) * K + j];
    if (l < lb) { lb = l; best = j; }
  }
  labels[s] = best;
}

int32_t launch_label_dispatch(int S, int K, int32_t* offsets, int32_t* perm, hipStream_t st) {
  ProfileScope ps(MOQE_PK_BUCKET, st);
  const int items = K * S > K + 1 ? K * S : K + 1;
  hipLaunchKernelGGL(k_label_dispatch, dim3((items + 255) / 256), dim3(256), 0, st, S, K, offsets, perm);
  return check_launch("label_pass(dispatch)");
}

int32_t launch_label_loss(const float* y, const int32_t* targets, int S, int T, int n, int K, float* losses, int32_t* labels,
                          hipStream_t st) {
  ProfileScope ps(MOQE_PK_OTHER, st);
  hipLaunchKernelGGL(k_label_loss, dim3(unsigned(S) * unsigned(K)), dim3(256), 0, st, y, targets, S, T, n, K, losses);
  hipLaunchKernelGGL(k_label_argmin, dim3((S + 255) / 256), dim3(256), 0, st, losses, S, K, labels);
  return check_launch("label_pass(loss)");
}

}  // namespace moqe
