// Router: mean pooling, [Linear -> ReLU ->] Linear, top-1 selection (MoQE Section 3.2: the
// router is a classifier whose last stage is an MLP producing one logit per expert; one
// expert is activated per sample, Section 3.1).  All reductions run in a fixed order, so
// results are bit-reproducible from launch to launch.
#include "moqe_internal.h"

namespace moqe {

static __device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

static __device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// partial[s][c][d] = sum over the tokens of chunk c of x[s][t][d].
// Block: 256 threads = CT column-threads (8 columns each) x TR token-rows.
__global__ __launch_bounds__(256) void k_pool_partial(const uint16_t* __restrict__ x, float* __restrict__ partial,
                                                       int T, int D, int C, int CT) {
  __shared__ float red[256 * 8];
  const int s = blockIdx.z, c = blockIdx.y;
  const int TR = 256 / CT;
  const int ct = threadIdx.x % CT, tr = threadIdx.x / CT;
  const int col = (blockIdx.x * CT + ct) * 8;
  const int tchunk = (T + C - 1) / C;
  const int t0 = c * tchunk, t1 = min(T, t0 + tchunk);
  float acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.f;
  if (col < D) {
    const uint16_t* base = x + (size_t(s) * T) * D + col;
    for (int t = t0 + tr; t < t1; t += TR) {
      uint4 v = *reinterpret_cast<const uint4*>(base + size_t(t) * D);
      acc[0] += bf16_bits_to_float(v.x & 0xffffu); acc[1] += bf16_bits_to_float(v.x >> 16);
      acc[2] += bf16_bits_to_float(v.y & 0xffffu); acc[3] += bf16_bits_to_float(v.y >> 16);
      acc[4] += bf16_bits_to_float(v.z & 0xffffu); acc[5] += bf16_bits_to_float(v.z >> 16);
      acc[6] += bf16_bits_to_float(v.w & 0xffffu); acc[7] += bf16_bits_to_float(v.w >> 16);
    }
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) red[threadIdx.x * 8 + i] = acc[i];
  __syncthreads();
  if (tr == 0 && col < D) {
    float* out = partial + (size_t(s) * C + c) * D + col;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float v = 0.f;
      for (int r = 0; r < TR; ++r) v += red[(r * CT + ct) * 8 + i];   // fixed order
      out[i] = v;
    }
  }
}

// pooled[s][d] = (sum_c partial[s][c][d]) / T
__global__ void k_pool_finish(const float* __restrict__ partial, float* __restrict__ pooled, int S, int T, int D, int C) {
  size_t i = size_t(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i >= size_t(S) * D) return;
  int s = int(i / D), d = int(i % D);
  float v = 0.f;
  for (int c = 0; c < C; ++c) v += partial[(size_t(s) * C + c) * D + d];
  pooled[i] = __fdiv_rn(v, float(T));
}

// hidden[s][j] = relu(b1[j] + <w1[j,:], pooled[s,:]>).  One wave per (hidden unit, 8 samples).
__global__ __launch_bounds__(256) void k_router_hidden(const float* __restrict__ pooled, const float* __restrict__ w1,
                                                        const float* __restrict__ b1, float* __restrict__ hidden,
                                                        int S, int D, int Hd) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = blockIdx.x * 4 + wave;
  const int s0 = blockIdx.y * 8;
  if (j >= Hd) return;
  float acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.f;
  const float* wr = w1 + size_t(j) * D;
  for (int d = lane * 4; d < D; d += 256) {
    float4 w = *reinterpret_cast<const float4*>(wr + d);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (s0 + i < S) {
        float4 p = *reinterpret_cast<const float4*>(pooled + size_t(s0 + i) * D + d);
        acc[i] += w.x * p.x + w.y * p.y + w.z * p.z + w.w * p.w;
      }
    }
  }
  const float bias = b1 ? b1[j] : 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    float v = wave_sum(acc[i]);
    if (lane == 0 && s0 + i < S) hidden[size_t(s0 + i) * Hd + j] = fmaxf(v + bias, 0.f);
  }
}

// logits[s][k] = b2[k] + <w2[k,:], feat[s,:]>;  expert_idx[s] = first index of the maximum.
// One wave per sample.
__global__ __launch_bounds__(256) void k_router_logits_argmax(const float* __restrict__ feat, const float* __restrict__ w2,
                                                               const float* __restrict__ b2, int S, int Dk, int K,
                                                               int32_t* __restrict__ expert_idx, float* __restrict__ logits) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int s = blockIdx.x * 4 + wave;
  if (s >= S) return;
  const float* f = feat + size_t(s) * Dk;
  float best = 0.f;
  int best_k = 0;
  for (int k = 0; k < K; ++k) {
    const float* wr = w2 + size_t(k) * Dk;
    float acc = 0.f;
    for (int d = lane * 4; d < Dk; d += 256) {
      float4 w = *reinterpret_cast<const float4*>(wr + d);
      float4 p = *reinterpret_cast<const float4*>(f + d);
      acc += w.x * p.x + w.y * p.y + w.z * p.z + w.w * p.w;
    }
    float z = wave_sum(acc) + (b2 ? b2[k] : 0.f);
    if (logits && lane == 0) logits[size_t(s) * K + k] = z;
    if (k == 0 || z > best) { best = z; best_k = k; }   // strict >: ties keep the lowest index
  }
  if (lane == 0) expert_idx[s] = best_k;
}

static void pool_shape(int T, int D, int* C, int* CT) {
  int cols8 = D / 8;
  int ct = 1;
  while (ct < cols8 && ct < 256) ct <<= 1;
  *CT = ct;
  int c = T / 64;
  if (c < 1) c = 1;
  if (c > 16) c = 16;
  *C = c;
}

size_t route_ws_bytes(int S, int T, const moqe_router& r) {
  int C, CT;
  pool_shape(T, r.d, &C, &CT);
  size_t b = align256(size_t(S) * C * r.d * 4);          // partial sums
  b += align256(size_t(S) * r.d * 4);                    // pooled
  b += align256(size_t(S) * (r.h > 0 ? r.h : 1) * 4);    // hidden
  return b;
}

int32_t launch_route(const void* x, int S, int T, const moqe_router& r, int32_t* idx, float* logits,
                     void* ws, hipStream_t st) {
  int C, CT;
  pool_shape(T, r.d, &C, &CT);
  const int D = r.d;
  uint8_t* p = static_cast<uint8_t*>(ws);
  float* partial = reinterpret_cast<float*>(p);
  p += align256(size_t(S) * C * D * 4);
  float* pooled = reinterpret_cast<float*>(p);
  p += align256(size_t(S) * D * 4);
  float* hidden = reinterpret_cast<float*>(p);
  {
    ProfileScope ps(MOQE_PK_ROUTE, st);
    dim3 grid((D / 8 + CT - 1) / CT, C, S);
    hipLaunchKernelGGL(k_pool_partial, grid, dim3(256), 0, st, static_cast<const uint16_t*>(x), partial, T, D, C, CT);
  }
  {
    ProfileScope ps(MOQE_PK_ROUTE, st);
    size_t nel = size_t(S) * D;
    hipLaunchKernelGGL(k_pool_finish, dim3(unsigned((nel + 255) / 256)), dim3(256), 0, st, partial, pooled, S, T, D, C);
  }
  const float* feat = pooled;
  int Dk = D;
  if (r.h > 0) {
    ProfileScope ps(MOQE_PK_ROUTE, st);
    dim3 grid((r.h + 3) / 4, (S + 7) / 8);
    hipLaunchKernelGGL(k_router_hidden, grid, dim3(256), 0, st, pooled, r.w1, r.b1, hidden, S, D, r.h);
    feat = hidden;
    Dk = r.h;
  }
  {
    ProfileScope ps(MOQE_PK_ROUTE, st);
    hipLaunchKernelGGL(k_router_logits_argmax, dim3((S + 3) / 4), dim3(256), 0, st, feat, r.w2, r.b2, S, Dk,
                       r.n_experts, idx, logits);
  }
  return check_launch("route");
}

}  // namespace moqe
