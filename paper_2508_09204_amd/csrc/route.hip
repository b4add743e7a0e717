// Router: mean pooling, [Linear -> ReLU ->] Linear, top-1 selection (MoQE Section 3.2: the
// router is a classifier whose last stage is an MLP producing one logit per expert; one
// expert is activated per sample, Section 3.1).  All reductions run in a fixed order, so
// results are bit-reproducible from launch to launch.
#include "bucket_device.h"

namespace moqe {

static __device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

static __device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// partial[s][c][d] = sum over the tokens of chunk c of x[s][t][d].
// Block: 256 threads = CT column-threads (8 columns each) x TR token-rows.
// With one chunk (C == 1, `finish` set) the sum is divided by T here and written as the pooled feature: the
// arithmetic of k_pool_finish on a single chunk (0 + sum, then the division), without its launch.
__global__ __launch_bounds__(256) void k_pool_partial(const uint16_t* __restrict__ x, float* __restrict__ partial,
                                                       int T, int D, int C, int CT, int finish) {
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
    // eight rows' loads in flight (rows past the chunk's end are clamped, loaded and not added); the additions keep
    // their order
    for (int t = t0 + tr; t < t1; t += 8 * TR) {
      uint4 v4[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v4[u] = *reinterpret_cast<const uint4*>(base + size_t(min(t + u * TR, t1 - 1)) * D);
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (t + u * TR < t1) {
          const uint4 v = v4[u];
          acc[0] += bf16_bits_to_float(v.x & 0xffffu); acc[1] += bf16_bits_to_float(v.x >> 16);
          acc[2] += bf16_bits_to_float(v.y & 0xffffu); acc[3] += bf16_bits_to_float(v.y >> 16);
          acc[4] += bf16_bits_to_float(v.z & 0xffffu); acc[5] += bf16_bits_to_float(v.z >> 16);
          acc[6] += bf16_bits_to_float(v.w & 0xffffu); acc[7] += bf16_bits_to_float(v.w >> 16);
        }
      }
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
      out[i] = finish ? __fdiv_rn(v, float(T)) : v;
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

// Hidden layer on the fp32 matrix cores.  part[kz][s][j] = sum over k-slice kz of feat[s][k] * w1[j][k]
// for one tile of 16 samples x 16 hidden units.  The tile's operands are first copied to LDS with
// coalesced loads (one round trip: every load of the work-group is issued before any is used; a
// direct operand-shaped read touches 64 cache lines per instruction and is bound by the texture
// path), then each of the 4 waves multiplies a quarter of the slice and the four partial tiles
// are added through LDS in wave order.  Bias and ReLU are applied by the consumer, which adds the
// slices in order, so the result does not depend on scheduling.
// XBF16: feat is the bf16 activation matrix itself (T == 1, pooling is the identity).
typedef float f32x4_t __attribute__((ext_vector_type(4)));
static __device__ __forceinline__ float4 keep4(float4 v, bool ok) {
  return make_float4(ok ? v.x : 0.f, ok ? v.y : 0.f, ok ? v.z : 0.f, ok ? v.w : 0.f);
}
constexpr int HID_KC = 512;                       // columns per k-slice
constexpr int HID_STRIDE = HID_KC + 4;            // LDS row stride in floats (bank-conflict free b128 reads)

template <bool XBF16>
__global__ __launch_bounds__(256) void k_router_hidden(const void* __restrict__ feat, const float* __restrict__ w1,
                                                        float* __restrict__ part, int S, int D, int Hd) {
  __shared__ __align__(16) float wt[16 * HID_STRIDE];
  __shared__ __align__(16) float xt[16 * HID_STRIDE];
  __shared__ float red[3][4][64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int h0 = blockIdx.x * 16, s0 = blockIdx.y * 16, kz = blockIdx.z;
  const int kbeg = kz * HID_KC;
  // ---- stage: thread t copies columns 4*(t%128) .. +3 of rows t/128, t/128 + 2, ... ----
  {
    const int c4 = (tid & 127) * 4;
    const bool kin = kbeg + c4 < D;
    const int kc = kin ? kbeg + c4 : 0;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const int row = (tid >> 7) + 2 * r;
      const int hr = min(h0 + row, Hd - 1), sr = min(s0 + row, S - 1);
      const float4 wv = *reinterpret_cast<const float4*>(w1 + size_t(hr) * D + kc);
      float4 xv;
      if constexpr (XBF16) {
        const uint2 v = *reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(feat) + size_t(sr) * D + kc);
        xv = make_float4(__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xffff0000u),
                         __uint_as_float(v.y << 16), __uint_as_float(v.y & 0xffff0000u));
      } else {
        xv = *reinterpret_cast<const float4*>(static_cast<const float*>(feat) + size_t(sr) * D + kc);
      }
      const bool wok = kin && h0 + row < Hd, xok = kin && s0 + row < S;
      *reinterpret_cast<float4*>(wt + row * HID_STRIDE + c4) = keep4(wv, wok);
      *reinterpret_cast<float4*>(xt + row * HID_STRIDE + c4) = keep4(xv, xok);
    }
  }
  __syncthreads();
  // ---- multiply: wave w takes columns [128w, 128w + 128): 8 steps of 16 columns ----
  const int i = lane & 15, q = lane >> 4;
  f32x4_t acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int st = 0; st < 8; ++st) {
    const int c = wave * 128 + st * 16 + 4 * q;
    const float4 a = *reinterpret_cast<const float4*>(xt + i * HID_STRIDE + c);
    const float4 b = *reinterpret_cast<const float4*>(wt + i * HID_STRIDE + c);
    acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(a.x, b.x, acc0, 0, 0, 0);
    acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(a.y, b.y, acc1, 0, 0, 0);
    acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(a.z, b.z, acc0, 0, 0, 0);
    acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(a.w, b.w, acc1, 0, 0, 0);
  }
  const f32x4_t acc = acc0 + acc1;
  if (wave > 0) {
#pragma unroll
    for (int r = 0; r < 4; ++r) red[wave - 1][r][lane] = acc[r];
  }
  __syncthreads();
  if (wave == 0) {
    const int j = h0 + i;                                  // result column i, rows 4q + r
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float v = ((acc[r] + red[0][r][lane]) + red[1][r][lane]) + red[2][r][lane];
      const int sm = s0 + 4 * q + r;
      if (sm < S && j < Hd) part[(size_t(kz) * S + sm) * Hd + j] = v;
    }
  }
}

// Features of sample s for the last layer: the pooled input itself, or relu(b1 + the hidden layer's
// k-slices added in order).
static __device__ __forceinline__ float4 feature4(const float* __restrict__ feat, int nslices, size_t slice_stride,
                                                  const float* __restrict__ b1, size_t off, int d) {
  float4 p = *reinterpret_cast<const float4*>(feat + off);
  if (nslices > 0) {
#pragma unroll 8
    for (int z = 1; z < nslices; ++z) {
      const float4 t = *reinterpret_cast<const float4*>(feat + z * slice_stride + off);
      p.x += t.x; p.y += t.y; p.z += t.z; p.w += t.w;
    }
    if (b1) { const float4 t = *reinterpret_cast<const float4*>(b1 + d); p.x += t.x; p.y += t.y; p.z += t.z; p.w += t.w; }
    p.x = fmaxf(p.x, 0.f); p.y = fmaxf(p.y, 0.f); p.z = fmaxf(p.z, 0.f); p.w = fmaxf(p.w, 0.f);
  }
  return p;
}

// One sample per wave (any batch size): logits[s][k] = b2[k] + <w2[k,:], f_s> and the first index of
// the maximum.  KP = number of experts rounded up to 4, 8 or 16: all loops have fixed bounds, and
// the KP cross-lane sums advance together so that their shuffles overlap.
template <int KP>
__global__ __launch_bounds__(256) void k_router_logits_argmax(const float* __restrict__ feat, int nslices, size_t slice_stride,
                                                               const float* __restrict__ b1, const float* __restrict__ w2,
                                                               const float* __restrict__ b2, int S, int Dk, int K,
                                                               int32_t* __restrict__ expert_idx, float* __restrict__ logits) {
  const int lane = threadIdx.x & 63;
  const int s = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (s >= S) return;
  // every feature is formed once (its slices are added here) and meets all K weight rows
  float acc[KP];
#pragma unroll
  for (int k = 0; k < KP; ++k) acc[k] = 0.f;
  for (int d = lane * 4; d < Dk; d += 256) {
    const float4 p = feature4(feat, nslices, slice_stride, b1, size_t(s) * Dk + d, d);
#pragma unroll
    for (int k = 0; k < KP; ++k) {
      const float4 w = *reinterpret_cast<const float4*>(w2 + size_t(k < K ? k : 0) * Dk + d);     // rows past K: row 0, unused
      acc[k] += w.x * p.x + w.y * p.y + w.z * p.z + w.w * p.w;
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
#pragma unroll
    for (int k = 0; k < KP; ++k) acc[k] += __shfl_xor(acc[k], off, 64);
  }
  float best = 0.f;
  int best_k = 0;
#pragma unroll
  for (int k = 0; k < KP; ++k) {
    if (k < K) {
      const float z = acc[k] + (b2 ? b2[k] : 0.f);
      if (logits && lane == 0) logits[size_t(s) * K + k] = z;
      if (k == 0 || z > best) { best = z; best_k = k; }   // strict >: ties keep the lowest index
    }
  }
  if (lane == 0) expert_idx[s] = best_k;
}

static void launch_logits_argmax(const float* feat, int nslices, size_t stride, const moqe_router& r, int S, int Dk,
                                 int32_t* idx, float* logits, hipStream_t st) {
  const dim3 grid((S + 3) / 4), block(256);
  const int K = r.n_experts;
  if (K <= 4) hipLaunchKernelGGL(k_router_logits_argmax<4>, grid, block, 0, st, feat, nslices, stride, r.b1, r.w2, r.b2, S, Dk, K, idx, logits);
  else if (K <= 8) hipLaunchKernelGGL(k_router_logits_argmax<8>, grid, block, 0, st, feat, nslices, stride, r.b1, r.w2, r.b2, S, Dk, K, idx, logits);
  else hipLaunchKernelGGL(k_router_logits_argmax<16>, grid, block, 0, st, feat, nslices, stride, r.b1, r.w2, r.b2, S, Dk, K, idx, logits);
}

// Logits, top-1 and the stable bucketing in ONE work-group (small batches: saves launches).
// A single work-group cannot hide latency behind other waves, so the kernel avoids chains of
// dependent accesses: all loads of a hidden-layer slice are issued together, features and last-
// layer weights sit in LDS, every (sample, expert) dot product belongs to one thread (independent
// 16-byte LDS reads, no cross-lane reductions), the chosen experts stay in LDS for the bucketing,
// and results are only stored.
// Needs S * K <= TAIL_MAX_PAIRS, S * (Dk + 4) <= TAIL_FEAT_FLOATS, S * Dk <= 1024 * TAIL_EPT (256 threads x TAIL_EPT
// groups of four floats) and
// K * (Dk + 4) <= TAIL_MAX_W2.
constexpr int TAIL_EPT = 16;               // float4 feature elements per thread, at most
constexpr int TAIL_FEAT_FLOATS = 16384 + 4096;
constexpr int TAIL_MAX_W2 = 4096 + 64;     // last-layer weights (rows padded by four floats)
constexpr int TAIL_MAX_PAIRS = 2048;       // (sample, expert) pairs
constexpr int TAIL_MAX_S = 1024;
constexpr int TAIL_LDS_BYTES = (TAIL_FEAT_FLOATS + TAIL_MAX_W2 + TAIL_MAX_PAIRS + TAIL_MAX_S) * 4;

__global__ __launch_bounds__(256) void k_router_tail(const float* __restrict__ feat, int nslices, size_t slice_stride,
                                                      const float* __restrict__ b1, const float* __restrict__ w2,
                                                      const float* __restrict__ b2, int S, int Dk, int K,
                                                      int32_t* __restrict__ expert_idx, float* __restrict__ logits,
                                                      int32_t* __restrict__ counts, int32_t* __restrict__ offsets,
                                                      int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm) {
  extern __shared__ __align__(16) float tail_lds[];
  float* fl = tail_lds;                                   // [S][Dk + 4]
  float* wl = tail_lds + TAIL_FEAT_FLOATS;                // [K][Dk + 4]
  float* zl = wl + TAIL_MAX_W2;                           // [S][K] logits
  int32_t* idx_l = reinterpret_cast<int32_t*>(zl + TAIL_MAX_PAIRS);
  const int tid = threadIdx.x;
  const int FS = Dk + 4;
  const int nel = S * Dk;
  for (int i = tid * 4; i < K * Dk; i += 1024) {
    const int k = i / Dk, d = i - k * Dk;
    *reinterpret_cast<float4*>(wl + k * FS + d) = *reinterpret_cast<const float4*>(w2 + i);
  }
  // features: element e of this thread is the float4 at flat index 4 * (tid + 256 e)
  float4 acc[TAIL_EPT];
#pragma unroll
  for (int e = 0; e < TAIL_EPT; ++e) {
    const int i = (tid + 256 * e) * 4;
    acc[e] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i < nel) acc[e] = *reinterpret_cast<const float4*>(feat + i);
  }
  for (int z = 1; z < nslices; ++z) {                     // slices of the hidden layer, added in order
    const float* fz = feat + z * slice_stride;
#pragma unroll
    for (int e = 0; e < TAIL_EPT; ++e) {
      const int i = (tid + 256 * e) * 4;
      if (i < nel) {
        const float4 t = *reinterpret_cast<const float4*>(fz + i);
        acc[e].x += t.x; acc[e].y += t.y; acc[e].z += t.z; acc[e].w += t.w;
      }
    }
  }
#pragma unroll
  for (int e = 0; e < TAIL_EPT; ++e) {
    const int i = (tid + 256 * e) * 4;
    if (i < nel) {
      const int sm = i / Dk, d = i - sm * Dk;
      float4 p = acc[e];
      if (nslices > 0) {                                  // hidden layer: bias and ReLU
        if (b1) { const float4 t = *reinterpret_cast<const float4*>(b1 + d); p.x += t.x; p.y += t.y; p.z += t.z; p.w += t.w; }
        p.x = fmaxf(p.x, 0.f); p.y = fmaxf(p.y, 0.f); p.z = fmaxf(p.z, 0.f); p.w = fmaxf(p.w, 0.f);
      }
      *reinterpret_cast<float4*>(fl + sm * FS + d) = p;
    }
  }
  __syncthreads();
  for (int pr = tid; pr < S * K; pr += 256) {
    const int sm = pr / K, k = pr - sm * K;
    const float4* f = reinterpret_cast<const float4*>(fl + sm * FS);
    const float4* w = reinterpret_cast<const float4*>(wl + k * FS);
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
    for (int d = 0; d < Dk / 4; ++d) {
      const float4 fv = f[d], wv = w[d];
      a0 += wv.x * fv.x; a1 += wv.y * fv.y; a2 += wv.z * fv.z; a3 += wv.w * fv.w;
    }
    const float z = ((a0 + a1) + (a2 + a3)) + (b2 ? b2[k] : 0.f);
    zl[pr] = z;
    if (logits) logits[pr] = z;
  }
  __syncthreads();
  for (int sm = tid; sm < S; sm += 256) {
    float best = zl[sm * K];
    int best_k = 0;
    for (int k = 1; k < K; ++k) {
      const float z = zl[sm * K + k];
      if (z > best) { best = z; best_k = k; }               // strict >: ties keep the lowest index
    }
    idx_l[sm] = best_k;
    expert_idx[sm] = best_k;
  }
  __syncthreads();
  bucket_body(idx_l, S, K, counts, offsets, perm, inv_perm);
}

// Samples of different lengths: pooled[s][d] = mean over the rows cu_rows[s] .. cu_rows[s+1] of x[., d].
// A thread owns 8 columns of one sample and adds that sample's rows in order (fp32).
__global__ __launch_bounds__(256) void k_pool_ragged(const uint16_t* __restrict__ x, const int32_t* __restrict__ cu_rows,
                                                      float* __restrict__ pooled, int D) {
  const int s = blockIdx.y;
  const int c8 = blockIdx.x * 256 + threadIdx.x;
  if (c8 * 8 >= D) return;
  const int r0 = cu_rows[s], r1 = cu_rows[s + 1];
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int r = r0; r < r1; ++r) {
    const uint4 v = *reinterpret_cast<const uint4*>(x + size_t(r) * D + c8 * 8);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      acc[2 * j] += bf16_bits_to_float(w[j] & 0xffffu);
      acc[2 * j + 1] += bf16_bits_to_float(w[j] >> 16);
    }
  }
  const float inv = r1 > r0 ? 1.0f / float(r1 - r0) : 0.f;      // a sample without rows has all-zero features
  float4 o0 = {acc[0] * inv, acc[1] * inv, acc[2] * inv, acc[3] * inv};
  float4 o1 = {acc[4] * inv, acc[5] * inv, acc[6] * inv, acc[7] * inv};
  float* dst = pooled + size_t(s) * D + c8 * 8;
  *reinterpret_cast<float4*>(dst) = o0;
  *reinterpret_cast<float4*>(dst + 4) = o1;
}

// Chunks of a sample's tokens (C) and column-threads per work-group (CT).  A batch that fills the chip with one
// work-group per sample and column block, and whose samples are short, is pooled in one chunk - and then in one launch.
static void pool_shape(int S, int T, int D, int* C, int* CT) {
  int cols8 = D / 8;
  int ct = 1;
  while (ct < cols8 && ct < 256) ct <<= 1;
  *CT = ct;
  int c = T / 64;
  if (c < 1) c = 1;
  if (c > 16) c = 16;
  if (T <= 256 && long(S) * ((cols8 + ct - 1) / ct) >= 256) c = 1;
  *C = c;
}

static int hidden_slices(int D) { return (D + HID_KC - 1) / HID_KC; }

size_t route_ws_bytes(int S, int T, const moqe_router& r) {
  int C, CT;
  pool_shape(S, T, r.d, &C, &CT);
  size_t b = align256(size_t(S) * C * r.d * 4);                   // partial sums of the pooling
  b += align256(size_t(S) * r.d * 4);                             // pooled features
  b += align256(size_t(hidden_slices(r.d)) * S * (r.h > 0 ? r.h : 1) * 4);   // hidden layer, one slab per k-slice
  return b;
}

// Pooling and hidden layer; returns the feature description for the logits stage.
struct RouteFeat { const float* feat; int nslices; size_t stride; int Dk; };

static int32_t route_front(const void* x, const int32_t* cu_rows, int S, int T, const moqe_router& r, void* ws, hipStream_t st,
                           RouteFeat* rf) {
  int C, CT;
  pool_shape(S, T, r.d, &C, &CT);
  const int D = r.d;
  uint8_t* p = static_cast<uint8_t*>(ws);
  float* partial = reinterpret_cast<float*>(p);
  p += align256(size_t(S) * C * D * 4);
  float* pooled = reinterpret_cast<float*>(p);
  p += align256(size_t(S) * D * 4);
  float* hidden = reinterpret_cast<float*>(p);
  const bool direct = (!cu_rows && T == 1 && r.h > 0);      // the hidden layer reads the bf16 rows themselves
  if (cu_rows) {
    ProfileScope ps(MOQE_PK_ROUTE, st);
    hipLaunchKernelGGL(k_pool_ragged, dim3((D / 8 + 255) / 256, S), dim3(256), 0, st, static_cast<const uint16_t*>(x), cu_rows,
                       pooled, D);
  } else if (!direct) {
    {
      ProfileScope ps(MOQE_PK_ROUTE, st);
      dim3 grid((D / 8 + CT - 1) / CT, C, S);
      hipLaunchKernelGGL(k_pool_partial, grid, dim3(256), 0, st, static_cast<const uint16_t*>(x), C == 1 ? pooled : partial, T, D, C,
                         CT, C == 1 ? 1 : 0);
    }
    if (C > 1) {
      ProfileScope ps(MOQE_PK_ROUTE, st);
      size_t nel = size_t(S) * D;
      hipLaunchKernelGGL(k_pool_finish, dim3(unsigned((nel + 255) / 256)), dim3(256), 0, st, partial, pooled, S, T, D, C);
    }
  }
  if (r.h > 0) {
    const int KS = hidden_slices(D);
    ProfileScope ps(MOQE_PK_ROUTE, st);
    dim3 grid((r.h + 15) / 16, (S + 15) / 16, KS);
    if (direct) hipLaunchKernelGGL(k_router_hidden<true>, grid, dim3(256), 0, st, x, r.w1, hidden, S, D, r.h);
    else hipLaunchKernelGGL(k_router_hidden<false>, grid, dim3(256), 0, st, static_cast<const void*>(pooled), r.w1, hidden, S, D, r.h);
    *rf = RouteFeat{hidden, KS, size_t(S) * r.h, r.h};
  } else {
    *rf = RouteFeat{pooled, 0, 0, D};
  }
  return check_launch("route");
}

int32_t launch_route(const void* x, int S, int T, const moqe_router& r, int32_t* idx, float* logits,
                     void* ws, hipStream_t st) {
  RouteFeat rf;
  int32_t rc = route_front(x, nullptr, S, T, r, ws, st, &rf);
  if (rc) return rc;
  ProfileScope ps(MOQE_PK_ROUTE, st);
  launch_logits_argmax(rf.feat, rf.nslices, rf.stride, r, S, rf.Dk, idx, logits, st);
  return check_launch("route");
}

// The router's MLP on feature vectors that are already there (feat: fp32 [S, r.d]); workspace route_ws_bytes(S, 1, r).
int32_t launch_route_features(const float* feat, int S, const moqe_router& r, int32_t* idx, float* logits, void* ws, hipStream_t st) {
  RouteFeat rf{feat, 0, 0, r.d};
  if (r.h > 0) {
    int C, CT;
    pool_shape(S, 1, r.d, &C, &CT);
    float* hidden = reinterpret_cast<float*>(static_cast<uint8_t*>(ws) + align256(size_t(S) * C * r.d * 4) + align256(size_t(S) * r.d * 4));
    const int KS = hidden_slices(r.d);
    ProfileScope ps(MOQE_PK_ROUTE, st);
    hipLaunchKernelGGL(k_router_hidden<false>, dim3((r.h + 15) / 16, (S + 15) / 16, KS), dim3(256), 0, st,
                       static_cast<const void*>(feat), r.w1, hidden, S, r.d, r.h);
    rf = RouteFeat{hidden, KS, size_t(S) * r.h, r.h};
  }
  ProfileScope ps(MOQE_PK_ROUTE, st);
  launch_logits_argmax(rf.feat, rf.nslices, rf.stride, r, S, rf.Dk, idx, logits, st);
  return check_launch("route");
}

// Samples of different lengths (cu_rows: device int32 [S + 1], first row of every sample): the
// workspace is that of route_ws_bytes(S, 2, r).
int32_t launch_route_ragged(const void* x, const int32_t* cu_rows, int S, const moqe_router& r, int32_t* idx, float* logits,
                            void* ws, hipStream_t st) {
  RouteFeat rf;
  int32_t rc = route_front(x, cu_rows, S, 2, r, ws, st, &rf);
  if (rc) return rc;
  ProfileScope ps(MOQE_PK_ROUTE, st);
  launch_logits_argmax(rf.feat, rf.nslices, rf.stride, r, S, rf.Dk, idx, logits, st);
  return check_launch("route");
}

// Router and bucketing together; small batches finish in one work-group.
int32_t launch_route_bucket(const void* x, int S, int T, const moqe_router& r, int32_t* idx, float* logits,
                            int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv_perm, void* ws, hipStream_t st) {
  const int Dk = r.h > 0 ? r.h : r.d;
  if (S > TAIL_MAX_S || S * r.n_experts > TAIL_MAX_PAIRS || size_t(S) * (Dk + 4) > size_t(TAIL_FEAT_FLOATS) ||
      size_t(S) * Dk > size_t(1024) * TAIL_EPT || r.n_experts * (Dk + 4) > TAIL_MAX_W2) {
    int32_t rc = launch_route(x, S, T, r, idx, logits, ws, st);
    if (rc) return rc;
    return launch_bucket(idx, S, r.n_experts, counts, offsets, perm, inv_perm, st);
  }
  RouteFeat rf;
  int32_t rc = route_front(x, nullptr, S, T, r, ws, st, &rf);
  if (rc) return rc;
  if (rf.nslices > 1) {
    // the slices of the hidden layer are best added by many work-groups: separate logits and bucket kernels
    {
      ProfileScope ps(MOQE_PK_ROUTE, st);
      launch_logits_argmax(rf.feat, rf.nslices, rf.stride, r, S, rf.Dk, idx, logits, st);
    }
    return launch_bucket(idx, S, r.n_experts, counts, offsets, perm, inv_perm, st);
  }
  rc = ensure_dynamic_lds(LDSK_ROUTER_TAIL, reinterpret_cast<const void*>(&k_router_tail), TAIL_LDS_BYTES, "route");
  if (rc) return rc;
  ProfileScope ps(MOQE_PK_BUCKET, st);
  hipLaunchKernelGGL(k_router_tail, dim3(1), dim3(256), TAIL_LDS_BYTES, st, rf.feat, rf.nslices, rf.stride, r.b1, r.w2,
                     r.b2, S, rf.Dk, r.n_experts, idx, logits, counts, offsets, perm, inv_perm);
  return check_launch("route+bucket");
}

}  // namespace moqe
