// The CV router model (MoQE Section 3.2): per-pixel three-layer MLP with batch normalisation and ReLU -> three
// squeeze-and-excitation basic blocks (16 / 32 / 64 channels, strides 1 / 2 / 2 in the paper) -> multi-head
// self-attention over the positions of the last feature map -> mean -> linear logits -> top-1.
// The whole model has about 0.1 M parameters and a few hundred MFLOP per batch: plain fp32 arithmetic in
// small LDS-tiled kernels, every sum in a fixed order.
//
//   k_cv_conv       out = [relu] [bn] (conv(in) + bias): 1x1 or 3x3 (padding 1), stride 1 or 2, NHWC, as an
//                   implicit GEMM: 4096 / CT output pixels x CT output channels per work-group (CT = 16, 32, 64),
//                   k in chunks of 32 through LDS, a thread owns 4 pixels x 4 channels
//   k_cv_se_gate    per image: channel means of u, two small linear layers, sigmoid
//   k_cv_se_apply   relu(u * gate + shortcut)
//   k_cv_attn_pool  per image: queries/keys/values, softmax attention per head, mean over positions, output projection
// The logits and the arg-max are the small router's last-layer kernel (route.hip).
#include "moqe_internal.h"

#include <cstring>

namespace moqe {

constexpr float CV_BN_EPS = 1e-5f;
constexpr int CV_MAX_C = 64;             // widest layer
constexpr int CV_MAX_POS = 36;           // positions of the last feature map
constexpr int CV_MAX_DH = 16;            // head width

struct CvConvArgs {
  const void* in;          // [S, hi, wi, cin], bf16 or fp32
  const float* w;          // [cout, taps, cin]
  const float* bias;       // [cout] or NULL
  const float *bn_g, *bn_o, *bn_m, *bn_v;   // all NULL: no normalisation
  float* out;              // [S, ho, wo, cout]
  int in_bf16, S, hi, wi, cin, ho, wo, cout, taps, stride, relu;
};

// CT = output channels per work-group (16, 32 or 64); the work-group takes 4096 / CT output pixels, a thread 4 x 4.
// Both operands are staged four channels at a time (cin is a multiple of 4, so a group of four never straddles a tap).
template <int CT>
__global__ __launch_bounds__(256) void k_cv_conv(const CvConvArgs a) {
  constexpr int PT = 4096 / CT;                    // pixels per work-group
  constexpr int CG = CT / 4;                       // thread groups along the output channels
  constexpr int PI = PT / 32;                      // pixels a thread stages per chunk
  __shared__ __align__(16) float As[32][PT];       // [k][pixel]
  __shared__ __align__(16) float Ws[32][CT];       // [k][output channel]
  const int tid = threadIdx.x;
  const int pg = tid / CG, cg = tid % CG;
  const int M = a.S * a.ho * a.wo, K = a.taps * a.cin;
  const int p0 = blockIdx.x * PT, c0 = blockIdx.y * CT;
  const int pad = a.taps == 9 ? 1 : 0;
  const int kq = tid & 7, r_l = tid >> 3;          // staging: channels 4 kq .. 4 kq + 3 of the chunk, rows r_l + 32 i
  int s_img[PI], s_iy[PI], s_ix[PI];
#pragma unroll
  for (int i = 0; i < PI; ++i) {
    const int px = p0 + r_l + 32 * i;
    if (px < M) {
      const int s = px / (a.ho * a.wo), rem = px - s * (a.ho * a.wo), oy = rem / a.wo, ox = rem - oy * a.wo;
      s_img[i] = s; s_iy[i] = oy * a.stride - pad; s_ix[i] = ox * a.stride - pad;
    } else {
      s_img[i] = -1; s_iy[i] = 0; s_ix[i] = 0;
    }
  }
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

  for (int kc = 0; kc < K; kc += 32) {
    const int k = kc + 4 * kq;
    const bool kin = k < K;                         // K is a multiple of 4: the four channels are in or out together
    const int tap = kin ? k / a.cin : 0, c = kin ? k - tap * a.cin : 0;
    const int kh = a.taps == 9 ? tap / 3 : 0, kw = a.taps == 9 ? tap - kh * 3 : 0;
#pragma unroll
    for (int i = 0; i < PI; ++i) {
      const int iy = s_iy[i] + kh, ix = s_ix[i] + kw;
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (kin && s_img[i] >= 0 && iy >= 0 && iy < a.hi && ix >= 0 && ix < a.wi) {
        const size_t at = ((size_t(s_img[i]) * a.hi + iy) * a.wi + ix) * a.cin + c;
        if (a.in_bf16) {
          const uint2 b = *reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(a.in) + at);
          v = make_float4(__uint_as_float(b.x << 16), __uint_as_float(b.x & 0xffff0000u), __uint_as_float(b.y << 16),
                          __uint_as_float(b.y & 0xffff0000u));
        } else {
          v = *reinterpret_cast<const float4*>(static_cast<const float*>(a.in) + at);
        }
      }
      const int px_l = r_l + 32 * i;
      As[4 * kq + 0][px_l] = v.x; As[4 * kq + 1][px_l] = v.y; As[4 * kq + 2][px_l] = v.z; As[4 * kq + 3][px_l] = v.w;
    }
#pragma unroll
    for (int i = 0; i < (CT + 31) / 32; ++i) {
      const int co_l = r_l + 32 * i;
      if (co_l < CT) {
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (kin && c0 + co_l < a.cout) v = *reinterpret_cast<const float4*>(a.w + size_t(c0 + co_l) * K + k);
        Ws[4 * kq + 0][co_l] = v.x; Ws[4 * kq + 1][co_l] = v.y; Ws[4 * kq + 2][co_l] = v.z; Ws[4 * kq + 3][co_l] = v.w;
      }
    }
    __syncthreads();
#pragma unroll 8
    for (int kk = 0; kk < 32; ++kk) {
      const float4 av = *reinterpret_cast<const float4*>(&As[kk][pg * 4]);
      const float4 wv = *reinterpret_cast<const float4*>(&Ws[kk][cg * 4]);
      const float ar[4] = {av.x, av.y, av.z, av.w}, wr[4] = {wv.x, wv.y, wv.z, wv.w};
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(ar[i], wr[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int co = c0 + cg * 4 + j;
    if (co >= a.cout) continue;
    const float bv = a.bias ? a.bias[co] : 0.f;
    float mean = 0.f, inv = 1.f, gain = 1.f, off = 0.f;
    if (a.bn_g) {
      mean = a.bn_m[co];
      inv = 1.0f / sqrtf(a.bn_v[co] + CV_BN_EPS);
      gain = a.bn_g[co];
      off = a.bn_o[co];
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int px = p0 + pg * 4 + i;
      if (px >= M) continue;
      float v = acc[i][j] + bv;
      if (a.bn_g) v = (v - mean) * inv * gain + off;
      if (a.relu) v = fmaxf(v, 0.f);
      a.out[size_t(px) * a.cout + co] = v;
    }
  }
}

// gate[s][c] = sigmoid(W2 relu(W1 mean_p u[s][p][:] + b1) + b2)[c]; one work-group per image, C <= 64.
__global__ __launch_bounds__(256) void k_cv_se_gate(const float* __restrict__ u, int P, int C, const float* __restrict__ w1,
                                                     const float* __restrict__ b1, const float* __restrict__ w2,
                                                     const float* __restrict__ b2, float* __restrict__ gate) {
  __shared__ float part[4][CV_MAX_C];
  __shared__ float z[CV_MAX_C];
  __shared__ float hid[CV_MAX_C / 4];
  const int s = blockIdx.x, c = threadIdx.x & 63, q = threadIdx.x >> 6, Cr = C / 4;
  float acc = 0.f;
  if (c < C)
    for (int p = q; p < P; p += 4) acc += u[(size_t(s) * P + p) * C + c];
  part[q][c] = acc;
  __syncthreads();
  if (threadIdx.x < C) z[threadIdx.x] = (((part[0][threadIdx.x] + part[1][threadIdx.x]) + part[2][threadIdx.x]) + part[3][threadIdx.x]) / float(P);
  __syncthreads();
  if (threadIdx.x < Cr) {
    float h = b1[threadIdx.x];
    for (int i = 0; i < C; ++i) h = fmaf(w1[threadIdx.x * C + i], z[i], h);
    hid[threadIdx.x] = fmaxf(h, 0.f);
  }
  __syncthreads();
  if (threadIdx.x < C) {
    float g = b2[threadIdx.x];
    for (int i = 0; i < Cr; ++i) g = fmaf(w2[threadIdx.x * Cr + i], hid[i], g);
    gate[size_t(s) * C + threadIdx.x] = 1.0f / (1.0f + expf(-g));
  }
}

__global__ __launch_bounds__(256) void k_cv_se_apply(const float* __restrict__ u, const float* __restrict__ gate,
                                                      const float* __restrict__ shortcut, float* __restrict__ out, int S, int P, int C) {
  const size_t i = size_t(blockIdx.x) * 256 + threadIdx.x, total = size_t(S) * P * C;
  if (i >= total) return;
  const int c = int(i % size_t(C)), s = int(i / (size_t(P) * C));
  out[i] = fmaxf(fmaf(u[i], gate[size_t(s) * C + c], shortcut[i]), 0.f);
}

// One work-group per image: tokens [P, dm] -> queries, keys, values -> per head softmax(q k^T / sqrt(dh)) v -> mean over
// the positions -> output projection -> pooled[s][dm].  (The mean of projected rows is the projection of the mean row.)
__global__ __launch_bounds__(256) void k_cv_attn_pool(const float* __restrict__ x, int P, int dm, int heads, const float* __restrict__ wqkv,
                                                       const float* __restrict__ bqkv, const float* __restrict__ wo,
                                                       const float* __restrict__ bo, float* __restrict__ pooled) {
  extern __shared__ __align__(16) float cv_lds[];
  float* tok = cv_lds;                       // [P][dm]
  float* qkv = tok + P * dm;                 // [P][3 dm]
  float* att = qkv + P * 3 * dm;             // [P][dm]
  float* mean_att = att + P * dm;            // [dm]
  const int s = blockIdx.x, tid = threadIdx.x, dh = dm / heads;
  const float scale = 1.0f / sqrtf(float(dh));
  for (int i = tid; i < P * dm; i += 256) tok[i] = x[size_t(s) * P * dm + i];
  __syncthreads();
  for (int o = tid; o < P * 3 * dm; o += 256) {
    const int p = o / (3 * dm), j = o - p * 3 * dm;
    float v = bqkv[j];
    for (int c = 0; c < dm; ++c) v = fmaf(tok[p * dm + c], wqkv[j * dm + c], v);
    qkv[o] = v;
  }
  __syncthreads();
  for (int item = tid; item < heads * P; item += 256) {
    const int h = item / P, q = item - h * P;
    const float* qv = qkv + q * 3 * dm + h * dh;
    float mx = -INFINITY;
    for (int k = 0; k < P; ++k) {
      const float* kv = qkv + k * 3 * dm + dm + h * dh;
      float d = 0.f;
      for (int c = 0; c < dh; ++c) d = fmaf(qv[c], kv[c], d);
      mx = fmaxf(mx, d * scale);
    }
    float sum = 0.f, acc[CV_MAX_DH];
#pragma unroll
    for (int c = 0; c < CV_MAX_DH; ++c) acc[c] = 0.f;
    for (int k = 0; k < P; ++k) {
      const float* kv = qkv + k * 3 * dm + dm + h * dh;
      const float* vv = qkv + k * 3 * dm + 2 * dm + h * dh;
      float d = 0.f;
      for (int c = 0; c < dh; ++c) d = fmaf(qv[c], kv[c], d);
      const float e = expf(d * scale - mx);
      sum += e;
#pragma unroll
      for (int c = 0; c < CV_MAX_DH; ++c)
        if (c < dh) acc[c] = fmaf(e, vv[c], acc[c]);
    }
    const float inv = 1.0f / sum;
#pragma unroll
    for (int c = 0; c < CV_MAX_DH; ++c)
      if (c < dh) att[q * dm + h * dh + c] = acc[c] * inv;
  }
  __syncthreads();
  if (tid < dm) {
    float m = 0.f;
    for (int p = 0; p < P; ++p) m += att[p * dm + tid];
    mean_att[tid] = m / float(P);
  }
  __syncthreads();
  if (tid < dm) {
    float v = bo[tid];
    for (int c = 0; c < dm; ++c) v = fmaf(mean_att[c], wo[tid * dm + c], v);
    pooled[size_t(s) * dm + tid] = v;
  }
}

// ---- host side -------------------------------------------------------------------------------------------------
namespace {
int out_size(int n, int taps, int stride) { return taps == 9 ? (n + 2 - 3) / stride + 1 : (n - 1) / stride + 1; }

struct CvLayout {
  size_t buf[4], gate, pooled, head, total;
  int h[4], w[4];            // feature-map size entering stage 0, 1, 2 and leaving stage 2
};

CvLayout cv_layout(int S, int h, int w, const moqe_cv_router& r) {
  CvLayout L;
  L.h[0] = h; L.w[0] = w;
  for (int i = 0; i < 3; ++i) {
    L.h[i + 1] = out_size(L.h[i], 9, r.stage[i].stride);
    L.w[i + 1] = out_size(L.w[i], 9, r.stage[i].stride);
  }
  size_t o = 0;
  const size_t big = align256(size_t(S) * h * w * CV_MAX_C * 4);        // any feature map fits
  for (int i = 0; i < 4; ++i) { L.buf[i] = o; o += big; }
  L.gate = o;   o += align256(size_t(S) * CV_MAX_C * 4);
  L.pooled = o; o += align256(size_t(S) * CV_MAX_C * 4);
  moqe_router head{nullptr, nullptr, r.w_out, r.b_out, r.stage[2].cout, 0, r.n_experts};
  L.head = o;   o += align256(route_ws_bytes(S, 1, head));
  L.total = o;
  return L;
}

int32_t conv(const void* in, bool in_bf16, const float* w, const float* bias, const moqe_bn* bn, float* out, int S, int hi, int wi, int cin,
             int cout, int taps, int stride, bool relu, hipStream_t st) {
  CvConvArgs a;
  memset(&a, 0, sizeof(a));
  a.in = in; a.in_bf16 = in_bf16 ? 1 : 0; a.w = w; a.bias = bias; a.out = out;
  if (bn) { a.bn_g = bn->gain; a.bn_o = bn->offset; a.bn_m = bn->mean; a.bn_v = bn->var; }
  a.S = S; a.hi = hi; a.wi = wi; a.cin = cin; a.cout = cout; a.taps = taps; a.stride = stride; a.relu = relu ? 1 : 0;
  a.ho = out_size(hi, taps, stride); a.wo = out_size(wi, taps, stride);
  const long M = long(S) * a.ho * a.wo;
  ProfileScope ps(MOQE_PK_ROUTE, st);
  if (cout <= 16) hipLaunchKernelGGL(k_cv_conv<16>, dim3(unsigned((M + 255) / 256), (cout + 15) / 16), dim3(256), 0, st, a);
  else if (cout <= 32) hipLaunchKernelGGL(k_cv_conv<32>, dim3(unsigned((M + 127) / 128), (cout + 31) / 32), dim3(256), 0, st, a);
  else hipLaunchKernelGGL(k_cv_conv<64>, dim3(unsigned((M + 63) / 64), (cout + 63) / 64), dim3(256), 0, st, a);
  return check_launch("route_cv(convolution)");
}

bool bn_ok(const moqe_bn& b) { return b.gain && b.offset && b.mean && b.var; }
}  // namespace

int32_t check_cv_router(const moqe_cv_router* r, int h, int w, const char* who) {
  if (!r) return set_error(MOQE_E_NULL, "%s: router is NULL", who);
  if (r->n_experts < 1 || r->n_experts > MOQE_MAX_EXPERTS) return set_error(MOQE_E_SHAPE, "%s: n_experts=%d", who, r->n_experts);
  if (r->c_in <= 0 || r->c_in % 4 || h <= 0 || w <= 0)
    return set_error(MOQE_E_SHAPE, "%s: image %d x %d x %d (channels a multiple of 4)", who, h, w, r->c_in);
  for (int i = 0; i < 3; ++i) {
    if (!r->mlp_w[i] || !r->mlp_b[i] || !bn_ok(r->mlp_bn[i])) return set_error(MOQE_E_NULL, "%s: MLP layer %d has a NULL parameter", who, i);
    if (r->mlp_n[i] <= 0 || r->mlp_n[i] > CV_MAX_C || r->mlp_n[i] % 4)
      return set_error(MOQE_E_SHAPE, "%s: MLP width %d must be a multiple of 4, at most %d", who, r->mlp_n[i], CV_MAX_C);
    const moqe_cv_stage& s = r->stage[i];
    const int cin = i == 0 ? r->mlp_n[2] : r->stage[i - 1].cout;
    if (!s.conv_a || !s.conv_b || !bn_ok(s.bn_a) || !bn_ok(s.bn_b) || !s.se_w1 || !s.se_b1 || !s.se_w2 || !s.se_b2)
      return set_error(MOQE_E_NULL, "%s: stage %d has a NULL parameter", who, i);
    if (s.cout <= 0 || s.cout > CV_MAX_C || s.cout % 4 || (s.stride != 1 && s.stride != 2))
      return set_error(MOQE_E_SHAPE, "%s: stage %d: %d channels (multiple of 4, at most %d), stride %d (1 or 2)", who, i, s.cout, CV_MAX_C, s.stride);
    if (!s.short_w && (s.stride != 1 || s.cout != cin))
      return set_error(MOQE_E_SHAPE, "%s: stage %d changes stride or width and needs a shortcut convolution", who, i);
    if (s.short_w && !bn_ok(s.short_bn)) return set_error(MOQE_E_NULL, "%s: stage %d: the shortcut's batch norm is NULL", who, i);
  }
  if (!r->wqkv || !r->bqkv || !r->wo || !r->bo || !r->w_out) return set_error(MOQE_E_NULL, "%s: an attention or output parameter is NULL", who);
  for (int i = 0; i < 3; ++i) {
    const void* mats[] = {r->mlp_w[i], r->stage[i].conv_a, r->stage[i].conv_b, r->stage[i].short_w};
    for (const void* m : mats)
      if (reinterpret_cast<uintptr_t>(m) % 16) return set_error(MOQE_E_SHAPE, "%s: weight matrices and filters must be 16-byte aligned", who);
  }
  const int dm = r->stage[2].cout;
  if (r->n_heads <= 0 || dm % r->n_heads || dm / r->n_heads > CV_MAX_DH || dm % 8)
    return set_error(MOQE_E_SHAPE, "%s: %d heads on %d channels (head width at most %d, channels a multiple of 8)", who, r->n_heads, dm, CV_MAX_DH);
  if (reinterpret_cast<uintptr_t>(r->w_out) % 16) return set_error(MOQE_E_SHAPE, "%s: w_out must be 16-byte aligned", who);
  int hh = h, ww = w;
  for (int i = 0; i < 3; ++i) { hh = out_size(hh, 9, r->stage[i].stride); ww = out_size(ww, 9, r->stage[i].stride); }
  if (hh * ww > CV_MAX_POS) return set_error(MOQE_E_SHAPE, "%s: the last feature map has %d positions, at most %d", who, hh * ww, CV_MAX_POS);
  return MOQE_OK;
}

size_t route_cv_ws_bytes(int S, int h, int w, const moqe_cv_router& r) { return cv_layout(S, h, w, r).total; }

int32_t launch_route_cv(const void* x, int S, int h, int w, const moqe_cv_router& r, int32_t* idx, float* logits, void* ws, hipStream_t st) {
  const CvLayout L = cv_layout(S, h, w, r);
  uint8_t* p = static_cast<uint8_t*>(ws);
  float* buf[4];
  for (int i = 0; i < 4; ++i) buf[i] = reinterpret_cast<float*>(p + L.buf[i]);
  float* gate = reinterpret_cast<float*>(p + L.gate);
  float* pooled = reinterpret_cast<float*>(p + L.pooled);
  int32_t rc;
  // per-pixel MLP: x -> buf0 -> buf1 -> buf0
  if ((rc = conv(x, true, r.mlp_w[0], r.mlp_b[0], &r.mlp_bn[0], buf[0], S, h, w, r.c_in, r.mlp_n[0], 1, 1, true, st))) return rc;
  if ((rc = conv(buf[0], false, r.mlp_w[1], r.mlp_b[1], &r.mlp_bn[1], buf[1], S, h, w, r.mlp_n[0], r.mlp_n[1], 1, 1, true, st))) return rc;
  if ((rc = conv(buf[1], false, r.mlp_w[2], r.mlp_b[2], &r.mlp_bn[2], buf[0], S, h, w, r.mlp_n[1], r.mlp_n[2], 1, 1, true, st))) return rc;
  float* cur = buf[0];                      // the stage's input
  int cin = r.mlp_n[2];
  for (int i = 0; i < 3; ++i) {
    const moqe_cv_stage& sg = r.stage[i];
    float* free_buf[3];
    int nf = 0;
    for (int b = 0; b < 4; ++b)
      if (buf[b] != cur) free_buf[nf++] = buf[b];
    float *a = free_buf[0], *u = free_buf[1], *sc = free_buf[2];
    const int hi = L.h[i], wi = L.w[i], ho = L.h[i + 1], wo = L.w[i + 1], P = ho * wo;
    if ((rc = conv(cur, false, sg.conv_a, nullptr, &sg.bn_a, a, S, hi, wi, cin, sg.cout, 9, sg.stride, true, st))) return rc;
    if ((rc = conv(a, false, sg.conv_b, nullptr, &sg.bn_b, u, S, ho, wo, sg.cout, sg.cout, 9, 1, false, st))) return rc;
    const float* shortcut = cur;
    if (sg.short_w) {
      if ((rc = conv(cur, false, sg.short_w, nullptr, &sg.short_bn, sc, S, hi, wi, cin, sg.cout, 1, sg.stride, false, st))) return rc;
      shortcut = sc;
    }
    {
      ProfileScope ps(MOQE_PK_ROUTE, st);
      hipLaunchKernelGGL(k_cv_se_gate, dim3(S), dim3(256), 0, st, u, P, sg.cout, sg.se_w1, sg.se_b1, sg.se_w2, sg.se_b2, gate);
      const size_t total = size_t(S) * P * sg.cout;
      hipLaunchKernelGGL(k_cv_se_apply, dim3(unsigned((total + 255) / 256)), dim3(256), 0, st, u, gate, shortcut, a, S, P, sg.cout);
      if ((rc = check_launch("route_cv(squeeze and excitation)"))) return rc;
    }
    cur = a;                                 // a is free again once u has been computed from it
    cin = sg.cout;
  }
  const int P = L.h[3] * L.w[3], dm = cin;
  {
    ProfileScope ps(MOQE_PK_ROUTE, st);
    const size_t lds = size_t(P) * 5 * dm * 4 + size_t(dm) * 4;
    hipLaunchKernelGGL(k_cv_attn_pool, dim3(S), dim3(256), lds, st, cur, P, dm, r.n_heads, r.wqkv, r.bqkv, r.wo, r.bo, pooled);
    if ((rc = check_launch("route_cv(attention)"))) return rc;
  }
  moqe_router head{nullptr, nullptr, r.w_out, r.b_out, dm, 0, r.n_experts};
  return launch_route_features(pooled, S, head, idx, logits, p + L.head, st);
}

}  // namespace moqe
