// The NLP router model (MoQE Section 3.2): token vectors -> projection -> one post-norm Transformer encoder
// layer -> a second self-attention module (residual, LayerNorm) -> mean over the tokens -> MLP head -> top-1.
// The paper fixes the order of the stages, not their sizes; widths come with the parameter struct.
//
// Kernels of this file:
//   k_to_bf16      fp32 parameters -> bf16 copies (one launch for all matrices)
//   k_lin          C = A W^T + bias [+ residual] [ReLU] on the bf16 matrix cores, fp32 accumulation; A and W
//                  are bf16, C is written as fp32 and/or bf16
//   k_attention    softmax(Q K^T / sqrt(dh)) V per (sample, head) in fp32 on the fp32 matrix cores, one wave per
//                  32 queries, keys streamed in tiles of 16 with a running maximum and sum (no LDS, no barrier)
//   k_layer_norm   per row, fp32, biased variance; writes fp32 and/or bf16
//   k_pool_f32     mean over a sample's tokens, added in token order
// The MLP head on the pooled vector is the small router of route.hip.
#include "qgemm_device.h"

#include <algorithm>
#include <cstring>

namespace moqe {

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

static __device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {   // round to nearest even, a in the low half
  const f32x2_t v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// ---- parameters to bf16 ---------------------------------------------------------------------------------
constexpr int CVT_MAX_SEG = 8;
struct CvtSegs {
  const float* src[CVT_MAX_SEG];
  uint16_t* dst[CVT_MAX_SEG];
  long long first[CVT_MAX_SEG + 1];      // first[i] = index (in units of 4 elements) where segment i starts
  int n;
};

__global__ __launch_bounds__(256) void k_to_bf16(const CvtSegs sg) {
  const long long total = sg.first[sg.n];
  for (long long i = blockIdx.x * 256ll + threadIdx.x; i < total; i += gridDim.x * 256ll) {
    int s = 0;
#pragma unroll
    for (int j = 1; j < CVT_MAX_SEG; ++j) s += (j < sg.n && i >= sg.first[j]) ? 1 : 0;
    const long long e = (i - sg.first[s]) * 4;
    const float4 v = *reinterpret_cast<const float4*>(sg.src[s] + e);
    uint2 o;
    o.x = pack_bf16x2(v.x, v.y);
    o.y = pack_bf16x2(v.z, v.w);
    *reinterpret_cast<uint2*>(sg.dst[s] + e) = o;
  }
}

// ---- C = A W^T ---------------------------------------------------------------------------------------------
// Work-group tile 128 rows x 128 columns, k-tiles of 64; 4 waves as 2 x 2, a wave owns 64 x 64 (4 x 4
// matrix-core blocks).  Both operand tiles go through LDS (rows of 128 bytes, 16-byte units XOR-swizzled by
// the row so that operand reads are conflict free), double-buffered, one barrier per k-tile.
constexpr int LBM = 128, LBN = 128, LBK = 64;
constexpr int L_TILE_BYTES = LBM * LBK * 2;                  // one operand tile
constexpr int L_LDS_BYTES = 4 * L_TILE_BYTES;               // A and W, two buffers each

struct LinArgs {
  const uint16_t* a;      // bf16 [M, k]
  const uint16_t* w;      // bf16 [n, k]
  const float* bias;      // [n] or NULL
  const float* residual;  // fp32 [M, n] or NULL, added after the bias
  float* c32;             // fp32 [M, n] or NULL
  uint16_t* c16;          // bf16 [M, n] or NULL
  int M, n, k;
  int relu;
  int ksplit;             // > 1: work-group z multiplies its share of the k-tiles and stores the raw sums to part[z]
  float* part;            // fp32 [ksplit, M, n]
};

__global__ __launch_bounds__(256, 2) void k_lin(const LinArgs la) {
  extern __shared__ __align__(16) uint8_t lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 15, lq = lane >> 4;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = blockIdx.y * LBM, n0 = blockIdx.x * LBN;
  const int KT = la.k / LBK;
  const int kt0 = int(blockIdx.z) * KT / la.ksplit, kt1 = (int(blockIdx.z) + 1) * KT / la.ksplit;   // this work-group's k-tiles
  // staging: a tile is 128 rows x 8 units of 16 bytes = 1024 units, 4 per thread per operand
  const int s_unit = tid & 7, s_row0 = tid >> 3;             // rows s_row0 + 32 i
  const uint16_t* a_src[4];
  const uint16_t* w_src[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = s_row0 + 32 * i;
    a_src[i] = la.a + size_t(min(m0 + row, la.M - 1)) * la.k + s_unit * 8;    // rows past the end repeat the last row
    w_src[i] = la.w + size_t(n0 + row) * la.k + s_unit * 8;                    // n is a multiple of the tile
  }
  // two register stages: the loads of k-tile j are issued two iterations before they are written to LDS
  u32x4 a_reg[2][4], w_reg[2][4];
  auto fetch = [&](int set, int kt) {
    const int ko = min(kt, KT - 1) * LBK;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      a_reg[set][i] = *reinterpret_cast<const u32x4*>(a_src[i] + ko);
      w_reg[set][i] = *reinterpret_cast<const u32x4*>(w_src[i] + ko);
    }
  };
  auto store = [&](int set, int buf) {
    uint8_t* ab = lds + buf * 2 * L_TILE_BYTES;
    uint8_t* wb = ab + L_TILE_BYTES;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = s_row0 + 32 * i;
      const int off = row * 128 + ((s_unit ^ (row & 7)) * 16);
      *reinterpret_cast<u32x4*>(ab + off) = a_reg[set][i];
      *reinterpret_cast<u32x4*>(wb + off) = w_reg[set][i];
    }
  };
  f32x4 acc[4][4];
#pragma unroll
  for (int mb = 0; mb < 4; ++mb)
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) acc[mb][nb] = f32x4{0.f, 0.f, 0.f, 0.f};

  auto compute = [&](int buf) {
    const uint8_t* ab = lds + buf * 2 * L_TILE_BYTES + (wm * 64 + lr) * 128;
    const uint8_t* wb = lds + buf * 2 * L_TILE_BYTES + L_TILE_BYTES + (wn * 64 + lr) * 128;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int uo = ((j * 4 + lq) ^ (lr & 7)) * 16;        // rows lr + 16 b share lr & 7
      bf16x8 af[4];
      u32x4 wf[4];
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        af[b] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(ab + b * 16 * 128 + uo));
        wf[b] = *reinterpret_cast<const u32x4*>(wb + b * 16 * 128 + uo);
      }
      // the weights are the FIRST operand: the result block is C^T, a lane then holds four neighbouring columns of one row
#pragma unroll
      for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int nb = 0; nb < 4; ++nb) acc[mb][nb] = mfma_bf16(wf[nb], af[mb], acc[mb][nb]);
    }
  };
  // k-tile kt0 + j: register set j & 1, LDS buffer j & 1
  fetch(0, kt0);
  store(0, 0);
  fetch(1, kt0 + 1);
  fetch(0, kt0 + 2);
  __syncthreads();
  int kt = kt0;
  for (; kt + 2 <= kt1; kt += 2) {
    compute(0);
    store(1, 1);               // k-tile kt + 1; that buffer was last read in the iteration before
    fetch(1, kt + 3);
    __syncthreads();
    compute(1);
    store(0, 0);               // k-tile kt + 2
    fetch(0, kt + 4);
    __syncthreads();
  }
  if (kt < kt1) compute(0);    // an odd number of k-tiles: the last one sits in buffer 0
  // ---- epilogue: lane (lr, lq) holds row m0 + wm*64 + mb*16 + lr, columns n0 + wn*64 + nb*16 + 4 lq .. + 3
#pragma unroll
  for (int mb = 0; mb < 4; ++mb) {
    const int row = m0 + wm * 64 + mb * 16 + lr;
    if (row >= la.M) continue;
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) {
      const int col = n0 + wn * 64 + nb * 16 + 4 * lq;
      const size_t o = size_t(row) * la.n + col;
      float4 v = make_float4(acc[mb][nb][0], acc[mb][nb][1], acc[mb][nb][2], acc[mb][nb][3]);
      if (la.ksplit > 1) {
        *reinterpret_cast<float4*>(la.part + size_t(blockIdx.z) * la.M * la.n + o) = v;
        continue;
      }
      if (la.bias) { const float4 t = *reinterpret_cast<const float4*>(la.bias + col); v.x += t.x; v.y += t.y; v.z += t.z; v.w += t.w; }
      if (la.residual) { const float4 t = *reinterpret_cast<const float4*>(la.residual + o); v.x += t.x; v.y += t.y; v.z += t.z; v.w += t.w; }
      if (la.relu) { v.x = fmaxf(v.x, 0.f); v.y = fmaxf(v.y, 0.f); v.z = fmaxf(v.z, 0.f); v.w = fmaxf(v.w, 0.f); }
      if (la.c32) *reinterpret_cast<float4*>(la.c32 + o) = v;
      if (la.c16) {
        uint2 h;
        h.x = pack_bf16x2(v.x, v.y);
        h.y = pack_bf16x2(v.z, v.w);
        *reinterpret_cast<uint2*>(la.c16 + o) = h;
      }
    }
  }
}

// Split launches: C = (sum over the k-shares, in order) + bias [+ residual] [ReLU]; four columns per thread.
__global__ __launch_bounds__(256) void k_lin_finish(const LinArgs la) {
  const size_t i = (size_t(blockIdx.x) * 256 + threadIdx.x) * 4, total = size_t(la.M) * la.n;
  if (i >= total) return;
  float4 v = *reinterpret_cast<const float4*>(la.part + i);
  for (int z = 1; z < la.ksplit; ++z) {
    const float4 t = *reinterpret_cast<const float4*>(la.part + size_t(z) * total + i);
    v.x += t.x; v.y += t.y; v.z += t.z; v.w += t.w;
  }
  const int col = int(i % size_t(la.n));
  if (la.bias) { const float4 t = *reinterpret_cast<const float4*>(la.bias + col); v.x += t.x; v.y += t.y; v.z += t.z; v.w += t.w; }
  if (la.residual) { const float4 t = *reinterpret_cast<const float4*>(la.residual + i); v.x += t.x; v.y += t.y; v.z += t.z; v.w += t.w; }
  if (la.relu) { v.x = fmaxf(v.x, 0.f); v.y = fmaxf(v.y, 0.f); v.z = fmaxf(v.z, 0.f); v.w = fmaxf(v.w, 0.f); }
  if (la.c32) *reinterpret_cast<float4*>(la.c32 + i) = v;
  if (la.c16) {
    uint2 o;
    o.x = pack_bf16x2(v.x, v.y);
    o.y = pack_bf16x2(v.z, v.w);
    *reinterpret_cast<uint2*>(la.c16 + i) = o;
  }
}

// ---- attention -----------------------------------------------------------------------------------------------
// qkv: fp32 [S*T, 3*dm] (queries, keys, values); out: bf16 [S*T, dm].  One wave = 16 queries of one head.
// Scores of a 16-key tile are computed TRANSPOSED (keys x queries), so that a lane's four accumulator values are
// four keys of ITS query (lane % 16): the softmax of a query then needs its own lane's values and those of the three
// lanes 16, 32, 48 further on, and the probabilities already sit where the second product wants them.
// The sum over the head's dimensions and the sum over a tile's keys are order-free, which lets lane group q
// (= lane / 16) take the contiguous quarter q of a row (dimensions) and the keys 4q .. 4q+3 of a tile.
// A wave takes QT tiles of 16 queries against the same stream of key tiles (each key / value tile is loaded once per
// wave and multiplied QT times), and the next key tile's loads are issued before the current tile's arithmetic.
constexpr int ATT_QT = 1;

template <int DH>
__global__ __launch_bounds__(256) void k_attention(const float* __restrict__ qkv, uint16_t* __restrict__ out, int S, int T, int dm,
                                                    float scale) {
  constexpr int QS = DH / 4;            // dimensions per lane group = matrix-core steps of the first product
  constexpr int CB = DH / 16;           // 16-column blocks of the output
  constexpr int QT = ATT_QT;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int lr = lane & 15, lq = lane >> 4;
  const int q0 = (blockIdx.x * 4 + wave) * 16 * QT;
  const int head = blockIdx.y, s = blockIdx.z;
  if (q0 >= T) return;                                      // uniform over the wave; the kernel has no barrier
  const size_t ld = size_t(3) * dm;
  const float* base = qkv + size_t(s) * T * ld + head * DH;
  // queries: lane (lr, lq) holds Q[q0 + 16 t + lr][lq*QS .. +QS) of query tile t
  float qf[QT][QS];
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    const float* qp = base + size_t(min(q0 + 16 * t + lr, T - 1)) * ld + lq * QS;
#pragma unroll
    for (int i = 0; i < QS; i += 4) {
      const float4 v = *reinterpret_cast<const float4*>(qp + i);
      qf[t][i] = v.x * scale; qf[t][i + 1] = v.y * scale; qf[t][i + 2] = v.z * scale; qf[t][i + 3] = v.w * scale;
    }
  }
  f32x4 o[QT][CB];
  float m_run[QT], l_run[QT];
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    m_run[t] = -INFINITY; l_run[t] = 0.f;
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) o[t][cb] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  // key tile k0: lane (lr, lq) holds K[k0 + lr][lq*QS .. +QS) and V[k0 + 4 lq + r][16 cb + lr]; rows past T repeat row T - 1
  float kf[QS], vf[4][CB];
  auto load_tile = [&](int k0) {
    const float* kp = base + dm + size_t(min(k0 + lr, T - 1)) * ld + lq * QS;
#pragma unroll
    for (int i = 0; i < QS; i += 4) {
      const float4 v = *reinterpret_cast<const float4*>(kp + i);
      kf[i] = v.x; kf[i + 1] = v.y; kf[i + 2] = v.z; kf[i + 3] = v.w;
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float* vp = base + 2 * dm + size_t(min(k0 + 4 * lq + r, T - 1)) * ld + lr;
#pragma unroll
      for (int cb = 0; cb < CB; ++cb) vf[r][cb] = vp[cb * 16];
    }
  };
  load_tile(0);
  for (int k0 = 0; k0 < T; k0 += 16) {
    float kc[QS], vc[4][CB];
#pragma unroll
    for (int i = 0; i < QS; ++i) kc[i] = kf[i];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int cb = 0; cb < CB; ++cb) vc[r][cb] = vf[r][cb];
    load_tile(k0 + 16);                                     // clamped rows: valid addresses also past the last tile
#pragma unroll
    for (int t = 0; t < QT; ++t) {
      if (q0 + 16 * t >= T) continue;                       // uniform: this query tile does not exist
      // ---- scores^T[key][query] for keys k0 .. k0+15
      f32x4 sc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int i = 0; i < QS; ++i) sc = __builtin_amdgcn_mfma_f32_16x16x4f32(kc[i], qf[t][i], sc, 0, 0, 0);
      // lane (lr, lq) now holds the scores of query q0 + 16 t + lr against keys k0 + 4 lq + r
      float p[4];
      float tmax = -INFINITY;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const bool live = k0 + 4 * lq + r < T;
        p[r] = live ? sc[r] : -INFINITY;
        tmax = fmaxf(tmax, p[r]);
      }
      tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
      const float m_new = fmaxf(m_run[t], tmax);            // finite: key k0 itself is live
      const float alpha = __expf(m_run[t] - m_new);         // exp(-inf) = 0 on the first tile
      float tsum = 0.f;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        p[r] = __expf(p[r] - m_new);
        tsum += p[r];
      }
      tsum += __shfl_xor(tsum, 16);
      tsum += __shfl_xor(tsum, 32);
      l_run[t] = l_run[t] * alpha + tsum;
      m_run[t] = m_new;
      // ---- out^T[c][query] += V^T P^T: step r multiplies the keys k0 + 4 kk + r (kk = lane group) of the tile
#pragma unroll
      for (int cb = 0; cb < CB; ++cb) {
#pragma unroll
        for (int r = 0; r < 4; ++r) o[t][cb][r] *= alpha;
      }
#pragma unroll
      for (int r = 0; r < 4; ++r)                           // dead keys have p = 0
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) o[t][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(vc[r][cb], p[r], o[t][cb], 0, 0, 0);
    }
  }
  // lane (lr, lq) holds out[q0 + 16 t + lr][16 cb + 4 lq + r]
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    if (q0 + 16 * t + lr < T) {
      const float inv = 1.f / l_run[t];
      uint16_t* op = out + (size_t(s) * T + q0 + 16 * t + lr) * dm + head * DH + 4 * lq;
#pragma unroll
      for (int cb = 0; cb < CB; ++cb) {
        uint2 v;
        v.x = pack_bf16x2(o[t][cb][0] * inv, o[t][cb][1] * inv);
        v.y = pack_bf16x2(o[t][cb][2] * inv, o[t][cb][3] * inv);
        *reinterpret_cast<uint2*>(op + cb * 16) = v;
      }
    }
  }
}

// ---- LayerNorm -----------------------------------------------------------------------------------------------
static __device__ __forceinline__ float wave_sum_f(float v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d);
  return v;
}

constexpr int LN_MAX_PER_LANE = 32;      // rows of up to 2048 elements
__global__ __launch_bounds__(256) void k_layer_norm(const float* __restrict__ x, const float* __restrict__ g, const float* __restrict__ b,
                                                     int M, int n, float* __restrict__ y32, uint16_t* __restrict__ y16) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= M) return;
  const float* xr = x + size_t(row) * n;
  float v[LN_MAX_PER_LANE];
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < LN_MAX_PER_LANE; ++i) {
    const int c = lane + 64 * i;
    v[i] = c < n ? xr[c] : 0.f;
    sum += v[i];
  }
  const float mu = wave_sum_f(sum) / float(n);
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < LN_MAX_PER_LANE; ++i) {
    const int c = lane + 64 * i;
    const float d = c < n ? v[i] - mu : 0.f;
    sq += d * d;
  }
  const float rstd = 1.0f / sqrtf(wave_sum_f(sq) / float(n) + 1e-5f);
#pragma unroll
  for (int i = 0; i < LN_MAX_PER_LANE; ++i) {
    const int c = lane + 64 * i;
    if (c < n) {
      const float r = (v[i] - mu) * rstd * g[c] + b[c];
      if (y32) y32[size_t(row) * n + c] = r;
      if (y16) y16[size_t(row) * n + c] = float_to_bf16_rne(r);
    }
  }
}

// pooled[s][c] = (sum over the sample's tokens of z[s][t][c]) / T.  A work-group takes 64 columns of one sample; wave w
// adds the tokens w, w + 16, ... in order, the 16 partial sums are added in wave order.
__global__ __launch_bounds__(1024) void k_pool_f32(const float* __restrict__ z, float* __restrict__ pooled, int S, int T, int n) {
  __shared__ float part[16][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int s = blockIdx.y, c = blockIdx.x * 64 + lane;
  float acc = 0.f;
  if (c < n) {
    const float* p = z + size_t(s) * T * n + c;
    for (int t = wave; t < T; t += 16) acc += p[size_t(t) * n];
  }
  part[wave][lane] = acc;
  __syncthreads();
  if (wave == 0 && c < n) {
    float v = part[0][lane];
#pragma unroll
    for (int w = 1; w < 16; ++w) v += part[w][lane];
    pooled[size_t(s) * n + c] = __fdiv_rn(v, float(T));
  }
}

// ---- host side -------------------------------------------------------------------------------------------------
namespace {
constexpr int LIN_SPLIT_MAX = 16;            // most k-shares of one product
constexpr int LIN_SPLIT_MAX_ROWS = 512;      // products with more rows fill the chip without splitting

struct NlpLayout {
  size_t w_in, wqkv1, wo1, wff1, wff2, wqkv2, wo2;          // bf16 parameter copies
  size_t t32a, t32b, t32c, t16a, t16b, qkv, hid, part, pooled, head, total;
};

NlpLayout nlp_layout(int S, int T, const moqe_nlp_router& r) {
  NlpLayout L;
  const size_t M = size_t(S) * T, dm = r.dm;
  size_t o = 0;
  auto take = [&](size_t bytes) { const size_t at = o; o += align256(bytes); return at; };
  L.w_in = take(dm * r.d * 2);
  L.wqkv1 = take(3 * dm * dm * 2);
  L.wo1 = take(dm * dm * 2);
  L.wff1 = take(size_t(r.d_ff) * dm * 2);
  L.wff2 = take(size_t(r.d_ff) * dm * 2);
  L.wqkv2 = take(3 * dm * dm * 2);
  L.wo2 = take(dm * dm * 2);
  L.t32a = take(M * dm * 4);
  L.t32b = take(M * dm * 4);
  L.t32c = take(M * dm * 4);
  L.t16a = take(M * dm * 2);
  L.t16b = take(M * dm * 2);
  L.qkv = take(M * 3 * dm * 4);
  L.hid = take(M * size_t(r.d_ff) * 2);
  const size_t widest = std::max<size_t>(3 * dm, size_t(r.d_ff));
  L.part = take(M <= size_t(LIN_SPLIT_MAX_ROWS) ? size_t(LIN_SPLIT_MAX) * M * widest * 4 : 0);   // k-shares of launches with few rows
  L.pooled = take(size_t(S) * dm * 4);
  L.head = take(route_ws_bytes(S, 1, r.head));
  L.total = o;
  return L;
}

int32_t lin(const uint16_t* a, const uint16_t* w, const float* bias, const float* residual, float* c32, uint16_t* c16, int M, int n,
            int k, bool relu, float* part, hipStream_t st) {
  LinArgs la{a, w, bias, residual, c32, c16, M, n, k, relu ? 1 : 0, 1, part};
  const int wgs = (n / LBN) * ((M + LBM - 1) / LBM), KT = k / LBK;
  // few rows: the k-tiles are shared out over more work-groups (at least two tiles each), summed by a second launch
  if (M <= LIN_SPLIT_MAX_ROWS)
    while (wgs * la.ksplit < 96 && la.ksplit * 4 <= KT && la.ksplit < LIN_SPLIT_MAX) la.ksplit *= 2;
  ProfileScope ps(MOQE_PK_ROUTE, st);
  hipLaunchKernelGGL(k_lin, dim3(n / LBN, (M + LBM - 1) / LBM, la.ksplit), dim3(256), L_LDS_BYTES, st, la);
  if (la.ksplit > 1)
    hipLaunchKernelGGL(k_lin_finish, dim3(unsigned((size_t(M) * n / 4 + 255) / 256)), dim3(256), 0, st, la);
  return check_launch("route_nlp(linear)");
}

int32_t attention(const float* qkv, uint16_t* out, int S, int T, int dm, int heads, hipStream_t st) {
  const int dh = dm / heads;
  const float scale = 1.0f / sqrtf(float(dh));
  const dim3 grid((T + 64 * ATT_QT - 1) / (64 * ATT_QT), heads, S);
  ProfileScope ps(MOQE_PK_ROUTE, st);
  switch (dh) {
    case 16:  hipLaunchKernelGGL(k_attention<16>, grid, dim3(256), 0, st, qkv, out, S, T, dm, scale); break;
    case 32:  hipLaunchKernelGGL(k_attention<32>, grid, dim3(256), 0, st, qkv, out, S, T, dm, scale); break;
    case 64:  hipLaunchKernelGGL(k_attention<64>, grid, dim3(256), 0, st, qkv, out, S, T, dm, scale); break;
    default:  hipLaunchKernelGGL(k_attention<128>, grid, dim3(256), 0, st, qkv, out, S, T, dm, scale); break;
  }
  return check_launch("route_nlp(attention)");
}

int32_t layer_norm(const float* x, const float* g, const float* b, int M, int n, float* y32, uint16_t* y16, hipStream_t st) {
  ProfileScope ps(MOQE_PK_ROUTE, st);
  hipLaunchKernelGGL(k_layer_norm, dim3((M + 3) / 4), dim3(256), 0, st, x, g, b, M, n, y32, y16);
  return check_launch("route_nlp(layer norm)");
}
}  // namespace

int32_t check_nlp_router(const moqe_nlp_router* r, const char* who) {
  if (!r) return set_error(MOQE_E_NULL, "%s: router is NULL", who);
  const void* need[] = {r->w_in, r->b_in, r->wqkv1, r->bqkv1, r->wo1, r->bo1, r->ln1_g, r->ln1_b, r->w_ff1, r->b_ff1, r->w_ff2,
                        r->b_ff2, r->ln2_g, r->ln2_b, r->wqkv2, r->bqkv2, r->wo2, r->bo2, r->ln3_g, r->ln3_b};
  for (const void* p : need)
    if (!p) return set_error(MOQE_E_NULL, "%s: a parameter pointer is NULL", who);
  const void* mats[] = {r->w_in, r->wqkv1, r->wo1, r->w_ff1, r->w_ff2, r->wqkv2, r->wo2};
  for (const void* p : mats)
    if (reinterpret_cast<uintptr_t>(p) % 16) return set_error(MOQE_E_SHAPE, "%s: parameter matrices must be 16-byte aligned", who);
  const void* vecs[] = {r->b_in, r->bqkv1, r->bo1, r->b_ff1, r->b_ff2, r->bqkv2, r->bo2};
  for (const void* p : vecs)
    if (reinterpret_cast<uintptr_t>(p) % 16) return set_error(MOQE_E_SHAPE, "%s: bias vectors must be 16-byte aligned", who);
  if (r->d <= 0 || r->d % 64 || r->dm <= 0 || r->dm % 128 || r->dm > 64 * LN_MAX_PER_LANE || r->d_ff <= 0 || r->d_ff % 128)
    return set_error(MOQE_E_SHAPE, "%s: d=%d must be a multiple of 64, dm=%d and d_ff=%d multiples of 128, dm <= %d", who, r->d,
                     r->dm, r->d_ff, 64 * LN_MAX_PER_LANE);
  if (r->n_heads <= 0 || r->dm % r->n_heads) return set_error(MOQE_E_SHAPE, "%s: %d heads do not divide dm=%d", who, r->n_heads, r->dm);
  const int dh = r->dm / r->n_heads;
  if (dh != 16 && dh != 32 && dh != 64 && dh != 128)
    return set_error(MOQE_E_SHAPE, "%s: head width %d must be 16, 32, 64 or 128", who, dh);
  if (r->head.d != r->dm) return set_error(MOQE_E_SHAPE, "%s: the MLP head takes %d features, dm is %d", who, r->head.d, r->dm);
  return MOQE_OK;
}

size_t route_nlp_ws_bytes(int S, int T, const moqe_nlp_router& r) { return nlp_layout(S, T, r).total; }

int32_t launch_route_nlp(const void* x, int S, int T, const moqe_nlp_router& r, int32_t* idx, float* logits, void* ws, hipStream_t st) {
  const NlpLayout L = nlp_layout(S, T, r);
  uint8_t* p = static_cast<uint8_t*>(ws);
  auto b16 = [&](size_t off) { return reinterpret_cast<uint16_t*>(p + off); };
  auto f32 = [&](size_t off) { return reinterpret_cast<float*>(p + off); };
  const int M = S * T, dm = r.dm, dff = r.d_ff;
  int32_t rc;
  {
    CvtSegs sg;
    memset(&sg, 0, sizeof(sg));
    const float* src[7] = {r.w_in, r.wqkv1, r.wo1, r.w_ff1, r.w_ff2, r.wqkv2, r.wo2};
    const size_t dst[7] = {L.w_in, L.wqkv1, L.wo1, L.wff1, L.wff2, L.wqkv2, L.wo2};
    const long long cnt[7] = {(long long)dm * r.d, 3ll * dm * dm, (long long)dm * dm, (long long)dff * dm, (long long)dff * dm,
                              3ll * dm * dm, (long long)dm * dm};
    sg.n = 7;
    for (int i = 0; i < 7; ++i) {
      sg.src[i] = src[i];
      sg.dst[i] = b16(dst[i]);
      sg.first[i + 1] = sg.first[i] + cnt[i] / 4;          // every count is a multiple of 64
    }
    ProfileScope ps(MOQE_PK_ROUTE, st);
    const long long blocks = (sg.first[7] + 255) / 256;
    hipLaunchKernelGGL(k_to_bf16, dim3(unsigned(blocks < 2048 ? blocks : 2048)), dim3(256), 0, st, sg);
    rc = check_launch("route_nlp(parameters)");
    if (rc) return rc;
  }
  rc = ensure_dynamic_lds(LDSK_NLP_LIN, reinterpret_cast<const void*>(&k_lin), L_LDS_BYTES, "route_nlp");
  if (rc) return rc;
  const uint16_t* xb = static_cast<const uint16_t*>(x);
  // u = x W_in^T + b_in                                             u: t32a / t16a
  if ((rc = lin(xb, b16(L.w_in), r.b_in, nullptr, f32(L.t32a), b16(L.t16a), M, dm, r.d, false, f32(L.part), st))) return rc;
  // encoder layer: v = LN1(u + attention(u))                         v: t32c / t16a
  if ((rc = lin(b16(L.t16a), b16(L.wqkv1), r.bqkv1, nullptr, f32(L.qkv), nullptr, M, 3 * dm, dm, false, f32(L.part), st))) return rc;
  if ((rc = attention(f32(L.qkv), b16(L.t16b), S, T, dm, r.n_heads, st))) return rc;
  if ((rc = lin(b16(L.t16b), b16(L.wo1), r.bo1, f32(L.t32a), f32(L.t32b), nullptr, M, dm, dm, false, f32(L.part), st))) return rc;
  if ((rc = layer_norm(f32(L.t32b), r.ln1_g, r.ln1_b, M, dm, f32(L.t32c), b16(L.t16a), st))) return rc;
  //                w = LN2(v + W2 relu(W1 v + b1) + b2)              w: t32a / t16a
  if ((rc = lin(b16(L.t16a), b16(L.wff1), r.b_ff1, nullptr, nullptr, b16(L.hid), M, dff, dm, true, f32(L.part), st))) return rc;
  if ((rc = lin(b16(L.hid), b16(L.wff2), r.b_ff2, f32(L.t32c), f32(L.t32b), nullptr, M, dm, dff, false, f32(L.part), st))) return rc;
  if ((rc = layer_norm(f32(L.t32b), r.ln2_g, r.ln2_b, M, dm, f32(L.t32a), b16(L.t16a), st))) return rc;
  // attention module: z = LN3(w + attention2(w))                     z: t32c
  if ((rc = lin(b16(L.t16a), b16(L.wqkv2), r.bqkv2, nullptr, f32(L.qkv), nullptr, M, 3 * dm, dm, false, f32(L.part), st))) return rc;
  if ((rc = attention(f32(L.qkv), b16(L.t16b), S, T, dm, r.n_heads, st))) return rc;
  if ((rc = lin(b16(L.t16b), b16(L.wo2), r.bo2, f32(L.t32a), f32(L.t32b), nullptr, M, dm, dm, false, f32(L.part), st))) return rc;
  if ((rc = layer_norm(f32(L.t32b), r.ln3_g, r.ln3_b, M, dm, f32(L.t32c), nullptr, st))) return rc;
  {
    ProfileScope ps(MOQE_PK_ROUTE, st);
    hipLaunchKernelGGL(k_pool_f32, dim3((dm + 63) / 64, S), dim3(1024), 0, st, f32(L.t32c), f32(L.pooled), S, T, dm);
    if ((rc = check_launch("route_nlp(pool)"))) return rc;
  }
  return launch_route_features(f32(L.pooled), S, r.head, idx, logits, p + L.head, st);
}

}  // namespace moqe
