// Weight preparation and activation preparation kernels:
//   round-to-nearest quantizers (canonical layout), canonical <-> packed layout,
//   per-row dynamic int8 activation quantization (W8A8 expert).
// The quantizers use fp32 IEEE operations with explicit rounding intrinsics so that no
// multiply-add contraction changes a code.
#include "moqe_internal.h"

namespace moqe {

static __device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}
static __device__ __forceinline__ float wave_min(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v = fminf(v, __shfl_xor(v, off, 64));
  return v;
}

// Block-wide max of non-negative values, every thread gets the result.
static __device__ __forceinline__ float block_max_256(float v, float* sh) {
  v = wave_max(v);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = fmaxf(fmaxf(sh[0], sh[1]), fmaxf(sh[2], sh[3]));
  __syncthreads();
  return r;
}

// ---- symmetric per-output-channel: one work-group per row ---------------------------------
__global__ __launch_bounds__(256) void k_quant_sym(const float* __restrict__ w, int n, int k, int bits,
                                                    int8_t* __restrict__ q, float* __restrict__ scale) {
  __shared__ float sh[4];
  const int row = blockIdx.x;
  const float* wr = w + size_t(row) * k;
  float a = 0.f;
  for (int c = threadIdx.x; c < k; c += 256) a = fmaxf(a, fabsf(wr[c]));
  a = block_max_256(a, sh);
  const float qmax = float((1 << (bits - 1)) - 1);
  const float s = (a == 0.f) ? 1.0f : __fdiv_rn(a, qmax);
  if (threadIdx.x == 0) scale[row] = s;
  int8_t* qr = q + size_t(row) * k;
  for (int c = threadIdx.x; c < k; c += 256) {
    float v = rintf(__fdiv_rn(wr[c], s));
    v = fminf(fmaxf(v, -qmax), qmax);
    qr[c] = int8_t(int(v));
  }
}

// ---- asymmetric group-wise: one wave per (row, group) ---------------------------------------
__global__ __launch_bounds__(256) void k_quant_asym(const float* __restrict__ w, int n, int k, int bits, int group,
                                                     float clip, uint8_t* __restrict__ q, float* __restrict__ scale,
                                                     uint8_t* __restrict__ zero) {
  const int lane = threadIdx.x & 63;
  const size_t gid = size_t(blockIdx.x) * 4 + (threadIdx.x >> 6);
  const int gpr = k / group;
  if (gid >= size_t(n) * gpr) return;
  const int row = int(gid / gpr), g = int(gid % gpr);
  const float* wg = w + size_t(row) * k + size_t(g) * group;
  float mn = 0.f, mx = 0.f;
  for (int c = lane; c < group; c += 64) { float v = wg[c]; mn = fminf(mn, v); mx = fmaxf(mx, v); }
  mn = wave_min(mn);
  mx = wave_max(mx);
  const float L = float((1 << bits) - 1);
  const float lo = __fmul_rn(clip, mn), hi = __fmul_rn(clip, mx);
  const float s = (hi == lo) ? 1.0f : __fdiv_rn(__fsub_rn(hi, lo), L);
  const float z = fminf(fmaxf(rintf(__fdiv_rn(-lo, s)), 0.f), L);
  if (lane == 0) { scale[gid] = s; zero[gid] = uint8_t(int(z)); }
  uint8_t* qg = q + size_t(row) * k + size_t(g) * group;
  for (int c = lane; c < group; c += 64) {
    float v = __fadd_rn(rintf(__fdiv_rn(wg[c], s)), z);
    v = fminf(fmaxf(v, 0.f), L);
    qg[c] = uint8_t(int(v));
  }
}

int32_t launch_quantize(const float* w, float clip, const moqe_qmat& out, hipStream_t st) {
  ProfileScope ps(MOQE_PK_OTHER, st);
  if (out.symmetric) {
    hipLaunchKernelGGL(k_quant_sym, dim3(out.n), dim3(256), 0, st, w, out.n, out.k, out.bits,
                       static_cast<int8_t*>(const_cast<void*>(out.qdata)), const_cast<float*>(out.scale));
  } else {
    size_t groups = size_t(out.n) * (out.k / out.group);
    hipLaunchKernelGGL(k_quant_asym, dim3(unsigned((groups + 3) / 4)), dim3(256), 0, st, w, out.n, out.k, out.bits,
                       out.group, clip, static_cast<uint8_t*>(const_cast<void*>(out.qdata)),
                       const_cast<float*>(out.scale), const_cast<uint8_t*>(out.zero));
  }
  return check_launch("quantize_rtn");
}

// ---- canonical -> packed -------------------------------------------------------------------
// One thread per code; codes are OR-ed into the (pre-zeroed) blob at the position code_pos() gives.
__global__ void k_pack_codes(const uint8_t* __restrict__ q, int n, int k, int symmetric, PackedInfo pi,
                             uint8_t* __restrict__ out) {
  size_t i = size_t(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i >= size_t(n) * k) return;
  const int row = int(i / k), col = int(i % k);
  uint32_t code;
  if (pi.fmt == FMT_I8A8) code = q[i];                                   // two's complement byte as is
  else if (symmetric) code = uint32_t(int(reinterpret_cast<const int8_t*>(q)[i]) + pi.zc);
  else code = q[i];
  const CodePos p = code_pos(pi, row, col);
  atomicOr(reinterpret_cast<unsigned int*>(out + p.byte0), (code & ((1u << p.bits0) - 1u)) << p.shift0);
  if (p.bits1) atomicOr(reinterpret_cast<unsigned int*>(out + p.byte1), ((code >> p.bits0) & ((1u << p.bits1) - 1u)) << p.shift1);
}

__global__ void k_pack_meta(const float* __restrict__ scale, const uint8_t* __restrict__ zero, int n, int k, PackedInfo pi,
                            uint8_t* __restrict__ out) {
  const int gpr = pi.gpt ? k / (128 / pi.gpt) : 1;
  size_t i = size_t(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i >= size_t(n) * gpr) return;
  const int row = int(i / gpr), g = int(i % gpr);
  const int col = pi.gpt ? g * (128 / pi.gpt) : 0;
  const size_t mi = meta_index(pi, row, col);
  reinterpret_cast<float*>(out + pi.scale_off)[mi] = scale[i];
  if (pi.asym) (out + pi.zero_off)[mi] = zero[i];
}

int32_t launch_pack(const moqe_qmat& c, const PackedInfo& pi, uint8_t* out, hipStream_t st) {
  ProfileScope ps(MOQE_PK_OTHER, st);
  hipError_t err = hipMemsetAsync(out, 0, pi.total, st);
  if (err != hipSuccess) return set_error(MOQE_E_HIP, "pack: memset failed: %s", hipGetErrorString(err));
  size_t nel = size_t(c.n) * c.k;
  hipLaunchKernelGGL(k_pack_codes, dim3(unsigned((nel + 255) / 256)), dim3(256), 0, st,
                     static_cast<const uint8_t*>(c.qdata), c.n, c.k, c.symmetric, pi, out);
  size_t nmeta = size_t(c.n) * (pi.gpt ? c.k / (128 / pi.gpt) : 1);
  hipLaunchKernelGGL(k_pack_meta, dim3(unsigned((nmeta + 255) / 256)), dim3(256), 0, st, c.scale, c.zero, c.n, c.k, pi, out);
  return check_launch("pack_qmat");
}

// ---- packed -> integer weights (code - zero) and scales in canonical shape ------------------
__global__ void k_unpack(const uint8_t* __restrict__ blob, int n, int k, PackedInfo pi, int16_t* __restrict__ out,
                         float* __restrict__ scale_out) {
  size_t i = size_t(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i >= size_t(n) * k) return;
  const int row = int(i / k), col = int(i % k);
  const CodePos p = code_pos(pi, row, col);
  uint32_t code = (*reinterpret_cast<const uint32_t*>(blob + p.byte0) >> p.shift0) & ((1u << p.bits0) - 1u);
  if (p.bits1) code |= ((*reinterpret_cast<const uint32_t*>(blob + p.byte1) >> p.shift1) & ((1u << p.bits1) - 1u)) << p.bits0;
  const size_t mi = meta_index(pi, row, col);
  int v;
  if (pi.fmt == FMT_I8A8) v = int(int8_t(code));
  else if (pi.asym) v = int(code) - int((blob + pi.zero_off)[mi]);
  else v = int(code) - pi.zc;
  out[i] = int16_t(v);
  if (scale_out) {
    const int gsz = pi.gpt ? 128 / pi.gpt : k;
    if (col % gsz == 0) {
      const size_t ci = pi.gpt ? size_t(row) * (k / gsz) + col / gsz : size_t(row);
      scale_out[ci] = reinterpret_cast<const float*>(blob + pi.scale_off)[mi];
    }
  }
}

int32_t launch_unpack(const moqe_qmat& p, const PackedInfo& pi, int16_t* out, float* scale_out, hipStream_t st) {
  ProfileScope ps(MOQE_PK_OTHER, st);
  size_t nel = size_t(p.n) * p.k;
  hipLaunchKernelGGL(k_unpack, dim3(unsigned((nel + 255) / 256)), dim3(256), 0, st,
                     static_cast<const uint8_t*>(p.qdata), p.n, p.k, pi, out, scale_out);
  return check_launch("unpack_qmat");
}

// ---- per-row dynamic int8 quantization of the rows of one expert's bucket --------------------
// Row b of the bucket (b < rows of the bucket) is read from x (gathered through perm when given)
// and written, as int8 with its scale, at its bucket-order position.
//   a = max|x|, sx = a/127 (1 if a == 0), xq = clamp(rint(x / sx), -127, 127)   (fp32 IEEE)
__global__ __launch_bounds__(256) void k_act_quant(const uint16_t* __restrict__ x, int kdim, int T,
                                                    const int32_t* __restrict__ offsets, const int32_t* __restrict__ perm,
                                                    int expert, int8_t* __restrict__ out, float* __restrict__ scales) {
  __shared__ float sh[4];
  const int off = offsets[expert];
  const int rows = (offsets[expert + 1] - off) * T;
  const int b = blockIdx.x;
  if (b >= rows) return;
  const int slot = off + b / T, t = b % T;
  const size_t src = perm ? size_t(perm[slot]) * T + t : size_t(off) * T + b;
  const size_t dst = size_t(off) * T + b;
  const uint16_t* xr = x + src * kdim;
  float a = 0.f;
  for (int c = threadIdx.x * 2; c < kdim; c += 512) {
    uint32_t v = *reinterpret_cast<const uint32_t*>(xr + c);
    a = fmaxf(a, fabsf(__uint_as_float(v << 16)));
    a = fmaxf(a, fabsf(__uint_as_float(v & 0xffff0000u)));
  }
  a = block_max_256(a, sh);
  const float sx = (a == 0.f) ? 1.0f : __fdiv_rn(a, 127.0f);
  if (threadIdx.x == 0) scales[dst] = sx;
  int8_t* o = out + dst * kdim;
  for (int c = threadIdx.x * 2; c < kdim; c += 512) {
    uint32_t v = *reinterpret_cast<const uint32_t*>(xr + c);
    float q0 = fminf(fmaxf(rintf(__fdiv_rn(__uint_as_float(v << 16), sx)), -127.f), 127.f);
    float q1 = fminf(fmaxf(rintf(__fdiv_rn(__uint_as_float(v & 0xffff0000u), sx)), -127.f), 127.f);
    uint16_t pk = uint16_t(uint8_t(int8_t(int(q0)))) | uint16_t(uint16_t(uint8_t(int8_t(int(q1)))) << 8);
    *reinterpret_cast<uint16_t*>(o + c) = pk;
  }
}

int32_t launch_act_quant(const void* x_bf16, int kdim, int T, const int32_t* offsets, const int32_t* perm,
                         int expert, int max_rows, int8_t* out, float* scales, hipStream_t st) {
  if (max_rows <= 0) return MOQE_OK;
  ProfileScope ps(MOQE_PK_ACTQUANT, st);
  hipLaunchKernelGGL(k_act_quant, dim3(max_rows), dim3(256), 0, st, static_cast<const uint16_t*>(x_bf16), kdim, T,
                     offsets, perm, expert, out, scales);
  return check_launch("act_quant");
}

}  // namespace moqe
