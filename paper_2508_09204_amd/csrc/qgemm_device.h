// Device helpers shared by the grouped dequantize-GEMM kernels: how packed codes become exact
// bf16 matrix-core operands, small conversions.
#pragma once

#include "moqe_internal.h"

#include <type_traits>

namespace moqe {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));


// How a stored code c appears to the matrix cores: the bf16 value BASE + CM * c.
//   FMT_I8 : c itself (converted through fp32; integers up to 255 are exact in bf16).
//   nibble / bit-plane formats: the code bits are OR-ed into the top mantissa bits of the bf16
//   constant BASE = 2^e, whose mantissa step is BASE/128, so that the value is BASE + c/2.
//   A small BASE keeps sum_k x (BASE + c/2) close in size to the wanted sum_k x (c - z), which
//   limits the cancellation error of removing the offset afterwards.
template <int FMT> struct CodeMap;
template <> struct CodeMap<FMT_I8>   { static constexpr float BASE = 0.f,  CM = 1.f;  };
template <> struct CodeMap<FMT_I8A8> { static constexpr float BASE = 0.f,  CM = 1.f;  };
template <> struct CodeMap<FMT_N4>   { static constexpr float BASE = 8.f,  CM = 0.5f; };   // 0x4100 | c << 3
template <> struct CodeMap<FMT_N3>   { static constexpr float BASE = 4.f,  CM = 0.5f; };   // 0x4080 | c << 4
template <> struct CodeMap<FMT_N6>   { static constexpr float BASE = 32.f, CM = 0.5f; };   // 0x4200 | c << 1

template <int FMT> struct Raw;
template <> struct Raw<FMT_I8>   { static constexpr int N = 8; static constexpr int PF = 2; };
template <> struct Raw<FMT_I8A8> { static constexpr int N = 8; static constexpr int PF = 2; };
template <> struct Raw<FMT_N4>   { static constexpr int N = 4; static constexpr int PF = 4; };
template <> struct Raw<FMT_N3>   { static constexpr int N = 3; static constexpr int PF = 4; };
template <> struct Raw<FMT_N6>   { static constexpr int N = 6; static constexpr int PF = 2; };

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// A buffer descriptor over a packed blob (a blob is smaller than 4 GiB): a load through it takes a scalar byte
// offset and a per-lane byte offset of 32 bits each, so a tile's address costs a scalar multiply-add and no
// 64-bit arithmetic in the vector unit (a global load of base + uniform offset + lane offset was compiled to four
// to six 64-bit vector additions per tile).  It also keeps such loads out of the flat path: a pointer that the
// compiler cannot trace back to a kernel argument (one put together from integers, say) is loaded with flat
// instructions, and a pending flat load turns every later wait for memory into a wait for ALL memory operations,
// so that a ring of loads in flight drains at each use.
typedef __amdgpu_buffer_rsrc_t buf_rsrc;
static __device__ __forceinline__ buf_rsrc blob_rsrc(const uint8_t* p) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(p), 0, -1, 0x00020000);   // raw buffer, 32-bit data format
}
static __device__ __forceinline__ u32x4 buf_load128(buf_rsrc rs, int voff, uint32_t soff) {
  return __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, voff, int(soff), 0));
}
static __device__ __forceinline__ u32x2 buf_load64(buf_rsrc rs, int voff, uint32_t soff) {
  return __builtin_bit_cast(u32x2, __builtin_amdgcn_raw_buffer_load_b64(rs, voff, int(soff), 0));
}
static __device__ __forceinline__ uint32_t buf_load32(buf_rsrc rs, int voff, uint32_t soff) {
  return uint32_t(__builtin_amdgcn_raw_buffer_load_b32(rs, voff, int(soff), 0));
}

// The packed codes of the tile that starts `soff` bytes into the blob, this lane's share.
template <int FMT>
static __device__ __forceinline__ void load_raw(uint32_t (&r)[Raw<FMT>::N], buf_rsrc rs, uint32_t soff, int lane) {
  if constexpr (FMT == FMT_I8 || FMT == FMT_I8A8) {
    const u32x4 a = buf_load128(rs, lane * 16, soff), b = buf_load128(rs, lane * 16 + 1024, soff);
    r[0] = a.x; r[1] = a.y; r[2] = a.z; r[3] = a.w; r[4] = b.x; r[5] = b.y; r[6] = b.z; r[7] = b.w;
  } else if constexpr (FMT == FMT_N4) {
    const u32x4 a = buf_load128(rs, lane * 16, soff);
    r[0] = a.x; r[1] = a.y; r[2] = a.z; r[3] = a.w;
  } else if constexpr (FMT == FMT_N3) {
    const u32x2 a = buf_load64(rs, lane * 8, soff);
    r[0] = a.x; r[1] = a.y;
    r[2] = buf_load32(rs, lane * 4 + 512, soff);
  } else {
    const u32x4 a = buf_load128(rs, lane * 16, soff);
    const u32x2 b = buf_load64(rs, lane * 8 + 1024, soff);
    r[0] = a.x; r[1] = a.y; r[2] = a.z; r[3] = a.w; r[4] = b.x; r[5] = b.y;
  }
}

template <int FMT>
static __device__ __forceinline__ void load_raw(uint32_t (&r)[Raw<FMT>::N], const uint8_t* tile, int lane) {
  if constexpr (FMT == FMT_I8 || FMT == FMT_I8A8) {
    uint4 a = *reinterpret_cast<const uint4*>(tile + lane * 16);
    uint4 b = *reinterpret_cast<const uint4*>(tile + 1024 + lane * 16);
    r[0] = a.x; r[1] = a.y; r[2] = a.z; r[3] = a.w; r[4] = b.x; r[5] = b.y; r[6] = b.z; r[7] = b.w;
  } else if constexpr (FMT == FMT_N4) {
    uint4 a = *reinterpret_cast<const uint4*>(tile + lane * 16);
    r[0] = a.x; r[1] = a.y; r[2] = a.z; r[3] = a.w;
  } else if constexpr (FMT == FMT_N3) {
    uint2 a = *reinterpret_cast<const uint2*>(tile + lane * 8);
    r[0] = a.x; r[1] = a.y;
    r[2] = *reinterpret_cast<const uint32_t*>(tile + 512 + lane * 4);
  } else {
    uint4 a = *reinterpret_cast<const uint4*>(tile + lane * 16);
    uint2 b = *reinterpret_cast<const uint2*>(tile + 1024 + lane * 8);
    r[0] = a.x; r[1] = a.y; r[2] = a.z; r[3] = a.w; r[4] = b.x; r[5] = b.y;
  }
}

// Constants of the unpacking, made opaque to the optimizer once per kernel: the mask lives in a
// scalar register and the bf16 exponent pattern in a vector register, so that (x & mask) | pattern
// is selected as ONE three-operand instruction (two literals do not fit its encoding, and with
// visible literals the compiler falls back to two instructions).  The unpacking itself stays plain
// C: the compiler must see every vector instruction that runs next to the matrix-core operations
// to place the wait states their register hazards need, which it cannot do for inline assembly.
template <uint32_t V> static __device__ __forceinline__ uint32_t opaque_sgpr() {
  uint32_t r;
  asm("s_mov_b32 %0, %1" : "=s"(r) : "n"(V));
  return r;
}
template <uint32_t V> static __device__ __forceinline__ uint32_t opaque_vgpr() {
  uint32_t r;
  asm("v_mov_b32 %0, %1" : "=v"(r) : "n"(V));
  return r;
}

template <int FMT> struct FragK { uint32_t m0, m1, pat; };
template <int FMT> static __device__ __forceinline__ FragK<FMT> frag_constants() {
  FragK<FMT> k{0u, 0u, 0u};
  if constexpr (FMT == FMT_N4) { k.m0 = opaque_sgpr<0x00780078u>(); k.pat = opaque_vgpr<0x41004100u>(); }
  if constexpr (FMT == FMT_N3) { k.m0 = opaque_sgpr<0x00300030u>(); k.m1 = opaque_sgpr<0x00400040u>(); k.pat = opaque_vgpr<0x40804080u>(); }
  if constexpr (FMT == FMT_N6) { k.m0 = opaque_sgpr<0x001E001Eu>(); k.m1 = opaque_sgpr<0x00600060u>(); k.pat = opaque_vgpr<0x42004200u>(); }
  return k;
}

static __device__ __forceinline__ uint32_t and_or(uint32_t x, uint32_t mask, uint32_t orv) { return (x & mask) | orv; }
// A value the optimizer must take as it is (no instruction is emitted).  Two-field codes are put together as
// (a & m0) | ((b & m1) | pattern): seen whole, the expression is regrouped into two ANDs and a three-input OR;
// with the inner part kept apart both halves stay and-or instructions, one instruction less per code pair.
static __device__ __forceinline__ uint32_t kept(uint32_t v) { asm("" : "+v"(v)); return v; }

template <int SH> static __device__ __forceinline__ uint32_t shift_by(uint32_t v) {
  if constexpr (SH >= 0) return v >> SH; else return v << (-SH);
}

// The matrix-core operand of step J (columns 32J + 8kq + 0..7 of the lane's row) as 8 bf16
// values BASE + CM * code.
template <int FMT, int J>
static __device__ __forceinline__ bf16x8 frag(const uint32_t (&r)[Raw<FMT>::N], const FragK<FMT>& k) {
  u32x4 d;
  if constexpr (FMT == FMT_I8) {
    const uint32_t u0 = r[(J / 2) * 4 + (J % 2) * 2], u1 = r[(J / 2) * 4 + (J % 2) * 2 + 1];
    // integers up to 255 are exact in fp32 and their bf16 is the upper half of the fp32 pattern
    const uint32_t f0 = __float_as_uint(float(u0 & 0xffu)), f1 = __float_as_uint(float((u0 >> 8) & 0xffu));
    const uint32_t f2 = __float_as_uint(float((u0 >> 16) & 0xffu)), f3 = __float_as_uint(float(u0 >> 24));
    const uint32_t f4 = __float_as_uint(float(u1 & 0xffu)), f5 = __float_as_uint(float((u1 >> 8) & 0xffu));
    const uint32_t f6 = __float_as_uint(float((u1 >> 16) & 0xffu)), f7 = __float_as_uint(float(u1 >> 24));
    d.x = __builtin_amdgcn_perm(f1, f0, 0x07060302u);
    d.y = __builtin_amdgcn_perm(f3, f2, 0x07060302u);
    d.z = __builtin_amdgcn_perm(f5, f4, 0x07060302u);
    d.w = __builtin_amdgcn_perm(f7, f6, 0x07060302u);
  } else if constexpr (FMT == FMT_N4) {
    const uint32_t w = r[J];                      // 0x4100 | c << 3 per 16-bit half
    d.x = and_or(shift_by<-3>(w), k.m0, k.pat);
    d.y = and_or(shift_by<1>(w), k.m0, k.pat);
    d.z = and_or(shift_by<5>(w), k.m0, k.pat);
    d.w = and_or(shift_by<9>(w), k.m0, k.pat);
  } else if constexpr (FMT == FMT_N3) {
    const uint32_t lo = r[J / 2], hi = r[2];      // 0x4080 | c << 4: two low bits from `lo`, the high bit from `hi`
    constexpr int P0 = 4 * (J % 2);       // first 2-bit field of this step inside `lo`
    constexpr int Q0 = 4 * J;             // first 1-bit field of this step inside `hi`
    d.x = and_or(shift_by<2 * (P0 + 0) - 4>(lo), k.m0, kept(and_or(shift_by<Q0 + 0 - 6>(hi), k.m1, k.pat)));
    d.y = and_or(shift_by<2 * (P0 + 1) - 4>(lo), k.m0, kept(and_or(shift_by<Q0 + 1 - 6>(hi), k.m1, k.pat)));
    d.z = and_or(shift_by<2 * (P0 + 2) - 4>(lo), k.m0, kept(and_or(shift_by<Q0 + 2 - 6>(hi), k.m1, k.pat)));
    d.w = and_or(shift_by<2 * (P0 + 3) - 4>(lo), k.m0, kept(and_or(shift_by<Q0 + 3 - 6>(hi), k.m1, k.pat)));
  } else {  // FMT_N6: 0x4200 | c << 1: four low bits from `w`, two high bits from `hi`
    const uint32_t w = r[J], hi = r[4 + J / 2];
    constexpr int P0 = 4 * (J % 2);
    d.x = and_or(shift_by<-1>(w), k.m0, kept(and_or(shift_by<2 * (P0 + 0) - 5>(hi), k.m1, k.pat)));
    d.y = and_or(shift_by<3>(w), k.m0, kept(and_or(shift_by<2 * (P0 + 1) - 5>(hi), k.m1, k.pat)));
    d.z = and_or(shift_by<7>(w), k.m0, kept(and_or(shift_by<2 * (P0 + 2) - 5>(hi), k.m1, k.pat)));
    d.w = and_or(shift_by<11>(w), k.m0, kept(and_or(shift_by<2 * (P0 + 3) - 5>(hi), k.m1, k.pat)));
  }
  return __builtin_bit_cast(bf16x8, d);
}

static __device__ __forceinline__ f32x4 mfma_bf16(const u32x4& a, const bf16x8& b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), b, c, 0, 0, 0);
}

static __device__ __forceinline__ uint16_t float_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return uint16_t(u >> 16);
}

static __device__ __forceinline__ float silu_mul(float g, float u) {
  return (g / (1.0f + __expf(-g))) * u;
}

}  // namespace moqe
