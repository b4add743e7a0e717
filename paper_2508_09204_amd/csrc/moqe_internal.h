// Internal declarations shared by the translation units of libmoqe (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/moqe.h"

namespace moqe {

// ---------------------------------------------------------------------------------------
// Packed device layout
//
// A matrix [n, k] (n % 16 == 0, k % 128 == 0) is cut into tiles of 16 rows x 128 columns,
// stored row-tile major: tile (nt, kt) has index nt * (k/128) + kt.  Inside a tile the
// codes are ordered for a 64-lane wavefront feeding 16x16x32 bf16 matrix-core steps: lane
// l = kq*16 + r owns row r and, for step j = 0..3, the eight columns 32j + 8kq + 0..7.
// Each lane's share of a tile is contiguous, so one wave reads a tile with one (or a few)
// fully coalesced 16-byte-per-lane loads and needs no shuffles before the matrix cores.
//
// Code storage per format (all codes are stored unsigned; a symmetric code q is stored as
// q + 2^(bits-1)):
//   FMT_I8   : 1 byte per code.  Two 1 KiB halves per tile (steps 0-1, steps 2-3); in a
//              half, lane l has 16 bytes: step-major, column-minor.
//   FMT_N4   : 4 bits.  Lane l has 16 bytes = one dword per step; in a dword, column i sits
//              in nibble i/2 (i even) or 4 + i/2 (i odd), so that (w >> 4p) & 0x000F000F
//              yields the pair (2p, 2p+1) as two 16-bit lanes.
//   FMT_N3   : 3 bits as a 2-bit plane (512 B per tile, 8 bytes per lane: one dword per two
//              steps, fields paired like the nibbles) and a 1-bit plane (256 B, one dword per
//              lane: bit 4j + i/2 for even i, +16 for odd i).
//   FMT_N6   : 6 bits as a 4-bit plane (like FMT_N4) and a 2-bit plane (like FMT_N3's).
//   FMT_I8A8 : signed bytes ordered for 16x16x64 int8 matrix-core steps: two 1 KiB halves
//              (columns 0-63, 64-127); lane l = kq*16 + r has the 16 columns 16kq + 0..15.
//
// After the codes come the scales (fp32) and, for asymmetric formats, the zero-points (u8):
// group formats store them per tile as [tile][row 16][groups per tile], per-channel formats
// as [n].  Each region starts on a 256-byte boundary.
// ---------------------------------------------------------------------------------------
enum Fmt : int { FMT_I8 = 0, FMT_N4 = 1, FMT_N3 = 2, FMT_N6 = 3, FMT_I8A8 = 4, FMT_NONE = -1 };
enum GroupMode : int { GM_PC = 0, GM_G128 = 1, GM_G64 = 2 };

struct PackedInfo {
  int      fmt;          // Fmt
  int      gm;           // GroupMode
  int      gpt;          // groups per 128-column tile: 0 (per channel), 1, 2
  int      zc;           // implicit zero of stored codes for symmetric formats, else 0
  int      asym;         // 1: per-group zero-points are stored
  int      nt, kt;       // tiles along n and k
  uint32_t tile_bytes;
  size_t   scale_off, zero_off, total;
};

__host__ __device__ inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

// Returns false when the format / shape is not supported.
__host__ __device__ inline bool packed_info(int n, int k, int bits, int group, int symmetric,
                                            int act_mode, PackedInfo* pi) {
  if (n <= 0 || k <= 0 || (n % 16) != 0 || (k % 128) != 0) return false;
  int fmt = FMT_NONE;
  if (symmetric) {
    if (group != 0) return false;
    if (bits == 8) fmt = act_mode ? FMT_I8A8 : FMT_I8;
    else if (bits == 6 && !act_mode) fmt = FMT_N6;
    else if (bits == 4 && !act_mode) fmt = FMT_N4;
  } else {
    if (act_mode) return false;
    if (group != 64 && group != 128) return false;
    if (bits == 4) fmt = FMT_N4;
    else if (bits == 3) fmt = FMT_N3;
  }
  if (fmt == FMT_NONE) return false;
  pi->fmt = fmt;
  pi->gm = group == 0 ? GM_PC : (group == 128 ? GM_G128 : GM_G64);
  pi->gpt = group == 0 ? 0 : 128 / group;
  pi->asym = symmetric ? 0 : 1;
  pi->zc = symmetric ? (fmt == FMT_I8A8 ? 0 : (1 << (bits - 1))) : 0;
  pi->nt = n / 16;
  pi->kt = k / 128;
  pi->tile_bytes = fmt == FMT_I8 || fmt == FMT_I8A8 ? 2048u : fmt == FMT_N4 ? 1024u : fmt == FMT_N3 ? 768u : 1536u;
  size_t tiles = size_t(pi->nt) * size_t(pi->kt);
  pi->scale_off = align256(tiles * pi->tile_bytes);
  size_t nscale = pi->gpt ? tiles * 16 * size_t(pi->gpt) : size_t(n);
  pi->zero_off = align256(pi->scale_off + nscale * 4);
  pi->total = pi->asym ? align256(pi->zero_off + nscale) : pi->zero_off;
  return true;
}

// Position of the code of element (row, col) inside the packed blob.
struct CodePos {
  size_t   byte0;  uint32_t shift0, bits0;   // first (or only) bit field, inside the dword at byte0
  size_t   byte1;  uint32_t shift1, bits1;   // second plane (bits1 == 0: none)
};

__host__ __device__ inline CodePos code_pos(const PackedInfo& pi, int row, int col) {
  CodePos p{};
  size_t t = size_t(row / 16) * size_t(pi.kt) + size_t(col / 128);
  int r = row % 16, kk = col % 128;
  size_t base = t * pi.tile_bytes;
  if (pi.fmt == FMT_I8A8) {
    int js = kk / 64, kq = (kk % 64) / 16, i = kk % 16, lane = kq * 16 + r;
    size_t b = base + size_t(js) * 1024 + size_t(lane) * 16 + size_t(i);
    p.byte0 = b & ~size_t(3); p.shift0 = uint32_t(b & 3) * 8; p.bits0 = 8;
    return p;
  }
  int j = kk / 32, kq = (kk % 32) / 8, i = kk % 8, lane = kq * 16 + r;
  int pairfield = (i & 1) ? 1 : 0;   // odd columns live in the upper 16-bit half
  if (pi.fmt == FMT_I8) {
    size_t b = base + size_t(j / 2) * 1024 + size_t(lane) * 16 + size_t(j % 2) * 8 + size_t(i);
    p.byte0 = b & ~size_t(3); p.shift0 = uint32_t(b & 3) * 8; p.bits0 = 8;
    return p;
  }
  if (pi.fmt == FMT_N4 || pi.fmt == FMT_N6) {
    p.byte0 = base + size_t(lane) * 16 + size_t(j) * 4;
    p.shift0 = uint32_t(4 * (i / 2) + 16 * pairfield); p.bits0 = 4;
    if (pi.fmt == FMT_N6) {
      p.byte1 = base + 1024 + size_t(lane) * 8 + size_t(j / 2) * 4;
      p.shift1 = uint32_t(2 * (4 * (j % 2) + i / 2) + 16 * pairfield); p.bits1 = 2;
    }
    return p;
  }
  // FMT_N3
  p.byte0 = base + size_t(lane) * 8 + size_t(j / 2) * 4;
  p.shift0 = uint32_t(2 * (4 * (j % 2) + i / 2) + 16 * pairfield); p.bits0 = 2;
  p.byte1 = base + 512 + size_t(lane) * 4;
  p.shift1 = uint32_t(4 * j + i / 2 + 16 * pairfield); p.bits1 = 1;
  return p;
}

// Index of the scale / zero-point of (row, col) inside their regions.
__host__ __device__ inline size_t meta_index(const PackedInfo& pi, int row, int col) {
  if (pi.gpt == 0) return size_t(row);
  size_t t = size_t(row / 16) * size_t(pi.kt) + size_t(col / 128);
  int g = (col % 128) / (128 / pi.gpt);
  return (t * 16 + size_t(row % 16)) * size_t(pi.gpt) + size_t(g);
}

// ---------------------------------------------------------------------------------------
// Kernel-side description of the experts of one grouped GEMM launch
// ---------------------------------------------------------------------------------------
struct ExpertDev {
  const uint8_t* w[2];       // packed blobs: [0] = the matrix (or gate), [1] = up (gate/up launch)
  int32_t  fmt, gm;
  int32_t  zc;               // implicit zero of symmetric codes
  int32_t  asym;
  uint32_t tile_bytes;
  uint32_t scale_off, zero_off;   // region offsets inside a blob (< 4 GiB)
};

struct GemmArgs {
  ExpertDev ex[MOQE_MAX_EXPERTS];
  int32_t   n_experts;
  int32_t   n, k;                      // per-matrix output / input features
  int32_t   S, T;
  const void*    a;          // bf16 [M, k] (act_mode 0) rows
  const int8_t*  a_q;        // int8 [M, k] bucket order (act_mode 1 experts), may be NULL
  const float*   a_scale;    // per-row scales of a_q
  const int32_t* offsets;    // [K+1] samples
  const int32_t* a_perm;     // bucket slot -> sample for reading a; NULL: a is in bucket order
  const int32_t* y_perm;     // bucket slot -> sample for writing y; NULL: bucket order
  void*     y;               // float [M, n] (plain) or bf16 [M, n] (gate/up, bucket order; plain with y_bf16)
  int32_t   y_bf16;          // plain launch: results are rounded to bf16 (nearest even) and stored as 16-bit rows
  int32_t   conv_h, conv_w, conv_c;   // tiled kernel, 3x3 convolution: a is the NHWC image [S, h, w, c] and the
                             // k = (kh*3 + kw)*c + ch columns of a row are gathered from its pixel's neighbours
  int32_t   min_rows, max_rows;   // this launch handles the experts whose bucket has min_rows .. max_rows rows
  // Streaming kernel, at most 64 samples: the launch buckets the samples itself from the router's choice (every
  // work-group works the same stable counting sort out in registers) instead of reading offsets and perm, and its first
  // work-group writes counts / offsets / perm / inv_perm (any may be NULL) for whatever runs after it.
  const int32_t* expert_idx;      // [S] or NULL: offsets and perm come from memory
  int32_t*  out_counts; int32_t* out_offsets; int32_t* out_perm; int32_t* out_inv_perm;
};

// ---------------------------------------------------------------------------------------
// Errors, profiling, launchers (implemented across the .hip files)
// ---------------------------------------------------------------------------------------
int32_t set_error(int32_t code, const char* fmt, ...);
bool    dry_run();

// Times kernel launches with HIP events when profiling is on.  The default scope records one event
// before and one after whatever is launched inside it.  An `exact` scope records nothing itself: its one
// kernel is launched through launch(), which hands the two events to the launch, so that they carry the
// kernel's own begin and end time stamps (what a kernel trace reports) without the dispatch gap.
struct ProfileScope {
  ProfileScope(int kind, hipStream_t s, bool exact = false);
  ~ProfileScope();
  template <typename F, typename... Args>
  void launch(F kernel, dim3 grid, dim3 block, size_t lds_bytes, Args... args) {
    if (slot >= 0 && exact) hipExtLaunchKernelGGL(kernel, grid, block, lds_bytes, stream, ev_begin, ev_end, 0, args...);
    else hipLaunchKernelGGL(kernel, grid, block, lds_bytes, stream, args...);
  }
  int slot; hipStream_t stream; bool exact;
  hipEvent_t ev_begin, ev_end;
};

int32_t check_launch(const char* what);

// Kernels that need more than 64 KiB of dynamic LDS must ask for it once per kernel: `slot` is a
// process-wide id of the kernel (LdsKernel); the request is made by the first caller only, under a
// lock, and every caller gets its outcome.
enum LdsKernel : int { LDSK_STREAM0 = 0, LDSK_TILE0 = 8, LDSK_ROUTER_TAIL = 12, LDSK_NLP_LIN = 13, LDSK_COUNT = 16 };
int32_t ensure_dynamic_lds(int slot, const void* kernel, int bytes, const char* what);

int32_t launch_route(const void* x, int S, int T, const moqe_router& r, int32_t* idx, float* logits,
                     void* ws, hipStream_t st);
size_t  route_ws_bytes(int S, int T, const moqe_router& r);
int32_t launch_route_features(const float* feat, int S, const moqe_router& r, int32_t* idx, float* logits, void* ws, hipStream_t st);
int32_t check_cv_router(const moqe_cv_router* r, int h, int w, const char* who);
size_t  route_cv_ws_bytes(int S, int h, int w, const moqe_cv_router& r);
int32_t launch_route_cv(const void* x, int S, int h, int w, const moqe_cv_router& r, int32_t* idx, float* logits, void* ws, hipStream_t st);
int32_t check_nlp_router(const moqe_nlp_router* r, const char* who);
size_t  route_nlp_ws_bytes(int S, int T, const moqe_nlp_router& r);
int32_t launch_route_nlp(const void* x, int S, int T, const moqe_nlp_router& r, int32_t* idx, float* logits, void* ws, hipStream_t st);
int32_t launch_route_ragged(const void* x, const int32_t* cu_rows, int S, const moqe_router& r, int32_t* idx, float* logits,
                            void* ws, hipStream_t st);
int32_t launch_expand_rows(const int32_t* cu_rows, const int32_t* offsets, const int32_t* perm, int S, int K,
                           int32_t* slot_rows, int32_t* row_offsets, int32_t* row_perm, hipStream_t st);
int32_t launch_route_bucket(const void* x, int S, int T, const moqe_router& r, int32_t* idx, float* logits,
                            int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv_perm, void* ws, hipStream_t st);
int32_t launch_bucket(const int32_t* idx, int S, int K, int32_t* counts, int32_t* offsets,
                      int32_t* perm, int32_t* inv_perm, hipStream_t st);
int32_t launch_label_dispatch(int S, int K, int32_t* offsets, int32_t* perm, hipStream_t st);
int32_t launch_label_loss(const float* y, const int32_t* targets, int S, int T, int n, int K, float* losses, int32_t* labels,
                          hipStream_t st);
int32_t launch_balance_stats(const float* logits, const int32_t* counts, int S, int K, float alpha, float* out,
                             hipStream_t st);
int32_t launch_quantize(const float* w, float clip, const moqe_qmat& out, hipStream_t st);
int32_t launch_pack(const moqe_qmat& c, const PackedInfo& pi, uint8_t* out, hipStream_t st);
int32_t launch_unpack(const moqe_qmat& p, const PackedInfo& pi, int16_t* out, float* scale_out, hipStream_t st);
// Two streaming kernels for buckets of a few rows: activations resident in registers (rows of up to
// STREAM_REG_MAX_KT k-tiles of 128 columns, which one phase of that kernel covers), activations marching
// through LDS (longer rows).
constexpr int STREAM_REG_MAX_KT = 32;
int32_t launch_qgemm_stream(const GemmArgs& ga, bool gateup, hipStream_t st);
int32_t launch_qgemm_stream_lds(const GemmArgs& ga, bool gateup, hipStream_t st);
int32_t launch_qgemm_tile(const GemmArgs& ga, bool gateup, hipStream_t st);
int32_t launch_act_quant(const void* x_bf16, int kdim, int T, const int32_t* offsets, const int32_t* perm,
                         int expert, int max_rows, int8_t* out, float* scales, hipStream_t st);

}  // namespace moqe
