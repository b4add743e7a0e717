// Grouped dequantize-GEMM, weight-streaming kernel for buckets of a few rows and LONG rows (k beyond what
// the register-resident kernel covers in one phase, e.g. the down projection of an MLP block).
//
// Each sample is processed by its selected expert only (MoQE Section 3.1), so for expert e the
// rows of its bucket (a few rows in decode) meet the whole weight matrix of that expert: the
// work is bound by reading packed weights once.  One wavefront owns two 16-row weight tiles
// and streams them along its k-slice with two tiles in flight; the lanes' packed codes are already
// ordered as matrix-core operands, so a tile goes
//     16-byte load -> a handful of bit operations -> bf16 MFMA
// with no shuffles, and the weights never touch LDS.  The bucket's activation rows march through LDS
// in double-buffered chunks shared by the 8 waves of a work-group (one barrier per chunk), so rows of
// any length stream without a restart.  Integer codes enter the matrix cores exactly, as the bf16
// value BASE + c/2 (or c for 8-bit codes), i.e. with a constant offset; a second MFMA against an
// all-ones operand gives the row sums of the activations over the same columns, which removes offset
// and zero-point exactly: sum_k x (off + c) - (off + z) sum_k x.  The fp32 scale multiplies the
// fp32 partial sum of each group, so no weight is ever rounded.
#include "qgemm_device.h"

#include <algorithm>

namespace moqe {

// Launch geometry: experts in the order their work-groups are laid out (heaviest first), work-groups per expert.
struct StreamLdsGeom { int32_t order[MOQE_MAX_EXPERTS]; int32_t wg_per_expert; };

namespace lds_stream {
constexpr int NS = 2;        // weight tiles (streams) per wave
constexpr int MT = 2;        // 16-row activation tiles per pass (32 bucket rows)

// Work-group geometry: 8 waves = WN tasks x WK k-slices (WK = 2 or 4, chosen per launch).  A task is a pair
// of weight tiles; slice ks of a task covers the k-tiles [ks*ceil(KT/WK), ...).  The activation
// rows of the pass (at most 32) are staged in LDS in chunks of CH = 8/WK k-tiles per slice,
// double-buffered, and shared by all waves, so activations cross the L2 once per work-group
// instead of once per wave and the work-group meets at a barrier once per chunk only: while a
// chunk is multiplied, each step copies one k-tile of the next chunk into the other buffer.
// Inside the tile loop every global load is unconditional (addresses are clamped, unused data is
// masked), which lets the compiler keep the whole prefetch ring in flight instead of draining
// it at control-flow joins.
constexpr int ROWS = 16 * MT;                 // bucket rows per pass
constexpr int WAVES = 8;                      // waves per work-group
constexpr int A_SLOT = 256;                   // LDS bytes per staged row and k-tile (int8 rows use half)

// A staged row is 16 units of 16 bytes; unit u of row r is stored at position u ^ (r & 15), which
// keeps the 16-byte-per-lane operand reads (16 rows x 4 units per instruction) free of bank conflicts.
static __device__ __forceinline__ int a_unit_pos(int row, int unit) { return (unit ^ (row & 15)) * 16; }

// LDS bytes: two buffers of (WK slices x CH k-tiles = 8) x ROWS rows; the k-slice reduction reuses them.
static constexpr int LDS_BYTES = 2 * 8 * ROWS * A_SLOT;

template <int FMT, int GM, bool GATEUP, int WK>
static __device__ __forceinline__ void stream_lds_task(const GemmArgs& ga, const ExpertDev& ex, const int off_e, const int M_e,
                                                   const int wgi, uint8_t* lds) {
  constexpr bool A8 = (FMT == FMT_I8A8);
  // tiles in flight per stream (a deeper ring was measured and bought nothing)
  constexpr int PF = 2;
  constexpr int CH = 8 / WK;                  // k-tiles per staged chunk and slice
  constexpr int U = PF > CH ? PF : CH;        // steps per loop iteration: ring slot and chunk position are static
  static_assert(U % PF == 0 && U % CH == 0, "the unrolled loop indexes the prefetch ring and the chunk statically");
  constexpr int NR = Raw<FMT>::N;
  constexpr int GPT = GM == GM_PC ? 0 : (GM == GM_G128 ? 1 : 2);
  constexpr int EB = A8 ? 1 : 2;              // bytes per activation element
  constexpr int nthreads = WAVES * 64;
  const int tid = threadIdx.x;
  // the wave index is uniform over the wave: telling the compiler so keeps everything derived
  // from it (task, k-slice, tile addresses) in scalar registers
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lr = lane & 15, lq = lane >> 4;
  const int KT = ga.k >> 7, NT = ga.n >> 4;
  const int T = ga.T;
  constexpr int wk = WK;
  constexpr int WN = WAVES / WK;                // tasks per work-group

  const int ks = wave % wk;
  const int task = wgi * WN + wave / wk;
  const int ntasks = GATEUP ? NT : (NT + 1) / 2;
  const bool active_task = task < ntasks;

  int nt[NS];
  bool sv[NS];
  const uint8_t* blob[NS];
  if constexpr (GATEUP) {
    nt[0] = nt[1] = task; sv[0] = sv[1] = active_task;
    blob[0] = ex.w[0]; blob[1] = ex.w[1];
  } else {
    nt[0] = 2 * task; nt[1] = 2 * task + 1;
    sv[0] = active_task && nt[0] < NT; sv[1] = active_task && nt[1] < NT;
    blob[0] = blob[1] = ex.w[0];
  }
  // weights are read through buffer descriptors: scalar tile offset + lane offset, no vector address arithmetic
  const buf_rsrc rsrc[NS] = {blob_rsrc(blob[0]), blob_rsrc(blob[1])};
  const int slice_tiles = (KT + wk - 1) / wk;              // k-tiles per slice (last slice may be shorter)
  const int kt0 = ks * slice_tiles, kt1 = min(KT, kt0 + slice_tiles);
  constexpr int KC = 128;                                  // columns staged per slice and step
  constexpr int buf_bytes = wk * CH * ROWS * A_SLOT;
  // streams without a tile of their own (odd tile count, padding tasks) and waves whose slice is
  // empty still run the loop on clamped addresses; their results are never stored
  const int nt_ld[NS] = {sv[0] ? nt[0] : 0, sv[1] ? nt[1] : 0};
  const int kt_last = max(kt0, kt1 - 1) < KT ? max(kt0, kt1 - 1) : KT - 1;

  // ---- weight ring; its first tile is requested right here, before the bucket's size is looked at and before
  // the staging plan: nothing in the request depends on them, and the tile is the longest wait of the set-up
  uint32_t raw[PF][NS][NR];
  float sc[PF][NS][GPT ? GPT : 1];
  uint16_t zp[PF][NS];      // as loaded: widened where it is used, so that nothing between request and use touches it

  auto issue_w = [&](int p, int kt_want) {
    const int kt = min(kt_want, kt_last);
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const uint32_t t = uint32_t(nt_ld[s]) * uint32_t(KT) + uint32_t(kt);          // uniform; byte offsets fit 32 bits
      load_raw<FMT>(raw[p][s], rsrc[s], t * ex.tile_bytes, lane);
      if constexpr (GPT > 0) {          // group formats are asymmetric: scale and zero-point per group
        if constexpr (GPT == 1) {
          sc[p][s][0] = __uint_as_float(buf_load32(rsrc[s], lr * 4, ex.scale_off + t * 64u));
          zp[p][s] = uint16_t(__builtin_amdgcn_raw_buffer_load_b8(rsrc[s], lr, int(ex.zero_off + t * 16u), 0));
        } else {
          const u32x2 v = buf_load64(rsrc[s], lr * 8, ex.scale_off + t * 128u);
          sc[p][s][0] = __uint_as_float(v.x); sc[p][s][1] = __uint_as_float(v.y);
          zp[p][s] = uint16_t(__builtin_amdgcn_raw_buffer_load_b16(rsrc[s], lr * 2, int(ex.zero_off + t * 32u), 0));
        }
      }
    }
  };

  issue_w(0, kt0);
  if (M_e <= 0 || M_e < ga.min_rows || M_e > ga.max_rows) return;     // uniform over the work-group (one expert per work-group)

  // sum_k x (c - z) = (1/CM) * (sum_k x (BASE + CM c) - (BASE + CM z) sum_k x)
  constexpr float BASE = CodeMap<FMT>::BASE, CM = CodeMap<FMT>::CM, INV_CM = 1.f / CodeMap<FMT>::CM;
  const float off_sym = BASE + CM * float(ex.zc);
  const FragK<FMT> fk = frag_constants<FMT>();
  const u32x4 ones = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
  const bf16x8 ones_b = __builtin_bit_cast(bf16x8, ones);

  // ---- staging plan: which 16-byte units of a chunk this thread copies -----------------------
  constexpr int upr = KC * EB / 16;                        // units per row
  constexpr int n_units = wk * ROWS * upr;
  constexpr int AU_MAX = n_units >= nthreads ? n_units / nthreads : 1;   // 16-byte units per thread and step
  static_assert(n_units % nthreads == 0 || n_units * 2 == nthreads, "whole units per thread, or half the threads idle");
  constexpr bool ALL_STAGE = n_units >= nthreads;          // false: only the lower half of the threads stages

  for (int pass0 = 0; pass0 < M_e; pass0 += ROWS) {
    const int rows_here = min(ROWS, M_e - pass0);
    // Per staged unit: byte offset of its step-0 source from the activation base, and the largest
    // step offset that stays inside the unit's slice.  Nothing is zero-filled: rows past the end of
    // the bucket repeat its last row (their products land in result rows that are never stored), and
    // steps past the end of a slice re-read its last tile and are not multiplied.
    // the activation matrix is smaller than 4 GiB (checked before the launch): 32-bit offsets through a descriptor
    const buf_rsrc a_rsrc = blob_rsrc(reinterpret_cast<const uint8_t*>(A8 ? static_cast<const void*>(ga.a_q) : ga.a));
    uint32_t uoff[AU_MAX];
    int ukend[AU_MAX];
    int32_t src_row[AU_MAX];               // source row of the unit in the activation matrix
#pragma unroll
    for (int i = 0; i < AU_MAX; ++i) {
      const int u = tid + i * nthreads;
      const int row = (u % (ROWS * upr)) / upr;
      src_row[i] = off_e * T + pass0 + min(row, rows_here - 1);
    }
    if constexpr (!A8) {
      if (ga.a_perm != nullptr) {          // uniform; all gather indices requested before any of them is used
        int32_t g[AU_MAX];
#pragma unroll
        for (int i = 0; i < AU_MAX; ++i) {
          const int mc = src_row[i] - off_e * T;
          g[i] = ga.a_perm[off_e + (T == 1 ? mc : mc / T)];
        }
#pragma unroll
        for (int i = 0; i < AU_MAX; ++i) {
          const int mc = src_row[i] - off_e * T;
          src_row[i] = T == 1 ? g[i] : g[i] * T + (mc % T);
        }
      }
    }
#pragma unroll
    for (int i = 0; i < AU_MAX; ++i) {
      const int u = tid + i * nthreads;
      uoff[i] = 0u; ukend[i] = 0;
      if (ALL_STAGE || u < n_units) {
        const int sl = u / (ROWS * upr), cu = u % upr;
        const int sk0 = min(sl * slice_tiles, KT - 1), sk1 = min(KT, sl * slice_tiles + slice_tiles);
        uoff[i] = (uint32_t(src_row[i]) * uint32_t(ga.k) + uint32_t(sk0) * 128u) * uint32_t(EB) + uint32_t(cu) * 16u;   // < 4 GiB
        ukend[i] = max(sk1 - sk0 - 1, 0) * 128 * EB;      // offset of the slice's last tile
      }
    }
    u32x4 areg[2][AU_MAX];                 // two sets: a k-tile is requested one step before it is stored
    auto a_fetch = [&](int set, int c) {   // global -> registers, k-tile c of every slice
      const int koff = c * KC * EB;
#pragma unroll
      for (int i = 0; i < AU_MAX; ++i)
        areg[set][i] = buf_load128(a_rsrc, int(uoff[i] + uint32_t(min(koff, ukend[i]))), 0u);
    };
    auto a_store = [&](int set, uint8_t* dst) {     // registers -> LDS; dst = buffer + k-tile position inside the chunk
#pragma unroll
      for (int i = 0; i < AU_MAX; ++i) {
        const int u = tid + i * nthreads;
        const int sl = u / (ROWS * upr), rem = u % (ROWS * upr), row = rem / upr, cu = rem % upr;
        if (ALL_STAGE || u < n_units)
          *reinterpret_cast<u32x4*>(dst + (sl * CH * ROWS + row) * A_SLOT + a_unit_pos(row, cu)) = areg[set][i];
      }
    };

    f32x4 tot[NS][MT];     // bf16 path: fp32 results; int8 path: int32 bit patterns
    f32x4 xs_tot[MT];      // per-channel formats: running row sums of the activations
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      xs_tot[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s = 0; s < NS; ++s) tot[s][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // One k-tile: activation operands come from LDS (tile `tl` of the current chunk buffer).
    auto consume = [&](int p, const uint8_t* abuf) {
      const uint8_t* arow0 = abuf + (ks * CH * ROWS + lr) * A_SLOT;      // row lr: unit u sits at (u ^ lr) * 16
      if constexpr (A8) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          if (mt * 16 < rows_here) {
            i32x4 a0 = *reinterpret_cast<const i32x4*>(arow0 + mt * 16 * A_SLOT + ((lq ^ lr) * 16));
            i32x4 a1 = *reinterpret_cast<const i32x4*>(arow0 + mt * 16 * A_SLOT + (((4 + lq) ^ lr) * 16));
#pragma unroll
            for (int s = 0; s < NS; ++s) {
              i32x4 acc = __builtin_bit_cast(i32x4, tot[s][mt]);
              i32x4 b0 = {int(raw[p][s][0]), int(raw[p][s][1]), int(raw[p][s][2]), int(raw[p][s][3])};
              i32x4 b1 = {int(raw[p][s][4]), int(raw[p][s][5]), int(raw[p][s][6]), int(raw[p][s][7])};
              acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(a0, b0, acc, 0, 0, 0);
              acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(a1, b1, acc, 0, 0, 0);
              tot[s][mt] = __builtin_bit_cast(f32x4, acc);
            }
          }
        }
      } else {
        // The operands of the activations are read from LDS once per k-tile, all of them at the top and without a
        // branch around them (rows past the end of the bucket repeat its last row), and meet both weight streams:
        // read where they were used, inside the per-block branches, every read was followed by a wait for it.
        u32x4 aop[MT][4];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int j = 0; j < 4; ++j)
            aop[mt][j] = *reinterpret_cast<const u32x4*>(arow0 + mt * 16 * A_SLOT + (((j * 4 + lq) ^ lr) * 16));
        f32x4 xs[MT][GPT ? GPT : 1];
#pragma unroll
        for (int s = 0; s < NS; ++s) {
          const bf16x8 b0 = frag<FMT, 0>(raw[p][s], fk);
          const bf16x8 b1 = frag<FMT, 1>(raw[p][s], fk);
          const bf16x8 b2 = frag<FMT, 2>(raw[p][s], fk);
          const bf16x8 b3 = frag<FMT, 3>(raw[p][s], fk);
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            if (mt * 16 < rows_here) {
              const u32x4 a0 = aop[mt][0], a1 = aop[mt][1], a2 = aop[mt][2], a3 = aop[mt][3];
              const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
              if (s == 0) {                 // row sums of the activations over the tile's groups, once per tile
                if constexpr (GM == GM_PC) {
                  xs_tot[mt] = mfma_bf16(a0, ones_b, xs_tot[mt]);
                  xs_tot[mt] = mfma_bf16(a1, ones_b, xs_tot[mt]);
                  xs_tot[mt] = mfma_bf16(a2, ones_b, xs_tot[mt]);
                  xs_tot[mt] = mfma_bf16(a3, ones_b, xs_tot[mt]);
                } else if constexpr (GM == GM_G128) {
                  f32x4 v = mfma_bf16(a0, ones_b, zero);
                  v = mfma_bf16(a1, ones_b, v);
                  v = mfma_bf16(a2, ones_b, v);
                  xs[mt][0] = mfma_bf16(a3, ones_b, v);
                } else {
                  xs[mt][0] = mfma_bf16(a1, ones_b, mfma_bf16(a0, ones_b, zero));
                  xs[mt][GPT == 2 ? 1 : 0] = mfma_bf16(a3, ones_b, mfma_bf16(a2, ones_b, zero));
                }
              }
              if constexpr (GM == GM_PC) {
                f32x4 v = tot[s][mt];
                v = mfma_bf16(a0, b0, v);
                v = mfma_bf16(a1, b1, v);
                v = mfma_bf16(a2, b2, v);
                v = mfma_bf16(a3, b3, v);
                tot[s][mt] = v;
              } else if constexpr (GM == GM_G128) {
                f32x4 v = mfma_bf16(a0, b0, zero);
                v = mfma_bf16(a1, b1, v);
                v = mfma_bf16(a2, b2, v);
                v = mfma_bf16(a3, b3, v);
                const float o = BASE + CM * float(uint32_t(zp[p][s]) & 0xffu);
                const float scv = sc[p][s][0] * INV_CM;
#pragma unroll
                for (int r = 0; r < 4; ++r) tot[s][mt][r] += scv * (v[r] - o * xs[mt][0][r]);
              } else {
                f32x4 v0 = mfma_bf16(a1, b1, mfma_bf16(a0, b0, zero));
                f32x4 v1 = mfma_bf16(a3, b3, mfma_bf16(a2, b2, zero));
                const float o0 = BASE + CM * float(uint32_t(zp[p][s]) & 0xffu);
                const float o1 = BASE + CM * float((uint32_t(zp[p][s]) >> 8) & 0xffu);
                const float s0 = sc[p][s][0] * INV_CM, s1 = sc[p][s][GPT == 2 ? 1 : 0] * INV_CM;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                  tot[s][mt][r] += s0 * (v0[r] - o0 * xs[mt][0][r]);
                  tot[s][mt][r] += s1 * (v1[r] - o1 * xs[mt][GPT == 2 ? 1 : 0][r]);
                }
              }
            }
          }
        }
      }
    };

    // What the epilogue needs from global memory is requested here, ahead of the tile loop, so that the end of the
    // kernel waits for no load: the destination rows of the scatter, per-channel scales, the row scales of int8
    // activations (rows past the end of the bucket take the last row's, and are never stored).
    int32_t out_row[MT][4];
    float sx_row[MT][4];
    float pcs[NS] = {1.f, 1.f};
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int mc = min(pass0 + mt * 16 + lq * 4 + r, M_e - 1);
        out_row[mt][r] = off_e * T + mc;
        sx_row[mt][r] = 1.f;
        if constexpr (A8) sx_row[mt][r] = ga.a_scale[size_t(off_e) * T + mc];
      }
    if constexpr (!GATEUP) {
      if (ga.y_perm != nullptr) {          // uniform branches: one sample per row group is the common case
        if (T == 1) {
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 4; ++r) out_row[mt][r] = ga.y_perm[out_row[mt][r]];
        } else {
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const int mc = out_row[mt][r] - off_e * T;
              out_row[mt][r] = ga.y_perm[off_e + mc / T] * T + (mc % T);
            }
        }
      }
    }
    if constexpr (GM == GM_PC) {
#pragma unroll
      for (int s = 0; s < NS; ++s) pcs[s] = __uint_as_float(buf_load32(rsrc[s], lr * 4, ex.scale_off + uint32_t(nt_ld[s]) * 64u));
    }

    // ---- prologue: (the first weight tile is in flight) the first chunk of the activations into LDS; then the
    // requests the first step expects behind it, in the order a step leaves them.  The waits of the loop are
    // counts of requests still in flight, fixed when the kernel is compiled and valid for the way in from here
    // as well as for the way round the loop: with any other order here, every step would wait for loads that
    // the step before has only just requested.
    if (pass0 > 0) issue_w(0, kt0);
#pragma unroll
    for (int c = 0; c < CH; c += 2) {
      a_fetch(0, c);
      if (c + 1 < CH) a_fetch(1, c + 1);
      a_store(0, lds + c * ROWS * A_SLOT);
      if (c + 1 < CH) a_store(1, lds + (c + 1) * ROWS * A_SLOT);
    }
    __builtin_amdgcn_sched_barrier(0);
    a_fetch(0, CH);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int p = 1; p < PF; ++p) issue_w(p, kt0 + p);
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();

    // ---- main loop over the slice's k-tiles: step ti requests the activations of tile ti+CH+1, multiplies
    // tile ti, requests weight tile ti+PF and stores the activations of tile ti+CH (the same position in the next
    // chunk, requested during the step before) into the other LDS buffer.  Loads complete in the order of their
    // requests, so a wait for one of them is a wait for everything requested before it: with the activations
    // requested a step ahead of their store, that wait covers only weight tiles that have been multiplied
    // already, and the tiles requested last keep their full lead.  U tiles per iteration so that the ring
    // slot, the register set and the position inside the chunk are static; the work-group meets once per
    // chunk.  Tiles past the end of a shorter slice are skipped (uniform over the wave).
    static_assert(U % 2 == 0, "the register set of the staged activations alternates with the step");
    auto step = [&](int ti, int i) {                        // i = ti % U, known at compile time where it matters
      const int cur = (ti / CH) & 1;
      uint8_t* const rd = lds + cur * buf_bytes + (i % CH) * ROWS * A_SLOT;
      uint8_t* const wr = lds + (cur ^ 1) * buf_bytes + (i % CH) * ROWS * A_SLOT;
      a_fetch((i + 1) & 1, ti + CH + 1);
      if (kt0 + ti < kt1) consume(i % PF, rd);
      issue_w(i % PF, kt0 + ti + PF);
      a_store(i & 1, wr);
      if ((i + 1) % CH == 0) __syncthreads();
      __builtin_amdgcn_sched_barrier(0);                    // keep the steps apart: their temporaries must not pile up
    };
    int tb = 0;
#pragma unroll 1
    for (; tb + U <= slice_tiles; tb += U) {
#pragma unroll
      for (int i = 0; i < U; ++i) step(tb + i, i);
    }
#pragma unroll
    for (int i = 0; i < U - 1; ++i)
      if (tb + i < slice_tiles) step(tb + i, i);            // uniform over the work-group
    __syncthreads();                                        // all reads of the staged rows are done

    // ---- combine the k-slices of a task (fixed order), then the epilogue -------------------
    if (wk > 1) {
      float* red = reinterpret_cast<float*>(lds);
      constexpr int SLOT = (NS * MT + MT) * 4 * 64;
      float* mine = red + size_t(wave) * SLOT;
      if (ks > 0) {
#pragma unroll
        for (int s = 0; s < NS; ++s)
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 4; ++r) mine[((s * MT + mt) * 4 + r) * 64 + lane] = tot[s][mt][r];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int r = 0; r < 4; ++r) mine[((NS * MT + mt) * 4 + r) * 64 + lane] = xs_tot[mt][r];
      }
      __syncthreads();
      if (ks == 0) {
        for (int o = 1; o < wk; ++o) {
          const float* other = red + size_t(wave + o) * SLOT;
#pragma unroll
          for (int s = 0; s < NS; ++s)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
              for (int r = 0; r < 4; ++r) {
                const float v = other[((s * MT + mt) * 4 + r) * 64 + lane];
                if constexpr (A8) tot[s][mt][r] = __int_as_float(__float_as_int(tot[s][mt][r]) + __float_as_int(v));
                else tot[s][mt][r] += v;
              }
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 4; ++r) xs_tot[mt][r] += other[((NS * MT + mt) * 4 + r) * 64 + lane];
        }
      }
    }

    if (ks == 0 && (sv[0] || sv[1])) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int m = pass0 + mt * 16 + lq * 4 + r;
          if (m < M_e) {
            float val[NS];
#pragma unroll
            for (int s = 0; s < NS; ++s) {
              if constexpr (A8) {
                val[s] = float(__float_as_int(tot[s][mt][r])) * sx_row[mt][r] * pcs[s];
              } else if constexpr (GM == GM_PC) {
                val[s] = (pcs[s] * INV_CM) * (tot[s][mt][r] - off_sym * xs_tot[mt][r]);
              } else {
                val[s] = tot[s][mt][r];
              }
            }
            const size_t brow = size_t(off_e) * T + m;
            if constexpr (GATEUP) {
              if (sv[0]) {
                uint16_t* h = static_cast<uint16_t*>(ga.y);
                h[brow * size_t(ga.n) + nt[0] * 16 + lr] = float_to_bf16_rne(silu_mul(val[0], val[1]));
              }
            } else {
              const size_t drow = size_t(out_row[mt][r]);
              if (ga.y_bf16) {
                uint16_t* y = static_cast<uint16_t*>(ga.y) + drow * size_t(ga.n);
                if (sv[0]) y[nt[0] * 16 + lr] = float_to_bf16_rne(val[0]);
                if (sv[1]) y[nt[1] * 16 + lr] = float_to_bf16_rne(val[1]);
              } else {
                float* y = static_cast<float*>(ga.y) + drow * size_t(ga.n);
                if (sv[0]) y[nt[0] * 16 + lr] = val[0];
                if (sv[1]) y[nt[1] * 16 + lr] = val[1];
              }
            }
          }
        }
      }
    }
    __syncthreads();                             // LDS is reused by the next pass
  }
}

}  // namespace lds_stream
using namespace lds_stream;

template <bool GATEUP, int WK>
__global__ __launch_bounds__(WAVES * 64, 2) void k_qgemm_stream_lds(const GemmArgs ga, const StreamLdsGeom geo) {
  extern __shared__ __align__(16) uint8_t lds[];
  // grid: x = work-group of the expert, y = the expert's place in `order` (no division, and nothing to wait for
  // before the expert is known)
  const int e = geo.order[blockIdx.y];
  const int wgi = blockIdx.x;
  const ExpertDev& ex = ga.ex[e];
  // the bucket's place is read here, before the branch on the format: its load travels together with the loads of
  // the expert's description instead of after them
  const int off_e = ga.offsets[e];
  const int M_e = (ga.offsets[e + 1] - off_e) * ga.T;
  switch (ex.fmt * 4 + ex.gm) {
    case FMT_I8 * 4 + GM_PC:     stream_lds_task<FMT_I8, GM_PC, GATEUP, WK>(ga, ex, off_e, M_e, wgi, lds); break;
    case FMT_I8A8 * 4 + GM_PC:   stream_lds_task<FMT_I8A8, GM_PC, GATEUP, WK>(ga, ex, off_e, M_e, wgi, lds); break;
    case FMT_N6 * 4 + GM_PC:     stream_lds_task<FMT_N6, GM_PC, GATEUP, WK>(ga, ex, off_e, M_e, wgi, lds); break;
    case FMT_N4 * 4 + GM_PC:     stream_lds_task<FMT_N4, GM_PC, GATEUP, WK>(ga, ex, off_e, M_e, wgi, lds); break;
    case FMT_N4 * 4 + GM_G128:   stream_lds_task<FMT_N4, GM_G128, GATEUP, WK>(ga, ex, off_e, M_e, wgi, lds); break;
    case FMT_N4 * 4 + GM_G64:    stream_lds_task<FMT_N4, GM_G64, GATEUP, WK>(ga, ex, off_e, M_e, wgi, lds); break;
    case FMT_N3 * 4 + GM_G128:   stream_lds_task<FMT_N3, GM_G128, GATEUP, WK>(ga, ex, off_e, M_e, wgi, lds); break;
    case FMT_N3 * 4 + GM_G64:    stream_lds_task<FMT_N3, GM_G64, GATEUP, WK>(ga, ex, off_e, M_e, wgi, lds); break;
    default: break;
  }
}

typedef void (*StreamLdsKernel)(const GemmArgs, const StreamLdsGeom);

int32_t launch_qgemm_stream_lds(const GemmArgs& ga, bool gateup, hipStream_t st) {
  // this kernel reads `a` as a plain [rows, k] matrix; an image that still needs its 3x3 gather must not get here
  if (ga.conv_c != 0) return set_error(MOQE_E_SHAPE, "grouped_qgemm: the streaming kernel cannot gather a convolution's rows");
  const int NT = ga.n / 16, KT = ga.k / 128;
  const int ntasks = gateup ? NT : (NT + 1) / 2;
  // Long rows are cut into four k-slices per task, short ones into two: a wave should keep a
  // dozen or more tiles to amortise its set-up, and there should be a few work-groups per CU.
  const int wk = KT >= 64 ? 4 : 2;
  const int wn = WAVES / wk;
  StreamLdsGeom geo;
  geo.wg_per_expert = (ntasks + wn - 1) / wn;
  // heaviest experts first, so that the long tasks start early
  int idx[MOQE_MAX_EXPERTS];
  for (int i = 0; i < MOQE_MAX_EXPERTS; ++i) idx[i] = i;
  std::stable_sort(idx, idx + ga.n_experts, [&](int a, int b) { return ga.ex[a].tile_bytes > ga.ex[b].tile_bytes; });
  for (int i = 0; i < MOQE_MAX_EXPERTS; ++i) geo.order[i] = idx[i];
  const int slot_bytes = (NS * MT + MT) * 4 * 64 * 4;
  int lds_bytes = LDS_BYTES;
  if (WAVES * slot_bytes > lds_bytes) lds_bytes = WAVES * slot_bytes;
  const int ki = (gateup ? 2 : 0) + (wk == 4 ? 1 : 0);
  static const StreamLdsKernel kernels[4] = {k_qgemm_stream_lds<false, 2>, k_qgemm_stream_lds<false, 4>, k_qgemm_stream_lds<true, 2>,
                                             k_qgemm_stream_lds<true, 4>};
  int32_t rc = ensure_dynamic_lds(LDSK_STREAM0 + 2 + ki, reinterpret_cast<const void*>(kernels[ki]), LDS_BYTES, "grouped_qgemm");
  if (rc) return rc;
  ProfileScope ps(gateup ? MOQE_PK_GEMM_GATEUP : MOQE_PK_GEMM_PLAIN, st, true);
  ps.launch(kernels[ki], dim3(unsigned(geo.wg_per_expert), unsigned(ga.n_experts)), dim3(WAVES * 64), lds_bytes, ga, geo);
  return check_launch("grouped_qgemm");
}

}  // namespace moqe
