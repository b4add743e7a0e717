// Grouped dequantize-GEMM, tile kernel for large buckets (prefill, images).
//
// Each sample is processed by its selected expert only (MoQE Section 3.1); when an expert's bucket
// holds hundreds of rows the work is a dense contraction and belongs on the matrix cores.  A
// work-group of 4 waves owns 64 bucket rows x 256 weight rows of one expert (for the SiLU-gated
// pair: 128 gate rows and the 128 up rows of the same features, so the gate meets its up value in
// registers); a wave owns 64 x 64.  Two work-groups share a CU (256 registers per wave) and meet at
// their barriers independently, so one computes while the other waits.
//
//  * Activations: the 64 x 128 tile of a k-step is gathered through the permutation into
//    registers and written to LDS (rows of 256 bytes, 16-byte units XOR-swizzled by the row so
//    that the 16-byte-per-lane operand reads are free of bank conflicts), double-buffered, one
//    barrier per k-step.
//  * Weights never touch LDS: the packed layout already is the matrix-core operand order, so each
//    wave loads the four packed 16-row tiles of its 64 weight rows with one coalesced 16-byte-per-
//    lane load each (two k-steps ahead) and unpacks them in registers to exact bf16 operands
//    BASE + c/2.  LDS traffic is thus one 16-byte read per lane for every four matrix-core
//    operations.
//  * Offset and zero-point are removed with the row sums of the activations (an MFMA against
//    ones), as in the streaming kernel.  Per-group scales use ONE accumulator: entering group g
//    the accumulator is multiplied by s_{g-1}/s_g, so that it always holds the sum in units of the
//    current group's scale, and the last scale multiplies the result.  No weight is rounded; the
//    extra roundings are one fp32 multiply per group on the accumulator.
#include "qgemm_device.h"

#include <algorithm>
#include <cstring>

namespace moqe {

constexpr int TBM = 64;                  // bucket rows per work-group tile
constexpr int TWM = 1, TWN = 4;          // waves along rows / weight rows
constexpr int TWAVES = TWM * TWN;
constexpr int TMB = 4, TNB = 4;          // 16 x 16 blocks per wave: 64 rows x 64 weight rows
constexpr int TBN = TWN * TNB * 16;      // 256 weight rows per work-group tile
constexpr int T_SLOT = 256;              // LDS bytes per staged row and k-step (int8 rows use half)
constexpr int T_LDS_BYTES = 2 * TBM * T_SLOT;

// What the launcher works out on the host for one launch.
struct TileGeom {
  uint64_t order_bits;                // 4 bits per position: experts in the order their row tiles are enumerated, dearest format first
  int32_t  patch_n_log2;              // a patch is 2^patch_n_log2 weight tiles x PATCH_M row tiles
  uint32_t conv_c_magic;              // ceil(2^32 / conv_c): column / conv_c = umulhi(column, magic) for every column < 9 * conv_c
};

template <int FMT, int GM, bool GATEUP, bool CONV>
static __device__ __forceinline__ void tile_task(const GemmArgs& ga, const TileGeom& tg, const ExpertDev& ex, const int off_e, const int M_e,
                                                 const int m0, const int ntile, uint8_t* lds) {
  constexpr bool A8 = (FMT == FMT_I8A8);
  constexpr int NR = Raw<FMT>::N;
  constexpr int GPT = GM == GM_PC ? 0 : (GM == GM_G128 ? 1 : 2);
  constexpr int EB = A8 ? 1 : 2;
  constexpr int A_UNITS = 128 * EB / 16;             // 16-byte units per activation row and k-step
  constexpr int A_ROWS_PER_IT = TWAVES * 64 / A_UNITS;
  constexpr int A_ITERS = TBM / A_ROWS_PER_IT;
  constexpr float BASE = CodeMap<FMT>::BASE, CM = CodeMap<FMT>::CM, INV_CM = 1.f / CodeMap<FMT>::CM;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);       // uniform: keeps tile addresses scalar
  const int lr = lane & 15, lq = lane >> 4;
  const int wm = wave / TWN, wn = wave % TWN;
  const int KT = ga.k >> 7, NT = ga.n >> 4;
  const int T = ga.T;
  const float off_sym = BASE + CM * float(ex.zc);
  const FragK<FMT> fk = frag_constants<FMT>();

  // ---- the four packed weight tiles of this wave (16 weight rows each) -----------------------------
  const uint8_t* blob[TNB];
  uint32_t tbase[TNB];                        // index of the tile's first k-step inside the blob
  int ncol[TNB];                              // weight row (plain) / feature (gate-up) of block b at lane column lr
  bool nok[TNB];
#pragma unroll
  for (int b = 0; b < TNB; ++b) {
    int nt16;
    if constexpr (GATEUP) {
      nt16 = ntile * 8 + wn * 2 + (b & 1);    // blocks 0,1: gate rows; blocks 2,3: up rows of the same features
      blob[b] = ex.w[b >> 1];
    } else {
      nt16 = ntile * 16 + wn * 4 + b;
      blob[b] = ex.w[0];
    }
    nok[b] = nt16 < NT;
    ncol[b] = nt16 * 16 + lr;
    tbase[b] = uint32_t((nok[b] ? nt16 : 0) * KT);      // clamped: rows outside the matrix are computed on other rows' codes, never stored
  }

  // ---- activation rows this thread copies per k-step ------------------------------------------------
  // activations and weights are read through buffer descriptors (each matrix is smaller than 4 GiB, checked before
  // the launch): 32-bit offsets, a scalar one and a per-lane one, and no 64-bit address arithmetic in the vector unit
  const uint8_t* abase = reinterpret_cast<const uint8_t*>(A8 ? static_cast<const void*>(ga.a_q) : ga.a);
  const buf_rsrc a_rsrc = blob_rsrc(abase);
  const buf_rsrc w_rsrc[2] = {blob_rsrc(ex.w[0]), blob_rsrc(ex.w[GATEUP ? 1 : 0])};
  uint32_t a_off[A_ITERS];
  const int a_unit = tid % A_UNITS, a_row0 = tid / A_UNITS;
  uint32_t a_taps[CONV ? A_ITERS : 1];       // convolution: bit t set = filter tap t of the row's pixel lies inside its image
  int32_t a_srow[A_ITERS];                   // source row of each copied row in the activation matrix
  int32_t a_rin[A_ITERS];                    // the row's place inside its sample (0 when samples have one row)
  const bool one_row = T == 1;               // uniform: the divisions below are some forty instructions each
#pragma unroll
  for (int i = 0; i < A_ITERS; ++i) {
    const int m = min(m0 + a_row0 + i * A_ROWS_PER_IT, M_e - 1);      // rows past the bucket repeat its last row
    const int smp = one_row ? m : m / T;
    a_rin[i] = one_row ? 0 : m - smp * T;
    a_srow[i] = off_e + smp;                 // the sample, for now
  }
  if constexpr (!A8) {
    if (ga.a_perm != nullptr) {              // uniform; all gather indices are requested before any of them is used
#pragma unroll
      for (int i = 0; i < A_ITERS; ++i) a_srow[i] = ga.a_perm[a_srow[i]];
    }
  }
#pragma unroll
  for (int i = 0; i < A_ITERS; ++i) {
    a_srow[i] = a_srow[i] * T + a_rin[i];
    // each matrix is smaller than 4 GiB: 32-bit byte offsets
    if constexpr (CONV && !A8) {
      a_off[i] = uint32_t(a_srow[i]) * uint32_t(ga.conv_c) * 2u;     // byte offset of the pixel in the NHWC image
      const int p = a_rin[i];                                         // the pixel inside its image
      const int py = p / ga.conv_w, px = p - py * ga.conv_w;
      uint32_t taps = 0;
#pragma unroll
      for (int t = 0; t < 9; ++t) {
        const int yy = py + t / 3 - 1, xx = px + t % 3 - 1;
        if (yy >= 0 && yy < ga.conv_h && xx >= 0 && xx < ga.conv_w) taps |= 1u << t;
      }
      a_taps[i] = taps;
    } else {
      a_off[i] = uint32_t(a_srow[i]) * uint32_t(ga.k) * uint32_t(EB) + uint32_t(a_unit) * 16u;
    }
  }
  // Where each of the tile's rows goes (and, for int8 activations, its scale): worked out now by the
  // first TBM threads, one row each, handed to every lane through LDS after the main loop.  -1: no such row.
  int my_drow = -1;
  float my_sx = 0.f;
  if (tid < TBM) {
    const int m = m0 + tid;
    if (m < M_e) {
      my_drow = off_e * T + m;
      if constexpr (A8) my_sx = ga.a_scale[my_drow];
      if constexpr (!GATEUP) {
        if (ga.y_perm) my_drow = ga.y_perm[off_e + m / T] * T + (m % T);
      }
    }
  }
  u32x4 a_reg[A_ITERS];
  uint32_t a_ok = 0u;                          // convolution: bit i = the tap of a_reg[i] lies inside the image
  // Convolution: the 8 columns of this thread's unit are 8 neighbouring channels of ONE filter tap
  // (k = tap * C + channel), i.e. 16 contiguous bytes of the pixel at that tap's offset, or zeros
  // outside the image.  Tap and channel follow from the unit's first column by one multiply-high.
  auto a_fetch = [&](int kt) {
    if constexpr (CONV && !A8) {
      const uint32_t col = uint32_t(kt) * 128u + uint32_t(a_unit) * 8u;
      const uint32_t tap = __umulhi(col, tg.conv_c_magic);           // k-steps past the end give taps >= 9: never multiplied
      const int ch = int(col - tap * uint32_t(ga.conv_c));
      const int ty = int((tap * 11u) >> 5);                           // tap / 3 for tap < 12
      const int dy = ty - 1, dx = int(tap) - ty * 3 - 1;
      const int delta = ((dy * ga.conv_w + dx) * ga.conv_c + ch) * 2;  // bytes from the row's pixel to the tap's channels
      const uint32_t bit = tap < 9u ? (1u << tap) : 0u;
      a_ok = 0u;
#pragma unroll
      for (int i = 0; i < A_ITERS; ++i) {
        const bool ok = (a_taps[i] & bit) != 0u;
        const uint32_t off = a_off[i] + uint32_t(ok ? delta : 0);     // always a valid address
        a_reg[i] = *reinterpret_cast<const u32x4*>(abase + off);
        a_ok |= ok ? (1u << i) : 0u;                                   // taps outside the image become zeros when the row is stored
      }
    } else {
      const uint32_t koff = uint32_t(min(kt, KT - 1)) * (128 * EB);
#pragma unroll
      for (int i = 0; i < A_ITERS; ++i) a_reg[i] = buf_load128(a_rsrc, int(a_off[i]), koff);
    }
  };
  auto a_store = [&](uint8_t* buf) {
#pragma unroll
    for (int i = 0; i < A_ITERS; ++i) {
      const int row = a_row0 + i * A_ROWS_PER_IT;
      u32x4 v = a_reg[i];
      if constexpr (CONV && !A8) {
        // the loaded words are first touched here, a k-step after the load was issued
        const bool ok = (a_ok >> i) & 1u;
        v.x = ok ? v.x : 0u; v.y = ok ? v.y : 0u; v.z = ok ? v.z : 0u; v.w = ok ? v.w : 0u;
      }
      *reinterpret_cast<u32x4*>(buf + row * T_SLOT + ((a_unit ^ (row & 15)) * 16)) = v;
    }
  };

  // ---- weight ring: two k-steps in flight ------------------------------------------------------------
  uint32_t raw[2][TNB][NR];
  float sc[2][TNB][GPT ? GPT : 1];
  uint32_t zp[2][TNB];
  auto issue_w = [&](int p, int kt_want) {
    const uint32_t kt = uint32_t(min(kt_want, KT - 1));
#pragma unroll
    for (int b = 0; b < TNB; ++b) {
      const uint32_t t = tbase[b] + kt;
      if constexpr (CONV) {
        // plain loads: with the descriptors the convolution's kernel ran out of registers (spills inside its loops)
        load_raw<FMT>(raw[p][b], blob[b] + t * ex.tile_bytes, lane);
        if constexpr (GPT > 0) {
          const uint8_t* sp = blob[b] + (ex.scale_off + t * uint32_t(16 * GPT * 4));
          const uint8_t* zq = blob[b] + (ex.zero_off + t * uint32_t(16 * GPT));
          if constexpr (GPT == 1) {
            sc[p][b][0] = *reinterpret_cast<const float*>(sp + uint32_t(lr) * 4u);
            zp[p][b] = *reinterpret_cast<const uint32_t*>(zq + (uint32_t(lr) & ~3u));
          } else {
            const float2 v = *reinterpret_cast<const float2*>(sp + uint32_t(lr) * 8u);
            sc[p][b][0] = v.x; sc[p][b][1] = v.y;
            zp[p][b] = *reinterpret_cast<const uint32_t*>(zq + ((uint32_t(lr) * 2u) & ~3u));
          }
        }
      } else {
        const buf_rsrc rs = w_rsrc[GATEUP ? (b >> 1) : 0];
        load_raw<FMT>(raw[p][b], rs, t * ex.tile_bytes, lane);
        if constexpr (GPT > 0) {
          // zero-points: the aligned dword holding the lane's byte(s), shifted down where it is used
          if constexpr (GPT == 1) {
            sc[p][b][0] = __uint_as_float(buf_load32(rs, lr * 4, ex.scale_off + t * 64u));
            zp[p][b] = buf_load32(rs, lr & ~3, ex.zero_off + t * 16u);
          } else {
            const u32x2 v = buf_load64(rs, lr * 8, ex.scale_off + t * 128u);
            sc[p][b][0] = __uint_as_float(v.x); sc[p][b][1] = __uint_as_float(v.y);
            zp[p][b] = buf_load32(rs, (lr * 2) & ~3, ex.zero_off + t * 32u);
          }
        }
      }
    }
  };
  const uint32_t zp_shift = GPT == 2 ? 16u * (uint32_t(lr) & 1u) : 8u * (uint32_t(lr) & 3u);

  f32x4 tot[TMB][TNB];        // bf16 path: fp32 sums in units of the current group's scale; int8 path: int32 bit patterns
  f32x4 xs_tot[TMB];          // per-channel formats: row sums of the activations over all of k
  float s_cur[TNB];           // scale of the group the accumulators are expressed in
#pragma unroll
  for (int mb = 0; mb < TMB; ++mb) {
    xs_tot[mb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int b = 0; b < TNB; ++b) tot[mb][b] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
#pragma unroll
  for (int b = 0; b < TNB; ++b) s_cur[b] = 1.f;
  const u32x4 ones = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
  const bf16x8 ones_b = __builtin_bit_cast(bf16x8, ones);
  const f32x4 zero = {0.f, 0.f, 0.f, 0.f};

  // One k-step: activation operands from LDS buffer `abuf`, weights from ring slot p.
  auto compute = [&](int p, const uint8_t* abuf) {
    // The ring values arrive through the loop's back edge; the fence keeps the optimizer from moving
    // arithmetic on them to the end of the previous iteration, right behind their loads.
#pragma unroll
    for (int b = 0; b < TNB; ++b) {
#pragma unroll
      for (int i = 0; i < NR; ++i) asm volatile("" : "+v"(raw[p][b][i]));
      if constexpr (GPT > 0) {
        asm volatile("" : "+v"(zp[p][b]));
#pragma unroll
        for (int g = 0; g < GPT; ++g) asm volatile("" : "+v"(sc[p][b][g]));
      }
    }
    const uint8_t* arow = abuf + (wm * 64 + lr) * T_SLOT;       // + mb * 16 rows; unit u of row lr sits at (u ^ lr) * 16
    if constexpr (A8) {
#pragma unroll
      for (int js = 0; js < 2; ++js) {
        i32x4 a[TMB];
#pragma unroll
        for (int mb = 0; mb < TMB; ++mb)
          a[mb] = *reinterpret_cast<const i32x4*>(arow + mb * 16 * T_SLOT + (((js * 4 + lq) ^ lr) * 16));
#pragma unroll
        for (int b = 0; b < TNB; ++b) {
          const i32x4 bv = {int(raw[p][b][js * 4 + 0]), int(raw[p][b][js * 4 + 1]), int(raw[p][b][js * 4 + 2]),
                            int(raw[p][b][js * 4 + 3])};
#pragma unroll
          for (int mb = 0; mb < TMB; ++mb)
            tot[mb][b] = __builtin_bit_cast(
                f32x4, __builtin_amdgcn_mfma_i32_16x16x64_i8(a[mb], bv, __builtin_bit_cast(i32x4, tot[mb][b]), 0, 0, 0));
        }
      }
    } else {
      constexpr int GSTEPS = GM == GM_G64 ? 2 : 4;     // matrix-core steps per quantization group
      f32x4 xs[TMB];
      auto do_j = [&](auto jc) {
        constexpr int J = decltype(jc)::value;
        if constexpr (GM != GM_PC && J % GSTEPS == 0) {     // entering a group: accumulators into its scale's units
          constexpr int G = J / GSTEPS;
#pragma unroll
          for (int b = 0; b < TNB; ++b) {
            const float s_new = sc[p][b][G < GPT ? G : 0];
            // s_cur / s_new from the hardware reciprocal and one Newton step (within an ulp or two of
            // the true quotient; any error only moves rounding points, the factor is applied and
            // divided out consistently)
            float rinv = __builtin_amdgcn_rcpf(s_new);
            rinv = fmaf(fmaf(-s_new, rinv, 1.0f), rinv, rinv);
            const float rho = s_cur[b] * rinv;
            s_cur[b] = s_new;
#pragma unroll
            for (int mb = 0; mb < TMB; ++mb)
#pragma unroll
              for (int r = 0; r < 4; ++r) tot[mb][b][r] *= rho;
          }
        }
        u32x4 a[TMB];
        bf16x8 bv[TNB];
#pragma unroll
        for (int mb = 0; mb < TMB; ++mb)
          a[mb] = *reinterpret_cast<const u32x4*>(arow + mb * 16 * T_SLOT + (((J * 4 + lq) ^ lr) * 16));
#pragma unroll
        for (int b = 0; b < TNB; ++b) bv[b] = frag<FMT, J>(raw[p][b], fk);
#pragma unroll
        for (int mb = 0; mb < TMB; ++mb) {
          if constexpr (GM == GM_PC) xs_tot[mb] = mfma_bf16(a[mb], ones_b, xs_tot[mb]);
          else xs[mb] = mfma_bf16(a[mb], ones_b, (J % GSTEPS == 0) ? zero : xs[mb]);
        }
#pragma unroll
        for (int b = 0; b < TNB; ++b)
#pragma unroll
          for (int mb = 0; mb < TMB; ++mb) {
            if constexpr (GM != GM_PC && J % GSTEPS == 0) {
              // The accumulator was just rewritten by vector arithmetic, so the matrix-core result may be
              // given other registers than its input.  Keeping the input alive across the operation
              // makes the two register ranges disjoint; the schedule the compiler then finds is also
              // the faster one (876 against 832 TFLOP/s on the prefill gate/up launch without it).
              const f32x4 c_in = tot[mb][b];
              tot[mb][b] = mfma_bf16(a[mb], bv[b], c_in);
              asm volatile("" :: "v"(c_in));
            } else {
              tot[mb][b] = mfma_bf16(a[mb], bv[b], tot[mb][b]);
            }
          }
        if constexpr (GM != GM_PC && (J + 1) % GSTEPS == 0) {   // leaving a group: remove offset and zero-point
          constexpr int G = J / GSTEPS;
#pragma unroll
          for (int b = 0; b < TNB; ++b) {
            const float o = BASE + CM * float(((zp[p][b] >> zp_shift) >> (8 * G)) & 0xffu);
#pragma unroll
            for (int mb = 0; mb < TMB; ++mb)
#pragma unroll
              for (int r = 0; r < 4; ++r) tot[mb][b][r] -= o * xs[mb][r];
          }
        }
      };
      do_j(std::integral_constant<int, 0>{});
      do_j(std::integral_constant<int, 1>{});
      do_j(std::integral_constant<int, 2>{});
      do_j(std::integral_constant<int, 3>{});
    }
  };

  // factor that turns the accumulator into the result; per-channel scales are requested here, ahead of the main
  // loop (these formats have no group scales in flight, so the registers are there), instead of at its end.
  // Not for the convolution, whose gather leaves no register free: it asks for them after the loop.
  constexpr bool FIN_EARLY = GM == GM_PC && !CONV;
  float fin[TNB];
  auto load_fin = [&]() {
#pragma unroll
    for (int b = 0; b < TNB; ++b)
      fin[b] = nok[b] ? reinterpret_cast<const float*>(blob[b] + ex.scale_off)[ncol[b]] : 1.f;
  };
  if constexpr (FIN_EARLY) load_fin();

  // ---- prologue: k-step 0 of the activations into LDS, k-step 1 in registers, two weight steps in flight.
  // The requests are left in the order a step of the loop leaves them (weights of the step after next, then the
  // next step's activations), with the first step's weights already there: the loop's waits are counts of requests
  // in flight, fixed at compile time for both ways into the loop's head, and with any other order here every
  // second step would wait for most of the weights requested half a step before.
  issue_w(0, 0);
  __builtin_amdgcn_sched_barrier(0);
  a_fetch(0);
  a_store(lds);                                     // loads complete in request order: the weights of step 0 are there too
  __builtin_amdgcn_sched_barrier(0);
  issue_w(1, 1);
  __builtin_amdgcn_sched_barrier(0);
  a_fetch(1);
  __syncthreads();
  __builtin_amdgcn_sched_barrier(0);

  // ---- main loop, two k-steps per iteration so that ring slot and LDS buffer are static ----------
  auto step = [&](int kt, int p) {
    compute(p, lds + p * (TBM * T_SLOT));
    issue_w(p, kt + 2);
    // the stored activations were requested a k-step ago; their wait must stay BEHIND the weight requests above,
    // or it is a wait for everything in flight (the convolution's masking of the loaded words was moved up otherwise)
    __builtin_amdgcn_sched_barrier(0);
    a_store(lds + (p ^ 1) * (TBM * T_SLOT));       // k-step kt+1; that buffer was last read in step kt-1
    a_fetch(kt + 2);
    __syncthreads();
    __builtin_amdgcn_sched_barrier(0);
  };
  int kt = 0;
#pragma unroll 1
  for (; kt + 2 <= KT; kt += 2) {
    step(kt, 0);
    step(kt + 1, 1);
  }
  if (kt < KT) step(kt, 0);                         // uniform over the grid

  // ---- epilogue -----------------------------------------------------------------------------------------
  if constexpr (GM != GM_PC) {
#pragma unroll
    for (int b = 0; b < TNB; ++b) fin[b] = s_cur[b] * INV_CM;
  } else if constexpr (!FIN_EARLY) {
    load_fin();
  }
  // every wave is past its last operand read (the loop ends with a barrier): the staging buffer is free
  int32_t* row_tab = reinterpret_cast<int32_t*>(lds);
  float* sx_tab = reinterpret_cast<float*>(lds + TBM * 4);
  if (tid < TBM) {
    row_tab[tid] = my_drow;
    if constexpr (A8) sx_tab[tid] = my_sx;
  }
  __syncthreads();
#pragma unroll
  for (int mb = 0; mb < TMB; ++mb) {
    const i32x4 drow4 = *reinterpret_cast<const i32x4*>(row_tab + wm * 64 + mb * 16 + lq * 4);
    f32x4 sx4 = {0.f, 0.f, 0.f, 0.f};
    if constexpr (A8) sx4 = *reinterpret_cast<const f32x4*>(sx_tab + wm * 64 + mb * 16 + lq * 4);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      if (drow4[r] >= 0) {
        float val[TNB];
#pragma unroll
        for (int b = 0; b < TNB; ++b) {
          if constexpr (A8) {
            val[b] = float(__float_as_int(tot[mb][b][r])) * sx4[r] * fin[b];
          } else if constexpr (GM == GM_PC) {
            val[b] = (fin[b] * INV_CM) * (tot[mb][b][r] - off_sym * xs_tot[mb][r]);
          } else {
            val[b] = tot[mb][b][r] * fin[b];
          }
        }
        const size_t drow = size_t(drow4[r]);
        if constexpr (GATEUP) {
          uint16_t* h = static_cast<uint16_t*>(ga.y) + drow * size_t(ga.n);
          if (nok[0]) h[ncol[0]] = float_to_bf16_rne(silu_mul(val[0], val[2]));
          if (nok[1]) h[ncol[1]] = float_to_bf16_rne(silu_mul(val[1], val[3]));
        } else if (ga.y_bf16) {
          uint16_t* y = static_cast<uint16_t*>(ga.y) + drow * size_t(ga.n);
#pragma unroll
          for (int b = 0; b < TNB; ++b)
            if (nok[b]) y[ncol[b]] = float_to_bf16_rne(val[b]);
        } else {
          float* y = static_cast<float*>(ga.y) + drow * size_t(ga.n);
#pragma unroll
          for (int b = 0; b < TNB; ++b)
            if (nok[b]) y[ncol[b]] = val[b];
        }
      }
    }
  }
}

// A launch with fewer than 8 weight tiles makes the patch narrower (2^patch_n_log2 weight tiles), so no
// work-group is launched for weight tiles that do not exist, and consecutive groups of PATCH_M row
// tiles still go round the XCDs.  Row tiles are enumerated expert by expert in the order of
// `TileGeom::order` (formats with the most arithmetic per tile first: what runs last, when the chip
// drains, are the cheap tiles).
constexpr int PATCH_M = 8;

template <bool GATEUP, bool CONV>
__global__ __launch_bounds__(TWAVES * 64, 2) void k_qgemm_tile(const GemmArgs ga, const TileGeom tg) {
  extern __shared__ __align__(16) uint8_t lds[];
  const int n_tiles = GATEUP ? (ga.n + TBN / 2 - 1) / (TBN / 2) : (ga.n + TBN - 1) / TBN;
  const int pn_log2 = tg.patch_n_log2, patch_wgs = PATCH_M << pn_log2;
  const int patches_n = (n_tiles + (1 << pn_log2) - 1) >> pn_log2;
  const int id = blockIdx.x, xcd = id & 7, j = id >> 3;
  const int patch = (j / patch_wgs) * 8 + xcd, q = j % patch_wgs;
  const int ntile = ((patch % patches_n) << pn_log2) + q / PATCH_M;
  if (ntile >= n_tiles) return;               // uniform over the work-group
  // Which expert and which row tile of its bucket: `slot` counts row tiles over all experts in the launch's
  // order.  Lane i takes the expert at position i: one load of the offsets, a prefix sum over 16 lanes.
  const int slot = (patch / patches_n) * PATCH_M + q % PATCH_M;
  const int lane = threadIdx.x & 63;
  const int mine = int((tg.order_bits >> (4 * (lane & 15))) & 15u);
  int o0 = 0, o1 = 0;
  if (lane < ga.n_experts) { o0 = ga.offsets[mine]; o1 = ga.offsets[mine + 1]; }
  int rows = (o1 - o0) * ga.T;
  if (rows < ga.min_rows || rows > ga.max_rows) rows = 0;         // that bucket belongs to the streaming kernel's launch
  const int tiles = (rows + TBM - 1) / TBM;
  int incl = tiles;
#pragma unroll
  for (int d = 1; d < MOQE_MAX_EXPERTS; d <<= 1) {
    const int v = __shfl_up(incl, d);
    if (lane >= d) incl += v;
  }
  const unsigned long long hit = __ballot(lane < ga.n_experts && slot >= incl - tiles && slot < incl);
  if (hit == 0ull) return;                    // uniform: a surplus work-group
  const int src = __ffsll(hit) - 1;
  const int e = __builtin_amdgcn_readfirstlane(__shfl(mine, src));
  const int off_e = __builtin_amdgcn_readfirstlane(__shfl(o0, src));
  const int M_e = __builtin_amdgcn_readfirstlane(__shfl((o1 - o0) * ga.T, src));
  const int m0 = __builtin_amdgcn_readfirstlane(__shfl((slot - (incl - tiles)) * TBM, src));
  const ExpertDev& ex = ga.ex[e];
  switch (ex.fmt * 4 + ex.gm) {
    case FMT_I8 * 4 + GM_PC:     tile_task<FMT_I8, GM_PC, GATEUP, CONV>(ga, tg, ex, off_e, M_e, m0, ntile, lds); break;
    case FMT_I8A8 * 4 + GM_PC:   tile_task<FMT_I8A8, GM_PC, GATEUP, CONV>(ga, tg, ex, off_e, M_e, m0, ntile, lds); break;
    case FMT_N6 * 4 + GM_PC:     tile_task<FMT_N6, GM_PC, GATEUP, CONV>(ga, tg, ex, off_e, M_e, m0, ntile, lds); break;
    case FMT_N4 * 4 + GM_PC:     tile_task<FMT_N4, GM_PC, GATEUP, CONV>(ga, tg, ex, off_e, M_e, m0, ntile, lds); break;
    case FMT_N4 * 4 + GM_G128:   tile_task<FMT_N4, GM_G128, GATEUP, CONV>(ga, tg, ex, off_e, M_e, m0, ntile, lds); break;
    case FMT_N4 * 4 + GM_G64:    tile_task<FMT_N4, GM_G64, GATEUP, CONV>(ga, tg, ex, off_e, M_e, m0, ntile, lds); break;
    case FMT_N3 * 4 + GM_G128:   tile_task<FMT_N3, GM_G128, GATEUP, CONV>(ga, tg, ex, off_e, M_e, m0, ntile, lds); break;
    case FMT_N3 * 4 + GM_G64:    tile_task<FMT_N3, GM_G64, GATEUP, CONV>(ga, tg, ex, off_e, M_e, m0, ntile, lds); break;
    default: break;
  }
}

// Relative arithmetic per tile of a format (measured on one launch per format): only the order matters.
static int tile_cost(const ExpertDev& ex) {
  const bool g64 = ex.gm == GM_G64, grp = ex.gm != GM_PC;
  switch (ex.fmt) {
    case FMT_I8A8: return 60;
    case FMT_I8:   return 119;
    case FMT_N6:   return 134;
    case FMT_N4:   return g64 ? 166 : (grp ? 125 : 108);
    default:       return g64 ? 172 : (grp ? 131 : 114);      // FMT_N3
  }
}

int32_t launch_qgemm_tile(const GemmArgs& ga, bool gateup, hipStream_t st) {
  const int M = ga.S * ga.T;
  const int row_tiles = (M + TBM - 1) / TBM + ga.n_experts;      // upper bound on sum_e ceil(M_e / TBM)
  const int n_tiles = gateup ? (ga.n + TBN / 2 - 1) / (TBN / 2) : (ga.n + TBN - 1) / TBN;
  TileGeom tg;
  memset(&tg, 0, sizeof(tg));
  while ((1 << tg.patch_n_log2) < n_tiles && tg.patch_n_log2 < 3) ++tg.patch_n_log2;
  const int pn = 1 << tg.patch_n_log2;
  const long patches = long((row_tiles + PATCH_M - 1) / PATCH_M) * ((n_tiles + pn - 1) / pn);
  const long grid = (patches + 7) / 8 * 8 * (PATCH_M * pn);
  if (grid > 0x7fffffffL) return set_error(MOQE_E_SHAPE, "grouped_qgemm: %d rows exceed the tile kernel's grid", M);
  static_assert(MOQE_MAX_EXPERTS <= 16, "the order is packed in 4-bit fields");
  int order[MOQE_MAX_EXPERTS];
  for (int e = 0; e < ga.n_experts; ++e) order[e] = e;
  std::stable_sort(order, order + ga.n_experts, [&](int a, int b) { return tile_cost(ga.ex[a]) > tile_cost(ga.ex[b]); });
  for (int e = 0; e < ga.n_experts; ++e) tg.order_bits |= uint64_t(order[e]) << (4 * e);
  const bool conv = ga.conv_c > 0;
  if (conv) {
    // column / conv_c by multiply-high is exact while column * conv_c < 2^32; columns stay below 10 * conv_c
    if (ga.conv_c > 16384) return set_error(MOQE_E_SHAPE, "grouped_qgemm: %d input channels exceed the convolution gather's 16384", ga.conv_c);
    tg.conv_c_magic = uint32_t(((1ull << 32) + uint32_t(ga.conv_c) - 1) / uint32_t(ga.conv_c));
  }
  const int ki = gateup ? 1 : (conv ? 2 : 0);
  const void* fns[3] = {reinterpret_cast<const void*>(&k_qgemm_tile<false, false>), reinterpret_cast<const void*>(&k_qgemm_tile<true, false>),
                        reinterpret_cast<const void*>(&k_qgemm_tile<false, true>)};
  int32_t rc = ensure_dynamic_lds(LDSK_TILE0 + ki, fns[ki], T_LDS_BYTES, "grouped_qgemm(tile)");
  if (rc) return rc;
  ProfileScope ps(gateup ? MOQE_PK_GEMM_GATEUP : MOQE_PK_GEMM_PLAIN, st, true);
  if (gateup) ps.launch(k_qgemm_tile<true, false>, dim3(unsigned(grid)), dim3(TWAVES * 64), T_LDS_BYTES, ga, tg);
  else if (conv) ps.launch(k_qgemm_tile<false, true>, dim3(unsigned(grid)), dim3(TWAVES * 64), T_LDS_BYTES, ga, tg);
  else ps.launch(k_qgemm_tile<false, false>, dim3(unsigned(grid)), dim3(TWAVES * 64), T_LDS_BYTES, ga, tg);
  return check_launch("grouped_qgemm(tile)");
}

}  // namespace moqe
