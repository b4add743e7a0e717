// Grouped dequantize-GEMM, tile kernel for large buckets (prefill, images).
//
// Each sample is processed by its selected expert only (MoQE Section 3.1); when an expert's bucket
// holds hundreds of rows the work is a dense contraction and belongs on the matrix cores with both
// operands staged through LDS.  A work-group of 8 waves owns a 128 x 128 output tile of one
// expert: 128 bucket rows (gathered through the permutation on load) times 128 weight rows (for
// the SiLU-gated pair: 64 gate rows and the 64 up rows of the same features, so the gate meets its
// up value in registers).  Per 128-column k-tile every wave fetches one packed 16-row weight tile
// with the same coalesced 16-byte-per-lane load as the streaming kernel, unpacks it to exact bf16
// operands (BASE + c/2) and stores them to LDS; the activation tile goes global -> registers ->
// LDS; the next k-tile's loads are in flight while the current one is multiplied.  Offsets and
// zero-points are removed with the activation row sums (an MFMA against ones) and the fp32 scale
// multiplies each group's fp32 partial sum, exactly as in the streaming kernel: no weight is
// rounded.
#include "qgemm_device.h"

namespace moqe {

constexpr int TBM = 128;                 // bucket rows per work-group tile
constexpr int TBN = 128;                 // weight rows per work-group tile
constexpr int TWAVES = 8;
constexpr int TMB = 2;                   // 16-row blocks per wave (rows)
constexpr int TNB = 4;                   // 16-row blocks per wave (weight rows)

template <bool A8> __host__ __device__ constexpr int tile_row_stride() { return 128 * (A8 ? 1 : 2) + 16; }

template <int FMT, int GM, bool GATEUP>
static __device__ __forceinline__ void tile_task(const GemmArgs& ga, const ExpertDev& ex, const int e, const int m0,
                                                 const int ntile, uint8_t* lds) {
  constexpr bool A8 = (FMT == FMT_I8A8);
  constexpr int NR = Raw<FMT>::N;
  constexpr int GPT = GM == GM_PC ? 0 : (GM == GM_G128 ? 1 : 2);
  constexpr int EB = A8 ? 1 : 2;
  constexpr int RS = tile_row_stride<A8>();
  constexpr int A_CHUNKS = 128 * EB / 16;            // 16-byte chunks per activation row and k-tile
  constexpr int A_ROWS_PER_IT = TWAVES * 64 / A_CHUNKS;
  constexpr int A_ITERS = TBM / A_ROWS_PER_IT;
  constexpr float BASE = CodeMap<FMT>::BASE, CM = CodeMap<FMT>::CM, INV_CM = 1.f / CodeMap<FMT>::CM;

  uint8_t* const lds_a = lds;
  uint8_t* const lds_b = lds + TBM * RS;
  float* const lds_sc = reinterpret_cast<float*>(lds + (TBM + TBN) * RS);        // [TBN][2]
  float* const lds_o = lds_sc + TBN * 2;                                            // [TBN][2]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 15, lq = lane >> 4;
  const int wm = wave >> 1, wn = wave & 1;
  const int KT = ga.k >> 7, NT = ga.n >> 4;
  const int T = ga.T;
  const int off_e = ga.offsets[e];
  const int M_e = (ga.offsets[e + 1] - off_e) * T;
  const float off_sym = BASE + CM * float(ex.zc);

  // ---- the packed weight tile this wave fetches per k-tile, and where its rows go in LDS -------
  int nt16;                                   // 16-row tile index inside the matrix
  const uint8_t* blob;
  if constexpr (GATEUP) {
    nt16 = ntile * 4 + (wave & 3);            // waves 0-3: gate rows, waves 4-7: up rows of the same features
    blob = ex.w[wave >> 2];
  } else {
    nt16 = ntile * 8 + wave;
    blob = ex.w[0];
  }
  const bool nt_ok = nt16 < NT;
  const int nt_ld = nt_ok ? nt16 : 0;         // clamped: rows outside the matrix are computed on garbage, never stored
  // ---- the weight-row blocks this wave multiplies (LDS rows) -------------------------------------
  int nb_row[TNB];
#pragma unroll
  for (int b = 0; b < TNB; ++b)
    nb_row[b] = GATEUP ? ((b >> 1) * 64 + wn * 32 + (b & 1) * 16) : (wn * 64 + b * 16);

  // ---- activation rows this thread copies per k-tile ----------------------------------------------
  const uint8_t* abase = reinterpret_cast<const uint8_t*>(A8 ? static_cast<const void*>(ga.a_q) : ga.a);
  uint32_t a_off[A_ITERS];
  const int a_chunk = tid % A_CHUNKS, a_row0 = tid / A_CHUNKS;
#pragma unroll
  for (int i = 0; i < A_ITERS; ++i) {
    const int m = min(m0 + a_row0 + i * A_ROWS_PER_IT, M_e - 1);      // rows past the bucket repeat its last row
    size_t src;
    if constexpr (A8) src = size_t(off_e) * T + m;
    else if (ga.a_perm) src = size_t(ga.a_perm[off_e + m / T]) * T + (m % T);
    else src = size_t(off_e) * T + m;
    a_off[i] = uint32_t(src * size_t(ga.k) * EB + a_chunk * 16);
  }

  u32x4 a_reg[A_ITERS];
  uint32_t raw[NR];
  float sc_reg[GPT ? GPT : 1];
  uint32_t zp_reg = 0;
  auto prefetch = [&](int kt) {
#pragma unroll
    for (int i = 0; i < A_ITERS; ++i)
      a_reg[i] = *reinterpret_cast<const u32x4*>(abase + size_t(a_off[i]) + size_t(kt) * 128 * EB);
    const size_t t = size_t(nt_ld) * KT + kt;
    load_raw<FMT>(raw, blob + t * ex.tile_bytes, lane);
    if constexpr (GPT > 0) {
      const float* sp = reinterpret_cast<const float*>(blob + ex.scale_off) + (t * 16 + lr) * GPT;
      const uint8_t* zq = blob + ex.zero_off + (t * 16 + lr) * GPT;
      if constexpr (GPT == 1) {
        sc_reg[0] = sp[0];
        zp_reg = uint32_t(zq[0]);
      } else {
        const float2 v = *reinterpret_cast<const float2*>(sp);
        sc_reg[0] = v.x; sc_reg[1] = v.y;
        zp_reg = uint32_t(*reinterpret_cast<const uint16_t*>(zq));
      }
    }
  };
  auto stage = [&]() {                        // registers -> LDS (weights are unpacked on the way)
#pragma unroll
    for (int i = 0; i < A_ITERS; ++i)
      *reinterpret_cast<u32x4*>(lds_a + (a_row0 + i * A_ROWS_PER_IT) * RS + a_chunk * 16) = a_reg[i];
    uint8_t* brow = lds_b + (wave * 16 + lr) * RS;
    if constexpr (A8) {
      *reinterpret_cast<u32x4*>(brow + lq * 16) = u32x4{raw[0], raw[1], raw[2], raw[3]};
      *reinterpret_cast<u32x4*>(brow + 64 + lq * 16) = u32x4{raw[4], raw[5], raw[6], raw[7]};
    } else {
      *reinterpret_cast<bf16x8*>(brow + (0 * 32 + lq * 8) * 2) = frag<FMT, 0>(raw);
      *reinterpret_cast<bf16x8*>(brow + (1 * 32 + lq * 8) * 2) = frag<FMT, 1>(raw);
      *reinterpret_cast<bf16x8*>(brow + (2 * 32 + lq * 8) * 2) = frag<FMT, 2>(raw);
      *reinterpret_cast<bf16x8*>(brow + (3 * 32 + lq * 8) * 2) = frag<FMT, 3>(raw);
      if constexpr (GPT > 0) {
        if (lq == 0) {
#pragma unroll
          for (int g = 0; g < GPT; ++g) {
            lds_sc[(wave * 16 + lr) * 2 + g] = sc_reg[g] * INV_CM;
            lds_o[(wave * 16 + lr) * 2 + g] = BASE + CM * float((zp_reg >> (8 * g)) & 0xffu);
          }
        }
      }
    }
  };

  f32x4 tot[TMB][TNB];        // bf16 path: fp32 results; int8 path: int32 bit patterns
  f32x4 xs_tot[TMB];
#pragma unroll
  for (int mb = 0; mb < TMB; ++mb) {
    xs_tot[mb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int b = 0; b < TNB; ++b) tot[mb][b] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  const u32x4 ones = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
  const bf16x8 ones_b = __builtin_bit_cast(bf16x8, ones);
  const uint8_t* a_rd = lds_a + (wm * 32 + lr) * RS;     // + mb*16*RS + column bytes
  const uint8_t* b_rd = lds_b + lr * RS;                 // + nb_row*RS + column bytes

  prefetch(0);
  for (int kt = 0; kt < KT; ++kt) {
    __syncthreads();                          // the previous k-tile is no longer read
    stage();
    __syncthreads();
    prefetch(min(kt + 1, KT - 1));            // unconditional (clamped): stays in flight during the multiply
    if constexpr (A8) {
#pragma unroll
      for (int js = 0; js < 2; ++js) {
        i32x4 a[TMB], b[TNB];
#pragma unroll
        for (int mb = 0; mb < TMB; ++mb) a[mb] = *reinterpret_cast<const i32x4*>(a_rd + mb * 16 * RS + js * 64 + lq * 16);
#pragma unroll
        for (int nb = 0; nb < TNB; ++nb) b[nb] = *reinterpret_cast<const i32x4*>(b_rd + nb_row[nb] * RS + js * 64 + lq * 16);
#pragma unroll
        for (int mb = 0; mb < TMB; ++mb)
#pragma unroll
          for (int nb = 0; nb < TNB; ++nb) {
            i32x4 acc = __builtin_bit_cast(i32x4, tot[mb][nb]);
            acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[mb], b[nb], acc, 0, 0, 0);
            tot[mb][nb] = __builtin_bit_cast(f32x4, acc);
          }
      }
    } else {
      constexpr int GSTEPS = GM == GM_G64 ? 2 : 4;      // MFMA steps per quantization group
      f32x4 v[TMB][TNB], xs[TMB];
      auto do_step = [&](auto jc) {
        constexpr int J = decltype(jc)::value;
        if constexpr (GM != GM_PC && J % GSTEPS == 0) {
#pragma unroll
          for (int mb = 0; mb < TMB; ++mb) {
            xs[mb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int nb = 0; nb < TNB; ++nb) v[mb][nb] = f32x4{0.f, 0.f, 0.f, 0.f};
          }
        }
        u32x4 a[TMB];
        bf16x8 b[TNB];
#pragma unroll
        for (int mb = 0; mb < TMB; ++mb) a[mb] = *reinterpret_cast<const u32x4*>(a_rd + mb * 16 * RS + (J * 32 + lq * 8) * 2);
#pragma unroll
        for (int nb = 0; nb < TNB; ++nb) b[nb] = *reinterpret_cast<const bf16x8*>(b_rd + nb_row[nb] * RS + (J * 32 + lq * 8) * 2);
#pragma unroll
        for (int mb = 0; mb < TMB; ++mb) {
          if constexpr (GM == GM_PC) xs_tot[mb] = mfma_bf16(a[mb], ones_b, xs_tot[mb]);
          else xs[mb] = mfma_bf16(a[mb], ones_b, xs[mb]);
#pragma unroll
          for (int nb = 0; nb < TNB; ++nb) {
            if constexpr (GM == GM_PC) tot[mb][nb] = mfma_bf16(a[mb], b[nb], tot[mb][nb]);
            else v[mb][nb] = mfma_bf16(a[mb], b[nb], v[mb][nb]);
          }
        }
        if constexpr (GM != GM_PC && (J + 1) % GSTEPS == 0) {
          constexpr int G = J / GSTEPS;
#pragma unroll
          for (int nb = 0; nb < TNB; ++nb) {
            const float scv = lds_sc[(nb_row[nb] + lr) * 2 + G];
            const float o = lds_o[(nb_row[nb] + lr) * 2 + G];
#pragma unroll
            for (int mb = 0; mb < TMB; ++mb)
#pragma unroll
              for (int r = 0; r < 4; ++r) tot[mb][nb][r] += scv * (v[mb][nb][r] - o * xs[mb][r]);
          }
        }
      };
      do_step(std::integral_constant<int, 0>{});
      do_step(std::integral_constant<int, 1>{});
      do_step(std::integral_constant<int, 2>{});
      do_step(std::integral_constant<int, 3>{});
    }
  }

  // ---- epilogue ---------------------------------------------------------------------------------------
  // global weight row of block nb, column lr
  int ncol[TNB];
  bool nok[TNB];
  float pcs[TNB];
#pragma unroll
  for (int nb = 0; nb < TNB; ++nb) {
    if constexpr (GATEUP) ncol[nb] = ntile * 64 + wn * 32 + (nb & 1) * 16 + lr;       // feature index (gate and up)
    else ncol[nb] = ntile * 128 + wn * 64 + nb * 16 + lr;
    nok[nb] = ncol[nb] < ga.n;
    pcs[nb] = 1.f;
    if constexpr (GM == GM_PC) {
      const uint8_t* bl = GATEUP ? ex.w[nb >> 1] : ex.w[0];
      if (nok[nb]) pcs[nb] = reinterpret_cast<const float*>(bl + ex.scale_off)[ncol[nb]];
    }
  }
#pragma unroll
  for (int mb = 0; mb < TMB; ++mb) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int m = m0 + wm * 32 + mb * 16 + lq * 4 + r;
      if (m < M_e) {
        float val[TNB];
#pragma unroll
        for (int nb = 0; nb < TNB; ++nb) {
          if constexpr (A8) {
            const float sx = ga.a_scale[size_t(off_e) * T + m];
            val[nb] = float(__float_as_int(tot[mb][nb][r])) * sx * pcs[nb];
          } else if constexpr (GM == GM_PC) {
            val[nb] = (pcs[nb] * INV_CM) * (tot[mb][nb][r] - off_sym * xs_tot[mb][r]);
          } else {
            val[nb] = tot[mb][nb][r];
          }
        }
        const size_t brow = size_t(off_e) * T + m;
        if constexpr (GATEUP) {
          uint16_t* h = static_cast<uint16_t*>(ga.y) + brow * size_t(ga.n);
          if (nok[0]) h[ncol[0]] = float_to_bf16_rne(silu_mul(val[0], val[2]));
          if (nok[1]) h[ncol[1]] = float_to_bf16_rne(silu_mul(val[1], val[3]));
        } else {
          size_t drow = brow;
          if (ga.y_perm) drow = size_t(ga.y_perm[off_e + m / T]) * T + (m % T);
          float* y = static_cast<float*>(ga.y) + drow * size_t(ga.n);
#pragma unroll
          for (int nb = 0; nb < TNB; ++nb)
            if (nok[nb]) y[ncol[nb]] = val[nb];
        }
      }
    }
  }
}

template <bool GATEUP>
__global__ __launch_bounds__(TWAVES * 64) void k_qgemm_tile(const GemmArgs ga) {
  extern __shared__ __align__(16) uint8_t lds[];
  // which expert and which 128-row tile of its bucket: blockIdx.y counts row tiles over all experts
  int slot = blockIdx.y, e = -1, m0 = 0;
  for (int i = 0; i < ga.n_experts; ++i) {
    const int rows = (ga.offsets[i + 1] - ga.offsets[i]) * ga.T;
    const int tiles = (rows + TBM - 1) / TBM;
    if (slot < tiles) { e = i; m0 = slot * TBM; break; }
    slot -= tiles;
  }
  if (e < 0) return;                          // uniform over the work-group
  const ExpertDev& ex = ga.ex[e];
  const int ntile = blockIdx.x;
  switch (ex.fmt * 4 + ex.gm) {
    case FMT_I8 * 4 + GM_PC:     tile_task<FMT_I8, GM_PC, GATEUP>(ga, ex, e, m0, ntile, lds); break;
    case FMT_I8A8 * 4 + GM_PC:   tile_task<FMT_I8A8, GM_PC, GATEUP>(ga, ex, e, m0, ntile, lds); break;
    case FMT_N6 * 4 + GM_PC:     tile_task<FMT_N6, GM_PC, GATEUP>(ga, ex, e, m0, ntile, lds); break;
    case FMT_N4 * 4 + GM_PC:     tile_task<FMT_N4, GM_PC, GATEUP>(ga, ex, e, m0, ntile, lds); break;
    case FMT_N4 * 4 + GM_G128:   tile_task<FMT_N4, GM_G128, GATEUP>(ga, ex, e, m0, ntile, lds); break;
    case FMT_N4 * 4 + GM_G64:    tile_task<FMT_N4, GM_G64, GATEUP>(ga, ex, e, m0, ntile, lds); break;
    case FMT_N3 * 4 + GM_G128:   tile_task<FMT_N3, GM_G128, GATEUP>(ga, ex, e, m0, ntile, lds); break;
    case FMT_N3 * 4 + GM_G64:    tile_task<FMT_N3, GM_G64, GATEUP>(ga, ex, e, m0, ntile, lds); break;
    default: break;
  }
}

int32_t launch_qgemm_tile(const GemmArgs& ga, bool gateup, hipStream_t st) {
  const int M = ga.S * ga.T;
  const int row_tiles = (M + TBM - 1) / TBM + ga.n_experts;      // upper bound on sum_e ceil(M_e / 128)
  const int n_tiles = gateup ? (ga.n + 63) / 64 : (ga.n + TBN - 1) / TBN;
  if (row_tiles > 65535) return set_error(MOQE_E_SHAPE, "grouped_qgemm: %d rows exceed the tile kernel's grid", M);
  const int lds_bytes = (TBM + TBN) * tile_row_stride<false>() + TBN * 2 * 4 * 2;
  static bool lds_ok[2] = {false, false};
  const void* fn = gateup ? reinterpret_cast<const void*>(&k_qgemm_tile<true>) : reinterpret_cast<const void*>(&k_qgemm_tile<false>);
  if (!lds_ok[gateup ? 1 : 0]) {
    hipError_t err = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (err != hipSuccess) return set_error(MOQE_E_HIP, "grouped_qgemm: cannot reserve LDS: %s", hipGetErrorString(err));
    lds_ok[gateup ? 1 : 0] = true;
  }
  ProfileScope ps(gateup ? MOQE_PK_GEMM_GATEUP : MOQE_PK_GEMM_PLAIN, st);
  if (gateup) hipLaunchKernelGGL(k_qgemm_tile<true>, dim3(n_tiles, row_tiles), dim3(TWAVES * 64), lds_bytes, st, ga);
  else hipLaunchKernelGGL(k_qgemm_tile<false>, dim3(n_tiles, row_tiles), dim3(TWAVES * 64), lds_bytes, st, ga);
  return check_launch("grouped_qgemm(tile)");
}

}  // namespace moqe
