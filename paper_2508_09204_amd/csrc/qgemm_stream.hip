// Grouped dequantize-GEMM, weight-streaming kernel for buckets of a few rows (decode).
//
// Each sample is processed by its selected expert only (MoQE Section 3.1), so for expert e the
// few rows of its bucket meet the whole weight matrix of that expert: the work is bound by
// reading the packed weights once, and everything else is arranged so that nothing but weights
// moves in the inner loop.
//
//  * One work-group (8 waves) per compute unit, resident for the whole launch.  The work-groups
//    are dealt to the experts in proportion to the bytes each expert has to stream (its tile size
//    times the passes its bucket needs), and an expert's 16-row weight tiles are split evenly among
//    its work-groups; every work-group computes this deal itself from the bucket offsets.
//  * The activations stay in REGISTERS: the k range (at most 32 k-tiles of 128 columns; longer rows
//    take the other streaming kernel) is cut across the 8 waves, 4 k-tiles per wave, and a wave loads
//    its slice of the bucket's rows once, already shaped as matrix-core operands.  It then streams
//    the matching 4-tile piece of every weight tile row of the work-group (4 KiB contiguous for
//    4-bit codes), a piece or two ahead, through 16-byte load -> a few bit operations -> bf16 MFMA.
//    No LDS traffic and no barrier sits between a weight load and its MFMA.
//  * Integer codes enter the matrix cores exactly as the bf16 value BASE + c/2 (or c for 8-bit
//    codes).  The offset and the zero-point are removed exactly: for group formats by ONE fp32
//    matrix-core operation per weight tile row, row sums of the activations (kept as its A operand,
//    one register) times -scale*(BASE + z/2) (its B operand); for per-channel formats by the wave's
//    row sum once per tile row.  The fp32 scale multiplies the fp32 partial sum of each group, so no
//    weight is ever rounded.
//  * The 8 partial sums of a tile row (one per k slice) are added in wave order through LDS, a
//    batch of tile rows per barrier, every wave adding its share.  Then the epilogue: fp32 rows scattered through the permutation, or
//    bf16(silu(gate) * up).  Every sum has a fixed order: results do not depend on scheduling.
#include "qgemm_device.h"

#include <mutex>

namespace moqe {

constexpr int SW = 8;                      // waves per work-group
constexpr int KPW = 4;                     // k-tiles (128 columns) a wave keeps as register operands
constexpr int MAX_KT = SW * KPW;           // k-tiles a work-group covers: longer rows go to the other streaming kernel
static_assert(MAX_KT == STREAM_REG_MAX_KT, "the launcher's limit is what the waves' register operands cover");
constexpr int STREAM_ROWS = 32;            // bucket rows per pass (two 16-row blocks)
constexpr int BMT = 4;                     // (tile rows per batch) x (16-row blocks): results exchanged per barrier
constexpr int PART_BYTES = 2 * BMT * SW * 64 * 16;     // two buffers of per-wave partial sums
constexpr int PERM_LDS_BYTES = SW * 64 * 4;           // a private copy of the permutation per wave (launches that bucket themselves)
constexpr int ROWTAB_BYTES = STREAM_ROWS * 8;          // per row of the pass: where its result goes, its activation scale
constexpr int STREAM_LDS_BYTES = PART_BYTES + PERM_LDS_BYTES + ROWTAB_BYTES;

// ---- which expert and which of its weight tiles a work-group streams ---------------------------------
struct StreamSeg {
  int e, u0, u1;          // expert and its weight tiles [u0, u1) for this work-group
  int off_e, rows_e;      // first sample of the expert's bucket, rows in it
  ExpertDev ex;           // the expert's descriptor, uniform over the work-group
};

// Units are 16-row weight tiles (gate/up: the gate tile and the up tile of the same 16 features).  The cost of
// an expert's unit is its tile bytes times the passes over its bucket; work-groups are dealt in proportion:
// the floor of each expert's share, then the work-groups left over one at a time to the expert whose
// work-groups carry the most.  Lane e of every 16-lane row holds expert e and the sums are cross-lane
// reductions, so the deal costs a few dozen instructions; every work-group runs the same arithmetic on the
// same inputs and gets the same deal.
// Reductions over a row of 16 lanes with data-parallel-primitive moves (vector instructions of a few cycles; a
// shuffle through the LDS crossbar costs a hundred and these chains are serial): partner lane^1 and lane^2 inside a
// quad, then the mirrored half row and the mirrored row, which pair lanes that already agree within their quad
// and half row.  Every lane ends with the reduction of its row.
template <int CTRL> static __device__ __forceinline__ int dpp_move(int v) {
  return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xf, 0xf, false);
}
constexpr int DPP_QUAD_XOR1 = 0xB1, DPP_QUAD_XOR2 = 0x4E, DPP_ROW_HALF_MIRROR = 0x141, DPP_ROW_MIRROR = 0x140;
static __device__ __forceinline__ int row16_sum(int v) {
  v += dpp_move<DPP_QUAD_XOR1>(v);
  v += dpp_move<DPP_QUAD_XOR2>(v);
  v += dpp_move<DPP_ROW_HALF_MIRROR>(v);
  v += dpp_move<DPP_ROW_MIRROR>(v);
  return v;
}
static __device__ __forceinline__ int row16_max(int v) {
  v = max(v, dpp_move<DPP_QUAD_XOR1>(v));
  v = max(v, dpp_move<DPP_QUAD_XOR2>(v));
  v = max(v, dpp_move<DPP_ROW_HALF_MIRROR>(v));
  v = max(v, dpp_move<DPP_ROW_MIRROR>(v));
  return v;
}
// Inclusive prefix sum over the 16 lanes of a row: shifts by 1, 2, 4, 8 lanes to the right, zero shifted in.
template <int N> static __device__ __forceinline__ int row_shr_or_zero(int v) {
  return __builtin_amdgcn_update_dpp(0, v, 0x110 + N, 0xf, 0xf, true);
}
static __device__ __forceinline__ int row16_prefix_sum(int v) {
  v += row_shr_or_zero<1>(v);
  v += row_shr_or_zero<2>(v);
  v += row_shr_or_zero<4>(v);
  v += row_shr_or_zero<8>(v);
  return v;
}

// Lane e (of every 16-lane row) fetches bucket e's bounds and expert e's descriptor, all in one round trip:
// the kernel arguments live in memory that is slow to touch for the first time, and a chain of dependent
// reads there would cost microseconds before the first weight is requested.
static __device__ __forceinline__ StreamSeg stream_schedule(const GemmArgs& ga, const int wg, const int G, int32_t* perm_l) {
  const int K = ga.n_experts, NU = ga.n >> 4;
  const int e = threadIdx.x & 15;
  const int el_safe = e < K ? e : 0;
  int o0, o1;
  if (ga.expert_idx) {
    // Stable counting sort of at most 64 samples, a sample per lane: the count of expert k is the population of the ballot
    // "my sample goes to k", a sample's place in its bucket the population below its lane (the bucket kernel's arithmetic).
    const int L = threadIdx.x & 63;
    int es = L < ga.S ? ga.expert_idx[L] : -1;
    if (es >= K) es = -1;
    const unsigned long long below = L == 0 ? 0ull : (~0ull >> (64 - L));
    int base = 0, my_pos = 0;
    o0 = 0; o1 = 0;
    for (int k = 0; k < K; ++k) {
      const unsigned long long b = __ballot(es == k);
      const int c = __popcll(b);
      if (es == k) my_pos = base + __popcll(b & below);
      if (e == k) { o0 = base; o1 = base + c; }
      base += c;
    }
    if (es >= 0) perm_l[my_pos] = L;                    // this wave's own copy: read back by the same wave only
    __builtin_amdgcn_wave_barrier();
    if (wg == 0 && threadIdx.x < 64) {                  // first wave of the first work-group publishes the result
      if (L < K) {
        if (ga.out_counts) ga.out_counts[L] = o1 - o0;
        if (ga.out_offsets) ga.out_offsets[L] = o0;
      }
      if (L == 0 && ga.out_offsets) ga.out_offsets[K] = base;
      if (es >= 0) {
        if (ga.out_perm) ga.out_perm[my_pos] = L;
        if (ga.out_inv_perm) ga.out_inv_perm[L] = my_pos;
      }
    }
  } else {
    o0 = ga.offsets[el_safe];
    o1 = ga.offsets[el_safe + 1];
  }
  const ExpertDev mine_ex = ga.ex[el_safe];                        // per-lane copy (vector loads from the argument block)
  const int rows = e < K ? (o1 - o0) * ga.T : 0;
  const bool mine = rows >= ga.min_rows && rows <= ga.max_rows && rows > 0;
  // Relative time of one weight tile row: mostly its bytes, plus what unpacking costs (measured per format on
  // MI355X), a little more when the bucket needs both 16-row blocks; times the passes over the bucket.
  const int f = mine_ex.fmt;
  const int per_tile = f == FMT_I8 ? 31 : (f == FMT_I8A8 ? 24 : (f == FMT_N6 ? 25 : (f == FMT_N4 ? 20 : 25)));
  const int passes = (rows + STREAM_ROWS - 1) / STREAM_ROWS;
  const int last = rows - (passes - 1) * STREAM_ROWS;              // rows of the last pass
  const int parts = (passes - 1) * 21 + (last > 16 ? 21 : 16);     // a pass with two blocks counts 21/16
  const int cost = mine ? per_tile * parts : 0;                    // small integers
  const int total = row16_sum(cost);
  StreamSeg sg;
  sg.e = -1; sg.u0 = 0; sg.u1 = 0; sg.off_e = 0; sg.rows_e = 0;
  if (total <= 0) return sg;
  // cost is at most a few hundred (price x passes) and G the number of compute units: the product fits 32 bits
  int g = cost > 0 ? max(1, min(NU, int(unsigned(cost) * unsigned(G) / unsigned(total)))) : 0;
  int sum = row16_sum(g);
  // more than G (tiny shares rounded up to one): take from the largest
  for (int it = 0; it < MOQE_MAX_EXPERTS && sum > G; ++it) {
    const int top = row16_max((g << 4) | (15 - e));                // ties: the lowest expert index
    const int cut = min(sum - G, (top >> 4) - 1);
    if (cut <= 0) break;
    if ((15 - (top & 15)) == e) g -= cut;
    sum -= cut;
  }
  // work-groups left over go, one at a time, to the expert whose work-groups carry the most
  for (int it = 0; it < MOQE_MAX_EXPERTS && sum < G; ++it) {
    const float load = (g > 0 && g < NU) ? float(cost) / float(g) : 0.f;
    const int key = (__float_as_int(load) & ~15) | (15 - e);       // positive floats order like their bit patterns
    const int top = row16_max(key);
    if ((top & ~15) == 0) break;                                   // nobody can take more
    if ((15 - (top & 15)) == e) g += 1;
    sum += 1;
  }
  // first work-group of each expert: exclusive prefix sum over the lanes of the row
  const int first = row16_prefix_sum(g) - g;
  const bool here = g > 0 && wg >= first && wg < first + g;
  const unsigned long long who = __ballot(here) & 0xffffull;       // row 0 of the wave; at most one lane
  if (who == 0ull) return sg;
  const int el = __ffsll(who) - 1;
  // everything of the chosen expert is read from its lane into scalar registers (el is uniform)
  auto from_lane = [&](int v) { return __builtin_amdgcn_readlane(v, el); };
  const int ge = from_lane(g), fe = from_lane(first);
  const unsigned i = unsigned(wg - fe);
  sg.e = el;
  // NU = q ge + r units over ge work-groups: the first r take q + 1 (one division instead of two)
  const unsigned q = unsigned(NU) / unsigned(ge), r = unsigned(NU) - q * unsigned(ge);
  sg.u0 = int(i * q + min(i, r));
  sg.u1 = sg.u0 + int(q) + (i < r ? 1 : 0);
  sg.off_e = from_lane(o0);
  sg.rows_e = from_lane(rows);
  const uint64_t w0 = reinterpret_cast<uint64_t>(mine_ex.w[0]), w1 = reinterpret_cast<uint64_t>(mine_ex.w[1]);
  const uint64_t w0u = (uint64_t(uint32_t(from_lane(int(w0 >> 32)))) << 32) | uint32_t(from_lane(int(uint32_t(w0))));
  const uint64_t w1u = (uint64_t(uint32_t(from_lane(int(w1 >> 32)))) << 32) | uint32_t(from_lane(int(uint32_t(w1))));
  sg.ex.w[0] = reinterpret_cast<const uint8_t*>(w0u);
  sg.ex.w[1] = reinterpret_cast<const uint8_t*>(w1u);
  sg.ex.fmt = from_lane(mine_ex.fmt);
  sg.ex.gm = from_lane(mine_ex.gm);
  sg.ex.zc = from_lane(mine_ex.zc);
  sg.ex.asym = from_lane(mine_ex.asym);
  sg.ex.tile_bytes = uint32_t(from_lane(int(mine_ex.tile_bytes)));
  sg.ex.scale_off = uint32_t(from_lane(int(mine_ex.scale_off)));
  sg.ex.zero_off = uint32_t(from_lane(int(mine_ex.zero_off)));
  return sg;
}

template <typename V> static __device__ __forceinline__ V pick4(int q, V a, V b, V c, V d) {
  return q == 0 ? a : (q == 1 ? b : (q == 2 ? c : d));
}

// One pass (at most 32 bucket rows, MT blocks of 16) of one expert's weight tiles [u0, u1).
template <int FMT, int GM, bool GATEUP, int MT>
static __device__ __forceinline__ void stream_pass(const GemmArgs& ga, const ExpertDev& ex, const int off_e, const int u0,
                                                   const int u1, const int pass0, const int rows_here, uint8_t* lds,
                                                   const int32_t* perm_l) {
  constexpr bool A8 = (FMT == FMT_I8A8);
  constexpr int NR = Raw<FMT>::N;
  constexpr int GPT = GM == GM_PC ? 0 : (GM == GM_G128 ? 1 : 2);
  constexpr int GP1 = GPT ? GPT : 1;
  constexpr int B = BMT / MT;                          // tile rows per batch
  // Tile rows in flight (the one being multiplied and those behind it): as many as the registers allow, a
  // budget of 24 registers of codes and group parameters per k-tile for one 16-row block, 12 for two.
  constexpr int RING_REGS = NR + (GM == GM_PC ? 0 : (GM == GM_G128 ? 2 : 3));
  constexpr int D_FIT = (MT == 1 ? 24 : 12) / RING_REGS;
  constexpr int D = D_FIT >= 4 && B % 4 == 0 ? 4 : ((D_FIT >= 2 && !(MT == 2 && GM == GM_G64)) ? 2 : 1);      // two blocks and two groups per k-tile: no room
  constexpr int AJ = A8 ? 2 : 4;                        // matrix-core steps per k-tile
  constexpr float BASE = CodeMap<FMT>::BASE, CM = CodeMap<FMT>::CM, INV_CM = 1.f / CodeMap<FMT>::CM;
  static_assert(B % D == 0 && (!GATEUP || B % 2 == 0), "ring slot and gate/up pairing are static inside a batch");
  static_assert(KPW == 4, "a wave's k-tiles map onto the four k positions of the fp32 matrix-core operation");

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lr = lane & 15, lq = lane >> 4;
  const int KT = ga.k >> 7, T = ga.T;
  const int ntr = (u1 - u0) * (GATEUP ? 2 : 1);         // weight tile rows of this work-group
  const int ktw0 = wave * KPW;                          // first k-tile of this wave
  const int nkt = max(0, min(KPW, KT - ktw0));          // its k-tiles (0 .. KPW)
  const float off_sym = BASE + CM * float(ex.zc);
  const FragK<FMT> fk = frag_constants<FMT>();
  const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};

  const uint32_t zp_shift = 8u * uint32_t((lr * GPT) & 3);      // position of the lane's zero-point(s) in their dword

  uint8_t* part = lds;                                  // [2][B][SW][MT][64] x 16 bytes

  // ---- rows of this pass ---------------------------------------------------------------------------------
  // operand rows: lane (lr, lq) feeds row mt*16 + lr of the pass; result rows: register r of lane (lr, lq) is
  // row mt*16 + 4 lq + r.  Rows past the end repeat the last one and are never stored.
  // The rows' gather / scatter indices and activation scales.  (An integer division by a run-time number is some
  // forty instructions, and there are twenty of them here: one row per sample, the decode case, skips them.)
  const bool one_row = T == 1;                          // uniform
  auto div_t = [&](int m) { return one_row ? m : m / T; };
  auto mod_t = [&](int m) { return one_row ? 0 : m % T; };
  const uint8_t* abase = reinterpret_cast<const uint8_t*>(A8 ? static_cast<const void*>(ga.a_q) : ga.a);
  int a_src[MT];                // sample of operand row mt*16 + lr (its gather index), before the row offset inside the sample
  int a_m[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    a_m[mt] = pass0 + min(mt * 16 + lr, rows_here - 1);
    a_src[mt] = off_e + div_t(a_m[mt]);
    if (!A8 && ga.a_perm) a_src[mt] = perm_l ? perm_l[a_src[mt]] : ga.a_perm[a_src[mt]];
  }
  int out_row[MT][4];           // destination row of each result register
  float sx[MT][4];              // W8A8: activation scale of each result row
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int m = pass0 + min(mt * 16 + lq * 4 + r, rows_here - 1);
      const int brow = off_e * T + m;
      int dsmp = off_e + div_t(m);
      if (!GATEUP && ga.y_perm) dsmp = perm_l ? perm_l[dsmp] : ga.y_perm[dsmp];
      out_row[mt][r] = dsmp;                                       // turned into a row index after the ring's first row
      sx[mt][r] = 1.f;
      if constexpr (A8) sx[mt][r] = ga.a_scale[brow];
    }
  size_t a_row_off[MT];

  // ---- weight ring -----------------------------------------------------------------------------------------
  // The work-group walks its tile rows in order, whole batches first, the rows left over last (requests past
  // the last row repeat it and are never used).  The ring holds D consecutive rows, KPW tiles each; tile (row, t) is requested
  // again, for the row D places further on, right after its matrix-core operations, so KPW * D - 1 tiles are in
  // flight behind the one being multiplied, across batch boundaries alike.  `cur_i` is the next row to request.
  uint32_t raw[D][KPW][NR];
  float sc[D][KPW][GP1];                                // group scales; per-channel formats: [0] of tile 0 is the row's scale
  uint32_t zp[D][KPW];
  const uint32_t tile_bytes = ex.tile_bytes, scale_off = ex.scale_off, zero_off = ex.zero_off;
  // weights are read through buffer descriptors: scalar tile offset + lane offset, no vector address arithmetic
  const buf_rsrc blob0 = blob_rsrc(ex.w[0]);
  const buf_rsrc blob1 = blob_rsrc(ex.w[GATEUP ? 1 : 0]);
  int cur_i = 0;
  // derived from the position: which blob, first tile index of the row's KPW tiles, tile row
  buf_rsrc cur_blob = blob0;
  uint32_t cur_t0 = 0u;
  int cur_nt = u0;
  const int cur_tmax = max(nkt - 1, 0);                  // tiles the wave does not have repeat its last one (or the row's last)
  auto cur_derive = [&]() {
    const int i = min(cur_i, ntr - 1);                   // rows past the end: the last row again
    cur_nt = GATEUP ? u0 + (i >> 1) : u0 + i;
    cur_blob = (GATEUP && (i & 1)) ? blob1 : blob0;
    cur_t0 = uint32_t(cur_nt) * uint32_t(KT) + uint32_t(min(ktw0, KT - 1));
  };
  auto cur_advance = [&]() {
    cur_i += 1;
    cur_derive();
  };
  auto issue_tile = [&](int d, int t) {                  // d, t are compile-time constants at every call
    const uint32_t tl = cur_t0 + uint32_t(min(t, cur_tmax));                      // uniform; byte offsets below fit 32 bits
    load_raw<FMT>(raw[d][t], cur_blob, tl * tile_bytes, lane);
    if constexpr (GPT > 0) {
      // zero-points: the aligned dword that holds the lane's byte(s); shifted down where it is used (a
      // narrower load would get its zero-extension placed right behind the load, which waits for the ring)
      zp[d][t] = buf_load32(cur_blob, (lr * GPT) & ~3, zero_off + tl * uint32_t(16 * GPT));
      if constexpr (GPT == 1) {
        sc[d][t][0] = __uint_as_float(buf_load32(cur_blob, lr * 4, scale_off + tl * 64u));
      } else {
        const u32x2 v = buf_load64(cur_blob, lr * 8, scale_off + tl * 128u);
        sc[d][t][0] = __uint_as_float(v.x); sc[d][t][GP1 - 1] = __uint_as_float(v.y);
      }
    } else {
      zp[d][t] = 0u;
      sc[d][t][0] = 1.f;
      if (t == 0) sc[d][t][0] = __uint_as_float(buf_load32(cur_blob, lr * 4, scale_off + uint32_t(cur_nt) * 64u));
    }
  };
  // ---- this wave's slice of the activations, as matrix-core operands ---------------------------------------------
  u32x4 areg[KPW][AJ][MT];
  auto load_a = [&]() {
#pragma unroll
    for (int t = 0; t < KPW; ++t)
#pragma unroll
      for (int j = 0; j < AJ; ++j)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          areg[t][j][mt] = u32x4{0u, 0u, 0u, 0u};
          if (t < nkt) {                                         // uniform over the wave
            const size_t col = A8 ? size_t(ktw0 + t) * 128 + j * 64 + lq * 16 : (size_t(ktw0 + t) * 128 + j * 32 + lq * 8) * 2;
            areg[t][j][mt] = *reinterpret_cast<const u32x4*>(abase + a_row_off[mt] + col);
          }
        }
  };

  // The activations are requested before any weight: a compute unit serves its requests
  // in order, and once the 8 waves have filled its queues with ring loads (misses to HBM), a load that hits
  // in L2 issued behind them would still wait for them all.
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    a_row_off[mt] = (size_t(a_src[mt]) * T + size_t(mod_t(a_m[mt]))) * size_t(ga.k) * (A8 ? 1 : 2);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int m = pass0 + min(mt * 16 + lq * 4 + r, rows_here - 1);
      out_row[mt][r] = out_row[mt][r] * T + mod_t(m);
    }
  }
  // The epilogue picks a row's destination by a run-time register number.  Held in registers, the eight values
  // end up as an indexed array in scratch memory, and the one scratch load per batch makes the epilogue wait for
  // every load in flight (loads return in order), i.e. for the whole weight ring.  They go through LDS instead.
  int2* const row_tab = reinterpret_cast<int2*>(lds + PART_BYTES + PERM_LDS_BYTES);
  if (wave == 0 && lr == 0) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 4; ++r) row_tab[mt * 16 + lq * 4 + r] = make_int2(out_row[mt][r], __float_as_int(sx[mt][r]));
  }
  load_a();
  cur_derive();
  // the ring's first row right behind the activations; the rows after it once the activations have been
  // used (below): a wave that requested its whole ring first would sit behind the other waves' rings too
  // (scheduling barriers: the first fill must request the tiles in the loop's order, see the loop's head)
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int t = 0; t < KPW; ++t) {
    issue_tile(0, t);
    __builtin_amdgcn_sched_barrier(0);
  }
  cur_advance();

  {
    {
      // ---- row sums of this wave's slice of the activations ------------------------------------------------
      // group formats: xs_op[mt][g], lane (lr, lq) = sum of row lr over group g of k-tile lq: the A operand of
      //   the fp32 matrix-core operation that removes offset and zero-point;
      // per-channel formats: xs_c[mt], register r of lane (lr, lq) = sum of row 4 lq + r over the wave's k-tiles.
      float xs_op[MT][GP1];
      f32x4 xs_c[MT];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        xs_c[mt] = zero4;
#pragma unroll
        for (int g = 0; g < GP1; ++g) xs_op[mt][g] = 0.f;
      }
      const u32x4 ones_u = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
      if constexpr (!A8 && GPT > 0) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int g = 0; g < GPT; ++g) {
            // all-ones first operand, the activations as second: every result register of lane (lr, .) is the sum
            // of row lr over the columns multiplied (fp32 accumulation inside the matrix core)
            float pt[KPW];
#pragma unroll
            for (int t = 0; t < KPW; ++t) {
              f32x4 v = zero4;
#pragma unroll
              for (int j = (GPT == 1 ? 0 : 2 * g); j < (GPT == 1 ? 4 : 2 * g + 2); ++j)
                v = mfma_bf16(ones_u, __builtin_bit_cast(bf16x8, areg[t][j][mt]), v);
              pt[t] = v[0];                                        // zero for k-tiles the wave does not have
            }
            xs_op[mt][g] = pick4(lq, pt[0], pt[1], pt[2], pt[3]);
          }
      }
      if constexpr (!A8 && GPT == 0) {
        const bf16x8 ones_b = __builtin_bit_cast(bf16x8, ones_u);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          f32x4 v = zero4;
#pragma unroll
          for (int t = 0; t < KPW; ++t)
#pragma unroll
            for (int j = 0; j < 4; ++j) v = mfma_bf16(areg[t][j][mt], ones_b, v);
          xs_c[mt] = v;
        }
      }

      // the rest of the ring, in the order the loop below requests it again
#pragma unroll
      for (int d = 1; d < D; ++d) {
#pragma unroll
        for (int t = 0; t < KPW; ++t) {
          __builtin_amdgcn_sched_barrier(0);
          issue_tile(d, t);
        }
        cur_advance();
      }
      __builtin_amdgcn_sched_barrier(0);

      // The ring values arrive through the loop's back edge.  Pinning a tile's registers where the tile is
      // used keeps the optimizer from moving arithmetic on them (a mask, a conversion) up to the end of the
      // previous iteration, right behind their loads, where it would wait for the whole ring.
      auto pin_tile = [&](int d, int t) {
#pragma unroll
        for (int i = 0; i < NR; ++i) asm volatile("" : "+v"(raw[d][t][i]));
        asm volatile("" : "+v"(zp[d][t]));
#pragma unroll
        for (int g = 0; g < GP1; ++g) asm volatile("" : "+v"(sc[d][t][g]));
      };
      // ---- one tile row from ring slot d: the wave's partial result, ready to be added across waves.  Straight-
      // line code: a k-tile the wave does not have is multiplied by all-zero activation operands.  With no branch
      // around a load the waits can be exact, and the compiler may overlap one tile's unpacking with the
      // matrix-core operations of another. -------
      auto multiply = [&](int d, f32x4 (&res)[MT], float& row_scale) {
        pin_tile(d, 0);
        row_scale = sc[d][0][0];                                   // per-channel formats: kept for the epilogue
        if constexpr (A8) {
          i32x4 acc[MT];
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) acc[mt] = i32x4{0, 0, 0, 0};
#pragma unroll
          for (int t = 0; t < KPW; ++t) {
            if (t > 0) pin_tile(d, t);
            {
              const i32x4 b0 = {int(raw[d][t][0]), int(raw[d][t][1]), int(raw[d][t][2]), int(raw[d][t][3])};
              const i32x4 b1 = {int(raw[d][t][4]), int(raw[d][t][5]), int(raw[d][t][6]), int(raw[d][t][7])};
#pragma unroll
              for (int mt = 0; mt < MT; ++mt) {
                acc[mt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(i32x4, areg[t][0][mt]), b0, acc[mt], 0, 0, 0);
                acc[mt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(i32x4, areg[t][1][mt]), b1, acc[mt], 0, 0, 0);
              }
            }
            issue_tile(d, t);
          }
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) res[mt] = __builtin_bit_cast(f32x4, acc[mt]);
        } else if constexpr (GPT == 0) {
          f32x4 acc[MT];
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) acc[mt] = zero4;
#pragma unroll
          for (int t = 0; t < KPW; ++t) {
            if (t > 0) pin_tile(d, t);
            {
              const bf16x8 b0 = frag<FMT, 0>(raw[d][t], fk), b1 = frag<FMT, 1>(raw[d][t], fk);
              const bf16x8 b2 = frag<FMT, 2>(raw[d][t], fk), b3 = frag<FMT, 3>(raw[d][t], fk);
#pragma unroll
              for (int mt = 0; mt < MT; ++mt) {
                f32x4 v = acc[mt];
                v = mfma_bf16(areg[t][0][mt], b0, v);
                v = mfma_bf16(areg[t][1][mt], b1, v);
                v = mfma_bf16(areg[t][2][mt], b2, v);
                v = mfma_bf16(areg[t][3][mt], b3, v);
                acc[mt] = v;
              }
            }
            issue_tile(d, t);
          }
          const float s = row_scale * INV_CM;
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 4; ++r) res[mt][r] = s * (acc[mt][r] - off_sym * xs_c[mt][r]);
        } else {
          f32x4 acc[MT];
          float so[GP1];                                           // lane (n = lr, g = lq): -scale * (BASE + CM z) / CM of k-tile lq
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) acc[mt] = zero4;
#pragma unroll
          for (int g = 0; g < GP1; ++g) so[g] = 0.f;
#pragma unroll
          for (int t = 0; t < KPW; ++t) {
            if (t > 0) pin_tile(d, t);
            const float s0 = sc[d][t][0] * INV_CM, s1 = sc[d][t][GP1 - 1] * INV_CM;
#pragma unroll
            for (int g = 0; g < GPT; ++g) {
              const float z = float((zp[d][t] >> (zp_shift + 8 * g)) & 0xffu);
              const float v = -(g == 0 ? s0 : s1) * (BASE + CM * z);
              so[g] = lq == t ? v : so[g];
            }
            {
              const bf16x8 b0 = frag<FMT, 0>(raw[d][t], fk), b1 = frag<FMT, 1>(raw[d][t], fk);
              const bf16x8 b2 = frag<FMT, 2>(raw[d][t], fk), b3 = frag<FMT, 3>(raw[d][t], fk);
#pragma unroll
              for (int mt = 0; mt < MT; ++mt) {
                if constexpr (GPT == 1) {
                  f32x4 v = mfma_bf16(areg[t][0][mt], b0, zero4);
                  v = mfma_bf16(areg[t][1][mt], b1, v);
                  v = mfma_bf16(areg[t][2][mt], b2, v);
                  v = mfma_bf16(areg[t][3][mt], b3, v);
#pragma unroll
                  for (int r = 0; r < 4; ++r) acc[mt][r] += s0 * v[r];
                } else {
                  const f32x4 v0 = mfma_bf16(areg[t][1][mt], b1, mfma_bf16(areg[t][0][mt], b0, zero4));
                  const f32x4 v1 = mfma_bf16(areg[t][3][mt], b3, mfma_bf16(areg[t][2][mt], b2, zero4));
#pragma unroll
                  for (int r = 0; r < 4; ++r) acc[mt][r] += s0 * v0[r] + s1 * v1[r];
                }
              }
            }
            issue_tile(d, t);
          }
          // offset and zero-point of all the wave's groups in one fp32 matrix-core operation per 4 groups:
          //   acc[m][n] += sum_g xs[m][g] * so[g][n]
#pragma unroll
          for (int g = 0; g < GPT; ++g)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
              acc[mt] = __builtin_amdgcn_mfma_f32_16x16x4f32(xs_op[mt][g], so[g], acc[mt], 0, 0, 0);
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) res[mt] = acc[mt];
        }
        cur_advance();
      };

      // ---- the tile rows, a batch per barrier ---------------------------------------------------------------
      // Wait counts are static: at the loop's head the compiler takes, per register, the stricter of the count
      // the loop's back edge needs and the count the code before the loop needs.  The first fill above requests
      // the ring in the loop's own order, so both agree and a tile waits for its own load only.
      // A batch of B tile rows starting at row i0.  Full batches run in the loop below, whose code has no branch
      // around a row.  The rows left over (fewer than B) run once through a second copy of the same code that
      // skips the absent rows: its wait counts are the cautious ones of branching code, which costs nothing
      // when no further row is on its way, and a work-group with 22 rows pays for 22, not for 24.
      auto batch = [&](auto tail_tag, const int i0, const int bi) {
        constexpr bool TAIL = decltype(tail_tag)::value;
        uint8_t* pbuf = part + (bi & 1) * (PART_BYTES / 2);
        float pcs_b[B];                                            // the per-channel scales of this batch's tile rows
#pragma unroll
        for (int b = 0; b < B; ++b) {
          const bool row_live = !TAIL || i0 + b < ntr;             // uniform over the work-group
          f32x4 res[MT];
          pcs_b[b] = 0.f;
          if (row_live) multiply(b % D, res, pcs_b[b]);
          if (row_live) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
              *reinterpret_cast<f32x4*>(pbuf + (((b * SW + wave) * MT + mt) * 64 + lane) * 16) = res[mt];
          }
        }
        __syncthreads();

        // All waves share the additions evenly: a result (64 lanes x 4 registers of one tile row and 16-row block;
        // gate/up: of the gate row and of the up row) belongs to SW / ITEMS waves, RPW registers each.  A thread adds
        // the 8 partial sums of its registers in wave order and stores them.
        constexpr int NV = GATEUP ? 2 : 1;                         // gate and up results meet in one thread
        constexpr int ITEMS = B * MT / NV;                         // results per batch
        constexpr int WPI = SW / ITEMS;                            // waves per result
        constexpr int RPW = 4 / WPI;                               // registers per wave
        static_assert(ITEMS * WPI == SW && RPW * WPI == 4, "the results of a batch divide evenly among the waves");
        {
          const int item = wave / WPI, r0 = (wave % WPI) * RPW;    // uniform over the wave
          const int ib = item / MT, mt_dyn = item % MT;            // tile row (or pair) inside the batch, 16-row block
          const int i_first = i0 + ib * NV;                        // tile row index
          if (i_first < ntr) {
            float v[NV][RPW];
#pragma unroll
            for (int s = 0; s < NV; ++s) {
              const uint8_t* src = pbuf + (((ib * NV + s) * SW * MT + mt_dyn) * 64 + lane) * 16 + r0 * 4;
#pragma unroll
              for (int rr = 0; rr < RPW; ++rr) v[s][rr] = reinterpret_cast<const float*>(src)[rr];
#pragma unroll
              for (int w = 1; w < SW; ++w) {
#pragma unroll
                for (int rr = 0; rr < RPW; ++rr) {
                  const float o = reinterpret_cast<const float*>(src + w * (MT * 64 * 16))[rr];
                  if constexpr (A8) v[s][rr] = __int_as_float(__float_as_int(v[s][rr]) + __float_as_int(o));
                  else v[s][rr] += o;
                }
              }
            }
            {
              const int i_glob = i_first;
              const int nt = GATEUP ? u0 + (i_glob >> 1) : u0 + i_glob;
              const int ncol = nt * 16 + lr;
#pragma unroll
              for (int rr = 0; rr < RPW; ++rr) {
                const int r = r0 + rr;
                // this register's result row (written before the batch's barrier, by the first wave)
                const int2 rt = row_tab[mt_dyn * 16 + lq * 4 + r];
                const int orow = rt.x;
                const float osx = __int_as_float(rt.y);
                float val[NV];
#pragma unroll
                for (int s = 0; s < NV; ++s) {
                  val[s] = v[s][rr];
                  if constexpr (A8) {
                    float ps = pcs_b[0];
#pragma unroll
                    for (int b = 1; b < B; ++b) if (ib * NV + s == b) ps = pcs_b[b];
                    val[s] = float(__float_as_int(val[s])) * osx * ps;
                  }
                }
                if (mt_dyn * 16 + lq * 4 + r < rows_here) {
                  const size_t o = size_t(orow) * size_t(ga.n) + ncol;
                  if constexpr (GATEUP) static_cast<uint16_t*>(ga.y)[o] = float_to_bf16_rne(silu_mul(val[0], val[NV - 1]));
                  else if (ga.y_bf16) static_cast<uint16_t*>(ga.y)[o] = float_to_bf16_rne(val[0]);
                  else static_cast<float*>(ga.y)[o] = val[0];
                }
              }
            }
          }
        }
      };
      int bi = 0, i0 = 0;
#pragma unroll 1
      for (; i0 + B <= ntr; i0 += B, ++bi) batch(std::false_type{}, i0, bi);
      if (i0 < ntr) batch(std::true_type{}, i0, bi);
      __syncthreads();          // the partial-sum buffers are free again before the next pass writes them
    }
  }
}

template <int FMT, int GM, bool GATEUP>
static __device__ __forceinline__ void stream_expert(const GemmArgs& ga, const StreamSeg& sg, uint8_t* lds, const int32_t* perm_l) {
  for (int pass0 = 0; pass0 < sg.rows_e; pass0 += STREAM_ROWS) {
    const int rows_here = min(STREAM_ROWS, sg.rows_e - pass0);
    if (rows_here <= 16) stream_pass<FMT, GM, GATEUP, 1>(ga, sg.ex, sg.off_e, sg.u0, sg.u1, pass0, rows_here, lds, perm_l);
    else stream_pass<FMT, GM, GATEUP, 2>(ga, sg.ex, sg.off_e, sg.u0, sg.u1, pass0, rows_here, lds, perm_l);
  }
}

template <bool GATEUP>
__global__ __launch_bounds__(SW * 64, 2) void k_qgemm_stream(const GemmArgs ga) {
  extern __shared__ __align__(16) uint8_t lds[];
  // the permutation of a launch that buckets itself: one copy per wave behind the partial-sum buffers
  int32_t* perm_l = ga.expert_idx ? reinterpret_cast<int32_t*>(lds + PART_BYTES) + (threadIdx.x >> 6) * 64 : nullptr;
  StreamSeg sg = stream_schedule(ga, int(blockIdx.x), int(gridDim.x), perm_l);
  if (sg.e < 0 || sg.u1 <= sg.u0) return;             // uniform over the work-group
  sg.u0 = __builtin_amdgcn_readfirstlane(sg.u0); sg.u1 = __builtin_amdgcn_readfirstlane(sg.u1);
  sg.off_e = __builtin_amdgcn_readfirstlane(sg.off_e); sg.rows_e = __builtin_amdgcn_readfirstlane(sg.rows_e);
  switch (sg.ex.fmt * 4 + sg.ex.gm) {
    case FMT_I8 * 4 + GM_PC:     stream_expert<FMT_I8, GM_PC, GATEUP>(ga, sg, lds, perm_l); break;
    case FMT_I8A8 * 4 + GM_PC:   stream_expert<FMT_I8A8, GM_PC, GATEUP>(ga, sg, lds, perm_l); break;
    case FMT_N6 * 4 + GM_PC:     stream_expert<FMT_N6, GM_PC, GATEUP>(ga, sg, lds, perm_l); break;
    case FMT_N4 * 4 + GM_PC:     stream_expert<FMT_N4, GM_PC, GATEUP>(ga, sg, lds, perm_l); break;
    case FMT_N4 * 4 + GM_G128:   stream_expert<FMT_N4, GM_G128, GATEUP>(ga, sg, lds, perm_l); break;
    case FMT_N4 * 4 + GM_G64:    stream_expert<FMT_N4, GM_G64, GATEUP>(ga, sg, lds, perm_l); break;
    case FMT_N3 * 4 + GM_G128:   stream_expert<FMT_N3, GM_G128, GATEUP>(ga, sg, lds, perm_l); break;
    case FMT_N3 * 4 + GM_G64:    stream_expert<FMT_N3, GM_G64, GATEUP>(ga, sg, lds, perm_l); break;
    default: break;
  }
}

// One work-group per compute unit of the current device.
static int32_t stream_grid(int* out) {
  static std::mutex mu;
  static int cus[64] = {};
  int dev = 0;
  hipError_t err = hipGetDevice(&dev);
  if (err != hipSuccess) return set_error(MOQE_E_HIP, "grouped_qgemm: hipGetDevice: %s", hipGetErrorString(err));
  if (dev < 0 || dev >= 64) return set_error(MOQE_E_HIP, "grouped_qgemm: device %d", dev);
  std::lock_guard<std::mutex> lk(mu);
  if (cus[dev] == 0) {
    int n = 0;
    err = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
    if (err != hipSuccess || n <= 0) return set_error(MOQE_E_HIP, "grouped_qgemm: compute unit count: %s", hipGetErrorString(err));
    cus[dev] = n;
  }
  *out = cus[dev];
  return MOQE_OK;
}

int32_t launch_qgemm_stream(const GemmArgs& ga, bool gateup, hipStream_t st) {
  // this kernel reads `a` as a plain [rows, k] matrix; an image that still needs its 3x3 gather must not get here
  if (ga.conv_c != 0) return set_error(MOQE_E_SHAPE, "grouped_qgemm: the streaming kernel cannot gather a convolution's rows");
  int grid = 0;
  int32_t rc = stream_grid(&grid);
  if (rc) return rc;
  const void* fn = gateup ? reinterpret_cast<const void*>(&k_qgemm_stream<true>) : reinterpret_cast<const void*>(&k_qgemm_stream<false>);
  rc = ensure_dynamic_lds(LDSK_STREAM0 + (gateup ? 1 : 0), fn, STREAM_LDS_BYTES, "grouped_qgemm");
  if (rc) return rc;
  ProfileScope ps(gateup ? MOQE_PK_GEMM_GATEUP : MOQE_PK_GEMM_PLAIN, st, true);
  if (gateup) ps.launch(k_qgemm_stream<true>, dim3(grid), dim3(SW * 64), STREAM_LDS_BYTES, ga);
  else ps.launch(k_qgemm_stream<false>, dim3(grid), dim3(SW * 64), STREAM_LDS_BYTES, ga);
  return check_launch("grouped_qgemm");
}

}  // namespace moqe
