// C-ABI entry points: argument validation on the host, workspace carving, kernel sequencing.
// Nothing here allocates device memory or synchronises the host (moqe_profile_read aside).
#include "moqe_internal.h"

#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <mutex>
#include <vector>

namespace moqe {

static thread_local char g_err[512] = "";
static std::atomic<int> g_dry{0};

int32_t set_error(int32_t code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

bool dry_run() { return g_dry.load() != 0; }

int32_t check_launch(const char* what) {
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return set_error(MOQE_E_HIP, "%s: launch failed: %s", what, hipGetErrorString(err));
  return MOQE_OK;
}

int32_t ensure_dynamic_lds(int slot, const void* kernel, int bytes, const char* what) {
  static std::mutex mu;
  static int state[LDSK_COUNT] = {};        // 0: not asked yet, 1: granted
  std::lock_guard<std::mutex> lk(mu);
  if (slot < 0 || slot >= LDSK_COUNT) return set_error(MOQE_E_SHAPE, "%s: bad kernel slot %d", what, slot);
  if (state[slot] == 1) return MOQE_OK;
  hipError_t err = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (err != hipSuccess) return set_error(MOQE_E_HIP, "%s: cannot reserve %d bytes of LDS: %s", what, bytes, hipGetErrorString(err));
  state[slot] = 1;
  return MOQE_OK;
}

// ---- profiling ---------------------------------------------------------------------------
// Event pairs come from a pool that only grows, so that recording inside a timed region costs two
// hipEventRecord calls per launch and no event creation once the pool is warm.
struct ProfRec { int ev; int kind; };
static std::mutex g_prof_mu;
static uint32_t g_prof_mask = 0;
static std::vector<ProfRec> g_prof;
static std::vector<hipEvent_t> g_pool;     // events 2i, 2i+1 form pair i

ProfileScope::ProfileScope(int kind, hipStream_t s, bool exact_) : slot(-1), stream(s), exact(exact_), ev_begin(nullptr), ev_end(nullptr) {
  if (!((g_prof_mask >> kind) & 1u)) return;
  std::lock_guard<std::mutex> lk(g_prof_mu);
  if (!((g_prof_mask >> kind) & 1u) || g_prof.size() >= MOQE_PROFILE_MAX_LAUNCHES) return;
  const size_t pair = g_prof.size();
  while (g_pool.size() < 2 * (pair + 1)) {
    hipEvent_t e;
    if (hipEventCreate(&e) != hipSuccess) return;
    g_pool.push_back(e);
  }
  ev_begin = g_pool[2 * pair];
  ev_end = g_pool[2 * pair + 1];
  if (!exact) (void)hipEventRecord(ev_begin, s);
  g_prof.push_back(ProfRec{int(pair), kind});
  slot = int(pair);
}

ProfileScope::~ProfileScope() {
  if (slot < 0 || exact) return;
  (void)hipEventRecord(ev_end, stream);
}

// ---- validation helpers --------------------------------------------------------------------
static bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

static int32_t check_qmat_format(const moqe_qmat& m, PackedInfo* pi, const char* who) {
  if (!packed_info(m.n, m.k, m.bits, m.group, m.symmetric, m.act_mode, pi)) {
    if (m.n <= 0 || m.k <= 0 || m.n % 16 || m.k % 128)
      return set_error(MOQE_E_SHAPE, "%s: matrix %d x %d needs n %% 16 == 0 and k %% 128 == 0", who, m.n, m.k);
    return set_error(MOQE_E_FORMAT, "%s: unsupported format bits=%d group=%d symmetric=%d act_mode=%d", who, m.bits,
                     m.group, m.symmetric, m.act_mode);
  }
  // the kernels address a packed matrix with 32-bit byte offsets from its start
  if (pi->total >= (size_t(1) << 32))
    return set_error(MOQE_E_SHAPE, "%s: packed matrix %d x %d takes %zu bytes, the limit is 4 GiB", who, m.n, m.k, pi->total);
  return MOQE_OK;
}

static int32_t check_packed(const moqe_qmat& m, PackedInfo* pi, const char* who) {
  int32_t rc = check_qmat_format(m, pi, who);
  if (rc) return rc;
  if (m.layout != MOQE_LAYOUT_PACKED) return set_error(MOQE_E_FORMAT, "%s: matrix must be in the packed layout", who);
  if (!m.qdata) return set_error(MOQE_E_NULL, "%s: qdata is NULL", who);
  if (!aligned(m.qdata, 256)) return set_error(MOQE_E_SHAPE, "%s: packed blob must be 256-byte aligned", who);
  return MOQE_OK;
}

static int32_t check_router(const moqe_router* r, const char* who) {
  if (!r) return set_error(MOQE_E_NULL, "%s: router is NULL", who);
  if (r->n_experts < 1 || r->n_experts > MOQE_MAX_EXPERTS)
    return set_error(MOQE_E_SHAPE, "%s: n_experts %d outside [1, %d]", who, r->n_experts, MOQE_MAX_EXPERTS);
  if (r->d <= 0 || r->d % 8) return set_error(MOQE_E_SHAPE, "%s: router input dim %d must be a positive multiple of 8", who, r->d);
  if (r->h < 0 || r->h % 4) return set_error(MOQE_E_SHAPE, "%s: router hidden dim %d must be a multiple of 4", who, r->h);
  if (!r->w2) return set_error(MOQE_E_NULL, "%s: router w2 is NULL", who);
  if (r->h > 0 && !r->w1) return set_error(MOQE_E_NULL, "%s: router w1 is NULL", who);
  if (!aligned(r->w2, 16) || (r->w1 && !aligned(r->w1, 16)) || (r->b1 && !aligned(r->b1, 16)))
    return set_error(MOQE_E_SHAPE, "%s: router weights must be 16-byte aligned", who);
  return MOQE_OK;
}

static void fill_expert(const moqe_qmat& m0, const moqe_qmat* m1, const PackedInfo& pi, ExpertDev* ex) {
  ex->w[0] = static_cast<const uint8_t*>(m0.qdata);
  ex->w[1] = m1 ? static_cast<const uint8_t*>(m1->qdata) : nullptr;
  ex->fmt = pi.fmt; ex->gm = pi.gm; ex->zc = pi.zc; ex->asym = pi.asym;
  ex->tile_bytes = pi.tile_bytes;
  ex->scale_off = uint32_t(pi.scale_off);
  ex->zero_off = uint32_t(pi.zero_off);
}

// Byte offsets into an activation matrix are 32-bit inside the kernels.
static int32_t check_activation_bytes(long long M, int k, const char* who) {
  if (size_t(M) * size_t(k) * 2 >= (size_t(1) << 32))
    return set_error(MOQE_E_SHAPE, "%s: activation matrix of %lld x %d exceeds 4 GiB", who, M, k);
  return MOQE_OK;
}

// Workspace for the int8 copies of activation rows needed by act_mode-1 experts.
static size_t a8_bytes(bool any_a8, int M, int kmax) {
  if (!any_a8) return 0;
  return align256(size_t(M) * kmax) + align256(size_t(M) * 4);
}

struct GroupedPlan {
  PackedInfo pi[MOQE_MAX_EXPERTS];
  bool any_a8;
};

static int32_t plan_experts(const moqe_qmat* experts, int K, const moqe_qmat* second, GroupedPlan* gp, const char* who) {
  gp->any_a8 = false;
  for (int e = 0; e < K; ++e) {
    int32_t rc = check_packed(experts[e], &gp->pi[e], who);
    if (rc) return rc;
    if (experts[e].n != experts[0].n || experts[e].k != experts[0].k)
      return set_error(MOQE_E_SHAPE, "%s: expert %d is %d x %d, expert 0 is %d x %d", who, e, experts[e].n, experts[e].k,
                       experts[0].n, experts[0].k);
    if (second) {
      PackedInfo p2;
      rc = check_packed(second[e], &p2, who);
      if (rc) return rc;
      if (second[e].n != experts[e].n || second[e].k != experts[e].k || p2.fmt != gp->pi[e].fmt || p2.gm != gp->pi[e].gm)
        return set_error(MOQE_E_FORMAT, "%s: gate and up of expert %d must share shape and format", who, e);
    }
    if (gp->pi[e].fmt == FMT_I8A8) gp->any_a8 = true;
  }
  return MOQE_OK;
}

// Which kernel an expert's bucket takes.  Buckets of a few rows stream the weights once (bound by HBM);
// buckets of many rows are a dense contraction and take the LDS-tiled kernel (bound by the matrix cores).
// The host does not know the bucket sizes, only bounds: every non-empty bucket has a multiple of T rows
// and at most M.  Where that decides, one kernel is launched; otherwise both are, and each takes, on the
// device, the experts whose bucket is on its side of STREAM_MAX_ROWS.
constexpr int STREAM_MAX_ROWS = 32;        // one pass of the streaming kernel
constexpr int STREAM_ONLY_ROWS = 128;      // up to here even one bucket holding every row streams (4 passes at most)
enum GemmPath { PATH_STREAM, PATH_TILE, PATH_BOTH };
static GemmPath choose_path(long long M, int T) {
  if (T > STREAM_MAX_ROWS) return PATH_TILE;
  if (M <= STREAM_ONLY_ROWS) return PATH_STREAM;
  return PATH_BOTH;
}

// Enqueues one grouped GEMM (plus the int8 row quantization its act_mode-1 experts need).
// A launch of at most 64 samples that can bucket them itself (see GemmArgs::expert_idx).
struct SelfBucket {
  const int32_t* expert_idx;
  int32_t *counts, *offsets, *perm, *inv_perm;
};

// True when run_grouped(..., &SelfBucket) is possible for this launch: the register-resident streaming kernel alone
// takes it, and no expert needs its rows quantized (that step reads the bucket arrays before the launch).
static bool can_self_bucket(int S, int T, int k, const GroupedPlan& gp) {
  return S <= 64 && !gp.any_a8 && choose_path((long long)S * T, T) == PATH_STREAM && k / 128 <= STREAM_REG_MAX_KT;
}

static int32_t run_grouped(const void* a, const int32_t* offsets, const int32_t* a_perm, const int32_t* y_perm, int S, int T,
                           const moqe_qmat* experts, const moqe_qmat* second, int K, const GroupedPlan& gp, void* y,
                           uint8_t* a8_ws, hipStream_t st, int conv_h = 0, int conv_w = 0, int conv_c = 0, bool y_bf16 = false,
                           const SelfBucket* sb = nullptr) {
  // conv_c > 0: a is the NHWC image and the tiled kernel gathers the 3x3 neighbourhoods itself
  GemmArgs ga;
  memset(&ga, 0, sizeof(ga));
  ga.n_experts = K;
  ga.n = experts[0].n; ga.k = experts[0].k;
  ga.S = S; ga.T = T;
  ga.a = a; ga.offsets = offsets; ga.a_perm = a_perm; ga.y_perm = y_perm; ga.y = y;
  ga.conv_h = conv_h; ga.conv_w = conv_w; ga.conv_c = conv_c;
  ga.y_bf16 = (y_bf16 && !second) ? 1 : 0;
  if (sb) {
    ga.expert_idx = sb->expert_idx;
    ga.out_counts = sb->counts; ga.out_offsets = sb->offsets; ga.out_perm = sb->perm; ga.out_inv_perm = sb->inv_perm;
  }
  for (int e = 0; e < K; ++e) fill_expert(experts[e], second ? &second[e] : nullptr, gp.pi[e], &ga.ex[e]);
  const int M = S * T;
  if (gp.any_a8) {
    int8_t* aq = reinterpret_cast<int8_t*>(a8_ws);
    float* as = reinterpret_cast<float*>(a8_ws + align256(size_t(M) * ga.k));
    ga.a_q = aq; ga.a_scale = as;
    for (int e = 0; e < K; ++e) {
      if (gp.pi[e].fmt != FMT_I8A8) continue;
      int32_t rc = launch_act_quant(a, ga.k, T, offsets, a_perm, e, M, aq, as, st);
      if (rc) return rc;
    }
  }
  // The 3x3 gather exists in the tiled kernel only: a convolution always goes there.
  const GemmPath path = conv_c > 0 ? PATH_TILE : choose_path(M, T);
  const int32_t all_rows = 0x7fffffff;
  if (path != PATH_TILE) {
    ga.min_rows = 1;
    ga.max_rows = path == PATH_STREAM ? all_rows : STREAM_MAX_ROWS;
    int32_t rc = (ga.k / 128 <= STREAM_REG_MAX_KT) ? launch_qgemm_stream(ga, second != nullptr, st)
                                                    : launch_qgemm_stream_lds(ga, second != nullptr, st);
    if (rc) return rc;
  }
  if (path != PATH_STREAM) {
    ga.min_rows = path == PATH_TILE ? 1 : STREAM_MAX_ROWS + 1;
    ga.max_rows = all_rows;
    return launch_qgemm_tile(ga, second != nullptr, st);
  }
  return MOQE_OK;
}

}  // namespace moqe

using namespace moqe;

extern "C" {

const char* moqe_version(void) { return "moqe-gfx950 0.1"; }
const char* moqe_last_error_string(void) { return g_err; }
void moqe_set_dry_run(int32_t on) { g_dry.store(on ? 1 : 0); }

// ---- routing -------------------------------------------------------------------------------
size_t moqe_route_workspace_bytes(int32_t S, int32_t T, const moqe_router* r) {
  if (!r || S < 0 || T <= 0 || r->d <= 0) return 0;
  return route_ws_bytes(S, T, *r);
}

int32_t moqe_route(const void* x, int32_t S, int32_t T, const moqe_router* r, int32_t* expert_idx, float* logits,
                   void* workspace, size_t workspace_bytes, void* stream) {
  int32_t rc = check_router(r, "moqe_route");
  if (rc) return rc;
  if (S < 0 || T <= 0) return set_error(MOQE_E_SHAPE, "moqe_route: S=%d T=%d", S, T);
  if (S == 0) return MOQE_OK;
  if (!x || !expert_idx) return set_error(MOQE_E_NULL, "moqe_route: x or expert_idx is NULL");
  if (!aligned(x, 16)) return set_error(MOQE_E_SHAPE, "moqe_route: x must be 16-byte aligned");
  const size_t need = route_ws_bytes(S, T, *r);
  if (!workspace || !aligned(workspace, 256) || workspace_bytes < need)
    return set_error(MOQE_E_WORKSPACE, "moqe_route: workspace needs %zu bytes, 256-byte aligned", need);
  if (dry_run()) return MOQE_OK;
  return launch_route(x, S, T, *r, expert_idx, logits, workspace, static_cast<hipStream_t>(stream));
}

int32_t moqe_bucket(const int32_t* expert_idx, int32_t S, int32_t K, int32_t* counts, int32_t* offsets, int32_t* perm,
                    int32_t* inv_perm, void* stream) {
  if (K < 1 || K > MOQE_MAX_EXPERTS) return set_error(MOQE_E_SHAPE, "moqe_bucket: K=%d outside [1, %d]", K, MOQE_MAX_EXPERTS);
  if (S < 0) return set_error(MOQE_E_SHAPE, "moqe_bucket: S=%d", S);
  if (!offsets) return set_error(MOQE_E_NULL, "moqe_bucket: offsets is NULL");
  if (S > 0 && !expert_idx) return set_error(MOQE_E_NULL, "moqe_bucket: expert_idx is NULL");
  if (dry_run()) return MOQE_OK;
  return launch_bucket(expert_idx, S, K, counts, offsets, perm, inv_perm, static_cast<hipStream_t>(stream));
}

size_t moqe_route_nlp_workspace_bytes(int32_t S, int32_t T, const moqe_nlp_router* r) {
  if (S < 0 || T <= 0 || (long long)S * T > 0x7fffffffLL) return 0;
  if (check_nlp_router(r, "moqe_route_nlp_workspace_bytes") || check_router(&r->head, "moqe_route_nlp_workspace_bytes")) return 0;
  return route_nlp_ws_bytes(S, T, *r);
}

int32_t moqe_route_nlp(const void* x, int32_t S, int32_t T, const moqe_nlp_router* r, int32_t* expert_idx, float* logits,
                       void* workspace, size_t workspace_bytes, void* stream) {
  int32_t rc = check_nlp_router(r, "moqe_route_nlp");
  if (rc) return rc;
  rc = check_router(&r->head, "moqe_route_nlp");
  if (rc) return rc;
  if (S < 0 || T <= 0 || (long long)S * T > 0x7fffffffLL) return set_error(MOQE_E_SHAPE, "moqe_route_nlp: S=%d T=%d", S, T);
  if (S == 0) return MOQE_OK;
  if (!x || !expert_idx) return set_error(MOQE_E_NULL, "moqe_route_nlp: x or expert_idx is NULL");
  if (!aligned(x, 16)) return set_error(MOQE_E_SHAPE, "moqe_route_nlp: x must be 16-byte aligned");
  if (S > 65535 || (long long)S * T > 65535LL * 128)
    return set_error(MOQE_E_SHAPE, "moqe_route_nlp: at most 65535 samples and 8388480 token rows per call");
  const size_t need = route_nlp_ws_bytes(S, T, *r);
  if (!workspace || !aligned(workspace, 256) || workspace_bytes < need)
    return set_error(MOQE_E_WORKSPACE, "moqe_route_nlp: workspace needs %zu bytes, 256-byte aligned", need);
  if (dry_run()) return MOQE_OK;
  return launch_route_nlp(x, S, T, *r, expert_idx, logits, workspace, static_cast<hipStream_t>(stream));
}

size_t moqe_route_cv_workspace_bytes(int32_t S, int32_t h, int32_t w, const moqe_cv_router* r) {
  if (S < 0 || h <= 0 || w <= 0 || (long long)S * h * w > 0x7fffffffLL) return 0;
  if (check_cv_router(r, h, w, "moqe_route_cv_workspace_bytes")) return 0;
  return route_cv_ws_bytes(S, h, w, *r);
}

int32_t moqe_route_cv(const void* x, int32_t S, int32_t h, int32_t w, const moqe_cv_router* r, int32_t* expert_idx, float* logits,
                      void* workspace, size_t workspace_bytes, void* stream) {
  if (S < 0 || h <= 0 || w <= 0 || (long long)S * h * w > 0x7fffffffLL) return set_error(MOQE_E_SHAPE, "moqe_route_cv: S=%d h=%d w=%d", S, h, w);
  int32_t rc = check_cv_router(r, h, w, "moqe_route_cv");
  if (rc) return rc;
  if (S == 0) return MOQE_OK;
  if (!x || !expert_idx) return set_error(MOQE_E_NULL, "moqe_route_cv: x or expert_idx is NULL");
  if (!aligned(x, 16)) return set_error(MOQE_E_SHAPE, "moqe_route_cv: x must be 16-byte aligned");
  const size_t need = route_cv_ws_bytes(S, h, w, *r);
  if (!workspace || !aligned(workspace, 256) || workspace_bytes < need)
    return set_error(MOQE_E_WORKSPACE, "moqe_route_cv: workspace needs %zu bytes, 256-byte aligned", need);
  if (dry_run()) return MOQE_OK;
  return launch_route_cv(x, S, h, w, *r, expert_idx, logits, workspace, static_cast<hipStream_t>(stream));
}

size_t moqe_route_ragged_workspace_bytes(int32_t S, const moqe_router* r) {
  if (!r || S < 0 || r->d <= 0) return 0;
  return route_ws_bytes(S, 2, *r);
}

int32_t moqe_route_ragged(const void* x, const int32_t* cu_rows, int32_t S, const moqe_router* r, int32_t* expert_idx,
                          float* logits, void* workspace, size_t workspace_bytes, void* stream) {
  int32_t rc = check_router(r, "moqe_route_ragged");
  if (rc) return rc;
  if (S < 0) return set_error(MOQE_E_SHAPE, "moqe_route_ragged: S=%d", S);
  if (S == 0) return MOQE_OK;
  if (!x || !cu_rows || !expert_idx) return set_error(MOQE_E_NULL, "moqe_route_ragged: x, cu_rows or expert_idx is NULL");
  if (!aligned(x, 16)) return set_error(MOQE_E_SHAPE, "moqe_route_ragged: x must be 16-byte aligned");
  if (r->d % 8) return set_error(MOQE_E_SHAPE, "moqe_route_ragged: d=%d must be a multiple of 8", r->d);
  const size_t need = route_ws_bytes(S, 2, *r);
  if (!workspace || !aligned(workspace, 256) || workspace_bytes < need)
    return set_error(MOQE_E_WORKSPACE, "moqe_route_ragged: workspace needs %zu bytes, 256-byte aligned", need);
  if (dry_run()) return MOQE_OK;
  return launch_route_ragged(x, cu_rows, S, *r, expert_idx, logits, workspace, static_cast<hipStream_t>(stream));
}

int32_t moqe_expand_rows(const int32_t* cu_rows, const int32_t* offsets, const int32_t* perm, int32_t S, int32_t K,
                         int32_t* slot_rows, int32_t* row_offsets, int32_t* row_perm, void* stream) {
  if (K < 1 || K > MOQE_MAX_EXPERTS) return set_error(MOQE_E_SHAPE, "moqe_expand_rows: K=%d outside [1, %d]", K, MOQE_MAX_EXPERTS);
  if (S < 0) return set_error(MOQE_E_SHAPE, "moqe_expand_rows: S=%d", S);
  if (!cu_rows || !offsets || !slot_rows || !row_offsets) return set_error(MOQE_E_NULL, "moqe_expand_rows: NULL argument");
  if (S > 0 && (!perm || !row_perm)) return set_error(MOQE_E_NULL, "moqe_expand_rows: perm or row_perm is NULL");
  if (dry_run()) return MOQE_OK;
  return launch_expand_rows(cu_rows, offsets, perm, S, K, slot_rows, row_offsets, row_perm, static_cast<hipStream_t>(stream));
}

int32_t moqe_balance_stats(const float* logits, const int32_t* counts, int32_t S, int32_t K, float alpha, float* out,
                           void* stream) {
  if (K < 1 || K > MOQE_MAX_EXPERTS) return set_error(MOQE_E_SHAPE, "moqe_balance_stats: K=%d outside [1, %d]", K, MOQE_MAX_EXPERTS);
  if (S < 1) return set_error(MOQE_E_SHAPE, "moqe_balance_stats: S=%d", S);
  if (!logits || !counts || !out) return set_error(MOQE_E_NULL, "moqe_balance_stats: logits, counts or out is NULL");
  if (dry_run()) return MOQE_OK;
  return launch_balance_stats(logits, counts, S, K, alpha, out, static_cast<hipStream_t>(stream));
}

// ---- expert weights ------------------------------------------------------------------------
int32_t moqe_quantize_rtn(const float* w, float clip, const moqe_qmat* out, void* stream) {
  if (!w || !out) return set_error(MOQE_E_NULL, "moqe_quantize_rtn: w or out is NULL");
  PackedInfo pi;
  moqe_qmat m = *out;
  m.act_mode = 0;
  int32_t rc = check_qmat_format(m, &pi, "moqe_quantize_rtn");
  if (rc) return rc;
  if (out->layout != MOQE_LAYOUT_CANONICAL) return set_error(MOQE_E_FORMAT, "moqe_quantize_rtn: output must be canonical");
  if (!out->qdata || !out->scale || (!out->symmetric && !out->zero))
    return set_error(MOQE_E_NULL, "moqe_quantize_rtn: output buffers missing");
  if (!(clip > 0.f) || clip > 1.f) return set_error(MOQE_E_SHAPE, "moqe_quantize_rtn: clip %g outside (0, 1]", double(clip));
  if (dry_run()) return MOQE_OK;
  return launch_quantize(w, clip, *out, static_cast<hipStream_t>(stream));
}

size_t moqe_packed_bytes(int32_t n, int32_t k, int32_t bits, int32_t group, int32_t symmetric, int32_t act_mode) {
  PackedInfo pi;
  if (!packed_info(n, k, bits, group, symmetric, act_mode, &pi)) return 0;
  return pi.total;
}

int32_t moqe_pack_qmat(const moqe_qmat* c, void* packed_out, size_t bytes, void* stream) {
  if (!c || !packed_out) return set_error(MOQE_E_NULL, "moqe_pack_qmat: NULL argument");
  PackedInfo pi;
  int32_t rc = check_qmat_format(*c, &pi, "moqe_pack_qmat");
  if (rc) return rc;
  if (c->layout != MOQE_LAYOUT_CANONICAL) return set_error(MOQE_E_FORMAT, "moqe_pack_qmat: input must be canonical");
  if (!c->qdata || !c->scale || (!c->symmetric && !c->zero)) return set_error(MOQE_E_NULL, "moqe_pack_qmat: input buffers missing");
  if (bytes < pi.total || !aligned(packed_out, 256))
    return set_error(MOQE_E_SHAPE, "moqe_pack_qmat: output needs %zu bytes, 256-byte aligned", pi.total);
  if (dry_run()) return MOQE_OK;
  return launch_pack(*c, pi, static_cast<uint8_t*>(packed_out), static_cast<hipStream_t>(stream));
}

int32_t moqe_unpack_qmat(const moqe_qmat* p, int16_t* q_minus_z, float* scale_out, void* stream) {
  if (!p || !q_minus_z) return set_error(MOQE_E_NULL, "moqe_unpack_qmat: NULL argument");
  PackedInfo pi;
  int32_t rc = check_packed(*p, &pi, "moqe_unpack_qmat");
  if (rc) return rc;
  if (dry_run()) return MOQE_OK;
  return launch_unpack(*p, pi, q_minus_z, scale_out, static_cast<hipStream_t>(stream));
}

// ---- grouped GEMM --------------------------------------------------------------------------
size_t moqe_grouped_qgemm_workspace_bytes(const moqe_qmat* experts, int32_t K, int32_t S, int32_t T) {
  if (!experts || K < 1 || K > MOQE_MAX_EXPERTS || S < 0 || T <= 0) return 0;
  bool any = false;
  for (int e = 0; e < K; ++e) any = any || experts[e].act_mode != 0;
  return a8_bytes(any, S * T, experts[0].k);
}

int32_t moqe_grouped_qgemm(const void* a, const int32_t* offsets, const int32_t* perm, int32_t S, int32_t T,
                           const moqe_qmat* experts, int32_t K, void* y, int32_t scatter, void* workspace,
                           size_t workspace_bytes, void* stream) {
  if (!experts) return set_error(MOQE_E_NULL, "moqe_grouped_qgemm: experts is NULL");
  if (K < 1 || K > MOQE_MAX_EXPERTS) return set_error(MOQE_E_SHAPE, "moqe_grouped_qgemm: K=%d outside [1, %d]", K, MOQE_MAX_EXPERTS);
  if (S < 0 || T <= 0 || (long long)S * T > 0x7fffffffLL) return set_error(MOQE_E_SHAPE, "moqe_grouped_qgemm: S=%d T=%d", S, T);
  GroupedPlan gp;
  int32_t rc = plan_experts(experts, K, nullptr, &gp, "moqe_grouped_qgemm");
  if (rc) return rc;
  rc = check_activation_bytes((long long)S * T, experts[0].k, "moqe_grouped_qgemm");
  if (rc) return rc;
  if (S == 0) return MOQE_OK;
  if (!a || !offsets || !y) return set_error(MOQE_E_NULL, "moqe_grouped_qgemm: a, offsets or y is NULL");
  if (!aligned(a, 16) || !aligned(y, 16)) return set_error(MOQE_E_SHAPE, "moqe_grouped_qgemm: a and y must be 16-byte aligned");
  if (scatter & ~(MOQE_SCATTER_OUTPUT | MOQE_INPUT_IN_BUCKET_ORDER | MOQE_OUTPUT_BF16))
    return set_error(MOQE_E_SHAPE, "moqe_grouped_qgemm: unknown bits in scatter=%d", scatter);
  if ((scatter & MOQE_SCATTER_OUTPUT) && !perm) return set_error(MOQE_E_NULL, "moqe_grouped_qgemm: scatter needs perm");
  const size_t need = a8_bytes(gp.any_a8, S * T, experts[0].k);
  if (need && (!workspace || !aligned(workspace, 256) || workspace_bytes < need))
    return set_error(MOQE_E_WORKSPACE, "moqe_grouped_qgemm: workspace needs %zu bytes, 256-byte aligned", need);
  if (dry_run()) return MOQE_OK;
  return run_grouped(a, offsets, (scatter & MOQE_INPUT_IN_BUCKET_ORDER) ? nullptr : perm,
                     (scatter & MOQE_SCATTER_OUTPUT) ? perm : nullptr, S, T, experts, nullptr, K, gp, y,
                     static_cast<uint8_t*>(workspace), static_cast<hipStream_t>(stream), 0, 0, 0,
                     (scatter & MOQE_OUTPUT_BF16) != 0);
}

// ---- the whole block -----------------------------------------------------------------------
namespace {
struct FwdLayout {
  size_t route, idx, logits, counts, offsets, perm, inv_perm, h, a8, total;
};

// routed: the caller brings the experts' indices; the block's own router is neither checked nor used
int32_t forward_layout(const moqe_block* b, int S, int T, FwdLayout* L, GroupedPlan* gp0, GroupedPlan* gp2, bool routed = false) {
  if (!b) return set_error(MOQE_E_NULL, "moqe_forward: block is NULL");
  int32_t rc;
  const int K = b->n_experts;
  if (routed) {
    if (K < 1 || K > MOQE_MAX_EXPERTS) return set_error(MOQE_E_SHAPE, "moqe_forward_routed: n_experts=%d outside [1, %d]", K, MOQE_MAX_EXPERTS);
  } else {
    rc = check_router(&b->router, "moqe_forward");
    if (rc) return rc;
    if (K != b->router.n_experts) return set_error(MOQE_E_SHAPE, "moqe_forward: block has %d experts, router %d", K, b->router.n_experts);
  }
  if (S < 0 || T <= 0 || (long long)S * T > 0x7fffffffLL) return set_error(MOQE_E_SHAPE, "moqe_forward: S=%d T=%d", S, T);
  if (!b->w0) return set_error(MOQE_E_NULL, "moqe_forward: w0 is NULL");
  if (b->kind == MOQE_KIND_SILU_MLP) {
    if (!b->w1 || !b->w2) return set_error(MOQE_E_NULL, "moqe_forward: SILU_MLP needs w1 and w2");
    rc = plan_experts(b->w0, K, b->w1, gp0, "moqe_forward(gate/up)");
    if (rc) return rc;
    rc = plan_experts(b->w2, K, nullptr, gp2, "moqe_forward(down)");
    if (rc) return rc;
    if ((!routed && b->w0[0].k != b->router.d) || b->w2[0].k != b->w0[0].n || b->w2[0].n != b->w0[0].k)
      return set_error(MOQE_E_SHAPE, "moqe_forward: MLP shapes do not chain (d=%d, gate %dx%d, down %dx%d)", b->router.d,
                       b->w0[0].n, b->w0[0].k, b->w2[0].n, b->w2[0].k);
  } else if (b->kind == MOQE_KIND_LINEAR) {
    rc = plan_experts(b->w0, K, nullptr, gp0, "moqe_forward(linear)");
    if (rc) return rc;
    if (!routed && b->w0[0].k != b->router.d) return set_error(MOQE_E_SHAPE, "moqe_forward: linear k=%d but router d=%d", b->w0[0].k, b->router.d);
  } else if (b->kind == MOQE_KIND_CONV3X3) {
    rc = plan_experts(b->w0, K, nullptr, gp0, "moqe_forward(conv)");
    if (rc) return rc;
    if (b->img_h <= 0 || b->img_w <= 0 || b->cin <= 0 || b->img_h * b->img_w != T || (!routed && b->cin != b->router.d) ||
        b->w0[0].k != b->cin * 9 || (b->cin % 8) != 0)
      return set_error(MOQE_E_SHAPE, "moqe_forward: conv needs T = img_h*img_w, cin = router d (a multiple of 8), k = 9*cin");
    if (gp0->any_a8) return set_error(MOQE_E_FORMAT, "moqe_forward: conv experts take bf16 activations (act_mode 0)");
  } else {
    return set_error(MOQE_E_FORMAT, "moqe_forward: unknown block kind %d", b->kind);
  }
  if (b->y_bf16 != 0 && b->y_bf16 != 1) return set_error(MOQE_E_FORMAT, "moqe_forward: y_bf16=%d (0 or 1)", b->y_bf16);
  const size_t M = size_t(S) * T;
  // every activation matrix a kernel indexes: x itself, and the bf16 intermediate of the MLP
  rc = check_activation_bytes((long long)M, b->kind == MOQE_KIND_CONV3X3 ? b->cin : b->w0[0].k, "moqe_forward");
  if (rc) return rc;
  if (b->kind == MOQE_KIND_SILU_MLP) {
    rc = check_activation_bytes((long long)M, b->w0[0].n, "moqe_forward");
    if (rc) return rc;
  }
  size_t o = 0;
  L->route = o;    o += routed ? 0 : align256(route_ws_bytes(S, T, b->router));
  L->idx = o;      o += align256(size_t(S) * 4);
  L->logits = o;   o += align256(size_t(S) * K * 4);
  L->counts = o;   o += align256(size_t(K) * 4);
  L->offsets = o;  o += align256(size_t(K + 1) * 4);
  L->perm = o;     o += align256(size_t(S) * 4);
  L->inv_perm = o; o += align256(size_t(S) * 4);
  L->h = o;
  if (b->kind == MOQE_KIND_SILU_MLP) o += align256(M * size_t(b->w0[0].n) * 2);
  L->a8 = o;
  {
    bool any = gp0->any_a8 || (b->kind == MOQE_KIND_SILU_MLP && gp2->any_a8);
    int kmax = b->w0[0].k;
    if (b->kind == MOQE_KIND_SILU_MLP) kmax = std::max(kmax, b->w2[0].k);
    o += a8_bytes(any, int(M), kmax);
  }
  L->total = o;
  return MOQE_OK;
}
}  // namespace

size_t moqe_workspace_bytes(const moqe_block* blk, int32_t S, int32_t T) {
  FwdLayout L;
  GroupedPlan g0, g2;
  if (forward_layout(blk, S, T, &L, &g0, &g2)) return 0;
  return L.total;
}

// Scratch memory of moqe_forward_static: one array per GPU the library runs on, held until the
// process ends.  In host code the array's name is only a handle for hipGetSymbolAddress; kernels
// get the device address that call returns (kept per device).
static __device__ __align__(256) uint8_t scratch[MOQE_STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[MAX_DEVICES] = {};

int32_t static_scratch(void** out) {
  int dev = -1;
  hipError_t err = hipGetDevice(&dev);
  if (err != hipSuccess) return set_error(MOQE_E_HIP, "moqe_forward_static: hipGetDevice: %s", hipGetErrorString(err));
  if (dev < 0 || dev >= MAX_DEVICES) return set_error(MOQE_E_HIP, "moqe_forward_static: device %d outside [0, %d)", dev, MAX_DEVICES);
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (err != hipSuccess || !p)
      return set_error(MOQE_E_HIP, "moqe_forward_static: address of the built-in scratch buffer: %s", hipGetErrorString(err));
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return MOQE_OK;
}

int32_t forward_body(const moqe_block* blk, const void* x, int32_t S, int32_t T, void* y, const moqe_aux* aux,
                     const FwdLayout& L, const GroupedPlan& g0, const GroupedPlan& g2, void* workspace, void* stream,
                     const int32_t* given_idx = nullptr);
}  // namespace

int32_t moqe_forward(const moqe_block* blk, const void* x, int32_t S, int32_t T, void* y, const moqe_aux* aux,
                     void* workspace, size_t workspace_bytes, void* stream) {
  FwdLayout L;
  GroupedPlan g0, g2;
  int32_t rc = forward_layout(blk, S, T, &L, &g0, &g2);
  if (rc) return rc;
  if (S == 0) return MOQE_OK;
  if (!x || !y) return set_error(MOQE_E_NULL, "moqe_forward: x or y is NULL");
  if (!aligned(x, 16) || !aligned(y, 16)) return set_error(MOQE_E_SHAPE, "moqe_forward: x and y must be 16-byte aligned");
  if (!workspace || !aligned(workspace, 256) || workspace_bytes < L.total)
    return set_error(MOQE_E_WORKSPACE, "moqe_forward: workspace needs %zu bytes, 256-byte aligned", L.total);
  if (dry_run()) return MOQE_OK;
  return forward_body(blk, x, S, T, y, aux, L, g0, g2, workspace, stream);
}

int32_t moqe_forward_routed(const moqe_block* blk, const int32_t* expert_idx, const void* x, int32_t S, int32_t T, void* y,
                            const moqe_aux* aux, void* workspace, size_t workspace_bytes, void* stream) {
  FwdLayout L;
  GroupedPlan g0, g2;
  int32_t rc = forward_layout(blk, S, T, &L, &g0, &g2, true);
  if (rc) return rc;
  if (S == 0) return MOQE_OK;
  if (!x || !y || !expert_idx) return set_error(MOQE_E_NULL, "moqe_forward_routed: x, y or expert_idx is NULL");
  if (!aligned(x, 16) || !aligned(y, 16)) return set_error(MOQE_E_SHAPE, "moqe_forward_routed: x and y must be 16-byte aligned");
  if (!workspace || !aligned(workspace, 256) || workspace_bytes < L.total)
    return set_error(MOQE_E_WORKSPACE, "moqe_forward_routed: workspace needs %zu bytes, 256-byte aligned", L.total);
  if (dry_run()) return MOQE_OK;
  return forward_body(blk, x, S, T, y, aux, L, g0, g2, workspace, stream, expert_idx);
}

size_t moqe_workspace_bytes_routed(const moqe_block* blk, int32_t S, int32_t T) {
  FwdLayout L;
  GroupedPlan g0, g2;
  if (forward_layout(blk, S, T, &L, &g0, &g2, true)) return 0;
  return L.total;
}

int32_t moqe_forward_static(const moqe_block* blk, const void* x, int32_t S, int32_t T, void* y, const moqe_aux* aux,
                            void* stream) {
  FwdLayout L;
  GroupedPlan g0, g2;
  int32_t rc = forward_layout(blk, S, T, &L, &g0, &g2);
  if (rc) return rc;
  if (L.total > size_t(MOQE_STATIC_SCRATCH_BYTES))
    return set_error(MOQE_E_WORKSPACE, "moqe_forward_static: this batch needs %zu bytes of scratch, the built-in buffer holds %zu "
                     "(use moqe_forward with a workspace)", L.total, size_t(MOQE_STATIC_SCRATCH_BYTES));
  if (S == 0) return MOQE_OK;
  if (!x || !y) return set_error(MOQE_E_NULL, "moqe_forward_static: x or y is NULL");
  if (!aligned(x, 16) || !aligned(y, 16)) return set_error(MOQE_E_SHAPE, "moqe_forward_static: x and y must be 16-byte aligned");
  if (dry_run()) return MOQE_OK;
  void* ws = nullptr;
  rc = static_scratch(&ws);
  if (rc) return rc;
  // every kernel of the block writes what it later reads, so nothing in the buffer has to start at zero
  return forward_body(blk, x, S, T, y, aux, L, g0, g2, ws, stream);
}

namespace {
int32_t forward_body(const moqe_block* blk, const void* x, int32_t S, int32_t T, void* y, const moqe_aux* aux,
                     const FwdLayout& L, const GroupedPlan& g0, const GroupedPlan& g2, void* workspace, void* stream,
                     const int32_t* given_idx) {
  int32_t rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  uint8_t* ws = static_cast<uint8_t*>(workspace);
  const int K = blk->n_experts;
  int32_t* idx = reinterpret_cast<int32_t*>(ws + L.idx);
  float* logits = reinterpret_cast<float*>(ws + L.logits);
  int32_t* counts = reinterpret_cast<int32_t*>(ws + L.counts);
  int32_t* offsets = reinterpret_cast<int32_t*>(ws + L.offsets);
  int32_t* perm = reinterpret_cast<int32_t*>(ws + L.perm);
  int32_t* inv_perm = reinterpret_cast<int32_t*>(ws + L.inv_perm);
  if (aux) {   // write straight into the caller's buffers where given
    if (aux->expert_idx) idx = aux->expert_idx;
    if (aux->logits) logits = aux->logits;
    if (aux->counts) counts = aux->counts;
    if (aux->offsets) offsets = aux->offsets;
    if (aux->perm) perm = aux->perm;
    if (aux->inv_perm) inv_perm = aux->inv_perm;
  }

  // Small batches whose first grouped launch is the streaming kernel: that launch buckets the samples itself, which takes
  // the bucket kernel (and one dependent read of its result) out of the chain router -> experts.
  const bool self = blk->kind != MOQE_KIND_CONV3X3 && can_self_bucket(S, T, blk->w0[0].k, g0);
  float* want_logits = (aux && aux->logits) ? logits : nullptr;
  int32_t* want_inv = (aux && aux->inv_perm) ? inv_perm : nullptr;
  const int32_t* chosen = idx;
  if (given_idx) {                      // routed by the caller: only the bucketing is left to do
    chosen = given_idx;
    rc = self ? MOQE_OK : launch_bucket(given_idx, S, K, counts, offsets, perm, want_inv, st);
  } else if (self) {
    rc = launch_route(x, S, T, blk->router, idx, want_logits, ws + L.route, st);
  } else {
    rc = launch_route_bucket(x, S, T, blk->router, idx, want_logits, counts, offsets, perm, want_inv, ws + L.route, st);
  }
  if (rc) return rc;
  const SelfBucket sb{chosen, counts, offsets, perm, want_inv};
  const SelfBucket* psb = self ? &sb : nullptr;

  const bool yb = blk->y_bf16 != 0;
  if (blk->kind == MOQE_KIND_LINEAR) {
    return run_grouped(x, offsets, perm, perm, S, T, blk->w0, nullptr, K, g0, y, ws + L.a8, st, 0, 0, 0, yb, psb);
  }
  if (blk->kind == MOQE_KIND_SILU_MLP) {
    void* h = (aux && aux->h) ? aux->h : static_cast<void*>(ws + L.h);
    rc = run_grouped(x, offsets, perm, nullptr, S, T, blk->w0, blk->w1, K, g0, h, ws + L.a8, st, 0, 0, 0, false, psb);
    if (rc) return rc;
    return run_grouped(h, offsets, nullptr, perm, S, T, blk->w2, nullptr, K, g2, y, ws + L.a8, st, 0, 0, 0, yb);
  }
  // CONV3X3: the tiled kernel gathers each row's 3x3 neighbourhood from the image itself
  return run_grouped(x, offsets, perm, perm, S, T, blk->w0, nullptr, K, g0, y, ws + L.a8, st, blk->img_h, blk->img_w, blk->cin, yb);
}
}  // namespace

// ---- the router's training labels ------------------------------------------------------------
namespace {
struct LabelLayout {
  size_t offsets, perm, y, h, a8, total;
  int n_out;
};

int32_t label_layout(const moqe_block* b, int S, int T, LabelLayout* L, GroupedPlan* gp0, GroupedPlan* gp2) {
  const char* who = "moqe_label_pass";
  if (!b) return set_error(MOQE_E_NULL, "%s: block is NULL", who);
  const int K = b->n_experts;
  if (K < 1 || K > MOQE_MAX_EXPERTS) return set_error(MOQE_E_SHAPE, "%s: n_experts=%d outside [1, %d]", who, K, MOQE_MAX_EXPERTS);
  if (b->kind != MOQE_KIND_LINEAR && b->kind != MOQE_KIND_SILU_MLP)
    return set_error(MOQE_E_FORMAT, "%s: kind %d (the rows of the block's output must be logits)", who, b->kind);
  if (S < 0 || T <= 0 || (long long)S * T * K > 0x7fffffffLL) return set_error(MOQE_E_SHAPE, "%s: S=%d T=%d K=%d", who, S, T, K);
  if (!b->w0) return set_error(MOQE_E_NULL, "%s: w0 is NULL", who);
  const bool mlp = b->kind == MOQE_KIND_SILU_MLP;
  int32_t rc = plan_experts(b->w0, K, mlp ? b->w1 : nullptr, gp0, who);
  if (rc) return rc;
  if (mlp) {
    if (!b->w1 || !b->w2) return set_error(MOQE_E_NULL, "%s: SILU_MLP needs w1 and w2", who);
    rc = plan_experts(b->w2, K, nullptr, gp2, who);
    if (rc) return rc;
    if (b->w2[0].k != b->w0[0].n) return set_error(MOQE_E_SHAPE, "%s: down takes %d features, gate/up give %d", who, b->w2[0].k, b->w0[0].n);
  }
  const long long MV = (long long)S * T * K;                 // rows of the K*S virtual samples
  rc = check_activation_bytes((long long)S * T, b->w0[0].k, who);
  if (rc) return rc;
  if (mlp) {
    rc = check_activation_bytes(MV, b->w0[0].n, who);
    if (rc) return rc;
  }
  L->n_out = mlp ? b->w2[0].n : b->w0[0].n;
  size_t o = 0;
  L->offsets = o; o += align256(size_t(K + 1) * 4);
  L->perm = o;    o += align256(size_t(K) * S * 4);
  L->y = o;       o += align256(size_t(MV) * L->n_out * 4);
  L->h = o;
  if (mlp) o += align256(size_t(MV) * size_t(b->w0[0].n) * 2);
  L->a8 = o;
  {
    bool any = gp0->any_a8 || (mlp && gp2->any_a8);
    int kmax = b->w0[0].k;
    if (mlp) kmax = std::max(kmax, b->w2[0].k);
    o += a8_bytes(any, int(MV), kmax);
  }
  L->total = o;
  return MOQE_OK;
}
}  // namespace

size_t moqe_label_pass_workspace_bytes(const moqe_block* blk, int32_t S, int32_t T) {
  LabelLayout L;
  GroupedPlan g0, g2;
  if (label_layout(blk, S, T, &L, &g0, &g2)) return 0;
  return L.total;
}

int32_t moqe_label_pass(const moqe_block* blk, const void* x, const int32_t* targets, int32_t S, int32_t T, float* losses,
                        int32_t* labels, void* workspace, size_t workspace_bytes, void* stream) {
  LabelLayout L;
  GroupedPlan g0, g2;
  int32_t rc = label_layout(blk, S, T, &L, &g0, &g2);
  if (rc) return rc;
  if (S == 0) return MOQE_OK;
  if (!x || !targets || !losses || !labels) return set_error(MOQE_E_NULL, "moqe_label_pass: x, targets, losses or labels is NULL");
  if (!aligned(x, 16)) return set_error(MOQE_E_SHAPE, "moqe_label_pass: x must be 16-byte aligned");
  if (!workspace || !aligned(workspace, 256) || workspace_bytes < L.total)
    return set_error(MOQE_E_WORKSPACE, "moqe_label_pass: workspace needs %zu bytes, 256-byte aligned", L.total);
  if (dry_run()) return MOQE_OK;
  hipStream_t st = static_cast<hipStream_t>(stream);
  uint8_t* ws = static_cast<uint8_t*>(workspace);
  const int K = blk->n_experts;
  int32_t* offsets = reinterpret_cast<int32_t*>(ws + L.offsets);
  int32_t* perm = reinterpret_cast<int32_t*>(ws + L.perm);
  float* yv = reinterpret_cast<float*>(ws + L.y);
  rc = launch_label_dispatch(S, K, offsets, perm, st);
  if (rc) return rc;
  // K*S virtual samples, expert j's bucket = every sample; the logits stay in bucket order
  if (blk->kind == MOQE_KIND_LINEAR) {
    rc = run_grouped(x, offsets, perm, nullptr, K * S, T, blk->w0, nullptr, K, g0, yv, ws + L.a8, st);
  } else {
    rc = run_grouped(x, offsets, perm, nullptr, K * S, T, blk->w0, blk->w1, K, g0, ws + L.h, ws + L.a8, st);
    if (rc) return rc;
    rc = run_grouped(ws + L.h, offsets, nullptr, nullptr, K * S, T, blk->w2, nullptr, K, g2, yv, ws + L.a8, st);
  }
  if (rc) return rc;
  return launch_label_loss(yv, targets, S, T, L.n_out, K, losses, labels, st);
}

// ---- the whole block, samples of different lengths -------------------------------------------
namespace {
struct RaggedLayout {
  size_t route, idx, logits, counts, offsets, perm, inv_perm, slot_rows, row_offsets, row_perm, h, a8, total;
};

int32_t ragged_layout(const moqe_block* b, int S, long long M, RaggedLayout* L, GroupedPlan* gp0, GroupedPlan* gp2) {
  if (!b) return set_error(MOQE_E_NULL, "moqe_forward_ragged: block is NULL");
  int32_t rc = check_router(&b->router, "moqe_forward_ragged");
  if (rc) return rc;
  const int K = b->n_experts;
  if (K < 1 || K > MOQE_MAX_EXPERTS || K != b->router.n_experts)
    return set_error(MOQE_E_SHAPE, "moqe_forward_ragged: n_experts=%d (router %d)", K, b->router.n_experts);
  if (b->kind != MOQE_KIND_LINEAR && b->kind != MOQE_KIND_SILU_MLP)
    return set_error(MOQE_E_FORMAT, "moqe_forward_ragged: kind %d (images have a fixed number of pixels)", b->kind);
  if (S < 0 || M < S || M > 0x7fffffffLL) return set_error(MOQE_E_SHAPE, "moqe_forward_ragged: S=%d M=%lld", S, M);
  if (b->y_bf16 != 0 && b->y_bf16 != 1) return set_error(MOQE_E_FORMAT, "moqe_forward_ragged: y_bf16=%d (0 or 1)", b->y_bf16);
  if (!b->w0) return set_error(MOQE_E_NULL, "moqe_forward_ragged: w0 is NULL");
  rc = plan_experts(b->w0, K, b->kind == MOQE_KIND_SILU_MLP ? b->w1 : nullptr, gp0, "moqe_forward_ragged");
  if (rc) return rc;
  if (b->w0[0].k != b->router.d) return set_error(MOQE_E_SHAPE, "moqe_forward_ragged: experts take %d features, the router %d", b->w0[0].k, b->router.d);
  if (b->router.d % 8) return set_error(MOQE_E_SHAPE, "moqe_forward_ragged: d=%d must be a multiple of 8", b->router.d);
  if (b->kind == MOQE_KIND_SILU_MLP) {
    if (!b->w1 || !b->w2) return set_error(MOQE_E_NULL, "moqe_forward_ragged: w1 or w2 is NULL");
    rc = plan_experts(b->w2, K, nullptr, gp2, "moqe_forward_ragged");
    if (rc) return rc;
    if (b->w2[0].k != b->w0[0].n) return set_error(MOQE_E_SHAPE, "moqe_forward_ragged: down takes %d features, gate/up give %d", b->w2[0].k, b->w0[0].n);
  }
  rc = check_activation_bytes(M, b->router.d, "moqe_forward_ragged");
  if (rc) return rc;
  if (b->kind == MOQE_KIND_SILU_MLP) {
    rc = check_activation_bytes(M, b->w0[0].n, "moqe_forward_ragged");
    if (rc) return rc;
  }
  size_t o = 0;
  L->route = o;       o += align256(route_ws_bytes(S, 2, b->router));
  L->idx = o;         o += align256(size_t(S) * 4);
  L->logits = o;      o += align256(size_t(S) * K * 4);
  L->counts = o;      o += align256(size_t(K) * 4);
  L->offsets = o;     o += align256(size_t(K + 1) * 4);
  L->perm = o;        o += align256(size_t(S) * 4);
  L->inv_perm = o;    o += align256(size_t(S) * 4);
  L->slot_rows = o;   o += align256(size_t(S + 1) * 4);
  L->row_offsets = o; o += align256(size_t(K + 1) * 4);
  L->row_perm = o;    o += align256(size_t(M) * 4);
  L->h = o;
  if (b->kind == MOQE_KIND_SILU_MLP) o += align256(size_t(M) * size_t(b->w0[0].n) * 2);
  L->a8 = o;
  {
    bool any = gp0->any_a8 || (b->kind == MOQE_KIND_SILU_MLP && gp2->any_a8);
    int kmax = b->w0[0].k;
    if (b->kind == MOQE_KIND_SILU_MLP) kmax = std::max(kmax, b->w2[0].k);
    o += a8_bytes(any, int(M), kmax);
  }
  L->total = o;
  return MOQE_OK;
}
}  // namespace

size_t moqe_workspace_bytes_ragged(const moqe_block* blk, int32_t S, int32_t M) {
  RaggedLayout L;
  GroupedPlan g0, g2;
  if (ragged_layout(blk, S, M, &L, &g0, &g2)) return 0;
  return L.total;
}

int32_t moqe_forward_ragged(const moqe_block* blk, const void* x, const int32_t* cu_rows, int32_t S, int32_t M, void* y,
                            const moqe_aux* aux, void* workspace, size_t workspace_bytes, void* stream) {
  RaggedLayout L;
  GroupedPlan g0, g2;
  int32_t rc = ragged_layout(blk, S, M, &L, &g0, &g2);
  if (rc) return rc;
  if (S == 0) return MOQE_OK;
  if (!x || !y || !cu_rows) return set_error(MOQE_E_NULL, "moqe_forward_ragged: x, y or cu_rows is NULL");
  if (!aligned(x, 16) || !aligned(y, 16)) return set_error(MOQE_E_SHAPE, "moqe_forward_ragged: x and y must be 16-byte aligned");
  if (!workspace || !aligned(workspace, 256) || workspace_bytes < L.total)
    return set_error(MOQE_E_WORKSPACE, "moqe_forward_ragged: workspace needs %zu bytes, 256-byte aligned", L.total);
  if (dry_run()) return MOQE_OK;

  hipStream_t st = static_cast<hipStream_t>(stream);
  uint8_t* ws = static_cast<uint8_t*>(workspace);
  const int K = blk->n_experts;
  int32_t* idx = reinterpret_cast<int32_t*>(ws + L.idx);
  float* logits = reinterpret_cast<float*>(ws + L.logits);
  int32_t* counts = reinterpret_cast<int32_t*>(ws + L.counts);
  int32_t* offsets = reinterpret_cast<int32_t*>(ws + L.offsets);
  int32_t* perm = reinterpret_cast<int32_t*>(ws + L.perm);
  int32_t* inv_perm = reinterpret_cast<int32_t*>(ws + L.inv_perm);
  if (aux) {
    if (aux->expert_idx) idx = aux->expert_idx;
    if (aux->logits) logits = aux->logits;
    if (aux->counts) counts = aux->counts;
    if (aux->offsets) offsets = aux->offsets;
    if (aux->perm) perm = aux->perm;
    if (aux->inv_perm) inv_perm = aux->inv_perm;
  }
  int32_t* slot_rows = reinterpret_cast<int32_t*>(ws + L.slot_rows);
  int32_t* row_offsets = reinterpret_cast<int32_t*>(ws + L.row_offsets);
  int32_t* row_perm = reinterpret_cast<int32_t*>(ws + L.row_perm);

  rc = launch_route_ragged(x, cu_rows, S, blk->router, idx, (aux && aux->logits) ? logits : nullptr, ws + L.route, st);
  if (rc) return rc;
  rc = launch_bucket(idx, S, K, counts, offsets, perm, (aux && aux->inv_perm) ? inv_perm : nullptr, st);
  if (rc) return rc;
  rc = launch_expand_rows(cu_rows, offsets, perm, S, K, slot_rows, row_offsets, row_perm, st);
  if (rc) return rc;
  // from here on every row is its own "sample": bucket offsets and permutation at row granularity
  if (blk->kind == MOQE_KIND_LINEAR)
    return run_grouped(x, row_offsets, row_perm, row_perm, M, 1, blk->w0, nullptr, K, g0, y, ws + L.a8, st, 0, 0, 0, blk->y_bf16 != 0);
  void* h = (aux && aux->h) ? aux->h : static_cast<void*>(ws + L.h);
  rc = run_grouped(x, row_offsets, row_perm, nullptr, M, 1, blk->w0, blk->w1, K, g0, h, ws + L.a8, st);
  if (rc) return rc;
  return run_grouped(h, row_offsets, nullptr, row_perm, M, 1, blk->w2, nullptr, K, g2, y, ws + L.a8, st, 0, 0, 0, blk->y_bf16 != 0);
}

// ---- timing --------------------------------------------------------------------------------
int32_t moqe_profile_enable(int32_t kind_mask) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  g_prof.clear();
  g_prof_mask = uint32_t(kind_mask) & ((1u << MOQE_PK_COUNT) - 1u);
  return MOQE_OK;
}

int32_t moqe_profile_read(int32_t kind, int32_t* launches, double* total_ms) {
  if (!launches || !total_ms) return set_error(MOQE_E_NULL, "moqe_profile_read: NULL argument");
  if (kind < 0 || kind >= MOQE_PK_COUNT) return set_error(MOQE_E_SHAPE, "moqe_profile_read: kind %d", kind);
  std::lock_guard<std::mutex> lk(g_prof_mu);
  int n = 0;
  double ms = 0.0;
  for (auto& r : g_prof) {
    if (r.kind != kind) continue;
    hipEvent_t a = g_pool[2 * r.ev], b = g_pool[2 * r.ev + 1];
    hipError_t err = hipEventSynchronize(b);
    if (err != hipSuccess) return set_error(MOQE_E_HIP, "moqe_profile_read: %s", hipGetErrorString(err));
    float t = 0.f;
    err = hipEventElapsedTime(&t, a, b);
    if (err != hipSuccess) return set_error(MOQE_E_HIP, "moqe_profile_read: %s", hipGetErrorString(err));
    ms += double(t);
    ++n;
  }
  *launches = n;
  *total_ms = ms;
  return MOQE_OK;
}

}  // extern "C"
