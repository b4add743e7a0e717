/*
 * moqe.h - C ABI of the MI355X (gfx950) library for the routed forward pass through
 * K quantization experts (MoQE, arXiv 2508.09204).
 *
 * The operation.  MoQE keeps several quantized variants ("quantization experts") of one
 * full-precision model.  A router model scores each data sample (a sequence, an image),
 * ONE expert is selected per sample, and that expert alone performs the inference on it
 * (Section 3.1, Figure 1; the system's prediction is f_{r(x)}(x), appendix on router
 * convergence; every input activates exactly one expert, appendix on the number of
 * experts).  This library runs that pattern for a BATCH of samples with all experts
 * resident: score and select (moqe_route), group samples by expert (moqe_bucket; its
 * counts are the n_i of Eq. 2), run each group through its expert's low-bit weights
 * (moqe_grouped_qgemm) and put results back in the caller's order; moqe_forward chains
 * these for one block.  The per-sample result is the same as serving samples one by one.
 * Beside the block: the paper's two router models (moqe_route_nlp, moqe_route_cv; Section 3.2), whose choice
 * drives the block through moqe_forward_routed; the router-training label pass and the load-balance
 * statistics of Section 3.3 (moqe_label_pass, moqe_balance_stats); samples of different lengths
 * (moqe_*_ragged); on-demand residency of the experts' weights (moqe_cache_*, Section 4.4).
 *
 * Conventions (all entry points).
 *  - Return value: 0 on success, a negative MOQE_E_* code on failure.  Every argument
 *    check (shapes, formats, sizes, alignment, workspace) runs before the first launch, so
 *    an argument error enqueues nothing; only MOQE_E_HIP (the runtime refused a launch) can
 *    come after part of a call's work was enqueued.  moqe_last_error_string() gives a
 *    thread-local description.
 *  - Pointers named in "device" comments are DEVICE pointers owned by the caller; the
 *    library does not allocate, free or retain device memory, with one exception: an expert
 *    cache (moqe_cache_create) owns the device slots it allocates until moqe_cache_destroy.
 *    An activation matrix (rows x features, bf16) and a packed weight matrix must each stay below 4 GiB
 *    (the kernels address them with 32-bit byte offsets; larger ones are refused with MOQE_E_SHAPE).  Descriptor structs
 *    (moqe_qmat, moqe_router, moqe_nlp_router, moqe_cv_router, moqe_block, moqe_aux) and arrays of them are HOST memory,
 *    read during the call only.  Scratch memory is a caller-provided device workspace
 *    whose size comes from the matching *_workspace_bytes query; it must be 256-byte
 *    aligned and may be reused between calls on the same stream.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *    enqueue work on it and never synchronise the host.
 *  - Activations are bfloat16 (raw 16-bit patterns), row-major.  A "sample" owns T
 *    consecutive rows; M = S*T.  Weight matrices are [n, k] = [out, in], groups run
 *    along k.
 *  - Shapes accepted by the packed layout: n % 16 == 0, k % 128 == 0.
 */
#ifndef MOQE_H
#define MOQE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MOQE_OK             0
#define MOQE_E_NULL        (-1)  /* a required pointer is NULL */
#define MOQE_E_SHAPE       (-2)  /* bad size, alignment or inconsistent shapes */
#define MOQE_E_FORMAT      (-3)  /* unsupported bits / group / symmetry / layout / act_mode */
#define MOQE_E_WORKSPACE   (-4)  /* workspace missing, misaligned or too small */
#define MOQE_E_HIP         (-5)  /* the HIP runtime reported an error */

#define MOQE_MAX_EXPERTS   16

#define MOQE_LAYOUT_CANONICAL 0  /* one code per byte, row-major [n, k] */
#define MOQE_LAYOUT_PACKED    1  /* the device layout written by moqe_pack_qmat */

#define MOQE_KIND_LINEAR    0
#define MOQE_KIND_SILU_MLP  1
#define MOQE_KIND_CONV3X3   2

/* One quantized weight matrix of one expert.  The real weight is scale * (code - zero).
 *
 * Supported formats (the paper names Int8 and Int4 experts, Sections 4.1-4.3; the formats
 * themselves are round-to-nearest ones):
 *   symmetric per output channel, bits 8 / 6 / 4: group = 0, zero = NULL, codes signed in
 *     [-(2^(bits-1)-1), 2^(bits-1)-1];
 *   asymmetric group-wise, bits 4 / 3: group = 64 or 128 along k, codes in [0, 2^bits-1],
 *     zero in the same range.
 * Canonical layout: qdata is int8 (symmetric) or uint8 (asymmetric), [n, k] row-major;
 *   scale is float [n] (group 0) or [n, k/group]; zero is uint8 with the shape of scale.
 * Packed layout: qdata is the blob written by moqe_pack_qmat (codes, scales and
 *   zero-points inside); scale and zero are ignored and may be NULL.
 * act_mode 1 (int8 per-channel symmetric only): activations are quantized per row to
 *   int8 with a dynamic scale and the product runs on integer matrix cores (W8A8). */
typedef struct moqe_qmat {
  const void*    qdata;      /* device */
  const float*   scale;      /* device */
  const uint8_t* zero;       /* device, NULL when symmetric */
  int32_t n, k;
  int32_t bits;              /* 8, 6, 4, 3 */
  int32_t group;             /* 0, 64, 128 */
  int32_t symmetric;         /* 0 / 1 */
  int32_t act_mode;          /* 0: bf16 activations, 1: per-row dynamic int8 activations */
  int32_t layout;            /* MOQE_LAYOUT_* */
} moqe_qmat;

/* Router: mean-pool the sample's rows, then [Linear(d->h), ReLU,] Linear(->K) giving one
 * logit per expert (the router ends in an MLP that maps features to routing logits,
 * Section 3.2).  h == 0: single linear layer, w1/b1 unused.  Weights fp32 row-major
 * [out, in]; biases may be NULL. */
typedef struct moqe_router {
  const float* w1; const float* b1;   /* device, [h, d], [h] */
  const float* w2; const float* b2;   /* device, [K, h or d], [K] */
  int32_t d, h, n_experts;
} moqe_router;

/* The NLP router model (Section 3.2, "NLP Router Model"): a Transformer encoder makes every token vector
 * context-aware, a dedicated self-attention module re-weights these representations, and an MLP maps the
 * refined features to one logit per expert.  The paper fixes the order of the stages, not their sizes; here
 *   u = x W_in^T + b_in                                         token vectors [T, d] -> width dm
 *   v = LN1(u + MHA1(u));  w = LN2(v + W_ff2 relu(W_ff1 v + b_ff1) + b_ff2)       one post-norm encoder layer
 *   z = LN3(w + MHA2(w))                                        the attention module
 *   logits = head(mean over the T tokens of z)                  head: Linear(dm -> h) -> ReLU -> Linear(h -> K)
 * MHA(u): n_heads heads of width dm / n_heads; [Q K V] = u Wqkv^T + bqkv (rows of Wqkv: queries, keys,
 * values); head h uses columns h*dh .. (h+1)*dh; softmax(Q K^T / sqrt(dh)) V, heads concatenated, then
 * Wo and bo.  No mask, no positional term.  LayerNorm: biased variance, eps 1e-5, gain g and offset b.
 * All parameters device fp32, matrices row-major [out, in].  d a multiple of 64; dm and d_ff multiples of
 * 128, dm <= 2048; dm / n_heads in {16, 32, 64, 128}; head.d == dm. */
typedef struct moqe_nlp_router {
  const float *w_in, *b_in;                              /* [dm, d], [dm] */
  const float *wqkv1, *bqkv1, *wo1, *bo1;                /* [3dm, dm], [3dm], [dm, dm], [dm] */
  const float *ln1_g, *ln1_b;                            /* [dm] */
  const float *w_ff1, *b_ff1, *w_ff2, *b_ff2;            /* [d_ff, dm], [d_ff], [dm, d_ff], [dm] */
  const float *ln2_g, *ln2_b;
  const float *wqkv2, *bqkv2, *wo2, *bo2;
  const float *ln3_g, *ln3_b;
  moqe_router head;
  int32_t d, dm, n_heads, d_ff;
} moqe_nlp_router;

/* The CV router model (Section 3.2, "CV Router Model"): a three-layer MLP, every linear layer followed by batch
 * normalisation and ReLU; a three-stage SEResNet-8 (the paper: 16, 32, 64 channels, strides 1, 2, 2); the last
 * feature map flattened into a sequence and fed to a multi-head self-attention module (the paper: 8 heads) that
 * gives the routing logits.  The paper fixes this order; the rest is read as follows.
 *   MLP      : on every pixel's channel vector, x <- relu(bn(W x + b)), three times (widths mlp_n).
 *   bn       : (x - mean) / sqrt(var + 1e-5) * gain + offset per channel (stored statistics).
 *   stage    : a = relu(bn_a(conv3x3(x, conv_a, stride)));  u = bn_b(conv3x3(a, conv_b, 1));
 *              g = sigmoid(se_w2 relu(se_w1 mean_pixels(u) + se_b1) + se_b2)   (squeeze width cout / 4);
 *              x <- relu(u * g + shortcut), shortcut = x, or short_bn(conv1x1(x, short_w, stride)) when short_w is
 *              given (required when the stride is 2 or the width changes).  3x3 convolutions pad by 1; filters are
 *              [cout, kh, kw, cin] (taps slow, channels fast), short_w is [cout, cin].
 *   attention: on the h' * w' positions of the last map (width dm = stage[2].cout): [Q K V] = x Wqkv^T + bqkv (rows of
 *              Wqkv: queries, keys, values), heads of width dm / n_heads, softmax(Q K^T / sqrt(dh)) V, Wo and bo,
 *              mean over the positions;  logits = w_out mean + b_out.
 * All parameters device fp32.  Widths multiples of 4 and at most 64, dm a multiple of 8, head width at most 16, at most
 * 36 positions in the last map (inputs up to 24 x 24 with the paper's strides); w_out 16-byte aligned. */
typedef struct moqe_bn { const float *gain, *offset, *mean, *var; } moqe_bn;
typedef struct moqe_cv_stage {
  const float* conv_a; moqe_bn bn_a;
  const float* conv_b; moqe_bn bn_b;
  const float *se_w1, *se_b1, *se_w2, *se_b2;
  const float* short_w; moqe_bn short_bn;                /* short_w NULL: identity shortcut */
  int32_t cout, stride;
} moqe_cv_stage;
typedef struct moqe_cv_router {
  const float* mlp_w[3]; const float* mlp_b[3]; moqe_bn mlp_bn[3]; int32_t mlp_n[3];
  moqe_cv_stage stage[3];
  const float *wqkv, *bqkv, *wo, *bo;                    /* [3dm, dm], [3dm], [dm, dm], [dm] */
  const float *w_out, *b_out;                            /* [K, dm], [K] or NULL */
  int32_t c_in, n_heads, n_experts;
} moqe_cv_router;

/* One routed block.  w0/w1/w2 are host arrays of n_experts PACKED matrices.
 *   LINEAR   : y = x W0^T.                         x [S*T, d], y [S*T, n]
 *   SILU_MLP : h = bf16(silu(x Wg^T) * (x Wu^T)), y = h Wd^T with w0 = gate, w1 = up,
 *              w2 = down; gate and up of an expert share one format.
 *   CONV3X3  : per image, 3x3 convolution, stride 1, zero padding 1, no bias.  x is NHWC
 *              [S, img_h, img_w, cin] (T = img_h*img_w), w0[e] is [cout, cin*9] with
 *              k = (kh*3 + kw)*cin + c (taps slow, channels fast, like x); y is NHWC fp32 (bf16 with y_bf16). */
typedef struct moqe_block {
  int32_t kind;
  moqe_router router;
  const moqe_qmat* w0;
  const moqe_qmat* w1;
  const moqe_qmat* w2;
  int32_t n_experts;
  int32_t img_h, img_w, cin;          /* CONV3X3 only */
  int32_t y_bf16;                     /* 0: y is fp32; 1: y is bf16 (each result rounded once, nearest even): half the
                                         output bytes where the next layer takes bf16 anyway */
} moqe_block;

/* Optional extra outputs of moqe_forward (any member may be NULL; all device). */
typedef struct moqe_aux {
  int32_t* expert_idx;   /* [S]    selected expert per sample */
  float*   logits;       /* [S, K] router logits */
  int32_t* counts;       /* [K]    samples per expert (n_i of Eq. 2) */
  int32_t* offsets;      /* [K+1]  exclusive prefix sum of counts */
  int32_t* perm;         /* [S]    bucket slot -> sample */
  int32_t* inv_perm;     /* [S]    sample -> bucket slot */
  void*    h;            /* SILU_MLP: the bf16 intermediate [S*T, F] in bucket order */
} moqe_aux;

const char* moqe_version(void);
const char* moqe_last_error_string(void);

/* When on, entry points validate their arguments and return without touching the GPU. */
void moqe_set_dry_run(int32_t on);

/* ---- routing ------------------------------------------------------------------------ */

/* Scores each sample and takes the top-1 expert (Section 3.1: the router decides which
 * expert is activated).  x: device bf16 [S*T, r->d].  expert_idx: device int32 [S];
 * among equal maxima the lowest index wins.  logits: device float [S, K] or NULL.
 * Pooling and both layers accumulate in fp32. */
size_t  moqe_route_workspace_bytes(int32_t S, int32_t T, const moqe_router* r);
int32_t moqe_route(const void* x, int32_t S, int32_t T, const moqe_router* r,
                   int32_t* expert_idx, float* logits,
                   void* workspace, size_t workspace_bytes, void* stream);

/* Groups samples by expert with a stable counting sort (the per-expert dispatch counts
 * n_i of Eq. 2 and the permutation that makes each expert's samples contiguous).
 *   counts[k] = #{s : e[s] = k};  offsets = exclusive prefix sum, offsets[K] = S;
 *   inv_perm[s] = offsets[e[s]] + #{s' < s : e[s'] = e[s]};  perm[inv_perm[s]] = s.
 * expert_idx values must lie in [0, K); K <= MOQE_MAX_EXPERTS.  All arrays device int32;
 * counts, perm or inv_perm may be NULL.  Results are deterministic. */
int32_t moqe_bucket(const int32_t* expert_idx, int32_t S, int32_t K,
                    int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv_perm,
                    void* stream);

/* The router's training labels (Section 3.3, first paragraph).  Every sample is run through ALL K experts
 * of the block, the prediction loss of each expert on the sample is computed, and the expert with the
 * lowest loss becomes the sample's label (ties: the lowest index).  The prediction loss of expert j on
 * sample s is the mean over the sample's T rows of the cross-entropy of the row's logits f_j(x_s)[t, :]
 * against targets[s, t]:  log(sum_c exp(logit_c)) - logit_target.  The router of the block is not used.
 *   blk     : LINEAR or SILU_MLP block (n = width of the logits); CONV3X3 is MOQE_E_FORMAT
 *   x       : device bf16 [S, T, d], 16-byte aligned;  targets: device int32 [S, T], values in [0, n)
 *             (a value outside is clamped into the range)
 *   losses  : device float [S, K] out;  labels: device int32 [S] out
 * The K forward passes are one grouped launch over K*S virtual samples in bucket order; logits fp32 in
 * the workspace, loss arithmetic fp32 with a fixed summation order (deterministic).  S*T*K rows must fit
 * int32 and the MLP's intermediate [S*T*K, F] bf16 must stay below 4 GiB.  S == 0 is a no-op. */
size_t moqe_label_pass_workspace_bytes(const moqe_block* blk, int32_t S, int32_t T);
int32_t moqe_label_pass(const moqe_block* blk, const void* x, const int32_t* targets, int32_t S, int32_t T,
                        float* losses, int32_t* labels, void* workspace, size_t workspace_bytes, void* stream);

/* Load-balance statistics of one routed batch (Section 3.2, Eq. 1-2), from the logits that
 * moqe_route wrote and the counts of moqe_bucket:
 *   P_i = mean over the S samples of softmax(logits[s, :])_i,   F_i = counts[i] / S,
 *   L_bal = K * sum_i P_i F_i,   sigma = std(counts) / mean(counts) (population std, mean = S / K),
 *   alpha_dyn = alpha * (1 + sigma), the weight that multiplies L_bal in the training loss.
 * logits: device float [S, K]; counts: device int32 [K]; out: device float [2K + 3] =
 * P[0..K), F[0..K), L_bal, sigma, alpha_dyn.  fp32 arithmetic, fixed summation order
 * (deterministic).  S >= 1, 1 <= K <= MOQE_MAX_EXPERTS.  One small kernel on `stream`. */
int32_t moqe_balance_stats(const float* logits, const int32_t* counts, int32_t S, int32_t K,
                           float alpha, float* out, void* stream);

/* Routing with the NLP router model (Section 3.2; the stages are listed at moqe_nlp_router).
 *   x          : device bf16 [S, T, d], 16-byte aligned (the token vectors the router model sees)
 *   expert_idx : device int32 [S] out (top-1, ties to the lowest index);  logits: device float [S, K] out or NULL
 * Arithmetic: the matrix products of the token stages multiply bf16 operands (x as given; parameters and the
 * activations between stages rounded to bf16, nearest even) on the matrix cores with fp32 accumulation;
 * softmax, LayerNorm, residual sums, the mean over the tokens and the MLP head are fp32.  All sums run in a
 * fixed order (deterministic).  About 16 launches on `stream` (23 for batches of at most 512 rows, whose products
 * are split along k); workspace as the query says, 256-byte aligned.  At most 65535 samples and 8388480 rows per call.
 * S == 0 is a no-op. */
size_t moqe_route_nlp_workspace_bytes(int32_t S, int32_t T, const moqe_nlp_router* r);
int32_t moqe_route_nlp(const void* x, int32_t S, int32_t T, const moqe_nlp_router* r,
                       int32_t* expert_idx, float* logits,
                       void* workspace, size_t workspace_bytes, void* stream);

/* Routing with the CV router model (Section 3.2; the stages are listed at moqe_cv_router).
 *   x          : device bf16 NHWC [S, h, w, c_in] (the tensor the routed stage sees)
 *   expert_idx : device int32 [S] out (top-1, ties to the lowest index);  logits: device float [S, K] out or NULL
 * fp32 arithmetic throughout, every sum in a fixed order (deterministic).  About 20 small launches on `stream`;
 * workspace as the query says, 256-byte aligned.  S == 0 is a no-op. */
size_t moqe_route_cv_workspace_bytes(int32_t S, int32_t h, int32_t w, const moqe_cv_router* r);
int32_t moqe_route_cv(const void* x, int32_t S, int32_t h, int32_t w, const moqe_cv_router* r,
                      int32_t* expert_idx, float* logits,
                      void* workspace, size_t workspace_bytes, void* stream);

/* ---- expert weights ----------------------------------------------------------------- */

/* Round-to-nearest quantization of a device fp32 matrix w [n, k] into the canonical layout
 * (how the workloads derive their experts from one full-precision model, Section 3.1).
 * fp32 IEEE arithmetic, ties to even:
 *   symmetric : s = max|w_row| / qmax (1 if 0), q = clamp(rint(w / s), -qmax, qmax)
 *   asymmetric: lo = clip*min(min,0), hi = clip*max(max,0), s = (hi-lo)/(2^bits-1) (1 if 0),
 *               z = clamp(rint(-lo/s)), q = clamp(rint(w/s) + z)
 * out->qdata/scale/zero must point to device buffers of the canonical sizes; the other
 * fields of `out` give the format. */
int32_t moqe_quantize_rtn(const float* w, float clip, const moqe_qmat* out, void* stream);

/* Size of the packed blob for a format; 0 if the format or shape is not supported. */
size_t  moqe_packed_bytes(int32_t n, int32_t k, int32_t bits, int32_t group,
                          int32_t symmetric, int32_t act_mode);

/* canonical -> packed.  packed_out: device, `bytes` >= moqe_packed_bytes(...), 256-byte aligned. */
int32_t moqe_pack_qmat(const moqe_qmat* canonical, void* packed_out, size_t bytes, void* stream);

/* packed -> the integer weights code - zero as device int16 [n, k] (for exact checks), and
 * optionally the scales in canonical shape (scale_out device float, may be NULL). */
int32_t moqe_unpack_qmat(const moqe_qmat* packed, int16_t* q_minus_z, float* scale_out, void* stream);

/* ---- grouped dequantize-GEMM -------------------------------------------------------- */

/* For every expert e and every row r of its bucket: y_row = a_row * W_e^T, where the
 * bucket of expert e is the samples perm[offsets[e] .. offsets[e+1]) and each sample brings
 * its T rows (each sample is processed by its selected expert only, Section 3.1).
 *   a       device bf16 [S*T, k], rows in the caller's order when perm != NULL (gathered on
 *           load), or already in bucket order when perm == NULL.
 *   offsets device int32 [K+1] in samples;  perm device int32 [S] or NULL.
 *   experts host array of K packed matrices with equal n and k.
 *   y       device float [S*T, n] (bfloat16 with MOQE_OUTPUT_BF16); scatter = 1 writes each row at
 *           its caller-order position (needs perm), scatter = 0 writes bucket order.
 *   scatter is a bit set: MOQE_SCATTER_OUTPUT (1) as above; MOQE_INPUT_IN_BUCKET_ORDER (2) says
 *           that a is already in bucket order although perm is given; MOQE_OUTPUT_BF16 (4) rounds
 *           each result once to bfloat16 (nearest even) and stores y as 16-bit rows, which is the
 *           input type of the next layer.  A stack of layers that is routed and bucketed once (the
 *           router selects the expert for the whole model, Section 3.1) runs its first layer with
 *           perm and scatter 4, the inner layers with perm NULL and scatter 4, and its last layer with
 *           perm and scatter 3: activations stay in bucket order and in bfloat16 in between, and
 *           nothing but this library touches them.
 * The integer codes enter bf16 matrix cores exactly and the fp32 scale is applied to fp32
 * partial sums per group, so no weight is rounded.  act_mode 1 experts quantize their rows
 * to int8 first (workspace). */
#define MOQE_SCATTER_OUTPUT          1
#define MOQE_INPUT_IN_BUCKET_ORDER   2
#define MOQE_OUTPUT_BF16             4
size_t  moqe_grouped_qgemm_workspace_bytes(const moqe_qmat* experts, int32_t K, int32_t S, int32_t T);
int32_t moqe_grouped_qgemm(const void* a, const int32_t* offsets, const int32_t* perm,
                           int32_t S, int32_t T, const moqe_qmat* experts, int32_t K,
                           void* y, int32_t scatter,
                           void* workspace, size_t workspace_bytes, void* stream);

/* ---- the whole block ---------------------------------------------------------------- */

/* y_s = f_{r(x_s)}(x_s) for all samples of the batch: route, bucket, grouped qGEMM(s) with
 * the fused SiLU gate, scatter back.  x: device bf16 [S*T, d]; y: device float [S*T, n_out]
 * in the caller's order.  aux may be NULL. */
size_t  moqe_workspace_bytes(const moqe_block* blk, int32_t S, int32_t T);
int32_t moqe_forward(const moqe_block* blk, const void* x, int32_t S, int32_t T, void* y,
                     const moqe_aux* aux, void* workspace, size_t workspace_bytes, void* stream);

/* moqe_forward for callers that cannot allocate device memory or bring a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid allocation.  Same operation, same
 * kernels and bit-identical results; the scratch memory is a buffer of MOQE_STATIC_SCRATCH_BYTES
 * built into the library (one per GPU the library runs on, held until the process ends; its
 * address is looked up once per device on the first call there).  The call allocates and frees
 * nothing.  Batches whose moqe_workspace_bytes exceeds the buffer are refused with
 * MOQE_E_WORKSPACE before anything is enqueued (16 MiB holds the decode-shaped workloads, e.g. 64
 * rows of the LLaMA-7B-shaped block need about 4 MiB).  All calls on one GPU share the buffer:
 * calls that may overlap in time (different streams, or threads) race on it, so keep them on one
 * stream or order them yourself.  Nothing in it has to be cleared between calls. */
#define MOQE_STATIC_SCRATCH_BYTES (16u << 20)
int32_t moqe_forward_static(const moqe_block* blk, const void* x, int32_t S, int32_t T, void* y,
                            const moqe_aux* aux, void* stream);

/* The block on experts that the caller has chosen: as moqe_forward, but the samples' experts come from
 * expert_idx (device int32 [S], values in [0, n_experts); e.g. the output of moqe_route_nlp or moqe_route_cv,
 * the router models of Section 3.2) and the block's own router is neither checked nor run.  aux->expert_idx and
 * aux->logits are not written; the other aux members as in moqe_forward. */
size_t  moqe_workspace_bytes_routed(const moqe_block* blk, int32_t S, int32_t T);
int32_t moqe_forward_routed(const moqe_block* blk, const int32_t* expert_idx, const void* x, int32_t S, int32_t T,
                            void* y, const moqe_aux* aux, void* workspace, size_t workspace_bytes, void* stream);

/* ---- samples of different lengths ---------------------------------------------------- */

/* The same path for samples that do not all have T rows (sequences of different lengths): x is device
 * bf16 [M, d] with sample s in the rows cu_rows[s] .. cu_rows[s+1) (cu_rows: device int32 [S+1],
 * cu_rows[0] = 0, cu_rows[S] = M, every sample should have at least one row; a sample without rows
 * gets all-zero router features and contributes no rows).  A sample's router feature is
 * the mean over its own rows; routing is per sample as before (Section 3.1).
 *
 * moqe_route_ragged: as moqe_route.
 * moqe_expand_rows: from the sample-level bucket result (offsets, perm of moqe_bucket) to rows:
 *   slot_rows[j]   first bucket-order row of bucket slot j (device int32 [S+1], slot_rows[S] = M)
 *   row_offsets[e] first bucket-order row of expert e      (device int32 [K+1])
 *   row_perm[i]    source row of bucket-order row i         (device int32 [M])
 *   so that moqe_grouped_qgemm(a, row_offsets, row_perm, S = M, T = 1, ...) runs the rows of every
 *   sample through its expert.
 * moqe_forward_ragged: route, bucket, expand, grouped GEMM(s), scatter; LINEAR and SILU_MLP blocks.
 *   M is passed by the host (it sizes the launch); y: device float [M, n_out] in the caller's row
 *   order; aux as in moqe_forward (aux->h, if given, is bf16 [M, F] in bucket-row order). */
size_t  moqe_route_ragged_workspace_bytes(int32_t S, const moqe_router* r);
int32_t moqe_route_ragged(const void* x, const int32_t* cu_rows, int32_t S, const moqe_router* r,
                          int32_t* expert_idx, float* logits,
                          void* workspace, size_t workspace_bytes, void* stream);
int32_t moqe_expand_rows(const int32_t* cu_rows, const int32_t* offsets, const int32_t* perm,
                         int32_t S, int32_t K, int32_t* slot_rows, int32_t* row_offsets,
                         int32_t* row_perm, void* stream);
size_t  moqe_workspace_bytes_ragged(const moqe_block* blk, int32_t S, int32_t M);
int32_t moqe_forward_ragged(const moqe_block* blk, const void* x, const int32_t* cu_rows, int32_t S,
                            int32_t M, void* y, const moqe_aux* aux,
                            void* workspace, size_t workspace_bytes, void* stream);

/* ---- on-demand residency of expert weights ------------------------------------------- */

/* The serving mode of Section 4.4 / the appendix on memory use: only the experts in use sit in
 * device memory, the others wait in host memory and are copied in when the router switches to
 * them.  A cache owns `slots` equal device buffers (each as large as the largest blob, allocated at
 * creation) and keeps the most recently used of K blobs (a blob = one packed matrix, or any
 * concatenation the caller defines).
 *   host_blobs[e], bytes[e]: host memory of blob e; it must stay valid for the cache's lifetime.
 *                            Pinned host memory makes the copies asynchronous.
 * moqe_cache_acquire makes the n <= slots distinct blobs want[0..n) resident and writes their device
 * addresses to dev_ptrs[0..n) (host array).  Missing blobs replace the least recently used ones and
 * are copied on `stream`: work enqueued on that stream afterwards sees the new contents, work
 * enqueued before still sees the old ones, so use the returned addresses on the same stream.
 * *copied (may be NULL) receives the number of copies issued.  Not thread-safe per cache.
 * moqe_cache_stats: totals since creation. */
typedef struct moqe_expert_cache moqe_expert_cache;
int32_t moqe_cache_create(moqe_expert_cache** out, const void* const* host_blobs, const size_t* bytes,
                          int32_t K, int32_t slots);
int32_t moqe_cache_destroy(moqe_expert_cache* cache);
int32_t moqe_cache_acquire(moqe_expert_cache* cache, const int32_t* want, int32_t n, void** dev_ptrs,
                           int32_t* copied, void* stream);
int32_t moqe_cache_stats(const moqe_expert_cache* cache, uint64_t* copies, uint64_t* copied_bytes);

/* ---- timing ------------------------------------------------------------------------- */

/* Per-kernel timing with HIP events recorded on the stream the kernels are launched on.
 * moqe_profile_enable(mask) discards earlier records and starts recording every launch whose
 * kernel kind k has bit (1 << k) set in mask (MOQE_PK_*; at most MOQE_PROFILE_MAX_LAUNCHES
 * launches are kept; mask 0 stops).  moqe_profile_read synchronises the recorded events of one
 * kind and returns the number of launches seen and their summed duration in milliseconds.
 * The two GEMM kinds hand their event pair to the launch itself, so that the pair carries the
 * kernel's own begin and end time stamps (the duration a kernel trace shows); the other kinds record
 * one event before and one after their launches, which includes the dispatch gap between them.
 * Do not enable profiling while a stream is being captured into a graph.
 * The record list is process-wide and unlocked: enable, run and read from one thread at a time. */
#define MOQE_PK_ROUTE      0
#define MOQE_PK_BUCKET     1
#define MOQE_PK_GEMM_GATEUP 2
#define MOQE_PK_GEMM_PLAIN 3
#define MOQE_PK_ACTQUANT   4
#define MOQE_PK_IM2COL     5   /* reserved (no kernel of this kind is launched) */
#define MOQE_PK_OTHER      6
#define MOQE_PK_COUNT      7
#define MOQE_PROFILE_MAX_LAUNCHES 65536
int32_t moqe_profile_enable(int32_t kind_mask);
int32_t moqe_profile_read(int32_t kind, int32_t* launches, double* total_ms);

#ifdef __cplusplus
}
#endif
#endif /* MOQE_H */
