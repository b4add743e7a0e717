"""CPU oracle for the routed quantization-expert forward pass (test infrastructure).

This module is TEST INFRASTRUCTURE.  It is a plain, slow, by-the-definition
numpy implementation used to check the HIP library; the product never calls
it, and it shares no code with the HIP path.

What it computes follows MoQE (arXiv 2508.09204):

* Section 3.1 and Figure 1: a data sample first goes through a router model,
  the router picks ONE quantization expert, and that expert alone performs the
  inference on the sample.  Appendix "Convergence Observations" writes this as
  the prediction f_{r(x)}(x) with r: X -> [M].
* Section 3.2: the router is a classifier that ends in an MLP producing one
  logit per expert.  Appendix "number of quantization experts": every input
  activates exactly one expert.
* Section 3.3, Eq. (1)-(2): n_i is the number of samples of the batch
  dispatched to expert i and F_i = n_i / B.  Section 3.3, first paragraph:
  the router's training label of a sample is the expert with the lowest
  prediction loss among all experts run on it (label_pass).

The paper prints no quantizer, no rounding rule and no batching scheme.  The
readings used here (round-to-nearest quantizers, tie rule, stable bucketing,
rounding points) are stated in the docstring of the function that applies them.

All floating-point work is fp64 unless a step is DEFINED in a narrower type
(quantizer arithmetic is fp32 IEEE; activations and the MLP intermediate are
bfloat16 values).

Pins (tests/test_oracle_*.py): hand-worked quantization groups, the s/2
round-trip bound, brute-force Python loops on tiny shapes, numpy/torch library
routines on special cases, one-hot-router == single quantized model,
permutation invariants.  Functions without a pin: none ("parity unpinned"
applies only to dataset-dependent quantities, which are not computed here).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np

KIND_LINEAR = 0
KIND_SILU_MLP = 1
KIND_CONV3X3 = 2


# --------------------------------------------------------------------------------------
# bfloat16 values
# --------------------------------------------------------------------------------------
def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round fp64 (or fp32) values to the nearest bfloat16 value, ties to even; returns fp64.

    bfloat16 has 8 significant bits and the fp32 exponent range.  The rounding is done
    directly from the input precision (no intermediate fp32 rounding).
    """
    x = np.asarray(x, dtype=np.float64)
    _, e = np.frexp(x)                      # x = m * 2**e, 0.5 <= |m| < 1
    e = np.maximum(e, -125)                 # below 2**-126 the spacing stays 2**-133 (subnormals)
    r = np.rint(np.ldexp(x, 8 - e))         # integer of at most 8 bits (+ carry), half-to-even
    return np.ldexp(r, e - 8)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """uint16 bfloat16 bit patterns -> fp64 values (exact)."""
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


# --------------------------------------------------------------------------------------
# Quantization experts: round-to-nearest formats (fp32 IEEE arithmetic, rint = half-to-even)
# --------------------------------------------------------------------------------------
@dataclass
class QMat:
    """One quantized weight matrix in canonical form.

    q      [n, k]  int8 codes in [-qmax, qmax] (symmetric) or uint8 codes in [0, 2^bits-1]
    scale  fp32 [n] (group == 0, one per output channel) or [n, k // group]
    zero   uint8, same shape as scale (asymmetric) or None (symmetric)
    The real weight is  scale * (q - zero).
    """
    q: np.ndarray
    scale: np.ndarray
    zero: Optional[np.ndarray]
    bits: int
    group: int
    symmetric: bool
    act_mode: int = 0   # 0: bf16 activations, 1: per-token dynamic int8 activations
    _deq: Optional[np.ndarray] = None   # memo of dequant(self); drop with release()

    def release(self) -> None:
        self._deq = None

    @property
    def n(self) -> int:
        return self.q.shape[0]

    @property
    def k(self) -> int:
        return self.q.shape[1]


def quantize_sym_per_channel(w: np.ndarray, bits: int, act_mode: int = 0) -> QMat:
    """Symmetric per-output-channel round-to-nearest.

    qmax = 2^(bits-1) - 1;  a_n = max_k |W[n,k]|;  s_n = a_n / qmax (s_n = 1 if a_n == 0);
    q = clamp(rint(W / s_n), -qmax, qmax).  The code -2^(bits-1) never appears.
    """
    w = np.ascontiguousarray(w, dtype=np.float32)
    qmax = np.float32(2 ** (bits - 1) - 1)
    a = np.max(np.abs(w), axis=1)
    s = (a / qmax).astype(np.float32)
    s[a == 0] = np.float32(1.0)
    q = np.rint(w / s[:, None])
    q = np.clip(q, -qmax, qmax).astype(np.int8)
    return QMat(q=q, scale=s, zero=None, bits=bits, group=0, symmetric=True, act_mode=act_mode)


def quantize_asym_group(w: np.ndarray, bits: int, group: int, clip: float = 1.0) -> QMat:
    """Asymmetric group-wise round-to-nearest along the input dimension.

    Per (row n, group of `group` consecutive k):
      lo = clip * min(min W, 0);  hi = clip * max(max W, 0);  L = 2^bits - 1
      s  = (hi - lo) / L   (s = 1 if hi == lo)
      z  = clamp(rint(-lo / s), 0, L)
      q  = clamp(rint(W / s) + z, 0, L)
    so that the real weight is s * (q - z) and the code z decodes to exactly 0.
    """
    w = np.ascontiguousarray(w, dtype=np.float32)
    n, k = w.shape
    if k % group:
        raise ValueError("k must be a multiple of the group size")
    wg = w.reshape(n, k // group, group)
    L = np.float32(2 ** bits - 1)
    c = np.float32(clip)
    lo = c * np.minimum(wg.min(axis=2), np.float32(0))
    hi = c * np.maximum(wg.max(axis=2), np.float32(0))
    s = ((hi - lo) / L).astype(np.float32)
    s[hi == lo] = np.float32(1.0)
    z = np.clip(np.rint(-lo / s), 0, L).astype(np.float32)
    q = np.rint(wg / s[:, :, None]) + z[:, :, None]
    q = np.clip(q, 0, L)
    return QMat(q=q.reshape(n, k).astype(np.uint8), scale=s, zero=z.astype(np.uint8),
                bits=bits, group=group, symmetric=False)


def quantize(w: np.ndarray, bits: int, group: int, symmetric: bool, clip: float = 1.0,
             act_mode: int = 0) -> QMat:
    if symmetric:
        if group != 0:
            raise ValueError("symmetric formats here are per output channel")
        return quantize_sym_per_channel(w, bits, act_mode)
    qm = quantize_asym_group(w, bits, group, clip)
    qm.act_mode = act_mode
    return qm


def dequant_int(qm: QMat) -> np.ndarray:
    """The integer weight q - zero, int16 [n, k]."""
    q = qm.q.astype(np.int16)
    if qm.zero is None:
        return q
    g = qm.group if qm.group else qm.k
    return q - np.repeat(qm.zero.astype(np.int16).reshape(qm.n, -1), g, axis=1)


def dequant(qm: QMat) -> np.ndarray:
    """The real weight scale * (q - zero), fp64 [n, k]; the fp32 scale is promoted, nothing is rounded."""
    g = qm.group if qm.group else qm.k
    s = np.repeat(qm.scale.astype(np.float64).reshape(qm.n, -1), g, axis=1)
    return s * dequant_int(qm).astype(np.float64)


def _dequant_memo(qm: QMat) -> np.ndarray:
    """dequant(qm), kept on the matrix so a per-sample loop does not redo it for every sample."""
    if qm._deq is None:
        qm._deq = dequant(qm)
    return qm._deq


# --------------------------------------------------------------------------------------
# Router (Section 3.2), top-1 selection, dispatch counts (Eq. 2), stable bucketing
# --------------------------------------------------------------------------------------
@dataclass
class Router:
    """pool -> [Linear(d->h) -> ReLU ->] Linear(->K).  w1/b1 are None when there is no hidden layer."""
    w1: Optional[np.ndarray]
    b1: Optional[np.ndarray]
    w2: np.ndarray
    b2: Optional[np.ndarray]


def pool(x: np.ndarray) -> np.ndarray:
    """Per-sample feature: arithmetic mean over the sample's T rows.  x fp64 [S, T, D] -> [S, D]."""
    x = np.asarray(x, dtype=np.float64)
    return x.sum(axis=1) / x.shape[1]


def router_logits(p: np.ndarray, r: Router) -> np.ndarray:
    """Logits [S, K] of the router's final MLP for pooled features p [S, D] (fp64)."""
    h = np.asarray(p, dtype=np.float64)
    if r.w1 is not None:
        h = h @ r.w1.astype(np.float64).T
        if r.b1 is not None:
            h = h + r.b1.astype(np.float64)
        h = np.maximum(h, 0.0)
    z = h @ r.w2.astype(np.float64).T
    if r.b2 is not None:
        z = z + r.b2.astype(np.float64)
    return z


def argmax_first(logits: np.ndarray) -> np.ndarray:
    """Top-1 expert per sample; among equal maxima the lowest index wins."""
    logits = np.asarray(logits)
    S, K = logits.shape
    out = np.zeros(S, dtype=np.int32)
    for s in range(S):
        best = 0
        for k in range(1, K):
            if logits[s, k] > logits[s, best]:
                best = k
        out[s] = best
    return out


def route(x: np.ndarray, r: Router) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """x fp64 [S, T, D] -> (expert index int32 [S], logits fp64 [S, K], margin top1 - top2 [S])."""
    logits = router_logits(pool(x), r)
    idx = argmax_first(logits)
    if logits.shape[1] > 1:
        srt = np.sort(logits, axis=1)
        margin = srt[:, -1] - srt[:, -2]
    else:
        margin = np.full(logits.shape[0], np.inf)
    return idx, logits, margin


def route_ragged(xs: Sequence[np.ndarray], r: Router) -> Tuple[np.ndarray, np.ndarray]:
    """Samples of different lengths: xs[s] fp64 [T_s, D], T_s >= 1.  Each sample's feature is the mean
    over its own rows; everything else as in route().  Returns (expert index int32 [S], logits [S, K])."""
    p = np.stack([np.asarray(x, dtype=np.float64).sum(axis=0) / x.shape[0] for x in xs])
    logits = router_logits(p, r)
    return argmax_first(logits), logits


def bucket(expert_idx: Sequence[int], K: int):
    """Dispatch counts and the stable permutation that groups samples by expert.

    counts[k]  = #{s : e[s] = k}                     (the n_i of Eq. 2)
    offsets    = exclusive prefix sum of counts, offsets[K] = S
    pos[s]     = offsets[e[s]] + #{s' < s : e[s'] = e[s]}
    perm[pos[s]] = s,  inv_perm[s] = pos[s]
    """
    e = np.asarray(expert_idx, dtype=np.int64)
    S = e.shape[0]
    counts = np.zeros(K, dtype=np.int32)
    for s in range(S):
        counts[e[s]] += 1
    offsets = np.zeros(K + 1, dtype=np.int32)
    for k in range(K):
        offsets[k + 1] = offsets[k] + counts[k]
    seen = np.zeros(K, dtype=np.int64)
    perm = np.zeros(S, dtype=np.int32)
    inv_perm = np.zeros(S, dtype=np.int32)
    for s in range(S):
        pos = offsets[e[s]] + seen[e[s]]
        seen[e[s]] += 1
        perm[pos] = s
        inv_perm[s] = pos
    return counts, offsets, perm, inv_perm


def balance_loss(logits: np.ndarray, expert_idx: np.ndarray) -> float:
    """L_bal = N * sum_i P_i F_i of Eq. (1)-(2): P_i mean softmax probability, F_i = n_i / B."""
    z = np.asarray(logits, dtype=np.float64)
    z = z - z.max(axis=1, keepdims=True)
    p = np.exp(z)
    p /= p.sum(axis=1, keepdims=True)
    B, N = z.shape
    P = p.mean(axis=0)
    F = np.bincount(np.asarray(expert_idx), minlength=N).astype(np.float64) / B
    return float(N * np.sum(P * F))


def balance_stats(logits: np.ndarray, expert_idx: np.ndarray, alpha: float):
    """The load-balance quantities of Section 3.2 for one batch, from the router's logits and its dispatch.

    P_i = mean over the batch of softmax(logits)_i, F_i = n_i / B with n_i the samples dispatched to
    expert i (Eq. 2), L_bal = N * sum_i P_i F_i (Eq. 1), sigma = relative standard deviation of the
    expert usage n_i (population standard deviation over its mean B / N), and the dynamic weight
    alpha * (1 + sigma) that scales L_bal in the training loss.  Returns (P, F, L_bal, sigma, alpha_dyn).
    """
    z = np.asarray(logits, dtype=np.float64)
    B, N = z.shape
    e = np.exp(z - z.max(axis=1, keepdims=True))
    p = e / e.sum(axis=1, keepdims=True)
    P = p.mean(axis=0)
    n = np.bincount(np.asarray(expert_idx), minlength=N).astype(np.float64)
    F = n / B
    l_bal = float(N * np.sum(P * F))
    mean = B / N
    sigma = float(np.sqrt(np.mean((n - mean) ** 2)) / mean)
    return P, F, l_bal, sigma, float(alpha * (1.0 + sigma))


# --------------------------------------------------------------------------------------
# Expert layers
# --------------------------------------------------------------------------------------
def act_quant_int8(x: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Per-row dynamic int8 quantization of bfloat16-valued rows x [m, k] (fp32 IEEE arithmetic).

    a = max_k |x|;  sx = a / 127 (sx = 1 if a == 0);  xq = clamp(rint(x / sx), -127, 127).
    """
    x32 = np.asarray(x, dtype=np.float32)
    a = np.max(np.abs(x32), axis=1)
    sx = (a / np.float32(127)).astype(np.float32)
    sx[a == 0] = np.float32(1.0)
    xq = np.clip(np.rint(x32 / sx[:, None]), -127, 127).astype(np.int8)
    return xq, sx


def qlinear(x: np.ndarray, qm: QMat) -> np.ndarray:
    """y = x W~^T for rows x [m, k] holding bfloat16 values; fp64 [m, n].

    act_mode 0: W~ = scale * (q - zero) unrounded, fp64 accumulation.
    act_mode 1 (W8A8): rows are quantized per token, the integer dot product is exact,
    and y[m, n] = (sum_k xq q) * sx_m * s_n.
    """
    x = np.asarray(x, dtype=np.float64)
    if qm.act_mode == 0:
        return x @ _dequant_memo(qm).T
    if not (qm.symmetric and qm.group == 0 and qm.bits == 8):
        raise ValueError("int8 activations are defined for the int8 per-channel expert only")
    xq, sx = act_quant_int8(x)
    acc = xq.astype(np.float64) @ qm.q.astype(np.float64).T      # integers < 2^53: exact
    return acc * sx.astype(np.float64)[:, None] * qm.scale.astype(np.float64)[None, :]


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def silu_mlp(x: np.ndarray, gate: QMat, up: QMat, down: QMat) -> Tuple[np.ndarray, np.ndarray]:
    """SiLU-gated MLP on rows x [m, D]: H = bf16(silu(x Wg^T) * (x Wu^T)),  Y = H Wd^T.

    Returns (Y fp64 [m, D], H fp64 [m, F] holding bfloat16 values).  H is rounded once to
    bfloat16 because the second GEMM consumes a bfloat16 tensor.
    """
    g = qlinear(x, gate)
    u = qlinear(x, up)
    h = bf16_round(silu(g) * u)
    return qlinear(h, down), h


def conv3x3(img: np.ndarray, qm: QMat, cin: int) -> np.ndarray:
    """3x3 convolution, stride 1, zero padding 1, no bias.  img fp64 [H, W, Cin] -> [H, W, Cout].

    The weight matrix row n is the filter of output channel n flattened channels-last, like the
    activations: k = (kh * 3 + kw) * Cin + cin (O, kh, kw, I order); quantization groups run along
    this k, so a group of 64 covers 64 neighbouring input channels of one filter tap.
    """
    img = np.asarray(img, dtype=np.float64)
    Hh, Ww, C = img.shape
    assert C == cin and qm.k == cin * 9
    w = _dequant_memo(qm).reshape(qm.n, 3, 3, cin)
    xp = np.zeros((Hh + 2, Ww + 2, C), dtype=np.float64)
    xp[1:-1, 1:-1, :] = img
    y = np.zeros((Hh, Ww, qm.n), dtype=np.float64)
    for kh in range(3):
        for kw in range(3):
            y += xp[kh:kh + Hh, kw:kw + Ww, :] @ w[:, kh, kw, :].T
    return y


@dataclass
class Block:
    """One routed block: a router and, per expert, its quantized matrices."""
    kind: int
    router: Router
    w0: List[QMat]                       # LINEAR / CONV: the matrix.  SILU_MLP: gate
    w1: Optional[List[QMat]] = None      # SILU_MLP: up
    w2: Optional[List[QMat]] = None      # SILU_MLP: down
    img_h: int = 0
    img_w: int = 0
    cin: int = 0

    @property
    def n_experts(self) -> int:
        return len(self.w0)


def expert_forward(blk: Block, e: int, xs: np.ndarray) -> np.ndarray:
    """f_e(x_s): the output of expert e alone on one sample's rows xs [T, D] (fp64, bf16 values)."""
    if blk.kind == KIND_LINEAR:
        return qlinear(xs, blk.w0[e])
    if blk.kind == KIND_SILU_MLP:
        return silu_mlp(xs, blk.w0[e], blk.w1[e], blk.w2[e])[0]
    if blk.kind == KIND_CONV3X3:
        img = xs.reshape(blk.img_h, blk.img_w, blk.cin)
        return conv3x3(img, blk.w0[e], blk.cin).reshape(blk.img_h * blk.img_w, -1)
    raise ValueError("unknown block kind")


def cross_entropy_rows(y: np.ndarray, targets: Sequence[int]) -> np.ndarray:
    """Prediction loss of rows of logits y [m, n] against class indices targets [m]:
    CE_r = log(sum_c exp(y[r, c])) - y[r, targets[r]]  (the negative log of the softmax probability of the target)."""
    y = np.asarray(y, dtype=np.float64)
    t = np.asarray(targets, dtype=np.int64)
    mx = y.max(axis=1)
    lse = mx + np.log(np.exp(y - mx[:, None]).sum(axis=1))
    return lse - y[np.arange(y.shape[0]), t]


def label_pass(blk: Block, x: np.ndarray, targets: np.ndarray):
    """The router's training labels (Section 3.3, first paragraph): every sample goes through ALL experts,
    each expert's prediction loss on the sample is computed, and the expert with the lowest loss is the
    sample's label (ties: the lowest index).  The prediction loss of a sample is the mean cross-entropy of
    its rows' logits f_j(x_s) [T, n] against the rows' target classes (the loss of both of the paper's task
    families: next-token prediction and classification).  x fp64 [S, T, D] holding bfloat16 values, targets
    int [S, T].  Returns (losses fp64 [S, K], labels int32 [S]).  LINEAR and SILU_MLP blocks."""
    if blk.kind == KIND_CONV3X3:
        raise ValueError("the label pass is defined for blocks whose rows are logits")
    x = np.asarray(x, dtype=np.float64)
    S, K = x.shape[0], blk.n_experts
    losses = np.zeros((S, K), dtype=np.float64)
    for s in range(S):
        for j in range(K):
            y = expert_forward(blk, j, x[s])
            losses[s, j] = cross_entropy_rows(y, targets[s]).sum() / y.shape[0]
    labels = np.zeros(S, dtype=np.int32)
    for s in range(S):
        best = 0
        for j in range(1, K):
            if losses[s, j] < losses[s, best]:
                best = j
        labels[s] = best
    return losses, labels


def forward_ragged(blk: Block, xs: Sequence[np.ndarray]):
    """y_s = f_{r(x_s)}(x_s) for samples of different lengths (LINEAR and SILU_MLP blocks): xs[s] fp64
    [T_s, D] holding bfloat16 values.  Returns (list of Y_s fp64 [T_s, N], expert index, logits)."""
    if blk.kind == KIND_CONV3X3:
        raise ValueError("images have a fixed number of pixels")
    idx, logits = route_ragged(xs, blk.router)
    return [expert_forward(blk, int(idx[s]), np.asarray(xs[s], dtype=np.float64)) for s in range(len(xs))], idx, logits


def forward(blk: Block, x: np.ndarray, expert_idx: Optional[np.ndarray] = None,
            rows: Optional[Sequence[int]] = None):
    """The MoQE prediction y_s = f_{r(x_s)}(x_s) for every sample, one sample at a time.

    x fp64 [S, T, D] holding bfloat16 values.  Returns (Y fp64 [S, T', N], expert_idx, logits).
    No bucketing takes part in computing Y.  `rows` (token indices within a sample) restricts
    the computed rows of LINEAR / SILU_MLP blocks, whose rows are independent of each other;
    T' = len(rows).  `expert_idx` overrides the router's decision (used to study one stage).
    """
    x = np.asarray(x, dtype=np.float64)
    S = x.shape[0]
    idx, logits, _ = route(x, blk.router)
    if expert_idx is not None:
        idx = np.asarray(expert_idx, dtype=np.int32)
    ys = []
    for s in range(S):
        xs = x[s]
        if rows is not None:
            if blk.kind == KIND_CONV3X3:
                raise ValueError("conv rows depend on their neighbours; compute whole images")
            xs = xs[np.asarray(rows)]
        ys.append(expert_forward(blk, int(idx[s]), xs))
    return np.stack(ys), idx, logits
