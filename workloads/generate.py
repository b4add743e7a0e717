"""Seeded tensor generators.

Every tensor comes from `numpy.random.default_rng(cfg.seed)` split into
independent child streams in a fixed order, so a given configuration always
yields the same bits no matter which consumer asks or in which order:

    child 0..m-1 : full-precision weight matrices, in `cfg.matrices()` order
    child m      : router first layer
    child m+1    : router second layer
    child m+2    : activations
    child m+3    : target classes of the label pass

Activations are stored at the library boundary as bfloat16.  The only
arithmetic here is the storage conversion fp32 -> bf16 bits (round to
nearest even) and back, which defines the input values themselves.
"""
from __future__ import annotations

from typing import Dict, Optional, Sequence

import numpy as np

from .configs import WorkloadConfig

_N_STREAMS = 8


def _streams(cfg: WorkloadConfig):
    return np.random.default_rng(cfg.seed).spawn(_N_STREAMS)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 array -> uint16 bfloat16 bit patterns, round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """uint16 bfloat16 bit patterns -> the fp32 values they denote (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def make_fp_weights(cfg: WorkloadConfig) -> Dict[str, np.ndarray]:
    """The shared full-precision weights, fp32 [out, in] ~ N(0, w_std)."""
    ss = _streams(cfg)
    out = {}
    for i, (name, (n, k)) in enumerate(cfg.matrices().items()):
        w = ss[i].standard_normal((n, k), dtype=np.float32)
        w *= np.float32(cfg.w_std)
        out[name] = w
    return out


def make_router(cfg: WorkloadConfig) -> Dict[str, Optional[np.ndarray]]:
    """Router weights, fp32.  hidden == 0: only w2 [K, D].  Biases are zero except cfg.router_bias."""
    ss = _streams(cfg)
    m = len(cfg.matrices())
    K, D, Hd = cfg.K, cfg.D, cfg.router_hidden
    r: Dict[str, Optional[np.ndarray]] = {"w1": None, "b1": None}
    if Hd:
        r["w1"] = (ss[m].standard_normal((Hd, D), dtype=np.float32) * np.float32(cfg.router_w_std))
        r["b1"] = np.zeros(Hd, dtype=np.float32)
        w2 = ss[m + 1].standard_normal((K, Hd), dtype=np.float32) * np.float32(cfg.router_w_std)
        # The hidden units are non-negative after the ReLU, so a row's sum would act as a large
        # per-expert constant and one expert would take most samples.  Rows are drawn zero-sum to
        # keep the routing of a random router roughly uniform, as the workloads call for.
        w2 -= w2.mean(axis=1, keepdims=True, dtype=np.float32)
        r["w2"] = w2
    else:
        r["w2"] = (ss[m + 1].standard_normal((K, D), dtype=np.float32) * np.float32(cfg.router_w_std))
    b2 = np.zeros(K, dtype=np.float32)
    if cfg.router_bias:
        b2[:] = np.asarray(cfg.router_bias, dtype=np.float32)
    r["b2"] = b2
    return r


def make_activations(cfg: WorkloadConfig, S: Optional[int] = None) -> np.ndarray:
    """Activations ~ N(0,1) as bfloat16 bit patterns, uint16 [S, T, D] (conv: [S, H, W, C] flattened to T=H*W)."""
    ss = _streams(cfg)
    m = len(cfg.matrices())
    S = cfg.S if S is None else S
    x = ss[m + 2].standard_normal((S, cfg.T, cfg.D), dtype=np.float32)
    return f32_to_bf16_bits(x)


def make_targets(cfg: WorkloadConfig, n_classes: int) -> np.ndarray:
    """Target class per row for the label pass, int32 [S, T], uniform in [0, n_classes) (child stream m+3)."""
    ss = _streams(cfg)
    m = len(cfg.matrices())
    return ss[m + 3].integers(0, n_classes, size=(cfg.S, cfg.T), dtype=np.int64).astype(np.int32)


def make_nlp_router(d: int, dm: int, n_heads: int, d_ff: int, head_hidden: int, K: int, seed: int) -> Dict[str, np.ndarray]:
    """Random fp32 parameters of the NLP router model (projection, encoder layer, attention module, MLP head).
    Matrices are [out, in] with N(0, 1/in) entries, biases N(0, 0.02), LayerNorm gains 1 + N(0, 0.05);
    the rows of the last layer are zero-sum (see make_router)."""
    ss = [np.random.default_rng(s) for s in np.random.SeedSequence(seed).spawn(32)]
    it = iter(ss)

    def mat(n, k):
        return (next(it).standard_normal((n, k), dtype=np.float32) * np.float32(1.0 / np.sqrt(k)))

    def vec(n, std=0.02, mean=0.0):
        return (next(it).standard_normal(n, dtype=np.float32) * np.float32(std) + np.float32(mean))

    p = {"w_in": mat(dm, d), "b_in": vec(dm)}
    for tag in ("1", "2"):
        p["wqkv" + tag] = mat(3 * dm, dm)
        p["bqkv" + tag] = vec(3 * dm)
        p["wo" + tag] = mat(dm, dm)
        p["bo" + tag] = vec(dm)
    p["w_ff1"], p["b_ff1"] = mat(d_ff, dm), vec(d_ff)
    p["w_ff2"], p["b_ff2"] = mat(dm, d_ff), vec(dm)
    for tag in ("1", "2", "3"):
        p["ln%s_g" % tag] = vec(dm, 0.05, 1.0)
        p["ln%s_b" % tag] = vec(dm)
    p["head_w1"], p["head_b1"] = mat(head_hidden, dm), vec(head_hidden)
    w2 = mat(K, head_hidden)
    w2 -= w2.mean(axis=1, keepdims=True, dtype=np.float32)
    p["head_w2"], p["head_b2"] = w2, vec(K)
    return p


def make_token_activations(S: int, T: int, D: int, seed: int, topic_std: float = 1.0) -> np.ndarray:
    """bf16 token vectors [S, T, D] as uint16 bit patterns: every sequence has its own N(0, topic_std) offset
    vector (sequences differ in content) plus N(0, 1) noise per token."""
    a, b = [np.random.default_rng(s) for s in np.random.SeedSequence(seed).spawn(2)]
    x = a.standard_normal((S, 1, D), dtype=np.float32) * np.float32(topic_std) + b.standard_normal((S, T, D), dtype=np.float32)
    return f32_to_bf16_bits(x)


def make_cv_router(c_in: int, mlp: Sequence[int], stages: Sequence[int], strides: Sequence[int], K: int, seed: int) -> Dict[str, np.ndarray]:
    """Random fp32 parameters of the CV router model.  Matrices [out, in] and filters [out, 3, 3, in] with N(0, 1/fan-in)
    entries, biases N(0, 0.05); batch-norm gains 1 + N(0, 0.1), offsets N(0, 0.1), means N(0, 0.1), variances in
    [0.5, 1.5]; zero-sum last layer (see make_router).  A stage has a 1x1 shortcut when its stride or width changes."""
    rng = iter(np.random.default_rng(s) for s in np.random.SeedSequence(seed).spawn(128))

    def mat(*shape):
        fan = int(np.prod(shape[1:]))
        return next(rng).standard_normal(shape, dtype=np.float32) * np.float32(1.0 / np.sqrt(fan))

    def vec(n, std=0.05, mean=0.0):
        return next(rng).standard_normal(n, dtype=np.float32) * np.float32(std) + np.float32(mean)

    def bn(prefix, n, p):
        p[prefix + "_g"], p[prefix + "_o"], p[prefix + "_m"] = vec(n, 0.1, 1.0), vec(n, 0.1), vec(n, 0.1)
        p[prefix + "_v"] = (next(rng).random(n, dtype=np.float32) + np.float32(0.5))

    p: Dict[str, np.ndarray] = {}
    prev = c_in
    for i, n in enumerate(mlp):
        p["mlp%d_w" % i], p["mlp%d_b" % i] = mat(n, prev), vec(n)
        bn("mlp%d_bn" % i, n, p)
        prev = n
    for i, (n, st) in enumerate(zip(stages, strides)):
        p["st%d_a" % i] = mat(n, 3, 3, prev)
        bn("st%d_abn" % i, n, p)
        p["st%d_b" % i] = mat(n, 3, 3, n)
        bn("st%d_bbn" % i, n, p)
        p["st%d_se1" % i], p["st%d_se1b" % i] = mat(n // 4, n), vec(n // 4)
        p["st%d_se2" % i], p["st%d_se2b" % i] = mat(n, n // 4), vec(n)
        if st != 1 or n != prev:
            p["st%d_s" % i] = mat(n, prev)
            bn("st%d_sbn" % i, n, p)
        prev = n
    p["wqkv"], p["bqkv"] = mat(3 * prev, prev), vec(3 * prev)
    p["wo"], p["bo"] = mat(prev, prev), vec(prev)
    w = mat(K, prev)
    w -= w.mean(axis=1, keepdims=True, dtype=np.float32)
    p["w_out"], p["b_out"] = w, vec(K)
    return p


def make_image_activations(S: int, h: int, w: int, c: int, seed: int) -> np.ndarray:
    """bf16 NHWC images [S, h, w, c] as uint16 bit patterns: a per-image N(0, 1) channel offset, a smooth per-image spatial
    pattern and N(0, 1) noise per pixel, so that images differ in content and positions differ within an image."""
    a, b, d = [np.random.default_rng(s) for s in np.random.SeedSequence(seed).spawn(3)]
    x = a.standard_normal((S, 1, 1, c), dtype=np.float32) + b.standard_normal((S, h, w, c), dtype=np.float32)
    yy, xx = np.meshgrid(np.linspace(-1, 1, h, dtype=np.float32), np.linspace(-1, 1, w, dtype=np.float32), indexing="ij")
    slope = d.standard_normal((S, 2, c), dtype=np.float32)
    x += slope[:, 0][:, None, None, :] * yy[None, :, :, None] + slope[:, 1][:, None, None, :] * xx[None, :, :, None]
    return f32_to_bf16_bits(x)
