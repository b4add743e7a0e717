"""CPU oracle for the CV router model of MoQE (test infrastructure).

This module is TEST INFRASTRUCTURE: a plain numpy fp64 implementation used to check the HIP library.
The product never calls it and it shares no code with the HIP path.

What it computes follows MoQE (arXiv 2508.09204), Section 3.2, "CV Router Model": a three-layer MLP, each
linear layer followed by batch normalisation and ReLU, transforms the input features; a three-stage
SEResNet-8 with 16, 32 and 64 channels and strides 1, 2, 2 extracts local representations; the resulting
feature map is flattened into a sequence and fed into an 8-head self-attention module that yields the
routing logits; the expert of the largest logit is activated (Section 3.1).  The paper gives this order,
the channel counts, the strides and the head count, and the total size (2.0 MB in full precision).
Readings fixed here, where it is silent:

* The router sees the same NHWC tensor [h, w, c] the routed stage sees.  The MLP acts on every pixel's
  channel vector (a 1x1 transformation): a pooled vector could not feed the convolution stages that follow.
* Batch normalisation is the inference form with stored statistics:
  (x - mean) / sqrt(var + 1e-5) * gain + offset, per channel.
* "SEResNet-8" = a residual network of 8 weight layers: one basic block per stage (two 3x3 convolutions,
  each with batch normalisation, ReLU between them), which with the MLP's last layer as stem and the final
  linear layer gives 8.  The first convolution of a stage carries the stride (padding 1).  Squeeze and
  excitation on the second convolution's output u: g = sigmoid(W2 relu(W1 mean_pixels(u) + b1) + b2) with
  reduction 4, then relu(u * g + shortcut).  The shortcut is the stage's input, or, when stride or width
  change, a strided 1x1 convolution with batch normalisation.
* Convolution filters are stored [out, kh, kw, in] (taps slow, channels fast), as for the routed stage.
* The attention module is multi-head self-attention with an output projection over the h'*w' positions of
  the last feature map (rows: queries, keys, values of Wqkv; scale 1/sqrt(head width)), no mask, no
  positional term; its outputs are averaged over the positions and one linear layer gives the logits.
* Ties of the arg-max go to the lowest index.  All arithmetic is fp64 here (fp32 in the library).

Pins (tests/test_oracle_router_cv.py): torch's conv2d / batch_norm / MultiheadAttention with the same
parameters, a stage against a composition of torch functions, scalar loops for one output pixel, closed forms
(identity batch norm, zero excitation weights give a gate of 1/2), output sizes of the strided stages.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Tuple

import numpy as np

from . import moqe_oracle as oc

BN_EPS = 1e-5


@dataclass
class BatchNorm:
    gain: np.ndarray
    offset: np.ndarray
    mean: np.ndarray
    var: np.ndarray


@dataclass
class Stage:
    conv_a: np.ndarray            # [cout, 3, 3, cin], stride = the stage's
    bn_a: BatchNorm
    conv_b: np.ndarray            # [cout, 3, 3, cout], stride 1
    bn_b: BatchNorm
    se_w1: np.ndarray             # [cout / 4, cout]
    se_b1: np.ndarray
    se_w2: np.ndarray             # [cout, cout / 4]
    se_b2: np.ndarray
    short_w: Optional[np.ndarray]  # [cout, cin] strided 1x1 shortcut, or None for the identity
    short_bn: Optional[BatchNorm]
    stride: int


@dataclass
class CvRouter:
    mlp_w: List[np.ndarray]       # three matrices [out, in]
    mlp_b: List[np.ndarray]
    mlp_bn: List[BatchNorm]
    stages: List[Stage]
    wqkv: np.ndarray              # [3 dm, dm]
    bqkv: np.ndarray
    wo: np.ndarray                # [dm, dm]
    bo: np.ndarray
    w_out: np.ndarray             # [K, dm]
    b_out: np.ndarray
    n_heads: int


def batch_norm(x: np.ndarray, bn: BatchNorm) -> np.ndarray:
    """Inference batch normalisation over the last axis (channels)."""
    f = lambda a: np.asarray(a, dtype=np.float64)
    return (np.asarray(x, dtype=np.float64) - f(bn.mean)) / np.sqrt(f(bn.var) + BN_EPS) * f(bn.gain) + f(bn.offset)


def conv(img: np.ndarray, w: np.ndarray, stride: int) -> np.ndarray:
    """img [h, w, cin], filter [cout, kh, kw, cin] with kh = kw = 3 (padding 1) or 1 (padding 0); output
    [h', w', cout] with h' = floor((h + 2 pad - kh) / stride) + 1."""
    img = np.asarray(img, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    cout, kh, kw, cin = w.shape
    pad = (kh - 1) // 2
    h, wd, _ = img.shape
    ho, wo = (h + 2 * pad - kh) // stride + 1, (wd + 2 * pad - kw) // stride + 1
    padded = np.zeros((h + 2 * pad, wd + 2 * pad, cin))
    padded[pad:pad + h, pad:pad + wd] = img
    out = np.zeros((ho, wo, cout))
    for oy in range(ho):
        for ox in range(wo):
            patch = padded[oy * stride:oy * stride + kh, ox * stride:ox * stride + kw]      # [kh, kw, cin]
            out[oy, ox] = np.tensordot(w, patch, axes=([1, 2, 3], [0, 1, 2]))
    return out


def sigmoid(z: np.ndarray) -> np.ndarray:
    return 1.0 / (1.0 + np.exp(-z))


def stage_forward(x: np.ndarray, st: Stage) -> np.ndarray:
    """One squeeze-and-excitation basic block, x [h, w, cin] -> [h', w', cout]."""
    f = lambda a: np.asarray(a, dtype=np.float64)
    a = np.maximum(batch_norm(conv(x, st.conv_a, st.stride), st.bn_a), 0.0)
    u = batch_norm(conv(a, st.conv_b, 1), st.bn_b)
    z = u.mean(axis=(0, 1))
    g = sigmoid(f(st.se_w2) @ np.maximum(f(st.se_w1) @ z + f(st.se_b1), 0.0) + f(st.se_b2))
    if st.short_w is None:
        short = np.asarray(x, dtype=np.float64)
    else:
        short = batch_norm(conv(x, f(st.short_w)[:, None, None, :], st.stride), st.short_bn)
    return np.maximum(u * g + short, 0.0)


def attention_pool(tokens: np.ndarray, r: CvRouter) -> np.ndarray:
    """Multi-head self-attention over tokens [P, dm], output projection, mean over the positions -> [dm]."""
    f = lambda a: np.asarray(a, dtype=np.float64)
    P, dm = tokens.shape
    dh = dm // r.n_heads
    qkv = tokens @ f(r.wqkv).T + f(r.bqkv)
    q, k, v = qkv[:, :dm], qkv[:, dm:2 * dm], qkv[:, 2 * dm:]
    out = np.zeros((P, dm))
    for h in range(r.n_heads):
        sl = slice(h * dh, (h + 1) * dh)
        s = q[:, sl] @ k[:, sl].T / np.sqrt(float(dh))
        s = np.exp(s - s.max(axis=1, keepdims=True))
        out[:, sl] = (s / s.sum(axis=1, keepdims=True)) @ v[:, sl]
    return (out @ f(r.wo).T + f(r.bo)).mean(axis=0)


def features(img: np.ndarray, r: CvRouter) -> np.ndarray:
    """img fp64 [h, w, c] -> the pooled attention output [dm]."""
    x = np.asarray(img, dtype=np.float64)
    for w, b, bn in zip(r.mlp_w, r.mlp_b, r.mlp_bn):
        x = np.maximum(batch_norm(x @ np.asarray(w, dtype=np.float64).T + np.asarray(b, dtype=np.float64), bn), 0.0)
    for st in r.stages:
        x = stage_forward(x, st)
    return attention_pool(x.reshape(-1, x.shape[-1]), r)


def route_cv(x: np.ndarray, r: CvRouter) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """x fp64 [S, h, w, c] -> (expert_idx int32 [S], logits fp64 [S, K], pooled fp64 [S, dm])."""
    pooled = np.stack([features(x[s], r) for s in range(x.shape[0])])
    logits = pooled @ np.asarray(r.w_out, dtype=np.float64).T + np.asarray(r.b_out, dtype=np.float64)
    return oc.argmax_first(logits), logits, pooled
