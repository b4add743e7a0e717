"""CPU oracle for the NLP router model of MoQE (test infrastructure).

This module is TEST INFRASTRUCTURE: a plain numpy fp64 implementation used to check the HIP library.
The product never calls it and it shares no code with the HIP path.

What it computes follows MoQE (arXiv 2508.09204), Section 3.2, "NLP Router Model": a Transformer
encoder turns every token vector into a context-aware one, a dedicated self-attention module re-weights
these representations, and an MLP maps the refined features to one logit per expert; the expert of the
largest logit is activated (Section 3.1).  The paper gives the order of the stages and the total size
(16.7 MB in full precision, Appendix "VRAM analysis"), not their dimensions.  Readings fixed here:

* The token vectors (the block's bf16 activations stand in for the embedding output) are first projected
  to the model width d_model by a linear layer, so that the router's size does not follow the base model.
* "Transformer encoder" = ONE standard post-norm encoder layer: multi-head self-attention with an output
  projection, residual, LayerNorm; feed-forward Linear -> ReLU -> Linear, residual, LayerNorm.  No mask
  and no positional term (none is mentioned): the router is a function of the SET of token vectors.
* "Dedicated self-attention module" = a second multi-head self-attention with its own weights, residual
  and LayerNorm.
* The MLP needs one vector per sample: the token vectors are averaged (the same pooling the small routers
  of the hot path use), then Linear -> ReLU -> Linear gives the logits (the `Router` of moqe_oracle).
* LayerNorm: biased variance, eps = 1e-5.  Softmax scale 1/sqrt(head width).  Ties of the arg-max go to
  the lowest index.
* Precision: parameters are fp32 values.  With `round_operands=True` the two operands of every matrix
  product of the token stages (projections, attention in/out projections, feed-forward) are rounded to
  bfloat16 first, which is what the library's matrix-core kernels multiply (products accumulate in fp32
  there, in fp64 here); everything else (softmax, LayerNorm, residuals, pooling, the MLP head) keeps full
  precision.  With `round_operands=False` the function is the plain fp64 definition, which the pins
  compare with torch.nn's encoder layer and attention module.

Pins (tests/test_oracle_router_nlp.py): torch.nn.TransformerEncoderLayer and torch.nn.MultiheadAttention
with the same weights in fp64, scalar loops for one attention row and one LayerNorm row, the closed form
for one token (attention returns the value vector), invariance of the logits under a permutation of the
tokens, and softmax rows that sum to one.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Tuple

import numpy as np

from . import moqe_oracle as oc

LN_EPS = 1e-5


@dataclass
class Attention:
    """Multi-head self-attention: wqkv [3*dm, dm] (rows: queries, keys, values), bqkv [3*dm], wo [dm, dm], bo [dm]."""
    wqkv: np.ndarray
    bqkv: np.ndarray
    wo: np.ndarray
    bo: np.ndarray


@dataclass
class NlpRouter:
    w_in: np.ndarray          # [dm, d]
    b_in: np.ndarray          # [dm]
    att1: Attention
    ln1_g: np.ndarray
    ln1_b: np.ndarray
    w_ff1: np.ndarray         # [d_ff, dm]
    b_ff1: np.ndarray
    w_ff2: np.ndarray         # [dm, d_ff]
    b_ff2: np.ndarray
    ln2_g: np.ndarray
    ln2_b: np.ndarray
    att2: Attention
    ln3_g: np.ndarray
    ln3_b: np.ndarray
    head: oc.Router           # Linear(dm -> h) -> ReLU -> Linear(h -> K) on the pooled vector
    n_heads: int


def _operand(a: np.ndarray, round_operands: bool) -> np.ndarray:
    a = np.asarray(a, dtype=np.float64)
    return oc.bf16_round(a) if round_operands else a


def linear(x: np.ndarray, w: np.ndarray, b: np.ndarray, round_operands: bool) -> np.ndarray:
    """y = x w^T + b for rows x [m, k], w [n, k]."""
    return _operand(x, round_operands) @ _operand(w, round_operands).T + np.asarray(b, dtype=np.float64)


def layer_norm(x: np.ndarray, g: np.ndarray, b: np.ndarray) -> np.ndarray:
    """Per row: (x - mean) / sqrt(var + eps) * g + b, biased variance."""
    x = np.asarray(x, dtype=np.float64)
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + LN_EPS) * np.asarray(g, dtype=np.float64) + np.asarray(b, dtype=np.float64)


def softmax_rows(z: np.ndarray) -> np.ndarray:
    z = z - z.max(axis=-1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=-1, keepdims=True)


def attention(u: np.ndarray, att: Attention, n_heads: int, round_operands: bool) -> np.ndarray:
    """Multi-head self-attention over the tokens of ONE sample, u [T, dm] -> [T, dm].
    Head h uses columns h*dh .. (h+1)*dh of the queries, keys and values; its output row t is
    sum_j softmax_j(q_t . k_j / sqrt(dh)) v_j; the heads are concatenated and projected by wo."""
    T, dm = u.shape
    dh = dm // n_heads
    qkv = linear(u, att.wqkv, att.bqkv, round_operands)
    q, k, v = qkv[:, :dm], qkv[:, dm:2 * dm], qkv[:, 2 * dm:]
    out = np.zeros((T, dm), dtype=np.float64)
    for h in range(n_heads):
        sl = slice(h * dh, (h + 1) * dh)
        p = softmax_rows(q[:, sl] @ k[:, sl].T / np.sqrt(float(dh)))
        out[:, sl] = p @ v[:, sl]
    return linear(out, att.wo, att.bo, round_operands)


def token_features(x: np.ndarray, r: NlpRouter, round_operands: bool = True) -> np.ndarray:
    """The refined token vectors of one sample: x [T, d] -> [T, dm] (projection, encoder layer, attention module)."""
    u = linear(x, r.w_in, r.b_in, round_operands)
    v = layer_norm(u + attention(u, r.att1, r.n_heads, round_operands), r.ln1_g, r.ln1_b)
    hid = np.maximum(linear(v, r.w_ff1, r.b_ff1, round_operands), 0.0)
    w = layer_norm(v + linear(hid, r.w_ff2, r.b_ff2, round_operands), r.ln2_g, r.ln2_b)
    return layer_norm(w + attention(w, r.att2, r.n_heads, round_operands), r.ln3_g, r.ln3_b)


def route_nlp(x: np.ndarray, r: NlpRouter, round_operands: bool = True) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """x fp64 [S, T, d] -> (expert_idx int32 [S], logits fp64 [S, K], pooled fp64 [S, dm])."""
    x = np.asarray(x, dtype=np.float64)
    pooled = np.stack([token_features(x[s], r, round_operands).mean(axis=0) for s in range(x.shape[0])])
    logits = oc.router_logits(pooled, r.head)
    return oc.argmax_first(logits), logits, pooled
