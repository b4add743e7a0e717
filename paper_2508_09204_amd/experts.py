"""Builds device-resident experts through the library: fp32 weights -> RTN codes -> packed blobs.

Helper on top of the binding (no arithmetic of its own): quantization runs in
moqe_quantize_rtn, the layout change in moqe_pack_qmat.
"""
from __future__ import annotations

from typing import Optional

import torch

from . import binding as mq


def alloc_canonical(n: int, k: int, bits: int, group: int, symmetric: bool, act_mode: int, device) -> mq.QMat:
    q = torch.empty((n, k), dtype=torch.int8 if symmetric else torch.uint8, device=device)
    ng = (k // group) if group else 1
    shape = (n, ng) if group else (n,)
    scale = torch.empty(shape, dtype=torch.float32, device=device)
    zero = None if symmetric else torch.empty(shape, dtype=torch.uint8, device=device)
    return mq.QMat(q, scale, zero, n, k, bits, group, symmetric, act_mode, mq.LAYOUT_CANONICAL)


def pack(canonical: mq.QMat) -> mq.QMat:
    nbytes = mq.moqe_packed_bytes(canonical.n, canonical.k, canonical.bits, canonical.group, canonical.symmetric,
                                  canonical.act_mode)
    if nbytes == 0:
        raise ValueError("unsupported format or shape for the packed layout")
    blob = torch.empty(nbytes, dtype=torch.uint8, device=canonical.qdata.device)
    mq.moqe_pack_qmat(canonical, blob)
    return mq.QMat(blob, None, None, canonical.n, canonical.k, canonical.bits, canonical.group, canonical.symmetric,
                   canonical.act_mode, mq.LAYOUT_PACKED)


def quantize_and_pack(w: torch.Tensor, bits: int, group: int, symmetric: bool, clip: float = 1.0,
                      act_mode: int = 0, keep_canonical: bool = False):
    """w: device fp32 [n, k].  Returns the packed QMat (and the canonical one if asked)."""
    n, k = w.shape
    can = alloc_canonical(n, k, bits, group, symmetric, act_mode, w.device)
    mq.moqe_quantize_rtn(w, clip, can)
    packed = pack(can)
    return (packed, can) if keep_canonical else packed
