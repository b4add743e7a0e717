"""Moves oracle-side objects to the device and wraps them for the HIP library (GPU tests only)."""
from __future__ import annotations

from typing import Dict, List

import numpy as np
import torch

import workloads as wl
from oracle import moqe_oracle as oc
from paper_2508_09204_amd import binding as mq
from paper_2508_09204_amd import experts as ex

DEV = "cuda:0"


def to_dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def bf16_dev(bits: np.ndarray) -> torch.Tensor:
    """uint16 bf16 bit patterns -> device tensor of dtype bfloat16 with the same bits."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(DEV).view(torch.bfloat16)


def canonical_dev(qm: oc.QMat) -> mq.QMat:
    return mq.QMat(to_dev(qm.q), to_dev(qm.scale), None if qm.zero is None else to_dev(qm.zero),
                   qm.n, qm.k, qm.bits, qm.group, qm.symmetric, qm.act_mode, mq.LAYOUT_CANONICAL)


def packed_dev(qm: oc.QMat) -> mq.QMat:
    return ex.pack(canonical_dev(qm))


def router_dev(r: oc.Router, K: int) -> mq.Router:
    d = r.w1.shape[1] if r.w1 is not None else r.w2.shape[1]
    h = r.w1.shape[0] if r.w1 is not None else 0
    return mq.Router(None if r.w1 is None else to_dev(r.w1), None if r.b1 is None else to_dev(r.b1),
                     to_dev(r.w2), None if r.b2 is None else to_dev(r.b2), d, h, K)


def block_dev(blk: oc.Block) -> mq.Block:
    K = blk.n_experts
    return mq.Block(kind=blk.kind, router=router_dev(blk.router, K),
                    w0=[packed_dev(q) for q in blk.w0],
                    w1=None if blk.w1 is None else [packed_dev(q) for q in blk.w1],
                    w2=None if blk.w2 is None else [packed_dev(q) for q in blk.w2],
                    img_h=blk.img_h, img_w=blk.img_w, cin=blk.cin)


def new_aux(S: int, K: int, M: int = 0, F: int = 0) -> mq.Aux:
    i32 = dict(dtype=torch.int32, device=DEV)
    return mq.Aux(expert_idx=torch.full((S,), -1, **i32), logits=torch.zeros((S, K), dtype=torch.float32, device=DEV),
                  counts=torch.full((K,), -1, **i32), offsets=torch.full((K + 1,), -1, **i32),
                  perm=torch.full((S,), -1, **i32), inv_perm=torch.full((S,), -1, **i32),
                  h=torch.zeros((M, F), dtype=torch.bfloat16, device=DEV) if F else None)


def bf16_tensor_to_f64(t: torch.Tensor) -> np.ndarray:
    return oc.bf16_bits_to_f64(t.view(torch.int16).cpu().numpy().view(np.uint16))
