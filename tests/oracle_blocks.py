"""Builds oracle-side objects (quantized experts, router, activations) from a workload config.

Used by the tests and by the smoke check; calls only `oracle/` and `workloads/`.
"""
from __future__ import annotations

from typing import Dict, List

import numpy as np

import workloads as wl
from oracle import moqe_oracle as oc


def quantize_experts(cfg: wl.WorkloadConfig, fpw: Dict[str, np.ndarray]) -> Dict[str, List[oc.QMat]]:
    """name -> per-expert QMat list; every expert is quantized from the same fp32 matrix."""
    out: Dict[str, List[oc.QMat]] = {}
    for name, w in fpw.items():
        out[name] = [oc.quantize(w, e.bits, e.group, e.symmetric, e.clip, e.act_mode) for e in cfg.experts]
    return out


def make_router(cfg: wl.WorkloadConfig) -> oc.Router:
    r = wl.make_router(cfg)
    return oc.Router(w1=r["w1"], b1=r["b1"], w2=r["w2"], b2=r["b2"])


def make_block(cfg: wl.WorkloadConfig, qms: Dict[str, List[oc.QMat]] = None) -> oc.Block:
    if qms is None:
        qms = quantize_experts(cfg, wl.make_fp_weights(cfg))
    router = make_router(cfg)
    if cfg.kind == wl.configs.KIND_SILU_MLP:
        return oc.Block(kind=cfg.kind, router=router, w0=qms["gate"], w1=qms["up"], w2=qms["down"])
    return oc.Block(kind=cfg.kind, router=router, w0=qms["w0"],
                    img_h=cfg.img_h, img_w=cfg.img_w, cin=cfg.D if cfg.kind == wl.configs.KIND_CONV3X3 else 0)


def activations_f64(cfg: wl.WorkloadConfig):
    """(uint16 bf16 bits [S,T,D], the same values as fp64)."""
    bits = wl.make_activations(cfg)
    return bits, oc.bf16_bits_to_f64(bits)


def tolerance_ok(y: np.ndarray, ref: np.ndarray, rel: float = 2e-3):
    """|y - ref| <= rel * max(|ref|, rms(ref)) for every element; returns (ok, worst ratio)."""
    ref = np.asarray(ref, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    bound = rel * np.maximum(np.abs(ref), rms)
    err = np.abs(y - ref)
    if ref.size == 0:
        return True, 0.0
    worst = float(np.max(err / np.maximum(bound, 1e-300)))
    return bool(np.all(err <= bound)), worst
