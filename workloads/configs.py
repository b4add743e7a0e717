"""Workload configurations: shapes, expert formats and seeds (data only).

Each configuration describes one routed block: a router, K quantization
experts that are all derived from ONE full-precision weight set (MoQE
Section 3.1: the experts are quantized variants of the same model), and a
batch of S samples of T rows each.  Real LLaMA / Qwen / ResNet weights and
the paper's datasets are not used; tensors are N(0, sigma) draws of the
same shapes.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, Tuple

SEED_BASE = 250809200

KIND_LINEAR = 0      # y = x W^T
KIND_SILU_MLP = 1    # y = (silu(x Wg^T) * (x Wu^T)) Wd^T
KIND_CONV3X3 = 2     # 3x3 conv, stride 1, zero pad 1, NHWC activations


@dataclass(frozen=True)
class ExpertSpec:
    """How one expert is quantized from the shared full-precision weights."""
    bits: int              # 8, 6, 4, 3
    group: int             # 0 = one scale per output channel, else 64 / 128 along the input dim
    symmetric: bool        # True: signed codes, no zero-point
    clip: float = 1.0      # range clip ratio (asymmetric group formats)
    act_mode: int = 0      # 0: bf16 activations; 1: per-token dynamic int8 activations (W8A8)

    def label(self) -> str:
        s = f"int{self.bits}" + (f"g{self.group}" if self.group else "pc")
        s += "sym" if self.symmetric else "asym"
        if self.clip != 1.0:
            s += f"c{self.clip:g}"
        if self.act_mode:
            s += "a8"
        return s


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    index: int                  # position in the list of benchmark configurations
    kind: int
    S: int                      # samples (sequences / images)
    T: int                      # rows per sample (tokens; pixels for conv)
    D: int                      # model / input-channel dim
    F: int                      # MLP intermediate dim, or output dim for LINEAR / CONV
    experts: Tuple[ExpertSpec, ...]
    router_hidden: int          # 0 = single Linear(D -> K)
    router_w_std: float
    w_std: float = 0.02
    router_bias: Tuple[float, ...] = ()   # b2; empty = zeros
    img_h: int = 0
    img_w: int = 0
    seed: int = 0
    unit: str = "tokens"

    @property
    def K(self) -> int:
        return len(self.experts)

    @property
    def M(self) -> int:
        return self.S * self.T

    @property
    def conv_k(self) -> int:
        return self.D * 9

    def matrices(self) -> Dict[str, Tuple[int, int]]:
        """name -> (out_features, in_features) of every weight matrix of the block."""
        if self.kind == KIND_LINEAR:
            return {"w0": (self.F, self.D)}
        if self.kind == KIND_SILU_MLP:
            return {"gate": (self.F, self.D), "up": (self.F, self.D), "down": (self.D, self.F)}
        return {"w0": (self.F, self.D * 9)}


def _asym(bits, group, clip=1.0):
    return ExpertSpec(bits=bits, group=group, symmetric=False, clip=clip)


def _sym(bits, act_mode=0):
    return ExpertSpec(bits=bits, group=0, symmetric=True, act_mode=act_mode)


# b2[0] of the skewed router.  Written by oracle/calibrate_skew_bias.py (bisection on the
# oracle's routing so that 60 % +- 2 % of the 128 sequences go to expert 0); a constant since.
QWEN_SKEW_BIAS0 = 0.023694349452853203


def _build() -> Dict[str, WorkloadConfig]:
    llama_experts = (_asym(4, 128), _asym(4, 128, 0.9), _asym(3, 128), _sym(8))
    cfgs = [
        WorkloadConfig(
            name="toy_linear", index=0, kind=KIND_LINEAR, S=32, T=16, D=256, F=256,
            experts=(_sym(8), _asym(4, 64), _asym(3, 64)),
            router_hidden=0, router_w_std=0.1),
        WorkloadConfig(
            name="llama7b_mlp_decode", index=1, kind=KIND_SILU_MLP, S=64, T=1, D=4096, F=11008,
            experts=llama_experts, router_hidden=256, router_w_std=0.02),
        WorkloadConfig(
            name="llama7b_mlp_prefill", index=2, kind=KIND_SILU_MLP, S=16, T=512, D=4096, F=11008,
            experts=llama_experts, router_hidden=256, router_w_std=0.02),
        WorkloadConfig(
            name="qwen_mlp_skew", index=3, kind=KIND_SILU_MLP, S=128, T=256, D=3584, F=18944,
            experts=(_asym(4, 128, 1.0), _asym(4, 128, 0.95), _asym(4, 128, 0.9), _asym(4, 128, 0.85),
                     _asym(3, 128, 1.0), _asym(3, 128, 0.9), _sym(8, act_mode=1), _sym(8)),
            router_hidden=256, router_w_std=0.02,
            router_bias=(QWEN_SKEW_BIAS0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0)),
        WorkloadConfig(
            name="resnet50_conv", index=4, kind=KIND_CONV3X3, S=256, T=196, D=256, F=256,
            experts=(_sym(8), _sym(6), _sym(4), _asym(4, 64)),
            router_hidden=64, router_w_std=0.02, img_h=14, img_w=14, unit="images"),
    ]
    out = {}
    for c in cfgs:
        out[c.name] = replace(c, seed=SEED_BASE + c.index + 1)
    return out


CONFIGS: Dict[str, WorkloadConfig] = _build()


def get_config(name: str) -> WorkloadConfig:
    return CONFIGS[name]


def scaled(cfg: WorkloadConfig, **overrides) -> WorkloadConfig:
    """A copy of `cfg` with some sizes replaced (reduced shapes for quick parity cases)."""
    return replace(cfg, **overrides)
