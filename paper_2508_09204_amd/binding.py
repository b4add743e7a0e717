"""ctypes binding of libmoqe.so: the functions of include/moqe.h under the same names.

Argument marshalling only: every step of the routed forward pass runs inside the HIP
library.  PyTorch appears here for device memory (tensors own the buffers) and for the
current stream handle.  If the shared library is missing, importing this module fails.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoqe.so")

MOQE_MAX_EXPERTS = 16
LAYOUT_CANONICAL, LAYOUT_PACKED = 0, 1
KIND_LINEAR, KIND_SILU_MLP, KIND_CONV3X3 = 0, 1, 2
PK_ROUTE, PK_BUCKET, PK_GEMM_GATEUP, PK_GEMM_PLAIN, PK_ACTQUANT, PK_IM2COL, PK_OTHER = range(7)


class MoqeError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"moqe error {code}: {msg}")
        self.code = code


class _QMat(C.Structure):
    _fields_ = [("qdata", C.c_void_p), ("scale", C.c_void_p), ("zero", C.c_void_p),
                ("n", C.c_int32), ("k", C.c_int32), ("bits", C.c_int32), ("group", C.c_int32),
                ("symmetric", C.c_int32), ("act_mode", C.c_int32), ("layout", C.c_int32)]


class _Router(C.Structure):
    _fields_ = [("w1", C.c_void_p), ("b1", C.c_void_p), ("w2", C.c_void_p), ("b2", C.c_void_p),
                ("d", C.c_int32), ("h", C.c_int32), ("n_experts", C.c_int32)]


_NLP_PTRS = ("w_in", "b_in", "wqkv1", "bqkv1", "wo1", "bo1", "ln1_g", "ln1_b", "w_ff1", "b_ff1", "w_ff2", "b_ff2",
             "ln2_g", "ln2_b", "wqkv2", "bqkv2", "wo2", "bo2", "ln3_g", "ln3_b")


class _NlpRouter(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _NLP_PTRS] + [("head", _Router), ("d", C.c_int32), ("dm", C.c_int32),
                                                         ("n_heads", C.c_int32), ("d_ff", C.c_int32)]


class _Bn(C.Structure):
    _fields_ = [("gain", C.c_void_p), ("offset", C.c_void_p), ("mean", C.c_void_p), ("var", C.c_void_p)]


class _CvStage(C.Structure):
    _fields_ = [("conv_a", C.c_void_p), ("bn_a", _Bn), ("conv_b", C.c_void_p), ("bn_b", _Bn),
                ("se_w1", C.c_void_p), ("se_b1", C.c_void_p), ("se_w2", C.c_void_p), ("se_b2", C.c_void_p),
                ("short_w", C.c_void_p), ("short_bn", _Bn), ("cout", C.c_int32), ("stride", C.c_int32)]


class _CvRouter(C.Structure):
    _fields_ = [("mlp_w", C.c_void_p * 3), ("mlp_b", C.c_void_p * 3), ("mlp_bn", _Bn * 3), ("mlp_n", C.c_int32 * 3),
                ("stage", _CvStage * 3), ("wqkv", C.c_void_p), ("bqkv", C.c_void_p), ("wo", C.c_void_p), ("bo", C.c_void_p),
                ("w_out", C.c_void_p), ("b_out", C.c_void_p), ("c_in", C.c_int32), ("n_heads", C.c_int32),
                ("n_experts", C.c_int32)]


class _Block(C.Structure):
    _fields_ = [("kind", C.c_int32), ("router", _Router),
                ("w0", C.POINTER(_QMat)), ("w1", C.POINTER(_QMat)), ("w2", C.POINTER(_QMat)),
                ("n_experts", C.c_int32), ("img_h", C.c_int32), ("img_w", C.c_int32), ("cin", C.c_int32),
                ("y_bf16", C.c_int32)]


class _Aux(C.Structure):
    _fields_ = [("expert_idx", C.c_void_p), ("logits", C.c_void_p), ("counts", C.c_void_p),
                ("offsets", C.c_void_p), ("perm", C.c_void_p), ("inv_perm", C.c_void_p), ("h", C.c_void_p)]


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2508_09204_amd.build` "
                          "(there is no fallback path)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    sig = {
        "moqe_version": (C.c_char_p, []),
        "moqe_last_error_string": (C.c_char_p, []),
        "moqe_set_dry_run": (None, [i32]),
        "moqe_route_workspace_bytes": (sz, [i32, i32, C.POINTER(_Router)]),
        "moqe_route": (i32, [vp, i32, i32, C.POINTER(_Router), vp, vp, vp, sz, vp]),
        "moqe_bucket": (i32, [vp, i32, i32, vp, vp, vp, vp, vp]),
        "moqe_balance_stats": (i32, [vp, vp, i32, i32, C.c_float, vp, vp]),
        "moqe_route_nlp_workspace_bytes": (sz, [i32, i32, C.POINTER(_NlpRouter)]),
        "moqe_route_nlp": (i32, [vp, i32, i32, C.POINTER(_NlpRouter), vp, vp, vp, sz, vp]),
        "moqe_route_cv_workspace_bytes": (sz, [i32, i32, i32, C.POINTER(_CvRouter)]),
        "moqe_route_cv": (i32, [vp, i32, i32, i32, C.POINTER(_CvRouter), vp, vp, vp, sz, vp]),
        "moqe_route_ragged_workspace_bytes": (sz, [i32, C.POINTER(_Router)]),
        "moqe_route_ragged": (i32, [vp, vp, i32, C.POINTER(_Router), vp, vp, vp, sz, vp]),
        "moqe_expand_rows": (i32, [vp, vp, vp, i32, i32, vp, vp, vp, vp]),
        "moqe_workspace_bytes_ragged": (sz, [C.POINTER(_Block), i32, i32]),
        "moqe_forward_ragged": (i32, [C.POINTER(_Block), vp, vp, i32, i32, vp, C.POINTER(_Aux), vp, sz, vp]),
        "moqe_quantize_rtn": (i32, [vp, C.c_float, C.POINTER(_QMat), vp]),
        "moqe_packed_bytes": (sz, [i32, i32, i32, i32, i32, i32]),
        "moqe_pack_qmat": (i32, [C.POINTER(_QMat), vp, sz, vp]),
        "moqe_unpack_qmat": (i32, [C.POINTER(_QMat), vp, vp, vp]),
        "moqe_grouped_qgemm_workspace_bytes": (sz, [C.POINTER(_QMat), i32, i32, i32]),
        "moqe_grouped_qgemm": (i32, [vp, vp, vp, i32, i32, C.POINTER(_QMat), i32, vp, i32, vp, sz, vp]),
        "moqe_workspace_bytes": (sz, [C.POINTER(_Block), i32, i32]),
        "moqe_forward": (i32, [C.POINTER(_Block), vp, i32, i32, vp, C.POINTER(_Aux), vp, sz, vp]),
        "moqe_workspace_bytes_routed": (sz, [C.POINTER(_Block), i32, i32]),
        "moqe_forward_routed": (i32, [C.POINTER(_Block), vp, vp, i32, i32, vp, C.POINTER(_Aux), vp, sz, vp]),
        "moqe_forward_static": (i32, [C.POINTER(_Block), vp, i32, i32, vp, C.POINTER(_Aux), vp]),
        "moqe_label_pass_workspace_bytes": (sz, [C.POINTER(_Block), i32, i32]),
        "moqe_label_pass": (i32, [C.POINTER(_Block), vp, vp, i32, i32, vp, vp, vp, sz, vp]),
        "moqe_cache_create": (i32, [C.POINTER(vp), C.POINTER(vp), C.POINTER(sz), i32, i32]),
        "moqe_cache_destroy": (i32, [vp]),
        "moqe_cache_acquire": (i32, [vp, C.POINTER(i32), i32, C.POINTER(vp), C.POINTER(i32), vp]),
        "moqe_cache_stats": (i32, [vp, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64)]),
        "moqe_profile_enable": (i32, [i32]),
        "moqe_profile_read": (i32, [i32, C.POINTER(i32), C.POINTER(C.c_double)]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    return lib


lib = _load()
SCATTER_OUTPUT = 1
INPUT_IN_BUCKET_ORDER = 2
OUTPUT_BF16 = 4

EXPORTED = ["moqe_version", "moqe_last_error_string", "moqe_set_dry_run", "moqe_route_workspace_bytes",
            "moqe_route", "moqe_route_nlp_workspace_bytes", "moqe_route_nlp", "moqe_route_cv_workspace_bytes", "moqe_route_cv", "moqe_bucket", "moqe_balance_stats", "moqe_route_ragged_workspace_bytes", "moqe_route_ragged",
            "moqe_expand_rows", "moqe_workspace_bytes_ragged", "moqe_forward_ragged", "moqe_quantize_rtn", "moqe_packed_bytes", "moqe_pack_qmat",
            "moqe_unpack_qmat", "moqe_grouped_qgemm_workspace_bytes", "moqe_grouped_qgemm",
            "moqe_workspace_bytes", "moqe_forward", "moqe_forward_static", "moqe_workspace_bytes_routed", "moqe_forward_routed", "moqe_label_pass_workspace_bytes", "moqe_label_pass", "moqe_cache_create", "moqe_cache_destroy", "moqe_cache_acquire",
            "moqe_cache_stats", "moqe_profile_enable", "moqe_profile_read"]


def _check(rc: int) -> None:
    if rc != 0:
        raise MoqeError(rc, lib.moqe_last_error_string().decode())


def _ptr(t) -> Optional[int]:
    """Address of a tensor's storage; a plain int (an address handed out by the library) passes through."""
    if t is None:
        return None
    return t if isinstance(t, int) else t.data_ptr()


def _stream() -> Optional[int]:
    return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None


# --------------------------------------------------------------------------------------
# Descriptors that keep their tensors alive
# --------------------------------------------------------------------------------------
@dataclass
class QMat:
    """A quantized matrix on the device.  Canonical: qdata int8/uint8 [n,k], scale, zero.
    Packed: qdata is the uint8 blob from moqe_pack_qmat, or its device address as an int (as handed
    out by moqe_cache_acquire)."""
    qdata: object
    scale: Optional[torch.Tensor]
    zero: Optional[torch.Tensor]
    n: int
    k: int
    bits: int
    group: int
    symmetric: bool
    act_mode: int = 0
    layout: int = LAYOUT_CANONICAL

    def c(self) -> _QMat:
        return _QMat(_ptr(self.qdata), _ptr(self.scale), _ptr(self.zero), self.n, self.k, self.bits, self.group,
                     int(self.symmetric), self.act_mode, self.layout)


@dataclass
class Router:
    w1: Optional[torch.Tensor]
    b1: Optional[torch.Tensor]
    w2: torch.Tensor
    b2: Optional[torch.Tensor]
    d: int
    h: int
    n_experts: int

    def c(self) -> _Router:
        return _Router(_ptr(self.w1), _ptr(self.b1), _ptr(self.w2), _ptr(self.b2), self.d, self.h, self.n_experts)


@dataclass
class NlpRouter:
    """The NLP router model: `params` maps the names of moqe_nlp_router's pointers to fp32 device tensors."""
    params: dict
    head: Router
    d: int
    dm: int
    n_heads: int
    d_ff: int

    def c(self) -> _NlpRouter:
        r = _NlpRouter()
        for n in _NLP_PTRS:
            setattr(r, n, _ptr(self.params[n]))
        r.head = self.head.c()
        r.d, r.dm, r.n_heads, r.d_ff = self.d, self.dm, self.n_heads, self.d_ff
        return r


@dataclass
class CvRouter:
    """The CV router model.  `params` holds fp32 device tensors under the names of workloads.make_cv_router:
    mlp{i}_w / _b / _bn_{g,o,m,v}, st{i}_a / _abn_* / _b / _bbn_* / _se1 / _se1b / _se2 / _se2b [/ _s / _sbn_*],
    wqkv, bqkv, wo, bo, w_out, b_out."""
    params: dict
    c_in: int
    strides: Sequence[int]
    n_heads: int
    n_experts: int

    def c(self) -> _CvRouter:
        p = self.params
        bn = lambda pre: _Bn(_ptr(p[pre + "_g"]), _ptr(p[pre + "_o"]), _ptr(p[pre + "_m"]), _ptr(p[pre + "_v"]))
        r = _CvRouter()
        for i in range(3):
            r.mlp_w[i], r.mlp_b[i], r.mlp_bn[i] = _ptr(p["mlp%d_w" % i]), _ptr(p["mlp%d_b" % i]), bn("mlp%d_bn" % i)
            r.mlp_n[i] = p["mlp%d_w" % i].shape[0]
            st = r.stage[i]
            st.conv_a, st.bn_a = _ptr(p["st%d_a" % i]), bn("st%d_abn" % i)
            st.conv_b, st.bn_b = _ptr(p["st%d_b" % i]), bn("st%d_bbn" % i)
            st.se_w1, st.se_b1 = _ptr(p["st%d_se1" % i]), _ptr(p["st%d_se1b" % i])
            st.se_w2, st.se_b2 = _ptr(p["st%d_se2" % i]), _ptr(p["st%d_se2b" % i])
            if ("st%d_s" % i) in p:
                st.short_w, st.short_bn = _ptr(p["st%d_s" % i]), bn("st%d_sbn" % i)
            st.cout, st.stride = p["st%d_a" % i].shape[0], self.strides[i]
        r.wqkv, r.bqkv, r.wo, r.bo = _ptr(p["wqkv"]), _ptr(p["bqkv"]), _ptr(p["wo"]), _ptr(p["bo"])
        r.w_out, r.b_out = _ptr(p["w_out"]), _ptr(p["b_out"])
        r.c_in, r.n_heads, r.n_experts = self.c_in, self.n_heads, self.n_experts
        return r


@dataclass
class Block:
    kind: int
    router: Router
    w0: List[QMat]
    w1: Optional[List[QMat]] = None
    w2: Optional[List[QMat]] = None
    img_h: int = 0
    img_w: int = 0
    cin: int = 0
    y_bf16: int = 0
    _keep: list = field(default_factory=list, repr=False)

    def c(self) -> _Block:
        def arr(ms):
            if ms is None:
                return None
            a = (_QMat * len(ms))(*[m.c() for m in ms])
            self._keep.append(a)
            return a
        self._keep.clear()
        return _Block(self.kind, self.router.c(), arr(self.w0), arr(self.w1), arr(self.w2), len(self.w0),
                      self.img_h, self.img_w, self.cin, self.y_bf16)


@dataclass
class Aux:
    expert_idx: Optional[torch.Tensor] = None
    logits: Optional[torch.Tensor] = None
    counts: Optional[torch.Tensor] = None
    offsets: Optional[torch.Tensor] = None
    perm: Optional[torch.Tensor] = None
    inv_perm: Optional[torch.Tensor] = None
    h: Optional[torch.Tensor] = None

    def c(self) -> _Aux:
        return _Aux(_ptr(self.expert_idx), _ptr(self.logits), _ptr(self.counts), _ptr(self.offsets),
                    _ptr(self.perm), _ptr(self.inv_perm), _ptr(self.h))


def _workspace(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


# --------------------------------------------------------------------------------------
# The entry points (same names as the C ABI)
# --------------------------------------------------------------------------------------
def moqe_version() -> str:
    return lib.moqe_version().decode()


def moqe_set_dry_run(on: bool) -> None:
    lib.moqe_set_dry_run(int(on))


def moqe_route_workspace_bytes(S: int, T: int, router: Router) -> int:
    r = router.c()
    return lib.moqe_route_workspace_bytes(S, T, C.byref(r))


def moqe_route(x: torch.Tensor, S: int, T: int, router: Router, expert_idx: torch.Tensor,
               logits: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> None:
    r = router.c()
    if workspace is None:
        workspace = _workspace(lib.moqe_route_workspace_bytes(S, T, C.byref(r)), x.device)
    _check(lib.moqe_route(_ptr(x), S, T, C.byref(r), _ptr(expert_idx), _ptr(logits), _ptr(workspace),
                          workspace.numel(), _stream()))


def moqe_bucket(expert_idx: torch.Tensor, S: int, K: int, counts: Optional[torch.Tensor], offsets: torch.Tensor,
                perm: Optional[torch.Tensor], inv_perm: Optional[torch.Tensor]) -> None:
    _check(lib.moqe_bucket(_ptr(expert_idx), S, K, _ptr(counts), _ptr(offsets), _ptr(perm), _ptr(inv_perm), _stream()))


def moqe_route_nlp_workspace_bytes(S: int, T: int, r: NlpRouter) -> int:
    rc = r.c()
    return lib.moqe_route_nlp_workspace_bytes(S, T, C.byref(rc))


def moqe_route_nlp(x: torch.Tensor, S: int, T: int, r: NlpRouter, expert_idx: torch.Tensor,
                   logits: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> None:
    rc = r.c()
    if workspace is None:
        workspace = _workspace(lib.moqe_route_nlp_workspace_bytes(S, T, C.byref(rc)), x.device)
    _check(lib.moqe_route_nlp(_ptr(x), S, T, C.byref(rc), _ptr(expert_idx), _ptr(logits), _ptr(workspace),
                              workspace.numel(), _stream()))


def moqe_route_cv_workspace_bytes(S: int, h: int, w: int, r: CvRouter) -> int:
    rc = r.c()
    return lib.moqe_route_cv_workspace_bytes(S, h, w, C.byref(rc))


def moqe_route_cv(x: torch.Tensor, S: int, h: int, w: int, r: CvRouter, expert_idx: torch.Tensor,
                  logits: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> None:
    rc = r.c()
    if workspace is None:
        workspace = _workspace(lib.moqe_route_cv_workspace_bytes(S, h, w, C.byref(rc)), x.device)
    _check(lib.moqe_route_cv(_ptr(x), S, h, w, C.byref(rc), _ptr(expert_idx), _ptr(logits), _ptr(workspace),
                             workspace.numel(), _stream()))


def moqe_balance_stats(logits: torch.Tensor, counts: torch.Tensor, S: int, K: int, alpha: float,
                       out: torch.Tensor) -> None:
    _check(lib.moqe_balance_stats(_ptr(logits), _ptr(counts), S, K, float(alpha), _ptr(out), _stream()))


def moqe_quantize_rtn(w: torch.Tensor, clip: float, out: QMat) -> None:
    o = out.c()
    _check(lib.moqe_quantize_rtn(_ptr(w), float(clip), C.byref(o), _stream()))


def moqe_packed_bytes(n: int, k: int, bits: int, group: int, symmetric: bool, act_mode: int = 0) -> int:
    return lib.moqe_packed_bytes(n, k, bits, group, int(symmetric), act_mode)


def moqe_pack_qmat(canonical: QMat, packed_out: torch.Tensor) -> None:
    c = canonical.c()
    _check(lib.moqe_pack_qmat(C.byref(c), _ptr(packed_out), packed_out.numel(), _stream()))


def moqe_unpack_qmat(packed: QMat, q_minus_z: torch.Tensor, scale_out: Optional[torch.Tensor] = None) -> None:
    p = packed.c()
    _check(lib.moqe_unpack_qmat(C.byref(p), _ptr(q_minus_z), _ptr(scale_out), _stream()))


def moqe_grouped_qgemm_workspace_bytes(experts: Sequence[QMat], S: int, T: int) -> int:
    arr = (_QMat * len(experts))(*[m.c() for m in experts])
    return lib.moqe_grouped_qgemm_workspace_bytes(arr, len(experts), S, T)


def moqe_grouped_qgemm(a: torch.Tensor, offsets: torch.Tensor, perm: Optional[torch.Tensor], S: int, T: int,
                       experts: Sequence[QMat], y: torch.Tensor, scatter: int,
                       workspace: Optional[torch.Tensor] = None) -> None:
    arr = (_QMat * len(experts))(*[m.c() for m in experts])
    if workspace is None:
        workspace = _workspace(lib.moqe_grouped_qgemm_workspace_bytes(arr, len(experts), S, T), a.device)
    _check(lib.moqe_grouped_qgemm(_ptr(a), _ptr(offsets), _ptr(perm), S, T, arr, len(experts), _ptr(y),
                                  int(scatter), _ptr(workspace), workspace.numel(), _stream()))


def moqe_cache_create(host_blobs: Sequence[torch.Tensor], slots: int) -> int:
    """host_blobs: CPU uint8 tensors (pinned for asynchronous copies); the caller keeps them alive.
    Returns the cache handle."""
    K = len(host_blobs)
    ptrs = (C.c_void_p * K)(*[t.data_ptr() for t in host_blobs])
    sizes = (C.c_size_t * K)(*[t.numel() * t.element_size() for t in host_blobs])
    handle = C.c_void_p()
    _check(lib.moqe_cache_create(C.byref(handle), ptrs, sizes, K, slots))
    return handle.value


def moqe_cache_destroy(handle: int) -> None:
    _check(lib.moqe_cache_destroy(handle))


def moqe_cache_acquire(handle: int, want: Sequence[int]):
    """Returns (device addresses of the wanted blobs, number of host->device copies issued)."""
    n = len(want)
    w = (C.c_int32 * n)(*want)
    out = (C.c_void_p * n)()
    copied = C.c_int32(0)
    _check(lib.moqe_cache_acquire(handle, w, n, out, C.byref(copied), _stream()))
    return [int(out[i]) for i in range(n)], copied.value


def moqe_cache_stats(handle: int):
    a, b = C.c_uint64(0), C.c_uint64(0)
    _check(lib.moqe_cache_stats(handle, C.byref(a), C.byref(b)))
    return a.value, b.value


def moqe_workspace_bytes(blk: Block, S: int, T: int) -> int:
    b = blk.c()
    return lib.moqe_workspace_bytes(C.byref(b), S, T)


def moqe_forward(blk: Block, x: torch.Tensor, S: int, T: int, y: torch.Tensor, aux: Optional[Aux] = None,
                 workspace: Optional[torch.Tensor] = None) -> None:
    b = blk.c()
    if workspace is None:
        workspace = _workspace(lib.moqe_workspace_bytes(C.byref(b), S, T), x.device)
    a = aux.c() if aux is not None else None
    _check(lib.moqe_forward(C.byref(b), _ptr(x), S, T, _ptr(y), C.byref(a) if a is not None else None,
                            _ptr(workspace), workspace.numel(), _stream()))


def moqe_label_pass_workspace_bytes(blk: Block, S: int, T: int) -> int:
    b = blk.c()
    return lib.moqe_label_pass_workspace_bytes(C.byref(b), S, T)


def moqe_label_pass(blk: Block, x: torch.Tensor, targets: torch.Tensor, S: int, T: int, losses: torch.Tensor,
                    labels: torch.Tensor, workspace: Optional[torch.Tensor] = None) -> None:
    b = blk.c()
    if workspace is None:
        workspace = _workspace(lib.moqe_label_pass_workspace_bytes(C.byref(b), S, T), x.device)
    _check(lib.moqe_label_pass(C.byref(b), _ptr(x), _ptr(targets), S, T, _ptr(losses), _ptr(labels),
                               _ptr(workspace), workspace.numel(), _stream()))


def moqe_forward_routed(blk: Block, expert_idx: torch.Tensor, x: torch.Tensor, S: int, T: int, y: torch.Tensor,
                        aux: Optional[Aux] = None, workspace: Optional[torch.Tensor] = None) -> None:
    """The block on experts chosen by the caller (e.g. by moqe_route_nlp or moqe_route_cv)."""
    b = blk.c()
    if workspace is None:
        workspace = _workspace(lib.moqe_workspace_bytes_routed(C.byref(b), S, T), x.device)
    a = aux.c() if aux is not None else None
    _check(lib.moqe_forward_routed(C.byref(b), _ptr(expert_idx), _ptr(x), S, T, _ptr(y),
                                   C.byref(a) if a is not None else None, _ptr(workspace), workspace.numel(), _stream()))


STATIC_SCRATCH_BYTES = 16 << 20


def moqe_forward_static(blk: Block, x: torch.Tensor, S: int, T: int, y: torch.Tensor, aux: Optional[Aux] = None) -> None:
    """moqe_forward on the library's built-in scratch buffer: no workspace, nothing allocated."""
    b = blk.c()
    a = aux.c() if aux is not None else None
    _check(lib.moqe_forward_static(C.byref(b), _ptr(x), S, T, _ptr(y), C.byref(a) if a is not None else None, _stream()))


def moqe_route_ragged_workspace_bytes(S: int, router: Router) -> int:
    r = router.c()
    return lib.moqe_route_ragged_workspace_bytes(S, C.byref(r))


def moqe_route_ragged(x: torch.Tensor, cu_rows: torch.Tensor, S: int, router: Router, expert_idx: torch.Tensor,
                      logits: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> None:
    r = router.c()
    if workspace is None:
        workspace = _workspace(lib.moqe_route_ragged_workspace_bytes(S, C.byref(r)), x.device)
    _check(lib.moqe_route_ragged(_ptr(x), _ptr(cu_rows), S, C.byref(r), _ptr(expert_idx), _ptr(logits), _ptr(workspace),
                                 workspace.numel(), _stream()))


def moqe_expand_rows(cu_rows: torch.Tensor, offsets: torch.Tensor, perm: Optional[torch.Tensor], S: int, K: int,
                     slot_rows: torch.Tensor, row_offsets: torch.Tensor, row_perm: Optional[torch.Tensor]) -> None:
    _check(lib.moqe_expand_rows(_ptr(cu_rows), _ptr(offsets), _ptr(perm), S, K, _ptr(slot_rows), _ptr(row_offsets),
                                _ptr(row_perm), _stream()))


def moqe_workspace_bytes_ragged(blk: Block, S: int, M: int) -> int:
    b = blk.c()
    return lib.moqe_workspace_bytes_ragged(C.byref(b), S, M)


def moqe_forward_ragged(blk: Block, x: torch.Tensor, cu_rows: torch.Tensor, S: int, M: int, y: torch.Tensor,
                        aux: Optional[Aux] = None, workspace: Optional[torch.Tensor] = None) -> None:
    b = blk.c()
    if workspace is None:
        workspace = _workspace(lib.moqe_workspace_bytes_ragged(C.byref(b), S, M), x.device)
    a = aux.c() if aux is not None else None
    _check(lib.moqe_forward_ragged(C.byref(b), _ptr(x), _ptr(cu_rows), S, M, _ptr(y), C.byref(a) if a is not None else None,
                                   _ptr(workspace), workspace.numel(), _stream()))


def moqe_profile_enable(kind_mask: int) -> None:
    _check(lib.moqe_profile_enable(int(kind_mask)))


def moqe_profile_read(kind: int):
    n = C.c_int32(0)
    ms = C.c_double(0.0)
    _check(lib.moqe_profile_read(kind, C.byref(n), C.byref(ms)))
    return n.value, ms.value


class ForwardCall:
    """moqe_forward with its arguments marshalled once; calling it only enqueues the work."""

    def __init__(self, blk: Block, x: torch.Tensor, S: int, T: int, y: torch.Tensor, aux: Optional[Aux] = None,
                 workspace: Optional[torch.Tensor] = None):
        self._blk_c = blk.c()
        self._keep = (blk, x, y, aux)
        if workspace is None:
            workspace = _workspace(lib.moqe_workspace_bytes(C.byref(self._blk_c), S, T), x.device)
        self.workspace = workspace
        self._aux_c = aux.c() if aux is not None else None
        self._args = (C.byref(self._blk_c), _ptr(x), S, T, _ptr(y),
                      C.byref(self._aux_c) if self._aux_c is not None else None,
                      _ptr(workspace), workspace.numel())

    def __call__(self, stream: Optional[int] = None) -> None:
        rc = lib.moqe_forward(*self._args, _stream() if stream is None else stream)
        if rc != 0:
            _check(rc)
