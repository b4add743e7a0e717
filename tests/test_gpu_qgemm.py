"""GPU parity: grouped dequantize-GEMM against the oracle, per format and for ragged buckets.

Tolerance: |y - ref| <= 2e-3 * max(|ref|, rms(ref)) element-wise (bf16 inputs, fp32 accumulation).
"""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import moqe_oracle as oc
from tests import oracle_blocks as ob

pytestmark = pytest.mark.gpu

FORMATS = [(8, 0, True, 1.0, 0), (8, 0, True, 1.0, 1), (6, 0, True, 1.0, 0), (4, 0, True, 1.0, 0),
           (4, 64, False, 1.0, 0), (4, 128, False, 0.9, 0), (3, 64, False, 1.0, 0), (3, 128, False, 1.0, 0)]


def _run(a_bits, e_idx, qms, S, T, scatter=True, use_perm=True):
    """Grouped GEMM on the GPU for routing e_idx; returns y (caller order) as numpy."""
    from paper_2508_09204_amd import binding as mq
    from tests import gpu_blocks as gb
    K = len(qms)
    counts, offsets, perm, inv = oc.bucket(e_idx, K)
    n, k = qms[0].n, qms[0].k
    a_host = a_bits.reshape(S, T, k)
    if not use_perm:
        a_host = a_host[perm]                         # hand the rows over already in bucket order
    a = gb.bf16_dev(a_host.reshape(S * T, k))
    y = torch.full((S * T, n), float("nan"), dtype=torch.float32, device=gb.DEV)
    packed = [gb.packed_dev(q) for q in qms]
    mq.moqe_grouped_qgemm(a, gb.to_dev(offsets), gb.to_dev(perm) if use_perm else None, S, T, packed, y,
                          scatter and use_perm)
    torch.cuda.synchronize()
    out = y.cpu().numpy().reshape(S, T, n)
    if not (scatter and use_perm):
        out = out[inv]                                # bucket order -> caller order
    return out


def _ref(a_bits, e_idx, qms, S, T):
    x = oc.bf16_bits_to_f64(a_bits).reshape(S, T, -1)
    return np.stack([oc.qlinear(x[s], qms[int(e_idx[s])]) for s in range(S)])


@pytest.mark.parametrize("bits,group,sym,clip,act", FORMATS)
@pytest.mark.parametrize("S,T,n,k", [(5, 3, 48, 384), (37, 1, 32, 1024), (3, 50, 16, 128)])
def test_single_format_single_expert(bits, group, sym, clip, act, S, T, n, k):
    rng = np.random.default_rng(bits * 13 + group + S)
    w = (rng.standard_normal((n, k)) * 0.02).astype(np.float32)
    qm = oc.quantize(w, bits, group, sym, clip, act)
    a_bits = wl.f32_to_bf16_bits(rng.standard_normal((S * T, k)).astype(np.float32))
    e = np.zeros(S, dtype=np.int32)
    y = _run(a_bits, e, [qm], S, T)
    ok, worst = ob.tolerance_ok(y, _ref(a_bits, e, [qm], S, T))
    assert ok, worst
    assert worst < 0.05          # far inside the 2e-3 budget: nothing is rounded but the accumulation


@pytest.mark.parametrize("scatter,use_perm", [(True, True), (False, True), (False, False)])
def test_mixed_experts_ragged_buckets(scatter, use_perm):
    rng = np.random.default_rng(21)
    S, T, n, k = 45, 3, 80, 640
    w = (rng.standard_normal((n, k)) * 0.02).astype(np.float32)
    specs = [(4, 128, False, 1.0, 0), (3, 128, False, 1.0, 0), (8, 0, True, 1.0, 0), (8, 0, True, 1.0, 1),
             (4, 64, False, 0.9, 0), (6, 0, True, 1.0, 0)]
    qms = [oc.quantize(w, *s) for s in specs]
    a_bits = wl.f32_to_bf16_bits(rng.standard_normal((S * T, k)).astype(np.float32))
    e = rng.integers(0, len(qms), S).astype(np.int32)
    e[e == 4] = 0                                     # expert 4 stays empty
    y = _run(a_bits, e, qms, S, T, scatter, use_perm)
    ok, worst = ob.tolerance_ok(y, _ref(a_bits, e, qms, S, T))
    assert ok, worst


@pytest.mark.parametrize("bits,group,sym,clip,act", FORMATS)
@pytest.mark.parametrize("S,T,n,k", [(5, 40, 208, 640), (3, 67, 272, 384)])
def test_large_bucket_kernel_per_format(bits, group, sym, clip, act, S, T, n, k):
    """Buckets of a few hundred rows take the LDS-tiled kernel: weight rows that do not fill the
    256-row work-group tile or a wave's 64, an odd number of 128-column steps, a ragged last row tile."""
    rng = np.random.default_rng(bits * 17 + group + n)
    w = (rng.standard_normal((n, k)) * 0.02).astype(np.float32)
    qm = oc.quantize(w, bits, group, sym, clip, act)
    a_bits = wl.f32_to_bf16_bits(rng.standard_normal((S * T, k)).astype(np.float32))
    e = np.zeros(S, dtype=np.int32)
    y = _run(a_bits, e, [qm], S, T)
    ok, worst = ob.tolerance_ok(y, _ref(a_bits, e, [qm], S, T))
    assert ok, worst
    assert worst < 0.05


@pytest.mark.parametrize("scatter,use_perm", [(True, True), (False, False)])
def test_large_bucket_kernel_mixed_experts(scatter, use_perm):
    """Six formats in one launch of the tiled kernel, ragged buckets (one of a single sample, one empty)."""
    rng = np.random.default_rng(22)
    S, T, n, k = 14, 37, 144, 512
    w = (rng.standard_normal((n, k)) * 0.02).astype(np.float32)
    specs = [(4, 128, False, 1.0, 0), (3, 128, False, 1.0, 0), (8, 0, True, 1.0, 0), (8, 0, True, 1.0, 1),
             (4, 64, False, 0.9, 0), (6, 0, True, 1.0, 0)]
    qms = [oc.quantize(w, *s) for s in specs]
    a_bits = wl.f32_to_bf16_bits(rng.standard_normal((S * T, k)).astype(np.float32))
    e = np.array([0, 1, 2, 3, 5, 0, 0, 1, 1, 1, 2, 3, 3, 0], dtype=np.int32)      # expert 4 empty, expert 5 one sample
    y = _run(a_bits, e, qms, S, T, scatter, use_perm)
    ok, worst = ob.tolerance_ok(y, _ref(a_bits, e, qms, S, T))
    assert ok, worst


@pytest.mark.parametrize("rows", [1, 15, 16, 17, 31, 32, 33, 64, 100])
def test_bucket_sizes_around_tile_edges(rows):
    rng = np.random.default_rng(rows)
    n, k = 32, 256
    w = (rng.standard_normal((n, k)) * 0.02).astype(np.float32)
    qms = [oc.quantize(w, 4, 128, False), oc.quantize(w, 8, 0, True)]
    S = rows + 3
    a_bits = wl.f32_to_bf16_bits(rng.standard_normal((S, k)).astype(np.float32))
    e = np.zeros(S, dtype=np.int32)
    e[[0, S // 2, S - 1]] = 1
    y = _run(a_bits, e, qms, S, 1)
    ok, worst = ob.tolerance_ok(y, _ref(a_bits, e, qms, S, 1))
    assert ok, worst


@pytest.mark.parametrize("S,T,counts", [
    (200, 1, [150, 20, 1, 0, 29]),        # more than 128 rows in all: both kernels run, the 150-row bucket is tiled
    (100, 2, [75, 16, 9]),                # the same with two rows per sample: buckets of 150, 32 and 18 rows
    (129, 1, [33, 32, 32, 32]),           # every bucket at the limit of one streaming pass, one just above it
    (1, 200, [1]),                        # one sample of 200 tokens: the tiled kernel alone
    (4, 32, [2, 1, 1]),                   # samples of exactly one streaming pass: 128 rows, the streaming kernel alone
    (5, 32, [3, 1, 1]),                   # 160 rows in samples of 32: a 96-row bucket tiled, two of 32 streamed
])
def test_launches_that_split_the_experts_between_the_kernels(S, T, counts):
    """Which kernel takes a bucket follows its number of rows; one launch can use both."""
    rng = np.random.default_rng(S * 7 + T)
    n, k = 48, 384
    w = (rng.standard_normal((n, k)) * 0.02).astype(np.float32)
    specs = [(4, 128, False, 1.0, 0), (8, 0, True, 1.0, 1), (3, 64, False, 1.0, 0), (6, 0, True, 1.0, 0),
             (8, 0, True, 1.0, 0)]
    qms = [oc.quantize(w, *specs[i]) for i in range(len(counts))]
    assert sum(counts) == S
    e = rng.permutation(np.repeat(np.arange(len(counts)), counts)).astype(np.int32)
    a_bits = wl.f32_to_bf16_bits(rng.standard_normal((S * T, k)).astype(np.float32))
    y = _run(a_bits, e, qms, S, T)
    ok, worst = ob.tolerance_ok(y, _ref(a_bits, e, qms, S, T))
    assert ok, worst


def test_w8a8_integer_accumulators_are_exact():
    """With unit scales the W8A8 output IS the int32 dot product: compare exactly."""
    rng = np.random.default_rng(3)
    S, n, k = 20, 32, 512
    q = rng.integers(-127, 128, (n, k)).astype(np.int8)
    qm = oc.QMat(q=q, scale=np.ones(n, dtype=np.float32), zero=None, bits=8, group=0, symmetric=True, act_mode=1)
    xi = rng.integers(-127, 128, (S, k)).astype(np.float32)
    xi[:, 0] = 127.0                                  # amax 127 -> activation scale exactly 1
    a_bits = wl.f32_to_bf16_bits(xi)                  # integers up to 127 are exact in bf16
    e = np.zeros(S, dtype=np.int32)
    y = _run(a_bits, e, [qm], S, 1)
    ref = xi.astype(np.int64) @ q.astype(np.int64).T
    assert np.array_equal(y.reshape(S, n).astype(np.int64), ref)


@pytest.mark.parametrize("bits,group,sym,clip,act", FORMATS)
@pytest.mark.parametrize("rows", [7, 29])
def test_long_rows_per_format(bits, group, sym, clip, act, rows):
    """k = 8192 (64 steps of 128 columns: the long-row geometry of the few-rows kernel) in every format,
    one and two 16-row blocks, weight rows that do not fill a work-group."""
    rng = np.random.default_rng(bits * 19 + group + rows)
    n, k = 48, 8192
    w = (rng.standard_normal((n, k)) * 0.02).astype(np.float32)
    qm = oc.quantize(w, bits, group, sym, clip, act)
    a_bits = wl.f32_to_bf16_bits(rng.standard_normal((rows, k)).astype(np.float32))
    e = np.zeros(rows, dtype=np.int32)
    y = _run(a_bits, e, [qm], rows, 1)
    ok, worst = ob.tolerance_ok(y, _ref(a_bits, e, [qm], rows, 1))
    assert ok, worst
    assert worst < 0.05


def test_decode_shape_llama_gate_matrix():
    """One decode-shaped problem at full width: 64 rows over 4 experts of an 11008 x 4096 matrix."""
    cfg = wl.get_config("llama7b_mlp_decode")
    rng = np.random.default_rng(4)
    w = (rng.standard_normal((cfg.F, cfg.D)) * 0.02).astype(np.float32)
    qms = [oc.quantize(w, s.bits, s.group, s.symmetric, s.clip, s.act_mode) for s in cfg.experts]
    a_bits = wl.make_activations(cfg).reshape(cfg.S, cfg.D)
    e = rng.integers(0, 4, cfg.S).astype(np.int32)
    y = _run(a_bits, e, qms, cfg.S, 1)
    ok, worst = ob.tolerance_ok(y, _ref(a_bits, e, qms, cfg.S, 1))
    assert ok, worst


def _random_case(seed):
    rng = np.random.default_rng(1000 + seed)
    K = int(rng.integers(1, 7))
    T = int(rng.choice([1, 1, 2, 3, 5, 17, 33, 40]))
    S = int(rng.integers(1, max(2, 260 // T)))
    n = 16 * int(rng.integers(1, 11))
    k = 128 * int(rng.choice([1, 2, 3, 5, 8, 33, 34]))       # 33 and 34 k-tiles: rows too long for the register-resident kernel
    specs = [FORMATS[int(i)] for i in rng.integers(0, len(FORMATS), K)]
    e = rng.integers(0, K, S).astype(np.int32)
    if K > 1 and rng.random() < 0.5:
        e[e == K - 1] = 0                                     # an empty expert, a heavier first one
    return rng, K, S, T, n, k, specs, e


@pytest.mark.parametrize("seed", range(24))
def test_random_shapes_formats_and_routings(seed):
    """Seeded random problems across the kernels' dispatch (few rows / many rows / both in one launch, short and long
    weight rows, every format, empty experts), compared element by element with the oracle."""
    rng, K, S, T, n, k, specs, e = _random_case(seed)
    w = (rng.standard_normal((n, k)) * 0.02).astype(np.float32)
    qms = [oc.quantize(w, *s) for s in specs]
    a_bits = wl.f32_to_bf16_bits(rng.standard_normal((S * T, k)).astype(np.float32))
    scatter, use_perm = bool(seed % 2 == 0), bool(seed % 3 != 0)
    y = _run(a_bits, e, qms, S, T, scatter, use_perm)
    ok, worst = ob.tolerance_ok(y, _ref(a_bits, e, qms, S, T))
    assert ok, (worst, K, S, T, n, k, specs)
