"""Pins for the oracle's round-to-nearest quantizers and bfloat16 rounding (CPU only).

The paper prints no quantizer; these pins are hand-worked groups whose arithmetic is exact
in binary (tests/golden/rtn_worked_examples.txt), the s/2 round-trip bound, range invariants,
an independent scalar loop, and torch's own bfloat16 conversion.
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import moqe_oracle as oc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "rtn_worked_examples.txt")


def _load_golden():
    cases = {}
    cur = None
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if not line:
            continue
        if line.startswith("["):
            cur = line.strip("[]")
            cases[cur] = {}
            continue
        key, val = line.split("=")
        cases[cur][key.strip()] = [float(v) for v in val.split()]
    return cases


def test_worked_int8_symmetric_row():
    g = _load_golden()["int8_sym"]
    qm = oc.quantize_sym_per_channel(np.array([g["w"]], dtype=np.float32), 8)
    assert qm.scale[0] == np.float32(g["scale"][0])
    assert qm.q[0].tolist() == [int(v) for v in g["q"]]      # 0.5 ties to 0 (half-to-even)


@pytest.mark.parametrize("case", ["int4_asym", "int4_asym_clip09"])
def test_worked_int4_asymmetric_group(case):
    g = _load_golden()[case]
    w = np.array([g["w"]], dtype=np.float32)
    qm = oc.quantize_asym_group(w, 4, w.shape[1], clip=g["clip"][0])
    assert qm.q[0].tolist() == [int(v) for v in g["q"]]
    assert int(qm.zero[0, 0]) == int(g["zero"][0])
    assert math.isclose(float(qm.scale[0, 0]), g["scale"][0], rel_tol=1e-6)
    np.testing.assert_allclose(oc.dequant(qm)[0], g["deq"], rtol=1e-6, atol=1e-9)
    assert oc.dequant_int(qm)[0].tolist() == [int(a) - int(g["zero"][0]) for a in g["q"]]


FORMATS = [(8, 0, True, 1.0), (6, 0, True, 1.0), (4, 0, True, 1.0),
           (4, 64, False, 1.0), (4, 128, False, 1.0), (3, 64, False, 1.0), (3, 128, False, 1.0),
           (4, 128, False, 0.9), (4, 128, False, 0.85), (3, 128, False, 0.9)]


def _rand_w(n, k, seed=0, std=0.02):
    return (np.random.default_rng(seed).standard_normal((n, k)) * std).astype(np.float32)


@pytest.mark.parametrize("bits,group,sym,clip", FORMATS)
def test_round_trip_error_at_most_half_scale(bits, group, sym, clip):
    w = _rand_w(48, 512, seed=bits * 100 + group)
    qm = oc.quantize(w, bits, group, sym, clip)
    deq = oc.dequant(qm)
    g = group if group else w.shape[1]
    s = np.repeat(qm.scale.astype(np.float64).reshape(w.shape[0], -1), g, axis=1)
    target = w.astype(np.float64)
    if not sym:
        wg = w.reshape(w.shape[0], -1, g)
        lo = np.float32(clip) * np.minimum(wg.min(axis=2), np.float32(0))
        hi = np.float32(clip) * np.maximum(wg.max(axis=2), np.float32(0))
        target = np.clip(target, np.repeat(lo.astype(np.float64), g, axis=1),
                         np.repeat(hi.astype(np.float64), g, axis=1))
    qrange = 2.0 ** bits
    # fp32 quotient W/s carries a relative error of 2^-24, i.e. up to qrange * 2^-24 code units
    assert np.all(np.abs(target - deq) <= s * (0.5 + 4 * qrange * 2.0 ** -24))
    # and the bound is tight: some element sits close to half a step away
    assert np.max(np.abs(target - deq) / s) > 0.45


@pytest.mark.parametrize("bits", [8, 6, 4])
def test_symmetric_invariants(bits):
    w = _rand_w(32, 256, seed=bits)
    qm = oc.quantize_sym_per_channel(w, bits)
    qmax = 2 ** (bits - 1) - 1
    assert qm.q.dtype == np.int8 and qm.zero is None
    assert np.all(np.abs(qm.q.astype(int)) <= qmax)
    am = np.argmax(np.abs(w), axis=1)
    rows = np.arange(w.shape[0])
    assert np.all(np.abs(qm.q[rows, am].astype(int)) == qmax)
    assert np.all(np.sign(qm.q[rows, am]) == np.sign(w[rows, am]))


@pytest.mark.parametrize("bits,group", [(4, 64), (3, 128)])
def test_asymmetric_invariants(bits, group):
    w = _rand_w(32, 256, seed=7 * bits)
    qm = oc.quantize_asym_group(w, bits, group)
    L = 2 ** bits - 1
    assert qm.q.dtype == np.uint8 and qm.zero.dtype == np.uint8
    assert qm.q.max() <= L and qm.zero.max() <= L
    assert qm.scale.shape == (32, 256 // group) and qm.zero.shape == qm.scale.shape
    # the code equal to the zero-point decodes to exactly 0
    qz = oc.QMat(q=np.repeat(qm.zero, group, axis=1), scale=qm.scale, zero=qm.zero,
                 bits=bits, group=group, symmetric=False)
    assert np.all(oc.dequant(qz) == 0.0)
    # both ends of the code range are used in (nearly) every group of a Gaussian matrix
    qg = qm.q.reshape(32, -1, group)
    assert np.mean(qg.min(axis=2) == 0) > 0.95 and np.mean(qg.max(axis=2) == L) > 0.95


def test_degenerate_groups():
    w = np.zeros((2, 128), dtype=np.float32)
    w[1, :64] = 0.25                      # constant positive group: lo = 0
    qs = oc.quantize_sym_per_channel(w, 8)
    assert qs.scale[0] == 1.0 and np.all(qs.q[0] == 0)
    qa = oc.quantize_asym_group(w, 4, 64)
    assert qa.scale[0, 0] == 1.0 and qa.zero[0, 0] == 0 and np.all(qa.q[0] == 0)
    assert qa.zero[1, 0] == 0 and np.all(qa.q[1, :64] == 15)
    np.testing.assert_allclose(oc.dequant(qa)[1, :64], 0.25, rtol=1e-6)
    # all-negative group: hi = 0, zero-point at the top of the range
    qn = oc.quantize_asym_group(-w, 4, 64)
    assert qn.zero[1, 0] == 15 and np.all(qn.q[1, :64] == 0)


def _scalar_asym(wrow, bits, clip):
    """Independent scalar loop in fp32 for one group."""
    f = np.float32
    lo, hi = f(0), f(0)
    for v in wrow:
        lo = min(lo, f(v))
        hi = max(hi, f(v))
    lo, hi = f(f(clip) * lo), f(f(clip) * hi)
    L = f(2 ** bits - 1)
    s = f(1) if hi == lo else f(f(hi - lo) / L)
    z = min(max(f(np.rint(f(-lo) / s)), f(0)), L)
    qs = [int(min(max(f(np.rint(f(v) / s)) + z, f(0)), L)) for v in wrow]
    return qs, float(s), int(z)


@pytest.mark.parametrize("bits,clip", [(4, 1.0), (3, 1.0), (4, 0.9), (3, 0.85)])
def test_asym_matches_scalar_loop(bits, clip):
    w = _rand_w(6, 32, seed=11)
    qm = oc.quantize_asym_group(w, bits, 16, clip)
    for n in range(6):
        for g in range(2):
            qs, s, z = _scalar_asym(w[n, 16 * g:16 * g + 16], bits, clip)
            assert qm.q[n, 16 * g:16 * g + 16].tolist() == qs
            assert float(qm.scale[n, g]) == s and int(qm.zero[n, g]) == z


def test_sym_matches_scalar_loop():
    w = _rand_w(5, 24, seed=12)
    for bits in (8, 6, 4):
        qm = oc.quantize_sym_per_channel(w, bits)
        f = np.float32
        for n in range(5):
            a = f(0)
            for v in w[n]:
                a = max(a, abs(f(v)))
            s = f(a / f(2 ** (bits - 1) - 1))
            assert float(qm.scale[n]) == float(s)
            for k in range(24):
                q = int(np.rint(f(w[n, k]) / s))
                assert int(qm.q[n, k]) == q


# ------------------------------- bfloat16 rounding -------------------------------------
def test_bf16_round_hand_ties():
    assert oc.bf16_round(1.0 + 2.0 ** -8) == 1.0                       # tie -> even mantissa
    assert oc.bf16_round(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6       # tie -> even mantissa
    assert oc.bf16_round(1.0 + 2.0 ** -8 + 2.0 ** -40) == 1.0 + 2.0 ** -7   # just above the tie: up
    assert oc.bf16_round(-0.3) == -0.30078125
    assert oc.bf16_round(0.0) == 0.0
    assert oc.bf16_round(255.5) == 256.0 and oc.bf16_round(254.5) == 254.0


def test_bf16_round_matches_torch_on_fp32_inputs():
    rng = np.random.default_rng(3)
    x = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-6, 6, 20000),
                        np.array([0.0, 1e-30, -1e-30, 3e38, 65504.0])]).astype(np.float32)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(oc.bf16_round(x), ref)
    assert np.array_equal(oc.bf16_round(ref), ref)                      # idempotent


def test_bf16_bits_to_f64():
    bits = np.array([0x3F80, 0xBF80, 0x4300, 0x0000, 0x3DCD], dtype=np.uint16)
    ref = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(oc.bf16_bits_to_f64(bits), ref)
    assert oc.bf16_bits_to_f64(bits)[:3].tolist() == [1.0, -1.0, 128.0]
