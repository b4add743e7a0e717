"""Pins for the oracle's expert layers and the routed forward (CPU only).

Pinned against scalar Python loops on tiny shapes, numpy / torch library routines in special
cases, and the structural facts the paper fixes: one expert per sample (Section 3.1, Fig. 1),
the prediction f_{r(x)}(x) (appendix on router convergence), so a router that always picks
expert e reproduces the single quantized model e.
"""
import math

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import moqe_oracle as oc
from tests import oracle_blocks as ob


def _bf16_vals(rng, shape, scale=1.0):
    return oc.bf16_round(rng.standard_normal(shape) * scale)


def _bf16_by_bits(v):
    """fp64 -> nearest bfloat16 value by integer arithmetic on the fp64 bit pattern (normal range)."""
    u = np.asarray(v, dtype=np.float64).view(np.uint64)
    drop = np.uint64(52 - 7)
    u = u + ((np.uint64(1) << (drop - np.uint64(1))) - np.uint64(1)) + ((u >> drop) & np.uint64(1))
    return ((u >> drop) << drop).view(np.float64)


def _loop_dequant(qm):
    n, k = qm.q.shape
    g = qm.group if qm.group else k
    w = [[0.0] * k for _ in range(n)]
    for i in range(n):
        for j in range(k):
            s = float(qm.scale[i]) if qm.scale.ndim == 1 else float(qm.scale[i, j // g])
            z = 0 if qm.zero is None else int(qm.zero[i, j // g])
            w[i][j] = s * (int(qm.q[i, j]) - z)
    return w


@pytest.mark.parametrize("bits,group,sym", [(8, 0, True), (6, 0, True), (4, 8, False), (3, 4, False)])
def test_qlinear_matches_scalar_loops(bits, group, sym):
    rng = np.random.default_rng(bits)
    w = (rng.standard_normal((5, 16)) * 0.02).astype(np.float32)
    qm = oc.quantize(w, bits, group, sym)
    x = _bf16_vals(rng, (3, 16))
    y = oc.qlinear(x, qm)
    wd = _loop_dequant(qm)
    for m in range(3):
        for n in range(5):
            ref = math.fsum(float(x[m, k]) * wd[n][k] for k in range(16))
            assert math.isclose(y[m, n], ref, rel_tol=1e-12, abs_tol=1e-15)
    assert np.array_equal(np.array(wd), oc.dequant(qm))


def test_w8a8_matches_scalar_loops():
    rng = np.random.default_rng(5)
    w = (rng.standard_normal((4, 12)) * 0.02).astype(np.float32)
    qm = oc.quantize_sym_per_channel(w, 8, act_mode=1)
    x = _bf16_vals(rng, (3, 12))
    x[2] = 0.0                                    # all-zero row: scale 1, codes 0
    y = oc.qlinear(x, qm)
    f = np.float32
    for m in range(3):
        a = max(abs(f(v)) for v in x[m])
        sx = f(1) if a == 0 else f(a / f(127))
        xq = [int(min(max(np.rint(f(v) / sx), -127), 127)) for v in x[m]]
        assert max(abs(v) for v in xq) == (127 if a else 0)
        for n in range(4):
            acc = sum(xq[k] * int(qm.q[n, k]) for k in range(12))
            assert math.isclose(y[m, n], acc * float(sx) * float(qm.scale[n]), rel_tol=1e-14, abs_tol=0)


def test_act_quant_hand_example():
    xq, sx = oc.act_quant_int8(np.array([[1.27, -0.635, 0.005, 0.0]]))
    assert xq[0].tolist()[:2] == [127, -64] or xq[0].tolist()[:2] == [127, -63]
    x = np.array([[127.0, 0.5, 1.5, 2.5, -63.5]])
    xq, sx = oc.act_quant_int8(x)
    assert sx[0] == 1.0 and xq[0].tolist() == [127, 0, 2, 2, -64]     # halves go to even


def test_silu_mlp_matches_scalar_loops():
    rng = np.random.default_rng(6)
    D, F = 8, 16
    wg, wu = [(rng.standard_normal((F, D)) * 0.3).astype(np.float32) for _ in range(2)]
    wd = (rng.standard_normal((D, F)) * 0.3).astype(np.float32)
    gate, up = oc.quantize_asym_group(wg, 4, 8), oc.quantize_asym_group(wu, 4, 8)
    down = oc.quantize_asym_group(wd, 4, 8)
    x = _bf16_vals(rng, (2, D))
    y, h = oc.silu_mlp(x, gate, up, down)
    g_, u_, d_ = _loop_dequant(gate), _loop_dequant(up), _loop_dequant(down)
    for m in range(2):
        hm = []
        for f in range(F):
            g = math.fsum(float(x[m, k]) * g_[f][k] for k in range(D))
            u = math.fsum(float(x[m, k]) * u_[f][k] for k in range(D))
            hv = (g / (1.0 + math.exp(-g))) * u
            hb = float(_bf16_by_bits(np.array([hv]))[0])
            hm.append(hb)
            assert h[m, f] == hb
        for n in range(D):
            ref = math.fsum(float(h[m, f]) * d_[n][f] for f in range(F))
            assert math.isclose(y[m, n], ref, rel_tol=1e-12, abs_tol=1e-15)
    assert np.array_equal(h, oc.bf16_round(h))


def test_silu_values():
    assert oc.silu(np.array([0.0]))[0] == 0.0
    assert math.isclose(oc.silu(np.array([1.0]))[0], 1.0 / (1.0 + math.exp(-1.0)))
    assert math.isclose(oc.silu(np.array([-2.0]))[0], -2.0 / (1.0 + math.exp(2.0)))
    assert math.isclose(oc.silu(np.array([30.0]))[0], 30.0, rel_tol=1e-12)


def test_conv_matches_scalar_loops_and_torch():
    rng = np.random.default_rng(7)
    Hh, Ww, Cin, Cout = 4, 4, 2, 3
    w = (rng.standard_normal((Cout, Cin * 9)) * 0.1).astype(np.float32)
    qm = oc.quantize_sym_per_channel(w, 6)
    img = _bf16_vals(rng, (Hh, Ww, Cin))
    y = oc.conv3x3(img, qm, Cin)
    wd = oc.dequant(qm)
    for h in range(Hh):
        for x_ in range(Ww):
            for n in range(Cout):
                acc = 0.0
                for c in range(Cin):
                    for kh in range(3):
                        for kw in range(3):
                            hh, ww = h + kh - 1, x_ + kw - 1
                            if 0 <= hh < Hh and 0 <= ww < Ww:
                                acc += img[hh, ww, c] * wd[n, (kh * 3 + kw) * Cin + c]
                assert math.isclose(y[h, x_, n], acc, rel_tol=1e-11, abs_tol=1e-14)
    t = torch.nn.functional.conv2d(torch.from_numpy(img).permute(2, 0, 1)[None],
                                   torch.from_numpy(wd).reshape(Cout, 3, 3, Cin).permute(0, 3, 1, 2), padding=1)
    np.testing.assert_allclose(y, t[0].permute(1, 2, 0).numpy(), rtol=1e-11, atol=1e-14)


def test_conv_group_format_is_im2col_matmul():
    rng = np.random.default_rng(8)
    Hh, Ww, Cin, Cout = 5, 6, 64, 4
    w = (rng.standard_normal((Cout, Cin * 9)) * 0.02).astype(np.float32)
    qm = oc.quantize_asym_group(w, 4, 64)
    img = _bf16_vals(rng, (Hh, Ww, Cin))
    y = oc.conv3x3(img, qm, Cin)
    xp = np.pad(img, ((1, 1), (1, 1), (0, 0)))
    cols = np.zeros((Hh * Ww, Cin * 9))
    for h in range(Hh):
        for x_ in range(Ww):
            for c in range(Cin):
                for kh in range(3):
                    for kw in range(3):
                        cols[h * Ww + x_, (kh * 3 + kw) * Cin + c] = xp[h + kh, x_ + kw, c]
    np.testing.assert_allclose(y.reshape(Hh * Ww, Cout), cols @ oc.dequant(qm).T, rtol=1e-11, atol=1e-14)


# ----------------------------------- routed forward -----------------------------------
def _small_cfg(kind):
    if kind == "linear":
        return wl.scaled(wl.get_config("toy_linear"), S=12, T=5, D=128, F=48)
    if kind == "mlp":
        return wl.scaled(wl.get_config("llama7b_mlp_decode"), S=10, T=3, D=128, F=256, router_hidden=16)
    if kind == "mlp8":
        return wl.scaled(wl.get_config("qwen_mlp_skew"), S=24, T=2, D=128, F=256, router_hidden=16)
    return wl.scaled(wl.get_config("resnet50_conv"), S=6, T=20, D=64, F=16, img_h=4, img_w=5, router_hidden=8)


@pytest.mark.parametrize("kind", ["linear", "mlp", "mlp8", "conv"])
def test_one_hot_router_is_the_single_quantized_model(kind):
    cfg = _small_cfg(kind)
    blk = ob.make_block(cfg)
    _, x = ob.activations_f64(cfg)
    for e in range(cfg.K):
        b2 = np.zeros(cfg.K, dtype=np.float32)
        b2[e] = 1e4
        blk.router.b2 = b2
        y, idx, _ = oc.forward(blk, x)
        assert np.all(idx == e)
        rows = x.reshape(cfg.S * cfg.T, cfg.D)
        if kind == "linear":
            ref = np.matmul(rows, np.array(_loop_dequant(blk.w0[e])).T)
        elif kind in ("mlp", "mlp8"):
            if blk.w0[e].act_mode:
                continue                         # W8A8 is pinned by its own scalar-loop test
            g = np.matmul(rows, np.array(_loop_dequant(blk.w0[e])).T)
            u = np.matmul(rows, np.array(_loop_dequant(blk.w1[e])).T)
            h = _bf16_by_bits(g / (1 + np.exp(-g)) * u)
            ref = np.matmul(h, np.array(_loop_dequant(blk.w2[e])).T)
        else:
            wd = torch.from_numpy(np.array(_loop_dequant(blk.w0[e]))).reshape(cfg.F, 3, 3, cfg.D).permute(0, 3, 1, 2)
            xi = torch.from_numpy(x.reshape(cfg.S, cfg.img_h, cfg.img_w, cfg.D)).permute(0, 3, 1, 2)
            ref = torch.nn.functional.conv2d(xi, wd, padding=1).permute(0, 2, 3, 1).numpy()
        ref = ref.reshape(y.shape)
        np.testing.assert_allclose(y, ref, rtol=1e-9, atol=1e-12)


def test_single_expert_block():
    cfg = wl.scaled(_small_cfg("linear"), experts=_small_cfg("linear").experts[1:2])
    blk = ob.make_block(cfg)
    _, x = ob.activations_f64(cfg)
    y, idx, logits = oc.forward(blk, x)
    assert np.all(idx == 0) and logits.shape == (cfg.S, 1)
    np.testing.assert_allclose(y.reshape(-1, cfg.F), x.reshape(-1, cfg.D) @ oc.dequant(blk.w0[0]).T, rtol=1e-12)


@pytest.mark.parametrize("kind", ["linear", "mlp", "conv"])
def test_each_sample_uses_exactly_its_expert_and_nothing_else(kind):
    cfg = _small_cfg(kind)
    blk = ob.make_block(cfg)
    _, x = ob.activations_f64(cfg)
    y, idx, logits = oc.forward(blk, x)
    assert len(set(idx.tolist())) > 1                       # the router really spreads this batch
    # permuting the samples permutes the outputs (equivariance)
    p = np.random.default_rng(0).permutation(cfg.S)
    yp, idxp, _ = oc.forward(blk, x[p])
    assert np.array_equal(idxp, idx[p]) and np.array_equal(yp, y[p])
    # a sample's output does not depend on the rest of the batch
    for s in (0, cfg.S - 1):
        ys, ids, _ = oc.forward(blk, x[s:s + 1])
        assert ids[0] == idx[s] and np.array_equal(ys[0], y[s])
        assert np.array_equal(y[s], oc.expert_forward(blk, int(idx[s]), x[s]))
    # and differs from what any other expert would give
    other = (int(idx[0]) + 1) % cfg.K
    assert not np.allclose(oc.expert_forward(blk, other, x[0]), y[0], rtol=1e-3)


def test_row_subset_equals_full_rows():
    cfg = _small_cfg("mlp8")
    blk = ob.make_block(cfg)
    _, x = ob.activations_f64(cfg)
    y, _, _ = oc.forward(blk, x)
    ysub, _, _ = oc.forward(blk, x, rows=[1])
    np.testing.assert_allclose(ysub[:, 0], y[:, 1], rtol=1e-10, atol=1e-14)   # BLAS sums in another order
    assert any(q.act_mode == 1 for q in blk.w0)


def test_routing_accuracy_against_itself_is_one():
    # RA = (1/N) sum 1{r(x_i) = j*(x_i)} (appendix on router convergence) used as a parity metric
    cfg = _small_cfg("mlp")
    blk = ob.make_block(cfg)
    _, x = ob.activations_f64(cfg)
    idx, _, _ = oc.route(x, blk.router)
    assert np.mean(idx == oc.forward(blk, x)[1]) == 1.0


def test_ragged_forward_reduces_to_the_uniform_one_and_is_per_sample():
    """Samples of different lengths: equal lengths give the uniform forward; a sample's result depends on
    nothing but its own rows (any other sample may change or vanish); a sample is routed by the mean of
    ITS rows (appending rows that change the mean can change the expert, appending copies cannot)."""
    rng = np.random.default_rng(9)
    D, F, K = 128, 256, 3
    fp = {n: (rng.standard_normal(sh) * 0.05).astype(np.float32) for n, sh in
          (("gate", (F, D)), ("up", (F, D)), ("down", (D, F)))}
    specs = [(8, 0, True, 1.0, 0), (4, 64, False, 1.0, 0), (3, 64, False, 0.9, 0)]
    router = oc.Router(None, None, (rng.standard_normal((K, D)) * 0.5).astype(np.float32), None)
    blk = oc.Block(oc.KIND_SILU_MLP, router, [oc.quantize(fp["gate"], *sp) for sp in specs],
                   [oc.quantize(fp["up"], *sp) for sp in specs], [oc.quantize(fp["down"], *sp) for sp in specs])
    x = oc.bf16_round(rng.standard_normal((5, 4, D)))
    y_u, idx_u, log_u = oc.forward(blk, x)
    ys, idx_r, log_r = oc.forward_ragged(blk, [x[s] for s in range(5)])
    assert np.array_equal(idx_u, idx_r) and np.allclose(log_u, log_r, rtol=0, atol=1e-12)
    assert all(np.allclose(ys[s], y_u[s], rtol=1e-12, atol=1e-12) for s in range(5))
    lens = [1, 7, 3, 4, 2]
    xs = [oc.bf16_round(rng.standard_normal((t, D))) for t in lens]
    ys, idx, logits = oc.forward_ragged(blk, xs)
    assert [y.shape for y in ys] == [(t, D) for t in lens]
    alone, idx1, _ = oc.forward_ragged(blk, [xs[1]])
    assert idx1[0] == idx[1] and np.allclose(alone[0], ys[1], rtol=1e-12, atol=1e-12)
    # the feature is the mean: a sample followed by a copy of itself is routed alike, row results repeat
    dup, idx2, log2 = oc.forward_ragged(blk, [np.concatenate([xs[2], xs[2]])])
    assert idx2[0] == idx[2] and np.allclose(log2[0], logits[2], rtol=1e-12, atol=1e-12)
    assert np.allclose(dup[0][:3], ys[2], rtol=1e-12, atol=1e-12) and np.allclose(dup[0][3:], ys[2], rtol=1e-12, atol=1e-12)
    # one row per sample is the T = 1 case of the uniform path
    single = [x[s, :1] for s in range(5)]
    y1, idx_s, _ = oc.forward_ragged(blk, single)
    y1u, idx_su, _ = oc.forward(blk, x[:, :1])
    assert np.array_equal(idx_s, idx_su) and all(np.allclose(y1[s], y1u[s], rtol=1e-12, atol=1e-12) for s in range(5))
