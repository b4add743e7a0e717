"""Pins of the oracle's CV router model (Section 3.2: three-layer MLP with batch norm and ReLU, three-stage
SEResNet-8 with 16/32/64 channels and strides 1/2/2, 8-head self-attention -> logits): torch's conv2d, batch_norm and
MultiheadAttention with the same parameters, a whole stage and the whole router as torch compositions, scalar loops,
closed forms."""
import math

import numpy as np
import torch
import torch.nn.functional as F

import workloads as wl
from oracle import moqe_oracle as oc
from oracle import router_cv_oracle as rc
from tests import oracle_router_cv as orc

C, MLP, STAGES, STRIDES, HEADS, K = 24, (20, 16, 16), (16, 32, 64), (1, 2, 2), 8, 3


def _setup(S=2, h=9, w=10, seed=5):
    p = wl.make_cv_router(C, MLP, STAGES, STRIDES, K, seed)
    r = orc.make(p, len(MLP), STRIDES, HEADS)
    x = oc.bf16_bits_to_f64(wl.make_image_activations(S, h, w, C, seed + 1))
    return p, r, x


def _t(a):
    return torch.from_numpy(np.asarray(a, dtype=np.float64))


def _tconv(x_hwc, w_okki, stride):
    pad = (w_okki.shape[1] - 1) // 2
    y = F.conv2d(_t(x_hwc).permute(2, 0, 1)[None], _t(w_okki).permute(0, 3, 1, 2), stride=stride, padding=pad)
    return y[0].permute(1, 2, 0)


def _tbn(x_hwc, bn):
    y = F.batch_norm(x_hwc.permute(2, 0, 1)[None], _t(bn.mean), _t(bn.var), _t(bn.gain), _t(bn.offset), False, 0.0, rc.BN_EPS)
    return y[0].permute(1, 2, 0)


def test_conv_and_batch_norm_match_torch_for_every_stride_and_filter_size():
    p, r, x = _setup()
    img = x[0][:, :, :16]
    for stride in (1, 2):
        got = rc.conv(img, p["st0_a"], stride)
        ref = _tconv(img, p["st0_a"], stride).numpy()
        assert got.shape == ref.shape and np.allclose(got, ref, rtol=1e-11, atol=1e-12)
    w1 = p["st1_s"][:, None, None, :]
    assert np.allclose(rc.conv(img, w1, 2), _tconv(img, w1, 2).numpy(), rtol=1e-11, atol=1e-12)
    bn = r.stages[0].bn_a
    y = rc.conv(img, p["st0_a"], 1)
    assert np.allclose(rc.batch_norm(y, bn), _tbn(_t(y), bn).numpy(), rtol=1e-11, atol=1e-12)
    assert rc.conv(np.zeros((14, 14, 16)), p["st1_a"], 2).shape == (7, 7, 32)
    assert rc.conv(np.zeros((7, 7, 32)), p["st2_a"], 2).shape == (4, 4, 64)


def _torch_stage(xt, st):
    a = torch.relu(_tbn(_tconv(xt.numpy(), st.conv_a, st.stride), st.bn_a))
    u = _tbn(_tconv(a.numpy(), st.conv_b, 1), st.bn_b)
    z = F.adaptive_avg_pool2d(u.permute(2, 0, 1)[None], 1)[0, :, 0, 0]
    g = torch.sigmoid(_t(st.se_w2) @ torch.relu(_t(st.se_w1) @ z + _t(st.se_b1)) + _t(st.se_b2))
    short = xt if st.short_w is None else _tbn(_tconv(xt.numpy(), st.short_w[:, None, None, :], st.stride), st.short_bn)
    return torch.relu(u * g + short)


def test_every_stage_matches_a_torch_composition():
    p, r, x = _setup()
    cur = _t(np.maximum(x[1][:, :, :16], 0.0))
    for st in r.stages:
        ref = _torch_stage(cur, st)
        got = rc.stage_forward(cur.numpy(), st)
        assert got.shape == tuple(ref.shape) and np.allclose(got, ref.numpy(), rtol=1e-10, atol=1e-12)
        cur = ref
    assert cur.shape == (3, 3, 64)                     # 9 x 10 -> 9 x 10 -> 5 x 5 -> 3 x 3


def test_whole_router_matches_a_torch_composition():
    p, r, x = _setup(S=3)
    mha = torch.nn.MultiheadAttention(64, HEADS, batch_first=True, dtype=torch.float64)
    with torch.no_grad():
        mha.in_proj_weight.copy_(_t(p["wqkv"])); mha.in_proj_bias.copy_(_t(p["bqkv"]))
        mha.out_proj.weight.copy_(_t(p["wo"])); mha.out_proj.bias.copy_(_t(p["bo"]))
        ref_logits = []
        for s in range(3):
            cur = _t(x[s])
            for w, b, bn in zip(r.mlp_w, r.mlp_b, r.mlp_bn):
                cur = torch.relu(_tbn(cur @ _t(w).T + _t(b), bn))
            for st in r.stages:
                cur = _torch_stage(cur, st)
            tok = cur.reshape(-1, 64)[None]
            pooled = mha(tok, tok, tok, need_weights=False)[0][0].mean(dim=0)
            ref_logits.append((pooled @ _t(p["w_out"]).T + _t(p["b_out"])).numpy())
    idx, logits, _ = rc.route_cv(x, r)
    assert np.allclose(logits, np.stack(ref_logits), rtol=1e-9, atol=1e-11)
    assert np.array_equal(idx, np.argmax(np.stack(ref_logits), axis=1))


def test_one_strided_output_pixel_by_scalar_loops_and_closed_forms():
    p, r, x = _setup()
    img = x[0][:, :, :16]
    w = p["st1_a"].astype(np.float64)                                    # [32, 3, 3, 16], stride 2
    oy, ox, co = 2, 4, 7
    acc = []
    for kh in range(3):
        for kw in range(3):
            iy, ix = oy * 2 + kh - 1, ox * 2 + kw - 1
            if 0 <= iy < img.shape[0] and 0 <= ix < img.shape[1]:
                acc += [img[iy, ix, c] * w[co, kh, kw, c] for c in range(16)]
    assert abs(rc.conv(img, p["st1_a"], 2)[oy, ox, co] - math.fsum(acc)) < 1e-12
    ident = rc.BatchNorm(np.ones(4), np.zeros(4), np.zeros(4), np.ones(4) - rc.BN_EPS)
    v = np.random.default_rng(0).standard_normal((3, 4))
    assert np.allclose(rc.batch_norm(v, ident), v, atol=1e-15)
    # excitation weights zero: the gate is sigmoid(0) = 1/2 for every channel
    st = r.stages[0]
    flat = rc.Stage(st.conv_a, st.bn_a, st.conv_b, st.bn_b, st.se_w1, st.se_b1, np.zeros_like(st.se_w2), np.zeros_like(st.se_b2),
                    None, None, 1)
    xin = np.maximum(x[0][:, :, :16], 0.0)
    u = rc.batch_norm(rc.conv(np.maximum(rc.batch_norm(rc.conv(xin, st.conv_a, 1), st.bn_a), 0.0), st.conv_b, 1), st.bn_b)
    assert np.allclose(rc.stage_forward(xin, flat), np.maximum(0.5 * u + xin, 0.0), rtol=1e-12, atol=1e-13)
