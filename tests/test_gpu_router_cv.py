"""GPU parity of the CV router model (moqe_route_cv, Section 3.2: three-layer MLP with batch norm and ReLU, three-stage
SEResNet-8, multi-head self-attention -> logits) against the oracle.

fp32 on the GPU, fp64 in the oracle: |logit - ref| <= 1e-3 * max(1, max|ref|).  The selected expert must be the first
arg-max of the logits the library wrote (bit-exact) and the oracle's expert wherever the oracle's margin between the two
largest logits exceeds twice that tolerance."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import moqe_oracle as oc
from oracle import router_cv_oracle as rc
from tests import oracle_router_cv as orc

pytestmark = pytest.mark.gpu

#           S   h   w   c_in  mlp            stages        strides    heads K
CASES = {
    "paper_shape": (6, 14, 14, 256, (64, 32, 16), (16, 32, 64), (1, 2, 2), 8, 4),
    "odd_image": (3, 9, 10, 24, (20, 16, 16), (16, 32, 64), (1, 2, 2), 8, 3),
    "no_strides": (2, 5, 6, 32, (24, 16, 16), (16, 16, 32), (1, 1, 1), 4, 5),
    "one_image_largest": (1, 24, 24, 8, (8, 8, 8), (8, 16, 24), (1, 2, 2), 3, 2),
    "many_images": (70, 7, 7, 16, (16, 16, 16), (16, 32, 64), (1, 2, 2), 8, 4),
}


def _run(case, seed=41):
    from paper_2508_09204_amd import binding as mq
    from tests import gpu_blocks as gb
    S, h, w, c_in, mlp, stages, strides, heads, K = CASES[case]
    p = wl.make_cv_router(c_in, mlp, stages, strides, K, seed)
    bits = wl.make_image_activations(S, h, w, c_in, seed + 1)
    dev = {k: gb.to_dev(np.ascontiguousarray(v)) for k, v in p.items()}
    r = mq.CvRouter(dev, c_in, strides, heads, K)
    x = gb.bf16_dev(bits.reshape(S * h * w, c_in))
    idx = torch.full((S,), -1, dtype=torch.int32, device=gb.DEV)
    logits = torch.full((S, K), float("nan"), dtype=torch.float32, device=gb.DEV)
    mq.moqe_route_cv(x, S, h, w, r, idx, logits)
    torch.cuda.synchronize()
    ref_idx, ref_logits, _ = rc.route_cv(oc.bf16_bits_to_f64(bits), orc.make(p, 3, strides, heads))
    return idx.cpu().numpy(), logits.cpu().numpy(), ref_idx, ref_logits


@pytest.mark.parametrize("case", list(CASES))
def test_route_cv_matches_oracle(case):
    idx, logits, ref_idx, ref_logits = _run(case)
    tol = 1e-3 * max(1.0, float(np.abs(ref_logits).max()))
    err = float(np.abs(logits.astype(np.float64) - ref_logits).max())
    assert err <= tol, (err, tol)
    first_max = np.array([int(np.flatnonzero(row == row.max())[0]) for row in logits])
    assert np.array_equal(idx, first_max)
    srt = np.sort(ref_logits, axis=1)
    clear = (srt[:, -1] - srt[:, -2]) > 2 * tol
    assert np.array_equal(idx[clear], ref_idx[clear])
    assert clear.mean() >= 0.5


def test_route_cv_is_deterministic():
    a, b = _run("odd_image"), _run("odd_image")
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


@pytest.mark.timeout(900)
def test_route_cv_full_size_conv_workload_shape():
    """The conv workload's batch shape (256 images of 14 x 14 x 256) with the paper's channels, strides and heads:
    the library routes all images, the oracle checks a sample of them (its convolutions are Python loops)."""
    from paper_2508_09204_amd import binding as mq
    from tests import gpu_blocks as gb
    S, h, w, c_in, mlp, stages, strides, heads, K = 256, 14, 14, 256, (64, 32, 16), (16, 32, 64), (1, 2, 2), 8, 4
    p = wl.make_cv_router(c_in, mlp, stages, strides, K, 61)
    bits = wl.make_image_activations(S, h, w, c_in, 62)
    dev = {k: gb.to_dev(np.ascontiguousarray(v)) for k, v in p.items()}
    r = mq.CvRouter(dev, c_in, strides, heads, K)
    x = gb.bf16_dev(bits.reshape(S * h * w, c_in))
    idx = torch.full((S,), -1, dtype=torch.int32, device=gb.DEV)
    logits = torch.full((S, K), float("nan"), dtype=torch.float32, device=gb.DEV)
    mq.moqe_route_cv(x, S, h, w, r, idx, logits)
    torch.cuda.synchronize()
    lg, ix = logits.cpu().numpy(), idx.cpu().numpy()
    assert np.all(np.isfinite(lg)) and np.array_equal(ix, np.argmax(lg, axis=1)) and len(set(ix.tolist())) > 1
    sample = [0, 1, 63, 64, 127, 200, 254, 255]
    ref_idx, ref_logits, _ = rc.route_cv(oc.bf16_bits_to_f64(bits[sample]), orc.make(p, 3, strides, heads))
    tol = 1e-3 * max(1.0, float(np.abs(ref_logits).max()))
    assert float(np.abs(lg[sample] - ref_logits).max()) <= tol
    srt = np.sort(ref_logits, axis=1)
    clear = (srt[:, -1] - srt[:, -2]) > 2 * tol
    assert np.array_equal(ix[sample][clear], ref_idx[clear])


def test_router_model_drives_the_routed_conv_stage():
    """moqe_route_cv -> moqe_forward_routed on a 3x3 convolution stage: experts against the oracle's router, the stage's
    output against the oracle's stage run on the experts the GPU router chose."""
    from paper_2508_09204_amd import binding as mq
    from tests import gpu_blocks as gb
    from tests import oracle_blocks as ob
    cfg = wl.scaled(wl.get_config("resnet50_conv"), S=9, T=30, D=128, F=48, img_h=5, img_w=6, router_hidden=16)
    blk = ob.make_block(cfg)
    mlp, stages, strides, heads = (32, 16, 16), (16, 32, 64), (1, 2, 2), 8
    p = wl.make_cv_router(cfg.D, mlp, stages, strides, cfg.K, 72)      # a seed whose random router uses two experts
    bits = wl.make_image_activations(cfg.S, cfg.img_h, cfg.img_w, cfg.D, 72)
    x64 = oc.bf16_bits_to_f64(bits).reshape(cfg.S, cfg.T, cfg.D)
    dev = {k: gb.to_dev(np.ascontiguousarray(v)) for k, v in p.items()}
    r = mq.CvRouter(dev, cfg.D, strides, heads, cfg.K)
    x = gb.bf16_dev(bits.reshape(cfg.M, cfg.D))
    idx = torch.full((cfg.S,), -1, dtype=torch.int32, device=gb.DEV)
    mq.moqe_route_cv(x, cfg.S, cfg.img_h, cfg.img_w, r, idx)
    y = torch.full((cfg.M, cfg.F), float("nan"), dtype=torch.float32, device=gb.DEV)
    mq.moqe_forward_routed(gb.block_dev(blk), idx, x, cfg.S, cfg.T, y)
    torch.cuda.synchronize()
    e = idx.cpu().numpy()
    ref_idx, _, _ = rc.route_cv(oc.bf16_bits_to_f64(bits), orc.make(p, 3, strides, heads))
    assert len(set(e.tolist())) > 1 and np.mean(e == ref_idx) >= 0.8
    y_ref, _, _ = oc.forward(blk, x64, expert_idx=e)
    ok, worst = ob.tolerance_ok(y.cpu().numpy().reshape(cfg.S, cfg.T, cfg.F), y_ref)
    assert ok, worst
