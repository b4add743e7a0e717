"""GPU parity of the whole routed block (moqe_forward) against the oracle on the five workloads.

Routing indices and the bucket permutation must match bit for bit; outputs must satisfy
|y - ref| <= 2e-3 * max(|ref|, rms(ref)).  Reduced shapes are compared in full; the large
workloads are compared on sampled rows that the oracle computes one by one.
"""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import moqe_oracle as oc
from tests import oracle_blocks as ob

pytestmark = pytest.mark.gpu
K_MLP = wl.configs.KIND_SILU_MLP


def _forward_gpu(cfg, blk, bits):
    from paper_2508_09204_amd import binding as mq
    from tests import gpu_blocks as gb
    dblk = gb.block_dev(blk)
    x = gb.bf16_dev(bits.reshape(cfg.M, cfg.D))
    n_out = cfg.D if cfg.kind == K_MLP else cfg.F
    y = torch.full((cfg.M, n_out), float("nan"), dtype=torch.float32, device=gb.DEV)
    aux = gb.new_aux(cfg.S, cfg.K, cfg.M, cfg.F if cfg.kind == K_MLP else 0)
    mq.moqe_forward(dblk, x, cfg.S, cfg.T, y, aux)
    torch.cuda.synchronize()
    return y.cpu().numpy().reshape(cfg.S, cfg.T, n_out), aux


def _check_routing(cfg, aux, ref_idx):
    assert np.array_equal(aux.expert_idx.cpu().numpy(), ref_idx)
    counts, offsets, perm, inv = oc.bucket(ref_idx, cfg.K)
    assert np.array_equal(aux.counts.cpu().numpy(), counts)
    assert np.array_equal(aux.offsets.cpu().numpy(), offsets)
    assert np.array_equal(aux.perm.cpu().numpy(), perm)
    assert np.array_equal(aux.inv_perm.cpu().numpy(), inv)
    return perm, inv


def _h_step(h_ref):
    """Allowed |H_gpu - H_oracle|: one bfloat16 step of the value, or, where gate or up nearly cancel
    to zero, the absolute error of an fp32 accumulation (1e-4 of the tensor's rms is ten times that)."""
    rms = float(np.sqrt(np.mean(h_ref * h_ref)))
    return np.maximum(np.abs(h_ref) * 2.0 ** -7, 1e-4 * rms)


def _check_mlp_stages(cfg, blk, x64, aux, y, ref_idx, rows=None):
    """Stage-wise check of the MLP: H against the oracle's H (one bf16 step at most, rarely), and the
    second GEMM against the oracle applied to the H the GPU actually produced.  This keeps the check
    exact where a bf16 rounding decision of H legitimately differs between fp32 and fp64 arithmetic
    (it matters for the W8A8 expert, whose row scale follows the largest |H|)."""
    from tests import gpu_blocks as gb
    _, inv = oc.bucket(ref_idx, cfg.K)[2:]
    h_gpu = gb.bf16_tensor_to_f64(aux.h).reshape(cfg.S, cfg.T, cfg.F)[inv]      # caller order
    trows = list(range(cfg.T)) if rows is None else list(rows)
    worst_h, worst_y = 0.0, 0.0
    for s in range(cfg.S):
        e = int(ref_idx[s])
        xs = x64[s][trows]
        _, h_ref = oc.silu_mlp(xs, blk.w0[e], blk.w1[e], blk.w2[e])
        hg = h_gpu[s][trows]
        assert np.all(np.abs(hg - h_ref) <= _h_step(h_ref)), (s, e)
        worst_h = max(worst_h, float(np.mean(hg != h_ref)))
        y_ref = oc.qlinear(hg, blk.w2[e])
        ok, worst = ob.tolerance_ok(y[s][trows], y_ref)
        assert ok, (s, e, worst)
        worst_y = max(worst_y, worst)
    assert worst_h < 0.02          # only a small fraction of H values may sit on the other side of a tie
    return worst_y


SMALL = {
    "linear": dict(base="toy_linear", S=21, T=5, D=384, F=80),
    "mlp": dict(base="llama7b_mlp_decode", S=37, T=1, D=256, F=384, router_hidden=32),
    "mlp_prefill": dict(base="llama7b_mlp_prefill", S=6, T=45, D=256, F=384, router_hidden=32),
    "mlp8": dict(base="qwen_mlp_skew", S=40, T=9, D=384, F=640, router_hidden=32),
    "conv": dict(base="resnet50_conv", S=9, T=30, D=128, F=48, img_h=5, img_w=6, router_hidden=16),
}


@pytest.mark.parametrize("which", list(SMALL))
def test_forward_reduced_shapes_full_compare(which):
    kw = dict(SMALL[which])
    cfg = wl.scaled(wl.get_config(kw.pop("base")), **kw)
    blk = ob.make_block(cfg)
    bits, x64 = ob.activations_f64(cfg)
    y_ref, ref_idx, ref_logits = oc.forward(blk, x64)
    assert len(set(ref_idx.tolist())) > 1
    y, aux = _forward_gpu(cfg, blk, bits)
    _check_routing(cfg, aux, ref_idx)
    if cfg.kind == K_MLP:
        _check_mlp_stages(cfg, blk, x64, aux, y, ref_idx)
        a8 = [e for e in range(cfg.K) if blk.w0[e].act_mode]
        keep = ~np.isin(ref_idx, a8)
        ok, worst = ob.tolerance_ok(y[keep], y_ref[keep])            # end to end, experts with bf16 activations
        assert ok, worst
    else:
        ok, worst = ob.tolerance_ok(y, y_ref)
        assert ok, worst


def test_forward_toy_linear_full_size():
    cfg = wl.get_config("toy_linear")
    blk = ob.make_block(cfg)
    bits, x64 = ob.activations_f64(cfg)
    y_ref, ref_idx, _ = oc.forward(blk, x64)
    y, aux = _forward_gpu(cfg, blk, bits)
    _check_routing(cfg, aux, ref_idx)
    ok, worst = ob.tolerance_ok(y, y_ref)
    assert ok, worst


def test_forward_resnet_conv_full_size():
    cfg = wl.get_config("resnet50_conv")
    blk = ob.make_block(cfg)
    bits, x64 = ob.activations_f64(cfg)
    y_ref, ref_idx, _ = oc.forward(blk, x64)
    y, aux = _forward_gpu(cfg, blk, bits)
    _check_routing(cfg, aux, ref_idx)
    ok, worst = ob.tolerance_ok(y, y_ref)
    assert ok, worst


@pytest.mark.timeout(900)
def test_forward_llama_decode_full_size():
    cfg = wl.get_config("llama7b_mlp_decode")
    blk = ob.make_block(cfg)
    bits, x64 = ob.activations_f64(cfg)
    ref_idx, _, _ = oc.route(x64, blk.router)
    y, aux = _forward_gpu(cfg, blk, bits)
    _check_routing(cfg, aux, ref_idx)
    _check_mlp_stages(cfg, blk, x64, aux, y, ref_idx)
    y_ref, _, _ = oc.forward(blk, x64)
    ok, worst = ob.tolerance_ok(y, y_ref)
    assert ok, worst


def _sampled_rows(T):
    """First 8 and last 8 token rows of a sequence plus three interior ones: with 64-row tiles that start at
    multiples of 64 these land in every 16-row block of a tile (positions 0-7, 17, 40, 23 + T/2 and 56-63)."""
    rows = list(range(8)) + [17, 40, T // 2 + 23] + list(range(T - 8, T))
    return sorted(set(r for r in rows if 0 <= r < T))


@pytest.mark.timeout(1500)
@pytest.mark.parametrize("name", ["llama7b_mlp_prefill", "qwen_mlp_skew"])
def test_forward_large_workloads_sampled_rows(name):
    """Full-size launch; the oracle computes nineteen token rows of every sequence (all columns)."""
    cfg = wl.get_config(name)
    blk = ob.make_block(cfg)
    bits, x64 = ob.activations_f64(cfg)
    ref_idx, _, _ = oc.route(x64, blk.router)
    y, aux = _forward_gpu(cfg, blk, bits)
    _check_routing(cfg, aux, ref_idx)
    assert np.all(np.isfinite(y))
    rows = _sampled_rows(cfg.T)
    order = np.argsort(ref_idx, kind="stable")          # visit samples expert by expert to bound host memory
    from tests import gpu_blocks as gb
    _, inv = oc.bucket(ref_idx, cfg.K)[2:]
    h_gpu_t = aux.h.view(cfg.S, cfg.T, cfg.F)
    last_e = -1
    for s in order:
        e = int(ref_idx[s])
        if e != last_e and last_e >= 0:
            for m in (blk.w0[last_e], blk.w1[last_e], blk.w2[last_e]):
                m.release()
        last_e = e
        xs = x64[s][rows]
        _, h_ref = oc.silu_mlp(xs, blk.w0[e], blk.w1[e], blk.w2[e])
        hg = gb.bf16_tensor_to_f64(h_gpu_t[int(inv[s])][rows])
        assert np.all(np.abs(hg - h_ref) <= _h_step(h_ref)), (s, e)
        assert np.mean(hg != h_ref) < 0.02
        y_ref = oc.qlinear(hg, blk.w2[e])
        ok, worst = ob.tolerance_ok(y[s][rows], y_ref)
        assert ok, (s, e, worst)
        if blk.w0[e].act_mode == 0:
            # End to end against the oracle's own H.  The two sides may round a few H values to
            # neighbouring bfloat16 numbers (checked and counted above); what such a difference adds to
            # an output is at most sum_f |w2[n, f]| * |dH_f|, and a single flipped large H value can by
            # itself exceed 2e-3 of the output's rms, so that bound is granted on top of the tolerance.
            y_e2e = oc.qlinear(h_ref, blk.w2[e])
            flip_allowance = np.abs(hg - h_ref) @ np.abs(oc._dequant_memo(blk.w2[e])).T
            rms = float(np.sqrt(np.mean(y_e2e * y_e2e)))
            bound = 2e-3 * np.maximum(np.abs(y_e2e), rms) + flip_allowance
            assert np.all(np.abs(y[s][rows] - y_e2e) <= bound), (s, e)


@pytest.mark.parametrize("S,hw", [(1, (14, 14)), (4, (14, 14)), (1, (5, 6)), (4, (5, 6))])
@pytest.mark.parametrize("forced", [0, 1, 2, 3, None])
def test_forward_conv_few_images(S, hw, forced):
    """One image per request is the serving mode of Section 4.4: batches of one and four images, every one
    of the conv workload's four formats (the router is biased to one expert; None = its own routing)."""
    base = wl.get_config("resnet50_conv")
    cfg = wl.scaled(base, S=S, T=hw[0] * hw[1], img_h=hw[0], img_w=hw[1])
    blk = ob.make_block(cfg)
    if forced is not None:
        blk.router.b2 = blk.router.b2.copy()
        blk.router.b2[forced] = 1e4
    bits, x64 = ob.activations_f64(cfg)
    y_ref, ref_idx, _ = oc.forward(blk, x64)
    if forced is not None:
        assert np.all(ref_idx == forced)
    y, aux = _forward_gpu(cfg, blk, bits)
    _check_routing(cfg, aux, ref_idx)
    ok, worst = ob.tolerance_ok(y, y_ref)
    assert ok, worst
    assert worst < 0.05


def test_forward_replays_from_a_captured_graph():
    """moqe_forward enqueues only kernels on the caller's stream (no allocation, no memset, no
    synchronisation), so after one eager call it can be captured into a graph; every replay, with eager
    work and synchronisations in between, must reproduce the eager result bit for bit."""
    from paper_2508_09204_amd import binding as mq
    from tests import gpu_blocks as gb
    kw = dict(SMALL["mlp_prefill"])
    cfg = wl.scaled(wl.get_config(kw.pop("base")), **kw)
    blk = ob.make_block(cfg)
    bits, _ = ob.activations_f64(cfg)
    dblk = gb.block_dev(blk)
    x = gb.bf16_dev(bits.reshape(cfg.M, cfg.D))
    y_eager = torch.empty((cfg.M, cfg.D), dtype=torch.float32, device=gb.DEV)
    y_graph = torch.full((cfg.M, cfg.D), float("nan"), dtype=torch.float32, device=gb.DEV)
    call_e = mq.ForwardCall(dblk, x, cfg.S, cfg.T, y_eager, mq.Aux())
    call_g = mq.ForwardCall(dblk, x, cfg.S, cfg.T, y_graph, mq.Aux())
    call_e(torch.cuda.current_stream().cuda_stream)                   # also does the one-time kernel set-up
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        call_g(torch.cuda.current_stream().cuda_stream)
    for rep in range(3):
        y_graph.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        call_e(torch.cuda.current_stream().cuda_stream)               # eager work between the replays
        torch.cuda.synchronize()
        assert torch.equal(y_graph, y_eager), rep


@pytest.mark.parametrize("S,hidden", [(300, 64), (256, 64), (260, 60), (1000, 16), (40, 500)])
def test_forward_router_batch_sizes_around_the_fused_tail_limits(S, hidden):
    """Batches around the capacity of the fused logits + arg-max + bucket work-group (S * hidden floats of features,
    S * K pairs): routing arrays bit-exact and outputs within tolerance on either side of each limit."""
    cfg = wl.scaled(wl.get_config("toy_linear"), S=S, T=2, D=128, F=32, router_hidden=hidden)
    blk = ob.make_block(cfg)
    bits, x64 = ob.activations_f64(cfg)
    y_ref, ref_idx, _ = oc.forward(blk, x64)
    y, aux = _forward_gpu(cfg, blk, bits)
    _check_routing(cfg, aux, ref_idx)
    ok, worst = ob.tolerance_ok(y, y_ref)
    assert ok, worst


@pytest.mark.parametrize("S,T", [(64, 1), (37, 2), (5, 20), (1, 7)])
def test_forward_small_batch_equals_the_separate_stages_bit_for_bit(S, T):
    """Batches of at most 64 samples are bucketed inside the first grouped launch; the same block through the separate
    entry points (route, bucket kernel, two grouped launches reading the bucket arrays from memory) must give the very
    same bits: routing arrays, H and Y."""
    from paper_2508_09204_amd import binding as mq
    from tests import gpu_blocks as gb
    cfg = wl.scaled(wl.get_config("llama7b_mlp_decode"), S=S, T=T, D=256, F=384, router_hidden=32)
    blk = ob.make_block(cfg)
    bits, _ = ob.activations_f64(cfg)
    dblk = gb.block_dev(blk)
    x = gb.bf16_dev(bits.reshape(cfg.M, cfg.D))
    y = torch.full((cfg.M, cfg.D), float("nan"), dtype=torch.float32, device=gb.DEV)
    aux = gb.new_aux(cfg.S, cfg.K, cfg.M, cfg.F)
    mq.moqe_forward(dblk, x, cfg.S, cfg.T, y, aux)
    # the stages one by one
    idx = torch.full((S,), -1, dtype=torch.int32, device=gb.DEV)
    ws = torch.empty(mq.moqe_route_workspace_bytes(S, T, dblk.router), dtype=torch.uint8, device=gb.DEV)
    mq.moqe_route(x, S, T, dblk.router, idx, None, ws)
    counts = torch.zeros(cfg.K, dtype=torch.int32, device=gb.DEV)
    offsets = torch.zeros(cfg.K + 1, dtype=torch.int32, device=gb.DEV)
    perm = torch.zeros(S, dtype=torch.int32, device=gb.DEV)
    inv = torch.zeros(S, dtype=torch.int32, device=gb.DEV)
    mq.moqe_bucket(idx, S, cfg.K, counts, offsets, perm, inv)
    y2 = torch.full((cfg.M, cfg.D), float("nan"), dtype=torch.float32, device=gb.DEV)
    mq.moqe_grouped_qgemm(aux.h, offsets, perm, S, T, dblk.w2, y2, mq.SCATTER_OUTPUT | mq.INPUT_IN_BUCKET_ORDER)
    y3 = torch.full((cfg.M, cfg.D), float("nan"), dtype=torch.float32, device=gb.DEV)
    mq.moqe_forward_routed(dblk, idx, x, S, T, y3)
    torch.cuda.synchronize()
    for a, b in ((aux.expert_idx, idx), (aux.counts, counts), (aux.offsets, offsets), (aux.perm, perm), (aux.inv_perm, inv)):
        assert torch.equal(a, b)
    assert torch.equal(y.view(torch.int32), y2.view(torch.int32))        # the down launch from memory-resident bucket arrays
    assert torch.equal(y.view(torch.int32), y3.view(torch.int32))        # the whole block on the given experts


@pytest.mark.parametrize("which", ["linear", "mlp", "mlp_prefill", "conv"])
def test_forward_bf16_output_is_the_fp32_output_rounded_once(which):
    """moqe_block.y_bf16: the same block with bf16 results must give exactly the fp32 results rounded to nearest even
    (the rounding is the last step of the same arithmetic), on the streaming and on the tiled kernel."""
    from paper_2508_09204_amd import binding as mq
    from tests import gpu_blocks as gb
    kw = dict(SMALL[which])
    cfg = wl.scaled(wl.get_config(kw.pop("base")), **kw)
    blk = ob.make_block(cfg)
    bits, _ = ob.activations_f64(cfg)
    x = gb.bf16_dev(bits.reshape(cfg.M, cfg.D))
    n_out = cfg.D if cfg.kind == K_MLP else cfg.F
    d32 = gb.block_dev(blk)
    y32 = torch.full((cfg.M, n_out), float("nan"), dtype=torch.float32, device=gb.DEV)
    mq.moqe_forward(d32, x, cfg.S, cfg.T, y32)
    d16 = gb.block_dev(blk)
    d16.y_bf16 = 1
    y16 = torch.full((cfg.M, n_out), float("nan"), dtype=torch.bfloat16, device=gb.DEV)
    mq.moqe_forward(d16, x, cfg.S, cfg.T, y16)
    torch.cuda.synchronize()
    assert torch.equal(y16.view(torch.int16), y32.to(torch.bfloat16).view(torch.int16))
    assert bool(torch.isfinite(y32).all())


_SPECS = [wl.configs.ExpertSpec(8, 0, True), wl.configs.ExpertSpec(8, 0, True, 1.0, 1), wl.configs.ExpertSpec(6, 0, True),
          wl.configs.ExpertSpec(4, 0, True), wl.configs.ExpertSpec(4, 64, False), wl.configs.ExpertSpec(4, 128, False, 0.9),
          wl.configs.ExpertSpec(3, 64, False), wl.configs.ExpertSpec(3, 128, False)]


@pytest.mark.parametrize("seed", range(12))
def test_forward_random_blocks(seed):
    """Seeded random MLP and linear blocks (sizes, formats, router with or without a hidden layer, rows per sample):
    routing and bucketing bit for bit, outputs stage by stage as for the named workloads."""
    rng = np.random.default_rng(500 + seed)
    mlp = seed % 3 != 0
    K = int(rng.integers(2, 7))
    T = int(rng.choice([1, 1, 2, 4, 9, 36]))
    S = int(rng.integers(2, max(3, 150 // T)))
    D = 128 * int(rng.integers(1, 5))
    F = 128 * int(rng.integers(1, 5)) if mlp else 16 * int(rng.integers(1, 9))
    experts = tuple(_SPECS[int(i)] for i in rng.integers(0, len(_SPECS), K))
    base = wl.get_config("llama7b_mlp_decode" if mlp else "toy_linear")
    cfg = wl.scaled(base, S=S, T=T, D=D, F=F, experts=experts, router_hidden=int(rng.choice([0, 16, 48])),
                    router_w_std=0.05, router_bias=(), seed=900 + seed)
    blk = ob.make_block(cfg)
    bits, x64 = ob.activations_f64(cfg)
    y_ref, ref_idx, _ = oc.forward(blk, x64)
    y, aux = _forward_gpu(cfg, blk, bits)
    _check_routing(cfg, aux, ref_idx)
    if mlp:
        _check_mlp_stages(cfg, blk, x64, aux, y, ref_idx)
    else:
        ok, worst = ob.tolerance_ok(y, y_ref)
        assert ok, (worst, K, S, T, D, F)
