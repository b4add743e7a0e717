"""GPU parity: router + top-1 selection, dispatch counts and the stable bucket permutation (bit-exact)."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import moqe_oracle as oc
from tests import oracle_blocks as ob

pytestmark = pytest.mark.gpu


def _route_gpu(bits, router, S, T, K):
    from paper_2508_09204_amd import binding as mq
    from tests import gpu_blocks as gb
    x = gb.bf16_dev(bits)
    idx = torch.full((S,), -1, dtype=torch.int32, device=gb.DEV)
    logits = torch.zeros((S, K), dtype=torch.float32, device=gb.DEV)
    mq.moqe_route(x, S, T, gb.router_dev(router, K), idx, logits)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), logits.cpu().numpy()


@pytest.mark.parametrize("name", ["toy_linear", "llama7b_mlp_decode", "llama7b_mlp_prefill", "qwen_mlp_skew",
                                  "resnet50_conv"])
def test_route_full_configs(name):
    cfg = wl.get_config(name)
    bits = wl.make_activations(cfg)
    router = ob.make_router(cfg)
    ref_idx, ref_logits, margin = oc.route(oc.bf16_bits_to_f64(bits), router)
    idx, logits = _route_gpu(bits, router, cfg.S, cfg.T, cfg.K)
    assert np.array_equal(idx, ref_idx)                                   # routing accuracy vs oracle = 100 %
    scale = np.abs(ref_logits).max()
    assert np.max(np.abs(logits - ref_logits)) <= 1e-5 * scale
    assert np.max(np.abs(logits - ref_logits)) < 0.1 * margin.min()


@pytest.mark.parametrize("S,T,D,H,K", [(1, 1, 128, 0, 1), (3, 7, 136, 12, 5), (70, 33, 264, 20, 16), (5, 200, 128, 8, 2),
                                       (3000, 1, 128, 16, 8), (2500, 2, 256, 0, 3)])
def test_route_ragged_shapes(S, T, D, H, K):
    rng = np.random.default_rng(S * 100 + T)
    bits = wl.f32_to_bf16_bits(rng.standard_normal((S, T, D)).astype(np.float32))
    r = oc.Router(w1=rng.standard_normal((H, D)).astype(np.float32) if H else None,
                  b1=rng.standard_normal(H).astype(np.float32) if H else None,
                  w2=rng.standard_normal((K, H if H else D)).astype(np.float32),
                  b2=rng.standard_normal(K).astype(np.float32))
    ref_idx, ref_logits, margin = oc.route(oc.bf16_bits_to_f64(bits), r)
    idx, logits = _route_gpu(bits, r, S, T, K)
    safe = margin > 1e-4 * np.abs(ref_logits).max()
    assert np.array_equal(idx[safe], ref_idx[safe])
    np.testing.assert_allclose(logits, ref_logits, rtol=0, atol=2e-5 * np.abs(ref_logits).max())


def test_route_exact_ties_take_lowest_index():
    rng = np.random.default_rng(9)
    S, T, D = 40, 3, 128
    bits = wl.f32_to_bf16_bits(rng.standard_normal((S, T, D)).astype(np.float32))
    w = rng.standard_normal((1, D)).astype(np.float32)
    r = oc.Router(w1=None, b1=None, w2=np.concatenate([w * 0.5, w, w, w]), b2=None)   # rows 1..3 identical
    ref_idx, _, _ = oc.route(oc.bf16_bits_to_f64(bits), r)
    idx, logits = _route_gpu(bits, r, S, T, 4)
    assert np.array_equal(idx, ref_idx)
    assert set(idx.tolist()) <= {0, 1}
    assert np.array_equal(logits[:, 1], logits[:, 2]) and np.array_equal(logits[:, 1], logits[:, 3])


def _bucket_gpu(e, K):
    from paper_2508_09204_amd import binding as mq
    from tests import gpu_blocks as gb
    S = len(e)
    i32 = dict(dtype=torch.int32, device=gb.DEV)
    counts, offsets = torch.full((K,), -7, **i32), torch.full((K + 1,), -7, **i32)
    perm, inv = torch.full((max(S, 1),), -7, **i32), torch.full((max(S, 1),), -7, **i32)
    mq.moqe_bucket(gb.to_dev(np.asarray(e, dtype=np.int32)) if S else None, S, K, counts, offsets, perm, inv)
    torch.cuda.synchronize()
    return counts.cpu().numpy(), offsets.cpu().numpy(), perm.cpu().numpy()[:S], inv.cpu().numpy()[:S]


@pytest.mark.parametrize("S,K,seed", [(1, 1, 0), (1, 4, 1), (64, 4, 2), (63, 3, 3), (65, 3, 4), (256, 8, 5), (257, 8, 6),
                                      (1000, 16, 7), (5000, 5, 8), (0, 4, 9), (200000, 16, 10)])
def test_bucket_matches_oracle_bit_exact(S, K, seed):
    e = np.random.default_rng(seed).integers(0, K, S)
    ref = oc.bucket(e, K)
    got = _bucket_gpu(e, K)
    for g, r in zip(got, ref):
        assert np.array_equal(g, r)


def test_bucket_degenerate_distributions():
    for e, K in [(np.full(300, 2), 4), (np.array([3, 3, 0, 0] * 40), 5), (np.arange(16).repeat(3), 16)]:
        ref = oc.bucket(e, K)
        got = _bucket_gpu(e, K)
        for g, r in zip(got, ref):
            assert np.array_equal(g, r)
    # repeated launches give identical results (no dependence on scheduling)
    e = np.random.default_rng(1).integers(0, 8, 777)
    a = _bucket_gpu(e, 8)
    for _ in range(3):
        b = _bucket_gpu(e, 8)
        assert all(np.array_equal(x, y) for x, y in zip(a, b))


def _balance_gpu(logits, counts, alpha):
    from paper_2508_09204_amd import binding as mq
    from tests import gpu_blocks as gb
    S, K = logits.shape
    out = torch.full((2 * K + 3,), float("nan"), dtype=torch.float32, device=gb.DEV)
    mq.moqe_balance_stats(gb.to_dev(logits.astype(np.float32)), gb.to_dev(counts.astype(np.int32)), S, K, alpha, out)
    torch.cuda.synchronize()
    o = out.cpu().numpy().astype(np.float64)
    return o[:K], o[K:2 * K], o[2 * K], o[2 * K + 1], o[2 * K + 2]


@pytest.mark.parametrize("S,K,seed", [(1, 1, 0), (64, 4, 1), (256, 3, 2), (5000, 16, 3), (300, 8, 4)])
def test_balance_stats_match_oracle(S, K, seed):
    """P_i, F_i, L_bal (Eq. 1-2), the usage spread and the dynamic weight, fp32 on the GPU against fp64."""
    rng = np.random.default_rng(seed)
    logits = (rng.standard_normal((S, K)) * 3.0).astype(np.float32)
    if seed == 4:
        logits[:, 2] += 50.0                       # everything to one expert: the degenerate dispatch
    idx = np.argmax(logits, axis=1)
    counts = np.bincount(idx, minlength=K)
    ref = oc.balance_stats(logits, idx, 0.02)
    got = _balance_gpu(logits, counts, 0.02)
    assert np.allclose(got[0], ref[0], rtol=2e-5, atol=1e-7)
    assert np.array_equal(got[1].astype(np.float32), (counts / S).astype(np.float32))
    for g, r in zip(got[2:], ref[2:]):
        assert np.isclose(g, r, rtol=2e-5, atol=1e-7)
    again = _balance_gpu(logits, counts, 0.02)
    assert all(np.array_equal(a, b) for a, b in zip(got, again))        # fixed summation order


def test_balance_stats_on_routed_workload():
    """From the logits and counts that the router and the bucket step leave on the device."""
    from paper_2508_09204_amd import binding as mq
    from tests import gpu_blocks as gb
    cfg = wl.get_config("qwen_mlp_skew")
    bits = wl.make_activations(cfg)
    router = ob.make_router(cfg)
    idx_ref, logits_ref, _ = oc.route(oc.bf16_bits_to_f64(bits), router)
    x = gb.bf16_dev(bits)
    idx = torch.empty(cfg.S, dtype=torch.int32, device=gb.DEV)
    logits = torch.empty((cfg.S, cfg.K), dtype=torch.float32, device=gb.DEV)
    mq.moqe_route(x, cfg.S, cfg.T, gb.router_dev(router, cfg.K), idx, logits)
    counts = torch.empty(cfg.K, dtype=torch.int32, device=gb.DEV)
    offsets = torch.empty(cfg.K + 1, dtype=torch.int32, device=gb.DEV)
    mq.moqe_bucket(idx, cfg.S, cfg.K, counts, offsets, None, None)
    out = torch.empty(2 * cfg.K + 3, dtype=torch.float32, device=gb.DEV)
    mq.moqe_balance_stats(logits, counts, cfg.S, cfg.K, 0.02, out)
    torch.cuda.synchronize()
    o = out.cpu().numpy().astype(np.float64)
    P, F, l, sig, a = oc.balance_stats(logits_ref, idx_ref, 0.02)
    K = cfg.K
    assert np.allclose(o[:K], P, rtol=1e-4) and np.allclose(o[K:2 * K], F)
    assert np.isclose(o[2 * K], l, rtol=1e-4) and np.isclose(o[2 * K + 1], sig, rtol=1e-5)
    assert np.isclose(o[2 * K + 2], a, rtol=1e-5)
    assert F[0] > 0.5                               # the skewed workload: expert 0 takes most sequences
