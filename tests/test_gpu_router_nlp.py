"""GPU parity of the NLP router model (moqe_route_nlp, Section 3.2: Transformer encoder -> self-attention module
-> MLP) against the oracle with the same bf16 operand rounding.

Logits: |gpu - ref| <= 2e-3 * max(1, max|ref|) (fp32 accumulation, fp32 exp and the rare bf16 rounding decision
that differs between an fp32 and an fp64 intermediate).  The selected expert is an integer decided by fp32 logits: it
must be the first arg-max of the logits the library wrote (bit-exact) and the oracle's expert wherever the oracle's
margin between the two largest logits exceeds twice that tolerance."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import moqe_oracle as oc
from oracle import router_nlp_oracle as rn
from tests import oracle_router_nlp as orn

pytestmark = pytest.mark.gpu

#         S   T    d    dm  heads d_ff head_h K
CASES = {
    "small_dh32": (5, 7, 192, 128, 4, 256, 32, 4),
    "one_token": (6, 1, 128, 128, 4, 128, 16, 3),
    "ragged_tiles_dh64": (2, 70, 128, 256, 4, 256, 64, 5),
    "dh16_many_heads": (3, 19, 64, 128, 8, 128, 32, 2),
    "dh128": (2, 33, 64, 256, 2, 128, 32, 4),
    "many_rows": (3, 200, 256, 128, 2, 256, 32, 4),
    "paper_size": (4, 37, 4096, 384, 6, 1536, 384, 4),
}


def _gpu_router(p, d, dm, heads, dff, hh, K):
    from paper_2508_09204_amd import binding as mq
    from tests import gpu_blocks as gb
    dev = {k: gb.to_dev(np.ascontiguousarray(v)) for k, v in p.items()}
    head = mq.Router(dev["head_w1"], dev["head_b1"], dev["head_w2"], dev["head_b2"], dm, hh, K)
    return mq.NlpRouter(dev, head, d, dm, heads, dff)


def _run(case, seed=21):
    from paper_2508_09204_amd import binding as mq
    from tests import gpu_blocks as gb
    S, T, d, dm, heads, dff, hh, K = CASES[case]
    p = wl.make_nlp_router(d, dm, heads, dff, hh, K, seed)
    bits = wl.make_token_activations(S, T, d, seed + 1)
    r = _gpu_router(p, d, dm, heads, dff, hh, K)
    x = gb.bf16_dev(bits.reshape(S * T, d))
    idx = torch.full((S,), -1, dtype=torch.int32, device=gb.DEV)
    logits = torch.full((S, K), float("nan"), dtype=torch.float32, device=gb.DEV)
    mq.moqe_route_nlp(x, S, T, r, idx, logits)
    torch.cuda.synchronize()
    ref_idx, ref_logits, _ = rn.route_nlp(oc.bf16_bits_to_f64(bits), orn.make(p, heads), round_operands=True)
    return idx.cpu().numpy(), logits.cpu().numpy(), ref_idx, ref_logits


@pytest.mark.parametrize("case", list(CASES))
def test_route_nlp_matches_oracle(case):
    idx, logits, ref_idx, ref_logits = _run(case)
    tol = 2e-3 * max(1.0, float(np.abs(ref_logits).max()))
    err = float(np.abs(logits.astype(np.float64) - ref_logits).max())
    assert err <= tol, (err, tol)
    first_max = np.array([int(np.flatnonzero(row == row.max())[0]) for row in logits])
    assert np.array_equal(idx, first_max)
    srt = np.sort(ref_logits, axis=1)
    clear = (srt[:, -1] - srt[:, -2]) > 2 * tol
    assert np.array_equal(idx[clear], ref_idx[clear])
    assert clear.mean() >= 0.5          # the seeded cases are not all near-ties


def test_route_nlp_is_deterministic_and_feeds_the_bucket():
    from paper_2508_09204_amd import binding as mq
    from tests import gpu_blocks as gb
    a = _run("small_dh32")
    b = _run("small_dh32")
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    S, K = CASES["small_dh32"][0], CASES["small_dh32"][7]
    idx = gb.to_dev(a[0].astype(np.int32))
    counts = torch.zeros(K, dtype=torch.int32, device=gb.DEV)
    offsets = torch.zeros(K + 1, dtype=torch.int32, device=gb.DEV)
    perm = torch.zeros(S, dtype=torch.int32, device=gb.DEV)
    inv = torch.zeros(S, dtype=torch.int32, device=gb.DEV)
    mq.moqe_bucket(idx, S, K, counts, offsets, perm, inv)
    torch.cuda.synchronize()
    c, o, pm, iv = oc.bucket(a[0], K)
    assert np.array_equal(counts.cpu().numpy(), c) and np.array_equal(perm.cpu().numpy(), pm)


@pytest.mark.parametrize("S,T", [(11, 6), (5, 70)])         # a batch that buckets itself in the first launch / one that does not
def test_router_model_drives_the_routed_mlp_block(S, T):
    """The paper's router in front of the routed experts: moqe_route_nlp -> moqe_forward_routed (bucketing, grouped
    gate/up GEMM with the SiLU gate, grouped down GEMM, scatter).  The experts the GPU router chose are checked against the
    oracle's router, the block's output against the oracle's block run on those experts."""
    from paper_2508_09204_amd import binding as mq
    from tests import gpu_blocks as gb
    from tests import oracle_blocks as ob
    cfg = wl.scaled(wl.get_config("llama7b_mlp_decode"), S=S, T=T, D=256, F=384, router_hidden=32)
    blk = ob.make_block(cfg)
    dm, heads, dff, hh = 128, 4, 256, 32
    p = wl.make_nlp_router(cfg.D, dm, heads, dff, hh, cfg.K, 31)
    bits = wl.make_token_activations(cfg.S, cfg.T, cfg.D, 32)
    x64 = oc.bf16_bits_to_f64(bits)
    r = _gpu_router(p, cfg.D, dm, heads, dff, hh, cfg.K)
    x = gb.bf16_dev(bits.reshape(cfg.M, cfg.D))
    idx = torch.full((cfg.S,), -1, dtype=torch.int32, device=gb.DEV)
    mq.moqe_route_nlp(x, cfg.S, cfg.T, r, idx)
    dblk = gb.block_dev(blk)
    y = torch.full((cfg.M, cfg.D), float("nan"), dtype=torch.float32, device=gb.DEV)
    aux = gb.new_aux(cfg.S, cfg.K, cfg.M, cfg.F)
    aux.expert_idx = None
    aux.logits = None
    mq.moqe_forward_routed(dblk, idx, x, cfg.S, cfg.T, y, aux)
    torch.cuda.synchronize()
    e = idx.cpu().numpy()
    assert len(set(e.tolist())) > 1
    ref_idx, _, _ = rn.route_nlp(x64, orn.make(p, heads), round_operands=True)
    assert np.mean(e == ref_idx) >= 0.8
    c, o, pm, iv = oc.bucket(e, cfg.K)
    assert np.array_equal(aux.counts.cpu().numpy(), c) and np.array_equal(aux.offsets.cpu().numpy(), o)
    assert np.array_equal(aux.perm.cpu().numpy(), pm) and np.array_equal(aux.inv_perm.cpu().numpy(), iv)
    # stage-wise, as for moqe_forward: H against the oracle's H, the down projection against the oracle's on the GPU's H
    from tests.test_gpu_forward import _check_mlp_stages
    _check_mlp_stages(cfg, blk, x64, aux, y.cpu().numpy().reshape(cfg.S, cfg.T, cfg.D), e)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("S,T", [(64, 1), (16, 512)])
def test_route_nlp_full_size_workload_shapes(S, T):
    """The 16 MB router at the decode and prefill batch shapes the bench times (d = 4096): all logits against the oracle."""
    from paper_2508_09204_amd import binding as mq
    from tests import gpu_blocks as gb
    d, dm, heads, dff, hh, K = 4096, 384, 6, 1536, 384, 4
    p = wl.make_nlp_router(d, dm, heads, dff, hh, K, 51)
    bits = wl.make_token_activations(S, T, d, 52)
    r = _gpu_router(p, d, dm, heads, dff, hh, K)
    x = gb.bf16_dev(bits.reshape(S * T, d))
    idx = torch.full((S,), -1, dtype=torch.int32, device=gb.DEV)
    logits = torch.full((S, K), float("nan"), dtype=torch.float32, device=gb.DEV)
    mq.moqe_route_nlp(x, S, T, r, idx, logits)
    torch.cuda.synchronize()
    ref_idx, ref_logits, _ = rn.route_nlp(oc.bf16_bits_to_f64(bits), orn.make(p, heads), round_operands=True)
    tol = 2e-3 * max(1.0, float(np.abs(ref_logits).max()))
    lg = logits.cpu().numpy()
    assert float(np.abs(lg - ref_logits).max()) <= tol
    srt = np.sort(ref_logits, axis=1)
    clear = (srt[:, -1] - srt[:, -2]) > 2 * tol
    assert np.array_equal(idx.cpu().numpy()[clear], ref_idx[clear]) and clear.mean() >= 0.5
