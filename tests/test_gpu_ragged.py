"""GPU parity: samples of different lengths (a sample's feature is the mean over its own rows; routing,
bucketing and the grouped GEMMs then work on rows)."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import moqe_oracle as oc
from tests import oracle_blocks as ob

pytestmark = pytest.mark.gpu


def _block(kind, D, F, K, hidden, seed):
    rng = np.random.default_rng(seed)
    specs = [(4, 128, False, 1.0, 0), (8, 0, True, 1.0, 0), (3, 64, False, 0.9, 0), (8, 0, True, 1.0, 1), (6, 0, True, 1.0, 0)][:K]
    q = lambda n, k: [oc.quantize((rng.standard_normal((n, k)) * 0.05).astype(np.float32), *sp) for sp in specs]
    if hidden:
        w1 = (rng.standard_normal((hidden, D)) * 0.1).astype(np.float32)
        w2 = (rng.standard_normal((K, hidden)) * 0.3).astype(np.float32)
        router = oc.Router(w1, (rng.standard_normal(hidden) * 0.05).astype(np.float32), w2, None)
    else:
        router = oc.Router(None, None, (rng.standard_normal((K, D)) * 0.3).astype(np.float32),
                           (rng.standard_normal(K) * 0.05).astype(np.float32))
    if kind == oc.KIND_LINEAR:
        # one weight set quantized K ways: every expert is a variant of the same layer
        w = (rng.standard_normal((F, D)) * 0.05).astype(np.float32)
        return oc.Block(kind, router, [oc.quantize(w, *sp) for sp in specs])
    wg, wu, wd = [(rng.standard_normal(sh) * 0.05).astype(np.float32) for sh in ((F, D), (F, D), (D, F))]
    return oc.Block(kind, router, [oc.quantize(wg, *sp) for sp in specs], [oc.quantize(wu, *sp) for sp in specs],
                    [oc.quantize(wd, *sp) for sp in specs])


def _run(blk, xs_bits, want_h=False):
    from paper_2508_09204_amd import binding as mq
    from tests import gpu_blocks as gb
    lens = [b.shape[0] for b in xs_bits]
    S, M, K = len(lens), int(sum(lens)), blk.n_experts
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    x = gb.bf16_dev(np.concatenate(xs_bits, axis=0))
    n_out = blk.w0[0].n if blk.kind == oc.KIND_LINEAR else blk.w2[0].n
    y = torch.full((M, n_out), float("nan"), dtype=torch.float32, device=gb.DEV)
    aux = mq.Aux(expert_idx=torch.empty(S, dtype=torch.int32, device=gb.DEV),
                 logits=torch.empty((S, K), dtype=torch.float32, device=gb.DEV),
                 perm=torch.empty(S, dtype=torch.int32, device=gb.DEV),
                 h=torch.empty((M, blk.w0[0].n), dtype=torch.bfloat16, device=gb.DEV) if want_h else None)
    mq.moqe_forward_ragged(gb.block_dev(blk), x, gb.to_dev(cu), S, M, y, aux)
    torch.cuda.synchronize()
    return y.cpu().numpy(), aux, cu


@pytest.mark.parametrize("kind,lens,hidden", [
    (oc.KIND_LINEAR, [1, 7, 3, 4, 2, 9, 1, 1, 5], 0),                 # few rows per expert: streaming kernel
    (oc.KIND_LINEAR, [60, 1, 131, 17, 40, 77, 3, 90], 16),            # many rows: tiled kernel
    (oc.KIND_SILU_MLP, [2, 5, 1, 8, 3, 3, 6], 16),
    (oc.KIND_SILU_MLP, [33, 150, 8, 64, 1, 97, 120, 45, 70, 12], 0),
])
def test_ragged_forward_matches_oracle(kind, lens, hidden):
    D, F, K = 256, 384, 5
    blk = _block(kind, D, F, K, hidden, len(lens))
    rng = np.random.default_rng(sum(lens))
    xs_bits = [wl.f32_to_bf16_bits(rng.standard_normal((t, D)).astype(np.float32)) for t in lens]
    xs = [oc.bf16_bits_to_f64(b) for b in xs_bits]
    idx_ref, logits_ref = oc.route_ragged(xs, blk.router)
    srt = np.sort(logits_ref, axis=1)
    assert (srt[:, -1] - srt[:, -2]).min() > 1e-4            # the routing decision is not a coin flip in fp32
    y, aux, cu = _run(blk, xs_bits, want_h=(kind == oc.KIND_SILU_MLP))
    assert np.array_equal(aux.expert_idx.cpu().numpy(), idx_ref)
    assert np.max(np.abs(aux.logits.cpu().numpy() - logits_ref)) <= 1e-5 * np.abs(logits_ref).max()
    assert np.all(np.isfinite(y))
    if kind == oc.KIND_LINEAR:
        for s, x in enumerate(xs):
            ok, worst = ob.tolerance_ok(y[cu[s]:cu[s + 1]], oc.qlinear(x, blk.w0[int(idx_ref[s])]))
            assert ok, (s, worst)
        return
    # MLP: stage-wise, as for the uniform path: H against the oracle's H (bf16 neighbours at most), the down
    # projection against the oracle applied to the H the GPU produced (rows of H are in bucket-row order)
    from tests import gpu_blocks as gb
    from tests.test_gpu_forward import _h_step
    perm = aux.perm.cpu().numpy()
    h_all = gb.bf16_tensor_to_f64(aux.h)
    pos = 0
    for j in range(len(lens)):
        s = int(perm[j]); e = int(idx_ref[s]); t = lens[s]
        hg = h_all[pos:pos + t]; pos += t
        _, h_ref = oc.silu_mlp(xs[s], blk.w0[e], blk.w1[e], blk.w2[e])
        assert np.all(np.abs(hg - h_ref) <= _h_step(h_ref)), (s, e)
        ok, worst = ob.tolerance_ok(y[cu[s]:cu[s + 1]], oc.qlinear(hg, blk.w2[e]))
        assert ok, (s, e, worst)


def test_expand_rows_matches_host_model():
    from paper_2508_09204_amd import binding as mq
    from tests import gpu_blocks as gb
    rng = np.random.default_rng(3)
    for S, K in [(1, 1), (7, 3), (300, 4), (1000, 16)]:
        lens = rng.integers(1, 40, S)
        cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        e = rng.integers(0, K, S).astype(np.int32)
        counts, offsets, perm, inv = oc.bucket(e, K)
        M = int(cu[-1])
        slot_rows = torch.empty(S + 1, dtype=torch.int32, device=gb.DEV)
        row_offsets = torch.empty(K + 1, dtype=torch.int32, device=gb.DEV)
        row_perm = torch.empty(M, dtype=torch.int32, device=gb.DEV)
        mq.moqe_expand_rows(gb.to_dev(cu), gb.to_dev(offsets), gb.to_dev(perm), S, K, slot_rows, row_offsets, row_perm)
        torch.cuda.synchronize()
        ref_rows = np.concatenate([np.arange(cu[s], cu[s + 1]) for s in perm])
        ref_slot = np.concatenate([[0], np.cumsum(lens[perm])])
        assert np.array_equal(row_perm.cpu().numpy(), ref_rows)
        assert np.array_equal(slot_rows.cpu().numpy(), ref_slot)
        assert np.array_equal(row_offsets.cpu().numpy(), ref_slot[offsets])
