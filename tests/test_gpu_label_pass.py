"""GPU parity of the router's training labels (moqe_label_pass, Section 3.3: every sample through all experts,
label = the expert of lowest prediction loss) against the oracle.

The logits are within 2e-3 * max(|ref|, rms(ref)) of the oracle's (the library's tolerance); a row's
cross-entropy moves by at most twice the largest change of its logits, so every loss must satisfy
|loss - ref| <= 4e-3 * max|logits of that (sample, expert)|.  A label is an integer decided by fp32 losses:
it must be the first arg-min of the losses the library itself wrote (bit-exact), and equal the oracle's
label wherever the oracle's margin between best and second best exceeds twice that tolerance."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import moqe_oracle as oc
from tests import oracle_blocks as ob

pytestmark = pytest.mark.gpu
K_MLP = wl.configs.KIND_SILU_MLP

CASES = {
    "linear": dict(base="toy_linear", S=21, T=5, D=384, F=80),
    "linear_few_rows": dict(base="toy_linear", S=3, T=2, D=256, F=208),
    "mlp_decode": dict(base="llama7b_mlp_decode", S=7, T=1, D=256, F=384, router_hidden=32),
    "mlp_decode_many": dict(base="llama7b_mlp_decode", S=37, T=1, D=256, F=384, router_hidden=32),
    "mlp_prefill": dict(base="llama7b_mlp_prefill", S=6, T=45, D=256, F=384, router_hidden=32),
    "mlp8": dict(base="qwen_mlp_skew", S=10, T=9, D=384, F=640, router_hidden=32),
}


def _label_pass_gpu(cfg, blk, bits, targets):
    from paper_2508_09204_amd import binding as mq
    from tests import gpu_blocks as gb
    dblk = gb.block_dev(blk)
    x = gb.bf16_dev(bits.reshape(cfg.M, cfg.D))
    tg = gb.to_dev(targets.astype(np.int32))
    losses = torch.full((cfg.S, cfg.K), float("nan"), dtype=torch.float32, device=gb.DEV)
    labels = torch.full((cfg.S,), -1, dtype=torch.int32, device=gb.DEV)
    mq.moqe_label_pass(dblk, x, tg, cfg.S, cfg.T, losses, labels)
    torch.cuda.synchronize()
    return losses.cpu().numpy(), labels.cpu().numpy()


def _check(cfg, blk, x64, targets, losses, labels):
    ref_losses, ref_labels = oc.label_pass(blk, x64, targets)
    tol = np.zeros_like(ref_losses)
    for s in range(cfg.S):
        for j in range(cfg.K):
            tol[s, j] = 4e-3 * np.abs(oc.expert_forward(blk, j, x64[s])).max()
    err = np.abs(losses.astype(np.float64) - ref_losses)
    assert np.all(err <= tol), float((err / tol).max())
    first_min = np.array([int(np.flatnonzero(losses[s] == losses[s].min())[0]) for s in range(cfg.S)])
    assert np.array_equal(labels, first_min)
    for s in range(cfg.S):
        order = np.sort(ref_losses[s])
        margin = order[1] - order[0] if cfg.K > 1 else np.inf
        if margin > 2 * tol[s].max():
            assert labels[s] == ref_labels[s], (s, margin)
        else:
            assert ref_losses[s, labels[s]] - order[0] <= 2 * tol[s].max()
    return float((err / tol).max()), float(np.mean(labels == ref_labels))


@pytest.mark.parametrize("which", list(CASES))
def test_label_pass_matches_oracle(which):
    kw = dict(CASES[which])
    cfg = wl.scaled(wl.get_config(kw.pop("base")), **kw)
    blk = ob.make_block(cfg)
    bits, x64 = ob.activations_f64(cfg)
    n_out = cfg.D if cfg.kind == K_MLP else cfg.F
    targets = wl.make_targets(cfg, n_out)
    losses, labels = _label_pass_gpu(cfg, blk, bits, targets)
    worst, agree = _check(cfg, blk, x64, targets, losses, labels)
    assert agree >= 0.9, agree         # seeded inputs: nearly every sample has a clear winner


def test_label_pass_decisive_targets_and_ties():
    """Targets taken from expert 1's own predictions with large logits: the labels are mostly 1 and match the
    oracle; then two identical experts: every label is 0 (the lowest index of a tie)."""
    E = wl.configs.ExpertSpec
    cfg = wl.scaled(wl.get_config("toy_linear"), S=12, T=4, D=256, F=16, experts=(E(3, 64, False), E(8, 0, True), E(3, 64, False, 0.7)))
    blk = ob.make_block(cfg)
    for q in blk.w0:
        q.scale = (q.scale * np.float32(40.0)).astype(np.float32); q.release()
    bits, x64 = ob.activations_f64(cfg)
    targets = np.stack([np.argmax(oc.qlinear(x64[s], blk.w0[1]), axis=1) for s in range(cfg.S)]).astype(np.int32)
    losses, labels = _label_pass_gpu(cfg, blk, bits, targets)
    _check(cfg, blk, x64, targets, losses, labels)
    assert np.mean(labels == 1) >= 0.75

    cfg2 = wl.scaled(wl.get_config("toy_linear"), S=9, T=3, D=128, F=32, experts=(E(4, 64, False), E(4, 64, False)))
    blk2 = ob.make_block(cfg2)
    blk2.w0[1] = blk2.w0[0]
    bits2, x2 = ob.activations_f64(cfg2)
    t2 = wl.make_targets(cfg2, cfg2.F)
    losses2, labels2 = _label_pass_gpu(cfg2, blk2, bits2, t2)
    _check(cfg2, blk2, x2, t2, losses2, labels2)
    assert np.array_equal(losses2[:, 0], losses2[:, 1]) and np.all(labels2 == 0)


def test_label_pass_clamps_targets_and_empty_batch():
    from paper_2508_09204_amd import binding as mq
    from tests import gpu_blocks as gb
    cfg = wl.scaled(wl.get_config("toy_linear"), S=4, T=3, D=128, F=48)
    blk = ob.make_block(cfg)
    bits, x64 = ob.activations_f64(cfg)
    targets = wl.make_targets(cfg, cfg.F)
    wild = targets.copy()
    wild[0, 0], wild[1, 2] = -5, 10_000
    clamped = np.clip(wild, 0, cfg.F - 1)
    l_wild, lab_wild = _label_pass_gpu(cfg, blk, bits, wild)
    l_cl, lab_cl = _label_pass_gpu(cfg, blk, bits, clamped)
    assert np.array_equal(l_wild, l_cl) and np.array_equal(lab_wild, lab_cl)
    _check(cfg, blk, x64, clamped, l_cl, lab_cl)
    dblk = gb.block_dev(blk)
    mq.moqe_label_pass(dblk, gb.bf16_dev(bits.reshape(cfg.M, cfg.D)), gb.to_dev(targets), 0, cfg.T,
                       torch.empty(0, device=gb.DEV), torch.empty(0, dtype=torch.int32, device=gb.DEV),
                       torch.empty(256, dtype=torch.uint8, device=gb.DEV))
    torch.cuda.synchronize()


@pytest.mark.timeout(900)
def test_label_pass_llama_decode_full_size():
    """The decode workload at its full size (64 sequences x 1 token, 4096 -> 11008 -> 4096, 4 experts): every expert on
    every sequence, i.e. the grouped launches of the bench with four full buckets."""
    cfg = wl.get_config("llama7b_mlp_decode")
    blk = ob.make_block(cfg)
    bits, x64 = ob.activations_f64(cfg)
    targets = wl.make_targets(cfg, cfg.D)
    losses, labels = _label_pass_gpu(cfg, blk, bits, targets)
    worst, agree = _check(cfg, blk, x64, targets, losses, labels)
    assert len(set(labels.tolist())) > 1
