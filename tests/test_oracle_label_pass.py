"""Pins of the oracle's label pass (Section 3.3: every sample through all experts, the expert with the lowest
prediction loss is the router's training label): the cross-entropy against a library routine and scalar
loops, closed forms, shift invariance, and the argmin rule on constructed cases."""
import math

import numpy as np
import torch

import workloads as wl
from oracle import moqe_oracle as oc
from tests import oracle_blocks as ob


def test_cross_entropy_matches_torch_and_scalar_loops():
    rng = np.random.default_rng(1)
    y = rng.standard_normal((7, 13)) * 3.0
    t = rng.integers(0, 13, 7)
    got = oc.cross_entropy_rows(y, t)
    ref = torch.nn.functional.cross_entropy(torch.from_numpy(y), torch.from_numpy(t), reduction="none").numpy()
    assert np.allclose(got, ref, rtol=1e-12, atol=1e-12)
    for r in range(7):
        den = math.fsum(math.exp(v) for v in y[r])
        assert abs(got[r] - (math.log(den) - y[r, t[r]])) < 1e-12


def test_cross_entropy_closed_forms():
    n = 11
    assert np.allclose(oc.cross_entropy_rows(np.zeros((3, n)), [0, 5, 10]), math.log(n))       # uniform logits
    y = np.full((1, n), -50.0); y[0, 4] = 50.0
    assert oc.cross_entropy_rows(y, [4])[0] < 1e-30                                             # certain and right
    assert abs(oc.cross_entropy_rows(y, [3])[0] - 100.0) < 1e-9                                 # certain and wrong
    y = np.array([[1.0, 2.0, 3.0]])
    assert np.allclose(oc.cross_entropy_rows(y + 1000.0, [1]), oc.cross_entropy_rows(y, [1]))   # shift invariance
    assert np.allclose(oc.cross_entropy_rows(y, [2]), math.log(math.e ** 1 + math.e ** 2 + math.e ** 3) - 3.0)


def _toy(K_specs, S=5, T=3, D=128, F=32, seed=3):
    cfg = wl.scaled(wl.get_config("toy_linear"), S=S, T=T, D=D, F=F, experts=tuple(K_specs))
    blk = ob.make_block(cfg)
    _, x64 = ob.activations_f64(cfg)
    return cfg, blk, x64


def test_label_pass_is_loss_argmin_over_all_experts():
    E = wl.configs.ExpertSpec
    cfg, blk, x64 = _toy([E(8, 0, True), E(4, 64, False), E(3, 64, False)])
    targets = wl.make_targets(cfg, cfg.F)
    losses, labels = oc.label_pass(blk, x64, targets)
    assert losses.shape == (cfg.S, cfg.K) and labels.shape == (cfg.S,)
    for s in range(cfg.S):
        for j in range(cfg.K):
            y = oc.qlinear(x64[s], blk.w0[j])                        # the single quantized model j on this sample
            ref = torch.nn.functional.cross_entropy(torch.from_numpy(y), torch.from_numpy(targets[s].astype(np.int64))).item()
            assert abs(losses[s, j] - ref) < 1e-10
        assert labels[s] == int(np.argmin(losses[s]))
    # the routed prediction of a router that follows the labels has, per sample, the lowest loss of all experts
    assert np.all(losses[np.arange(cfg.S), labels] == losses.min(axis=1))


def test_label_pass_ties_take_the_lowest_index_and_single_expert():
    E = wl.configs.ExpertSpec
    cfg, blk, x64 = _toy([E(4, 64, False), E(4, 64, False)], S=4)    # two identical experts: exact ties
    targets = wl.make_targets(cfg, cfg.F)
    losses, labels = oc.label_pass(blk, x64, targets)
    assert np.array_equal(losses[:, 0], losses[:, 1]) and np.all(labels == 0)
    cfg1, blk1, x1 = _toy([E(8, 0, True)], S=3)
    _, labels1 = oc.label_pass(blk1, x1, wl.make_targets(cfg1, cfg1.F))
    assert np.all(labels1 == 0)


def test_label_pass_prefers_the_expert_whose_prediction_is_the_target():
    """Targets taken from expert 1's own arg-max rows: its loss is the smallest wherever the experts disagree
    enough, so expert 1 is the label of most samples and never has the highest loss."""
    E = wl.configs.ExpertSpec
    cfg, blk, x64 = _toy([E(3, 64, False), E(8, 0, True), E(3, 64, False, 0.7)], S=12, T=4, D=256, F=16, seed=5)
    for q in blk.w0:                                                  # larger logits: predictions are decisive
        q.scale = (q.scale * np.float32(40.0)).astype(np.float32); q.release()
    targets = np.stack([np.argmax(oc.qlinear(x64[s], blk.w0[1]), axis=1) for s in range(cfg.S)]).astype(np.int32)
    losses, labels = oc.label_pass(blk, x64, targets)
    assert np.mean(labels == 1) >= 0.75
    assert np.all(np.argmax(losses, axis=1) != 1)
