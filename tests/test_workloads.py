"""The synthetic workloads: determinism, shapes, and the routing structure the configs promise (CPU only)."""
import numpy as np
import pytest

import workloads as wl
from oracle import moqe_oracle as oc
from tests import oracle_blocks as ob


def test_generators_are_deterministic_and_bf16():
    cfg = wl.get_config("toy_linear")
    a, b = wl.make_activations(cfg), wl.make_activations(cfg)
    assert a.dtype == np.uint16 and a.shape == (32, 16, 256) and np.array_equal(a, b)
    w = wl.make_fp_weights(cfg)["w0"]
    assert w.shape == (256, 256) and abs(float(w.std()) - 0.02) < 1e-3
    x = wl.bf16_bits_to_f32(a)
    assert abs(float(x.std()) - 1.0) < 0.02
    assert np.array_equal(wl.f32_to_bf16_bits(x), a)
    assert np.array_equal(x.astype(np.float64), oc.bf16_bits_to_f64(a))


def test_config_shapes():
    c = wl.CONFIGS
    assert [v.index for v in c.values()] == [0, 1, 2, 3, 4]
    assert c["llama7b_mlp_decode"].M == 64 and c["llama7b_mlp_prefill"].M == 8192
    assert c["qwen_mlp_skew"].K == 8 and c["qwen_mlp_skew"].M == 32768
    assert c["resnet50_conv"].matrices() == {"w0": (256, 2304)} and c["resnet50_conv"].T == 196
    assert sum(e.act_mode for e in c["qwen_mlp_skew"].experts) == 1


@pytest.mark.parametrize("name", ["toy_linear", "llama7b_mlp_decode", "llama7b_mlp_prefill", "qwen_mlp_skew",
                                  "resnet50_conv"])
def test_routing_structure_and_margins(name):
    """Every expert is used (except under the deliberate skew) and no sample sits near a tie, so fp32
    summation order on the GPU cannot change an index."""
    cfg = wl.get_config(name)
    x = oc.bf16_bits_to_f64(wl.make_activations(cfg))
    idx, logits, margin = oc.route(x, ob.make_router(cfg))
    hist = np.bincount(idx, minlength=cfg.K)
    assert hist.sum() == cfg.S
    assert margin.min() > 1e-4 * np.abs(logits).max(), (margin.min(), np.abs(logits).max())
    if name == "qwen_mlp_skew":
        assert abs(hist[0] / cfg.S - 0.60) <= 0.02
        assert np.all(hist > 0)
    else:
        assert np.all(hist > 0)
        assert hist.max() <= 0.5 * cfg.S
