"""Finds the router bias that skews the Qwen-style workload: about 60 % of sequences to expert 0.

Run once (python -m oracle.calibrate_skew_bias); the printed value is stored as the constant
QWEN_SKEW_BIAS0 of workloads/configs.py.  Calls only the oracle and the input generators.
"""
import numpy as np

import workloads as wl
from oracle import moqe_oracle as oc


def main(target=0.60):
    cfg = wl.scaled(wl.get_config("qwen_mlp_skew"), router_bias=())
    r = wl.make_router(cfg)
    x = oc.bf16_bits_to_f64(wl.make_activations(cfg))
    p = oc.pool(x)
    router = oc.Router(w1=r["w1"], b1=r["b1"], w2=r["w2"], b2=None)
    base = oc.router_logits(p, router)
    # sample s goes to expert 0 exactly when bias > t_s = max_{k>0} z_k - z_0; put the bias midway
    # between two neighbouring thresholds so that no sample sits on the decision boundary
    t = np.sort(base[:, 1:].max(axis=1) - base[:, 0])
    n0 = int(round(target * cfg.S))
    beta = float(np.float32(0.5 * (t[n0 - 1] + t[n0])))
    z = base.copy()
    z[:, 0] += beta
    idx = oc.argmax_first(z)
    print("QWEN_SKEW_BIAS0 =", repr(beta))
    print("fraction to expert 0:", np.mean(idx == 0), "histogram:", np.bincount(idx, minlength=cfg.K).tolist())
    print("logit abs max:", float(np.abs(base).max()))


if __name__ == "__main__":
    main()
