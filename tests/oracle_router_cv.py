"""Builds the oracle's CV router from the generator's parameter dictionary (shared by CPU and GPU tests)."""
from oracle import router_cv_oracle as rc


def _bn(p, prefix):
    return rc.BatchNorm(p[prefix + "_g"], p[prefix + "_o"], p[prefix + "_m"], p[prefix + "_v"])


def make(p, n_mlp, strides, n_heads):
    stages = []
    for i, st in enumerate(strides):
        has_short = ("st%d_s" % i) in p
        stages.append(rc.Stage(p["st%d_a" % i], _bn(p, "st%d_abn" % i), p["st%d_b" % i], _bn(p, "st%d_bbn" % i),
                               p["st%d_se1" % i], p["st%d_se1b" % i], p["st%d_se2" % i], p["st%d_se2b" % i],
                               p["st%d_s" % i] if has_short else None, _bn(p, "st%d_sbn" % i) if has_short else None, st))
    return rc.CvRouter([p["mlp%d_w" % i] for i in range(n_mlp)], [p["mlp%d_b" % i] for i in range(n_mlp)],
                       [_bn(p, "mlp%d_bn" % i) for i in range(n_mlp)], stages, p["wqkv"], p["bqkv"], p["wo"], p["bo"],
                       p["w_out"], p["b_out"], n_heads)
