"""Builds the oracle's NLP router from the generator's parameter dictionary (shared by CPU and GPU tests)."""
import numpy as np

from oracle import moqe_oracle as oc
from oracle import router_nlp_oracle as rn


def make(p, n_heads):
    a1 = rn.Attention(p["wqkv1"], p["bqkv1"], p["wo1"], p["bo1"])
    a2 = rn.Attention(p["wqkv2"], p["bqkv2"], p["wo2"], p["bo2"])
    head = oc.Router(p["head_w1"], p["head_b1"], p["head_w2"], p["head_b2"])
    return rn.NlpRouter(p["w_in"], p["b_in"], a1, p["ln1_g"], p["ln1_b"], p["w_ff1"], p["b_ff1"], p["w_ff2"], p["b_ff2"],
                        p["ln2_g"], p["ln2_b"], a2, p["ln3_g"], p["ln3_b"], head, n_heads)
