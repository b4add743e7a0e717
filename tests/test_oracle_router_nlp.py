"""Pins of the oracle's NLP router model (Section 3.2: Transformer encoder -> self-attention module -> MLP):
torch.nn's encoder layer and attention module with the same weights, scalar loops, closed forms, invariants."""
import math

import numpy as np
import torch

import workloads as wl
from oracle import moqe_oracle as oc
from oracle import router_nlp_oracle as rn
from tests import oracle_router_nlp as orn

D, DM, NH, DFF, HH, K = 48, 32, 4, 64, 24, 3


def _setup(T=7, S=3, seed=11):
    p = wl.make_nlp_router(D, DM, NH, DFF, HH, K, seed)
    r = orn.make(p, NH)
    x = oc.bf16_bits_to_f64(wl.make_token_activations(S, T, D, seed + 1))
    return p, r, x


def _t(a):
    return torch.from_numpy(np.asarray(a, dtype=np.float64))


def test_attention_matches_torch_multihead_attention():
    p, r, x = _setup()
    u = rn.linear(x[0], r.w_in, r.b_in, False)
    mha = torch.nn.MultiheadAttention(DM, NH, batch_first=True, dtype=torch.float64)
    with torch.no_grad():
        mha.in_proj_weight.copy_(_t(p["wqkv1"])); mha.in_proj_bias.copy_(_t(p["bqkv1"]))
        mha.out_proj.weight.copy_(_t(p["wo1"])); mha.out_proj.bias.copy_(_t(p["bo1"]))
        ref = mha(_t(u)[None], _t(u)[None], _t(u)[None], need_weights=False)[0][0].numpy()
    got = rn.attention(u, r.att1, NH, False)
    assert np.allclose(got, ref, rtol=1e-10, atol=1e-12)


def test_encoder_layer_matches_torch_transformer_encoder_layer():
    p, r, x = _setup()
    u = rn.linear(x[1], r.w_in, r.b_in, False)
    layer = torch.nn.TransformerEncoderLayer(DM, NH, dim_feedforward=DFF, dropout=0.0, activation="relu",
                                             layer_norm_eps=rn.LN_EPS, batch_first=True, norm_first=False, dtype=torch.float64)
    layer.eval()
    with torch.no_grad():
        layer.self_attn.in_proj_weight.copy_(_t(p["wqkv1"])); layer.self_attn.in_proj_bias.copy_(_t(p["bqkv1"]))
        layer.self_attn.out_proj.weight.copy_(_t(p["wo1"])); layer.self_attn.out_proj.bias.copy_(_t(p["bo1"]))
        layer.linear1.weight.copy_(_t(p["w_ff1"])); layer.linear1.bias.copy_(_t(p["b_ff1"]))
        layer.linear2.weight.copy_(_t(p["w_ff2"])); layer.linear2.bias.copy_(_t(p["b_ff2"]))
        layer.norm1.weight.copy_(_t(p["ln1_g"])); layer.norm1.bias.copy_(_t(p["ln1_b"]))
        layer.norm2.weight.copy_(_t(p["ln2_g"])); layer.norm2.bias.copy_(_t(p["ln2_b"]))
        ref = layer(_t(u)[None])[0].numpy()
    v = rn.layer_norm(u + rn.attention(u, r.att1, NH, False), r.ln1_g, r.ln1_b)
    hid = np.maximum(rn.linear(v, r.w_ff1, r.b_ff1, False), 0.0)
    got = rn.layer_norm(v + rn.linear(hid, r.w_ff2, r.b_ff2, False), r.ln2_g, r.ln2_b)
    assert np.allclose(got, ref, rtol=1e-10, atol=1e-12)


def test_whole_router_matches_a_torch_composition():
    """The three stages and the head chained as torch modules, end to end on the logits."""
    p, r, x = _setup(T=5, S=4)
    with torch.no_grad():
        enc = torch.nn.TransformerEncoderLayer(DM, NH, dim_feedforward=DFF, dropout=0.0, layer_norm_eps=rn.LN_EPS,
                                               batch_first=True, dtype=torch.float64).eval()
        sa = enc.self_attn
        sa.in_proj_weight.copy_(_t(p["wqkv1"])); sa.in_proj_bias.copy_(_t(p["bqkv1"])); sa.out_proj.weight.copy_(_t(p["wo1"])); sa.out_proj.bias.copy_(_t(p["bo1"]))
        enc.linear1.weight.copy_(_t(p["w_ff1"])); enc.linear1.bias.copy_(_t(p["b_ff1"])); enc.linear2.weight.copy_(_t(p["w_ff2"])); enc.linear2.bias.copy_(_t(p["b_ff2"]))
        enc.norm1.weight.copy_(_t(p["ln1_g"])); enc.norm1.bias.copy_(_t(p["ln1_b"])); enc.norm2.weight.copy_(_t(p["ln2_g"])); enc.norm2.bias.copy_(_t(p["ln2_b"]))
        m2 = torch.nn.MultiheadAttention(DM, NH, batch_first=True, dtype=torch.float64)
        m2.in_proj_weight.copy_(_t(p["wqkv2"])); m2.in_proj_bias.copy_(_t(p["bqkv2"])); m2.out_proj.weight.copy_(_t(p["wo2"])); m2.out_proj.bias.copy_(_t(p["bo2"]))
        u = _t(x) @ _t(p["w_in"]).T + _t(p["b_in"])
        w = enc(u)
        z = torch.nn.functional.layer_norm(w + m2(w, w, w, need_weights=False)[0], (DM,), _t(p["ln3_g"]), _t(p["ln3_b"]), rn.LN_EPS)
        pooled = z.mean(dim=1)
        ref = torch.relu(pooled @ _t(p["head_w1"]).T + _t(p["head_b1"])) @ _t(p["head_w2"]).T + _t(p["head_b2"])
    idx, logits, pooled_o = rn.route_nlp(x, r, round_operands=False)
    assert np.allclose(pooled_o, pooled.numpy(), rtol=1e-9, atol=1e-12)
    assert np.allclose(logits, ref.numpy(), rtol=1e-9, atol=1e-12)
    assert np.array_equal(idx, np.argmax(ref.numpy(), axis=1))


def test_one_attention_row_and_one_layer_norm_row_by_scalar_loops():
    p, r, x = _setup(T=4)
    u = rn.linear(x[0], r.w_in, r.b_in, False)
    dh = DM // NH
    qkv = [[math.fsum(u[t, k] * float(p["wqkv1"][j, k]) for k in range(DM)) + float(p["bqkv1"][j]) for j in range(3 * DM)] for t in range(4)]
    t0, h = 2, 1
    sc = [math.fsum(qkv[t0][h * dh + c] * qkv[j][DM + h * dh + c] for c in range(dh)) / math.sqrt(dh) for j in range(4)]
    mx = max(sc); e = [math.exp(v - mx) for v in sc]; den = math.fsum(e)
    head_out = [math.fsum(e[j] / den * qkv[j][2 * DM + h * dh + c] for j in range(4)) for c in range(dh)]
    # the oracle's concatenated heads before the output projection, recovered by undoing wo (solve) is awkward:
    # compare through a router whose output projection is the identity
    att = rn.Attention(p["wqkv1"], p["bqkv1"], np.eye(DM), np.zeros(DM))
    got = rn.attention(u, att, NH, False)[t0, h * dh:(h + 1) * dh]
    assert np.allclose(got, head_out, rtol=1e-11, atol=1e-13)
    row = u[1]
    mu = math.fsum(row) / DM
    var = math.fsum((v - mu) ** 2 for v in row) / DM
    ref = [(row[i] - mu) / math.sqrt(var + 1e-5) * float(p["ln1_g"][i]) + float(p["ln1_b"][i]) for i in range(DM)]
    assert np.allclose(rn.layer_norm(u, r.ln1_g, r.ln1_b)[1], ref, rtol=1e-12, atol=1e-13)


def test_single_token_attention_returns_the_projected_value():
    p, r, x = _setup(T=1)
    u = rn.linear(x[2], r.w_in, r.b_in, False)                       # [1, dm]
    v = u @ p["wqkv1"][2 * DM:].astype(np.float64).T + p["bqkv1"][2 * DM:]
    ref = v @ p["wo1"].astype(np.float64).T + p["bo1"]
    assert np.allclose(rn.attention(u, r.att1, NH, False), ref, rtol=1e-12, atol=1e-13)


def test_logits_do_not_depend_on_the_order_of_the_tokens_and_softmax_rows_sum_to_one():
    p, r, x = _setup(T=9, S=2)
    perm = np.random.default_rng(0).permutation(9)
    for ro in (False, True):
        _, l0, _ = rn.route_nlp(x, r, ro)
        _, l1, _ = rn.route_nlp(x[:, perm], r, ro)
        assert np.allclose(l0, l1, rtol=1e-9, atol=1e-11)
    z = np.random.default_rng(1).standard_normal((5, 11)) * 30
    assert np.allclose(rn.softmax_rows(z).sum(axis=1), 1.0, atol=1e-14)


def test_operand_rounding_is_bf16_of_both_operands_and_changes_little():
    p, r, x = _setup(T=6, S=3)
    xr = np.random.default_rng(2).standard_normal((4, DM))
    got = rn.linear(xr, p["wo1"], p["bo1"], True)
    ref = oc.bf16_round(xr) @ oc.bf16_round(p["wo1"].astype(np.float64)).T + p["bo1"]
    assert np.array_equal(got, ref)
    _, l_exact, _ = rn.route_nlp(x, r, False)
    _, l_round, _ = rn.route_nlp(x, r, True)
    assert np.abs(l_exact - l_round).max() < 0.05 * max(1.0, np.abs(l_exact).max())
    assert np.abs(l_exact - l_round).max() > 0.0
