"""GPU parity: a stack of routed layers that is routed and bucketed ONCE.

The router selects the expert for the whole model (Section 3.1), so one bucket result drives every
quantized layer: the first grouped GEMM gathers the samples' rows through the permutation, the
activations then stay in bucket order (rounded to bfloat16 between layers, as the next layer's
input type requires), and only the last layer scatters back to the caller's order.
"""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import moqe_oracle as oc
from tests import oracle_blocks as ob

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("S,T", [(20, 3), (9, 41)])        # small buckets (streaming kernel) / large (tiled kernel)
def test_three_layer_stack_bucketed_once(S, T):
    from paper_2508_09204_amd import binding as mq
    from tests import gpu_blocks as gb
    rng = np.random.default_rng(S)
    dims = [256, 384, 128, 256]                              # layer i: dims[i] -> dims[i + 1]
    specs = [(4, 128, False, 1.0, 0), (8, 0, True, 1.0, 0), (3, 64, False, 1.0, 0), (6, 0, True, 1.0, 0)]
    K = len(specs)
    layers = []
    for i in range(3):
        w = (rng.standard_normal((dims[i + 1], dims[i])) * 0.05).astype(np.float32)
        layers.append([oc.quantize(w, *sp) for sp in specs])
    a_bits = wl.f32_to_bf16_bits(rng.standard_normal((S * T, dims[0])).astype(np.float32))
    e = rng.integers(0, K, S).astype(np.int32)
    e[e == 2] = 1                                             # one expert stays empty
    counts, offsets, perm, inv = oc.bucket(e, K)
    offs_d, perm_d = gb.to_dev(offsets), gb.to_dev(perm)

    packed = [[gb.packed_dev(q) for q in L] for L in layers]
    x0 = gb.bf16_dev(a_bits.reshape(S * T, dims[0]))
    # every tensor between the layers is written and read by the library alone: bf16, bucket order
    x1 = torch.full((S * T, dims[1]), float("nan"), dtype=torch.bfloat16, device=gb.DEV)
    mq.moqe_grouped_qgemm(x0, offs_d, perm_d, S, T, packed[0], x1, mq.OUTPUT_BF16)             # gather, bucket order out
    x2 = torch.full((S * T, dims[2]), float("nan"), dtype=torch.bfloat16, device=gb.DEV)
    mq.moqe_grouped_qgemm(x1, offs_d, None, S, T, packed[1], x2, mq.OUTPUT_BF16)               # bucket order in and out
    y3 = torch.full((S * T, dims[3]), float("nan"), dtype=torch.float32, device=gb.DEV)
    mq.moqe_grouped_qgemm(x2, offs_d, perm_d, S, T, packed[2], y3,
                          mq.SCATTER_OUTPUT | mq.INPUT_IN_BUCKET_ORDER)                        # scatter only here
    torch.cuda.synchronize()

    # stage-wise against the oracle: each layer on the bfloat16 input the GPU actually fed it; a bf16 output
    # must be the oracle's fp64 result rounded once, give or take one bf16 step where fp32 accumulation lands
    # on the other side of a rounding boundary
    x0_f = oc.bf16_bits_to_f64(a_bits).reshape(S, T, dims[0])
    x1_f = gb.bf16_tensor_to_f64(x1).reshape(S, T, dims[1])[inv]      # bucket order -> caller order
    x2_f = gb.bf16_tensor_to_f64(x2).reshape(S, T, dims[2])[inv]
    y3_g = y3.cpu().numpy().reshape(S, T, dims[3])                    # already in caller order
    assert np.all(np.isfinite(x1_f)) and np.all(np.isfinite(x2_f)) and np.all(np.isfinite(y3_g))
    flips = 0
    for s in range(S):
        k = int(e[s])
        for (xin, xout, L) in ((x0_f, x1_f, layers[0]), (x1_f, x2_f, layers[1])):
            ref = oc.qlinear(xin[s], L[k])
            ref16 = oc.bf16_round(ref)
            rms = float(np.sqrt(np.mean(ref * ref)))
            step = np.maximum(np.abs(ref) * 2.0 ** -7, 1e-4 * rms)
            assert np.all(np.abs(xout[s] - ref16) <= step), (s, k)
            flips += int(np.sum(xout[s] != ref16))
        ok, worst = ob.tolerance_ok(y3_g[s], oc.qlinear(x2_f[s], layers[2][k]))
        assert ok, (s, k, worst)
    assert flips < 0.02 * S * T * (dims[1] + dims[2])
