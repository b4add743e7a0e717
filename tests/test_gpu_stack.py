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
    y1 = torch.empty((S * T, dims[1]), dtype=torch.float32, device=gb.DEV)
    mq.moqe_grouped_qgemm(x0, offs_d, perm_d, S, T, packed[0], y1, 0)                          # gather, bucket order out
    x1 = y1.to(torch.bfloat16)
    y2 = torch.empty((S * T, dims[2]), dtype=torch.float32, device=gb.DEV)
    mq.moqe_grouped_qgemm(x1, offs_d, None, S, T, packed[1], y2, 0)                            # bucket order in and out
    x2 = y2.to(torch.bfloat16)
    y3 = torch.full((S * T, dims[3]), float("nan"), dtype=torch.float32, device=gb.DEV)
    mq.moqe_grouped_qgemm(x2, offs_d, perm_d, S, T, packed[2], y3,
                          mq.SCATTER_OUTPUT | mq.INPUT_IN_BUCKET_ORDER)                        # scatter only here
    torch.cuda.synchronize()

    # stage-wise against the oracle: each layer on the bfloat16 input the GPU actually fed it
    x0_f = oc.bf16_bits_to_f64(a_bits).reshape(S, T, dims[0])
    y1_g = y1.cpu().numpy().reshape(S, T, dims[1])[inv]       # bucket order -> caller order
    x1_f = gb.bf16_tensor_to_f64(x1).reshape(S, T, dims[1])[inv]
    y2_g = y2.cpu().numpy().reshape(S, T, dims[2])[inv]
    x2_f = gb.bf16_tensor_to_f64(x2).reshape(S, T, dims[2])[inv]
    y3_g = y3.cpu().numpy().reshape(S, T, dims[3])            # already in caller order
    assert np.all(np.isfinite(y3_g))
    for s in range(S):
        k = int(e[s])
        for (xin, yout, L) in ((x0_f, y1_g, layers[0]), (x1_f, y2_g, layers[1]), (x2_f, y3_g, layers[2])):
            ok, worst = ob.tolerance_ok(yout[s], oc.qlinear(xin[s], L[k]))
            assert ok, (s, k, worst)
    # and the intermediate roundings are those of the values the GPU produced (round to nearest even)
    assert np.array_equal(gb.bf16_tensor_to_f64(x1).reshape(-1), oc.bf16_round(y1.cpu().numpy().astype(np.float64)).reshape(-1))
