"""GPU parity: round-to-nearest quantizer, packed layout round trip, int8 activation quantization.

Integer results (codes, zero-points, code - zero) must match the oracle bit for bit.
"""
import numpy as np
import pytest
import torch

from oracle import moqe_oracle as oc

pytestmark = pytest.mark.gpu

FORMATS = [(8, 0, True, 1.0, 0), (8, 0, True, 1.0, 1), (6, 0, True, 1.0, 0), (4, 0, True, 1.0, 0),
           (4, 64, False, 1.0, 0), (4, 128, False, 1.0, 0), (3, 64, False, 1.0, 0), (3, 128, False, 1.0, 0),
           (4, 128, False, 0.9, 0), (3, 128, False, 0.85, 0)]


def _w(n, k, seed):
    w = (np.random.default_rng(seed).standard_normal((n, k)) * 0.02).astype(np.float32)
    w[0, :128] = 0.0            # an all-zero group / (almost) zero row start
    w[1, :] = 0.0               # an all-zero row
    w[2, :128] = 0.01           # a constant group
    return w


@pytest.mark.parametrize("bits,group,sym,clip,act", FORMATS)
@pytest.mark.parametrize("n,k", [(48, 384), (16, 128)])
def test_quantize_rtn_matches_oracle_bit_exact(bits, group, sym, clip, act, n, k):
    from paper_2508_09204_amd import binding as mq, experts as ex
    from tests import gpu_blocks as gb
    w = _w(n, k, seed=bits * 7 + group)
    ref = oc.quantize(w, bits, group, sym, clip)
    can = ex.alloc_canonical(n, k, bits, group, sym, 0, gb.DEV)
    mq.moqe_quantize_rtn(gb.to_dev(w), clip, can)
    torch.cuda.synchronize()
    assert np.array_equal(can.qdata.cpu().numpy(), ref.q)
    assert np.array_equal(can.scale.cpu().numpy().view(np.uint32), ref.scale.view(np.uint32))
    if not sym:
        assert np.array_equal(can.zero.cpu().numpy(), ref.zero)


@pytest.mark.parametrize("bits,group,sym,clip,act", FORMATS)
@pytest.mark.parametrize("n,k", [(48, 384), (16, 128), (256, 256)])
def test_pack_unpack_round_trip_bit_exact(bits, group, sym, clip, act, n, k):
    from paper_2508_09204_amd import binding as mq
    from tests import gpu_blocks as gb
    w = _w(n, k, seed=bits * 11 + group + n)
    ref = oc.quantize(w, bits, group, sym, clip, act)
    packed = gb.packed_dev(ref)
    assert packed.qdata.numel() == mq.moqe_packed_bytes(n, k, bits, group, sym, act)
    out = torch.full((n, k), -999, dtype=torch.int16, device=gb.DEV)
    sc = torch.zeros(ref.scale.shape, dtype=torch.float32, device=gb.DEV)
    mq.moqe_unpack_qmat(packed, out, sc)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), oc.dequant_int(ref))
    assert np.array_equal(sc.cpu().numpy().view(np.uint32), ref.scale.view(np.uint32))


def test_quantize_full_llama_matrix_matches_oracle():
    """One full-size matrix (11008 x 4096, int4 g128): codes, scales and zero-points bit-exact."""
    from paper_2508_09204_amd import binding as mq, experts as ex
    from tests import gpu_blocks as gb
    w = (np.random.default_rng(5).standard_normal((11008, 4096)) * 0.02).astype(np.float32)
    ref = oc.quantize_asym_group(w, 4, 128, 0.9)
    can = ex.alloc_canonical(11008, 4096, 4, 128, False, 0, gb.DEV)
    mq.moqe_quantize_rtn(gb.to_dev(w), 0.9, can)
    torch.cuda.synchronize()
    assert np.array_equal(can.qdata.cpu().numpy(), ref.q)
    assert np.array_equal(can.scale.cpu().numpy(), ref.scale)
    assert np.array_equal(can.zero.cpu().numpy(), ref.zero)
