"""GPU check of moqe_forward_static, the variant of moqe_forward for callers that cannot allocate:
its scratch memory is a buffer built into the library.  Two calls in a row (the second on a smaller
batch, so stale contents of the shared buffer would show) must reproduce moqe_forward bit for bit,
and a batch that does not fit the buffer is refused before anything runs."""
import numpy as np
import pytest
import torch

import workloads as wl
from tests import oracle_blocks as ob

pytestmark = pytest.mark.gpu


def _pair(mq, gb, dblk, cfg, bits, static):
    x = gb.bf16_dev(bits.reshape(cfg.M, cfg.D))
    y = torch.full((cfg.M, cfg.D), float("nan"), dtype=torch.float32, device=gb.DEV)
    aux = gb.new_aux(cfg.S, cfg.K, cfg.M, cfg.F)
    if static:
        mq.moqe_forward_static(dblk, x, cfg.S, cfg.T, y, aux)
    else:
        mq.moqe_forward(dblk, x, cfg.S, cfg.T, y, aux)
    torch.cuda.synchronize()
    return y, aux


def test_static_scratch_forward_matches_workspace_forward():
    from paper_2508_09204_amd import binding as mq
    from tests import gpu_blocks as gb
    base = wl.get_config("llama7b_mlp_decode")
    big = wl.scaled(base, S=45, T=3, D=384, F=640, router_hidden=32)
    small = wl.scaled(base, S=7, T=1, D=384, F=640, router_hidden=32)
    blk = ob.make_block(big)                       # same weights and router for both batches
    dblk = gb.block_dev(blk)
    for cfg in (big, small):                       # second call: smaller input on the same buffer
        bits, _ = ob.activations_f64(cfg)
        y_ref, aux_ref = _pair(mq, gb, dblk, cfg, bits, static=False)
        y, aux = _pair(mq, gb, dblk, cfg, bits, static=True)
        assert torch.equal(y, y_ref)
        assert torch.all(torch.isfinite(y))
        for name in ("expert_idx", "logits", "counts", "offsets", "perm", "inv_perm"):
            assert torch.equal(getattr(aux, name), getattr(aux_ref, name)), name
        assert torch.equal(aux.h.view(torch.int16), aux_ref.h.view(torch.int16))
        assert len(set(aux.expert_idx.cpu().tolist())) > 1


def test_static_scratch_forward_refuses_what_does_not_fit():
    from paper_2508_09204_amd import binding as mq
    from tests import gpu_blocks as gb
    base = wl.get_config("llama7b_mlp_decode")
    cfg = wl.scaled(base, S=64, T=200, D=384, F=1024, router_hidden=32)       # H alone: 64*200*1024*2 = 26 MB
    dblk = gb.block_dev(ob.make_block(cfg))
    assert mq.moqe_workspace_bytes(dblk, cfg.S, cfg.T) > mq.STATIC_SCRATCH_BYTES
    x = torch.zeros((cfg.M, cfg.D), dtype=torch.bfloat16, device=gb.DEV)
    y = torch.full((cfg.M, cfg.D), 7.0, dtype=torch.float32, device=gb.DEV)
    with pytest.raises(mq.MoqeError) as ei:
        mq.moqe_forward_static(dblk, x, cfg.S, cfg.T, y)
    assert ei.value.code == -4
    torch.cuda.synchronize()
    assert torch.all(y == 7.0)                     # nothing was enqueued
