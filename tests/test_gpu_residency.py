"""GPU: on-demand residency of expert weights (the serving mode in which only the experts in use sit in
device memory and the others are copied in from host memory when the router switches to them).

The kernels are the same as with all experts resident, so results must be bit-identical; the cache's
replacement order is checked against a least-recently-used model on the host.
"""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import moqe_oracle as oc
from tests import oracle_blocks as ob

pytestmark = pytest.mark.gpu

SPECS = [(4, 128, False, 1.0, 0), (8, 0, True, 1.0, 0), (3, 64, False, 1.0, 0), (6, 0, True, 1.0, 0), (4, 0, True, 1.0, 0)]


def _setup(n, k, seed):
    from tests import gpu_blocks as gb
    rng = np.random.default_rng(seed)
    w = (rng.standard_normal((n, k)) * 0.02).astype(np.float32)
    qms = [oc.quantize(w, *sp) for sp in SPECS]
    packed = [gb.packed_dev(q) for q in qms]                       # all resident: the comparison
    host = [p.qdata.cpu().pin_memory() for p in packed]             # the blobs as they wait in host memory
    return qms, packed, host


def test_one_expert_at_a_time_switching():
    """Requests served one by one, two slots for five experts: every result equals the all-resident one bit
    for bit, and a blob is copied exactly when a least-recently-used cache of two would miss."""
    from paper_2508_09204_amd import binding as mq
    from tests import gpu_blocks as gb
    n, k, T = 96, 256, 3
    qms, packed, host = _setup(n, k, 1)
    cache = mq.moqe_cache_create(host, 2)
    try:
        rng = np.random.default_rng(2)
        seq = [0, 1, 0, 2, 3, 3, 1, 4, 1, 4, 0, 2, 2, 0]
        lru, expected_copies = [], 0
        offsets = gb.to_dev(np.array([0, 1], dtype=np.int32))
        for step, e in enumerate(seq):
            a_bits = wl.f32_to_bf16_bits(rng.standard_normal((T, k)).astype(np.float32))
            a = gb.bf16_dev(a_bits)
            (addr,), copied = mq.moqe_cache_acquire(cache, [e])
            miss = e not in lru
            if miss:
                expected_copies += 1
                if len(lru) == 2:
                    lru.pop(0)
            else:
                lru.remove(e)
            lru.append(e)
            assert copied == int(miss), (step, e)
            p = packed[e]
            cached = mq.QMat(addr, None, None, p.n, p.k, p.bits, p.group, p.symmetric, p.act_mode, p.layout)
            y_c = torch.empty((T, n), dtype=torch.float32, device=gb.DEV)
            y_r = torch.empty((T, n), dtype=torch.float32, device=gb.DEV)
            mq.moqe_grouped_qgemm(a, offsets, None, 1, T, [cached], y_c, 0)
            mq.moqe_grouped_qgemm(a, offsets, None, 1, T, [p], y_r, 0)
            torch.cuda.synchronize()
            assert torch.equal(y_c, y_r), (step, e)
            ok, worst = ob.tolerance_ok(y_c.cpu().numpy(), oc.qlinear(oc.bf16_bits_to_f64(a_bits), qms[e]))
            assert ok, (step, e, worst)
        copies, nbytes = mq.moqe_cache_stats(cache)
        assert copies == expected_copies
        assert nbytes == sum(host[e].numel() for e in _misses(seq, 2))
    finally:
        mq.moqe_cache_destroy(cache)


def _misses(seq, slots):
    lru, out = [], []
    for e in seq:
        if e in lru:
            lru.remove(e)
        else:
            out.append(e)
            if len(lru) == slots:
                lru.pop(0)
        lru.append(e)
    return out


def test_batch_loads_only_the_experts_in_use():
    """A routed batch that uses two of five experts: both are acquired in one call, the grouped GEMM runs on the
    cached copies (empty buckets get a placeholder address that is never read) and matches the all-resident run."""
    from paper_2508_09204_amd import binding as mq
    from tests import gpu_blocks as gb
    n, k, S, T = 64, 384, 7, 2
    qms, packed, host = _setup(n, k, 3)
    cache = mq.moqe_cache_create(host, 3)
    try:
        e = np.array([3, 1, 1, 3, 3, 1, 3], dtype=np.int32)
        counts, offsets, perm, inv = oc.bucket(e, len(qms))
        used = [int(i) for i in np.nonzero(counts)[0]]
        addrs, copied = mq.moqe_cache_acquire(cache, used)
        assert copied == 2
        again, copied2 = mq.moqe_cache_acquire(cache, used)
        assert copied2 == 0 and again == addrs                       # hits: no copies, same addresses
        where = dict(zip(used, addrs))
        experts = []
        for i, p in enumerate(packed):
            experts.append(mq.QMat(where.get(i, addrs[0]), None, None, p.n, p.k, p.bits, p.group, p.symmetric, p.act_mode, p.layout))
        a_bits = wl.f32_to_bf16_bits(np.random.default_rng(4).standard_normal((S * T, k)).astype(np.float32))
        a = gb.bf16_dev(a_bits)
        y_c = torch.empty((S * T, n), dtype=torch.float32, device=gb.DEV)
        y_r = torch.empty((S * T, n), dtype=torch.float32, device=gb.DEV)
        mq.moqe_grouped_qgemm(a, gb.to_dev(offsets), gb.to_dev(perm), S, T, experts, y_c, 1)
        mq.moqe_grouped_qgemm(a, gb.to_dev(offsets), gb.to_dev(perm), S, T, packed, y_r, 1)
        torch.cuda.synchronize()
        assert torch.equal(y_c, y_r)
        with pytest.raises(mq.MoqeError):
            mq.moqe_cache_acquire(cache, [0, 1, 2, 3])               # more blobs than slots
        with pytest.raises(mq.MoqeError):
            mq.moqe_cache_acquire(cache, [1, 1])                     # a blob twice
    finally:
        mq.moqe_cache_destroy(cache)
