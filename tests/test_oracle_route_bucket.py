"""Pins for the oracle's router, top-1 selection, dispatch counts and stable bucketing (CPU only)."""
import numpy as np
import pytest

from oracle import moqe_oracle as oc


def _router(rng, D, H, K, bias=True):
    if H:
        return oc.Router(w1=rng.standard_normal((H, D)).astype(np.float32),
                         b1=rng.standard_normal(H).astype(np.float32) if bias else None,
                         w2=rng.standard_normal((K, H)).astype(np.float32),
                         b2=rng.standard_normal(K).astype(np.float32) if bias else None)
    return oc.Router(w1=None, b1=None, w2=rng.standard_normal((K, D)).astype(np.float32),
                     b2=rng.standard_normal(K).astype(np.float32) if bias else None)


def test_pool_hand_example():
    x = np.array([[[1.0, 2.0], [3.0, 6.0]], [[-1.0, 0.5], [-1.0, 0.5]]])
    assert oc.pool(x).tolist() == [[2.0, 4.0], [-1.0, 0.5]]
    x1 = np.random.default_rng(0).standard_normal((5, 1, 7))
    assert np.array_equal(oc.pool(x1), x1[:, 0, :])          # T = 1: the row itself


@pytest.mark.parametrize("H", [0, 5])
def test_router_matches_scalar_loops(H):
    rng = np.random.default_rng(1)
    S, T, D, K = 7, 3, 11, 4
    x = rng.standard_normal((S, T, D))
    r = _router(rng, D, H, K)
    idx, logits, margin = oc.route(x, r)
    for s in range(S):
        p = [sum(x[s, t, d] for t in range(T)) / T for d in range(D)]
        if H:
            h = []
            for j in range(H):
                a = float(r.b1[j]) + sum(float(r.w1[j, d]) * p[d] for d in range(D))
                h.append(a if a > 0 else 0.0)
        else:
            h = p
        z = [float(r.b2[k]) + sum(float(r.w2[k, j]) * h[j] for j in range(len(h))) for k in range(K)]
        np.testing.assert_allclose(logits[s], z, rtol=1e-12, atol=1e-12)
        assert idx[s] == max(range(K), key=lambda k: (z[k], -k))
        zs = sorted(z)
        assert np.isclose(margin[s], zs[-1] - zs[-2])


def test_single_linear_router_is_numpy_argmax():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((64, 4, 32))
    r = _router(rng, 32, 0, 3, bias=False)
    idx, logits, _ = oc.route(x, r)
    ref = np.argmax(x.mean(axis=1) @ r.w2.astype(np.float64).T, axis=1)
    assert np.array_equal(idx, ref)
    assert set(idx.tolist()) == {0, 1, 2}


def test_ties_go_to_lowest_index():
    assert oc.argmax_first(np.array([[1.0, 3.0, 3.0], [2.0, 2.0, 2.0], [0.0, -1.0, 0.0],
                                     [-5.0, -4.0, -4.0]])).tolist() == [1, 0, 0, 1]
    # duplicated router rows give bit-identical logits
    rng = np.random.default_rng(3)
    w = rng.standard_normal((1, 16)).astype(np.float32)
    r = oc.Router(w1=None, b1=None, w2=np.concatenate([w * 0.5, w, w]), b2=None)
    x = rng.standard_normal((20, 2, 16))
    idx, logits, margin = oc.route(x, r)
    pos = logits[:, 1] > 0
    assert np.all(idx[pos] == 1) and np.all(idx[~pos] == 0)
    assert np.all(margin[pos] == 0.0)


def test_relu_is_applied():
    r = oc.Router(w1=np.array([[1.0], [-1.0]], dtype=np.float32), b1=None,
                  w2=np.array([[1.0, 0.0], [0.0, 1.0]], dtype=np.float32), b2=None)
    lg = oc.router_logits(np.array([[2.0], [-3.0]]), r)
    assert lg.tolist() == [[2.0, 0.0], [0.0, 3.0]]


def test_bucket_hand_example():
    counts, offsets, perm, inv = oc.bucket([2, 0, 2, 1, 0], 3)
    assert counts.tolist() == [2, 1, 2]
    assert offsets.tolist() == [0, 2, 3, 5]
    assert perm.tolist() == [1, 4, 3, 0, 2]
    assert inv.tolist() == [3, 0, 4, 2, 1]


@pytest.mark.parametrize("S,K,seed", [(1, 1, 0), (1, 4, 1), (64, 4, 2), (257, 8, 3), (1000, 3, 4), (0, 4, 5)])
def test_bucket_invariants(S, K, seed):
    e = np.random.default_rng(seed).integers(0, K, S)
    counts, offsets, perm, inv = oc.bucket(e, K)
    assert counts.sum() == S and offsets[0] == 0 and offsets[K] == S
    assert np.array_equal(np.diff(offsets), counts)
    assert np.array_equal(counts, np.bincount(e, minlength=K))
    assert sorted(perm.tolist()) == list(range(S))                 # every sample in exactly one slot
    assert np.array_equal(inv[perm], np.arange(S))
    assert np.all(np.diff(e[perm]) >= 0)                           # grouped by expert
    for k in range(K):                                             # stable inside a bucket
        assert np.all(np.diff(perm[offsets[k]:offsets[k + 1]]) > 0)
    assert np.array_equal(perm, np.argsort(e, kind="stable"))      # library routine, same definition


def test_bucket_empty_and_all_to_one():
    counts, offsets, perm, inv = oc.bucket([3, 3, 3], 5)
    assert counts.tolist() == [0, 0, 0, 3, 0]
    assert offsets.tolist() == [0, 0, 0, 0, 3, 3]
    assert perm.tolist() == [0, 1, 2] and inv.tolist() == [0, 1, 2]


def test_balance_loss_closed_forms():
    # uniform probabilities and uniform dispatch: N * sum (1/N)(1/N) = 1  (Eq. 1-2)
    N = 4
    logits = np.zeros((8, N))
    assert np.isclose(oc.balance_loss(logits, np.arange(8) % N), 1.0)
    # everything to one expert with probability ~1: N * 1 * 1 = N
    logits = np.full((8, N), -1e3)
    logits[:, 2] = 1e3
    assert np.isclose(oc.balance_loss(logits, np.full(8, 2)), float(N))


def test_balance_stats_closed_forms():
    """Eq. (1)-(2) and the dynamic weight on cases with known values."""
    N, B = 4, 12
    # uniform probabilities, perfectly even dispatch: P = F = 1/N, L_bal = 1, sigma = 0, alpha_dyn = alpha
    P, F, l, sig, a = oc.balance_stats(np.zeros((B, N)), np.arange(B) % N, 0.02)
    assert np.allclose(P, 0.25) and np.allclose(F, 0.25)
    assert np.isclose(l, 1.0) and sig == 0.0 and np.isclose(a, 0.02)
    # everything dispatched to expert 1: n = (0, B, 0, 0); population std = mean * sqrt(N - 1)
    P, F, l, sig, a = oc.balance_stats(np.zeros((B, N)), np.full(B, 1), 0.02)
    assert np.allclose(F, [0, 1, 0, 0]) and np.isclose(l, N * 0.25)
    assert np.isclose(sig, np.sqrt(N - 1)) and np.isclose(a, 0.02 * (1 + np.sqrt(3)))
    # two-expert batch with hand-computed softmax: logits (0, ln 3) -> p = (1/4, 3/4)
    z = np.array([[0.0, np.log(3.0)], [np.log(3.0), 0.0], [0.0, np.log(3.0)], [0.0, np.log(3.0)]])
    P, F, l, sig, a = oc.balance_stats(z, np.array([1, 0, 1, 1]), 1.0)
    assert np.allclose(P, [(0.25 * 3 + 0.75) / 4, (0.75 * 3 + 0.25) / 4])
    assert np.allclose(F, [0.25, 0.75])
    assert np.isclose(l, 2 * (0.375 * 0.25 + 0.625 * 0.75))
    assert np.isclose(sig, 0.5) and np.isclose(a, 1.5)           # n = (1, 3): std 1, mean 2
    # agrees with the scalar form used elsewhere, and a constant added to a row changes nothing
    rng = np.random.default_rng(5)
    z = rng.standard_normal((33, 5))
    idx = rng.integers(0, 5, 33)
    assert np.isclose(oc.balance_stats(z, idx, 0.1)[2], oc.balance_loss(z, idx))
    assert np.allclose(oc.balance_stats(z + 100.0, idx, 0.1)[0], oc.balance_stats(z, idx, 0.1)[0])
    assert np.isclose(oc.balance_stats(z, idx, 0.1)[0].sum(), 1.0)
