"""Pins for the oracle's aggregation divergence (Sec. 4.3, Definition 2 of the paper:
distance between a worker's model and the aggregate of all workers).  CPU only."""
import numpy as np
import pytest


def test_divergence_equals_numpy_float64(ref):
    rng = np.random.default_rng(0)
    X = rng.normal(0, 0.02, (12, 30_001)).astype(np.float32)
    X64 = X.astype(np.float64)
    want = ((X64 - X64.mean(axis=0)) ** 2).sum(axis=1)
    got = ref.aggregation_divergence(X)
    assert np.allclose(got, want, rtol=1e-12, atol=0)
    d = rng.integers(100, 2000, 12).astype(np.float32)
    mean = (d[:, None].astype(np.float64) * X64).sum(axis=0) / d.astype(np.float64).sum()
    want = ((X64 - mean) ** 2).sum(axis=1)
    assert np.allclose(ref.aggregation_divergence(X, d=d), want, rtol=1e-12, atol=0)


def test_divergence_closed_forms(ref):
    x = np.random.default_rng(1).normal(0, 1, 5000).astype(np.float32)
    # identical workers: zero (Sec. 4.1: common initialisation)
    assert np.all(ref.aggregation_divergence(np.stack([x] * 7)) == 0.0)
    # x and -x: the mean is 0, each worker is |x| away
    got = ref.aggregation_divergence(np.stack([x, -x]))
    n2 = float((x.astype(np.float64) ** 2).sum())
    assert np.allclose(got, [n2, n2], rtol=1e-13)
    # a pitch does not change anything
    buf = np.full((3, 5056), 9.0, np.float32)
    buf[:, :5000] = np.stack([0 * x, x, 2 * x])      # all exact in binary32; the mean is x
    assert np.allclose(ref.aggregation_divergence(buf[:, :5000]), [n2, 0.0, n2], rtol=1e-12, atol=1e-25)


def test_divergence_after_full_aggregation_is_rounding_only(ref):
    """R = N-1: every worker ends at the FedAvg mean, the divergence drops to zero
    (Sec. 4.3) - here to binary32 rounding."""
    N, P, S = 10, 20_000, 4
    X = np.random.default_rng(2).normal(0, 0.02, (N, P)).astype(np.float32)
    before = ref.aggregation_divergence(X)
    Y = ref.gossip_round(X, ref.make_peer_table(N, S, N - 1, 0, 0), P, S, N - 1)
    after = ref.aggregation_divergence(Y)
    assert after.max() < 1e-10 * before.min()


def test_more_replicas_mean_less_divergence(ref):
    """The trade-off R controls (Sec. 4.3, Sec. 5.2): after one round from independent
    models the largest distance to the global mean shrinks as R grows."""
    N, P, S = 30, 50_000, 10
    X = np.random.default_rng(3).normal(0, 0.02, (N, P)).astype(np.float32)
    rho = []
    for R in (1, 2, 4, 8, 16, 29):
        Y = ref.gossip_round(X, ref.make_peer_table(N, S, R, 0, 0), P, S, R)
        rho.append(np.sqrt(ref.aggregation_divergence(Y).max()))
    assert all(a > b for a, b in zip(rho, rho[1:]))
    # independent models of variance v: one round leaves about v*(1/(R+1) - 1/N) per element
    for R, r in zip((1, 2, 4, 8, 16), rho):
        expect = np.sqrt(P * 0.02 ** 2 * (1 / (R + 1) - 1 / N))
        assert abs(r - expect) / expect < 0.05
