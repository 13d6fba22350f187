"""Pins for the CPU oracle: every check here compares the oracle with something that
is NOT the oracle - published generator outputs, closed forms, hand-worked literal
examples, textbook/library routines (dense matmul, column mean), brute force on tiny
inputs and invariants the paper states.  CPU only.

Paper passages behind the properties:
  Eq. (1) and Sec. 5.1 (segments do not overlap and together are the model),
  Sec. 4.1 step (2) (R peers per segment, other workers, without replacement),
  Eq. (3) (weighted mean over the worker itself and its R providers), Eq. (4),
  Sec. 4.1 (identical initialisation), Sec. 4.3 / 5.2 (R = n-1 is FedAvg),
  Sec. 5.1 (S = 1 is plain gossip; the process is synchronous).
"""
import itertools
import os

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
M64 = (1 << 64) - 1


# ----------------------------------------------------------------------------- bounds
def test_bounds_values_of_the_five_workloads(ref):
    # (P, S) -> (common length, last length), worked out by hand from P = S*L + rem
    table = {
        (65_536, 8): (8192, 8192),
        (11_689_512, 32): (365_297, 365_305),
        (25_557_032, 10): (2_555_703, 2_555_705),
        (1_000_003, 7): (142_857, 142_861),
        (335_141_888, 16): (20_946_368, 20_946_368),
    }
    for (P, S), (L, last) in table.items():
        lo, hi = ref.segment_bounds(P, S)
        assert lo[0] == 0 and hi[-1] == P
        assert np.all(hi[:-1] - lo[:-1] == L)
        assert hi[-1] - lo[-1] == last
        assert np.all(lo[1:] == hi[:-1])


@pytest.mark.parametrize("P", [1, 2, 6, 7, 64, 97, 1000])
def test_bounds_cover_every_column_exactly_once(ref, P):
    for S in sorted({1, 2, 3, min(7, P), P}):
        if S > P:
            continue
        lo, hi = ref.segment_bounds(P, S)
        owner = np.zeros(P, np.int64)
        for s in range(S):
            assert hi[s] > lo[s]
            owner[lo[s]:hi[s]] += 1
        assert np.all(owner == 1)
        # "same number of parameters": all but the last are floor(P/S)
        assert np.all((hi - lo)[:-1] == P // S)
        assert (hi - lo)[-1] == P - (S - 1) * (P // S)


def test_bounds_reject_bad_arguments(ref):
    with pytest.raises(ValueError):
        ref.segment_bounds(4, 5)
    with pytest.raises(ValueError):
        ref.segment_bounds(4, 0)


# ------------------------------------------------------------------------------- hash
def _golden_vectors():
    out = []
    with open(os.path.join(HERE, "golden", "splitmix64_vectors.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            seed, idx, val = line.split()
            out.append((int(seed), int(idx), int(val)))
    return out


def test_mix64_reproduces_published_splitmix64_outputs(ref):
    gamma = 0x9E3779B97F4A7C15
    for seed, idx, val in _golden_vectors():
        assert ref.mix64((seed + idx * gamma) & M64) == val


def test_hash_chain_structure(ref):
    """hash(seed, r, w, s, j) = absorb(absorb(absorb(absorb(first SplitMix64 output of
    seed, r), w), s), j), absorb(h, c) = mix64((h ^ c) + GAMMA).  The chain is this
    repository's own definition (the paper names no hash); this test pins the ORDER
    in which the counters enter and that each is used, via the pinned mix64."""
    gamma = 0x9E3779B97F4A7C15
    mix = ref.mix64
    for seed, r, w, s, j in [(0, 0, 0, 0, 0), (7, 3, 31, 9, 1), (1234567, 19, 99, 6, 2),
                             (M64, 1 << 40, 5, 4, 3)]:
        h = mix((seed + gamma) & M64)
        for c in (r, w, s, j):
            h = mix(((h ^ c) + gamma) & M64)
        assert ref.peer_hash(seed, r, w, s, j) == h
    # the five arguments are not interchangeable
    vals = {ref.peer_hash(*p) for p in itertools.permutations((1, 2, 3, 4, 5))}
    assert len(vals) == 120
    # seed 0 / 1234567 start from the published first outputs
    assert mix((1234567 + gamma) & M64) == 6457827717110365317


def test_reduce_is_the_exact_multiply_shift(ref):
    rng = np.random.default_rng(1)
    for m in [1, 2, 3, 5, 15, 31, 98, 99, 1000, 16383, (1 << 31) - 1, (1 << 32) - 1]:
        hs = [0, M64, 1 << 32, (1 << 32) - 1, 0x8000000000000000] + [int(x) for x in
              rng.integers(0, 1 << 63, 50, dtype=np.int64) * 2 + 1]
        for h in hs:
            h &= M64
            want = ((h >> 32) * m) >> 32       # python integers: exact
            got = ref.reduce(h, m)
            assert got == want and 0 <= got < m
    assert ref.reduce(M64, 7) == 6 and ref.reduce(0, 7) == 0


# ------------------------------------------------------------------------- peer table
def _fisher_yates_prefix(N, R, w, words):
    """Textbook partial Fisher-Yates over 'all the other workers' (increasing order,
    w skipped), swap partner of step j taken from words[j]; written independently."""
    others = [v for v in range(N) if v != w]
    M = len(others)
    for j in range(R):
        r = j + (((words[j] >> 32) * (M - j)) >> 32)
        others[j], others[r] = others[r], others[j]
    return others[:R]


@pytest.mark.parametrize("N,S,R,seed,rnd", [(4, 8, 2, 0, 0), (32, 32, 4, 0, 9), (32, 10, 2, 7, 3),
                                            (100, 7, 3, 0, 19), (16, 16, 4, 0, 4), (5, 3, 4, 11, 2),
                                            (2, 4, 1, 3, 3), (1, 2, 0, 0, 0), (9, 1, 0, 5, 5)])
def test_peer_table_is_fisher_yates_on_the_hash_words(ref, N, S, R, seed, rnd):
    T = ref.make_peer_table(N, S, R, seed, rnd)
    assert T.shape == (N, S, R) and T.dtype == np.int32
    for w in range(N):
        for s in range(S):
            words = [ref.peer_hash(seed, rnd, w, s, j) for j in range(R)]
            assert list(T[w, s]) == _fisher_yates_prefix(N, R, w, words)


@pytest.mark.parametrize("N,S,R", [(4, 8, 2), (32, 32, 4), (100, 7, 3), (16, 16, 15), (7, 5, 6)])
def test_peer_table_structure(ref, N, S, R):
    for rnd in range(3):
        T = ref.make_peer_table(N, S, R, 0, rnd)
        assert T.min() >= 0 and T.max() < N
        for w in range(N):
            assert not np.any(T[w] == w)                       # never itself
            for s in range(S):
                assert len(set(T[w, s].tolist())) == R          # without replacement
                if R == N - 1:                                  # all the others
                    assert sorted(T[w, s].tolist()) == [v for v in range(N) if v != w]


def test_peer_table_two_workers_and_determinism(ref):
    T = ref.make_peer_table(2, 5, 1, 123, 4)
    assert np.all(T[0] == 1) and np.all(T[1] == 0)
    a = ref.make_peer_table(32, 32, 4, 0, 5)
    b = ref.make_peer_table(32, 32, 4, 0, 5)
    c = ref.make_peer_table(32, 32, 4, 0, 6)
    d = ref.make_peer_table(32, 32, 4, 1, 5)
    assert np.array_equal(a, b) and not np.array_equal(a, c) and not np.array_equal(a, d)
    with pytest.raises(ValueError):
        ref.make_peer_table(4, 2, 4, 0, 0)    # cannot pick 4 distinct others out of 3


def test_peer_table_draws_are_uniform(ref):
    """N=4, R=2: each worker has 6 equally likely ordered pairs of others.  Chi-square
    over 4000 (round, segment) draws per worker; 5 degrees of freedom, the 99.99 %
    quantile is 25.7."""
    N, S, R = 4, 50, 2
    counts = {w: {} for w in range(N)}
    for rnd in range(80):
        T = ref.make_peer_table(N, S, R, 2024, rnd)
        for w in range(N):
            for s in range(S):
                key = (int(T[w, s, 0]), int(T[w, s, 1]))
                counts[w][key] = counts[w].get(key, 0) + 1
    for w in range(N):
        assert len(counts[w]) == 6
        n = sum(counts[w].values())
        chi2 = sum((c - n / 6) ** 2 / (n / 6) for c in counts[w].values())
        assert chi2 < 25.7, (w, counts[w])
    # N=100: the first peer is uniform over the 99 others (98 dof, 99.99 % ~ 157)
    T = np.concatenate([ref.make_peer_table(100, 7, 3, 5, r) for r in range(30)], axis=1)
    for w in (0, 37, 99):
        h = np.bincount(T[w, :, 0], minlength=100)
        assert h[w] == 0
        e = T.shape[1] / 99
        chi2 = float(np.sum((np.delete(h, w) - e) ** 2 / e))
        assert chi2 < 157


def test_peer_table_golden_file(ref):
    """Regression guard: a table written once by tests/golden/make_peer_table_golden.py
    (which calls only the oracle)."""
    path = os.path.join(HERE, "golden", "peer_table_N4_S8_R2_seed0_round0.txt")
    rows = [list(map(int, l.split())) for l in open(path) if not l.startswith("#")]
    T = ref.make_peer_table(4, 8, 2, 0, 0)
    assert np.array_equal(T.reshape(4, 16), np.array(rows, np.int32))


# ------------------------------------------------------------------ aggregation, Eq. 3
def _f32(a):
    return np.array(a, dtype=np.float32)


def test_round_hand_worked_R1_S2(ref):
    """N=3, P=6, S=2, R=1; integers whose pair sums halve exactly in binary32."""
    X = _f32([[3, 6, 9, 12, 15, 18],
              [0, 3, 30, 6, 9, 3],
              [9, 0, 3, 0, 3, 9]])
    peers = np.array([[[1], [2]], [[2], [0]], [[0], [1]]], np.int32)   # [w][s][j]
    want = _f32([[1.5, 4.5, 19.5, 6.0, 9.0, 13.5],      # w0: cols 0-2 with w1, 3-5 with w2
                 [4.5, 1.5, 16.5, 9.0, 12.0, 10.5],     # w1: cols 0-2 with w2, 3-5 with w0
                 [6.0, 3.0, 6.0, 3.0, 6.0, 6.0]])       # w2: cols 0-2 with w0, 3-5 with w1
    Y = ref.gossip_round(X, peers, P=6, S=2, R=1)
    assert np.array_equal(Y, want)
    Y64 = ref.gossip_round_f64(X, peers, P=6, S=2, R=1)
    assert np.array_equal(Y64, want.astype(np.float64))


def test_round_hand_worked_R1_S3_distinct_peer_per_segment(ref):
    X = _f32([[2, 4, 6, 8, 10, 12],
              [4, 0, 2, 2, 0, 4],
              [0, 8, 0, 4, 6, 0]])
    peers = np.array([[[1], [2], [1]], [[0], [0], [2]], [[1], [0], [0]]], np.int32)
    want = _f32([[3, 2, 3, 6, 5, 8],       # (0,1)|w1  (2,3)|w2  (4,5)|w1
                 [3, 2, 4, 5, 3, 2],       # (0,1)|w0  (2,3)|w0  (4,5)|w2
                 [2, 4, 3, 6, 8, 6]])      # (0,1)|w1  (2,3)|w0  (4,5)|w0
    assert np.array_equal(ref.gossip_round(X, peers, P=6, S=3, R=1), want)


def test_round_hand_worked_R2_full_mean(ref):
    """N=3, R=2: every worker averages all three.  Column sums are multiples of 3 and
    small, so fl(sum * fl(1/3)) is the exact third."""
    X = _f32([[3, 6, 9, 12, 15, 18],
              [0, 3, 30, 6, 9, 3],
              [9, 0, 3, 0, 3, 9]])
    peers = np.array([[[1, 2], [2, 1]], [[2, 0], [0, 2]], [[0, 1], [1, 0]]], np.int32)
    want_row = _f32([4, 3, 14, 6, 9, 10])
    Y = ref.gossip_round(X, peers, P=6, S=2, R=2)
    assert np.array_equal(Y, np.stack([want_row] * 3))


def test_round_hand_worked_weighted(ref):
    """Eq. (3) with unequal dataset sizes, N=3, P=4, S=2, R=1, d=(1,3,4):
       w0 seg0 with w1: (1*x0 + 3*x1)/4 ; w0 seg1 with w2: (1*x0 + 4*x2)/5 ; ..."""
    d = _f32([1, 3, 4])
    X = _f32([[4, 8, 5, 10],
              [0, 4, 7, 14],
              [8, 1, 0, 5]])
    peers = np.array([[[1], [2]], [[2], [0]], [[1], [0]]], np.int32)
    want = _f32([[(4 + 0) / 4, (8 + 12) / 4, (5 + 0) / 5, (10 + 20) / 5],
                 [(0 + 32) / 7, (12 + 4) / 7, (21 + 5) / 4, (42 + 10) / 4],
                 [(32 + 0) / 7, (4 + 12) / 7, (0 + 5) / 5, (20 + 10) / 5]])
    Y = ref.gossip_round(X, peers, P=4, S=2, R=1, d=d)
    # quotients by 7 are correctly rounded binary32 divisions of exact integers
    assert np.array_equal(Y, want)


def _dense_mixing(peers, N, S, R, d=None):
    """A[s] (N x N, float64, row-stochastic): Y[:, seg s] = A[s] @ X[:, seg s]."""
    A = np.zeros((S, N, N))
    dd = np.ones(N) if d is None else np.asarray(d, np.float64)
    for w in range(N):
        for s in range(S):
            members = [w] + [int(p) for p in peers[w, s]]
            tot = sum(dd[m] for m in members)
            for m in members:
                A[s, w, m] += dd[m] / tot
    return A


@pytest.mark.parametrize("N,P,S,R,weighted", [(4, 65, 8, 2, False), (6, 1003, 7, 3, False),
                                              (9, 257, 1, 4, False), (5, 40, 40, 4, False),
                                              (6, 1003, 7, 3, True), (8, 130, 4, 7, True)])
def test_round_equals_dense_row_stochastic_matmul(ref, N, P, S, R, weighted):
    rng = np.random.default_rng(N * 1000 + P)
    X = rng.normal(0, 0.05, (N, P)).astype(np.float32)
    d = rng.integers(100, 2000, N).astype(np.float32) if weighted else None
    peers = ref.make_peer_table(N, S, R, 3, 1)
    lo, hi = ref.segment_bounds(P, S)
    A = _dense_mixing(peers, N, S, R, d)
    want = np.empty((N, P))
    for s in range(S):
        want[:, lo[s]:hi[s]] = A[s] @ X[:, lo[s]:hi[s]].astype(np.float64)
    Y64 = ref.gossip_round_f64(X, peers, P, S, R, d=d)
    assert np.allclose(Y64, want, rtol=0, atol=1e-15)
    Y = ref.gossip_round(X, peers, P, S, R, d=d)
    # binary32: R adds (+ products) and one scale, each within 2^-24 relative
    bound = (R + 3) * 2.0 ** -24 * np.abs(X).max() * 1.01
    assert np.max(np.abs(Y.astype(np.float64) - want)) <= bound


def test_round_R0_is_the_identity_bitwise(ref):
    rng = np.random.default_rng(3)
    X = rng.normal(0, 1, (5, 1001)).astype(np.float32)
    peers = np.empty((5, 4, 0), np.int32)
    Y = ref.gossip_round(X, peers, P=1001, S=4, R=0)
    assert np.array_equal(Y.view(np.uint32), X.view(np.uint32))


def test_round_all_peers_is_the_fedavg_mean(ref):
    """R = N-1: every worker ends at the global mean (Sec. 4.3).  Each row sums the same
    N numbers in its own order, so agreement with the float64 column mean is to
    N * 2^-24 * max|x|, not bitwise."""
    N, P, S = 12, 5003, 5
    rng = np.random.default_rng(4)
    X = rng.normal(0, 0.02, (N, P)).astype(np.float32)
    peers = ref.make_peer_table(N, S, N - 1, 0, 0)
    Y = ref.gossip_round(X, peers, P, S, N - 1)
    mean = X.astype(np.float64).mean(axis=0)
    assert np.max(np.abs(Y - mean[None, :])) <= (N + 1) * 2.0 ** -24 * np.abs(X).max()
    Y64 = ref.gossip_round_f64(X, peers, P, S, N - 1)
    assert np.allclose(Y64, np.broadcast_to(mean, (N, P)), rtol=0, atol=1e-16)


def test_round_S1_is_whole_model_gossip(ref):
    """S = 1: each worker averages whole rows of its R peers (plain gossip, Sec. 5.1)."""
    N, P, R = 7, 333, 2
    rng = np.random.default_rng(5)
    X = rng.normal(0, 1, (N, P)).astype(np.float32)
    peers = ref.make_peer_table(N, 1, R, 9, 0)
    Y = ref.gossip_round(X, peers, P, 1, R)
    for w in range(N):
        acc = X[w].copy()
        for j in range(R):
            acc = acc + X[peers[w, 0, j]]            # numpy float32 vector adds, same order
        assert np.array_equal(Y[w], acc * np.float32(1.0 / 3.0))


def test_round_invariants(ref):
    N, P, S, R = 10, 4099, 6, 3
    rng = np.random.default_rng(6)
    X = rng.uniform(-0.1, 0.1, (N, P)).astype(np.float32)
    peers = ref.make_peer_table(N, S, R, 1, 2)
    Y = ref.gossip_round(X, peers, P, S, R)
    # convex combination: stays inside the per-column hull (1 ulp slack)
    eps = 2.0 ** -23 * 0.1
    assert np.all(Y <= X.max(axis=0)[None, :] + eps) and np.all(Y >= X.min(axis=0)[None, :] - eps)
    # a column that is constant across workers stays constant (to 2 ulp) and rows agree bitwise
    Xc = np.repeat(X[:1], N, axis=0)
    Yc = ref.gossip_round(Xc, peers, P, S, R)
    assert np.all(Yc.view(np.uint32) == Yc[:1].view(np.uint32))
    assert np.max(np.abs(Yc - Xc)) <= 2 * 2.0 ** -24 * 0.1 * 1.01
    # linearity
    Z = rng.normal(0, 0.05, (N, P)).astype(np.float32)
    lhs = ref.gossip_round_f64((2 * X + 3 * Z).astype(np.float32), peers, P, S, R)
    rhs = 2 * ref.gossip_round_f64(X, peers, P, S, R) + 3 * ref.gossip_round_f64(Z, peers, P, S, R)
    assert np.max(np.abs(lhs - rhs)) < 1e-6
    # mass is NOT conserved in general (the mixing matrix is only row-stochastic), but a
    # second round never widens the per-column range
    Y2 = ref.gossip_round(Y, ref.make_peer_table(N, S, R, 1, 3), P, S, R)
    assert np.all(np.ptp(Y2, axis=0) <= np.ptp(Y, axis=0) + eps)


def test_round_writes_each_element_once_and_leaves_padding(ref):
    N, P, S, R, ld = 5, 1003, 7, 2, 1024
    rng = np.random.default_rng(7)
    Xbuf = np.full((N, ld), np.float32(777.0))
    Xbuf[:, :P] = rng.normal(0, 1, (N, P)).astype(np.float32)
    Ybuf = np.full((N, ld), np.nan, np.float32)
    peers = ref.make_peer_table(N, S, R, 0, 0)
    ref.gossip_round(Xbuf[:, :P], peers, P, S, R, out=Ybuf[:, :P])
    assert not np.any(np.isnan(Ybuf[:, :P]))
    assert np.all(np.isnan(Ybuf[:, P:]))
    assert np.all(Xbuf[:, P:] == 777.0)
    # the padding was not read either: the result equals the one on a tight copy
    tight = np.ascontiguousarray(Xbuf[:, :P])
    assert np.array_equal(ref.gossip_round(tight, peers, P, S, R), Ybuf[:, :P])


def test_round_is_column_separable(ref):
    """A window of the round equals the round on the window (used to check samples of
    rounds too large to recompute in full)."""
    N, P, S, R = 6, 10007, 7, 3
    rng = np.random.default_rng(8)
    X = rng.normal(0, 0.02, (N, P)).astype(np.float32)
    peers = ref.make_peer_table(N, S, R, 0, 0)
    full = ref.gossip_round(X, peers, P, S, R)
    for c0, nc in [(0, 100), (1400, 100), (1429 - 3, 7), (P - 50, 50), (4000, 3000)]:
        win = np.ascontiguousarray(X[:, c0:c0 + nc])
        assert np.array_equal(ref.gossip_round(win, peers, P, S, R, col0=c0), full[:, c0:c0 + nc])


def test_weighted_with_equal_sizes_matches_uniform(ref):
    N, P, S, R = 8, 2050, 4, 3
    rng = np.random.default_rng(9)
    X = rng.normal(0, 0.05, (N, P)).astype(np.float32)
    peers = ref.make_peer_table(N, S, R, 0, 0)
    Yu = ref.gossip_round(X, peers, P, S, R)
    Yw = ref.gossip_round(X, peers, P, S, R, d=np.full(N, 500, np.float32))
    # power-of-two-free scale: products round, so agreement is a few ulp of max|x|
    assert np.max(np.abs(Yu - Yw)) <= (R + 3) * 2.0 ** -24 * np.abs(X).max()
    # sizes equal to 1: products exact, sum order identical, /4 == *0.25 exactly
    Y1 = ref.gossip_round(X, peers, P, S, R, d=np.ones(N, np.float32))
    assert np.array_equal(Y1, Yu)


# -------------------------------------------------------- local step, then aggregation
def test_fused_lr0_equals_plain_round(ref):
    N, P, S, R = 6, 999, 7, 3
    rng = np.random.default_rng(10)
    X = rng.uniform(-0.1, 0.1, (N, P)).astype(np.float32)
    G = rng.normal(0, 1e-3, (N, P)).astype(np.float32)
    peers = ref.make_peer_table(N, S, R, 0, 0)
    want = ref.gossip_round(X, peers, P, S, R)
    Xc = X.copy()
    got = ref.local_sgd_then_gossip(Xc, G, 0.0, peers, P, S, R)
    assert np.array_equal(got, want) and np.array_equal(Xc, X)


def test_fused_hand_worked(ref):
    """lr = 0.5, gradients even integers: x - 0.5*g is exact.  N=3, P=4, S=2, R=1."""
    X = _f32([[4, 8, 12, 16], [2, 2, 2, 2], [10, 20, 30, 40]])
    G = _f32([[4, 4, 4, 4], [-4, 0, 4, 8], [0, 8, 20, 40]])
    # stepped: [[2,6,10,14],[4,2,0,-2],[10,16,20,20]]
    peers = np.array([[[1], [2]], [[2], [0]], [[0], [1]]], np.int32)
    want = _f32([[3, 4, 15, 17], [7, 9, 5, 6], [6, 11, 10, 9]])
    Xc = X.copy()
    got = ref.local_sgd_then_gossip(Xc, G, 0.5, peers, P=4, S=2, R=1)
    assert np.array_equal(got, want)
    assert np.array_equal(Xc, _f32([[2, 6, 10, 14], [4, 2, 0, -2], [10, 16, 20, 20]]))


def test_fused_every_row_is_stepped_before_any_is_averaged(ref):
    """Matmul form A_s (X - lr G) in float64: would fail if peers' rows were read
    un-stepped (Sec. 4.1: segments are served after the provider's local update)."""
    N, P, S, R, lr = 7, 1003, 7, 3, 0.01
    rng = np.random.default_rng(11)
    X = rng.uniform(-0.1, 0.1, (N, P)).astype(np.float32)
    G = rng.normal(0, 1.0, (N, P)).astype(np.float32)       # large, so a missing step shows
    peers = ref.make_peer_table(N, S, R, 0, 0)
    lo, hi = ref.segment_bounds(P, S)
    A = _dense_mixing(peers, N, S, R)
    Xs = X.astype(np.float64) - np.float64(np.float32(lr)) * G.astype(np.float64)
    want = np.empty((N, P))
    for s in range(S):
        want[:, lo[s]:hi[s]] = A[s] @ Xs[:, lo[s]:hi[s]]
    got = ref.local_sgd_then_gossip(X.copy(), G, lr, peers, P, S, R)
    assert np.max(np.abs(got - want)) <= (R + 5) * 2.0 ** -24 * np.abs(Xs).max()
    # constant gradient, identical rows: Y = X - lr*G up to 2 ulp
    Xi = np.repeat(X[:1], N, axis=0)
    Gi = np.full((N, P), np.float32(0.25))
    got = ref.local_sgd_then_gossip(Xi.copy(), Gi, lr, peers, P, S, R)
    assert np.max(np.abs(got - (Xi - np.float32(lr) * np.float32(0.25)))) <= 3 * 2.0 ** -24 * 0.11


def test_f32_and_f64_oracles_agree_to_rounding(ref):
    N, P, S, R = 32, 20011, 32, 4
    rng = np.random.default_rng(12)
    X = rng.normal(0, 0.02, (N, P)).astype(np.float32)
    peers = ref.make_peer_table(N, S, R, 0, 0)
    Y = ref.gossip_round(X, peers, P, S, R)
    Y64 = ref.gossip_round_f64(X, peers, P, S, R)
    assert np.max(np.abs(Y - Y64)) / np.max(np.abs(Y64)) < 1e-6


def test_planted_mistakes_are_caught(ref):
    """Sanity of the pins themselves: plausible wrong variants of the round, written
    here in numpy, fail the hand-worked example."""
    X = _f32([[3, 6, 9, 12, 15, 18], [0, 3, 30, 6, 9, 3], [9, 0, 3, 0, 3, 9]])
    peers = np.array([[[1], [2]], [[2], [0]], [[0], [1]]], np.int32)
    good = ref.gossip_round(X, peers, P=6, S=2, R=1)
    no_self = np.stack([np.concatenate([X[peers[w, 0, 0], :3], X[peers[w, 1, 0], 3:]]) for w in range(3)])
    transposed = np.stack([np.concatenate([(X[w, :3] + X[peers[w, 1, 0], :3]) / 2,
                                           (X[w, 3:] + X[peers[w, 0, 0], 3:]) / 2]) for w in range(3)])
    assert not np.array_equal(good, no_self) and not np.array_equal(good, transposed)


# ------------------------------------------- several local steps (interval tau), then a round
def test_multi_step_tau1_is_the_single_step(ref):
    N, P, S, R = 6, 999, 7, 3
    rng = np.random.default_rng(20)
    X = rng.uniform(-0.1, 0.1, (N, P)).astype(np.float32)
    G = rng.normal(0, 1e-2, (1, N, P)).astype(np.float32)
    peers = ref.make_peer_table(N, S, R, 0, 0)
    a, b = X.copy(), X.copy()
    ya = ref.local_sgd_steps_then_gossip(a, G, 0.01, peers, P, S, R)
    yb = ref.local_sgd_then_gossip(b, np.ascontiguousarray(G[0]), 0.01, peers, P, S, R)
    assert np.array_equal(ya, yb) and np.array_equal(a, b)
    # tau = 0: no local step at all
    c = X.copy()
    y0 = ref.local_sgd_steps_then_gossip(c, G[:0], 0.01, peers, P, S, R)
    assert np.array_equal(y0, ref.gossip_round(X, peers, P, S, R)) and np.array_equal(c, X)


def test_multi_step_equals_numpy_float32_passes(ref):
    """tau elementwise binary32 passes x <- x - lr*g done by numpy (IEEE multiply and
    subtract, no fusion), in step order, then the pinned round."""
    N, P, S, R, tau = 5, 1003, 4, 2, 4
    rng = np.random.default_rng(21)
    X = rng.uniform(-0.1, 0.1, (N, P)).astype(np.float32)
    G = rng.normal(0, 1.0, (tau, N, P)).astype(np.float32)
    lr = np.float32(0.1)
    peers = ref.make_peer_table(N, S, R, 1, 1)
    Xs = X.copy()
    for k in range(tau):
        Xs = Xs - lr * G[k]
        assert Xs.dtype == np.float32
    Xc = X.copy()
    Y = ref.local_sgd_steps_then_gossip(Xc, G, float(lr), peers, P, S, R)
    assert np.array_equal(Xc, Xs)
    assert np.array_equal(Y, ref.gossip_round(Xs, peers, P, S, R))
    # order of the steps matters in binary32: reversing the gradients changes some bits
    Xr = X.copy()
    ref.local_sgd_steps_then_gossip(Xr, np.ascontiguousarray(G[::-1]), float(lr), peers, P, S, R)
    assert not np.array_equal(Xr, Xs) and np.allclose(Xr, Xs, rtol=0, atol=1e-6)
