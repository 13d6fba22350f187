"""Pins for the oracle's dynamic-worker functions (Sec. 4.2 of the paper: workers that
drop out are marked offline and the request goes to someone else; a newcomer pulls and
aggregates as normal but without its local model, and is not yet a provider).  CPU only.
status: 0 = offline, 1 = active, 2 = newcomer."""
import numpy as np
import pytest


def _f32(a):
    return np.array(a, dtype=np.float32)


@pytest.mark.parametrize("N,S,R", [(4, 8, 2), (32, 32, 4), (100, 7, 3), (7, 3, 6), (2, 2, 1), (1, 3, 0)])
def test_all_active_reduces_to_the_static_functions(ref, N, S, R):
    st = np.ones(N, np.uint8)
    T = ref.make_peer_table_dynamic(st, N, S, R, 5, 6)
    assert np.array_equal(T, ref.make_peer_table(N, S, R, 5, 6))
    P = 501
    X = np.random.default_rng(N).normal(0, 0.05, (N, P)).astype(np.float32)
    if S <= P:
        for d in (None, np.random.default_rng(1).integers(100, 2000, N).astype(np.float32)):
            a = ref.gossip_round_dynamic(X, T, st, P, S, R, d=d)
            b = ref.gossip_round(X, T, P, S, R, d=d)
            assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


def test_selection_respects_status(ref):
    N, S, R = 12, 6, 3
    st = np.ones(N, np.uint8)
    st[[2, 7]] = 0          # offline
    st[[4, 11]] = 2         # newcomers
    for rnd in range(5):
        T = ref.make_peer_table_dynamic(st, N, S, R, 3, rnd)
        assert np.all(T[[2, 7]] == -1)                       # offline workers ask nobody
        asked = T[st != 0]
        assert asked.min() >= 0                               # 8 active others >= R: all slots used
        assert not np.isin(asked, [2, 7, 4, 11]).any()        # nobody asks offline or newcomers
        for w in np.nonzero(st)[0]:
            for s in range(S):
                row = T[w, s].tolist()
                assert w not in row and len(set(row)) == R


def test_selection_with_fewer_candidates_than_R(ref):
    # N=5, R=3, workers 1 and 3 offline, 4 a newcomer: candidates for w=0 are {2}, for
    # w=2 {0}, for the newcomer {0, 2}
    st = np.array([1, 0, 1, 0, 2], np.uint8)
    T = ref.make_peer_table_dynamic(st, 5, 4, 3, 0, 0)
    assert np.all(T[0] == [2, -1, -1]) and np.all(T[2] == [0, -1, -1])
    assert np.all(T[1] == -1) and np.all(T[3] == -1)
    for s in range(4):
        assert sorted(T[4, s, :2].tolist()) == [0, 2] and T[4, s, 2] == -1
    # a lone active worker has nobody to ask
    st = np.array([0, 1, 0], np.uint8)
    assert np.all(ref.make_peer_table_dynamic(st, 3, 2, 2, 0, 0) == -1)


def test_selection_is_uniform_over_the_active_others(ref):
    N = 9
    st = np.ones(N, np.uint8)
    st[[1, 5]] = 0
    st[8] = 2
    first = np.concatenate([ref.make_peer_table_dynamic(st, N, 20, 2, 11, r)[0, :, 0] for r in range(100)])
    h = np.bincount(first, minlength=N)
    assert h[[0, 1, 5, 8]].sum() == 0
    cand = [2, 3, 4, 6, 7]
    e = len(first) / len(cand)
    assert float(np.sum((h[cand] - e) ** 2 / e)) < 23.5       # 4 dof, 99.99 %


def test_round_hand_worked_with_offline_and_newcomer(ref):
    """N=4, P=4, S=2, R=2.  w1 offline, w3 newcomer.
       w0 (active): seg0 terms (self, w2)      -> (x0+x2)/2 ; seg1 terms (self, w2) -> same
       w1 (offline): unchanged
       w2 (active): seg0 (self, w0), seg1 (self, w0)
       w3 (newcomer): seg0 terms (w0, w2) -> (x0+x2)/2 without its own value; seg1 (w2, w0)"""
    st = np.array([1, 0, 1, 2], np.uint8)
    X = _f32([[2, 4, 6, 8], [100, 100, 100, 100], [4, 8, 2, 0], [1000, 1000, 1000, 1000]])
    T = np.array([[[2, -1], [2, -1]], [[-1, -1], [-1, -1]], [[0, -1], [0, -1]], [[0, 2], [2, 0]]], np.int32)
    Y = ref.gossip_round_dynamic(X, T, st, P=4, S=2, R=2)
    want = _f32([[3, 6, 4, 4], [100, 100, 100, 100], [3, 6, 4, 4], [3, 6, 4, 4]])
    assert np.array_equal(Y, want)
    # weighted: d = (1, 9, 3, 5): w0 seg -> (1*x0 + 3*x2)/4 ; newcomer -> (1*x0 + 3*x2)/4 and (3*x2 + 1*x0)/4
    d = _f32([1, 9, 3, 5])
    Yw = ref.gossip_round_dynamic(X, T, st, P=4, S=2, R=2, d=d)
    m = _f32([(2 + 12) / 4, (4 + 24) / 4, (6 + 6) / 4, (8 + 0) / 4])
    assert np.array_equal(Yw, np.stack([m, X[1], m, m]))


def test_rows_that_must_not_be_read_are_not_read(ref):
    """Offline rows and newcomers' own rows are poisoned with NaN: no active worker and
    no newcomer result may see them."""
    N, P, S, R = 10, 403, 5, 3
    rng = np.random.default_rng(2)
    st = np.ones(N, np.uint8)
    st[[3, 6]] = 0
    st[[0, 9]] = 2
    X = rng.normal(0, 0.05, (N, P)).astype(np.float32)
    X[[3, 6, 0, 9]] = np.nan
    T = ref.make_peer_table_dynamic(st, N, S, R, 1, 1)
    Y = ref.gossip_round_dynamic(X, T, st, P, S, R)
    assert np.isnan(Y[[3, 6]]).all()                          # offline rows are copied as they are
    assert not np.isnan(np.delete(Y, [3, 6], axis=0)).any()


@pytest.mark.parametrize("weighted", [False, True])
def test_dynamic_round_equals_dense_matmul(ref, weighted):
    N, P, S, R = 9, 700, 7, 4
    rng = np.random.default_rng(5)
    st = np.array([1, 1, 0, 1, 2, 1, 1, 0, 2], np.uint8)
    X = rng.normal(0, 0.05, (N, P)).astype(np.float32)
    d = rng.integers(100, 2000, N).astype(np.float32) if weighted else None
    dd = np.ones(N) if d is None else d.astype(np.float64)
    T = ref.make_peer_table_dynamic(st, N, S, R, 2, 3)
    lo, hi = ref.segment_bounds(P, S)
    want = np.empty((N, P))
    for s in range(S):
        A = np.zeros((N, N))
        for w in range(N):
            terms = ([w] if st[w] == 1 else []) + ([int(p) for p in T[w, s] if p >= 0] if st[w] else [])
            if not terms:
                A[w, w] = 1.0
            else:
                tot = sum(dd[t] for t in terms)
                for t in terms:
                    A[w, t] += dd[t] / tot
        want[:, lo[s]:hi[s]] = A @ X[:, lo[s]:hi[s]].astype(np.float64)
    Y = ref.gossip_round_dynamic(X, T, st, P, S, R, d=d)
    assert np.max(np.abs(Y - want)) <= (R + 3) * 2.0 ** -24 * np.abs(X).max() * 1.01


def test_newcomer_with_nobody_to_ask_keeps_its_parameters(ref):
    st = np.array([2, 0, 0], np.uint8)
    X = _f32([[1, 2, 3], [4, 5, 6], [7, 8, 9]])
    T = ref.make_peer_table_dynamic(st, 3, 1, 2, 0, 0)
    assert np.all(T == -1)
    assert np.array_equal(ref.gossip_round_dynamic(X, T, st, P=3, S=1, R=2), X)


def test_offline_worker_keeps_its_row_whatever_its_table_row_says(ref):
    """The round goes by the status, not by the table: an offline worker whose table row
    still holds stale valid entries does not aggregate."""
    N, P, S, R = 6, 50, 5, 2
    X = np.random.default_rng(1).normal(0, 1, (N, P)).astype(np.float32)
    T = ref.make_peer_table(N, S, R, 0, 0)             # every row full of valid entries
    st = np.array([1, 0, 1, 1, 0, 1], np.uint8)
    Y = ref.gossip_round_dynamic(X, T, st, P, S, R)
    assert np.array_equal(Y[[1, 4]], X[[1, 4]])
    assert not np.array_equal(Y[0], X[0])
