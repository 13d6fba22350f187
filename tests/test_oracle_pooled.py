"""Pins for the oracle's pooled peer selection (Sec. 4.1 step 2 of the paper read
literally: one pool of the other workers for all S*R requests of a worker, drawn
without replacement until no option is left) and the serve-load histogram.  CPU only."""
import numpy as np
import pytest

POOL_TAG = 0x706F6F6C65642121
M64 = (1 << 64) - 1


def _queue_model(ref, N, S, R, w, seed, rnd):
    """Independent re-implementation with a python list as the queue."""
    M = N - 1
    queue, epoch, out = [], 0, []
    for s in range(S):
        picks = []
        for j in range(R):
            if not queue:
                queue = [v for v in range(N) if v != w]
                for i in range(M - 1):
                    h = ref.peer_hash((seed ^ POOL_TAG) & M64, rnd, w, epoch, i)
                    r = i + (((h >> 32) * (M - i)) >> 32)
                    queue[i], queue[r] = queue[r], queue[i]
                epoch += 1
            k = next(k for k, v in enumerate(queue) if v not in picks)
            picks.append(queue.pop(k))
        out.append(picks)
    return out


@pytest.mark.parametrize("N,S,R,seed,rnd", [(30, 10, 2, 0, 0), (4, 8, 2, 0, 0), (32, 32, 4, 0, 3),
                                            (100, 7, 3, 5, 19), (5, 9, 4, 1, 1), (2, 3, 1, 0, 0),
                                            (7, 3, 6, 2, 2), (1, 4, 0, 0, 0), (16, 16, 0, 0, 0)])
def test_pooled_table_matches_queue_model(ref, N, S, R, seed, rnd):
    T = ref.make_peer_table_pooled(N, S, R, seed, rnd)
    assert T.shape == (N, S, R)
    for w in range(N):
        assert T[w].tolist() == _queue_model(ref, N, S, R, w, seed, rnd)


@pytest.mark.parametrize("N,S,R", [(30, 10, 2), (40, 10, 2), (21, 10, 2), (100, 7, 3), (17, 4, 4)])
def test_all_requests_go_to_different_workers_when_they_fit(ref, N, S, R):
    """S*R <= N-1 (the paper writes n): every one of a worker's S*R targets is distinct."""
    assert S * R <= N - 1
    for rnd in range(3):
        T = ref.make_peer_table_pooled(N, S, R, 9, rnd)
        for w in range(N):
            flat = T[w].ravel().tolist()
            assert len(set(flat)) == S * R and w not in flat


@pytest.mark.parametrize("N,S,R", [(4, 8, 2), (32, 32, 4), (5, 9, 4), (7, 3, 6), (20, 10, 2), (3, 50, 2)])
def test_pool_is_exhausted_before_it_is_refilled(ref, N, S, R):
    """Requests are spread evenly: per requesting worker every other worker is asked
    floor or ceil of S*R/(N-1) times; segments never hold a duplicate or the worker."""
    T = ref.make_peer_table_pooled(N, S, R, 4, 2)
    lo, hi = (S * R) // (N - 1), -(-(S * R) // (N - 1))
    for w in range(N):
        cnt = np.bincount(T[w].ravel(), minlength=N)
        assert cnt[w] == 0
        others = np.delete(cnt, w)
        assert others.min() >= lo and others.max() <= hi
        for s in range(S):
            assert len(set(T[w, s].tolist())) == R


def test_pooled_determinism_and_mode_independence(ref):
    a = ref.make_peer_table_pooled(32, 10, 2, 0, 5)
    assert np.array_equal(a, ref.make_peer_table_pooled(32, 10, 2, 0, 5))
    assert not np.array_equal(a, ref.make_peer_table_pooled(32, 10, 2, 0, 6))
    assert not np.array_equal(a, ref.make_peer_table_pooled(32, 10, 2, 1, 5))
    assert not np.array_equal(a, ref.make_peer_table(32, 10, 2, 0, 5))
    with pytest.raises(ValueError):
        ref.make_peer_table_pooled(4, 2, 4, 0, 0)


def test_pooled_first_target_is_uniform(ref):
    N = 11
    first = np.concatenate([ref.make_peer_table_pooled(N, 1, 1, 77, r)[:, 0, 0] for r in range(600)])
    who = np.tile(np.arange(N), 600)
    for w in (0, 5, 10):
        h = np.bincount(first[who == w], minlength=N)
        assert h[w] == 0
        e = 600 / (N - 1)
        chi2 = float(np.sum((np.delete(h, w) - e) ** 2 / e))
        assert chi2 < 35.6            # 9 dof, 99.995 %


def test_in_degree_is_a_bincount(ref):
    for maker in (ref.make_peer_table, ref.make_peer_table_pooled):
        T = maker(32, 32, 4, 0, 1)
        deg = ref.peer_in_degree(T, 32, 32, 4)
        assert np.array_equal(deg, np.bincount(T.ravel(), minlength=32))
        assert deg.sum() == 32 * 32 * 4
    # the pooled draw balances what each REQUESTER asks for, so the serve load is much
    # tighter than with independent draws per segment
    Tp = ref.make_peer_table_pooled(30, 10, 2, 0, 0)
    Ti = ref.make_peer_table(30, 10, 2, 0, 0)
    assert ref.peer_in_degree(Tp, 30, 10, 2).sum() == ref.peer_in_degree(Ti, 30, 10, 2).sum() == 600


def test_pooled_table_drives_the_round(ref):
    """The aggregation is agnostic to how the table was drawn."""
    N, P, S, R = 30, 1000, 10, 2
    X = np.random.default_rng(0).normal(0, 0.05, (N, P)).astype(np.float32)
    T = ref.make_peer_table_pooled(N, S, R, 0, 0)
    Y = ref.gossip_round(X, T, P, S, R)
    lo, hi = ref.segment_bounds(P, S)
    for w in (0, 17):
        for s in (0, 9):
            want = (X[w, lo[s]:hi[s]] + X[T[w, s, 0], lo[s]:hi[s]]) + X[T[w, s, 1], lo[s]:hi[s]]
            assert np.array_equal(Y[w, lo[s]:hi[s]], want * np.float32(1 / 3))
