"""GPU parity for the pooled peer selection and the serve-load histogram (integer work:
bit-exact against the CPU oracle), and the round driven by a pooled table."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def combo():
    import paper_1908_07782_amd as c
    assert torch.cuda.is_available()
    c.lib()
    return c


CASES = [(30, 10, 2, 0, 0), (4, 8, 2, 0, 0), (32, 32, 4, 0, 3), (32, 10, 2, 7, 9), (100, 7, 3, 5, 19),
         (16, 16, 4, 0, 4), (5, 9, 4, 1, 1), (2, 3, 1, 0, 0), (7, 3, 6, 2, 2), (100, 3, 99, 1, 0),
         (1000, 2, 5, 2**63 + 1, 2**33), (3, 200, 2, 8, 8),
         # around the limit of the register-resident kernel (64 candidates), R up to N-1 there,
         # segments that straddle many refills
         (65, 5, 64, 3, 1), (65, 7, 3, 0, 2), (66, 7, 3, 0, 2), (64, 9, 63, 4, 4), (33, 17, 5, 6, 6),
         (17, 40, 16, 1, 3), (2, 50, 1, 9, 9), (48, 64, 7, 2**40, 5), (9, 11, 8, 0, 1)]


@pytest.mark.parametrize("N,S,R,seed,rnd", CASES)
def test_pooled_table_bit_exact(combo, ref, N, S, R, seed, rnd):
    t = torch.full((N * S * R,), -7, dtype=torch.int32, device="cuda")
    combo.make_peer_table_pooled(t, N, S, R, seed, rnd)
    torch.cuda.synchronize()
    want = ref.make_peer_table_pooled(N, S, R, seed, rnd)
    assert np.array_equal(t.cpu().numpy().reshape(want.shape), want)


@pytest.mark.parametrize("N,S,R,seed,rnd", CASES[:8])
@pytest.mark.parametrize("pooled", [False, True])
def test_in_degree_bit_exact(combo, ref, N, S, R, seed, rnd, pooled):
    t = torch.empty(N * S * R, dtype=torch.int32, device="cuda")
    (combo.make_peer_table_pooled if pooled else combo.make_peer_table)(t, N, S, R, seed, rnd)
    deg = torch.full((N,), -1, dtype=torch.int32, device="cuda")
    combo.peer_in_degree(deg, t, N, S, R)
    torch.cuda.synchronize()
    want = ref.peer_in_degree(t.cpu().numpy(), N, S, R)
    assert np.array_equal(deg.cpu().numpy(), want) and int(deg.sum()) == N * S * R


def test_pooled_R0_and_errors(combo):
    combo.make_peer_table_pooled(None, 4, 2, 0, 0, 0)
    t = torch.empty(8, dtype=torch.int32, device="cuda")
    with pytest.raises(combo.ComboError):
        combo.make_peer_table_pooled(t, 2, 2, 2, 0, 0)


def test_round_with_pooled_table_paper_default(combo, ref):
    """The paper's default setting (S, R) = (10, 2) at 30 workers: S*R = 20 <= 29, so all
    of a worker's segments come from different providers; the round matches the oracle."""
    N, P, S, R = 30, 200_003, 10, 2
    Xh = np.random.default_rng(3).normal(0, 0.05, (N, P)).astype(np.float32)
    ld = combo.workloads.row_pitch(P)
    src = torch.zeros((N, ld), dtype=torch.float32, device="cuda")
    src[:, :P] = torch.from_numpy(Xh).cuda()
    dst = torch.zeros_like(src)
    t = torch.empty(N * S * R, dtype=torch.int32, device="cuda")
    combo.make_peer_table_pooled(t, N, S, R, 0, 0)
    combo.segment_gossip_round(dst, src, t, P, S, R)
    torch.cuda.synchronize()
    T = ref.make_peer_table_pooled(N, S, R, 0, 0)
    assert np.array_equal(t.cpu().numpy().reshape(T.shape), T)
    for w in range(N):
        assert len(set(T[w].ravel().tolist())) == S * R
    want = ref.gossip_round(Xh, T, P, S, R)
    got = dst[:, :P].cpu().numpy()
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
