"""GPU parity for the table-free round (peer selection + local steps + aggregation in one
launch): must equal the oracle's table followed by the oracle's round, bit for bit."""
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


def np_unpack(flat, N, P, Wt):
    T = -(-P // Wt)
    return np.ascontiguousarray(flat.reshape(T, N, Wt).transpose(1, 0, 2).reshape(N, T * Wt)[:, :P])


CASES = [
    # N, P, S, R
    (4, 65_536, 8, 2), (5, 10_007, 7, 3), (8, 40_001, 3, 4), (32, 9_999, 32, 4), (7, 4_096, 1, 2),
    (6, 130, 130, 1), (9, 5_000, 2, 0), (9, 20_000, 5, 8), (100, 20_003, 7, 3), (2, 8_193, 2, 1),
    (32, 70_000, 32, 4), (16, 30_011, 4, 7), (1, 3_000, 3, 0), (200, 3_001, 3, 5),
    # many workers: narrow tiles (the row-major slab does not fit: tiled only)
    (300, 4_003, 4, 3), (600, 2_001, 3, 2),
]


@pytest.mark.parametrize("N,P,S,R", CASES)
@pytest.mark.parametrize("layout", ["rows", "tiled"])
@pytest.mark.parametrize("mode", ["plain", "weighted", "fused2"])
def test_hashed_round_matches_oracle(combo, ref, N, P, S, R, layout, mode):
    if layout == "rows" and combo.round_kernel_kind(N, R) != 1:
        pytest.skip("N rows of 64 columns do not fit in LDS: the one-launch round needs the tiled arena")
    rng = np.random.default_rng(N * 17 + P + R)
    seed, rnd = int(rng.integers(0, 2**63)), int(rng.integers(0, 2**30))
    Xh = rng.normal(0, 0.05, (N, P)).astype(np.float32)
    tau = 2 if mode == "fused2" else 0
    Gh = rng.normal(0, 1e-2, (tau, N, P)).astype(np.float32)
    d_h = rng.integers(100, 2000, N).astype(np.float32) if mode == "weighted" else None
    T = ref.make_peer_table(N, S, R, seed, rnd)
    if tau:
        want = ref.local_sgd_steps_then_gossip(Xh.copy(), Gh, 0.05, T, P, S, R)
    else:
        want = ref.gossip_round(Xh, T, P, S, R, d=d_h)
    d = None if d_h is None else torch.from_numpy(d_h).cuda()
    ld = combo.workloads.row_pitch(P)
    rows = torch.full((N, ld), float("nan"), dtype=torch.float32, device="cuda")
    rows[:, :P] = torch.from_numpy(Xh).cuda()
    grows = torch.zeros((max(tau, 1), N, ld), dtype=torch.float32, device="cuda")
    if tau:
        grows[:, :, :P] = torch.from_numpy(Gh).cuda()
    if layout == "tiled":
        Wt = combo.tiled_cols(N, R)
        n = combo.tiled_elems(N, P, Wt)
        src = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
        dst = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
        combo.pack_tiled(src, rows, N, P, Wt)
        g = None
        if tau:
            g = torch.zeros((tau, n), dtype=torch.float32, device="cuda")
            for k in range(tau):
                combo.pack_tiled(g[k], grows[k], N, P, Wt)
        combo.round_hashed(dst, src, N, P, S, R, seed, rnd, grads=g, lr=0.05, tile_cols=Wt, dataset_sizes=d)
        torch.cuda.synchronize()
        got = np_unpack(dst.cpu().numpy(), N, P, Wt)
    else:
        out = torch.full((N, ld), float("nan"), dtype=torch.float32, device="cuda")
        combo.round_hashed(out, rows, N, P, S, R, seed, rnd, grads=grows[:tau] if tau else None, lr=0.05,
                           dataset_sizes=d)
        torch.cuda.synchronize()
        got = out[:, :P].cpu().numpy()
        assert bool(torch.isnan(out[:, P:]).all())
        assert np.array_equal(rows[:, :P].cpu().numpy(), Xh)           # source never modified
    assert np.all(np.abs(got - want) <= 1e-6 * np.maximum(np.abs(want), 1e-30))
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_hashed_round_errors(combo):
    a = torch.zeros((20, 1024), dtype=torch.float32, device="cuda")
    b = torch.zeros_like(a)
    with pytest.raises(combo.ComboError) as e:                      # R > 8: use the table
        combo.round_hashed(b, a, 20, 1000, 4, 9, 0, 0)
    assert e.value.status == -3
    with pytest.raises(combo.ComboError) as e:
        combo.round_hashed(a, a, 20, 1000, 4, 2, 0, 0)
    assert e.value.status == -2
    big = torch.zeros((300, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(combo.ComboError) as e:                      # slab does not fit
        combo.round_hashed(torch.zeros_like(big), big, 300, 64, 2, 2, 0, 0)
    assert e.value.status == -3


def test_hashed_full_size_benchmark_workload(combo, ref):
    """c2 at full size, tiled layout, three rounds of the one-launch path, on windows."""
    import tests.test_gpu_parity as tp
    wl = combo.workloads.WORKLOADS["c2_resnet18"]
    arena = combo.GossipArena(wl.N, wl.P, wl.S, wl.R, layout="tiled", seed=wl.hash_seed)
    rows = torch.zeros((wl.N, wl.ld), dtype=torch.float32, device="cuda")
    combo.workloads.fill_params(rows, wl)
    arena.load(rows)
    wins = tp.sample_windows(wl)
    X0 = {w: rows[:, w[0]:w[0] + w[1]].cpu().numpy() for w in wins}
    cur, other = arena.front, arena.back
    for rnd in range(3):
        combo.round_hashed(other, cur, wl.N, wl.P, wl.S, wl.R, wl.hash_seed, rnd, tile_cols=arena.tile_cols)
        cur, other = other, cur
    combo.unpack_tiled(rows, cur, wl.N, wl.P, arena.tile_cols)
    torch.cuda.synchronize()
    for w in wins:
        want = tp.oracle_rounds_on_window(ref, wl, X0[w], w[0], 3)
        assert np.array_equal(rows[:, w[0]:w[0] + w[1]].cpu().numpy().view(np.uint32), want.view(np.uint32)), w
