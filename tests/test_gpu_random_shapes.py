"""Randomised GPU-vs-oracle parity: 84 seeded random shapes (N, P, S, R, pitch, layout,
weights, fused steps, dynamic status), each compared bit for bit with the CPU oracle."""
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


@pytest.mark.parametrize("case", range(84))
def test_random_case(combo, ref, case):
    rng = np.random.default_rng(1000 + case)
    if case < 60:
        N = int(rng.choice([1, 2, 3, 5, 8, 16, 31, 32, 33, 64, 100, 130, 257]))
        P = int(rng.choice([1, 7, 63, 64, 65, 1000, 4097, 20_011, 65_536, 100_003]))
    else:                                           # many workers: narrow tiles, row-tile fallback
        N = int(rng.choice([40, 129, 257, 400, 513, 700, 1000]))
        P = int(rng.choice([9, 500, 4097, 20_011]))
    S = int(rng.integers(1, min(P, 40) + 1))
    R = int(rng.integers(0, min(N - 1, 12) + 1))
    mode = rng.choice(["plain", "weighted", "fused", "dynamic"])
    layout = rng.choice(["rows", "rows_pitch", "tiled"])
    seed, rnd = int(rng.integers(0, 2**63)), int(rng.integers(0, 2**20))
    tau = int(rng.integers(1, 4)) if mode == "fused" else 0
    print(f"case {case}: N={N} P={P} S={S} R={R} {mode} {layout} tau={tau}", flush=True)

    Xh = rng.normal(0, 0.05, (N, P)).astype(np.float32)
    Gh = rng.normal(0, 1e-2, (tau, N, P)).astype(np.float32)
    d_h = rng.integers(100, 2000, N).astype(np.float32) if mode == "weighted" else None
    status = rng.integers(0, 3, N).astype(np.uint8) if mode == "dynamic" else None

    # oracle
    if mode == "dynamic":
        T = ref.make_peer_table_dynamic(status, N, S, R, seed, rnd)
        want = ref.gossip_round_dynamic(Xh, T, status, P, S, R)
    else:
        T = ref.make_peer_table(N, S, R, seed, rnd)
        if mode == "fused":
            want = ref.local_sgd_steps_then_gossip(Xh.copy(), Gh, 0.05, T, P, S, R)
        else:
            want = ref.gossip_round(Xh, T, P, S, R, d=d_h)

    # GPU
    peers = torch.full((max(N * S * R, 1),), -9, dtype=torch.int32, device="cuda")
    d = None if d_h is None else torch.from_numpy(d_h).cuda()
    st = None if status is None else torch.from_numpy(status).cuda()
    if mode == "dynamic":
        combo.make_peer_table_dynamic(peers, st, N, S, R, seed, rnd)
    else:
        combo.make_peer_table(peers, N, S, R, seed, rnd)
    use_tiled = layout == "tiled"
    Wt = 0
    if use_tiled:
        try:
            Wt = combo.tiled_cols(N, R)
        except combo.ComboError:
            use_tiled = False                      # too many workers for the LDS slab
    ld = combo.workloads.row_pitch(P) + (int(rng.integers(1, 9)) if layout == "rows_pitch" else 0)
    rows = torch.full((N, ld), float("nan"), dtype=torch.float32, device="cuda")
    rows[:, :P] = torch.from_numpy(Xh).cuda()
    grows = torch.zeros((max(tau, 1), N, ld), dtype=torch.float32, device="cuda")
    if tau:
        grows[:, :, :P] = torch.from_numpy(Gh).cuda()
    if use_tiled:
        n = combo.tiled_elems(N, P, Wt)
        src = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
        dst = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
        combo.pack_tiled(src, rows, N, P, Wt)
        if mode == "fused":
            gt = torch.zeros(n * tau, dtype=torch.float32, device="cuda")
            for k in range(tau):
                combo.pack_tiled(gt[k * n:(k + 1) * n], grows[k], N, P, Wt)
            combo.local_sgd_steps_then_gossip_tiled(dst, src, gt, tau, 0.05, Wt, peers, N, P, S, R)
        else:
            combo.segment_gossip_round_tiled(dst, src, Wt, peers if R else None, N, P, S, R,
                                             dataset_sizes=d, status=st)
        torch.cuda.synchronize()
        got = np_unpack(dst.cpu().numpy(), N, P, Wt)
    else:
        out = torch.full((N, ld), float("nan"), dtype=torch.float32, device="cuda")
        if mode == "fused":
            combo.local_sgd_steps_then_gossip(out, rows, grows[:tau], 0.05, peers, P, S, R)
        elif mode == "dynamic":
            combo.segment_gossip_round_dynamic(out, rows, peers if R else None, st, P, S, R)
        else:
            combo.segment_gossip_round(out, rows, peers if R else None, P, S, R, dataset_sizes=d)
        torch.cuda.synchronize()
        got = out[:, :P].cpu().numpy()
        assert bool(torch.isnan(out[:, P:]).all())
    assert np.array_equal(peers.cpu().numpy()[:N * S * R].reshape(T.shape), T)
    assert np.all(np.abs(got - want) <= 1e-6 * np.maximum(np.abs(want), 1e-30))
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
