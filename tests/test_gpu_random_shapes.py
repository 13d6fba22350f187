"""Randomised GPU-vs-oracle parity: 84 seeded random shapes (N, P, S, R, pitch, layout,
weights, fused steps, dynamic status) through the single-layout entry points and 72 more through
the round between layouts under random performance knobs, each compared bit for bit with the CPU
oracle."""
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


@pytest.mark.parametrize("case", range(72))
def test_random_case_between_layouts_and_under_random_knobs(combo, ref, case):
    """Random shapes through combo_round_relayout (any pair of layouts), with many short
    segments, up to 20 replicas, and the performance knobs (strip order, workgroup size, LDS
    floor) set at random: results never depend on them."""
    from tests.test_gpu_relayout import Side, bits
    from tests.test_gpu_tiled import np_pack
    rng = np.random.default_rng(5000 + case)
    N = int(rng.choice([2, 3, 5, 8, 16, 21, 32, 33, 64, 100]))
    P = int(rng.choice([64, 65, 1000, 4097, 20_011, 65_536, 100_003]))
    S = int(rng.choice([1, 2, 7, min(P, 40), min(P, 333), min(P, 5000), P]))
    R = int(rng.integers(0, min(N - 1, 20) + 1))
    mode = rng.choice(["plain", "weighted", "fused", "dynamic", "dynamic+weights"])
    src_l, dst_l = rng.choice(["rows", "tiled"]), rng.choice(["rows", "tiled"])
    seed, rnd = int(rng.integers(0, 2**63)), int(rng.integers(0, 2**20))
    tau = int(rng.integers(1, 3)) if mode == "fused" else 0
    order = int(rng.choice([0, 1, 2, 5, 16]))
    threads = int(rng.choice([0, 256, 512]))
    floor = int(rng.choice([0, 1, 32 * 1024]))
    print(f"case {case}: N={N} P={P} S={S} R={R} {mode} {src_l}->{dst_l} tau={tau} order={order} "
          f"threads={threads} floor={floor}", flush=True)
    Xh = rng.normal(0, 0.05, (N, P)).astype(np.float32)
    Gh = rng.normal(0, 1e-2, (tau, N, P)).astype(np.float32)
    d_h = rng.integers(100, 2000, N).astype(np.float32) if "weight" in mode else None
    status = rng.integers(0, 3, N).astype(np.uint8) if mode.startswith("dynamic") else None
    if status is not None:
        T = ref.make_peer_table_dynamic(status, N, S, R, seed, rnd)
        want = ref.gossip_round_dynamic(Xh, T, status, P, S, R, d=d_h)
    else:
        T = ref.make_peer_table(N, S, R, seed, rnd)
        want = ref.local_sgd_steps_then_gossip(Xh.copy(), Gh, 0.05, T, P, S, R) if tau \
            else ref.gossip_round(Xh, T, P, S, R, d=d_h)

    Wt = combo.tiled_cols(N, R)
    src = Side(combo, N, P, Wt if src_l == "tiled" else 0, Xh)
    dst = Side(combo, N, P, Wt if dst_l == "tiled" else 0, None, extra_pitch=int(rng.choice([0, 4, 64])))
    grads = None
    if tau:
        if src.tile:
            grads = torch.stack([torch.from_numpy(np.nan_to_num(np_pack(Gh[k], Wt))).cuda() for k in range(tau)])
        else:
            grads = torch.zeros((tau,) + tuple(src.t.shape), dtype=torch.float32, device="cuda")
            grads[:, :, :P] = torch.from_numpy(Gh).cuda()
    peers = torch.from_numpy(np.ascontiguousarray(T).reshape(-1)).cuda() if R else None
    d = None if d_h is None else torch.from_numpy(d_h).cuda()
    st = None if status is None else torch.from_numpy(status).cuda()
    try:
        combo.tune(combo.TUNE_SLAB_ORDER, order)
        combo.tune(combo.TUNE_SLAB_THREADS, threads)
        combo.tune(combo.TUNE_SLAB_LDS_FLOOR, floor)
        combo.round_relayout(dst.t, dst.tile, src.t, src.tile, peers, N, P, S, R, grads=grads, lr=0.05,
                             dataset_sizes=d, status=st)
        torch.cuda.synchronize()
    finally:
        combo.tune(combo.TUNE_SLAB_ORDER, 0)
        combo.tune(combo.TUNE_SLAB_THREADS, 0)
        combo.tune(combo.TUNE_SLAB_LDS_FLOOR, 0)
    got, pad_ok = dst.values()
    nan_ok = np.array_equal(np.isnan(got), np.isnan(want))
    assert nan_ok and pad_ok
    ok = ~np.isnan(want)
    assert np.array_equal(bits(got)[ok], bits(want)[ok])
    assert np.array_equal(bits(src.values()[0]), bits(Xh))
