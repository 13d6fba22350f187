"""GPU parity for the tiled arena layout [T][N][Wt].  The layout itself is pinned against
numpy (pad the columns to T*Wt, reshape to (N, T, Wt), move the tile axis first); the
rounds on tiled buffers must equal the CPU oracle's row-major results bit for bit."""
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


def np_pack(X, Wt, fill=np.nan):
    N, P = X.shape
    T = -(-P // Wt)
    pad = np.full((N, T * Wt), fill, np.float32)
    pad[:, :P] = X
    return np.ascontiguousarray(pad.reshape(N, T, Wt).transpose(1, 0, 2)).reshape(-1)


def np_unpack(flat, N, P, Wt):
    T = -(-P // Wt)
    return np.ascontiguousarray(flat.reshape(T, N, Wt).transpose(1, 0, 2).reshape(N, T * Wt)[:, :P])


def to_tiled(combo, Xh, Wt):
    """Upload row-major, convert on the GPU; padding of the tiled buffer pre-set to NaN."""
    N, P = Xh.shape
    ld = combo.workloads.row_pitch(P)
    rows = torch.zeros((N, ld), dtype=torch.float32, device="cuda")
    rows[:, :P] = torch.from_numpy(Xh).cuda()
    tiled = torch.full((combo.tiled_elems(N, P, Wt),), float("nan"), dtype=torch.float32, device="cuda")
    combo.pack_tiled(tiled, rows, N, P, Wt)
    return tiled


@pytest.mark.parametrize("N,P,Wt", [(4, 1000, 64), (5, 10_007, 128), (32, 40_001, 64), (3, 64, 64),
                                    (7, 63, 64), (16, 100_000, 1024), (100, 5_003, 64),
                                    (300, 2_001, 16), (5, 1_003, 8), (70, 999, 32), (3, 7, 8)])
def test_pack_and_unpack_match_numpy(combo, N, P, Wt):
    Xh = np.random.default_rng(P).normal(0, 1, (N, P)).astype(np.float32)
    tiled = to_tiled(combo, Xh, Wt)
    torch.cuda.synchronize()
    want = np_pack(Xh, Wt)
    got = tiled.cpu().numpy()
    assert got.size == combo.tiled_elems(N, P, Wt) == want.size
    assert np.array_equal(np.isnan(got), np.isnan(want))            # padding untouched
    assert np.array_equal(got[~np.isnan(want)], want[~np.isnan(want)])
    ld = combo.workloads.row_pitch(P) + 64
    back = torch.full((N, ld), float("nan"), dtype=torch.float32, device="cuda")
    combo.unpack_tiled(back, tiled, N, P, Wt)
    torch.cuda.synchronize()
    assert np.array_equal(back[:, :P].cpu().numpy(), Xh) and bool(torch.isnan(back[:, P:]).all())
    assert np.array_equal(np_unpack(want, N, P, Wt), Xh)


@pytest.mark.parametrize("ld_extra,offset", [(1, 0), (0, 1), (3, 2), (4, 4)])
def test_pack_and_unpack_any_pitch_and_alignment(combo, ld_extra, offset):
    """Row pitches that are not multiples of four and base pointers off the 16-byte grid take
    the scalar conversion; (4, 4) is aligned again and takes the 128-bit one."""
    N, P, Wt = 6, 3_003, 64
    Xh = np.random.default_rng(1).normal(0, 1, (N, P)).astype(np.float32)
    ld = 3_008 + ld_extra
    raw = torch.full((N * ld + offset + 4,), float("nan"), dtype=torch.float32, device="cuda")
    rows = raw[offset:offset + N * ld].view(N, ld)
    rows[:, :P] = torch.from_numpy(Xh).cuda()
    tiled = torch.full((combo.tiled_elems(N, P, Wt),), float("nan"), dtype=torch.float32, device="cuda")
    combo.pack_tiled(tiled, rows, N, P, Wt)
    want = np_pack(Xh, Wt)
    got = tiled.cpu().numpy()
    assert np.array_equal(np.isnan(got), np.isnan(want))
    assert np.array_equal(got[~np.isnan(want)], want[~np.isnan(want)])
    raw2 = torch.full_like(raw, float("nan"))
    back = raw2[offset:offset + N * ld].view(N, ld)
    combo.unpack_tiled(back, tiled, N, P, Wt)
    torch.cuda.synchronize()
    assert np.array_equal(back[:, :P].cpu().numpy(), Xh) and bool(torch.isnan(back[:, P:]).all())
    assert bool(torch.isnan(raw2[:offset]).all()) and bool(torch.isnan(raw2[offset + N * ld:]).all())


ROUND_CASES = [
    # N, P, S, R, Wt
    (4, 65_536, 8, 2, 512), (5, 10_007, 7, 3, 64), (8, 40_001, 3, 4, 128), (32, 9_999, 32, 4, 64),
    (7, 4_096, 1, 2, 256), (6, 130, 130, 1, 64), (12, 20_000, 5, 11, 64), (16, 30_011, 4, 9, 128),
    (9, 5_000, 2, 0, 64), (100, 20_003, 7, 3, 64), (2, 8_193, 2, 1, 1024), (32, 70_000, 32, 4, 128),
    # narrow tiles: many workers on the LDS-slab kernel (more workers than threads in a workgroup,
    # run-time replica counts), and small cases at every narrow width
    (300, 5_003, 5, 3, 16), (600, 3_001, 3, 2, 8), (1000, 2_003, 2, 5, 8), (64, 9_999, 4, 4, 32),
    (12, 1_000, 3, 2, 8), (200, 4_001, 4, 12, 32), (513, 1_500, 3, 1, 16),
]


@pytest.mark.parametrize("N,P,S,R,Wt", ROUND_CASES)
@pytest.mark.parametrize("weighted", [False, True])
def test_tiled_round_matches_oracle(combo, ref, N, P, S, R, Wt, weighted):
    Xh = np.random.default_rng(N * 13 + P).normal(0, 0.05, (N, P)).astype(np.float32)
    src = to_tiled(combo, Xh, Wt)
    dst = torch.full_like(src, float("nan"))
    peers = torch.empty(max(N * S * R, 1), dtype=torch.int32, device="cuda")
    combo.make_peer_table(peers, N, S, R, 4, 5)
    d = combo.workloads.dataset_sizes(N, 2, "cuda") if weighted else None
    combo.segment_gossip_round_tiled(dst, src, Wt, peers if R else None, N, P, S, R, dataset_sizes=d)
    torch.cuda.synchronize()
    ph = ref.make_peer_table(N, S, R, 4, 5)
    want = ref.gossip_round(Xh, ph, P, S, R, d=None if d is None else d.cpu().numpy())
    got_flat = dst.cpu().numpy()
    got = np_unpack(got_flat, N, P, Wt)
    assert np.all(np.abs(got - want) <= 1e-6 * np.maximum(np.abs(want), 1e-30))
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    assert np.array_equal(np.isnan(got_flat), np.isnan(np_pack(Xh, Wt)))   # only padding is NaN
    assert np.array_equal(np_unpack(src.cpu().numpy(), N, P, Wt), Xh)       # source intact


@pytest.mark.parametrize("tau", [0, 1, 3])
@pytest.mark.parametrize("N,P,S,R,Wt", [(6, 10_007, 7, 3, 64), (100, 5_003, 7, 3, 64), (16, 30_000, 4, 4, 128),
                                        (300, 2_003, 3, 3, 16), (9, 3_000, 2, 2, 8)])
def test_tiled_fused_steps_match_oracle(combo, ref, tau, N, P, S, R, Wt):
    rng = np.random.default_rng(tau + N)
    Xh = rng.uniform(-0.1, 0.1, (N, P)).astype(np.float32)
    Gh = rng.normal(0, 1e-2, (tau, N, P)).astype(np.float32)
    src = to_tiled(combo, Xh, Wt)
    n = combo.tiled_elems(N, P, Wt)
    grads = torch.zeros(max(n * tau, 1), dtype=torch.float32, device="cuda")
    for k in range(tau):
        grads[k * n:(k + 1) * n] = to_tiled(combo, Gh[k], Wt).nan_to_num(0.0)
    dst = torch.full_like(src, float("nan"))
    peers = torch.empty(N * S * R, dtype=torch.int32, device="cuda")
    combo.make_peer_table(peers, N, S, R, 1, 1)
    combo.local_sgd_steps_then_gossip_tiled(dst, src, grads, tau, 0.05, Wt, peers, N, P, S, R)
    torch.cuda.synchronize()
    ph = ref.make_peer_table(N, S, R, 1, 1)
    want = ref.local_sgd_steps_then_gossip(Xh.copy(), np.ascontiguousarray(Gh), 0.05, ph, P, S, R)
    got = np_unpack(dst.cpu().numpy(), N, P, Wt)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    assert np.array_equal(np_unpack(src.cpu().numpy(), N, P, Wt), Xh)


@pytest.mark.parametrize("N,P,S,R,Wt", [(12, 30_011, 6, 3, 128), (300, 3_001, 4, 3, 16), (20, 2_000, 3, 4, 8)])
def test_tiled_dynamic_round(combo, ref, N, P, S, R, Wt):
    st = np.ones(N, np.uint8)
    st[[2, 7]] = 0
    st[[4, 11]] = 2
    Xh = np.random.default_rng(0).normal(0, 0.05, (N, P)).astype(np.float32)
    src = to_tiled(combo, Xh, Wt)
    dst = torch.full_like(src, float("nan"))
    std = torch.from_numpy(st).cuda()
    peers = torch.empty(N * S * R, dtype=torch.int32, device="cuda")
    combo.make_peer_table_dynamic(peers, std, N, S, R, 0, 0)
    combo.segment_gossip_round_tiled(dst, src, Wt, peers, N, P, S, R, status=std)
    torch.cuda.synchronize()
    T = ref.make_peer_table_dynamic(st, N, S, R, 0, 0)
    want = ref.gossip_round_dynamic(Xh, T, st, P, S, R)
    got = np_unpack(dst.cpu().numpy(), N, P, Wt)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_tiled_errors(combo):
    a = torch.zeros(combo.tiled_elems(4, 1000, 64), dtype=torch.float32, device="cuda")
    b = torch.zeros_like(a)
    peers = torch.zeros(4 * 2 * 2, dtype=torch.int32, device="cuda")
    with pytest.raises(combo.ComboError):
        combo.tiled_elems(4, 1000, 100)
    with pytest.raises(combo.ComboError) as e:
        combo.segment_gossip_round_tiled(a, a, 64, peers, 4, 1000, 2, 2)
    assert e.value.status == -2
    with pytest.raises(combo.ComboError) as e:
        combo.tiled_cols(3000, 2)
    assert e.value.status == -3
    assert combo.tiled_cols(32, 4) == 64 and combo.tiled_cols(16, 4) == 128
    # more workers: the widest of 64, 32, 16, 8 columns whose tile stays within 32 KiB
    assert combo.tiled_cols(100, 3) == 64 and combo.tiled_cols(200, 3) == 32
    assert combo.tiled_cols(300, 2) == 16 and combo.tiled_cols(1000, 5) == 8
    with pytest.raises(combo.ComboError):
        combo.tiled_cols(1000, 6)                    # the peer list no longer fits beside the slab
    with pytest.raises(combo.ComboError):
        combo.tiled_elems(4, 1000, 4)


@pytest.mark.parametrize("name,weighted", [("c2_resnet18", False), ("c3_resnet50", False),
                                           ("c4_prime_fused", False), ("c5_bertlarge", False),
                                           ("c2_resnet18", True), ("c4_prime_fused", True)])
def test_full_size_workloads_tiled_on_sampled_windows(combo, ref, name, weighted):
    """Full-size tiled arena, all rounds, the layout and launch configuration that the
    benchmark times (and the same with dataset-size weights); compared on column windows
    that the oracle recomputes round by round."""
    wl = combo.workloads.WORKLOADS[name]
    d = combo.workloads.dataset_sizes(wl.N, 1, "cuda") if weighted else None
    dh = None if d is None else d.cpu().numpy()
    Wt = combo.tiled_cols(wl.N, wl.R)
    n = combo.tiled_elems(wl.N, wl.P, Wt)
    T = n // (wl.N * Wt)
    arena = torch.full((2, n), float("nan"), dtype=torch.float32, device="cuda")
    view = arena[0].view(T, wl.N, Wt)
    g = torch.Generator(device="cuda")
    g.manual_seed(wl.data_seed)
    for t0 in range(0, T, 4096):                     # fill tile blocks; padding of the last tile too
        blk = view[t0:t0 + 4096]
        if wl.dist == "normal":
            blk.normal_(0.0, wl.scale, generator=g)
        else:
            blk.uniform_(-wl.scale, wl.scale, generator=g)
    grads = None
    if wl.fused:
        grads = torch.zeros(n, dtype=torch.float32, device="cuda")

    def window(buf, c0, nc):
        """Columns [c0, c0+nc) of all workers from a tiled buffer, as a host (N, nc) array."""
        t_lo, t_hi = c0 // Wt, (c0 + nc - 1) // Wt + 1
        blk = buf.view(T, wl.N, Wt)[t_lo:t_hi].permute(1, 0, 2).reshape(wl.N, -1)
        return blk[:, c0 - t_lo * Wt:c0 - t_lo * Wt + nc].contiguous().cpu().numpy()

    import tests.test_gpu_parity as tp
    wins = tp.sample_windows(wl)
    X0 = {w: window(arena[0], *w) for w in wins}
    G = {w: [] for w in wins}
    peers = torch.empty(wl.N * wl.S * wl.R, dtype=torch.int32, device="cuda")
    cur = 0
    for rnd in range(wl.rounds):
        combo.make_peer_table(peers, wl.N, wl.S, wl.R, wl.hash_seed, rnd)
        if wl.fused:
            gg = torch.Generator(device="cuda")
            gg.manual_seed(1000 + rnd)
            grads.normal_(0.0, wl.grad_std, generator=gg)
            for w in wins:
                G[w].append(window(grads, *w))
            combo.local_sgd_steps_then_gossip_tiled(arena[1 - cur], arena[cur], grads, 1, wl.lr, Wt, peers,
                                                    wl.N, wl.P, wl.S, wl.R, dataset_sizes=d)
        else:
            combo.segment_gossip_round_tiled(arena[1 - cur], arena[cur], Wt, peers, wl.N, wl.P, wl.S, wl.R,
                                             dataset_sizes=d)
        cur = 1 - cur
    torch.cuda.synchronize()
    for w in wins:
        want = tp.oracle_rounds_on_window(ref, wl, X0[w], w[0], wl.rounds, Gwins=G[w] if wl.fused else None,
                                          d=dh)
        got = window(arena[cur], *w)
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), (name, w)
    # nothing unwritten inside the rows; the last tile's padding columns stay NaN
    last = arena[cur].view(T, wl.N, Wt)
    assert not bool(torch.isnan(last[:T - 1]).any())
    tail = wl.P - (T - 1) * Wt
    assert not bool(torch.isnan(last[T - 1, :, :tail]).any())
    if tail < Wt:      # half 1 started as NaN everywhere: its padding was never written
        assert bool(torch.isnan(arena[1].view(T, wl.N, Wt)[T - 1, :, tail:]).all())


@pytest.mark.parametrize("layout", ["rows", "tiled"])
def test_more_than_two_to_the_32_columns(combo, ref, layout):
    """P > 2^32: column indices, segment lookup and offsets need 64 bits (a 17 GB row).
    N=2, S=3, R=1, two rounds, checked on windows at the row start and end, at both
    segment boundaries and across column 2^32."""
    from paper_1908_07782_amd.workloads import Workload
    import tests.test_gpu_parity as tp
    P = 2**32 + 4099
    wl = Workload("wide", N=2, P=P, S=3, R=1, rounds=2, dist="normal", scale=0.05)
    L = P // 3
    wins = [(0, 3000), (P - 3000, 3000), (L - 1500, 3000), (2 * L - 1500, 3000), (2**32 - 1500, 3000),
            (2**31 - 1500, 3000)]
    peers = torch.empty(wl.N * wl.S * wl.R, dtype=torch.int32, device="cuda")
    g = torch.Generator(device="cuda")
    g.manual_seed(5)
    if layout == "rows":
        arena = torch.empty((2, wl.N, wl.ld), dtype=torch.float32, device="cuda")
        arena[1].fill_(float("nan"))
        for w in range(wl.N):
            arena[0, w].normal_(0.0, wl.scale, generator=g)

        def window(buf, c0, nc):
            return buf[:, c0:c0 + nc].contiguous().cpu().numpy()
    else:
        Wt = combo.tiled_cols(wl.N, wl.R)
        n = combo.tiled_elems(wl.N, P, Wt)
        T = n // (wl.N * Wt)
        arena = torch.empty((2, n), dtype=torch.float32, device="cuda")
        arena[1].fill_(float("nan"))
        half = n // 2 // 4 * 4
        arena[0, :half].normal_(0.0, wl.scale, generator=g)
        arena[0, half:].normal_(0.0, wl.scale, generator=g)

        def window(buf, c0, nc):
            t_lo, t_hi = c0 // Wt, (c0 + nc - 1) // Wt + 1
            blk = buf.view(T, wl.N, Wt)[t_lo:t_hi].permute(1, 0, 2).reshape(wl.N, -1)
            return blk[:, c0 - t_lo * Wt:c0 - t_lo * Wt + nc].contiguous().cpu().numpy()
    X0 = {w: window(arena[0], *w) for w in wins}
    cur = 0
    for rnd in range(wl.rounds):
        combo.make_peer_table(peers, wl.N, wl.S, wl.R, wl.hash_seed, rnd)
        if layout == "rows":
            combo.segment_gossip_round(arena[1 - cur], arena[cur], peers, P, wl.S, wl.R)
        else:
            combo.segment_gossip_round_tiled(arena[1 - cur], arena[cur], Wt, peers, wl.N, P, wl.S, wl.R)
        cur = 1 - cur
    torch.cuda.synchronize()
    for w in wins:
        want = tp.oracle_rounds_on_window(ref, wl, X0[w], w[0], wl.rounds)
        got = window(arena[cur], *w)
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), (layout, w)
    # after one round the other half was written everywhere inside the rows
    if layout == "rows":
        assert not bool(torch.isnan(arena[1, :, :P]).any())
        assert bool(torch.isnan(arena[1, :, P:]).all())
