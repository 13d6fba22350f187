"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the
same seeded inputs.  Peer tables must match bit for bit.  Parameters must agree within
max relative error 1e-6 elementwise against the same-order binary32 oracle (the bar of
this build); because the summation order and roundings are part of the ABI, they are
also expected - and asserted - to be bitwise equal.  Against the binary64 oracle the
normwise error max|g - o64| / max|o64| is checked against (R+3) * 2^-24 * max|x| /
max|o64| and is what is reported as accuracy.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

REL_TOL = 1e-6


@pytest.fixture(scope="module")
def combo():
    import paper_1908_07782_amd as c
    assert torch.cuda.is_available(), "these tests need the GPU"
    c.lib()                                  # raises if libcombo.so is missing: no fallback
    return c


def set_variant(combo, variant):
    """variant: ("slab", strip columns or 0 for automatic) or ("tile", tile columns)."""
    kind, cols = variant
    if kind == "slab":
        combo.tune(combo.TUNE_KERNEL, 0)
        combo.tune(combo.TUNE_SLAB_COLS, cols)
    else:
        combo.tune(combo.TUNE_KERNEL, 1)
        combo.tune(combo.TUNE_TILE_COLS, cols)


VARIANTS = [("slab", 0), ("slab", 64), ("slab", 256), ("slab", 1024),
            ("slab", 128), ("slab", 512),
            ("tile", 1024), ("tile", 2048), ("tile", 4096)]


@pytest.fixture(autouse=True)
def _default_tuning(combo):
    yield
    combo.tune(combo.TUNE_KERNEL, 0)
    combo.tune(combo.TUNE_SLAB_COLS, 0)
    combo.tune(combo.TUNE_FUSED_MODE, 0)
    combo.tune(combo.TUNE_TILE_COLS, 0)
    combo.tune(combo.TUNE_XCD_SWIZZLE, 1)


def assert_params_match(got, want, what=""):
    """got, want: float32 numpy arrays.  1e-6 relative (the stated bar), then bitwise."""
    got = np.asarray(got)
    want = np.asarray(want)
    assert got.shape == want.shape
    err = np.abs(got.astype(np.float64) - want.astype(np.float64))
    bound = REL_TOL * np.maximum(np.abs(want.astype(np.float64)), 1e-30)
    bad = err > bound
    assert not bad.any(), f"{what}: {int(bad.sum())} elements beyond 1e-6 relative, max err {err.max()}"
    same = got.view(np.uint32) == want.view(np.uint32)
    assert same.all(), f"{what}: within 1e-6 but {int((~same).sum())} elements differ in the last bits"


def device_table(combo, N, S, R, seed, rnd):
    t = torch.full((max(N * S * R, 1),), -7, dtype=torch.int32, device="cuda")
    combo.make_peer_table(t, N, S, R, seed, rnd)
    torch.cuda.synchronize()
    return t


def make_arena(wl, ld=None, fill=float("nan")):
    ld = wl.ld if ld is None else ld
    return torch.full((2, wl.N, ld), fill, dtype=torch.float32, device="cuda")


# ------------------------------------------------------------------------ peer tables
@pytest.mark.parametrize("name", ["c1_tiny", "c2_resnet18", "c3_resnet50", "c4_prime_fused",
                                  "c5_bertlarge"])
def test_peer_tables_bit_exact_all_rounds(combo, ref, name):
    wl = combo.workloads.WORKLOADS[name]
    for rnd in range(wl.rounds):
        t = device_table(combo, wl.N, wl.S, wl.R, wl.hash_seed, rnd)
        want = ref.make_peer_table(wl.N, wl.S, wl.R, wl.hash_seed, rnd)
        assert np.array_equal(t.cpu().numpy().reshape(want.shape), want), (name, rnd)


@pytest.mark.parametrize("N,S,R,seed,rnd", [(2, 5, 1, 3, 0), (5, 3, 4, 11, 2), (100, 7, 99, 1, 1),
                                            (16, 16, 15, 0, 4), (1000, 3, 17, 2**63 + 5, 2**40 + 1),
                                            (16384, 1, 3, 9, 9), (3, 1000, 2, 4, 4)])
def test_peer_tables_edge_cases(combo, ref, N, S, R, seed, rnd):
    t = device_table(combo, N, S, R, seed, rnd)
    want = ref.make_peer_table(N, S, R, seed, rnd)
    assert np.array_equal(t.cpu().numpy().reshape(want.shape), want)


def test_peer_table_R0_writes_nothing(combo):
    t = torch.full((8,), -7, dtype=torch.int32, device="cuda")
    combo.make_peer_table(t, 4, 2, 0, 0, 0)
    combo.make_peer_table(None, 4, 2, 0, 0, 0)
    torch.cuda.synchronize()
    assert bool((t == -7).all())


# ----------------------------------------------------------------- one round, small
def run_small(combo, ref, N, P, S, R, *, ld=None, weighted=False, seed=0, rnd=0, offset=0,
              scale=0.05):
    """One round on the GPU and in the oracle; returns (gpu Y, oracle Y, X, peers).
    `offset` shifts the base pointers by that many floats (alignment cases)."""
    ld = combo.workloads.row_pitch(P) if ld is None else ld
    rng = np.random.default_rng(seed * 7919 + N * 31 + P)
    Xh = rng.normal(0, scale, (N, P)).astype(np.float32)
    raw = torch.full((2, N * ld + offset + 8), float("nan"), dtype=torch.float32, device="cuda")
    src = raw[0, offset:offset + N * ld].view(N, ld)
    dst = raw[1, offset:offset + N * ld].view(N, ld)
    src[:, :P] = torch.from_numpy(Xh).cuda()
    peers = device_table(combo, N, S, R, seed, rnd)
    d = combo.workloads.dataset_sizes(N, seed, "cuda") if weighted else None
    combo.segment_gossip_round(dst, src, peers if R > 0 else None, P, S, R, dataset_sizes=d)
    torch.cuda.synchronize()
    ph = ref.make_peer_table(N, S, R, seed, rnd)
    assert np.array_equal(peers.cpu().numpy()[:N * S * R].reshape(ph.shape), ph)
    want = ref.gossip_round(Xh, ph, P, S, R, d=None if d is None else d.cpu().numpy())
    got = dst[:, :P].cpu().numpy()
    # padding and guard words untouched, source intact
    assert bool(torch.isnan(dst[:, P:]).all())
    assert bool(torch.isnan(raw[1, :offset]).all()) and bool(torch.isnan(raw[1, offset + N * ld:]).all())
    assert np.array_equal(src[:, :P].cpu().numpy().view(np.uint32), Xh.view(np.uint32))
    return got, want, Xh, ph


SMALL_SHAPES = [
    # N, P, S, R : several tiles, ragged tails, segment boundaries inside tiles
    (4, 65_536, 8, 2),          # the tiny workload: 8192-column segments
    (5, 10_007, 7, 3),          # prime P, P % 4 == 3
    (8, 40_001, 3, 4),          # P % 4 == 1, long segments
    (32, 9_999, 32, 4),         # segments shorter than a tile: boundary path everywhere
    (7, 4_096, 1, 2),           # S = 1 (whole-model gossip)
    (3, 6, 2, 2),               # the hand-sized case
    (6, 130, 130, 1),           # S = P: one column per segment
    (12, 20_000, 5, 11),        # R = N-1 (FedAvg limit), run-time-R kernel
    (16, 30_011, 4, 9),         # R > 8: run-time-R kernel
    (9, 5_000, 2, 0),           # R = 0: copy
    (1, 3_000, 3, 0),           # single worker
    (2, 8_193, 2, 1),           # two workers
]


@pytest.mark.parametrize("N,P,S,R", SMALL_SHAPES + [(100, 20_003, 7, 3), (250, 3_001, 3, 5),
                                                    (300, 2_000, 2, 2)])
@pytest.mark.parametrize("variant", VARIANTS, ids=lambda v: f"{v[0]}{v[1]}")
def test_round_matches_oracle_small(combo, ref, N, P, S, R, variant):
    set_variant(combo, variant)
    got, want, _, _ = run_small(combo, ref, N, P, S, R)
    assert_params_match(got, want, f"N{N} P{P} S{S} R{R} {variant}")


@pytest.mark.parametrize("N,P,S,R", [(5, 10_007, 7, 3), (32, 40_000, 32, 4), (12, 20_000, 5, 11)])
def test_round_plain_workgroup_order(combo, ref, N, P, S, R):
    combo.tune(combo.TUNE_KERNEL, 1)
    combo.tune(combo.TUNE_XCD_SWIZZLE, 0)
    got, want, _, _ = run_small(combo, ref, N, P, S, R)
    assert_params_match(got, want)


@pytest.mark.parametrize("N,P,S,R", [(5, 10_007, 7, 3), (8, 40_001, 3, 4), (6, 130, 130, 1),
                                     (16, 30_011, 4, 9), (9, 5_000, 2, 0), (32, 70_000, 32, 4)])
@pytest.mark.parametrize("variant", [("slab", 0), ("slab", 64), ("slab", 512), ("tile", 2048)],
                         ids=lambda v: f"{v[0]}{v[1]}")
def test_round_dataset_size_weights(combo, ref, N, P, S, R, variant):
    set_variant(combo, variant)
    got, want, _, _ = run_small(combo, ref, N, P, S, R, weighted=True, seed=3)
    assert_params_match(got, want)


@pytest.mark.parametrize("ld,offset", [(10_007, 0), (10_009, 0), (10_048, 1), (10_048, 3), (10_010, 2)])
def test_round_unaligned_pitch_or_base(combo, ref, ld, offset):
    """ld % 4 != 0 or a base pointer off the 16-byte grid: the scalar kernel runs."""
    got, want, _, _ = run_small(combo, ref, 5, 10_007, 7, 3, ld=ld, offset=offset)
    assert_params_match(got, want)
    got, want, _, _ = run_small(combo, ref, 5, 10_007, 7, 3, ld=ld, offset=offset, weighted=True)
    assert_params_match(got, want)


def test_round_against_float64_oracle(combo, ref):
    N, P, S, R = 32, 200_003, 32, 4
    got, _, Xh, ph = run_small(combo, ref, N, P, S, R, scale=0.02)
    y64 = ref.gossip_round_f64(Xh, ph, P, S, R)
    normwise = np.max(np.abs(got - y64)) / np.max(np.abs(y64))
    assert normwise <= (R + 3) * 2.0 ** -24 * np.abs(Xh).max() / np.max(np.abs(y64))
    assert normwise < REL_TOL


def test_round_paper_invariants_on_gpu(combo, ref):
    # identical workers stay identical (Sec. 4.1: common initialisation)
    N, P, S, R = 8, 50_000, 10, 2
    row = torch.randn(P, device="cuda") * 0.05
    src = row.repeat(N, 1).contiguous()
    dst = torch.empty_like(src)
    peers = device_table(combo, N, S, R, 0, 0)
    combo.segment_gossip_round(dst, src, peers, P, S, R)
    torch.cuda.synchronize()
    assert bool((dst.view(torch.int32) == dst[:1].view(torch.int32)).all())
    assert float((dst - src).abs().max()) <= 2 * 2.0 ** -24 * float(row.abs().max()) * 1.01
    # R = N-1: every worker reaches the FedAvg mean (Sec. 4.3)
    N, P, S = 10, 30_000, 4
    src = torch.randn(N, P, device="cuda") * 0.02
    dst = torch.empty_like(src)
    peers = device_table(combo, N, S, N - 1, 0, 0)
    combo.segment_gossip_round(dst, src, peers, P, S, N - 1)
    torch.cuda.synchronize()
    mean = src.double().mean(dim=0)
    assert float((dst.double() - mean[None]).abs().max()) <= (N + 1) * 2.0 ** -24 * float(src.abs().max())


# ----------------------------------------------------- multi-round, with buffer swap
def run_rounds_gpu(combo, wl, arena, rounds, grads=None, dsz=None, tables_out=None):
    """T rounds through the C ABI, ping-ponging the two halves of the arena.  Returns
    the index of the half that holds the final parameters."""
    peers = torch.empty(max(wl.N * wl.S * wl.R, 1), dtype=torch.int32, device="cuda")
    cur = 0
    for rnd in range(rounds):
        combo.make_peer_table(peers, wl.N, wl.S, wl.R, wl.hash_seed, rnd)
        if tables_out is not None:
            tables_out.append(peers.clone())
        if grads is not None:
            combo.workloads.fill_grads(grads, wl, rnd)
            combo.local_sgd_then_gossip(arena[1 - cur], arena[cur], grads, wl.lr, peers,
                                        wl.P, wl.S, wl.R, dataset_sizes=dsz)
        else:
            combo.segment_gossip_round(arena[1 - cur], arena[cur], peers, wl.P, wl.S, wl.R,
                                       dataset_sizes=dsz)
        cur = 1 - cur
    torch.cuda.synchronize()
    return cur


def oracle_rounds_on_window(ref, wl, Xwin, c0, rounds, Gwins=None, d=None):
    """The same T rounds in the oracle on the column window [c0, c0 + ncols)."""
    X = np.ascontiguousarray(Xwin)
    for rnd in range(rounds):
        ph = ref.make_peer_table(wl.N, wl.S, wl.R, wl.hash_seed, rnd)
        if Gwins is not None:
            X = ref.local_sgd_then_gossip(X, np.ascontiguousarray(Gwins[rnd]), wl.lr, ph, wl.P, wl.S,
                                          wl.R, d=d, col0=c0)
        else:
            X = ref.gossip_round(X, ph, wl.P, wl.S, wl.R, d=d, col0=c0)
    return X


def sample_windows(wl, width=3000, tile=2048):
    """Column windows the oracle can afford: row start, row end (ragged tail), every
    kind of segment boundary (first, middle, last), and a few tile-interior spots."""
    L = wl.P // wl.S
    starts = {0, max(wl.P - width, 0)}
    for s in sorted({1, wl.S // 2, wl.S - 1}):
        if 0 < s < wl.S:
            starts.add(max(s * L - width // 2, 0))
    rng = np.random.default_rng(wl.P)
    for c in rng.integers(0, max(wl.P - width, 1), 3):
        starts.add(int(c))
    return [(c0, min(width, wl.P - c0)) for c0 in sorted(starts)]


def test_c1_tiny_full(combo, ref):
    wl = combo.workloads.WORKLOADS["c1_tiny"]
    arena = make_arena(wl)
    combo.workloads.fill_params(arena[0], wl)
    X0 = arena[0, :, :wl.P].cpu().numpy()
    cur = run_rounds_gpu(combo, wl, arena, wl.rounds)
    want = oracle_rounds_on_window(ref, wl, X0, 0, wl.rounds)
    assert_params_match(arena[cur, :, :wl.P].cpu().numpy(), want, "c1")
    assert bool(torch.isnan(arena[cur, :, wl.P:]).all()) if wl.ld > wl.P else True


@pytest.mark.parametrize("mode", ["fused_slab", "two_pass_slab", "two_pass_tile"])
def test_c4_prime_fused_full_three_rounds(combo, ref, mode):
    """N=100, P=1,000,003 (prime), S=7, R=3, x -= 0.01*g then gossip; full-size
    elementwise comparison over 3 of the 20 rounds (all 20 are covered on windows)."""
    wl = combo.workloads.WORKLOADS["c4_prime_fused"]
    combo.tune(combo.TUNE_FUSED_MODE, 0 if mode.startswith("fused") else 1)
    combo.tune(combo.TUNE_KERNEL, 1 if mode == "two_pass_tile" else 0)
    arena = make_arena(wl)
    combo.workloads.fill_params(arena[0], wl)
    grads = torch.zeros((wl.N, wl.ld), dtype=torch.float32, device="cuda")
    X = arena[0, :, :wl.P].cpu().numpy()
    rounds = 3
    Gs = []
    for rnd in range(rounds):
        combo.workloads.fill_grads(grads, wl, rnd)
        Gs.append(grads[:, :wl.P].cpu().numpy())
    cur = run_rounds_gpu(combo, wl, arena, rounds, grads=grads)
    want = oracle_rounds_on_window(ref, wl, X, 0, rounds, Gwins=Gs)
    assert_params_match(arena[cur, :, :wl.P].cpu().numpy(), want, "c4 full")
    assert bool(torch.isnan(arena[cur, :, wl.P:]).all())


def test_c4_prime_fused_all_rounds_on_windows(combo, ref):
    wl = combo.workloads.WORKLOADS["c4_prime_fused"]
    arena = make_arena(wl)
    combo.workloads.fill_params(arena[0], wl)
    grads = torch.zeros((wl.N, wl.ld), dtype=torch.float32, device="cuda")
    wins = sample_windows(wl)
    X0 = {w: arena[0, :, w[0]:w[0] + w[1]].cpu().numpy() for w in wins}
    G = {w: [] for w in wins}
    for rnd in range(wl.rounds):
        combo.workloads.fill_grads(grads, wl, rnd)
        for w in wins:
            G[w].append(grads[:, w[0]:w[0] + w[1]].cpu().numpy())
    cur = run_rounds_gpu(combo, wl, arena, wl.rounds, grads=grads)
    for w in wins:
        want = oracle_rounds_on_window(ref, wl, X0[w], w[0], wl.rounds, Gwins=G[w])
        assert_params_match(arena[cur, :, w[0]:w[0] + w[1]].cpu().numpy(), want, f"c4 window {w}")


@pytest.mark.parametrize("name", ["c2_resnet18", "c3_resnet50", "c5_bertlarge"])
@pytest.mark.parametrize("variant", [("slab", 0), ("tile", 2048)], ids=lambda v: f"{v[0]}{v[1]}")
def test_full_size_workloads_on_sampled_windows(combo, ref, name, variant):
    """Full-size arena, all rounds, in the launch configuration the benchmark times;
    compared on column windows that the oracle recomputes round by round (an output
    column depends only on the same input column, so a window of the full run equals the
    run on the window)."""
    wl = combo.workloads.WORKLOADS[name]
    set_variant(combo, variant)
    arena = make_arena(wl)
    combo.workloads.fill_params(arena[0], wl)
    wins = sample_windows(wl)
    X0 = {w: arena[0, :, w[0]:w[0] + w[1]].cpu().numpy() for w in wins}
    tables = []
    cur = run_rounds_gpu(combo, wl, arena, wl.rounds, tables_out=tables)
    for rnd, t in enumerate(tables):
        want = ref.make_peer_table(wl.N, wl.S, wl.R, wl.hash_seed, rnd)
        assert np.array_equal(t.cpu().numpy().reshape(want.shape), want)
    for w in wins:
        want = oracle_rounds_on_window(ref, wl, X0[w], w[0], wl.rounds)
        assert_params_match(arena[cur, :, w[0]:w[0] + w[1]].cpu().numpy(), want, f"{name} window {w}")
    # properties that hold at any size: nothing unwritten, padding untouched, and the
    # per-column range never grows (convex combinations)
    assert not bool(torch.isnan(arena[cur, :, :wl.P]).any())
    if wl.ld > wl.P:
        assert bool(torch.isnan(arena[cur, :, wl.P:]).all())


def test_c2_resnet18_full_one_round_elementwise(combo, ref):
    """One full-size round of the benchmark workload compared element by element."""
    wl = combo.workloads.WORKLOADS["c2_resnet18"]
    arena = make_arena(wl)
    combo.workloads.fill_params(arena[0], wl)
    X0 = arena[0, :, :wl.P].cpu().numpy()
    cur = run_rounds_gpu(combo, wl, arena, 1)
    want = oracle_rounds_on_window(ref, wl, X0, 0, 1)
    assert_params_match(arena[cur, :, :wl.P].cpu().numpy(), want, "c2 full round")


@pytest.mark.parametrize("mode,weighted", [("fused_slab", False), ("fused_slab", True),
                                           ("two_pass_slab", False), ("two_pass_tile", True)])
def test_fused_small_and_aliasing_contract(combo, ref, mode, weighted):
    combo.tune(combo.TUNE_FUSED_MODE, 0 if mode.startswith("fused") else 1)
    combo.tune(combo.TUNE_KERNEL, 1 if mode == "two_pass_tile" else 0)
    N, P, S, R, lr = 6, 10_007, 7, 3, 0.01
    rng = np.random.default_rng(5)
    Xh = rng.uniform(-0.1, 0.1, (N, P)).astype(np.float32)
    Gh = rng.normal(0, 1e-3, (N, P)).astype(np.float32)
    ld = combo.workloads.row_pitch(P)
    buf = torch.full((3, N, ld), float("nan"), dtype=torch.float32, device="cuda")
    buf[0, :, :P] = torch.from_numpy(Xh).cuda()
    buf[2, :, :P] = torch.from_numpy(Gh).cuda()
    peers = device_table(combo, N, S, R, 0, 0)
    d = combo.workloads.dataset_sizes(N, 1, "cuda") if weighted else None
    combo.local_sgd_then_gossip(buf[1], buf[0], buf[2], lr, peers, P, S, R, dataset_sizes=d)
    torch.cuda.synchronize()
    ph = ref.make_peer_table(N, S, R, 0, 0)
    Xs = Xh.copy()
    want = ref.local_sgd_then_gossip(Xs, Gh, lr, ph, P, S, R, d=None if d is None else d.cpu().numpy())
    assert_params_match(buf[1, :, :P].cpu().numpy(), want, "fused")
    # the old front buffer holds x (fused kernel) or the stepped x' (two passes)
    assert_params_match(buf[0, :, :P].cpu().numpy(), Xh if mode.startswith("fused") else Xs, "front buffer")
    assert_params_match(buf[2, :, :P].cpu().numpy(), Gh, "gradients untouched")
    assert bool(torch.isnan(buf[:, :, P:]).all())
    # overlapping buffers are refused and nothing is enqueued
    before = buf.clone()
    with pytest.raises(combo.ComboError) as e:
        combo.segment_gossip_round(buf[0], buf[0], peers, P, S, R)
    assert e.value.status == -2
    with pytest.raises(combo.ComboError):
        combo.local_sgd_then_gossip(buf[1], buf[0], buf[0], lr, peers, P, S, R)
    torch.cuda.synchronize()
    assert torch.equal(before.view(torch.int32), buf.view(torch.int32))


def test_runs_on_a_side_stream(combo, ref):
    N, P, S, R = 8, 100_003, 5, 3
    st = torch.cuda.Stream()
    Xh = np.random.default_rng(1).normal(0, 0.05, (N, P)).astype(np.float32)
    ld = combo.workloads.row_pitch(P)
    src = torch.zeros((N, ld), dtype=torch.float32, device="cuda")
    src[:, :P] = torch.from_numpy(Xh).cuda()
    dst = torch.zeros_like(src)
    peers = torch.empty(N * S * R, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    with torch.cuda.stream(st):
        combo.make_peer_table(peers, N, S, R, 5, 6, stream=st)
        combo.segment_gossip_round(dst, src, peers, P, S, R, stream=st)
    st.synchronize()
    ph = ref.make_peer_table(N, S, R, 5, 6)
    assert_params_match(dst[:, :P].cpu().numpy(), ref.gossip_round(Xh, ph, P, S, R))


# ------------------------------------------ several local steps (interval tau), then the round
@pytest.mark.parametrize("tau", [0, 1, 3])
@pytest.mark.parametrize("mode", ["fused_slab", "two_pass_slab", "two_pass_tile"])
@pytest.mark.parametrize("N,P,S,R,weighted", [(6, 10_007, 7, 3, False), (32, 40_000, 32, 4, True),
                                              (100, 5_003, 7, 3, False)])
def test_multi_step_local_update(combo, ref, tau, mode, N, P, S, R, weighted):
    combo.tune(combo.TUNE_FUSED_MODE, 0 if mode.startswith("fused") else 1)
    combo.tune(combo.TUNE_KERNEL, 1 if mode == "two_pass_tile" else 0)
    lr = 0.05
    rng = np.random.default_rng(tau * 100 + N)
    ld = combo.workloads.row_pitch(P)
    Xh = rng.uniform(-0.1, 0.1, (N, P)).astype(np.float32)
    Gh = np.zeros((tau, N, ld), np.float32)
    Gh[:, :, :P] = rng.normal(0, 1e-2, (tau, N, P)).astype(np.float32)
    buf = torch.full((2, N, ld), float("nan"), dtype=torch.float32, device="cuda")
    buf[0, :, :P] = torch.from_numpy(Xh).cuda()
    grads = torch.from_numpy(Gh).cuda()
    peers = device_table(combo, N, S, R, 2, 3)
    d = combo.workloads.dataset_sizes(N, 1, "cuda") if weighted else None
    combo.local_sgd_steps_then_gossip(buf[1], buf[0], grads, lr, peers, P, S, R, dataset_sizes=d)
    torch.cuda.synchronize()
    ph = ref.make_peer_table(N, S, R, 2, 3)
    Xs = np.zeros((N, ld), np.float32)
    Xs[:, :P] = Xh
    want = ref.local_sgd_steps_then_gossip(Xs[:, :P], Gh[:, :, :P], lr, ph, P, S, R,
                                           d=None if d is None else d.cpu().numpy())
    assert_params_match(buf[1, :, :P].cpu().numpy(), want, f"tau={tau} {mode}")
    front = buf[0, :, :P].cpu().numpy()
    assert_params_match(front, Xh if (mode.startswith("fused") or tau == 0) else Xs[:, :P], "front buffer")
    assert bool(torch.isnan(buf[:, :, P:]).all())


def test_rounds_can_be_captured_in_a_hip_graph(combo, ref):
    """The library neither allocates nor synchronises nor memsets, so a caller may capture
    peer-table + round launches in a HIP graph.  The graph (two rounds, A -> B -> A) is
    replayed several times with eager work and synchronisations in between; every replay
    must equal the same calls made eagerly."""
    N, P, S, R = 8, 50_003, 5, 3
    ld = combo.workloads.row_pitch(P)
    Xh = np.random.default_rng(7).normal(0, 0.05, (N, P)).astype(np.float32)
    A = torch.zeros((N, ld), dtype=torch.float32, device="cuda")
    A[:, :P] = torch.from_numpy(Xh).cuda()
    B = torch.zeros_like(A)
    peers = torch.empty(N * S * R, dtype=torch.int32, device="cuda")
    eA, eB, ep = A.clone(), B.clone(), peers.clone()

    def two_rounds(a, b, p, stream):
        combo.make_peer_table(p, N, S, R, 3, 0, stream=stream)
        combo.segment_gossip_round(b, a, p, P, S, R, stream=stream)
        combo.make_peer_table(p, N, S, R, 3, 1, stream=stream)
        combo.segment_gossip_round(a, b, p, P, S, R, stream=stream)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        two_rounds(A, B, peers, side)                 # warm-up on the capture stream
    side.synchronize()
    A.copy_(eA)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        two_rounds(A, B, peers, torch.cuda.current_stream())
    torch.cuda.synchronize()
    A.copy_(eA)                                       # capture does not execute; start clean
    for replay in range(4):
        graph.replay()
        two_rounds(eA, eB, ep, torch.cuda.current_stream())
        junk = torch.randn(1000, device="cuda").sum()   # unrelated eager work in between
        torch.cuda.synchronize()
        assert torch.equal(A.view(torch.int32), eA.view(torch.int32)), replay
        assert torch.equal(B.view(torch.int32), eB.view(torch.int32)), replay
        assert float(junk) == float(junk)
    # and the eager chain is the oracle's: 8 rounds alternating tables of round 0 and 1
    X = Xh
    for k in range(8):
        X = ref.gossip_round(X, ref.make_peer_table(N, S, R, 3, k % 2), P, S, R)
    assert_params_match(eA[:, :P].cpu().numpy(), X, "graph chain")


# ------------------------------------------------------- special values, bit for bit
def _special_matrix(N, P, seed):
    """Ordinary parameters with a third of the entries replaced by signed zeros, subnormal,
    tiny, huge, infinite and NaN values: every branch of the weighted quotient."""
    rng = np.random.default_rng(seed)
    X = rng.normal(0, 0.05, (N, P)).astype(np.float32)
    specials = np.array([0.0, -0.0, 1e-45, -1e-45, 1e-40, -3e-39, 1.2e-38, -1.2e-38, 1e-30, -1e-25,
                         2.0 ** -61, 2.0 ** -60, -2.0 ** -59, 1e-19, 2.0 ** 59, -2.0 ** 60, 2.0 ** 61,
                         1e19, -1e25, 1e30, -3e38, 3.4e38, np.inf, -np.inf, np.nan], dtype=np.float32)
    mask = rng.random((N, P)) < 0.33
    X[mask] = rng.choice(specials, size=int(mask.sum()))
    # whole columns of one special value, so that sums of only zeros (of either sign), only
    # subnormals, only huge values occur too
    cols = np.flatnonzero(rng.random(P) < 0.1)
    X[:, cols] = rng.choice(specials, size=cols.size)[None, :]
    return X


def _assert_same_bits_or_both_nan(got, want, what):
    nan_g, nan_w = np.isnan(got), np.isnan(want)
    assert np.array_equal(nan_g, nan_w), f"{what}: NaN positions differ"
    same = (got.view(np.uint32) == want.view(np.uint32)) | nan_w
    assert same.all(), f"{what}: {int((~same).sum())} elements differ, first at {np.argwhere(~same)[0]}"


@pytest.mark.parametrize("layout", ["rows", "tiled"])
@pytest.mark.parametrize("mode", ["plain", "weighted", "weighted_tiny_sizes", "weighted_huge_sizes",
                                  "dynamic", "dynamic_weighted"])
def test_special_values_bit_exact(combo, ref, layout, mode):
    N, P, S, R = 12, 40_003, 5, 3
    Xh = _special_matrix(N, P, 5)
    ld = combo.workloads.row_pitch(P)
    rows = torch.zeros((2, N, ld), dtype=torch.float32, device="cuda")
    rows[0, :, :P] = torch.from_numpy(Xh).cuda()
    d = None
    if "weighted" in mode:
        d = combo.workloads.dataset_sizes(N, 3, "cuda")
        if mode == "weighted_tiny_sizes":
            d = d * 1e-24            # denominators below 2^-60
        if mode == "weighted_huge_sizes":
            d = d * 1e17             # denominators above 2^60 for the larger sums
    status = None
    if mode.startswith("dynamic"):
        sh = np.ones(N, dtype=np.uint8)
        sh[3] = 0
        sh[7] = 2
        status = torch.from_numpy(sh).cuda()
        peers = torch.empty(N * S * R, dtype=torch.int32, device="cuda")
        combo.make_peer_table_dynamic(peers, status, N, S, R, 9, 2)
        ph = ref.make_peer_table_dynamic(sh, N, S, R, 9, 2)
    else:
        peers = device_table(combo, N, S, R, 9, 2)
        ph = ref.make_peer_table(N, S, R, 9, 2)
    dh = None if d is None else d.cpu().numpy()
    with np.errstate(all="ignore"):
        if status is None:
            want = ref.gossip_round(Xh, ph, P, S, R, d=dh)
        else:
            want = ref.gossip_round_dynamic(Xh, ph, sh, P, S, R, d=dh)
    if layout == "rows":
        if status is None:
            combo.segment_gossip_round(rows[1], rows[0], peers, P, S, R, dataset_sizes=d)
        else:
            combo.segment_gossip_round_dynamic(rows[1], rows[0], peers, status, P, S, R, dataset_sizes=d)
    else:
        Wt = combo.tiled_cols(N, R)
        t = torch.zeros((2, combo.tiled_elems(N, P, Wt)), dtype=torch.float32, device="cuda")
        combo.pack_tiled(t[0], rows[0], N, P, Wt)
        combo.segment_gossip_round_tiled(t[1], t[0], Wt, peers, N, P, S, R, dataset_sizes=d, status=status)
        combo.unpack_tiled(rows[1], t[1], N, P, Wt)
    torch.cuda.synchronize()
    _assert_same_bits_or_both_nan(rows[1, :, :P].cpu().numpy(), want, f"{layout} {mode}")


@pytest.mark.parametrize("layout", ["rows", "tiled"])
@pytest.mark.parametrize("sizes", [(1.0, 1.0), (3.0, 5.0), (1e3, 7e3), (0.1, 0.2), (2.0 ** -31, 2.0 ** -31),
                                   (2.0 ** 58, 2.0 ** 58), (2.0 ** 59, 2.0 ** 59), (2.0 ** -61, 2.0 ** -62),
                                   (float(np.float32(1.9999999)), 0.0), (float(np.float32(1.0000001)), 0.0),
                                   (1e-30, 3e-30), (12345.0, 0.0)])
def test_weighted_quotient_on_random_bit_patterns(combo, ref, layout, sizes):
    """Two workers that average each other with dataset sizes (d0, d1): every output is
    fl(fl(d0*x0 + d1*x1) / fl(d0 + d1)).  Numerators are arbitrary finite bit patterns, the
    denominators cover both sides of the range in which the kernel replaces the division by
    a multiplication with the shared reciprocal plus a residual correction."""
    N, P, S, R = 2, 300_001, 1, 1
    rng = np.random.default_rng(int(abs(hash(sizes)) % 2**31))
    bits = rng.integers(0, 2**32, size=(N, P), dtype=np.uint64).astype(np.uint32)
    Xh = bits.view(np.float32).copy()
    Xh[~np.isfinite(Xh)] = 0.0
    Xh[1, ::3] = 0.0                          # a third of the outputs are d0*x0 / (d0+d1) exactly
    dh = np.array(sizes, dtype=np.float32)
    ph = ref.make_peer_table(N, S, R, 0, 0)   # with two workers each one's only peer is the other
    with np.errstate(all="ignore"):
        want = ref.gossip_round(Xh, ph, P, S, R, d=dh)
    ld = combo.workloads.row_pitch(P)
    rows = torch.zeros((2, N, ld), dtype=torch.float32, device="cuda")
    rows[0, :, :P] = torch.from_numpy(Xh).cuda()
    peers = torch.from_numpy(ph.reshape(-1).astype(np.int32)).cuda()
    d = torch.from_numpy(dh).cuda()
    if layout == "rows":
        combo.segment_gossip_round(rows[1], rows[0], peers, P, S, R, dataset_sizes=d)
    else:
        Wt = combo.tiled_cols(N, R)
        t = torch.zeros((2, combo.tiled_elems(N, P, Wt)), dtype=torch.float32, device="cuda")
        combo.pack_tiled(t[0], rows[0], N, P, Wt)
        combo.segment_gossip_round_tiled(t[1], t[0], Wt, peers, N, P, S, R, dataset_sizes=d)
        combo.unpack_tiled(rows[1], t[1], N, P, Wt)
    torch.cuda.synchronize()
    _assert_same_bits_or_both_nan(rows[1, :, :P].cpu().numpy(), want, f"{layout} sizes {sizes}")
