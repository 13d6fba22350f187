"""GPU parity for rounds that read one arena layout and write another
(combo_round_relayout: Eq. 4's reassembly lands in the layout the caller wants next), for
strips that hold several segments (short segments, L < strip width: the slab is staged in
LDS all the same and the peer lists are looked up per word), and for the strip order knob.
Everything is compared with the CPU oracle bit for bit."""
import numpy as np
import pytest
import torch

from tests.test_gpu_tiled import np_pack, np_unpack

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def combo():
    import paper_1908_07782_amd as c
    assert torch.cuda.is_available()
    c.lib()
    return c


@pytest.fixture(autouse=True)
def default_knobs(combo):
    yield
    combo.tune(combo.TUNE_KERNEL, 0)
    combo.tune(combo.TUNE_SLAB_COLS, 0)
    combo.tune(combo.TUNE_SLAB_ORDER, 0)


def bits(a):
    return np.ascontiguousarray(a).view(np.uint32)


class Side:
    """One parameter matrix on the GPU in either layout, NaN wherever no parameter lives."""

    def __init__(self, combo, N, P, tile, Xh=None, extra_pitch=0):
        self.combo, self.N, self.P, self.tile = combo, N, P, tile
        if tile:
            flat = np_pack(Xh, tile) if Xh is not None else np.full(combo.tiled_elems(N, P, tile), np.nan, np.float32)
            self.t = torch.from_numpy(flat).cuda()
        else:
            ld = combo.workloads.row_pitch(P) + extra_pitch
            self.t = torch.full((N, ld), float("nan"), dtype=torch.float32, device="cuda")
            if Xh is not None:
                self.t[:, :P] = torch.from_numpy(Xh).cuda()

    def values(self):
        """(parameters as (N, P), True if nothing but the parameters was written)"""
        h = self.t.cpu().numpy()
        if self.tile:
            pad_ok = np.array_equal(np.isnan(h), np.isnan(np_pack(np.zeros((self.N, self.P), np.float32), self.tile)))
            return np_unpack(h, self.N, self.P, self.tile), pad_ok
        return h[:, :self.P].copy(), bool(np.isnan(h[:, self.P:]).all())


LAYOUTS = [("rows", "tiled"), ("tiled", "rows"), ("rows", "rows"), ("tiled", "tiled")]
SHAPES = [
    # N, P, S, R, Wt
    (4, 65_536, 8, 2, 512), (5, 10_007, 7, 3, 64), (32, 40_001, 32, 4, 64), (16, 30_011, 4, 9, 128),
    (100, 20_003, 7, 3, 64), (6, 130, 130, 1, 64), (12, 20_000, 5, 11, 64), (9, 5_000, 2, 0, 64),
    (300, 5_003, 5, 3, 16), (3, 63, 3, 2, 64),
]


@pytest.mark.parametrize("src_l,dst_l", LAYOUTS)
@pytest.mark.parametrize("N,P,S,R,Wt", SHAPES)
@pytest.mark.parametrize("weighted", [False, True])
def test_relayout_round_matches_oracle(combo, ref, src_l, dst_l, N, P, S, R, Wt, weighted):
    if N > 250 and "rows" in (src_l, dst_l) and Wt < 64 and src_l == dst_l == "rows":
        pytest.skip("row-major on both sides needs a 64-column slab, which 300 rows do not fit")
    Xh = np.random.default_rng(N * 13 + P).normal(0, 0.05, (N, P)).astype(np.float32)
    src = Side(combo, N, P, Wt if src_l == "tiled" else 0, Xh)
    dst = Side(combo, N, P, Wt if dst_l == "tiled" else 0, None, extra_pitch=64 if src_l == dst_l == "rows" else 0)
    peers = torch.empty(max(N * S * R, 1), dtype=torch.int32, device="cuda")
    combo.make_peer_table(peers, N, S, R, 4, 5)
    d = combo.workloads.dataset_sizes(N, 2, "cuda") if weighted else None
    combo.round_relayout(dst.t, dst.tile, src.t, src.tile, peers if R else None, N, P, S, R, dataset_sizes=d)
    torch.cuda.synchronize()
    ph = ref.make_peer_table(N, S, R, 4, 5)
    want = ref.gossip_round(Xh, ph, P, S, R, d=None if d is None else d.cpu().numpy())
    got, pad_ok = dst.values()
    assert np.all(np.abs(got - want) <= 1e-6 * np.maximum(np.abs(want), 1e-30))
    assert np.array_equal(bits(got), bits(want))
    assert pad_ok
    back, _ = src.values()
    assert np.array_equal(bits(back), bits(Xh))          # source intact


@pytest.mark.parametrize("src_l,dst_l", LAYOUTS[:2])
@pytest.mark.parametrize("tau", [1, 3])
@pytest.mark.parametrize("N,P,S,R,Wt", [(6, 10_007, 7, 3, 64), (100, 5_003, 7, 3, 64), (16, 30_000, 4, 4, 128),
                                        (10, 1_000, 250, 2, 64)])
def test_relayout_with_local_steps_matches_oracle(combo, ref, src_l, dst_l, tau, N, P, S, R, Wt):
    rng = np.random.default_rng(tau + N)
    Xh = rng.uniform(-0.1, 0.1, (N, P)).astype(np.float32)
    Gh = rng.normal(0, 1e-2, (tau, N, P)).astype(np.float32)
    src = Side(combo, N, P, Wt if src_l == "tiled" else 0, Xh)
    dst = Side(combo, N, P, Wt if dst_l == "tiled" else 0)
    if src.tile:
        grads = torch.stack([torch.from_numpy(np.nan_to_num(np_pack(Gh[k], Wt))).cuda() for k in range(tau)])
    else:
        grads = torch.zeros((tau,) + tuple(src.t.shape), dtype=torch.float32, device="cuda")
        grads[:, :, :P] = torch.from_numpy(Gh).cuda()
    peers = torch.empty(N * S * R, dtype=torch.int32, device="cuda")
    combo.make_peer_table(peers, N, S, R, 1, 1)
    combo.round_relayout(dst.t, dst.tile, src.t, src.tile, peers, N, P, S, R, grads=grads, lr=0.05)
    torch.cuda.synchronize()
    ph = ref.make_peer_table(N, S, R, 1, 1)
    want = ref.local_sgd_steps_then_gossip(Xh.copy(), np.ascontiguousarray(Gh), 0.05, ph, P, S, R)
    got, pad_ok = dst.values()
    assert np.array_equal(bits(got), bits(want)) and pad_ok
    assert np.array_equal(bits(src.values()[0]), bits(Xh))


@pytest.mark.parametrize("src_l,dst_l", LAYOUTS[:2])
@pytest.mark.parametrize("weighted", [False, True])
def test_relayout_with_dynamic_workers_matches_oracle(combo, ref, src_l, dst_l, weighted):
    N, P, S, R, Wt = 12, 30_011, 6, 3, 64
    st = np.ones(N, np.uint8)
    st[[2, 7]] = 0
    st[[4, 11]] = 2
    Xh = np.random.default_rng(5).normal(0, 0.05, (N, P)).astype(np.float32)
    src = Side(combo, N, P, Wt if src_l == "tiled" else 0, Xh)
    dst = Side(combo, N, P, Wt if dst_l == "tiled" else 0)
    std = torch.from_numpy(st).cuda()
    t = torch.empty(N * S * R, dtype=torch.int32, device="cuda")
    combo.make_peer_table_dynamic(t, std, N, S, R, 1, 2)
    d = combo.workloads.dataset_sizes(N, 3, "cuda") if weighted else None
    combo.round_relayout(dst.t, dst.tile, src.t, src.tile, t, N, P, S, R, dataset_sizes=d, status=std)
    torch.cuda.synchronize()
    T = ref.make_peer_table_dynamic(st, N, S, R, 1, 2)
    want = ref.gossip_round_dynamic(Xh, T, st, P, S, R, d=None if d is None else d.cpu().numpy())
    got, pad_ok = dst.values()
    assert np.array_equal(bits(got), bits(want)) and pad_ok


def test_enter_and_leave_a_tiled_arena_without_conversion_passes(combo, ref):
    """rows -> tiled (round 0), tiled -> tiled (rounds 1, 2), tiled -> rows (round 3) equals
    four oracle rounds on row-major data."""
    N, P, S, R = 16, 100_003, 8, 4
    Xh = np.random.default_rng(3).normal(0, 0.02, (N, P)).astype(np.float32)
    arena = combo.GossipArena(N, P, S, R, layout="tiled", seed=9)
    rows = torch.zeros((N, arena.ld), dtype=torch.float32, device="cuda")
    rows[:, :P] = torch.from_numpy(Xh).cuda()
    arena.step_in(rows)
    arena.step()
    arena.step()
    out = torch.full((N, arena.ld), float("nan"), dtype=torch.float32, device="cuda")
    arena.step_out(out)
    torch.cuda.synchronize()
    want = Xh
    for rnd in range(4):
        want = ref.gossip_round(want, ref.make_peer_table(N, S, R, 9, rnd), P, S, R)
    assert np.array_equal(bits(out[:, :P].cpu().numpy()), bits(want))
    assert bool(torch.isnan(out[:, P:]).all())


def test_relayout_argument_errors(combo):
    N, P, S, R = 8, 10_000, 4, 2
    rows = torch.zeros((N, 10_048), dtype=torch.float32, device="cuda")
    t64 = torch.zeros(combo.tiled_elems(N, P, 64), dtype=torch.float32, device="cuda")
    t128 = torch.zeros(combo.tiled_elems(N, P, 128), dtype=torch.float32, device="cuda")
    peers = torch.zeros(N * S * R, dtype=torch.int32, device="cuda")
    with pytest.raises(combo.ComboError) as e:
        combo.round_relayout(t128, 128, t64, 64, peers, N, P, S, R)       # two different tile widths
    assert e.value.status == -3
    with pytest.raises(combo.ComboError) as e:
        combo.round_relayout(t64, 64, t64, 64, peers, N, P, S, R)         # overlap
    assert e.value.status == -2
    with pytest.raises(combo.ComboError) as e:                            # dynamic + local steps
        combo.round_relayout(t64, 64, rows, 0, peers, N, P, S, R, grads=rows.reshape(1, N, -1).clone(), lr=0.1,
                             status=torch.ones(N, dtype=torch.uint8, device="cuda"))
    assert e.value.status == -3
    with pytest.raises(ValueError):
        combo.round_relayout(t64, 64, rows, 0, peers[:5], N, P, S, R)     # short table
    with pytest.raises(ValueError):
        combo.segment_gossip_round(rows.clone(), rows, peers[::2], P, S, R // 2)   # strided table
    with pytest.raises(ValueError):
        combo.segment_gossip_round(rows.clone(), rows, peers, P, S, R,
                                   dataset_sizes=torch.ones(N - 1, device="cuda"))


# ---- strips that hold several segments ------------------------------------------------
SHORT = [
    # N, P, S, R : L = P // S is below the strip width, or not a multiple of four
    (6, 4_096, 4_096, 2), (8, 10_007, 1_000, 3), (32, 9_999, 333, 4), (16, 20_000, 2_000, 9),
    (5, 1_003, 17, 2), (100, 5_003, 301, 3), (12, 8_191, 90, 11), (4, 70_001, 35_000, 1),
    (3, 300, 299, 2),
]


@pytest.mark.parametrize("N,P,S,R", SHORT)
@pytest.mark.parametrize("weighted", [False, True])
@pytest.mark.parametrize("layout", ["rows", "tiled"])
def test_short_segments_match_oracle(combo, ref, N, P, S, R, weighted, layout):
    Xh = np.random.default_rng(N + P).normal(0, 0.05, (N, P)).astype(np.float32)
    Wt = combo.tiled_cols(N, R) if layout == "tiled" else 0
    src = Side(combo, N, P, Wt, Xh)
    dst = Side(combo, N, P, Wt)
    peers = torch.empty(N * S * R, dtype=torch.int32, device="cuda")
    combo.make_peer_table(peers, N, S, R, 2, 3)
    d = combo.workloads.dataset_sizes(N, 2, "cuda") if weighted else None
    if layout == "tiled":
        combo.segment_gossip_round_tiled(dst.t, src.t, Wt, peers, N, P, S, R, dataset_sizes=d)
    else:
        assert combo.round_kernel_kind(N, R) == 1
        combo.segment_gossip_round(dst.t, src.t, peers, P, S, R, dataset_sizes=d)
    torch.cuda.synchronize()
    want = ref.gossip_round(Xh, ref.make_peer_table(N, S, R, 2, 3), P, S, R,
                            d=None if d is None else d.cpu().numpy())
    got, pad_ok = dst.values()
    assert np.array_equal(bits(got), bits(want)) and pad_ok


@pytest.mark.parametrize("N,P,S,R", SHORT[:6])
@pytest.mark.parametrize("tau", [1, 2])
def test_short_segments_with_local_steps(combo, ref, N, P, S, R, tau):
    rng = np.random.default_rng(N + P + tau)
    Xh = rng.uniform(-0.1, 0.1, (N, P)).astype(np.float32)
    Gh = rng.normal(0, 1e-2, (tau, N, P)).astype(np.float32)
    src = Side(combo, N, P, 0, Xh)
    dst = Side(combo, N, P, 0)
    grads = torch.zeros((tau,) + tuple(src.t.shape), dtype=torch.float32, device="cuda")
    grads[:, :, :P] = torch.from_numpy(Gh).cuda()
    peers = torch.empty(N * S * R, dtype=torch.int32, device="cuda")
    combo.make_peer_table(peers, N, S, R, 2, 3)
    d = combo.workloads.dataset_sizes(N, 2, "cuda")
    combo.local_sgd_steps_then_gossip(dst.t, src.t, grads, 0.05, peers, P, S, R, dataset_sizes=d)
    torch.cuda.synchronize()
    want = ref.local_sgd_steps_then_gossip(Xh.copy(), np.ascontiguousarray(Gh), 0.05,
                                           ref.make_peer_table(N, S, R, 2, 3), P, S, R, d=d.cpu().numpy())
    got, pad_ok = dst.values()
    assert np.array_equal(bits(got), bits(want)) and pad_ok


@pytest.mark.parametrize("N,P,S,R", SHORT[:6])
@pytest.mark.parametrize("weighted", [False, True])
def test_short_segments_with_dynamic_workers(combo, ref, N, P, S, R, weighted):
    st = np.ones(N, np.uint8)
    st[0] = 0
    st[N - 1] = 2
    st[N // 2] = 0
    Xh = np.random.default_rng(N * P).normal(0, 0.05, (N, P)).astype(np.float32)
    src = Side(combo, N, P, 0, Xh)
    dst = Side(combo, N, P, 0)
    std = torch.from_numpy(st).cuda()
    t = torch.empty(N * S * R, dtype=torch.int32, device="cuda")
    combo.make_peer_table_dynamic(t, std, N, S, R, 1, 2)
    d = combo.workloads.dataset_sizes(N, 3, "cuda") if weighted else None
    combo.segment_gossip_round_dynamic(dst.t, src.t, t, std, P, S, R, dataset_sizes=d)
    torch.cuda.synchronize()
    T = ref.make_peer_table_dynamic(st, N, S, R, 1, 2)
    want = ref.gossip_round_dynamic(Xh, T, st, P, S, R, d=None if d is None else d.cpu().numpy())
    got, pad_ok = dst.values()
    assert np.array_equal(bits(got), bits(want)) and pad_ok


@pytest.mark.parametrize("N,P,S,R", [c for c in SHORT if c[3] <= 8][:6])
@pytest.mark.parametrize("weighted", [False, True])
@pytest.mark.parametrize("layout", ["rows", "tiled"])
def test_short_segments_table_free_round(combo, ref, N, P, S, R, weighted, layout):
    Xh = np.random.default_rng(N + 2 * P).normal(0, 0.05, (N, P)).astype(np.float32)
    Wt = combo.tiled_cols(N, R) if layout == "tiled" else 0
    src = Side(combo, N, P, Wt, Xh)
    dst = Side(combo, N, P, Wt)
    d = combo.workloads.dataset_sizes(N, 2, "cuda") if weighted else None
    combo.round_hashed(dst.t, src.t, N, P, S, R, 6, 7, tile_cols=Wt, dataset_sizes=d)
    torch.cuda.synchronize()
    want = ref.gossip_round(Xh, ref.make_peer_table(N, S, R, 6, 7), P, S, R,
                            d=None if d is None else d.cpu().numpy())
    got, pad_ok = dst.values()
    assert np.array_equal(bits(got), bits(want)) and pad_ok


# ---- strip order ------------------------------------------------------------------------
@pytest.mark.parametrize("N,P,S,R", [(32, 100_003, 32, 4), (16, 64 * 8 * 5, 4, 2), (8, 1_000, 3, 2),
                                     (100, 64 * 9 + 1, 7, 3), (4, 63, 2, 1)])
@pytest.mark.parametrize("layout", ["rows", "tiled"])
def test_strip_order_does_not_change_results(combo, ref, N, P, S, R, layout):
    """Every XCD working through its own contiguous range of strips (strip counts that are and
    are not multiples of 8, fewer strips than XCDs) gives the same bits."""
    combo.tune(combo.TUNE_SLAB_ORDER, 2)
    Xh = np.random.default_rng(P).normal(0, 0.05, (N, P)).astype(np.float32)
    Wt = combo.tiled_cols(N, R) if layout == "tiled" else 0
    src = Side(combo, N, P, Wt, Xh)
    dst = Side(combo, N, P, Wt)
    peers = torch.empty(N * S * R, dtype=torch.int32, device="cuda")
    combo.make_peer_table(peers, N, S, R, 0, 1)
    if layout == "tiled":
        combo.segment_gossip_round_tiled(dst.t, src.t, Wt, peers, N, P, S, R)
    else:
        combo.segment_gossip_round(dst.t, src.t, peers, P, S, R)
    torch.cuda.synchronize()
    want = ref.gossip_round(Xh, ref.make_peer_table(N, S, R, 0, 1), P, S, R)
    got, pad_ok = dst.values()
    assert np.array_equal(bits(got), bits(want)) and pad_ok


# ---- more replicas than the fully unrolled kernels cover (the paper sweeps R up to 16) ----
@pytest.mark.parametrize("R", [9, 10, 11, 12, 13, 14, 15, 16, 17, 23, 29])
@pytest.mark.parametrize("weighted", [False, True])
@pytest.mark.parametrize("layout", ["rows", "tiled"])
def test_many_replicas_match_oracle(combo, ref, R, weighted, layout):
    N, P, S = 30, 50_021, 10
    Xh = np.random.default_rng(R).normal(0, 0.05, (N, P)).astype(np.float32)
    Wt = combo.tiled_cols(N, R) if layout == "tiled" else 0
    src = Side(combo, N, P, Wt, Xh)
    dst = Side(combo, N, P, Wt)
    peers = torch.empty(N * S * R, dtype=torch.int32, device="cuda")
    combo.make_peer_table(peers, N, S, R, 3, R)
    d = combo.workloads.dataset_sizes(N, 2, "cuda") if weighted else None
    if layout == "tiled":
        combo.segment_gossip_round_tiled(dst.t, src.t, Wt, peers, N, P, S, R, dataset_sizes=d)
    else:
        combo.segment_gossip_round(dst.t, src.t, peers, P, S, R, dataset_sizes=d)
    torch.cuda.synchronize()
    want = ref.gossip_round(Xh, ref.make_peer_table(N, S, R, 3, R), P, S, R,
                            d=None if d is None else d.cpu().numpy())
    got, pad_ok = dst.values()
    assert np.array_equal(bits(got), bits(want)) and pad_ok
