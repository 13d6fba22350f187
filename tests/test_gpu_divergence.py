"""GPU parity for the aggregation-divergence monitor (Sec. 4.3, Definition 2).

Tolerance: the kernel accumulates in binary64 with a fixed tree (6 shuffle levels, then
at most W/64 + strips-per-workgroup + 2048 sequential additions of non-negative terms),
so its relative error is below about 4000 * 2^-53 = 5e-13; the oracle accumulates in
extended precision.  The tests use 2e-12 relative."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu
RTOL = 2e-12


@pytest.fixture(scope="module")
def combo():
    import paper_1908_07782_amd as c
    assert torch.cuda.is_available()
    c.lib()
    return c


def gpu_divergence(combo, x, P, d=None):
    N = x.shape[0]
    ws = torch.full((combo.aggregation_divergence_workspace(N, P) // 8,), float("nan"),
                    dtype=torch.float64, device="cuda")
    out = torch.full((N,), float("nan"), dtype=torch.float64, device="cuda")
    combo.aggregation_divergence(out, x, P, ws, dataset_sizes=d)
    torch.cuda.synchronize()
    return out.cpu().numpy()


@pytest.mark.parametrize("N,P", [(4, 65_536), (12, 30_001), (32, 200_003), (100, 50_003), (1, 5_000),
                                 (2, 63), (224, 4_097), (256, 1_000), (16, 1_000_000), (300, 2_001),
                                 (512, 1_003), (513, 1_003), (1000, 2_001), (1024, 700)])
@pytest.mark.parametrize("weighted", [False, True])
def test_divergence_matches_oracle(combo, ref, N, P, weighted):
    rng = np.random.default_rng(N * 7 + P)
    Xh = rng.normal(0, 0.02, (N, P)).astype(np.float32)
    ld = combo.workloads.row_pitch(P)
    x = torch.full((N, ld), float("nan"), dtype=torch.float32, device="cuda")   # padding must not be read
    x[:, :P] = torch.from_numpy(Xh).cuda()
    d = combo.workloads.dataset_sizes(N, 5, "cuda") if weighted else None
    got = gpu_divergence(combo, x, P, d)
    want = ref.aggregation_divergence(Xh, d=None if d is None else d.cpu().numpy())
    assert np.all(np.abs(got - want) <= RTOL * want + 1e-300), (got, want)


@pytest.mark.parametrize("N,P,Wt", [(4, 65_536, 512), (32, 200_003, 64), (16, 100_000, 128),
                                    (100, 50_003, 64), (5, 1_000, 256), (256, 5_000, 64),
                                    # 8, 4 and 2 tiles per strip, ragged row counts, very wide tiles,
                                    # and fewer rows than one pass of the workgroup covers
                                    (16, 70_001, 64), (30, 123_457, 64), (48, 33_333, 64), (8, 99_999, 256),
                                    (2, 9_999, 512), (3, 7_777, 512), (8, 50_000, 64), (64, 20_000, 64),
                                    (17, 64 * 4 * 9, 64), (32, 11_689_512 // 16, 64),
                                    # tiles larger than one wavefront's register slots (workgroup kernel), odd row counts
                                    (33, 4_000, 64), (65, 7_000, 64), (128, 9_999, 64), (129, 3_000, 64),
                                    (40, 5_000, 128), (20, 6_001, 256), (100, 1_000_003 // 4, 64),
                                    # narrow tiles and up to 512 workers
                                    (300, 3_001, 16), (512, 2_000, 8), (200, 4_001, 32), (12, 1_000, 8),
                                    (1000, 2_003, 8), (700, 1_500, 16)])
@pytest.mark.parametrize("weighted", [False, True])
def test_divergence_tiled_matches_oracle(combo, ref, N, P, Wt, weighted):
    rng = np.random.default_rng(N + P)
    Xh = rng.normal(0, 0.02, (N, P)).astype(np.float32)
    rows = torch.zeros((N, combo.workloads.row_pitch(P)), dtype=torch.float32, device="cuda")
    rows[:, :P] = torch.from_numpy(Xh).cuda()
    tiled = torch.full((combo.tiled_elems(N, P, Wt),), float("nan"), dtype=torch.float32, device="cuda")
    combo.pack_tiled(tiled, rows, N, P, Wt)           # padding of the last tile stays NaN
    d = combo.workloads.dataset_sizes(N, 5, "cuda") if weighted else None
    ws = torch.empty(combo.aggregation_divergence_workspace(N, P) // 8, dtype=torch.float64, device="cuda")
    out = torch.full((N,), float("nan"), dtype=torch.float64, device="cuda")
    combo.aggregation_divergence_tiled(out, tiled, Wt, N, P, ws, dataset_sizes=d)
    torch.cuda.synchronize()
    want = ref.aggregation_divergence(Xh, d=None if d is None else d.cpu().numpy())
    got = out.cpu().numpy()
    assert np.all(np.abs(got - want) <= RTOL * want + 1e-300), (got, want)


def test_divergence_unaligned_and_reproducible(combo, ref):
    N, P, ld = 7, 10_007, 10_009
    Xh = np.random.default_rng(0).normal(0, 1, (N, P)).astype(np.float32)
    raw = torch.zeros(N * ld + 3, dtype=torch.float32, device="cuda")
    x = raw[1:1 + N * ld].view(N, ld)
    x[:, :P] = torch.from_numpy(Xh).cuda()
    a = gpu_divergence(combo, x, P)
    b = gpu_divergence(combo, x, P)
    assert np.array_equal(a.view(np.uint64), b.view(np.uint64))          # same bits every time
    want = ref.aggregation_divergence(Xh)
    assert np.all(np.abs(a - want) <= RTOL * want)


def test_divergence_of_identical_workers_is_zero_and_full_round_collapses_it(combo, ref):
    N, P, S = 10, 100_000, 4
    row = torch.randn(P, device="cuda") * 0.02
    x = row.repeat(N, 1).contiguous()
    assert np.all(gpu_divergence(combo, x, P) == 0.0)
    x = torch.randn(N, P, device="cuda") * 0.02
    before = gpu_divergence(combo, x, P)
    y = torch.empty_like(x)
    t = torch.empty(N * S * (N - 1), dtype=torch.int32, device="cuda")
    combo.make_peer_table(t, N, S, N - 1, 0, 0)
    combo.segment_gossip_round(y, x, t, P, S, N - 1)
    after = gpu_divergence(combo, y, P)
    assert after.max() < 1e-10 * before.min()          # R = N-1: FedAvg, divergence -> 0 (Sec. 4.3)


def test_divergence_on_the_benchmark_workload(combo, ref):
    """Full-size c2 arena; the oracle recomputes the whole thing (about a second)."""
    wl = combo.workloads.WORKLOADS["c2_resnet18"]
    x = torch.zeros((wl.N, wl.ld), dtype=torch.float32, device="cuda")
    combo.workloads.fill_params(x, wl)
    got = gpu_divergence(combo, x, wl.P)
    want = ref.aggregation_divergence(x[:, :wl.P].cpu().numpy())
    assert np.all(np.abs(got - want) <= RTOL * want)


def test_divergence_errors(combo):
    x = torch.zeros((300, 1024), dtype=torch.float32, device="cuda")
    with pytest.raises(combo.ComboError) as e:
        combo.aggregation_divergence_workspace(1100, 1000)
    assert e.value.status == -3
    with pytest.raises(combo.ComboError) as e:          # 100 rows of a 1024-column tile: too many slots
        combo.aggregation_divergence_tiled(torch.zeros(100, dtype=torch.float64, device="cuda"),
                                           torch.zeros(combo.tiled_elems(100, 2048, 1024), device="cuda"),
                                           1024, 100, 2048, torch.zeros(4096 * 100, dtype=torch.float64,
                                                                        device="cuda"))
    assert e.value.status in (-1, -3)
    out = torch.zeros(4, dtype=torch.float64, device="cuda")
    small = torch.zeros(1, dtype=torch.float64, device="cuda")
    with pytest.raises(combo.ComboError):
        combo.aggregation_divergence(out, x[:4], 1000, small)


@pytest.mark.parametrize("N,weighted", [(1, True), (3, False), (5, True), (30, False), (100, True)])
def test_identical_rows_have_no_divergence_up_to_the_rounding_of_the_mean(combo, ref, N, weighted):
    """All workers hold one model (Sec. 4.1 initialisation): Definition 2 gives zero.  The kernel
    forms the mean as a sum times a rounded reciprocal, so its mean is off by at most
    (N+3) * 2^-53 relative and dist^2 by at most the square of that times |mean|^2: far below
    anything a model distance can resolve, but not exactly zero unless N is a power of two."""
    P = 100_003
    rng = np.random.default_rng(N)
    row = rng.normal(0, 0.02, P).astype(np.float32)
    Xh = np.tile(row, (N, 1))
    ld = combo.workloads.row_pitch(P)
    x = torch.full((N, ld), float("nan"), dtype=torch.float32, device="cuda")
    x[:, :P] = torch.from_numpy(Xh).cuda()
    d = combo.workloads.dataset_sizes(N, 5, "cuda") if weighted else None
    got = gpu_divergence(combo, x, P, d)
    want = ref.aggregation_divergence(Xh, d=None if d is None else d.cpu().numpy())
    assert np.all(want == 0.0)
    bound = ((N + 3) * 2.0 ** -53) ** 2 * float(np.sum(row.astype(np.float64) ** 2))
    assert np.all(got >= 0.0) and np.all(got <= bound), (got, bound)
