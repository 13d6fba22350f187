"""GPU parity for dynamic workers (Sec. 4.2 of the paper): the masked peer selection is
integer work and must match the oracle bit for bit; the aggregation must match the
same-order binary32 oracle within 1e-6 relative (and, being order-defined, bitwise)."""
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


@pytest.fixture(autouse=True)
def _default_tuning(combo):
    yield
    combo.tune(combo.TUNE_KERNEL, 0)
    combo.tune(combo.TUNE_SLAB_COLS, 0)


def make_status(N, offline, newcomers):
    st = np.ones(N, np.uint8)
    st[list(offline)] = 0
    st[list(newcomers)] = 2
    return st


STATUS_CASES = [
    (12, 6, 3, [2, 7], [4, 11]),
    (5, 4, 3, [1, 3], [4]),            # fewer candidates than R
    (3, 2, 2, [0, 2], []),             # a lone active worker
    (32, 32, 4, [], []),               # everybody active: equals the static table
    (100, 7, 3, range(0, 100, 3), [1, 50]),
    (1000, 2, 5, range(5, 1000, 7), [0, 999]),
    (70, 3, 69, [10], [20]),           # R = N-1 requested, fewer available
    (4, 3, 2, [0, 1, 2, 3], []),       # everybody offline
]


@pytest.mark.parametrize("N,S,R,off,new", STATUS_CASES)
def test_dynamic_table_bit_exact(combo, ref, N, S, R, off, new):
    st = make_status(N, off, new)
    t = torch.full((N * S * R,), -7, dtype=torch.int32, device="cuda")
    combo.make_peer_table_dynamic(t, torch.from_numpy(st).cuda(), N, S, R, 3, 5)
    torch.cuda.synchronize()
    want = ref.make_peer_table_dynamic(st, N, S, R, 3, 5)
    assert np.array_equal(t.cpu().numpy().reshape(want.shape), want)
    if not list(off) and not list(new):
        assert np.array_equal(want, ref.make_peer_table(N, S, R, 3, 5))


def run_dynamic(combo, ref, N, P, S, R, off, new, weighted, poison=True, offset=0, ld=None):
    st = make_status(N, off, new)
    rng = np.random.default_rng(N + P)
    Xh = rng.normal(0, 0.05, (N, P)).astype(np.float32)
    if poison:                           # rows that nobody may read for somebody else
        Xh[list(off)] = np.nan
        Xh[list(new)] = np.nan
    ld = combo.workloads.row_pitch(P) if ld is None else ld
    raw = torch.full((2, N * ld + offset + 8), float("nan"), dtype=torch.float32, device="cuda")
    src = raw[0, offset:offset + N * ld].view(N, ld)
    dst = raw[1, offset:offset + N * ld].view(N, ld)
    src[:, :P] = torch.from_numpy(Xh).cuda()
    dst[:, :P] = 12345.0
    std = torch.from_numpy(st).cuda()
    t = torch.full((max(N * S * R, 1),), -7, dtype=torch.int32, device="cuda")
    combo.make_peer_table_dynamic(t, std, N, S, R, 1, 2)
    d = combo.workloads.dataset_sizes(N, 3, "cuda") if weighted else None
    combo.segment_gossip_round_dynamic(dst, src, t if R > 0 else None, std, P, S, R, dataset_sizes=d)
    torch.cuda.synchronize()
    T = ref.make_peer_table_dynamic(st, N, S, R, 1, 2)
    want = ref.gossip_round_dynamic(Xh, T, st, P, S, R, d=None if d is None else d.cpu().numpy())
    got = dst[:, :P].cpu().numpy()
    assert np.array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    assert np.all(np.abs(got[ok] - want[ok]) <= 1e-6 * np.maximum(np.abs(want[ok]), 1e-30))
    assert np.array_equal(got.view(np.uint32)[ok], want.view(np.uint32)[ok])
    # the poisoned rows reached nobody: only offline rows (copied) and newcomers with
    # nobody to ask (kept) may hold NaN, exactly as in the oracle (checked above)
    assert bool(torch.isnan(dst[:, P:]).all())


@pytest.mark.parametrize("N,P,S,R,off,new", [
    (12, 30_011, 6, 3, [2, 7], [4, 11]),
    (5, 10_007, 4, 3, [1, 3], [4]),
    (32, 70_000, 32, 4, [0, 31], [5]),
    (100, 20_003, 7, 3, range(0, 100, 3), [1, 50]),
    (300, 3_000, 3, 2, [5, 6], [7]),          # too many workers for the slab: elementwise kernel
    (3, 2_000, 2, 2, [0, 2], []),
    (4, 1_000, 3, 2, [0, 1, 2, 3], []),
    (6, 130, 130, 1, [3], [2]),
])
@pytest.mark.parametrize("weighted", [False, True])
@pytest.mark.parametrize("kernel", ["slab", "elementwise"])
def test_dynamic_round_matches_oracle(combo, ref, N, P, S, R, off, new, weighted, kernel):
    combo.tune(combo.TUNE_KERNEL, 0 if kernel == "slab" else 1)
    run_dynamic(combo, ref, N, P, S, R, off, new, weighted)


def test_dynamic_round_unaligned(combo, ref):
    run_dynamic(combo, ref, 12, 10_007, 6, 3, [2], [4], False, offset=1, ld=10_009)


def test_all_active_equals_static_round(combo, ref):
    N, P, S, R = 16, 50_000, 8, 4
    src = torch.randn(N, P, device="cuda") * 0.05
    a = torch.empty_like(src)
    b = torch.empty_like(src)
    st = torch.ones(N, dtype=torch.uint8, device="cuda")
    t = torch.empty(N * S * R, dtype=torch.int32, device="cuda")
    combo.make_peer_table(t, N, S, R, 0, 0)
    combo.segment_gossip_round(a, src, t, P, S, R)
    combo.segment_gossip_round_dynamic(b, src, t, st, P, S, R)
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int32), b.view(torch.int32))


def test_offline_rows_are_copied_even_with_stale_table_entries(combo, ref):
    N, P, S, R = 6, 10_007, 5, 2
    Xh = np.random.default_rng(1).normal(0, 1, (N, P)).astype(np.float32)
    st = np.array([1, 0, 1, 1, 0, 1], np.uint8)
    T = ref.make_peer_table(N, S, R, 0, 0)
    want = ref.gossip_round_dynamic(Xh, T, st, P, S, R)
    for kernel in (0, 1):
        combo.tune(combo.TUNE_KERNEL, kernel)
        src = torch.from_numpy(Xh).cuda()
        dst = torch.zeros_like(src)
        combo.segment_gossip_round_dynamic(dst, src, torch.from_numpy(T.reshape(-1)).cuda(),
                                           torch.from_numpy(st).cuda(), P, S, R)
        torch.cuda.synchronize()
        assert np.array_equal(dst.cpu().numpy().view(np.uint32), want.view(np.uint32))
