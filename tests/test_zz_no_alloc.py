"""The divergence monitor without a workspace argument (combo_aggregation_divergence_noalloc):
same kernels as the workspace forms, partial sums in an array the library holds itself.

Checked against the workspace forms bit for bit (same kernels, same fixed order) and against
the CPU oracle at the monitor's tolerance, on calls in a row that shrink, so that a later call
sees the earlier call's leftovers in the shared array."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu
RTOL = 2e-12          # see test_gpu_divergence.py


@pytest.fixture(scope="module")
def combo():
    import paper_1908_07782_amd as c
    assert torch.cuda.is_available()
    c.lib()
    return c


def _case(combo, N, P, seed):
    rng = np.random.default_rng(seed)
    Xh = rng.normal(0, 0.02, (N, P)).astype(np.float32)
    ld = combo.workloads.row_pitch(P)
    x = torch.full((N, ld), float("nan"), dtype=torch.float32, device="cuda")
    x[:, :P] = torch.from_numpy(Xh).cuda()
    return Xh, x


def _with_workspace(combo, x, P, d, Wt=0, xt=None):
    N = x.shape[0]
    ws = torch.full((combo.aggregation_divergence_workspace(N, P) // 8,), float("nan"),
                    dtype=torch.float64, device="cuda")
    out = torch.full((N,), float("nan"), dtype=torch.float64, device="cuda")
    if Wt:
        combo.aggregation_divergence_tiled(out, xt, Wt, N, P, ws, dataset_sizes=d)
    else:
        combo.aggregation_divergence(out, x, P, ws, dataset_sizes=d)
    torch.cuda.synchronize()
    return out.cpu().numpy()


@pytest.mark.parametrize("weighted", [False, True])
def test_two_calls_in_a_row_the_second_smaller(combo, ref, weighted):
    # large first (fills many workgroups' partials), then smaller shapes that use fewer rows
    # and fewer workgroups of the same array
    for N, P in [(100, 400_003), (32, 50_001), (3, 777)]:
        Xh, x = _case(combo, N, P, N + P)
        d = combo.workloads.dataset_sizes(N, 5, "cuda") if weighted else None
        out = torch.full((N,), float("nan"), dtype=torch.float64, device="cuda")
        combo.aggregation_divergence_noalloc(out, x, N, P, dataset_sizes=d)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        want_gpu = _with_workspace(combo, x, P, d)
        assert np.array_equal(got.view(np.uint64), want_gpu.view(np.uint64)), (N, P)
        want = ref.aggregation_divergence(Xh, d=None if d is None else d.cpu().numpy())
        assert np.all(np.abs(got - want) <= RTOL * want + 1e-300), (N, P, got, want)


def test_tiled_calls_in_a_row(combo, ref):
    for N, P, Wt in [(100, 250_003, 64), (16, 100_000, 128), (128, 9_999, 64), (5, 1_000, 256)]:
        Xh, x = _case(combo, N, P, 3 * N + P)
        xt = torch.full((combo.tiled_elems(N, P, Wt),), float("nan"), dtype=torch.float32, device="cuda")
        combo.pack_tiled(xt, x, N, P, Wt)
        out = torch.full((N,), float("nan"), dtype=torch.float64, device="cuda")
        combo.aggregation_divergence_noalloc(out, xt, N, P, tile_cols=Wt)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        want_gpu = _with_workspace(combo, x, P, None, Wt, xt)
        assert np.array_equal(got.view(np.uint64), want_gpu.view(np.uint64)), (N, P, Wt)
        want = ref.aggregation_divergence(Xh)
        assert np.all(np.abs(got - want) <= RTOL * want + 1e-300), (N, P, Wt)


def test_repeated_calls_give_identical_bits_and_limit_is_enforced(combo):
    N, P = 64, 123_457
    _, x = _case(combo, N, P, 1)
    a = torch.empty(N, dtype=torch.float64, device="cuda")
    b = torch.empty(N, dtype=torch.float64, device="cuda")
    combo.aggregation_divergence_noalloc(a, x, N, P)
    combo.aggregation_divergence_noalloc(b, x, N, P)
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int64), b.view(torch.int64))
    big = torch.zeros((129, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(combo.ComboError) as e:
        combo.aggregation_divergence_noalloc(torch.empty(129, dtype=torch.float64, device="cuda"), big, 129, 64)
    assert e.value.status == -3
