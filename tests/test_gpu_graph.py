"""The library under HIP graph capture: it never allocates, copies, synchronises or clears
memory with a memset, so a whole multi-round experiment - peer tables, rounds with buffer
swaps, local steps, the divergence monitor that needs no workspace - can be captured once
and replayed.  Every replay, with eager work and synchronisations in between, must give the
eager result bit for bit (and that equals the oracle's)."""
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


@pytest.mark.parametrize("layout", ["rows", "tiled"])
def test_a_captured_experiment_replays_to_the_eager_result(combo, ref, layout):
    N, P, S, R, T, lr = 12, 70_003, 6, 3, 4, 0.05
    ld = combo.workloads.row_pitch(P)
    rng = np.random.default_rng(11)
    Xh = rng.normal(0, 0.05, (N, P)).astype(np.float32)
    Gh = rng.normal(0, 1e-2, (N, P)).astype(np.float32)
    Wt = combo.tiled_cols(N, R) if layout == "tiled" else 0
    rows = torch.zeros((N, ld), dtype=torch.float32, device="cuda")
    rows[:, :P] = torch.from_numpy(Xh).cuda()
    grows = torch.zeros((1, N, ld), dtype=torch.float32, device="cuda")
    grows[0, :, :P] = torch.from_numpy(Gh).cuda()
    if Wt:
        n = combo.tiled_elems(N, P, Wt)
        x0 = torch.zeros(n, dtype=torch.float32, device="cuda")
        combo.pack_tiled(x0, rows, N, P, Wt)
        grads = torch.zeros((1, n), dtype=torch.float32, device="cuda")
        combo.pack_tiled(grads[0], grows[0], N, P, Wt)
        arena = torch.zeros((2, n), dtype=torch.float32, device="cuda")
    else:
        x0, grads = rows.clone(), grows
        arena = torch.zeros((2, N, ld), dtype=torch.float32, device="cuda")
    peers = torch.empty(N * S * R, dtype=torch.int32, device="cuda")
    div = torch.zeros((T, N), dtype=torch.float64, device="cuda")

    def experiment():
        """T iterations: fresh table, one local step + round (odd rounds: plain round), swap,
        then the divergence of the new models.  Ends with the result in arena[T % 2]."""
        cur = 0
        for rnd in range(T):
            combo.make_peer_table(peers, N, S, R, 3, rnd)
            g = grads if rnd % 2 == 0 else None
            combo.round_relayout(arena[1 - cur], Wt, arena[cur], Wt, peers, N, P, S, R, grads=g, lr=lr)
            cur = 1 - cur
            combo.aggregation_divergence_noalloc(div[rnd], arena[cur], N, P, tile_cols=Wt)
        return cur

    arena[0].copy_(x0)
    cur = experiment()                       # eager; also loads every kernel before the capture
    torch.cuda.synchronize()
    eager = arena[cur].clone()
    eager_div = div.clone()

    graph = torch.cuda.CUDAGraph()
    arena[0].copy_(x0)
    with torch.cuda.graph(graph):
        assert experiment() == cur
    other = torch.zeros_like(arena)
    for replay in range(3):
        arena[0].copy_(x0)
        arena[1].fill_(float("nan"))
        div.fill_(-1.0)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(arena[cur].view(torch.int32), eager.view(torch.int32)), replay
        assert torch.equal(div.view(torch.int64), eager_div.view(torch.int64)), replay
        # the program's own eager work between the replays
        other[0].copy_(x0)
        combo.round_relayout(other[1], Wt, other[0], Wt, peers, N, P, S, R)
        combo.aggregation_divergence_noalloc(torch.empty(N, dtype=torch.float64, device="cuda"), other[1], N, P,
                                             tile_cols=Wt)
        torch.cuda.synchronize()

    # and the eager result is the oracle's
    want = Xh
    for rnd in range(T):
        ph = ref.make_peer_table(N, S, R, 3, rnd)
        if rnd % 2 == 0:
            want = ref.local_sgd_then_gossip(want.copy(), Gh, lr, ph, P, S, R)
        else:
            want = ref.gossip_round(want, ph, P, S, R)
    if Wt:
        back = torch.zeros((N, ld), dtype=torch.float32, device="cuda")
        combo.unpack_tiled(back, eager, N, P, Wt)
        got = back[:, :P].cpu().numpy()
    else:
        got = eager[:, :P].cpu().numpy()
    assert np.array_equal(got.view(np.uint32), np.ascontiguousarray(want).view(np.uint32))
    d_want = ref.aggregation_divergence(np.ascontiguousarray(want))
    assert np.all(np.abs(eager_div[T - 1].cpu().numpy() - d_want) <= 2e-12 * d_want)
