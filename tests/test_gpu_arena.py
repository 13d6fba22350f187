"""The GossipArena helper (two buffers + table + round counter around the C ABI): whole
simulations of several rounds against the oracle, both layouts, both selection modes."""
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


@pytest.mark.parametrize("layout", ["tiled", "rows"])
@pytest.mark.parametrize("selection", ["segment", "pooled"])
def test_arena_simulation_matches_oracle(combo, ref, layout, selection):
    N, P, S, R, T = 30, 50_003, 10, 2, 6
    rng = np.random.default_rng(3)
    Xh = rng.normal(0, 0.05, (N, P)).astype(np.float32)
    d = rng.integers(100, 2000, N).astype(np.float32)
    arena = combo.GossipArena(N, P, S, R, layout=layout, seed=11, dataset_sizes=d, selection=selection)
    arena.load(torch.from_numpy(Xh).cuda())
    maker = ref.make_peer_table_pooled if selection == "pooled" else ref.make_peer_table
    X = Xh
    rho = []
    for t in range(T):
        if t % 2 == 0:                                   # plain round
            arena.step()
            X = ref.gossip_round(X, maker(N, S, R, 11, t), P, S, R, d=d)
        else:                                            # two local steps, then the round
            Gh = rng.normal(0, 1e-2, (2, N, P)).astype(np.float32)
            g = arena.like_front(2)
            for k in range(2):
                arena.pack_like_front(g[k], torch.from_numpy(Gh[k]).cuda())
            arena.step(grads=g, lr=0.05)
            X = ref.local_sgd_steps_then_gossip(X.copy(), Gh, 0.05, maker(N, S, R, 11, t), P, S, R, d=d)
        rho.append(arena.divergence().cpu().numpy())
        # the table of the step just taken stays readable until the next step
        assert np.array_equal(arena.peers.cpu().numpy()[:N * S * R], maker(N, S, R, 11, t).reshape(-1))
    got = arena.export().cpu().numpy()
    assert np.array_equal(got.view(np.uint32), X.view(np.uint32))
    assert arena.round == T
    want_rho = ref.aggregation_divergence(X, d=d)
    assert np.all(np.abs(rho[-1] - want_rho) <= 2e-12 * want_rho)
    assert rho[-1].max() < rho[0].max()                  # workers move towards consensus
    deg = arena.serve_load().cpu().numpy()
    assert np.array_equal(deg, ref.peer_in_degree(maker(N, S, R, 11, T - 1), N, S, R))


def test_arena_dynamic_workers(combo, ref):
    N, P, S, R = 12, 20_011, 6, 3
    Xh = np.random.default_rng(5).normal(0, 0.05, (N, P)).astype(np.float32)
    st = np.ones(N, np.uint8)
    st[[2, 7]] = 0
    st[11] = 2
    for layout in ("tiled", "rows"):
        arena = combo.GossipArena(N, P, S, R, layout=layout, seed=4).load(torch.from_numpy(Xh).cuda())
        arena.step(status=torch.from_numpy(st).cuda())
        T = ref.make_peer_table_dynamic(st, N, S, R, 4, 0)
        want = ref.gossip_round_dynamic(Xh, T, st, P, S, R)
        assert np.array_equal(arena.export().cpu().numpy().view(np.uint32), want.view(np.uint32))


def test_arena_many_short_rounds_with_interleaved_readers_and_dynamic_steps(combo, ref):
    """Many short rounds without host synchronisation, a serve-load histogram after every
    step, dynamic steps in the middle."""
    N, P, S, R, T = 16, 8_195, 4, 3, 24
    Xh = np.random.default_rng(9).normal(0, 0.05, (N, P)).astype(np.float32)
    st = np.ones(N, np.uint8)
    st[[1, 5]] = 0
    std = torch.from_numpy(st).cuda()
    arena = combo.GossipArena(N, P, S, R, layout="tiled", seed=3)
    arena.load(torch.from_numpy(Xh).cuda())
    degs = []
    for t in range(T):
        arena.step(status=std if t in (7, 8, 15) else None)
        degs.append(arena.serve_load())                  # stays on the device: no host sync in the loop
    torch.cuda.synchronize()
    X = Xh
    for t in range(T):
        if t in (7, 8, 15):
            tab = ref.make_peer_table_dynamic(st, N, S, R, 3, t)
            X = ref.gossip_round_dynamic(X, tab, st, P, S, R)
        else:
            tab = ref.make_peer_table(N, S, R, 3, t)
            X = ref.gossip_round(X, tab, P, S, R)
        flat = np.asarray(tab).reshape(-1)
        assert np.array_equal(degs[t].cpu().numpy(), np.bincount(flat[flat >= 0], minlength=N)), t
    assert np.array_equal(arena.export().cpu().numpy().view(np.uint32), X.view(np.uint32))


@pytest.mark.parametrize("selection", ["segment", "pooled"])
def test_arena_with_many_workers(combo, ref, selection):
    """600 workers: 8- or 16-column tiles keep the arena on the LDS-slab kernel; table,
    rounds, fused steps and the divergence monitor against the oracle."""
    N, P, S, R, T = 600, 3_001, 3, 2, 3
    rng = np.random.default_rng(21)
    Xh = rng.normal(0, 0.05, (N, P)).astype(np.float32)
    d = rng.integers(100, 2000, N).astype(np.float32)
    arena = combo.GossipArena(N, P, S, R, layout="tiled", seed=5, dataset_sizes=d, selection=selection)
    assert arena.tile_cols in (8, 16)
    arena.load(torch.from_numpy(Xh).cuda())
    maker = ref.make_peer_table_pooled if selection == "pooled" else ref.make_peer_table
    X = Xh
    for t in range(T):
        if t == 1:
            Gh = rng.normal(0, 1e-2, (1, N, P)).astype(np.float32)
            g = arena.like_front(1)
            arena.pack_like_front(g[0], torch.from_numpy(Gh[0]).cuda())
            arena.step(grads=g, lr=0.05)
            X = ref.local_sgd_steps_then_gossip(X.copy(), Gh, 0.05, maker(N, S, R, 5, t), P, S, R, d=d)
        else:
            arena.step()
            X = ref.gossip_round(X, maker(N, S, R, 5, t), P, S, R, d=d)
    assert np.array_equal(arena.export().cpu().numpy().view(np.uint32), X.view(np.uint32))
    want_rho = ref.aggregation_divergence(X, d=d)
    got_rho = arena.divergence().cpu().numpy()
    assert np.all(np.abs(got_rho - want_rho) <= 2e-12 * want_rho)
    deg = arena.serve_load().cpu().numpy()
    assert np.array_equal(deg, ref.peer_in_degree(maker(N, S, R, 5, T - 1), N, S, R))
