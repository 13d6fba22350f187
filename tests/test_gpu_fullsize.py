"""Full-size parity beyond the sampled windows of test_gpu_parity.py / test_gpu_tiled.py:

  * one whole round of the ResNet-50-sized workload (c3) compared element by element with
    the CPU oracle, in both arena layouts;
  * the BERT-large-sized workload (c5, 5.4e9 elements per half), all five rounds, both
    layouts, on windows placed where the flat element offset (and with it the byte offset)
    crosses 2^30, 2^31 and 2^32, plus a few hundred seeded random 64-column windows.  A
    round is column-separable (output column e depends on input column e only), so a
    window of the full run equals the oracle's run on the window.
Everything is bitwise."""
import numpy as np
import pytest
import torch

import tests.test_gpu_parity as tp

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def combo():
    import paper_1908_07782_amd as c
    assert torch.cuda.is_available()
    c.lib()
    return c


def bits(a):
    return np.ascontiguousarray(a).view(np.uint32)


def host_rows(dev_rows, P):
    out = np.empty((dev_rows.shape[0], P), np.float32)
    for w in range(dev_rows.shape[0]):
        torch.from_numpy(out[w]).copy_(dev_rows[w, :P])
    return out


@pytest.mark.parametrize("layout", ["rows", "tiled"])
def test_c3_resnet50_full_one_round_elementwise(combo, ref, layout):
    wl = combo.workloads.WORKLOADS["c3_resnet50"]
    N, P, S, R = wl.N, wl.P, wl.S, wl.R
    rows = torch.full((N, wl.ld), float("nan"), dtype=torch.float32, device="cuda")
    combo.workloads.fill_params(rows, wl)
    X0 = host_rows(rows, P)
    peers = torch.empty(N * S * R, dtype=torch.int32, device="cuda")
    combo.make_peer_table(peers, N, S, R, wl.hash_seed, 0)
    out = torch.full((N, wl.ld), float("nan"), dtype=torch.float32, device="cuda")
    if layout == "rows":
        combo.segment_gossip_round(out, rows, peers, P, S, R)
    else:
        Wt = combo.tiled_cols(N, R)
        t = torch.full((2, combo.tiled_elems(N, P, Wt)), float("nan"), dtype=torch.float32, device="cuda")
        combo.pack_tiled(t[0], rows, N, P, Wt)
        combo.segment_gossip_round_tiled(t[1], t[0], Wt, peers, N, P, S, R)
        combo.unpack_tiled(out, t[1], N, P, Wt)
    torch.cuda.synchronize()
    want = ref.gossip_round(X0, ref.make_peer_table(N, S, R, wl.hash_seed, 0), P, S, R)
    for w in range(N):                      # row by row: bounded host memory
        got = out[w, :P].cpu().numpy()
        assert np.array_equal(bits(got), bits(want[w])), (layout, w)
    assert bool(torch.isnan(out[:, P:]).all())


def c5_windows(wl, Wt):
    """(start, width) windows: where the flat element offset crosses 2^30, 2^31, 2^32 in the
    row-major layout (offset w*ld + e) and in the tiled one (offset (e/Wt)*N*Wt + w*Wt + e%Wt),
    row ends, segment boundaries, and 300 seeded random 64-column windows."""
    P, N, ld = wl.P, wl.N, wl.ld
    wide = 3000
    cols = {0, P - wide}
    for k in (30, 31, 32):
        cols.add((2 ** k) % ld - wide // 2)                     # row-major: column where row (2^k // ld) crosses
        cols.add(2 ** k // (N * Wt) * Wt - wide // 2)           # tiled: first column of the tile at offset 2^k
    L = P // wl.S
    for s in (1, wl.S // 2, wl.S - 1):
        cols.add(s * L - wide // 2)
    wins = [(int(c), wide) for c in sorted(cols) if 0 <= c <= P - wide]
    rng = np.random.default_rng(2 ** 20 + 5)
    wins += [(int(c), 64) for c in rng.integers(0, P - 64, 300)]
    return wins


@pytest.mark.parametrize("layout", ["rows", "tiled"])
def test_c5_bertlarge_all_rounds_on_offset_crossings_and_random_windows(combo, ref, layout):
    wl = combo.workloads.WORKLOADS["c5_bertlarge"]
    N, P, S, R = wl.N, wl.P, wl.S, wl.R
    Wt = combo.tiled_cols(N, R)
    assert (12 * wl.ld <= 2 ** 32 < 13 * wl.ld) and 2 ** 32 // (N * Wt) * Wt == 268_435_456
    wins = c5_windows(wl, Wt)
    # every window's columns in one index vector, gathered on the device
    col_idx = torch.from_numpy(np.concatenate([np.arange(c, c + n) for c, n in wins])).cuda()
    rows = torch.empty((N, wl.ld), dtype=torch.float32, device="cuda")
    combo.workloads.fill_params(rows, wl)
    peers = torch.empty(N * S * R, dtype=torch.int32, device="cuda")
    if layout == "rows":
        arena = torch.empty((2, N, wl.ld), dtype=torch.float32, device="cuda")
        arena[0].copy_(rows)
        del rows

        def gather(buf):
            return buf[:, col_idx].cpu().numpy()
    else:
        n = combo.tiled_elems(N, P, Wt)
        arena = torch.empty((2, n), dtype=torch.float32, device="cuda")
        combo.pack_tiled(arena[0], rows, N, P, Wt)
        del rows
        flat = (col_idx // Wt) * (N * Wt) + col_idx % Wt        # worker 0's element of each column

        def gather(buf):
            return torch.stack([buf[flat + w * Wt] for w in range(N)]).cpu().numpy()
    arena[1].fill_(float("nan"))
    X0 = gather(arena[0])
    cur = 0
    for rnd in range(wl.rounds):
        combo.make_peer_table(peers, N, S, R, wl.hash_seed, rnd)
        if layout == "rows":
            combo.segment_gossip_round(arena[1 - cur], arena[cur], peers, P, S, R)
        else:
            combo.segment_gossip_round_tiled(arena[1 - cur], arena[cur], Wt, peers, N, P, S, R)
        cur = 1 - cur
    torch.cuda.synchronize()
    got = gather(arena[cur])
    at = 0
    for c0, n in wins:
        want = tp.oracle_rounds_on_window(ref, wl, X0[:, at:at + n], c0, wl.rounds)
        assert np.array_equal(bits(got[:, at:at + n]), bits(want)), (layout, c0, n)
        at += n
