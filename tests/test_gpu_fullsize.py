"""Full-size parity beyond the sampled windows of test_gpu_parity.py / test_gpu_tiled.py:

  * one whole round of the ResNet-50-sized workload (c3) compared element by element with
    the CPU oracle, in both arena layouts;
  * the BERT-large-sized workload (c5, 5.4e9 elements per half), all five rounds, both
    layouts, on windows placed where the flat element offset (and with it the byte offset)
    crosses 2^30, 2^31 and 2^32, plus a few hundred seeded random 64-column windows.  A
    round is column-separable (output column e depends on input column e only), so a
    window of the full run equals the oracle's run on the window;
  * properties that hold at any size on every element of the c5 arena (constant rows pinned
    through the oracle's table, identical workers, all peers = column mean);
  * the weighted round (Eq. 3 with dataset sizes) and the dynamic-worker round (Sec. 4.2) on
    the whole c2 arena, both layouts.
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


# --- properties that hold at any size, checked on every element of the c5 arena in the launch
# --- configuration the benchmark times.  The inputs and the views of the tiled arena are made
# --- with torch alone (no pack / unpack kernel of the library is involved).

def c5_arena(combo, layout, fill_row):
    """(input half, NaN-filled output half, row view function, Wt) of a c5-sized arena whose
    row w is fill_row(w) (a 1-D tensor of P floats or a scalar)."""
    wl = combo.workloads.WORKLOADS["c5_bertlarge"]
    N, P, R = wl.N, wl.P, wl.R
    if layout == "rows":
        arena = torch.empty((2, N, wl.ld), dtype=torch.float32, device="cuda")
        arena[0].fill_(float("nan"))
        for w in range(N):
            arena[0][w, :P] = fill_row(w)
        arena[1].fill_(float("nan"))
        return arena, (lambda buf, w: buf[w, :P]), 0
    Wt = combo.tiled_cols(N, R)
    T = -(-P // Wt)
    arena = torch.empty((2, T * N * Wt), dtype=torch.float32, device="cuda")
    v = arena[0].view(T, N, Wt)
    for w in range(N):
        r = fill_row(w)
        if torch.is_tensor(r):
            padded = torch.full((T * Wt,), float("nan"), dtype=torch.float32, device="cuda")
            padded[:P] = r
            v[:, w, :] = padded.view(T, Wt)
            del padded
        else:
            v[:, w, :] = r
    arena[1].fill_(float("nan"))
    return arena, (lambda buf, w: buf.view(T, N, Wt)[:, w, :].reshape(-1)[:P]), Wt


def c5_round(combo, arena, Wt, peers, R=None):
    wl = combo.workloads.WORKLOADS["c5_bertlarge"]
    R = wl.R if R is None else R
    if Wt == 0:
        combo.segment_gossip_round(arena[1], arena[0], peers, wl.P, wl.S, R)
    else:
        combo.segment_gossip_round_tiled(arena[1], arena[0], Wt, peers, wl.N, wl.P, wl.S, R)
    torch.cuda.synchronize()


@pytest.mark.parametrize("layout", ["rows", "tiled"])
def test_c5_constant_rows_pin_every_element_to_its_segment_and_peers(combo, ref, layout):
    """Row w holds one value c_w everywhere.  Then every element of segment s of worker w must be
    the one number ((c_w + c_p0) + c_p1 ...) * fl(1/(R+1)) that the table fixes (Eq. 3), so a
    single misplaced segment boundary or peer index anywhere in the 5.4e9 elements shows."""
    wl = combo.workloads.WORKLOADS["c5_bertlarge"]
    N, P, S, R = wl.N, wl.P, wl.S, wl.R
    c = np.random.default_rng(77).standard_normal(N).astype(np.float32)
    arena, row_of, Wt = c5_arena(combo, layout, lambda w: float(c[w]))
    table = ref.make_peer_table(N, S, R, wl.hash_seed, 3)            # (N, S, R)
    peers = torch.from_numpy(np.ascontiguousarray(table).reshape(-1)).cuda()
    c5_round(combo, arena, Wt, peers)
    inv = np.float32(1.0) / np.float32(R + 1)
    L = P // S
    for w in range(N):
        row = row_of(arena[1], w).contiguous().view(torch.int32)
        for s in range(S):
            acc = c[w]
            for j in range(R):
                acc = np.float32(acc + c[table[w, s, j]])
            want = int(np.float32(acc * inv).view(np.int32))
            lo, hi = s * L, (P if s == S - 1 else (s + 1) * L)
            assert bool((row[lo:hi] == want).all()), (layout, w, s)
        del row


@pytest.mark.parametrize("layout", ["rows", "tiled"])
def test_c5_identical_workers_stay_identical(combo, layout):
    """All workers start from one model (Sec. 4.1 initialisation): after a round all rows are
    bitwise equal to each other, and equal to the input within 2 ulp."""
    wl = combo.workloads.WORKLOADS["c5_bertlarge"]
    N, P, S, R = wl.N, wl.P, wl.S, wl.R
    g = torch.Generator(device="cuda").manual_seed(11)
    x = torch.empty(P, dtype=torch.float32, device="cuda").normal_(0, 0.02, generator=g)
    arena, row_of, Wt = c5_arena(combo, layout, lambda w: x)
    peers = torch.empty(N * S * R, dtype=torch.int32, device="cuda")
    combo.make_peer_table(peers, N, S, R, wl.hash_seed, 1)
    c5_round(combo, arena, Wt, peers)
    first = row_of(arena[1], 0).contiguous()
    assert bool(((first - x).abs() <= 2.5e-7 * x.abs()).all())
    for w in range(1, N):
        assert torch.equal(row_of(arena[1], w).contiguous().view(torch.int32), first.view(torch.int32)), (layout, w)


@pytest.mark.parametrize("layout", ["rows", "tiled"])
def test_c5_size_all_peers_is_the_global_average(combo, layout):
    """R = N-1 (every other worker is pulled): each row is the column mean (the FedAvg limit of
    Sec. 4.3) up to the rounding of N-1 fp32 adds and one scale."""
    wl = combo.workloads.WORKLOADS["c5_bertlarge"]
    N, P, S = wl.N, wl.P, wl.S
    R = N - 1

    def fill(w):
        g = torch.Generator(device="cuda").manual_seed(100 + w)
        return torch.empty(P, dtype=torch.float32, device="cuda").normal_(0, 0.02, generator=g)

    wl_cols = combo.tiled_cols(N, R)
    if layout == "rows":
        arena, row_of, Wt = c5_arena(combo, "rows", fill)
    else:
        # the tile width follows R: build the arena for it
        T = -(-P // wl_cols)
        arena = torch.empty((2, T * N * wl_cols), dtype=torch.float32, device="cuda")
        v = arena[0].view(T, N, wl_cols)
        for w in range(N):
            padded = torch.full((T * wl_cols,), float("nan"), dtype=torch.float32, device="cuda")
            padded[:P] = fill(w)
            v[:, w, :] = padded.view(T, wl_cols)
            del padded
        arena[1].fill_(float("nan"))
        Wt = wl_cols
        row_of = lambda buf, w: buf.view(T, N, Wt)[:, w, :].reshape(-1)[:P]      # noqa: E731
    peers = torch.empty(N * S * R, dtype=torch.int32, device="cuda")
    combo.make_peer_table(peers, N, S, R, wl.hash_seed, 2)
    c5_round(combo, arena, Wt, peers, R=R)
    mean = torch.zeros(P, dtype=torch.float64, device="cuda")
    biggest = 0.0
    for w in range(N):
        r = row_of(arena[0], w)
        mean += r.double()
        biggest = max(biggest, float(r.abs().max()))
    mean /= N
    bound = (N + 1) * 2.0 ** -24 * biggest
    for w in range(N):
        err = float((row_of(arena[1], w).double() - mean).abs().max())
        assert err <= bound, (layout, w, err, bound)


# --- the other variants of the round at a full configuration size (c2), every element

def c2_run(combo, layout, rows, peers, *, dsz=None, status=None):
    wl = combo.workloads.WORKLOADS["c2_resnet18"]
    N, P, S, R = wl.N, wl.P, wl.S, wl.R
    out = torch.full((N, wl.ld), float("nan"), dtype=torch.float32, device="cuda")
    if layout == "rows":
        if status is None:
            combo.segment_gossip_round(out, rows, peers, P, S, R, dataset_sizes=dsz)
        else:
            combo.segment_gossip_round_dynamic(out, rows, peers, status, P, S, R, dataset_sizes=dsz)
    else:
        Wt = combo.tiled_cols(N, R)
        t = torch.full((2, combo.tiled_elems(N, P, Wt)), float("nan"), dtype=torch.float32, device="cuda")
        combo.pack_tiled(t[0], rows, N, P, Wt)
        combo.segment_gossip_round_tiled(t[1], t[0], Wt, peers, N, P, S, R, dataset_sizes=dsz, status=status)
        combo.unpack_tiled(out, t[1], N, P, Wt)
    torch.cuda.synchronize()
    return out


@pytest.mark.parametrize("layout", ["rows", "tiled"])
def test_c2_resnet18_full_weighted_round_elementwise(combo, ref, layout):
    """Eq. (3) with dataset sizes on the whole c2 arena, bit for bit (the quotient included)."""
    wl = combo.workloads.WORKLOADS["c2_resnet18"]
    N, P, S, R = wl.N, wl.P, wl.S, wl.R
    rows = torch.full((N, wl.ld), float("nan"), dtype=torch.float32, device="cuda")
    combo.workloads.fill_params(rows, wl)
    X0 = host_rows(rows, P)
    d = (np.random.default_rng(21).integers(100, 5000, N)).astype(np.float32)
    table = ref.make_peer_table(N, S, R, wl.hash_seed, 4)
    peers = torch.from_numpy(np.ascontiguousarray(table).reshape(-1)).cuda()
    out = c2_run(combo, layout, rows, peers, dsz=torch.from_numpy(d).cuda())
    want = ref.gossip_round(X0, table, P, S, R, d=d)
    for w in range(N):
        assert np.array_equal(bits(out[w, :P].cpu().numpy()), bits(want[w])), (layout, w)


@pytest.mark.parametrize("layout", ["rows", "tiled"])
def test_c2_resnet18_full_dynamic_round_elementwise(combo, ref, layout):
    """Sec. 4.2 on the whole c2 arena: offline workers, newcomers and active ones mixed."""
    wl = combo.workloads.WORKLOADS["c2_resnet18"]
    N, P, S, R = wl.N, wl.P, wl.S, wl.R
    rows = torch.full((N, wl.ld), float("nan"), dtype=torch.float32, device="cuda")
    combo.workloads.fill_params(rows, wl)
    X0 = host_rows(rows, P)
    status = np.ones(N, np.uint8)
    status[[3, 17, 30]] = 0                          # offline
    status[[5, 6, 22]] = 2                           # newcomers
    table = ref.make_peer_table_dynamic(status, N, S, R, wl.hash_seed, 2)
    st_dev = torch.from_numpy(status).cuda()
    peers = torch.empty(N * S * R, dtype=torch.int32, device="cuda")
    combo.make_peer_table_dynamic(peers, st_dev, N, S, R, wl.hash_seed, 2)
    assert np.array_equal(peers.cpu().numpy().reshape(table.shape), table)
    out = c2_run(combo, layout, rows, peers, status=st_dev)
    want = ref.gossip_round_dynamic(X0, table, status, P, S, R)
    for w in range(N):
        assert np.array_equal(bits(out[w, :P].cpu().numpy()), bits(want[w])), (layout, w)
