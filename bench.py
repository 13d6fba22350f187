#!/usr/bin/env python3
"""Benchmark of the segmented-gossip aggregation round on one MI355X.

A step is one pass of the whole hot path over the resident arena: the round's peer
table (hash kernel), the gather-average round (Eq. 3 / Eq. 4 of the segmented-gossip
paper; for the fused workload the local SGD step first), and the swap of the front and
back buffers.  The inputs are seeded and synthetic and already in HBM when the timed
region starts.  Prints ONE JSON line: rounds per second, the roofline of the dominant
kernel (the gather-average kernel, HBM bound) measured with HIP events on the launch
stream, and the CPU oracle timed on the host as a reported baseline.

usage: python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]
"""
import argparse
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X published HBM3E bandwidth


def kernel_source_digest():
    h = hashlib.sha256()
    for f in ("gossip_slab_kernel.h", "gossip_slab.hip", "round_device.h", "combo_internal.h"):
        h.update(open(os.path.join(ROOT, "paper_1908_07782_amd", "csrc", f), "rb").read())
    return h.hexdigest()[:16]


def recorded_traffic(workload, layout):
    """(HBM bytes per launch of the dominant kernel, the file they come from): the committed
    rocprofv3 --pmc summary (FETCH_SIZE and WRITE_SIZE, scaled by a copy of known size), or
    (None, None) when there is none or the kernel sources changed since it was taken."""
    tag = "" if layout == "rows" else "_tiled"
    name = f"profiles/gossip_slab_kernel_{workload}{tag}_pmc.txt"
    path = os.path.join(ROOT, name)
    if not os.path.exists(path):
        return None, None
    text = open(path).read()
    m = re.search(r"^kernel_source_digest:\s*(\w+)", text, flags=re.M)
    t = re.search(r"^hbm_bytes_per_launch:\s*([0-9.eE+]+)", text, flags=re.M)
    if not m or not t or m.group(1) != kernel_source_digest():
        return None, None
    return float(t.group(1)), name


def time_kernel(fn, stream, reps=20, warm=3):
    """Average milliseconds of fn() (which enqueues on `stream`), HIP events."""
    import torch
    for _ in range(warm):
        fn()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record(stream)
    for _ in range(reps):
        fn()
    b.record(stream)
    b.synchronize()
    return a.elapsed_time(b) / reps


def sweep_paper(combo, P, layout="rows"):
    """The paper's own sweeps as bandwidth curves (Sec. 5.2: 30 workers; R = 1..16 at
    S = 10; S = 1..10 at R = 2; and 20, 30, 40 workers at the default S = 10, R = 2).  One
    JSON line per point."""
    import torch
    sweep_paper_workers(combo, 30, P, layout,
                        [("R", 10, r) for r in (1, 2, 3, 4, 6, 8, 12, 16, 29)] +
                        [("S", s, 2) for s in (1, 2, 3, 4, 6, 8, 10)] + [("N", 10, 2)])
    for N in (20, 40):
        torch.cuda.empty_cache()
        sweep_paper_workers(combo, N, P, layout, [("N", 10, 2)])


def sweep_paper_workers(combo, N, P, layout, points):
    import torch
    ld = combo.workloads.row_pitch(P)
    wl = combo.workloads.small_case(N, P, 10, 2, scale=0.02)
    rows = torch.zeros((N, ld), dtype=torch.float32, device="cuda")
    combo.workloads.fill_params(rows, wl)
    stream = torch.cuda.current_stream()
    ws = torch.empty(combo.aggregation_divergence_workspace(N, P) // 8, dtype=torch.float64, device="cuda")
    d2 = torch.empty(N, dtype=torch.float64, device="cuda")
    tiled = layout == "tiled"
    if tiled:
        # the tile width follows the replica count (combo_tiled_cols): the arena is packed anew
        # when it changes
        state = {"Wt": 0, "arena": None}

        def arena_for(R):
            Wt = combo.tiled_cols(N, R)
            if Wt != state["Wt"]:
                state["arena"] = None
                state["arena"] = torch.zeros((2, combo.tiled_elems(N, P, Wt)), dtype=torch.float32, device="cuda")
                combo.pack_tiled(state["arena"][0], rows, N, P, Wt)
                state["Wt"] = Wt
            return state["arena"], Wt

        def one_round(peers, S, R):
            arena, Wt = arena_for(R)
            combo.segment_gossip_round_tiled(arena[1], arena[0], Wt, peers, N, P, S, R, stream=stream)

        def rho_of(which, R):
            arena, Wt = arena_for(R)
            combo.aggregation_divergence_tiled(d2, arena[which], Wt, N, P, ws, stream=stream)
            return float(d2.max().sqrt())
    else:
        arena = torch.zeros((2, N, ld), dtype=torch.float32, device="cuda")
        arena[0].copy_(rows)
        del rows

        def one_round(peers, S, R):
            combo.segment_gossip_round(arena[1], arena[0], peers, P, S, R, stream=stream)

        def rho_of(which, R):
            combo.aggregation_divergence(d2, arena[which], P, ws, stream=stream)
            return float(d2.max().sqrt())
    rho0 = rho_of(0, 2)
    for which, S, R in points:
        peers = torch.empty(N * S * R, dtype=torch.int32, device="cuda")
        combo.make_peer_table(peers, N, S, R, 0, 0)
        ms = time_kernel(lambda: one_round(peers, S, R), stream)
        # aggregation divergence (Sec. 4.3, Def. 2) after this one round from independent models
        rho = rho_of(1, R)
        print(json.dumps({"sweep": which, "layout": layout, "N": N, "P": P, "S": S, "R": R,
                          "tiled_cols": combo.tiled_cols(N, R) if tiled else 0, "kernel_ms": ms,
                          "rounds_per_s": 1e3 / ms,
                          "effective_GBs": 4 * (R + 2) * N * P / ms / 1e6,
                          "compulsory_GBs": 8 * N * P / ms / 1e6,
                          "rho_before": rho0, "rho_after_one_round": rho}), flush=True)


def extras(combo, wl):
    """Timings of the other entry points on the workload's shape.  One JSON line each."""
    import torch
    N, P, S, R, ld = wl.N, wl.P, wl.S, wl.R, wl.ld
    arena = torch.zeros((2, N, ld), dtype=torch.float32, device="cuda")
    combo.workloads.fill_params(arena[0], wl)
    stream = torch.cuda.current_stream()
    peers = torch.empty(N * S * R, dtype=torch.int32, device="cuda")

    def emit(name, ms, nbytes=None, **kw):
        rec = {"op": name, "workload": wl.name, "ms": ms}
        if nbytes:
            rec["GBs"] = nbytes / ms / 1e6
        rec.update(kw)
        print(json.dumps(rec), flush=True)

    # practical ceilings on this device for the same footprint: gather-free passes with the
    # kernels' access patterns (combo_bandwidth_probe), torch's own copy, and the library's
    # round with R = 0 (a copy through the slab kernel), both layouts
    foot = N * ld * 4
    for flight in (1, 2, 4, 8):
        emit(f"probe: flat copy, {flight} x 128-bit words in flight per thread", time_kernel(
            lambda: combo.bandwidth_probe(combo.PROBE_COPY, arena[1], arena[0], P, param=flight, stream=stream),
            stream), 2 * foot, note="bytes = read + write")
    for flight in (1, 2):
        # the same passes with the XCDs taking turns at runs of 512 KiB of consecutive blocks
        run = 512 * 1024 // (4096 * flight)
        for kind, what, nbytes in ((combo.PROBE_COPY, "flat copy", 2 * foot), (combo.PROBE_READ, "read only", foot),
                                   (combo.PROBE_WRITE, "write only", foot)):
            emit(f"probe: {what}, {flight} words in flight, XCD runs of {run} blocks (512 KiB)", time_kernel(
                lambda: combo.bandwidth_probe(kind, arena[1], None if kind == combo.PROBE_WRITE else arena[0], P,
                                              cols=run << 4, param=flight, stream=stream), stream), nbytes,
                note="bytes as for the plain probe")
            if kind != combo.PROBE_READ and flight == 1:
                emit(f"probe: {what}, 1 word in flight, XCD runs of {run} blocks, stores written through to "
                     "device scope", time_kernel(
                    lambda: combo.bandwidth_probe(kind, arena[1], None if kind == combo.PROBE_WRITE else arena[0], P,
                                                  cols=(run << 4) | 2, param=flight, stream=stream), stream), nbytes,
                    note="bytes as for the plain probe")
    for flight in (1, 2, 4, 8):
        emit(f"probe: read only, {flight} words in flight", time_kernel(
            lambda: combo.bandwidth_probe(combo.PROBE_READ, arena[1], arena[0], P, param=flight, stream=stream),
            stream), foot, note="bytes = read")
        emit(f"probe: write only, {flight} words in flight", time_kernel(
            lambda: combo.bandwidth_probe(combo.PROBE_WRITE, arena[1], None, P, param=flight, stream=stream),
            stream), foot, note="bytes = write")
    wt0 = combo.tiled_cols(N, R)
    widths = sorted({64, 128, 256, 512, 1024, wt0})
    for cols in widths:
        moved = 8 * N * (P // cols) * cols
        emit(f"probe: row-chunk copy, N chunks of {cols} columns per workgroup (row-major footprint)",
             time_kernel(lambda: combo.bandwidth_probe(combo.PROBE_ROW_CHUNKS, arena[1], arena[0], P, cols=cols,
                                                       stream=stream), stream), moved, note="bytes = read + write")
        emit(f"probe: tile copy, one contiguous N x {cols} tile per workgroup (tiled footprint)",
             time_kernel(lambda: combo.bandwidth_probe(combo.PROBE_TILES, arena[1], arena[0], P, cols=cols,
                                                       stream=stream), stream), moved, note="bytes = read + write")
        if cols <= 128:
            # the same copies with the strip orders the round uses: 2 KiB of consecutive columns of a row
            # per XCD turn on the row-major arena, runs of 16 tiles on the tiled one
            run = 512 // cols
            emit(f"probe: row-chunk copy, N chunks of {cols} columns per workgroup, XCD runs of {run} strips",
                 time_kernel(lambda: combo.bandwidth_probe(combo.PROBE_ROW_CHUNKS, arena[1], arena[0], P, cols=cols,
                                                           param=run, stream=stream), stream), moved,
                 note="bytes = read + write")
            emit(f"probe: tile copy, one contiguous N x {cols} tile per workgroup, XCD runs of 16 tiles",
                 time_kernel(lambda: combo.bandwidth_probe(combo.PROBE_TILES, arena[1], arena[0], P, cols=cols,
                                                           param=16, stream=stream), stream), moved,
                 note="bytes = read + write")
    for k in sorted({1, 3, R + 1}):
        emit(f"probe: {k} read streams + 1 write stream, no reuse out of LDS (worker-major order)",
             time_kernel(lambda: combo.bandwidth_probe(combo.PROBE_MULTI_READ, arena[1], arena[0], P, param=k,
                                                       stream=stream), stream),
             4 * (k + 1) * N * (P // 1024) * 1024, note="bytes = (k reads + 1 write) per element as issued")
    # what the aggregation phase draws on: conflict-free 128-bit LDS reads, 8 workgroups per CU
    lds_wgs, lds_iters = 2048, 4000
    emit("probe: LDS reads, 128-bit, conflict-free, 2048 workgroups of 256 threads", time_kernel(
        lambda: combo.bandwidth_probe(combo.PROBE_LDS_READ, arena[1], None, P, cols=lds_wgs, param=lds_iters,
                                      stream=stream), stream, reps=5, warm=1),
        lds_wgs * 256 * 8 * 16 * lds_iters, note="bytes = LDS bytes read (no HBM traffic)")
    emit("torch copy_ of one arena half", time_kernel(
        lambda: arena[1].copy_(arena[0]), stream), 8 * N * ld, note="bytes = read + write")
    emit("round with R=0, row-major (copy through the slab kernel)", time_kernel(
        lambda: combo.segment_gossip_round(arena[1], arena[0], None, P, S, 0, stream=stream), stream),
        8 * N * P, note="bytes = read + write")
    t0 = torch.zeros((2, combo.tiled_elems(N, P, wt0)), dtype=torch.float32, device="cuda")
    combo.pack_tiled(t0[0], arena[0], N, P, wt0)
    emit("round with R=0, tiled (copy through the slab kernel)", time_kernel(
        lambda: combo.segment_gossip_round_tiled(t0[1], t0[0], wt0, None, N, P, S, 0, stream=stream),
        stream), 8 * N * P, note="bytes = read + write", tiled_cols=wt0)
    # the round itself with the two strip orders (1: workgroup i takes strip i, 2: a contiguous
    # eighth of the strips per XCD; A/B in one process), and the rounds that change layout on
    # the way (no pack / unpack pass)
    combo.make_peer_table(peers, N, S, R, 0, 1)
    for rep in range(2):
        for order in (1, 2):
            combo.tune(combo.TUNE_SLAB_ORDER, order)
            emit(f"combo_segment_gossip_round, row-major, strip order {order} (pass {rep})", time_kernel(
                lambda: combo.segment_gossip_round(arena[1], arena[0], peers, P, S, R, stream=stream), stream),
                8 * N * P, note="bytes = compulsory read + write")
            emit(f"combo_segment_gossip_round_tiled, strip order {order} (pass {rep})", time_kernel(
                lambda: combo.segment_gossip_round_tiled(t0[1], t0[0], wt0, peers, N, P, S, R, stream=stream),
                stream), 8 * N * P, note="bytes = compulsory read + write", tiled_cols=wt0)
    combo.tune(combo.TUNE_SLAB_ORDER, 0)
    emit("combo_round_relayout rows -> tiled", time_kernel(
        lambda: combo.round_relayout(t0[1], wt0, arena[0], 0, peers, N, P, S, R, stream=stream), stream),
        8 * N * P, note="bytes = compulsory read + write", tiled_cols=wt0)
    emit("combo_round_relayout tiled -> rows", time_kernel(
        lambda: combo.round_relayout(arena[1], 0, t0[0], wt0, peers, N, P, S, R, stream=stream), stream),
        8 * N * P, note="bytes = compulsory read + write", tiled_cols=wt0)
    del t0
    emit("combo_make_peer_table", time_kernel(
        lambda: combo.make_peer_table(peers, N, S, R, 0, 1, stream=stream), stream))
    emit("combo_make_peer_table_pooled", time_kernel(
        lambda: combo.make_peer_table_pooled(peers, N, S, R, 0, 1, stream=stream), stream))
    deg = torch.empty(N, dtype=torch.int32, device="cuda")
    emit("combo_peer_in_degree", time_kernel(
        lambda: combo.peer_in_degree(deg, peers, N, S, R, stream=stream), stream))
    # aggregation divergence: read-only pass, 4 bytes per element
    ws = torch.empty(combo.aggregation_divergence_workspace(N, P) // 8, dtype=torch.float64, device="cuda")
    d2 = torch.empty(N, dtype=torch.float64, device="cuda")
    emit("combo_aggregation_divergence", time_kernel(
        lambda: combo.aggregation_divergence(d2, arena[0], P, ws, stream=stream), stream),
        4 * N * P, note="bytes = one read of every element")
    Wt = combo.tiled_cols(N, R)
    tiled = torch.zeros(combo.tiled_elems(N, P, Wt), dtype=torch.float32, device="cuda")
    combo.pack_tiled(tiled, arena[0], N, P, Wt)
    emit("combo_aggregation_divergence_tiled", time_kernel(
        lambda: combo.aggregation_divergence_tiled(d2, tiled, Wt, N, P, ws, stream=stream), stream),
        4 * N * P, note="bytes = one read of every element", tiled_cols=Wt)
    del tiled
    # dynamic round with every tenth worker offline and one newcomer
    st = torch.ones(N, dtype=torch.uint8)
    st[::10] = 0
    st[1] = 2
    st = st.cuda()
    combo.make_peer_table_dynamic(peers, st, N, S, R, 0, 1)
    emit("combo_segment_gossip_round_dynamic", time_kernel(
        lambda: combo.segment_gossip_round_dynamic(arena[1], arena[0], peers, st, P, S, R,
                                                   stream=stream), stream),
        8 * N * P, note="bytes = compulsory read + write")
    combo.make_peer_table(peers, N, S, R, 0, 1)
    dsz = combo.workloads.dataset_sizes(N, 0, "cuda")
    emit("combo_segment_gossip_round (dataset-size weights)", time_kernel(
        lambda: combo.segment_gossip_round(arena[1], arena[0], peers, P, S, R, dataset_sizes=dsz,
                                           stream=stream), stream), 8 * N * P,
        note="bytes = compulsory read + write")
    for tau in (1, 2, 4):
        grads = torch.zeros((tau, N, ld), dtype=torch.float32, device="cuda")
        grads.normal_(0, 1e-3)
        emit(f"combo_local_sgd_steps_then_gossip tau={tau}", time_kernel(
            lambda: combo.local_sgd_steps_then_gossip(arena[1], arena[0], grads, 0.01, peers, P, S, R,
                                                      stream=stream), stream),
            (8 + 4 * tau) * N * P, note="bytes = x read + tau gradient reads + write")
        del grads
    # the same variants on the tiled arena (the layout the round is timed on by default)
    del arena
    t = torch.zeros((2, combo.tiled_elems(N, P, Wt)), dtype=torch.float32, device="cuda")
    rows = torch.zeros((N, ld), dtype=torch.float32, device="cuda")
    combo.workloads.fill_params(rows, wl)
    combo.pack_tiled(t[0], rows, N, P, Wt)
    del rows
    rows2 = torch.zeros((N, ld), dtype=torch.float32, device="cuda")
    emit("combo_pack_tiled", time_kernel(lambda: combo.pack_tiled(t[1], rows2, N, P, Wt, stream=stream), stream),
         8 * N * P, note="bytes = read + write", tiled_cols=Wt)
    emit("combo_unpack_tiled", time_kernel(lambda: combo.unpack_tiled(rows2, t[0], N, P, Wt, stream=stream), stream),
         8 * N * P, note="bytes = read + write", tiled_cols=Wt)
    del rows2
    emit("combo_segment_gossip_round_tiled", time_kernel(
        lambda: combo.segment_gossip_round_tiled(t[1], t[0], Wt, peers, N, P, S, R, stream=stream),
        stream), 8 * N * P, note="bytes = compulsory read + write", tiled_cols=Wt)
    emit("combo_segment_gossip_round_tiled (dataset-size weights)", time_kernel(
        lambda: combo.segment_gossip_round_tiled(t[1], t[0], Wt, peers, N, P, S, R, dataset_sizes=dsz,
                                                 stream=stream), stream), 8 * N * P,
        note="bytes = compulsory read + write", tiled_cols=Wt)
    combo.make_peer_table_dynamic(peers, st, N, S, R, 0, 1)
    emit("combo_segment_gossip_round_tiled (dynamic workers)", time_kernel(
        lambda: combo.segment_gossip_round_tiled(t[1], t[0], Wt, peers, N, P, S, R, status=st,
                                                 stream=stream), stream), 8 * N * P,
        note="bytes = compulsory read + write", tiled_cols=Wt)
    combo.make_peer_table(peers, N, S, R, 0, 1)
    for tau in (1, 2):
        grads = torch.zeros(tau * combo.tiled_elems(N, P, Wt), dtype=torch.float32, device="cuda")
        grads.normal_(0, 1e-3)
        emit(f"combo_local_sgd_steps_then_gossip_tiled tau={tau}", time_kernel(
            lambda: combo.local_sgd_steps_then_gossip_tiled(t[1], t[0], grads, tau, 0.01, Wt, peers,
                                                            N, P, S, R, stream=stream), stream),
            (8 + 4 * tau) * N * P, note="bytes = x read + tau gradient reads + write", tiled_cols=Wt)
        del grads


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def host_memory_available():
    try:
        for line in open("/proc/meminfo"):
            if line.startswith("MemAvailable"):
                return int(line.split()[1]) * 1024
    except OSError:
        pass
    return 0


def to_host(dev_rows, out=None):
    """(N, ld) device matrix -> numpy (N, ld), row by row (bounded staging memory)."""
    import numpy as np
    import torch
    N, ld = dev_rows.shape
    if out is None:
        out = np.empty((N, ld), np.float32)
    for w in range(N):
        torch.from_numpy(out[w]).copy_(dev_rows[w])
    return out


def parity_windows(wl, budget_cols):
    """Column windows for the sampled check of a round too large for the host: row start
    and end, every segment boundary, the columns where the flat element offset crosses
    2^31 and 2^32 in either layout, and seeded random ones up to `budget_cols` columns."""
    import random
    width = 4096
    starts = {0, max(0, wl.P - width)}
    L = wl.P // wl.S
    for s in range(1, wl.S):
        starts.add(max(0, s * L - width // 2))
    rnd = random.Random(wl.P)
    while len(starts) * width < budget_cols:
        starts.add(rnd.randrange(0, max(1, wl.P - width)))
    return [(c, min(width, wl.P - c)) for c in sorted(starts)]


_ORACLE_ROUND_ZERO = {}      # workload name -> the oracle's round 0 on the whole arena (host array)
_ORACLE_F64_WINDOWS = {}     # workload name -> [(first column, width, binary64 oracle result)]


def check_against_oracle(combo, wl, rows, grad_rows, run_round_zero, budget_s):
    """Parity of the timed kernel's first round with the CPU oracle, and the oracle's own
    speed.  `rows` (device, (N, ld)) holds the initial parameters; run_round_zero() makes
    the device run round 0 from them with the timed entry point and returns the result as a
    row-major (N, ld) device matrix.  Returns (parity dict, cpu_baseline dict)."""
    import numpy as np
    from oracle import ref
    N, P, S, R, ld = wl.N, wl.P, wl.S, wl.R, wl.ld
    ph = ref.make_peer_table(N, S, R, wl.hash_seed, 0)
    need = (3 if wl.fused else 2) * N * ld * 4 + 2 * ld * 4
    full = need < 0.6 * host_memory_available()
    got_dev, peers_dev = run_round_zero()
    tables_ok = bool(np.array_equal(peers_dev.cpu().numpy()[:N * S * R].reshape(ph.shape), ph))
    worst, bitwise, checked = 0.0, True, 0

    def compare(got, want):
        nonlocal worst, bitwise, checked
        checked += want.size
        if np.array_equal(got.view(np.uint32), want.view(np.uint32)):
            return
        bitwise = False
        worst = max(worst, float(np.max(np.abs(got - want) / np.maximum(np.abs(want), 1e-30))))

    cpu_s, cpu_rounds, cpu_cols = 0.0, 0, 0
    if full and wl.name in _ORACLE_ROUND_ZERO:
        # the other layout of a workload already checked: same inputs, same table, same result
        Y = _ORACLE_ROUND_ZERO[wl.name]
        import torch
        row = np.empty(ld, np.float32)
        for w in range(N):
            torch.from_numpy(row).copy_(got_dev[w])
            compare(row[:P], Y[w])
        cpu = None
        mode = "every element of round 0"
    elif full:
        Xh = to_host(rows)
        Gh = to_host(grad_rows) if wl.fused else None
        X, Y = Xh[:, :P], np.empty((N, ld), np.float32)[:, :P]
        t0 = time.perf_counter()
        if wl.fused:
            Y = ref.local_sgd_then_gossip(X, Gh[:, :P], wl.lr, ph, P, S, R)
        else:
            ref.gossip_round(X, ph, P, S, R, out=Y)
        cpu_s += time.perf_counter() - t0
        cpu_rounds = 1
        row = np.empty(ld, np.float32)
        import torch
        for w in range(N):
            torch.from_numpy(row).copy_(got_dev[w])
            compare(row[:P], Y[w])
        _ORACLE_ROUND_ZERO[wl.name] = Y
        # binary64 results on a few windows (X holds the served values: the fused oracle call has
        # stepped it in place)
        _ORACLE_F64_WINDOWS[wl.name] = [
            (c0, wd, ref.gossip_round_f64(np.ascontiguousarray(X[:, c0:c0 + wd]), ph, P, S, R, col0=c0))
            for c0, wd in parity_windows(wl, budget_cols=0)[:12]]
        # the oracle of record keeps going on whole rounds until the budget is spent; round 0's
        # result stays intact for the check of the other layout (later rounds alternate between
        # the input buffer and a third one)
        src, dst, spare = Y, X, None
        while cpu_s < budget_s:
            ph_k = ref.make_peer_table(N, S, R, wl.hash_seed, cpu_rounds)
            if wl.fused and src is Y:                # the step is taken in place: work on a copy
                src = np.empty((N, ld), np.float32)[:, :P]
                src[:] = Y
            t0 = time.perf_counter()
            if wl.fused:
                src = ref.local_sgd_then_gossip(src, Gh[:, :P], wl.lr, ph_k, P, S, R)
            else:
                ref.gossip_round(src, ph_k, P, S, R, out=dst)
            cpu_s += time.perf_counter() - t0
            cpu_rounds += 1
            if not wl.fused:
                if spare is None:
                    spare = np.empty((N, ld), np.float32)[:, :P]
                src, dst = dst, (spare if dst is X else X)
        cpu = {"value": cpu_rounds / cpu_s, "unit": "rounds/s", "cores": 1, "kind": "oracle",
               "sample": f"{cpu_rounds} full rounds of {wl.name} (all N={N} workers, all P={P} columns), "
                         f"single thread, {cpu_s:.1f} s", "extrapolated": False}
        if budget_s > 0 and not wl.fused:
            # beside the figure of record: the same oracle library, untouched, called from parallel
            # threads on disjoint column windows of one more round (a round is column-separable)
            from concurrent.futures import ThreadPoolExecutor
            threads = min(16, os.cpu_count() or 1)
            ph_k = ref.make_peer_table(N, S, R, wl.hash_seed, cpu_rounds)
            step = max(64, P // (threads * 4) // 64 * 64)

            def one_window(c0):
                wd = min(step, P - c0)
                ref.gossip_round(src[:, c0:c0 + wd], ph_k, P, S, R, col0=c0, out=dst[:, c0:c0 + wd])

            t0 = time.perf_counter()
            with ThreadPoolExecutor(max_workers=threads) as pool:
                list(pool.map(one_window, range(0, P, step)))
            dt = time.perf_counter() - t0
            same = True
            for c0, wd in parity_windows(wl, budget_cols=0)[:6]:
                want = ref.gossip_round(np.ascontiguousarray(src[:, c0:c0 + wd]), ph_k, P, S, R, col0=c0)
                same = same and np.array_equal(np.ascontiguousarray(dst[:, c0:c0 + wd]).view(np.uint32),
                                               want.view(np.uint32))
            cpu["all_cores"] = {"value": 1.0 / dt, "unit": "rounds/s", "threads": threads,
                                "kind": "the oracle library, unchanged, called from parallel threads on disjoint "
                                        "column windows of one round", "equals_single_call_on_sampled_windows": bool(same)}
        mode = "every element of round 0"
    else:
        # too large for the host: column windows (a round is column-separable: output column e
        # depends on input column e only), oracle timed on the same windows and scaled to P
        wins = parity_windows(wl, budget_cols=1 << 22)
        for c0, wd in wins:
            Xw = np.ascontiguousarray(rows[:, c0:c0 + wd].cpu().numpy())
            t0 = time.perf_counter()
            if wl.fused:
                Gw = np.ascontiguousarray(grad_rows[:, c0:c0 + wd].cpu().numpy())
                want = ref.local_sgd_then_gossip(Xw, Gw, wl.lr, ph, P, S, R, col0=c0)
            else:
                want = ref.gossip_round(Xw, ph, P, S, R, col0=c0)
            cpu_s += time.perf_counter() - t0
            cpu_cols += wd
            compare(np.ascontiguousarray(got_dev[:, c0:c0 + wd].cpu().numpy()), np.ascontiguousarray(want))
        cpu = {"value": cpu_cols / cpu_s / P, "unit": "rounds/s", "cores": 1, "kind": "oracle",
               "sample": f"{len(wins)} column windows of round 0 of {wl.name} ({cpu_cols} of {P} columns, all "
                         f"N={N} workers), single thread, {cpu_s:.1f} s; scaled by P / columns",
               "extrapolated": True}
        mode = f"{len(wins)} column windows of round 0 (host memory too small for the whole arena)"
    # accuracy against the binary64 oracle (reported, not gated: the elementwise relative error of
    # an average of zero-mean values is unbounded, so this is the normwise figure) on a few windows
    norm64 = None
    if wl.name in _ORACLE_F64_WINDOWS:
        num = den = 0.0
        for c0, wd, y64 in _ORACLE_F64_WINDOWS[wl.name]:
            gw = got_dev[:, c0:c0 + wd].cpu().numpy().astype(np.float64)
            num = max(num, float(np.max(np.abs(gw - y64))))
            den = max(den, float(np.max(np.abs(y64))))
        norm64 = num / den if den > 0 else 0.0
    parity = {"tables_bit_exact": tables_ok, "bitwise_equal": bitwise, "max_rel_err": worst,
              "normwise_err_vs_f64_oracle": norm64,
              "elements_checked": checked, "columns_checked": checked // N, "of_columns": P,
              "coverage": mode, "tolerance": 1e-6, "ok": bool(tables_ok and worst <= 1e-6)}
    if cpu is not None:
        cpu["cpu_model"] = cpu_model()
        cpu["host_cores_visible"] = os.cpu_count()
    return parity, cpu


def measure(combo, wl, args, layout, steps, warmup, trials, with_oracle, cpu_budget):
    """One workload in one arena layout: parity of round 0 against the oracle (optional),
    then `trials` timed runs of `steps` steps each.  Returns a dict of results."""
    import torch
    dev = torch.device("cuda:0")
    N, P, S, R = wl.N, wl.P, wl.S, wl.R
    is_tiled = layout == "tiled"
    wt = (args.tiled_cols or combo.tiled_cols(N, R)) if is_tiled else 0
    stream = torch.cuda.current_stream()
    rows = torch.zeros((N, wl.ld), dtype=torch.float32, device=dev)
    combo.workloads.fill_params(rows, wl)
    grad_rows = None
    if wl.fused:
        grad_rows = torch.zeros((N, wl.ld), dtype=torch.float32, device=dev)
        combo.workloads.fill_grads(grad_rows, wl, 0)
    if is_tiled:
        arena = torch.zeros((2, combo.tiled_elems(N, P, wt)), dtype=torch.float32, device=dev)
        combo.pack_tiled(arena[0], rows, N, P, wt)
        grads = None
        if wl.fused:
            grads = torch.zeros_like(arena[0])
            combo.pack_tiled(grads, grad_rows, N, P, wt)
    else:
        arena = torch.zeros((2, N, wl.ld), dtype=torch.float32, device=dev)
        arena[0].copy_(rows)
        grads = grad_rows
    peers = torch.empty(max(N * S * R, 1), dtype=torch.int32, device=dev)
    state = {"cur": 0, "round": 0}
    one_launch = bool(args.one_launch) and R <= 8 and (is_tiled or combo.round_kernel_kind(N, R) == 1)
    g1 = None if grads is None else grads.reshape((1,) + tuple(grads.shape))

    def step(ev=None, stream=stream):
        cur, rnd = state["cur"], state["round"]
        if one_launch:
            if ev is not None:
                ev[0].record(stream)
            combo.round_hashed(arena[1 - cur], arena[cur], N, P, S, R, wl.hash_seed, rnd,
                               grads=g1, lr=wl.lr, tile_cols=wt, stream=stream)
            if ev is not None:
                ev[1].record(stream)
            state["cur"], state["round"] = 1 - cur, rnd + 1
            return
        combo.make_peer_table(peers, N, S, R, wl.hash_seed, rnd, stream=stream)
        if ev is not None:
            ev[0].record(stream)
        if is_tiled and wl.fused:
            combo.local_sgd_steps_then_gossip_tiled(arena[1 - cur], arena[cur], grads, 1, wl.lr, wt,
                                                    peers, N, P, S, R, stream=stream)
        elif is_tiled:
            combo.segment_gossip_round_tiled(arena[1 - cur], arena[cur], wt, peers, N, P, S, R, stream=stream)
        elif wl.fused:
            combo.local_sgd_then_gossip(arena[1 - cur], arena[cur], grads, wl.lr, peers, P, S, R, stream=stream)
        else:
            combo.segment_gossip_round(arena[1 - cur], arena[cur], peers, P, S, R, stream=stream)
        if ev is not None:
            ev[1].record(stream)
        state["cur"], state["round"] = 1 - cur, rnd + 1

    res = {"workload": wl.name, "N": N, "P": P, "S": S, "R": R, "layout": layout, "tiled_cols": wt,
           "fused_local_step": wl.fused, "one_launch_per_round": one_launch}
    if with_oracle:
        def run_round_zero():
            if one_launch:
                combo.make_peer_table(peers, N, S, R, wl.hash_seed, 0, stream=stream)   # for the table check
            step()
            out = arena[state["cur"]]
            if is_tiled:
                back = torch.empty((N, wl.ld), dtype=torch.float32, device=dev)
                combo.unpack_tiled(back, out, N, P, wt)
                out = back
            torch.cuda.synchronize()
            return out, peers
        res["parity"], res["cpu_baseline"] = check_against_oracle(combo, wl, rows, grad_rows, run_round_zero,
                                                                  cpu_budget)
    del rows

    for _ in range(warmup):
        step()
    runs = []
    for _ in range(trials):
        events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                  for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(steps):
            step(events[k])
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        runs.append((t1 - t0, sorted(a.elapsed_time(b) for a, b in events)))
    if args.graph:
        # the same `steps` steps captured once into a HIP graph (the library never allocates,
        # copies or synchronises) and replayed: what is left when launch overhead is taken away
        try:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for k in range(steps):
                    step(stream=torch.cuda.current_stream())
            graph.replay()
            torch.cuda.synchronize()
            walls = []
            for _ in range(trials):
                t0 = time.perf_counter()
                graph.replay()
                torch.cuda.synchronize()
                walls.append(time.perf_counter() - t0)
            walls.sort()
            res["graph_replay"] = {"rounds_per_s": steps / walls[len(walls) // 2],
                                   "ms_per_step": walls[len(walls) // 2] / steps * 1e3,
                                   "steps_per_graph": steps, "launches_per_graph": steps * (1 if one_launch else 2)}
            del graph
        except Exception as e:  # noqa: BLE001 - an extra: the eager figures stand on their own
            res["graph_replay"] = {"error": str(e)[:200]}
    runs.sort(key=lambda r: r[0])
    wall, kern_ms = runs[len(runs) // 2]                 # the median trial
    res["trial_rounds_per_s"] = sorted(steps / r[0] for r in runs)
    res["rounds_per_s"] = steps / wall
    res["ms_per_step"] = wall / steps * 1e3
    kern_avg_ms = sum(kern_ms) / len(kern_ms)
    slab = is_tiled or combo.round_kernel_kind(N, R) == 1
    fused_in_kernel = wl.fused and (is_tiled or one_launch or
                                    (slab and combo.get_tune(combo.TUNE_FUSED_MODE) == 0))
    two_pass = wl.fused and not fused_in_kernel
    # bytes that have to cross the HBM interface per launch: every element read once and
    # written once (+ the gradient when the local step is folded in); the R further reads of
    # an output are LDS reads.  The row-tile kernel re-reads provider rows out of L2.
    hbm_bytes = 8 * N * P + (4 * N * P if fused_in_kernel else 0)
    # (R+1) served values read + 1 written per element, + the gradient read of the local step
    alg_bytes = wl.algorithmic_bytes_per_round + (4 * N * P if wl.fused else 0)
    traffic, source = recorded_traffic(wl.name, layout)
    res["kernel"] = ("gossip_slab_kernel" if slab else "gossip_round_kernel") + \
        (" (after sgd_step_kernel)" if two_pass else "")
    res["kernel_ms_avg"] = kern_avg_ms
    res["kernel_ms_median"] = kern_ms[len(kern_ms) // 2]
    res["kernel_ms_min"] = kern_ms[0]
    res["hbm_bytes_per_launch"] = hbm_bytes
    res["algorithmic_bytes_per_launch"] = alg_bytes
    res["traffic"], res["traffic_source"] = traffic, source
    res["hbm_gbs"] = (traffic or hbm_bytes) / (kern_avg_ms * 1e-3) / 1e9
    res["hbm_frac"] = res["hbm_gbs"] / HBM_PEAK_GBS
    res["effective_gbs"] = alg_bytes / (kern_avg_ms * 1e-3) / 1e9
    res["effective_pct_of_hbm_peak"] = 100.0 * res["effective_gbs"] / HBM_PEAK_GBS   # LDS reuse: may exceed 100
    res["bandwidth_meaningful"] = 8 * N * P > 512 * 1024 * 1024   # below: the arena sits in cache
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--trials", type=int, default=3,
                    help="timed runs of --steps steps each; the line reports the median run")
    ap.add_argument("--workload", default="c5_bertlarge")
    ap.add_argument("--tile", type=int, default=0, help="override COMBO_TUNE_TILE_COLS")
    ap.add_argument("--swizzle", type=int, default=-1, help="override COMBO_TUNE_XCD_SWIZZLE")
    ap.add_argument("--kernel", type=int, default=-1, help="override COMBO_TUNE_KERNEL")
    ap.add_argument("--slab-cols", type=int, default=-1, help="override COMBO_TUNE_SLAB_COLS")
    ap.add_argument("--slab-order", type=int, default=-1, help="override COMBO_TUNE_SLAB_ORDER")
    ap.add_argument("--fused-mode", type=int, default=-1, help="override COMBO_TUNE_FUSED_MODE")
    ap.add_argument("--replicas", type=int, default=-1,
                    help="override R (0 turns the round into a plain copy of known size: the "
                         "calibration kernel for the HBM byte counters)")
    ap.add_argument("--layout", choices=["rows", "tiled"], default="tiled",
                    help="arena layout: tiled [T][N][Wt] (default, the faster one) or row-major "
                         "[N][ld]")
    ap.add_argument("--no-per-config", action="store_true",
                    help="skip the table of all five configurations (both layouts)")
    ap.add_argument("--one-launch", type=int, default=0,
                    help="0 (default): combo_make_peer_table, then the table-driven round; 1: a step is "
                         "ONE combo_round_hashed launch (peer selection inside the kernel; faster only "
                         "for launch-bound sizes)")
    ap.add_argument("--shape", default="", help="ad-hoc workload N,P,S,R instead of a named one")
    ap.add_argument("--tiled-cols", type=int, default=0, help="tile width of the tiled layout")
    ap.add_argument("--no-graph", dest="graph", action="store_false",
                    help="skip the HIP-graph replay of the timed steps (graph_replay in the record)")
    ap.add_argument("--no-cpu-baseline", action="store_true",
                    help="profiling runs: skip the oracle (no parity field, no cpu_baseline) and the graph replay")
    ap.add_argument("--cpu-budget", type=float, default=15.0,
                    help="seconds of CPU work for the oracle baseline (whole rounds)")
    ap.add_argument("--sweep-paper", action="store_true",
                    help="instead of the benchmark line: the paper's R and S sweeps (30 workers)")
    ap.add_argument("--extras", action="store_true",
                    help="instead of the benchmark line: bandwidth probes and timings of the other "
                         "entry points")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (all N simulated workers live in one "
                 "arena); --gpus must be 1")

    import torch
    import paper_1908_07782_amd as combo
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    combo.lib()
    if args.tile:
        combo.tune(combo.TUNE_TILE_COLS, args.tile)
    if args.swizzle >= 0:
        combo.tune(combo.TUNE_XCD_SWIZZLE, args.swizzle)
    if args.kernel >= 0:
        combo.tune(combo.TUNE_KERNEL, args.kernel)
    if args.slab_cols >= 0:
        combo.tune(combo.TUNE_SLAB_COLS, args.slab_cols)
    if args.slab_order >= 0:
        combo.tune(combo.TUNE_SLAB_ORDER, args.slab_order)
    if args.fused_mode >= 0:
        combo.tune(combo.TUNE_FUSED_MODE, args.fused_mode)
    wl = combo.workloads.WORKLOADS[args.workload]
    if args.shape:
        n_, p_, s_, r_ = (int(v) for v in args.shape.split(","))
        wl = combo.workloads.small_case(n_, p_, s_, r_, scale=0.02)
    if args.replicas >= 0:
        import dataclasses
        wl = dataclasses.replace(wl, R=args.replicas, name=f"{wl.name}_R{args.replicas}")
    torch.cuda.set_device(0)
    if args.sweep_paper:
        return sweep_paper(combo, wl.P, args.layout)
    if args.extras:
        return extras(combo, wl)

    oracle = not args.no_cpu_baseline
    if args.no_cpu_baseline:
        args.graph = False                     # profiling runs: the timed eager launches only
    head = measure(combo, wl, args, args.layout, args.steps, args.warmup, args.trials, oracle,
                   args.cpu_budget)
    torch.cuda.empty_cache()
    per_config = []
    if not args.no_per_config:
        # every configuration in both layouts (the headline one only in its other layout), at
        # least 50 steps per trial; parity of round 0 against the oracle on the whole arena
        short = max(args.steps, 50)
        for name, w in combo.workloads.WORKLOADS.items():
            for layout in ("tiled", "rows"):
                if name == wl.name and layout == args.layout:
                    continue
                r = measure(combo, w, args, layout, short, 10, args.trials, oracle, 0.0)
                r.pop("cpu_baseline", None)
                r["steps"] = short
                per_config.append(r)
                torch.cuda.empty_cache()

    out = {
        "metric": "gossip rounds/sec and effective HBM GB/s (% of peak) at N workers x P params",
        "value": head["rounds_per_s"],
        "unit": "rounds/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "trials": args.trials,
        "trial_values": head["trial_rounds_per_s"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": wl.name, "N": wl.N, "P": wl.P, "S": wl.S, "R": wl.R,
                   "fused_local_step": wl.fused, "one_launch_per_round": head["one_launch_per_round"],
                   "layout": args.layout, "tiled_cols": head["tiled_cols"],
                   "kernel": combo.get_tune(combo.TUNE_KERNEL),
                   "slab_cols": combo.get_tune(combo.TUNE_SLAB_COLS),
                   "slab_order": combo.get_tune(combo.TUNE_SLAB_ORDER),
                   "fused_mode": combo.get_tune(combo.TUNE_FUSED_MODE),
                   "tile_cols": combo.get_tune(combo.TUNE_TILE_COLS),
                   "xcd_swizzle": combo.get_tune(combo.TUNE_XCD_SWIZZLE)},
        # (R+1) reads + 1 write per element over the step time: R of the reads are LDS reads, so
        # this rate may exceed the HBM peak; it is not HBM utilisation (that is roofline.frac)
        "effective_gbs": head["algorithmic_bytes_per_launch"] / (head["ms_per_step"] * 1e-3) / 1e9,
        "effective_pct_of_hbm_peak": 100.0 * head["algorithmic_bytes_per_launch"] /
        (head["ms_per_step"] * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "roofline": {
            "bound": "hbm",
            "kernel": head["kernel"],
            "achieved": head["hbm_gbs"],
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": head["hbm_frac"],
            "bytes_per_launch": head["traffic"] or head["hbm_bytes_per_launch"],
            "bytes_source": head["traffic_source"] or
            "compulsory HBM bytes: every element read once and written once (8*N*P, +4*N*P gradient)",
            "traffic": head["traffic"],
            "traffic_source": head["traffic_source"],
            "compulsory_bytes_per_launch": head["hbm_bytes_per_launch"],
            "algorithmic_bytes_per_launch": head["algorithmic_bytes_per_launch"],
            "effective_gbs": head["effective_gbs"],
            "kernel_ms_avg": head["kernel_ms_avg"],
            "kernel_ms_median": head["kernel_ms_median"],
            "kernel_ms_min": head["kernel_ms_min"],
        },
    }
    if "parity" in head:
        out["parity"] = head["parity"]
    if "graph_replay" in head:
        out["graph_replay"] = head["graph_replay"]
    if per_config:
        out["per_config"] = per_config
    if "cpu_baseline" in head:
        out["cpu_baseline"] = head["cpu_baseline"]
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
