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
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc
    summary, or None when there is none or the kernel source changed since."""
    tag = "" if layout == "rows" else "_tiled"
    path = os.path.join(ROOT, "profiles", f"gossip_slab_kernel_{workload}{tag}_pmc.txt")
    if not os.path.exists(path):
        return None
    text = open(path).read()
    m = re.search(r"^kernel_source_digest:\s*(\w+)", text, flags=re.M)
    t = re.search(r"^hbm_bytes_per_launch:\s*([0-9.eE+]+)", text, flags=re.M)
    if not m or not t or m.group(1) != kernel_source_digest():
        return None
    return float(t.group(1))


def cpu_baseline(wl, X0_host, budget_s=15.0):
    """The oracle as it stands (single thread), timed on whole rounds of the same
    workload until about `budget_s` seconds of CPU work are spent."""
    import numpy as np
    from oracle import ref
    X = X0_host
    Y = np.empty_like(X)
    G = None
    if wl.fused:
        G = (np.random.default_rng(1).standard_normal(X.shape, dtype=np.float32) * wl.grad_std)
    t0 = time.perf_counter()
    rounds = 0
    while True:
        ph = ref.make_peer_table(wl.N, wl.S, wl.R, wl.hash_seed, rounds)
        if wl.fused:
            Y = ref.local_sgd_then_gossip(X, G, wl.lr, ph, wl.P, wl.S, wl.R)
        else:
            ref.gossip_round(X, ph, wl.P, wl.S, wl.R, out=Y)
        X, Y = Y, X
        rounds += 1
        dt = time.perf_counter() - t0
        if dt >= budget_s:
            break
    return {"value": rounds / dt, "unit": "rounds/s", "cores": 1, "kind": "oracle",
            "sample": f"{rounds} full rounds of {wl.name} (all N={wl.N} workers, all P={wl.P} "
                      f"columns), single thread, {dt:.1f} s"}


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
    S = 10; S = 1..10 at R = 2).  One JSON line per point."""
    import torch
    N = 30
    ld = combo.workloads.row_pitch(P)
    wl = combo.workloads.small_case(N, P, 10, 2, scale=0.02)
    rows = torch.zeros((N, ld), dtype=torch.float32, device="cuda")
    combo.workloads.fill_params(rows, wl)
    stream = torch.cuda.current_stream()
    points = [("R", 10, r) for r in (1, 2, 3, 4, 6, 8, 12, 16, 29)] + \
             [("S", s, 2) for s in (1, 2, 3, 4, 6, 8, 10)]
    ws = torch.empty(combo.aggregation_divergence_workspace(N, P) // 8, dtype=torch.float64, device="cuda")
    d2 = torch.empty(N, dtype=torch.float64, device="cuda")
    tiled = layout == "tiled"
    if tiled:
        Wt = combo.tiled_cols(N, 2)
        arena = torch.zeros((2, combo.tiled_elems(N, P, Wt)), dtype=torch.float32, device="cuda")
        combo.pack_tiled(arena[0], rows, N, P, Wt)
        del rows

        def one_round(peers, S, R):
            combo.segment_gossip_round_tiled(arena[1], arena[0], Wt, peers, N, P, S, R, stream=stream)

        def rho_of(x):
            combo.aggregation_divergence_tiled(d2, x, Wt, N, P, ws, stream=stream)
            return float(d2.max().sqrt())
    else:
        arena = torch.zeros((2, N, ld), dtype=torch.float32, device="cuda")
        arena[0].copy_(rows)
        del rows

        def one_round(peers, S, R):
            combo.segment_gossip_round(arena[1], arena[0], peers, P, S, R, stream=stream)

        def rho_of(x):
            combo.aggregation_divergence(d2, x, P, ws, stream=stream)
            return float(d2.max().sqrt())
    rho0 = rho_of(arena[0])
    for which, S, R in points:
        peers = torch.empty(N * S * R, dtype=torch.int32, device="cuda")
        combo.make_peer_table(peers, N, S, R, 0, 0)
        ms = time_kernel(lambda: one_round(peers, S, R), stream)
        # aggregation divergence (Sec. 4.3, Def. 2) after this one round from independent models
        rho = rho_of(arena[1])
        print(json.dumps({"sweep": which, "layout": layout, "N": N, "P": P, "S": S, "R": R, "kernel_ms": ms,
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

    # practical ceilings on this device for the same footprint: a plain device-to-device copy
    # and the library's own round with R = 0 (a copy through the slab kernel), both layouts
    emit("torch copy_ of one arena half (ceiling probe)", time_kernel(
        lambda: arena[1].copy_(arena[0]), stream), 8 * N * ld, note="bytes = read + write")
    emit("round with R=0, row-major (copy through the slab kernel)", time_kernel(
        lambda: combo.segment_gossip_round(arena[1], arena[0], None, P, S, 0, stream=stream), stream),
        8 * N * P, note="bytes = read + write")
    wt0 = combo.tiled_cols(N, R)
    t0 = torch.zeros((2, combo.tiled_elems(N, P, wt0)), dtype=torch.float32, device="cuda")
    combo.pack_tiled(t0[0], arena[0], N, P, wt0)
    emit("round with R=0, tiled (copy through the slab kernel)", time_kernel(
        lambda: combo.segment_gossip_round_tiled(t0[1], t0[0], wt0, None, N, P, S, 0, stream=stream),
        stream), 8 * N * P, note="bytes = read + write", tiled_cols=wt0)
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c2_resnet18")
    ap.add_argument("--tile", type=int, default=0, help="override COMBO_TUNE_TILE_COLS")
    ap.add_argument("--swizzle", type=int, default=-1, help="override COMBO_TUNE_XCD_SWIZZLE")
    ap.add_argument("--kernel", type=int, default=-1, help="override COMBO_TUNE_KERNEL")
    ap.add_argument("--slab-cols", type=int, default=-1, help="override COMBO_TUNE_SLAB_COLS")
    ap.add_argument("--fused-mode", type=int, default=-1, help="override COMBO_TUNE_FUSED_MODE")
    ap.add_argument("--replicas", type=int, default=-1,
                    help="override R (0 turns the round into a plain copy of known size: the "
                         "calibration kernel for the HBM byte counters)")
    ap.add_argument("--layout", choices=["rows", "tiled"], default="tiled",
                    help="arena layout: tiled [T][N][Wt] (default, the faster one) or row-major "
                         "[N][ld]")
    ap.add_argument("--no-other-layout", action="store_true",
                    help="skip the short side measurement of the other arena layout")
    ap.add_argument("--one-launch", type=int, default=0,
                    help="0 (default): combo_make_peer_table, then the table-driven round; 1: a step is "
                         "ONE combo_round_hashed launch (peer selection inside the kernel; faster only "
                         "for launch-bound sizes)")
    ap.add_argument("--shape", default="", help="ad-hoc workload N,P,S,R instead of a named one")
    ap.add_argument("--tiled-cols", type=int, default=0, help="tile width of the tiled layout")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-budget", type=float, default=15.0,
                    help="seconds of CPU work for the oracle baseline (whole rounds)")
    ap.add_argument("--sweep-paper", action="store_true",
                    help="instead of the benchmark line: the paper's R and S sweeps (30 workers)")
    ap.add_argument("--extras", action="store_true",
                    help="instead of the benchmark line: timings of the other entry points")
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
    if args.fused_mode >= 0:
        combo.tune(combo.TUNE_FUSED_MODE, args.fused_mode)
    wl = combo.workloads.WORKLOADS[args.workload]
    if args.shape:
        n_, p_, s_, r_ = (int(v) for v in args.shape.split(","))
        wl = combo.workloads.small_case(n_, p_, s_, r_, scale=0.02)
    if args.replicas >= 0:
        import dataclasses
        wl = dataclasses.replace(wl, R=args.replicas, name=f"{wl.name}_R{args.replicas}")
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.sweep_paper:
        return sweep_paper(combo, wl.P, args.layout)
    if args.extras:
        return extras(combo, wl)

    rows = torch.zeros((wl.N, wl.ld), dtype=torch.float32, device=dev)
    combo.workloads.fill_params(rows, wl)
    X0_host = None
    if not args.no_cpu_baseline:
        X0_host = rows[:, :wl.P].cpu().numpy()
    peers = torch.empty(max(wl.N * wl.S * wl.R, 1), dtype=torch.int32, device=dev)
    stream = torch.cuda.current_stream()

    used = {}

    def run_layout(layout, steps, warmup):
        """Time `steps` steps in one arena layout; returns (wall seconds, kernel ms list, Wt)."""
        is_tiled = layout == "tiled"
        wt = (args.tiled_cols or combo.tiled_cols(wl.N, wl.R)) if is_tiled else 0
        if is_tiled:
            arena = torch.zeros((2, combo.tiled_elems(wl.N, wl.P, wt)), dtype=torch.float32, device=dev)
            combo.pack_tiled(arena[0], rows, wl.N, wl.P, wt)
        else:
            arena = torch.zeros((2, wl.N, wl.ld), dtype=torch.float32, device=dev)
            arena[0].copy_(rows)
        grads = None
        if wl.fused:
            grads = torch.zeros_like(arena[0])
            grads.normal_(0.0, wl.grad_std)          # layout-agnostic: i.i.d. values
        state = {"cur": 0, "round": 0}

        one_launch = bool(args.one_launch) and wl.R <= 8 and \
            (is_tiled or combo.round_kernel_kind(wl.N, wl.R) == 1)
        used["one_launch"] = one_launch
        g1 = None if grads is None else grads.reshape((1,) + tuple(grads.shape))

        def step(ev=None):
            cur, rnd = state["cur"], state["round"]
            if one_launch:
                if ev is not None:
                    ev[0].record(stream)
                combo.round_hashed(arena[1 - cur], arena[cur], wl.N, wl.P, wl.S, wl.R, wl.hash_seed, rnd,
                                   grads=g1, lr=wl.lr, tile_cols=wt, stream=stream)
                if ev is not None:
                    ev[1].record(stream)
                state["cur"], state["round"] = 1 - cur, rnd + 1
                return
            combo.make_peer_table(peers, wl.N, wl.S, wl.R, wl.hash_seed, rnd, stream=stream)
            if ev is not None:
                ev[0].record(stream)
            if is_tiled and wl.fused:
                combo.local_sgd_steps_then_gossip_tiled(arena[1 - cur], arena[cur], grads, 1, wl.lr, wt,
                                                        peers, wl.N, wl.P, wl.S, wl.R, stream=stream)
            elif is_tiled:
                combo.segment_gossip_round_tiled(arena[1 - cur], arena[cur], wt, peers, wl.N, wl.P,
                                                 wl.S, wl.R, stream=stream)
            elif wl.fused:
                combo.local_sgd_then_gossip(arena[1 - cur], arena[cur], grads, wl.lr, peers, wl.P,
                                            wl.S, wl.R, stream=stream)
            else:
                combo.segment_gossip_round(arena[1 - cur], arena[cur], peers, wl.P, wl.S, wl.R,
                                           stream=stream)
            if ev is not None:
                ev[1].record(stream)
            state["cur"], state["round"] = 1 - cur, rnd + 1

        for _ in range(warmup):
            step()
        events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                  for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(steps):
            step(events[k])
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        return t1 - t0, sorted(a.elapsed_time(b) for a, b in events), wt

    tiled = args.layout == "tiled"
    wall, kern_ms, Wt = run_layout(args.layout, args.steps, args.warmup)
    one_launch = used["one_launch"]
    other = None
    if not args.no_other_layout:
        other_name = "rows" if tiled else "tiled"
        o_wall, o_ms, o_wt = run_layout(other_name, min(args.steps, 20), 3)
        other = {"layout": other_name, "tiled_cols": o_wt, "rounds_per_s": min(args.steps, 20) / o_wall,
                 "kernel_ms_avg": sum(o_ms) / len(o_ms)}
    del rows

    kern_avg_ms = sum(kern_ms) / len(kern_ms)
    # (R+1) served values read + 1 written per element; the fused local step adds the
    # read of the gradient (folded into the slab fill) or, in two passes, a read of x and
    # g and a write of x
    alg_bytes = wl.algorithmic_bytes_per_round
    if wl.fused:
        fused_in_kernel = tiled or one_launch or (combo.round_kernel_kind(wl.N, wl.R) == 1 and
                                                  combo.get_tune(combo.TUNE_FUSED_MODE) == 0)
        alg_bytes += 4 * wl.N * wl.P * (1 if fused_in_kernel else 3)
    achieved = alg_bytes / (kern_avg_ms * 1e-3) / 1e9
    slab = tiled or combo.round_kernel_kind(wl.N, wl.R) == 1
    two_pass = wl.fused and not tiled and not one_launch and \
        (not slab or combo.get_tune(combo.TUNE_FUSED_MODE) == 1)
    kernel_name = ("gossip_slab_kernel" if slab else "gossip_round_kernel") + \
        (" (+ sgd_step_kernel)" if two_pass else "")
    out = {
        "metric": "gossip rounds/sec and effective HBM GB/s (% of peak) at N workers x P params",
        "value": args.steps / wall,
        "unit": "rounds/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": wall / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": wl.name, "N": wl.N, "P": wl.P, "S": wl.S, "R": wl.R,
                   "fused_local_step": wl.fused, "one_launch_per_round": one_launch, "layout": args.layout, "tiled_cols": Wt, "kernel": combo.get_tune(combo.TUNE_KERNEL),
                   "slab_cols": combo.get_tune(combo.TUNE_SLAB_COLS),
                   "fused_mode": combo.get_tune(combo.TUNE_FUSED_MODE),
                   "tile_cols": combo.get_tune(combo.TUNE_TILE_COLS),
                   "xcd_swizzle": combo.get_tune(combo.TUNE_XCD_SWIZZLE)},
        "effective_hbm_gbs": alg_bytes / (wall / args.steps) / 1e9,
        "effective_hbm_pct_of_peak": 100.0 * alg_bytes / (wall / args.steps) / 1e9 / HBM_PEAK_GBS,
        "roofline": {
            "bound": "hbm",
            "kernel": kernel_name,
            "achieved": achieved,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": recorded_traffic(wl.name, args.layout),
            "algorithmic_bytes_per_launch": alg_bytes,
            "compulsory_bytes_per_launch": 8 * wl.N * wl.P + (4 * wl.N * wl.P if wl.fused else 0),
            "kernel_ms_avg": kern_avg_ms,
            "kernel_ms_median": kern_ms[len(kern_ms) // 2],
            "kernel_ms_min": kern_ms[0],
        },
    }
    if other is not None:
        out["other_layout"] = other
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, X0_host, args.cpu_budget)
        out["cpu_baseline"]["host_cores_visible"] = os.cpu_count()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
