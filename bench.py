#!/usr/bin/env python3
"""Benchmark of the fused MoE shuffle hot path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic routing:
    fusco_plan -> fusco_dispatch (x -> expert-major tensor) -> fusco_combine (identity experts)
with every input already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config dsv3] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published peak

TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "bench_dsv3_hbm_traffic_pmc.txt")


def measured_traffic(workload: str):
    """HBM-side bytes per launch of the two movers, read from the tracked rocprofv3 --pmc summary of this
    workload (FETCH_SIZE and WRITE_SIZE per dispatch, scaled there by what the same counters read for a plain
    1 GiB copy).  The counters need the profiler, so they cannot be taken inside a timed run; the summary names
    the library source it was taken with, and tests/test_profiles.py fails when that differs from the tree.
    Returns {"dispatch": bytes, "combine": bytes} or {} when there is no summary for the workload."""
    out = {}
    try:
        lines = open(TRAFFIC_PROFILE).read().splitlines()
    except OSError:
        return out
    if not any(l.startswith("workload:") and l.split(":", 1)[1].strip() == workload for l in lines):
        return out
    for l in lines:
        f = l.split()
        if len(f) >= 5 and f[0] in ("dispatch_kernel", "dispatch_tiled_kernel", "combine_kernel"):
            out[f[0].split("_")[0]] = int(f[3]) + int(f[4])          # read bytes + written bytes
    return out


def cpu_baseline(cfg, total_tokens, A, w, xb, min_seconds=8.0, max_passes=64):
    """The CPU oracle, as it stands, on the same workload: plan + two-hop dispatch + fp64 combine,
    repeated until about min_seconds of CPU work have been timed."""
    import oracle
    oracle.build()
    passes, t0 = 0, time.perf_counter()
    while True:
        pl = oracle.plan(A, cfg.E, cfg.D)
        _, eb = oracle.dispatch(pl, xb)
        oracle.combine_f64(eb, w, pl.pair_slot)
        passes += 1
        dt = time.perf_counter() - t0
        if dt >= min_seconds or passes >= max_passes:
            break
    return {"value": cfg.N * passes / dt, "unit": "tokens/s", "cores": 1, "kind": "oracle",
            "sample": "%d of %d tokens of the %s workload, %d passes of plan + two-hop dispatch + fp64 combine "
                      "on one host thread, %.1f s" % (cfg.N, total_tokens, cfg.name, passes, dt),
            "host_cores_available": os.cpu_count()}


def cpu_baseline_all_cores(cfg, total_tokens, A, w, xb, threads, min_seconds=5.0, max_passes=64):
    """The same oracle functions with the independent rows of dispatch and combine handed to `threads` host
    threads in contiguous ranges (its row-subset calls; the plan stays on one thread).  Results are the same
    rows, only computed side by side."""
    import oracle
    from concurrent.futures import ThreadPoolExecutor
    oracle.build()
    slot_cuts = np.linspace(0, cfg.P, threads + 1).astype(np.int64)
    tok_cuts = np.linspace(0, cfg.N, threads + 1).astype(np.int64)
    passes, t0 = 0, time.perf_counter()
    with ThreadPoolExecutor(max_workers=threads) as pool:
        while True:
            pl = oracle.plan(A, cfg.E, cfg.D)
            parts = list(pool.map(lambda i: oracle.dispatch_rows(pl, xb, np.arange(slot_cuts[i], slot_cuts[i + 1])),
                                  range(threads)))
            eb = np.concatenate(parts)
            list(pool.map(lambda i: oracle.combine_f64(eb, w, pl.pair_slot, np.arange(tok_cuts[i], tok_cuts[i + 1])),
                          range(threads)))
            passes += 1
            dt = time.perf_counter() - t0
            if dt >= min_seconds or passes >= max_passes:
                break
    return {"value": cfg.N * passes / dt, "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": "%d of %d tokens of the %s workload, %d passes; dispatch and combine rows split over %d host "
                      "threads, plan on one, %.1f s" % (cfg.N, total_tokens, cfg.name, passes, threads, dt)}


def time_variants(fusco, torch, cfg, L, d_A, d_x, d_w, d_expert, d_out, reps):
    """Event-timed means of the paths that are not the headline: the two-hop dispatch (level 1 then level 2
    as separate passes) and the disaggregated baseline (pack by device, exchange copy, re-pack by expert, and
    the mirror for combine).  Same inputs, same outputs as the fused step."""
    def mean_ms(fn):
        for _ in range(3):
            fn()
        e = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for a, b in e:
            a.record()
            fn()
            b.record()
        torch.cuda.synchronize()
        return sum(a.elapsed_time(b) for a, b in e) / reps

    d_send = torch.empty((L.send_cap, cfg.H), dtype=torch.bfloat16, device="cuda")
    two_hop = mean_ms(lambda: fusco.fusco_dispatch(L, d_x, d_expert, send_buf=d_send, flags=fusco.DISPATCH_TWO_HOP))
    wire = mean_ms(lambda: fusco.fusco_dispatch(L, d_x, d_expert, send_buf=d_send, flags=3))
    # level 1 alone, with and without the planner's duplicate removal ("Planner-off"): packing what would go
    # on the links, one row per (token, device) against one row per (token, expert) in device-major order
    wire_only = mean_ms(lambda: fusco.fusco_dispatch(L, d_x, None, send_buf=d_send, flags=fusco.DISPATCH_WIRE))
    del d_send
    d_part = torch.empty((L.send_cap, cfg.H), dtype=torch.float32, device="cuda")
    two_hop_c = mean_ms(lambda: fusco.fusco_combine_two_hop(L, d_expert, d_w, d_part, d_out))
    del d_part
    U = int(L.array("send_off")[cfg.D].item())
    # segment-descriptor engine on the same rows: the level-1 transfer written as (offset, size) descriptors,
    # packed into one contiguous stream cut into 1 MiB slices
    row = cfg.row_bytes
    src_tok = L.array("send_src")[:U].to(torch.int64)
    desc = torch.stack([src_tok * row, torch.full_like(src_tok, row)], dim=1).contiguous()
    cum = torch.empty(U + 1, dtype=torch.int64, device="cuda")
    seg_status = torch.zeros(1, dtype=torch.int32, device="cuda")
    cap = U * row
    stream_buf = torch.empty(cap, dtype=torch.uint8, device="cuda")
    fill = torch.empty((cap + (1 << 20) - 1) >> 20, dtype=torch.int32, device="cuda")
    seg_scan = mean_ms(lambda: fusco.fusco_segments_scan(desc, cum, seg_status))
    seg_pack = mean_ms(lambda: fusco.fusco_segments_copy(d_x, desc, stream_buf, None, cum, cap, seg_status,
                                                         slice_bytes=1 << 20, slice_fill=fill))
    seg_ok = int(seg_status.item()) == 0 and int(fill.sum().item()) == cap
    seg_pack_plain = mean_ms(lambda: fusco.fusco_segments_copy(d_x, desc, stream_buf, None, cum, cap, seg_status))
    del stream_buf, desc, cum, fill
    Lr = fusco.Layout(cfg.N, cfg.k, cfg.D, cfg.D)
    d_dev = torch.empty_like(d_A)
    rank_plan = mean_ms(lambda: fusco.fusco_disaggregated_plan(Lr, L, d_A, d_dev))
    wire_no_dedup = mean_ms(lambda: fusco.fusco_dispatch(Lr, d_x, d_expert))     # device-major, one row per pair
    st_a = torch.empty_like(d_expert)
    st_b = torch.empty_like(d_expert)
    dis_d = mean_ms(lambda: fusco.fusco_disaggregated_dispatch(L, Lr, d_x, st_a, st_b, d_expert))
    dis_c = mean_ms(lambda: fusco.fusco_disaggregated_combine(L, Lr, d_expert, d_w, st_a, st_b, d_out))
    return {"wire_rows_deduplicated": U, "wire_rows_one_per_pair": cfg.P, "wire_rows_ratio": U / cfg.P,
            "two_hop_dispatch_ms": two_hop, "two_hop_combine_ms": two_hop_c,
            "fused_dispatch_with_wire_tensor_ms": wire,
            "wire_pack_deduplicated_ms": wire_only, "wire_pack_one_per_pair_ms": wire_no_dedup,
            "segments_scan_ms": seg_scan, "segments_pack_ms": seg_pack,
            "segments_pack_GBps": 2.0 * cap / (seg_pack * 1e-3) / 1e9, "segments_ok": seg_ok,
            "segments_pack_without_slices_ms": seg_pack_plain,
            "disaggregated_plan_extra_ms": rank_plan, "disaggregated_dispatch_ms": dis_d,
            "disaggregated_combine_ms": dis_c, "reps": reps}


def measure_ceilings(fusco, torch, cfg, d_x, d_expert, d_out, reps):
    """What the memory system gives for plain row traffic of the same sizes, measured with the library's probe
    kernels (no plan, no arithmetic): the figures the shuffle kernels' bandwidth is to be read against."""
    row = cfg.row_bytes
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    xb = d_x.view(torch.uint8).view(cfg.N, -1)
    eb = d_expert.view(torch.uint8).view(cfg.P, -1)
    ob = d_out.view(torch.uint8).view(cfg.N, -1)
    eb2 = torch.empty_like(eb)

    def gbps(nbytes, fn):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return nbytes / (e0.elapsed_time(e1) / reps * 1e-3) / 1e9

    P, N = cfg.P, cfg.N
    out = {"row_bytes": row, "reps": reps, "unit": "GB/s"}
    for name, scatter in (("launch_order", False), ("scattered_rows", True)):
        out[name] = {
            "fill_P_rows": gbps(P * row, lambda: fusco.fusco_probe_rows(None, eb, 0, 1, scatter)),
            "read_P_rows": gbps(P * row, lambda: fusco.fusco_probe_rows(eb, None, 1, 0, scatter, sink=sink)),
            "copy_P_rows": gbps(2 * P * row, lambda: fusco.fusco_probe_rows(eb, eb2, 1, 1, scatter)),
            "read_1_write_8": gbps((N + P) * row, lambda: fusco.fusco_probe_rows(xb, eb, 1, 8, scatter)),
            "read_8_write_1": gbps((N + P) * row, lambda: fusco.fusco_probe_rows(eb, ob, 8, 1, scatter, True)),
        }
    # the same bytes as one stream of 4 KiB pieces, one 16-byte store (or load) per thread, in address order:
    # the best the memory system gives for writes (a single front) and for a copy
    if (P * row) % 4096 == 0:
        f1, f2 = eb.view(-1, 4096), eb2.view(-1, 4096)
        out["one_front_4KiB_pieces"] = {
            "fill": gbps(P * row, lambda: fusco.fusco_probe_rows(None, f1, 0, 1, False)),
            "read": gbps(P * row, lambda: fusco.fusco_probe_rows(f1, None, 1, 0, False, sink=sink)),
            "copy": gbps(2 * P * row, lambda: fusco.fusco_probe_rows(f1, f2, 1, 1, False)),
        }
    del eb2
    return out


def write_study(fusco, torch, cfg, L, d_x, d_expert, reps):
    """Where the write side of dispatch stands on this GPU: the expert tensor filled (and read) as 4 KiB pieces
    with different assignments of pieces to the 8 XCDs, as whole rows, and by the dispatch itself.  Every fill
    moves the same P * row_bytes bytes through the same address window; only which XCD writes which piece
    changes.  Each variant is launched once to warm up and then `reps` times between two stream events, in the
    order of the returned list (a profiler's per-dispatch rows follow the same order)."""
    nbytes = cfg.P * cfg.row_bytes
    flat = d_expert.view(torch.uint8).view(-1)
    rows = d_expert.view(torch.uint8).view(cfg.P, -1)
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    pieces = nbytes // 4096
    out = []

    def timed(name, moved, fn):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / reps * 1e3
        out.append({"variant": name, "us": us, "GBps": moved / (us * 1e-6) / 1e9, "launches": reps + 1})

    if nbytes % 4096 == 0 and pieces % 8 == 0:
        runs = [r for r in (1, 2, 4, 7, 8, 16, 32, 64, 256, pieces // 8) if (pieces // 8) % r == 0]
        for r in runs:
            timed("fill, 4 KiB pieces, runs of %d per XCD" % r, nbytes,
                  lambda r=r: fusco.fusco_probe_pieces(flat, True, r))
        timed("fill, 4 KiB pieces, scattered", nbytes, lambda: fusco.fusco_probe_pieces(flat, True, scatter=True))
        for r in runs:
            timed("read, 4 KiB pieces, runs of %d per XCD" % r, nbytes,
                  lambda r=r: fusco.fusco_probe_pieces(flat, False, r, sink=sink))
        timed("read, 4 KiB pieces, scattered", nbytes,
              lambda: fusco.fusco_probe_pieces(flat, False, scatter=True, sink=sink))
    timed("fill, whole rows in launch order", nbytes, lambda: fusco.fusco_probe_rows(None, rows, 0, 1, False))
    timed("fill, whole rows scattered", nbytes, lambda: fusco.fusco_probe_rows(None, rows, 0, 1, True))
    timed("read, whole rows in launch order", nbytes, lambda: fusco.fusco_probe_rows(rows, None, 1, 0, False, sink=sink))
    timed("read, whole rows scattered", nbytes, lambda: fusco.fusco_probe_rows(rows, None, 1, 0, True, sink=sink))
    timed("fusco_dispatch (reads N rows, writes P rows)", (cfg.N + cfg.P) * cfg.row_bytes,
          lambda: fusco.fusco_dispatch(L, d_x, d_expert))
    return {"workload": cfg.name, "row_bytes": cfg.row_bytes, "bytes_per_fill": nbytes, "reps": reps, "variants": out}


def cache_probe(fusco, torch, row_bytes, reps=5):
    """Reading a buffer that is cold, that has just been read, and that has just been written: what the 256 MB
    memory-side cache does to a read that follows a write of the same rows (combine after dispatch).  2 GiB are
    written between the measurements so that every one starts from the same state.  Median of `reps`."""
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    scrub = torch.empty((2 << 30) // 16384, 16384, dtype=torch.uint8, device="cuda")

    def timed(fn):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3

    out = []
    for mb in (64, 128, 192, 256, 384, 512, 940):
        rows = mb * (1 << 20) // row_bytes
        buf = torch.empty((rows, row_bytes), dtype=torch.uint8, device="cuda")
        read = lambda: fusco.fusco_probe_rows(buf, None, 1, 0, False, sink=sink)
        res = {"MB": mb, "bytes": rows * row_bytes}
        for mode, before in (("cold", None), ("after_read", read),
                             ("after_fill", lambda: fusco.fusco_probe_rows(None, buf, 0, 1, False)),
                             ("after_write_through_fill", lambda: fusco.fusco_probe_rows(None, buf, 0, 1, False, True))):
            ts = []
            for _ in range(reps):
                fusco.fusco_probe_rows(None, scrub, 0, 1, False)
                torch.cuda.synchronize()
                if before is not None:
                    before()
                ts.append(timed(read))
            ts.sort()
            res[mode + "_us"] = ts[len(ts) // 2]
        out.append(res)
        del buf
    return {"row_bytes": row_bytes, "reps": reps, "sizes": out}


def plan_scaling(fusco, torch, reps=20):
    """fusco_plan alone over growing inputs (k = 8, E = 256, D = 8, uniform random experts): event-timed mean."""
    out = []
    for N in (8192, 32768, 131072, 524288, 2097152):
        k, E, D = 8, 256, 8
        rng = np.random.default_rng(N)
        d_A = torch.from_numpy(rng.integers(0, E, size=(N, k), dtype=np.int32)).cuda()
        L = fusco.Layout(N, k, E, D)
        fusco.fusco_plan(L, d_A)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fusco.fusco_plan(L, d_A)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / reps * 1e3
        out.append({"N": N, "pairs": N * k, "plan_us": us, "ns_per_pair": us * 1e3 / (N * k)})
        del L, d_A
    return {"k": 8, "E": 256, "D": 8, "reps": reps, "sizes": out}


def row_sweep(fusco, torch, np, W, reps=30):
    """Dispatch and combine over the hidden size, at the dsv3 workload's routing (8192 tokens, top-8 of 256 experts,
    bf16 rows of 2 * hidden bytes), per-call kernel times as in the benchmark line.  x larger than 128 MiB is
    dispatched in source chunks; rows longer than 15 KiB are moved in column segments."""
    cfg = W.get_config("dsv3")
    A, w = W.make_routing(cfg)
    d_A, d_w = torch.from_numpy(A).cuda(), torch.from_numpy(w).cuda()
    L = fusco.Layout(cfg.N, cfg.k, cfg.E, cfg.D)
    fusco.fusco_plan(L, d_A)
    torch.cuda.synchronize()
    first = L.array("pair_slot").long()[::cfg.k][:64]
    rows = []
    for H in (2048, 4096, 6144, 7168, 7680, 7936, 8192, 10240, 12288, 16384, 20480, 24576, 32768):
        x = torch.randn((cfg.N, H), device="cuda").to(torch.bfloat16)
        eb = torch.empty((cfg.P, H), dtype=torch.bfloat16, device="cuda")
        out = torch.empty((cfg.N, H), dtype=torch.bfloat16, device="cuda")
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(reps)]
        for r in ev:
            for e in r:
                e.record()
        for _ in range(40):   # past the slower first milliseconds after the allocations' idle time (see token_sweep)
            fusco.fusco_dispatch(L, x, eb)
            fusco.fusco_combine(L, eb, d_w, out)
        torch.cuda.synchronize()
        for i in range(reps):
            fusco.fusco_probe_time_next_call(ev[i][0], ev[i][1])
            fusco.fusco_dispatch(L, x, eb)
            fusco.fusco_probe_time_next_call(ev[i][2], ev[i][3])
            fusco.fusco_combine(L, eb, d_w, out)
        torch.cuda.synchronize()
        if not torch.equal(eb[first], x[:64]):
            raise RuntimeError("row sweep: dispatch moved wrong rows at hidden %d" % H)
        d = float(np.mean([ev[i][0].elapsed_time(ev[i][1]) for i in range(reps)])) * 1e3
        c = float(np.mean([ev[i][2].elapsed_time(ev[i][3]) for i in range(reps)])) * 1e3
        nb = (cfg.N + cfg.P) * H * 2
        rows.append({"hidden": H, "row_bytes": H * 2, "transfer_order": bool(fusco.fusco_dispatch_in_transfer_order(L, H * 2)),
                     "dispatch_us": d, "dispatch_GBps": nb / d / 1e3, "combine_us": c, "combine_GBps": nb / c / 1e3,
                     "frac_of_peak": 2 * nb / ((d + c) * 1e-6) / 1e9 / HBM_PEAK_GBS})
        del x, eb, out
    return {"N": cfg.N, "k": cfg.k, "E": cfg.E, "reps": reps, "sizes": rows}


def token_sweep(fusco, torch, np, W, reps=20):
    """Plan, dispatch and combine over the token count, with the dsv3 workload's shape (bf16 rows of 14336 B, top-8 of
    256 experts, the same seeded routing recipe), per-call kernel times as in the benchmark line."""
    base = W.get_config("dsv3")
    rows = []
    for N in (1024, 2048, 4096, 8192, 12288, 16384, 32768, 65536):
        cfg = base.with_tokens(N)
        A, w = W.make_routing(cfg)
        d_A, d_w = torch.from_numpy(A).cuda(), torch.from_numpy(w).cuda()
        L = fusco.Layout(cfg.N, cfg.k, cfg.E, cfg.D)
        x = torch.randn((cfg.N, cfg.H), device="cuda").to(torch.bfloat16)
        eb = torch.empty((cfg.P, cfg.H), dtype=torch.bfloat16, device="cuda")
        out = torch.empty((cfg.N, cfg.H), dtype=torch.bfloat16, device="cuda")
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(reps)]
        for r in ev:
            for e in r:
                e.record()
        # the routing of every size is made on the host while the GPU idles; its first milliseconds of work after an
        # idle period run slower (dispatch 170-178 us instead of 158 us for some 30 steps at 8192 tokens): warm up past that
        for _ in range(40):
            fusco.fusco_plan(L, d_A)
            fusco.fusco_dispatch(L, x, eb)
            fusco.fusco_combine(L, eb, d_w, out)
        torch.cuda.synchronize()
        for i in range(reps):
            fusco.fusco_probe_time_next_call(ev[i][0], ev[i][1])
            fusco.fusco_plan(L, d_A)
            fusco.fusco_probe_time_next_call(ev[i][2], ev[i][3])
            fusco.fusco_dispatch(L, x, eb)
            fusco.fusco_probe_time_next_call(ev[i][4], ev[i][5])
            fusco.fusco_combine(L, eb, d_w, out)
        torch.cuda.synchronize()
        p, d, c = (float(np.mean([ev[i][2 * j].elapsed_time(ev[i][2 * j + 1]) for i in range(reps)])) * 1e3 for j in range(3))
        nb = (cfg.N + cfg.P) * cfg.row_bytes
        rows.append({"N": N, "tiles": L.tile_count, "transfer_order": bool(fusco.fusco_dispatch_in_transfer_order(L, cfg.row_bytes)),
                     "source_MB": cfg.N * cfg.row_bytes / 1e6, "plan_us": p, "dispatch_us": d, "dispatch_GBps": nb / d / 1e3,
                     "combine_us": c, "combine_GBps": nb / c / 1e3, "frac_of_peak": 2 * nb / ((d + c) * 1e-6) / 1e9 / HBM_PEAK_GBS})
        del x, eb, out, L
    return {"row_bytes": base.row_bytes, "k": base.k, "E": base.E, "reps": reps, "sizes": rows}


def shape_sweep(fusco, torch, np, W, reps=16):
    """Dispatch and combine for other MoE shapes (rows per token, experts, row size, token count), with fusco_dispatch
    on the token walk, on the transfer order where its workgroup shape allows, and as the library chooses: the
    evidence for the choice rules.  The combine reads the tensor dispatch wrote; per-call kernel times."""
    from dataclasses import replace
    base = W.get_config("dsv3")
    shapes = [  # name, N, hidden, k, E
        ("dsv3", 8192, 7168, 8, 256), ("dsv3, 1024 experts", 8192, 7168, 8, 1024), ("dsv3, 64 experts", 8192, 7168, 8, 64),
        ("top-6 of 160, 10 KiB rows", 8192, 5120, 6, 160), ("top-4 of 128, 12 KiB rows", 8192, 6144, 4, 128),
        ("top-4 of 128, 6 KiB rows", 16384, 3072, 4, 128), ("top-4 of 32, 5.6 KiB rows", 8192, 2880, 4, 32),
        ("top-2 of 8, 8 KiB rows", 16384, 4096, 2, 8),
        ("top-8, 8 KiB rows, x 256 MiB", 32768, 4096, 8, 128), ("top-8, 14 KiB rows, x 224 MiB", 16384, 7168, 8, 128),
        ("top-6, 8 KiB rows, x 256 MiB", 32768, 4096, 6, 128), ("top-6, 10 KiB rows, x 240 MiB", 24576, 5120, 6, 128),
        ("top-6, 14 KiB rows, x 224 MiB", 16384, 7168, 6, 128), ("top-5, 10 KiB rows, x 240 MiB", 24576, 5120, 5, 128),
        ("top-4, 7 KiB rows, x 224 MiB", 32768, 3584, 4, 128), ("top-4, 12 KiB rows, x 192 MiB", 16384, 6144, 4, 128),
        ("top-4, 14 KiB rows, x 448 MiB", 32768, 7168, 4, 128), ("top-2, 8 KiB rows, x 256 MiB", 32768, 4096, 2, 8),
    ]
    rows = []
    for name, N, H, k, E in shapes:
        cfg = replace(base, N=N, H=H, k=k, E=E, D=8)
        A, w = W.make_routing(cfg)
        d_A, d_w = torch.from_numpy(A).cuda(), torch.from_numpy(w).cuda()
        L = fusco.Layout(cfg.N, cfg.k, cfg.E, cfg.D)
        fusco.fusco_plan(L, d_A)
        x = torch.randn((cfg.N, cfg.H), device="cuda").to(torch.bfloat16)
        eb = torch.empty((cfg.P, cfg.H), dtype=torch.bfloat16, device="cuda")
        out = torch.empty((cfg.N, cfg.H), dtype=torch.bfloat16, device="cuda")
        nb = (cfg.N + cfg.P) * cfg.row_bytes
        row = {"name": name, "N": N, "hidden": H, "k": k, "E": E, "source_MiB": N * cfg.row_bytes / 2**20,
               "expert_tensor_MiB": cfg.P * cfg.row_bytes / 2**20,
               "library_takes_transfer_order": bool(fusco.fusco_dispatch_in_transfer_order(L, cfg.row_bytes))}
        try:
            for label, which in (("token_walk", 1), ("transfer_order", 2)):
                fusco.fusco_probe_dispatch_kernel(which)
                if which == 2 and not fusco.fusco_dispatch_in_transfer_order(L, cfg.row_bytes):
                    row[label] = None        # the workgroup shape does not allow it
                    continue
                ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(reps)]
                for r in ev:
                    for e in r:
                        e.record()
                for _ in range(40):
                    fusco.fusco_dispatch(L, x, eb)
                    fusco.fusco_combine(L, eb, d_w, out)
                torch.cuda.synchronize()
                for i in range(reps):
                    fusco.fusco_probe_time_next_call(ev[i][0], ev[i][1])
                    fusco.fusco_dispatch(L, x, eb)
                    fusco.fusco_probe_time_next_call(ev[i][2], ev[i][3])
                    fusco.fusco_combine(L, eb, d_w, out)
                torch.cuda.synchronize()
                d = float(np.mean([ev[i][0].elapsed_time(ev[i][1]) for i in range(reps)])) * 1e3
                c = float(np.mean([ev[i][2].elapsed_time(ev[i][3]) for i in range(reps)])) * 1e3
                row[label] = {"dispatch_us": d, "combine_us": c, "frac_of_peak": 2 * nb / ((d + c) * 1e-6) / 1e9 / HBM_PEAK_GBS}
        finally:
            fusco.fusco_probe_dispatch_kernel(0)
        rows.append(row)
        del x, eb, out, L
    return {"reps": reps, "shapes": rows}


def dispatch_study(fusco, torch, np, W, reps=16):
    """The tiled dispatch over the workgroups it keeps per compute unit (fusco_probe_dispatch_occupancy), with and
    without the pull of a tile's source rows (fusco_probe_dispatch_pull), with x in the memory-side cache and cold
    (rotating over copies of more than 700 MB in all): the evidence for the library's choice of both.  dsv3 routing,
    8192 tokens unless said otherwise; dispatch alternates with the combine as in a step; per-call kernel times."""
    base = W.get_config("dsv3")
    rows = []
    for N, H in ((8192, 2560), (8192, 3072), (8192, 4096), (8192, 5120), (8192, 6144), (8192, 6656), (8192, 7168), (8192, 7680),
                 (8192, 8192), (4096, 12288), (4096, 7168), (8704, 7168), (9216, 7168), (16384, 7168)):
        cfg = base.with_tokens(N)
        A, w = W.make_routing(cfg)
        d_A, d_w = torch.from_numpy(A).cuda(), torch.from_numpy(w).cuda()
        L = fusco.Layout(cfg.N, cfg.k, cfg.E, cfg.D)
        fusco.fusco_plan(L, d_A)
        copies = max(2, (700 << 20) // (N * H * 2) + 1)
        xs = [torch.randn((N, H), device="cuda").to(torch.bfloat16) for _ in range(copies)]
        eb = torch.empty((cfg.P, H), dtype=torch.bfloat16, device="cuda")
        out = torch.empty((N, H), dtype=torch.bfloat16, device="cuda")
        row = {"N": N, "hidden": H, "row_bytes": 2 * H, "source_MiB": N * H * 2 / 2**20, "cases": []}
        try:
            for pull in (1, 2):
                for rot in (1, copies):
                    times = {}
                    for wgs in (16, 12, 8, 7, 6, 5, 4):
                        fusco.fusco_probe_dispatch_pull(pull)
                        fusco.fusco_probe_dispatch_occupancy(wgs)
                        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(reps)]
                        for r in ev:
                            for e in r:
                                e.record()
                        turn = 0
                        for _ in range(40):
                            fusco.fusco_dispatch(L, xs[turn % rot], eb)
                            fusco.fusco_combine(L, eb, d_w, out)
                            turn += 1
                        torch.cuda.synchronize()
                        for i in range(reps):
                            fusco.fusco_probe_time_next_call(ev[i][0], ev[i][1])
                            fusco.fusco_dispatch(L, xs[turn % rot], eb)
                            fusco.fusco_combine(L, eb, d_w, out)
                            turn += 1
                        torch.cuda.synchronize()
                        times[str(wgs)] = float(np.mean([ev[i][0].elapsed_time(ev[i][1]) for i in range(reps)])) * 1e3
                    row["cases"].append({"pull": pull == 2, "x": "cold" if rot > 1 else "in the memory-side cache",
                                         "dispatch_us_by_workgroups_per_cu": times})
            fusco.fusco_probe_dispatch_pull(0)
            fusco.fusco_probe_dispatch_occupancy(0)
            ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(reps)]
            for r in ev:
                for e in r:
                    e.record()
            for _ in range(40):
                fusco.fusco_dispatch(L, xs[0], eb)
                fusco.fusco_combine(L, eb, d_w, out)
            torch.cuda.synchronize()
            for i in range(reps):
                fusco.fusco_probe_time_next_call(ev[i][0], ev[i][1])
                fusco.fusco_dispatch(L, xs[0], eb)
                fusco.fusco_combine(L, eb, d_w, out)
            torch.cuda.synchronize()
            row["library_choice_us"] = float(np.mean([ev[i][0].elapsed_time(ev[i][1]) for i in range(reps)])) * 1e3
        finally:
            fusco.fusco_probe_dispatch_pull(0)
            fusco.fusco_probe_dispatch_occupancy(0)
        rows.append(row)
        del xs, eb, out, L
    return {"reps": reps, "k": base.k, "E": base.E, "sizes": rows}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="dsv3")
    ap.add_argument("--cpu-sample-tokens", type=int, default=0, help="tokens for the CPU baseline (0 = all)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="capture the step (plan, dispatch, combine) into one HIP graph and time its replays")
    ap.add_argument("--cold-sets", type=int, default=1,
                    help="rotate the step over this many copies of its buffers (cache-cold figures for the small "
                         "configurations; choose enough copies to exceed 512 MB)")
    ap.add_argument("--no-variants", action="store_true",
                    help="skip timing the two-hop dispatch and the disaggregated multi-stage baseline")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip the plain row-traffic probes (fill, read, copy, 1:8 and 8:1 mixes) of the same sizes")
    ap.add_argument("--write-study", action="store_true",
                    help="instead of the benchmark line, print the write-side study: fills and reads of the expert "
                         "tensor with different assignments of 4 KiB pieces to the XCDs, whole rows, the dispatch")
    ap.add_argument("--cache-probe", action="store_true",
                    help="instead of the benchmark line, print the memory-side cache probe: a buffer read cold, "
                         "right after a read and right after a write of it")
    ap.add_argument("--plan-scaling", action="store_true",
                    help="instead of the benchmark line, print fusco_plan's time for 8 Ki to 2 Mi tokens")
    ap.add_argument("--row-sweep", action="store_true",
                    help="instead of the benchmark line, print dispatch and combine times for hidden sizes 2048 ... 32768")
    ap.add_argument("--token-sweep", action="store_true",
                    help="instead of the benchmark line, print plan, dispatch and combine times for 1 Ki to 64 Ki tokens")
    ap.add_argument("--shape-sweep", action="store_true",
                    help="instead of the benchmark line, print dispatch and combine times of other MoE shapes with "
                         "fusco_dispatch on the token walk and on the transfer order")
    ap.add_argument("--dispatch-study", action="store_true",
                    help="instead of the benchmark line, print the tiled dispatch's time over the workgroups per compute "
                         "unit, with and without the pull of the source rows, with x cached and cold")
    ap.add_argument("--probe-copy", action="store_true",
                    help="also launch the 1 GiB plain-copy probe 3 times (calibration of traffic counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (expert-parallel devices are virtual partitions of "
              "one GPU's buffers); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import workloads as W
    import paper_2512_22036_amd as fusco

    fusco.load_library()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    torch.cuda.set_device(0)

    cfg = W.get_config(args.config)
    if args.cache_probe:
        print(json.dumps({"cache_probe": cache_probe(fusco, torch, cfg.row_bytes)}))
        return 0
    if args.token_sweep:
        print(json.dumps({"token_sweep": token_sweep(fusco, torch, np, W)}))
        return 0
    if args.row_sweep:
        print(json.dumps({"row_sweep": row_sweep(fusco, torch, np, W)}))
        return 0
    if args.shape_sweep:
        print(json.dumps({"shape_sweep": shape_sweep(fusco, torch, np, W)}))
        return 0
    if args.dispatch_study:
        print(json.dumps({"dispatch_study": dispatch_study(fusco, torch, np, W)}))
        return 0
    if args.plan_scaling:
        print(json.dumps({"plan_scaling": plan_scaling(fusco, torch)}))
        return 0
    A, w = W.make_routing(cfg)
    d_A = torch.from_numpy(A).cuda()
    d_w = torch.from_numpy(w).cuda()
    L = fusco.Layout(cfg.N, cfg.k, cfg.E, cfg.D)
    d_out = torch.empty((cfg.N, cfg.H), dtype=torch.bfloat16, device="cuda")
    if cfg.payload == "bf16":
        xb = W.make_activations(cfg)
        d_x = torch.from_numpy(xb.view(np.int16)).cuda().view(torch.bfloat16)
        d_expert = torch.empty((cfg.P, cfg.H), dtype=torch.bfloat16, device="cuda")
        d_y = d_expert                                   # identity experts
        dispatch_kwargs = {}
    else:
        # fp8 payload + per-128-element scales travel as two planes; the experts' output is a bf16 tensor
        # of its own (dequantisation and expert compute are outside the library)
        q, sc = W.make_fp8_activations(cfg)
        xb = q
        d_x = torch.from_numpy(q).cuda()
        d_expert = torch.empty((cfg.P, cfg.H), dtype=torch.uint8, device="cuda")
        d_y = torch.from_numpy(W.make_expert_output(cfg).view(np.int16)).cuda().view(torch.bfloat16)
        dispatch_kwargs = {"x_aux": torch.from_numpy(sc).cuda(),
                           "expert_aux": torch.empty((cfg.P, sc.shape[1]), dtype=torch.float32, device="cuda")}

    # cold runs: the step walks over R copies of its buffers (same contents), so that a configuration
    # small enough to live in the 256 MB memory-side cache finds none of its rows there
    sets = [(d_x, d_expert, d_y, d_out, dispatch_kwargs)]
    for _ in range(1, max(1, args.cold_sets)):
        kw = {name: t.clone() for name, t in dispatch_kwargs.items()}
        e = torch.empty_like(d_expert)
        sets.append((d_x.clone(), e, e if d_y is d_expert else d_y.clone(), torch.empty_like(d_out), kw))
    turn = [0]

    def step():
        sx, se, sy, so, kw = sets[turn[0] % len(sets)]
        turn[0] += 1
        fusco.fusco_plan(L, d_A)
        fusco.fusco_dispatch(L, sx, se, **kw)
        fusco.fusco_combine(L, sy, d_w, so)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    if args.write_study:
        if cfg.payload != "bf16":
            print("bench.py: --write-study needs a bf16 configuration", file=sys.stderr)
            return 2
        print(json.dumps({"write_study": write_study(fusco, torch, cfg, L, d_x, d_expert, max(3, args.steps // 10))}))
        return 0

    run_step = step
    if args.graph and len(sets) > 1:
        print("bench.py: --graph replays one captured step and cannot rotate buffers", file=sys.stderr)
        return 2
    if args.graph:
        # the library only enqueues kernels on the given stream (no allocation, no memset, no sync), so a
        # step can be captured as it is; replays are checked against the eager result
        eager_out = d_out.clone()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            step()
            torch.cuda.synchronize()
            with torch.cuda.graph(graph, stream=side):
                step()
        torch.cuda.current_stream().wait_stream(side)
        for _ in range(3):
            d_out.zero_()
            graph.replay()
            torch.cuda.synchronize()
            if not torch.equal(d_out, eager_out):
                print("bench.py: graph replay differs from the eager step", file=sys.stderr)
                return 1
        run_step = graph.replay

    # timed region: exactly K steps, nothing but the library's launches between the two brackets
    K = args.steps
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(K):
        run_step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / K
    tokens_per_s = cfg.N * K / wall

    # per-kernel durations: the same K steps again, every call carrying a pair of HIP events that its own
    # kernels record (start of the first, end of the last; fusco_probe_time_next_call).  Nothing is put into
    # the stream between the kernels, so the steps run as in the region above; a pair of stream events
    # around each call would add about 5 us of barriers to it.
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(K)]
    for row in ev:
        for e in row:
            e.record()          # creates the HIP event
    torch.cuda.synchronize()
    for i in range(K):
        sx, se, sy, so, kw = sets[i % len(sets)]
        fusco.fusco_probe_time_next_call(ev[i][0], ev[i][1])
        fusco.fusco_plan(L, d_A)
        fusco.fusco_probe_time_next_call(ev[i][2], ev[i][3])
        fusco.fusco_dispatch(L, sx, se, **kw)
        fusco.fusco_probe_time_next_call(ev[i][4], ev[i][5])
        fusco.fusco_combine(L, sy, d_w, so)
    torch.cuda.synchronize()
    ms = np.array([[ev[i][2 * j].elapsed_time(ev[i][2 * j + 1]) for j in range(3)] for i in range(K)])   # [K, 3]
    plan_ms, disp_ms, comb_ms = ms.mean(axis=0)

    # the same step with the experts' output in a buffer of its own (an expert computation sits between dispatch
    # and combine in an MoE layer, section 2.1): combine then finds none of its rows in the memory-side cache, and
    # dispatch's freshly written rows are pushed out of it while combine runs
    own_y = None
    if cfg.payload == "bf16" and len(sets) == 1 and not args.graph:
        d_y2 = d_expert.clone()
        K2 = max(20, K // 4)
        nbytes2 = 2 * (cfg.N + cfg.P) * cfg.row_bytes

        def own_buffer_step(dispatch_flags):
            def step2():
                fusco.fusco_plan(L, d_A)
                fusco.fusco_dispatch(L, d_x, d_expert, flags=dispatch_flags)
                fusco.fusco_combine(L, d_y2, d_w, d_out)
            for _ in range(5):
                step2()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(K2):
                step2()
            torch.cuda.synchronize()
            wall2 = time.perf_counter() - t0
            ev2 = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(K2)]
            for row in ev2:
                for e in row:
                    e.record()
            torch.cuda.synchronize()
            for i in range(K2):
                fusco.fusco_plan(L, d_A)
                fusco.fusco_probe_time_next_call(ev2[i][0], ev2[i][1])
                fusco.fusco_dispatch(L, d_x, d_expert, flags=dispatch_flags)
                fusco.fusco_probe_time_next_call(ev2[i][2], ev2[i][3])
                fusco.fusco_combine(L, d_y2, d_w, d_out)
            torch.cuda.synchronize()
            d2 = float(np.mean([ev2[i][0].elapsed_time(ev2[i][1]) for i in range(K2)]))
            c2 = float(np.mean([ev2[i][2].elapsed_time(ev2[i][3]) for i in range(K2)]))
            return {"steps": K2, "ms_per_step": wall2 * 1e3 / K2, "tokens_per_s": cfg.N * K2 / wall2,
                    "dispatch_ms": d2, "combine_ms": c2,
                    "dispatch_plus_combine": {"ms": d2 + c2, "GBps": nbytes2 / ((d2 + c2) * 1e-3) / 1e9,
                                              "frac_of_peak": nbytes2 / ((d2 + c2) * 1e-3) / 1e9 / HBM_PEAK_GBS}}
        own_y = {"plain_dispatch": own_buffer_step(0),
                 "streaming_dispatch": own_buffer_step(fusco.DISPATCH_STREAMING)}
        del d_y2
        step()                       # leave the buffers as the headline step leaves them
        torch.cuda.synchronize()

    # where the source rows are when dispatch starts.  The timed loop above dispatches the same x every step, and
    # dispatch's streaming stores leave x in the 256 MB memory-side cache from one step to the next.  Two more
    # cases, per-call event times as above: a producer kernel rewrites x before every step (what a layer that has
    # just computed x looks like), and x rotates over enough copies that no step finds its rows in the cache.
    source_rows = token_walk = None
    if cfg.payload == "bf16" and len(sets) == 1 and not args.graph and not args.no_variants:
        K3 = max(20, K // 4)
        copies = max(2, -(-(512 << 20) // (cfg.N * cfg.row_bytes)) + 1)
        d_xs = [d_x] + [d_x.clone() for _ in range(copies - 1)]
        d_xsrc = d_x.clone()
        nbytes3 = 2 * (cfg.N + cfg.P) * cfg.row_bytes

        def source_case(before_step, x_of, flags=0):
            ev3 = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(K3)]
            for row in ev3:
                for e in row:
                    e.record()
            for i in range(-35, 5):   # past the slower first milliseconds after the idle time of the allocations above
                before_step()
                fusco.fusco_plan(L, d_A)
                fusco.fusco_dispatch(L, x_of(i), d_expert, flags=flags)
                fusco.fusco_combine(L, d_expert, d_w, d_out)
            torch.cuda.synchronize()
            for i in range(K3):
                before_step()
                fusco.fusco_plan(L, d_A)
                fusco.fusco_probe_time_next_call(ev3[i][0], ev3[i][1])
                fusco.fusco_dispatch(L, x_of(i + 5), d_expert, flags=flags)
                fusco.fusco_probe_time_next_call(ev3[i][2], ev3[i][3])
                fusco.fusco_combine(L, d_expert, d_w, d_out)
            torch.cuda.synchronize()
            d3 = float(np.mean([ev3[i][0].elapsed_time(ev3[i][1]) for i in range(K3)]))
            c3 = float(np.mean([ev3[i][2].elapsed_time(ev3[i][3]) for i in range(K3)]))
            return {"steps": K3, "dispatch_ms": d3, "combine_ms": c3,
                    "dispatch_plus_combine": {"ms": d3 + c3, "GBps": nbytes3 / ((d3 + c3) * 1e-3) / 1e9,
                                              "frac_of_peak": nbytes3 / ((d3 + c3) * 1e-3) / 1e9 / HBM_PEAK_GBS}}
        # the same step with fusco_dispatch kept on the token walk (one workgroup per token), when the library would
        # move the rows tile by tile in transfer order: what the transfer order is worth, in one run
        if fusco.fusco_dispatch_in_transfer_order(L, cfg.row_bytes, 0):
            try:
                fusco.fusco_probe_dispatch_kernel(1)
                fusco.fusco_probe_dispatch_walk(1)      # non-temporal loads, plain stores
                token_walk = {"plain_stores": source_case(lambda: None, lambda i: d_x)}
                fusco.fusco_probe_dispatch_walk(0)      # the library's choice for these sizes (cached loads, streaming stores)
                token_walk["streaming_stores"] = source_case(lambda: None, lambda i: d_x)
            finally:
                fusco.fusco_probe_dispatch_kernel(0)
                fusco.fusco_probe_dispatch_walk(0)
        # a layer's other traffic between two shuffles (weights, attention) leaves nothing of the previous step in the
        # memory-side cache: 1 GiB of another buffer is read before x is rewritten
        d_other = torch.empty((1 << 30) // 16384, 16384, dtype=torch.uint8, device="cuda")
        d_sink = torch.zeros(1, dtype=torch.int32, device="cuda")

        def other_traffic_then_x():
            fusco.fusco_probe_rows(d_other, None, 1, 0, False, sink=d_sink)
            d_x.copy_(d_xsrc)
        source_rows = {
            "same_x_every_step": source_case(lambda: None, lambda i: d_x),
            "x_rewritten_before_every_step": source_case(lambda: d_x.copy_(d_xsrc), lambda i: d_x),
            "1GiB_of_other_reads_then_x_rewritten_before_every_step": source_case(other_traffic_then_x, lambda i: d_x),
            "x_rotating_over_%d_copies" % copies: source_case(lambda: None, lambda i: d_xs[i % copies]),
        }
        del d_xs, d_xsrc, d_other
        step()
        torch.cuda.synchronize()

    variants = None
    if not args.no_variants and cfg.payload == "bf16":
        variants = time_variants(fusco, torch, cfg, L, d_A, d_x, d_w, d_expert, d_out, max(10, K // 4))

    # decode-sized inputs (one planner tile): the same step with plan and dispatch in one launch
    fused = None
    if cfg.N <= 2048 // cfg.k and len(sets) == 1:
        def fused_step():
            fusco.fusco_plan_dispatch(L, d_A, d_x, d_expert, **{k_: v for k_, v in dispatch_kwargs.items()})
            fusco.fusco_combine(L, d_y, d_w, d_out)
        want_layout, want_expert = L.mem.clone(), d_expert.clone()
        d_expert.zero_()
        for _ in range(args.warmup):
            fused_step()
        torch.cuda.synchronize()
        if not (torch.equal(L.mem, want_layout) and torch.equal(d_expert, want_expert)):
            print("bench.py: fused plan + dispatch differs from the two calls", file=sys.stderr)
            return 1
        run_fused, how = fused_step, "fusco_plan_dispatch + fusco_combine"
        if args.graph:
            side2 = torch.cuda.Stream()
            side2.wait_stream(torch.cuda.current_stream())
            fgraph = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side2):
                with torch.cuda.graph(fgraph, stream=side2):
                    fused_step()
            torch.cuda.current_stream().wait_stream(side2)
            d_expert.zero_()
            fgraph.replay()
            torch.cuda.synchronize()
            if not torch.equal(d_expert, want_expert):
                print("bench.py: graph replay of the fused step differs", file=sys.stderr)
                return 1
            run_fused, how = fgraph.replay, how + ", one HIP graph replay per step"
        t0 = time.perf_counter()
        for _ in range(K):
            run_fused()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        fused = {"ms_per_step": dt * 1e3 / K, "tokens_per_s": cfg.N * K / dt, "launches": how}

    ceilings = None
    if not args.no_ceilings and cfg.payload == "bf16":
        ceilings = measure_ceilings(fusco, torch, cfg, d_x, d_expert, d_out, max(10, K // 10))
        # the probes overwrote the shuffle's buffers: run one more step so the checks below see its results
        turn[0] = 0
        step()
        torch.cuda.synchronize()

    if args.probe_copy:
        src = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            fusco.fusco_probe_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst

    # sanity: the identity-expert round trip gives sum_j w_j * x[t] = x[t] up to rounding
    err = 0.0
    if cfg.payload == "bf16":
        for r0 in range(0, cfg.N, 4096):
            err = max(err, (d_out[r0:r0 + 4096].float() - d_x[r0:r0 + 4096].float()).abs().max().item())
    if not err < 0.05:
        print("bench.py: round trip is wrong (max error %g)" % err, file=sys.stderr)
        return 1
    status = int(L.array("status").item())

    bytes_dispatch = (cfg.N + cfg.P) * (cfg.row_bytes + cfg.aux_row_bytes)   # read N rows, write P rows
    bytes_combine = (cfg.P + cfg.N) * cfg.H * 2                 # read P rows, write N rows
    def spread(col):
        p10, med, p90 = np.percentile(ms[:, col], [10, 50, 90])
        return {"p10_ms": float(p10), "median_ms": float(med), "p90_ms": float(p90)}

    kernels = {
        "dispatch": {"ms": float(disp_ms), **spread(1), "algorithmic_bytes": bytes_dispatch,
                     "GBps": bytes_dispatch / (disp_ms * 1e-3) / 1e9},
        "combine": {"ms": float(comb_ms), **spread(2), "algorithmic_bytes": bytes_combine,
                    "GBps": bytes_combine / (comb_ms * 1e-3) / 1e9},
        "plan": {"ms": float(plan_ms), **spread(0)},
    }
    dom = "dispatch" if disp_ms >= comb_ms else "combine"
    achieved = kernels[dom]["GBps"]
    both = (bytes_dispatch + bytes_combine) / ((disp_ms + comb_ms) * 1e-3) / 1e9

    result = {
        "metric": "dispatch+combine tokens/s and achieved HBM GB/s (% of peak), 1 MI355X",
        "value": tokens_per_s,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if cfg.payload == "bf16" else "u8 rows + bf16 combine",
        "data": "synthetic",
        "config": {"workload": "%s: N=%d tokens, hidden=%d %s, E=%d, top-%d, D=%d virtual devices; step = plan + "
                               "dispatch + combine (identity experts)"
                               % (cfg.name, cfg.N, cfg.H, cfg.payload, cfg.E, cfg.k, cfg.D),
                   "N": cfg.N, "hidden": cfg.H, "E": cfg.E, "k": cfg.k, "D": cfg.D, "seed": cfg.seed},
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": measured_traffic(cfg.name).get(dom),
                     "traffic_source": "profiles/bench_dsv3_hbm_traffic_pmc.txt (rocprofv3 --pmc run of this bench)",
                     "timing": "mean over a second pass of the same K steps; each call's kernels record their own "
                               "start and end HIP events (no stream events between kernels)"},
        "kernels": kernels,
        "dispatch_plus_combine": {"ms": float(disp_ms + comb_ms), "tokens_per_s": cfg.N / ((disp_ms + comb_ms) * 1e-3),
                                  "GBps": both, "frac_of_peak": both / HBM_PEAK_GBS},
        "invalid_ids": status,
        "launch": "one HIP graph replay per step" if args.graph else "three library calls per step",
        "buffer_sets": len(sets),
    }
    if own_y is not None:
        result["expert_output_in_own_buffer"] = own_y
    if source_rows is not None:
        result["source_rows"] = source_rows
    if token_walk is not None:
        result["dispatch_kept_on_token_walk"] = token_walk
    if fused is not None:
        result["fused_plan_dispatch_step"] = fused
    if ceilings is not None:
        result["ceilings"] = ceilings
    if variants is not None:
        fused = float(disp_ms + comb_ms)
        variants["fused_dispatch_plus_combine_ms"] = fused
        variants["fused_speedup_over_disaggregated"] = (variants["disaggregated_dispatch_ms"]
                                                        + variants["disaggregated_combine_ms"]) / fused
        result["variants"] = variants
    if not args.no_cpu_baseline:
        n = args.cpu_sample_tokens or cfg.N
        sub = cfg.with_tokens(min(n, cfg.N))
        result["cpu_baseline"] = cpu_baseline(sub, cfg.N, A[:sub.N], w[:sub.N], xb[:sub.N])
        if cfg.payload == "bf16":
            result["cpu_baseline_all_cores"] = cpu_baseline_all_cores(sub, cfg.N, A[:sub.N], w[:sub.N], xb[:sub.N],
                                                                      min(16, os.cpu_count() or 1))
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
