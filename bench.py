#!/usr/bin/env python3
"""Benchmark of the one-sided hot path on one MI355X.

Headline (the workload the metric is quoted on): configuration 2, the put / get
bandwidth sweep over 8 emulated PEs in a ring.  One "step" is one pass over the
HBM-bound part of the sweep: for every message size in SIZES, one put cell and
one get cell (every PE issues OPS back-to-back messages to its ring neighbour
in one launch, rotating over slots so that a launch touches >= 2 GiB).  `value`
is the payload rate of the whole step; a copy moves two bytes of HBM traffic per
payload byte, which is what `roofline` prices against the 8 TB/s peak.

Prints ONE JSON line.  Inputs are resident in HBM before the timed region.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
NPES = 8
SEG = 1 << 30                       # 1 GiB per PE
SIZES = [1 << 20, 1 << 22, 1 << 24, 1 << 26]
BYTES_PER_PE_PER_CELL = 1 << 28     # 256 MiB of payload per PE per launch (2 GiB per launch)


def cells(wgs):
    out = []
    for nbytes in SIZES:
        ops = BYTES_PER_PE_PER_CELL // nbytes
        nslots = ops                 # every op has its own slot: 256 MiB local + 256 MiB remote per PE
        for kind in (0, 1):          # put, get
            out.append(dict(kind=kind, nbytes=nbytes, ops=ops, nslots=nslots, wgs=wgs))
    return out


def cpu_baseline(seconds=12.0):
    """The oracle as it stands, single-threaded, on a bounded sample of the same
    workload: put + quiet and get of SIZES between ring neighbours."""
    import numpy as np
    import oracle
    npes, seg = NPES, 160 << 20
    w = oracle.World(npes, seg, oracle.AT_QUIET, 0)
    for p in range(npes):
        w.heap(p)[: 1 << 20] = np.arange(1 << 20, dtype=np.uint8)
    moved, t0, k = 0, time.perf_counter(), 0
    while time.perf_counter() - t0 < seconds:
        nbytes = SIZES[k % len(SIZES)]
        for p in range(npes):
            peer = (p + 1) % npes
            if (k // len(SIZES)) % 2 == 0:
                w.put(p, 80 << 20, 0, nbytes, peer)
            else:
                w.get(p, 0, 80 << 20, nbytes, peer)
        w.barrier_all()
        moved += nbytes * npes
        k += 1
    dt = time.perf_counter() - t0
    w.close()
    return {"value": moved / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"{k} ring rounds of put+quiet / get over sizes {SIZES} B, 8 PEs, {dt:.1f} s of CPU time"}


def cpu_baseline_extras():
    """The oracle timed (one core) on bounded samples of the other configurations, in each one's unit."""
    import numpy as np
    import oracle
    import workgen
    out = {}
    # config 1: the whole table (it is small)
    ops = workgen.cfg1_op_table()
    w = oracle.World(4, 1 << 20, oracle.AT_QUIET, 0)
    t0 = time.perf_counter(); w.op_batch(ops, 100); dt = time.perf_counter() - t0
    out["config1_optable"] = {"Mops_per_s": round(len(ops) / dt / 1e6, 3), "sample": "all 10,000 ops"}
    w.close()
    # config 3: 2^22 fetch-adds, T = 1024, uniform
    n = 1 << 22
    pe, idx, a = workgen.cfg3_amo_ops(n=n, npes=64, T=1024, dist="uniform", addend="rand16")
    w = oracle.World(64, 1 << 16, oracle.AT_QUIET, 0)
    t0 = time.perf_counter(); w.amo_batch(oracle.AMO_FETCH_ADD, 0, pe, idx, a); dt = time.perf_counter() - t0
    out["config3_amo"] = {"Mops_per_s": round(n / dt / 1e6, 2), "sample": "2^22 fetch-adds, T=1024, uniform"}
    w.close()
    # config 4: 2^21 inserts at load 0.5 and 2^21 lookups
    n, npes = 1 << 21, 16
    slots = 2 * n // npes
    keys = workgen.cfg4_keys(n=n)
    q = workgen.cfg4_queries(keys, n=n)
    w = oracle.World(npes, slots * 8 + 4096, oracle.AT_QUIET, 0)
    tab = w.malloc(slots * 8)
    t0 = time.perf_counter(); w.hash_insert(tab, slots, keys); t1 = time.perf_counter()
    w.hash_lookup(tab, slots, q); t2 = time.perf_counter()
    out["config4_hash"] = {"Minserts_per_s": round(n / (t1 - t0) / 1e6, 2), "Mlookups_per_s": round(n / (t2 - t1) / 1e6, 2),
                           "sample": "2^21 keys into 2^22 slots, 2^21 lookups"}
    w.close()
    # config 5: one search on an R-MAT graph of scale 20
    scale = 20
    row, nbr = workgen.rmat_csr(scale)
    root = int(workgen.bfs_roots(row, 1)[0])
    vpp = (1 << scale) // 16
    w = oracle.World(16, ((vpp * 28 + vpp // 8 + (1 << 16)) + 255) // 256 * 256, oracle.AT_QUIET, 0)
    t0 = time.perf_counter(); _, _, st = w.bfs(row, nbr, root); dt = time.perf_counter() - t0
    out["config5_bfs"] = {"GTEPS": round(st["edges_traversed"] / dt / 1e9, 4), "sample": "one root, R-MAT scale 20, edge factor 16"}
    w.close()
    # MoE-shaped dispatch + combine: one batch of 128 tokens per PE at the paper's sizes
    from oracle import moe as omoe
    P, E, T, K, Hb = 8, 288, 128, 8, 14336
    topk, ntok = workgen.moe_routing(npes=P, num_experts=E, max_tokens=T, topk=K, ntok=T)
    x = workgen.moe_tokens(npes=P, max_tokens=T, hidden_bytes=Hb)
    lay = omoe.MoeLayout(P, E, T, K, Hb)
    w = oracle.World(P, lay.end, oracle.AT_QUIET, 0)
    t0 = time.perf_counter(); d = omoe.dispatch(w, lay, x, topk, ntok); t1 = time.perf_counter()
    omoe.combine(w, lay, d[0], d[1], d[2], topk, ntok); t2 = time.perf_counter()
    out["moe_low_latency"] = {"dispatch_us": round((t1 - t0) * 1e6), "combine_us": round((t2 - t1) * 1e6),
                              "sample": "one dispatch and one combine, 8 PEs x 128 tokens, 288 experts, top-8"}
    w.close()
    return {"cores": 1, "kind": "oracle", "cells": out}


def _median_ms(fn, reset, reps=5, warm=2):
    """Median HIP-event time of fn() on the current stream; reset() runs untimed before each rep."""
    import torch
    stream = torch.cuda.current_stream()
    out = []
    for r in range(warm + reps):
        reset()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        fn()
        b.record(stream)
        b.synchronize()
        if r >= warm:
            out.append(a.elapsed_time(b))
    out.sort()
    return out[len(out) // 2]


def _agg_hw_atomics(torch, d_pe, d_idx, T, n, npes, wgs, pass_ops=1024):
    """Hardware atomics the combining kernel issues for this batch: one per distinct word per pass of 1024 ops
    of a workgroup (a PE's block of ops is cut into consecutive passes) -- counted here from the op arrays."""
    per_pe = (n + npes - 1) // npes
    i = torch.arange(n, device=d_pe.device, dtype=torch.int64)
    within = i - (i // per_pe) * per_pe
    window = (i // per_pe) * ((per_pe + pass_ops - 1) // pass_ops) + within // pass_ops
    key = window * (npes * T) + d_pe.to(torch.int64) * T + d_idx.to(torch.int64)
    return int(torch.unique(key).numel())


def extra_amo(sh, torch, ceilings=None, n=1 << 24, npes=64, wgs=32):
    """Configuration 3: 2^24 AMOs on 64 PEs, T in {1, 1024, 2^20}, uniform / Zipf(1.0).  Every cell is held
    against the atomic ceiling of the same run that matches its footprint: 64 x the one-address rate for
    T = 1, the distinct-line rate over 8 MiB for T = 1024 (512 KiB of counters), over 1 GiB for T = 2^20."""
    import numpy as np
    import workgen
    dev = torch.device("cuda:0")
    seg = 8 << 20
    heap = torch.zeros(npes * seg, dtype=torch.uint8, device=dev)
    scratch = torch.zeros(sh.scratch_bytes(npes), dtype=torch.uint8, device=dev)
    sh.init(npes, seg, heap, scratch, torch.cuda.current_stream().cuda_stream)
    res = {}
    c = ceilings or {}
    ceil_of = {1: ("64 x atomic_same_address_Gops", 64e3 * c["atomic_same_address_Gops"] if "atomic_same_address_Gops" in c else None),
               1024: ("atomic_indep_8MiB_Gops", 1e3 * c["atomic_indep_8MiB_Gops"] if "atomic_indep_8MiB_Gops" in c else None),
               1 << 20: ("atomic_indep_1GiB_Gops", 1e3 * c["atomic_indep_1GiB_Gops"] if "atomic_indep_1GiB_Gops" in c else None)}
    try:
        d_old = torch.empty(n, dtype=torch.int64, device=dev)
        d_zero = torch.zeros(n, dtype=torch.int64, device=dev)
        d_tag = torch.arange(1, n + 1, dtype=torch.int64, device=dev)
        up = lambda a: torch.from_numpy(np.ascontiguousarray(a).view(np.uint8).reshape(-1)).to(dev)
        for T in (1, 1024, 1 << 20):
            ctr = sh.malloc(T * 8)
            off = ctr - heap.data_ptr()
            view = heap.view(npes, seg)[:, off:off + 8 * T]
            for dist in ("uniform", "zipf"):
                pe, idx, a16 = workgen.cfg3_amo_ops(n=n, npes=npes, T=T, dist=dist, addend="rand16")
                d_pe, d_idx, d_a16 = up(pe), up(idx), up(a16)
                d_one = torch.ones(n, dtype=torch.int64, device=dev)
                reset = lambda: view.zero_()
                agg_atomics = _agg_hw_atomics(torch, d_pe.view(torch.int32), d_idx.view(torch.int32), T, n, npes, wgs)
                cell = {}
                for name, kind, a, b, agg in (("fadd1", sh.AMO_FETCH_ADD, d_one, None, 0),
                                              ("fadd1_agg", sh.AMO_FETCH_ADD, d_one, None, 1),
                                              ("faddv", sh.AMO_FETCH_ADD, d_a16, None, 0),
                                              ("faddv_agg", sh.AMO_FETCH_ADD, d_a16, None, 1),
                                              ("cas_claim", sh.AMO_COMPARE_SWAP, d_zero, d_tag, 0),
                                              ("cas_min", sh.AMO_MIN_CAS_LOOP, d_tag, None, 0),
                                              ("cas_min_agg", sh.AMO_MIN_CAS_LOOP, d_tag, None, 1)):
                    ms = _median_ms(lambda: sh.amo_batch(kind, ctr, T, d_pe, d_idx, a, b, d_old, n, wgs, agg),
                                    reset, reps=3, warm=1)
                    mops = n / ms / 1e3
                    entry = {"Mops_per_s": round(mops, 1)}
                    if agg:
                        entry["ops_per_hw_atomic"] = round(n / agg_atomics, 2)
                    elif name != "cas_min":
                        entry["ops_per_hw_atomic"] = 1.0      # cas_min retries: more than one atomic per op, not counted here
                    cname, cval = ceil_of[T]
                    if cval:
                        # a combining kernel is priced by the hardware atomics it still issues
                        hw_rate = mops / entry["ops_per_hw_atomic"] if "ops_per_hw_atomic" in entry else mops
                        entry["roofline"] = {"bound": "atomic", "ceiling": round(cval, 1), "unit": "M hardware atomics/s",
                                             "ceiling_source": f"same run: {cname}", "achieved": round(hw_rate, 1),
                                             "frac": round(hw_rate / cval, 4)}
                    cell[name] = entry
                res[f"T{T}_{dist}"] = cell
                del d_pe, d_idx, d_a16
            sh.free(ctr)
        sh.stream_sync()
    finally:
        sh.finalize()
    return {"unit": "Mops/s", "ops": n, "npes": npes, "wgs_per_pe": wgs,
            "hbm_random_bound_Mops": 62000.0, "note": "T = 2^20 also against the 62 Gop/s HBM random-access bound (128 B of line traffic per op at 8 TB/s)",
            "cells": res}


def extra_config1(sh, torch, wgs=2):
    """Configuration 1: 10,000 random puts/gets (8 B..4 KiB) on 4 PEs, barrier every 100, one launch."""
    import numpy as np
    import workgen
    dev = torch.device("cuda:0")
    npes, seg = 4, 1 << 20
    heap = torch.zeros(npes * seg, dtype=torch.uint8, device=dev)
    heap.view(torch.int64).random_()
    scratch = torch.zeros(sh.scratch_bytes(npes), dtype=torch.uint8, device=dev)
    ops = workgen.cfg1_op_table()
    d_ops = torch.from_numpy(ops.view(np.uint8).reshape(-1)).to(dev)
    sh.init(npes, seg, heap, scratch, torch.cuda.current_stream().cuda_stream)
    try:
        res = {}
        for w in (1, wgs, 8):
            ms = _median_ms(lambda: sh.op_batch(d_ops, len(ops), 100, w), lambda: None, reps=5, warm=2)
            res[f"wgs{w}"] = {"ms": round(ms, 4), "us_per_batch_of_100": round(ms * 10, 3),
                             "Mops_per_s": round(len(ops) / ms / 1e3, 2)}
        sh.stream_sync()
        # the same table through the proxy-style executor (descriptor ring in host memory, host thread)
        px = sh.proxy_create(1 << 12)
        times = []
        for _ in range(4):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            sh.proxy_submit(px, d_ops, len(ops), 4)
            sh.proxy_quiet(px)
            times.append(time.perf_counter() - t0)
        sh.proxy_destroy(px)
        dt = sorted(times[1:])[1]
        res["proxy"] = {"ms": round(dt * 1e3, 3), "us_per_op": round(dt * 1e6 / len(ops), 3),
                        "Mops_per_s": round(len(ops) / dt / 1e6, 3)}
    finally:
        sh.finalize()
    return {"ops": int(len(ops)), "payload_bytes": int(ops["count"].sum()), "npes": npes, "cells": res}


def extra_latency(sh, torch):
    """Put-with-signal ping-pong between two PEs on different dies (the paper's latency experiment,
    Sec. V-A, here inside one GPU) and the in-kernel world barrier."""
    dev = torch.device("cuda:0")
    npes, seg = 16, 16 << 20
    heap = torch.zeros(npes * seg, dtype=torch.uint8, device=dev)
    scratch = torch.zeros(sh.scratch_bytes(npes), dtype=torch.uint8, device=dev)
    sh.init(npes, seg, heap, scratch, torch.cuda.current_stream().cuda_stream)
    try:
        base = heap.data_ptr()
        buf = sh.malloc(9 << 20)                                    # 2 x 4 MiB payload buffers
        gin = sh.gin_create(1, 0)
        sig_off = sh.gin_signal_sym(gin, 0) - base
        hv = heap.view(npes, seg)
        pp = {}
        for nbytes in (8, 128, 4096, 65536, 1 << 20, 4 << 20):
            iters = 2000 if nbytes <= 65536 else 200
            ms = _median_ms(lambda: sh.pingpong(buf, nbytes, gin, 0, iters),
                            lambda: hv[:2, sig_off:sig_off + 8].zero_(), reps=3, warm=1)
            pp[str(nbytes)] = round(ms * 1e3 / iters, 3)            # us per round trip
        slots = sh.malloc(8 * npes)
        bar = {}
        for wgs in (1, 4, 16):
            rounds = 2000
            ms = _median_ms(lambda: sh.barrier_epochs(slots, rounds, wgs, None), lambda: None, reps=3, warm=1)
            bar[f"{npes}x{wgs}_wgs"] = round(ms * 1e3 / rounds, 3)  # us per put-all + barrier_all round
        # barriers over teams of PEs: two teams of 8 (evens and odds) and four of 4, side by side in one launch
        tb = {}
        for name, layout in (("2_teams_of_8", [(0, 2, 8), (1, 2, 8)]), ("4_teams_of_4", [(r, 4, 4) for r in range(4)])):
            teams = [sh.team_create(*t) for t in layout]
            rounds = 2000
            ms = _median_ms(lambda: sh.team_epochs(teams, [rounds] * len(teams), slots, 1, None), lambda: None, reps=3, warm=1)
            tb[name] = round(ms * 1e3 / rounds, 3)                   # us per put-to-members + team barrier round
            sh.stream_sync()
            for t in teams:
                sh.team_destroy(t)
        sh.stream_sync()
    finally:
        sh.finalize()
    return {"pingpong_round_trip_us": pp, "barrier_round_us": bar, "team_barrier_round_us": tb}


def extra_moe(sh, torch, npes=8, num_experts=288, topk=8, hidden=14336, max_tokens=128, wgs=None):
    """MoE-shaped low-latency dispatch / combine (Sec. IV-E, sizes of Sec. V-C): 8 emulated PEs,
    288 experts, top-8 routing, 14,336-byte tokens (14,352-byte dispatch messages), 1-128 tokens
    per PE.  Per launch: microseconds, and payload bytes moved between PEs per second.  `pair_graph_us`:
    one dispatch + combine pair when ten pairs are replayed from one HIP graph (a serving loop's way of paying
    one launch for many), against `dispatch_us + combine_us` launched one by one."""
    import workgen
    dev = torch.device("cuda:0")
    side = torch.cuda.Stream()              # graphs cannot be captured on the default stream
    with torch.cuda.stream(side):
        return _extra_moe_on_current_stream(sh, torch, dev, workgen, npes, num_experts, topk, hidden, max_tokens, wgs)


def _extra_moe_on_current_stream(sh, torch, dev, workgen, npes, num_experts, topk, hidden, max_tokens, wgs):
    epp = num_experts // npes
    seg = (epp * npes * max_tokens * (hidden + 16) + max_tokens * topk * hidden + (1 << 20) + 255) // 256 * 256
    heap = torch.zeros(npes * seg, dtype=torch.uint8, device=dev)
    scratch = torch.zeros(sh.scratch_bytes(npes), dtype=torch.uint8, device=dev)
    sh.init(npes, seg, heap, scratch, torch.cuda.current_stream().cuda_stream)
    res = {}
    try:
        moe = sh.moe_create(num_experts, max_tokens, topk, hidden)
        x = torch.from_numpy(workgen.moe_tokens(npes=npes, max_tokens=max_tokens, hidden_bytes=hidden)).to(dev)
        recv_x = torch.zeros((npes, epp, npes * max_tokens, hidden), dtype=torch.uint8, device=dev)
        recv_info = torch.zeros((npes, epp, npes * max_tokens, 4), dtype=torch.int32, device=dev)
        recv_range = torch.zeros((npes, epp, npes, 2), dtype=torch.int32, device=dev)
        recv_count = torch.zeros((npes, epp), dtype=torch.int32, device=dev)
        combined = torch.zeros((npes, max_tokens, hidden), dtype=torch.uint8, device=dev)
        for ntok in (1, 8, 32, 128):
            topk_np, ntok_np = workgen.moe_routing(npes=npes, num_experts=num_experts, max_tokens=max_tokens, topk=topk,
                                                   ntok=ntok)
            tk, nt = torch.from_numpy(topk_np).to(dev), torch.from_numpy(ntok_np).to(dev)
            routes = int((topk_np >= 0).sum())
            # team size: 36 workgroups per PE (one per local expert) while the batch is latency-bound; 32
            # (one workgroup per CU over the 8 PEs, no CU shared by two) once it is bandwidth-bound
            w = wgs if wgs else (36 if ntok < 32 else 32)
            d_ms = _median_ms(lambda: sh.moe_dispatch(moe, x, tk, nt, recv_x, recv_info, recv_range, recv_count, w),
                              lambda: None, reps=20, warm=3)
            c_ms = _median_ms(lambda: sh.moe_combine(moe, recv_x, recv_info, recv_range, tk, nt, combined, w),
                              lambda: None, reps=20, warm=3)
            sh.stream_sync()
            assert int(recv_count.sum().item()) == routes
            pairs = 10
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=torch.cuda.current_stream()):
                for _ in range(pairs):
                    sh.moe_dispatch(moe, x, tk, nt, recv_x, recv_info, recv_range, recv_count, w)
                    sh.moe_combine(moe, recv_x, recv_info, recv_range, tk, nt, combined, w)
            g_ms = _median_ms(graph.replay, lambda: None, reps=10, warm=2)
            sh.stream_sync()
            assert int(recv_count.sum().item()) == routes
            del graph
            res[str(ntok)] = {"dispatch_us": round(d_ms * 1e3, 2), "combine_us": round(c_ms * 1e3, 2),
                              "pair_graph_us": round(g_ms * 1e3 / pairs, 2),
                              "dispatch_GBs": round(routes * (hidden + 16) / d_ms / 1e6, 1),
                              "combine_GBs": round(routes * hidden / c_ms / 1e6, 1), "routes": routes, "wgs_per_pe": w,
                              # HBM traffic per route: dispatch writes the remote slot and the packed row and reads both
                              # sources (4 x message); combine moves a row there, reads it in the sum (3 x) and writes the
                              # token once per top-k routes
                              "dispatch_hbm_frac": round(routes * 4 * (hidden + 16) / d_ms / 1e6 / HBM_PEAK_GBS, 4),
                              "combine_hbm_frac": round((routes * 3 * hidden + npes * ntok * hidden) / c_ms / 1e6 / HBM_PEAK_GBS, 4)}
        sh.moe_destroy(moe)
    finally:
        sh.finalize()
    return {"npes": npes, "num_experts": num_experts, "topk": topk, "hidden_bytes": hidden, "tokens_per_pe": res}


def extra_transpose(sh, torch, npes=8, n=16384, wgs=256):
    """Distributed transpose by one-sided gets (an iget-shaped variant): 16384 x 16384 uint32 over 8 PEs."""
    dev = torch.device("cuda:0")
    blk = (n // npes) * n * 4
    heap = torch.empty(npes * 2 * blk, dtype=torch.uint8, device=dev)
    heap.view(torch.int64).random_()
    scratch = torch.zeros(sh.scratch_bytes(npes), dtype=torch.uint8, device=dev)
    sh.init(npes, 2 * blk, heap, scratch, torch.cuda.current_stream().cuda_stream)
    try:
        base = heap.data_ptr()
        res = {}
        for w in (64, wgs):
            ms = _median_ms(lambda: sh.transpose(base + blk, base, n, 4, w), lambda: None, reps=9, warm=2)
            res[f"wgs{w}"] = {"ms": round(ms, 4), "traffic_GBs": round(2 * n * n * 4 / ms / 1e6, 1),
                             "hbm_frac": round(2 * n * n * 4 / ms / 1e6 / HBM_PEAK_GBS, 4)}
        sh.stream_sync()
    finally:
        sh.finalize()
    return {"n": n, "elem_bytes": 4, "npes": npes, "matrix_bytes": n * n * 4, "cells": res}


def extra_hash(sh, torch, ceilings=None, n=1 << 26, npes=16, wgs=256):
    """Configuration 4: 2^26 inserts at load factor 0.5, then 2^26 lookups (50 % present)."""
    import numpy as np
    import workgen
    dev = torch.device("cuda:0")
    slots = 2 * n // npes
    seg = slots * 8 + (1 << 20)
    heap = torch.zeros(npes * seg, dtype=torch.uint8, device=dev)
    scratch = torch.zeros(sh.scratch_bytes(npes), dtype=torch.uint8, device=dev)
    sh.init(npes, seg, heap, scratch, torch.cuda.current_stream().cuda_stream)
    try:
        keys = workgen.cfg4_keys(n=n)
        queries = workgen.cfg4_queries(keys, n=n)
        d_keys = torch.from_numpy(keys.view(np.int64)).to(dev)
        d_q = torch.from_numpy(queries.view(np.int64)).to(dev)
        d_st = torch.empty(n, dtype=torch.uint8, device=dev)
        d_fo = torch.empty(n, dtype=torch.uint8, device=dev)
        tab = sh.malloc(slots * 8)
        ins_ms = _median_ms(lambda: sh.hash_insert(tab, slots, d_keys, n, d_st, wgs), lambda: heap.zero_(), reps=3, warm=1)
        look_ms = _median_ms(lambda: sh.hash_lookup(tab, slots, d_q, n, d_fo, wgs), lambda: None, reps=3, warm=1)
        sh.stream_sync()
        found = float(d_fo.float().mean().item())
        inserted = int((d_st == 0).sum().item())
    finally:
        sh.finalize()
    c = ceilings or {}
    # algorithmic bytes: insert = 8 B key + 128 B sector read-modify-write + 1 B status; lookup = 8 + 64 + 1
    ins_gbs, look_gbs = n * 137 / ins_ms / 1e6, n * 73 / look_ms / 1e6
    out = {"keys": n, "npes": npes, "slots_per_pe": slots, "wgs_per_pe": wgs,
           "Minserts_per_s": round(n / ins_ms / 1e3, 1), "Mlookups_per_s": round(n / look_ms / 1e3, 1),
           "inserted": inserted, "found_fraction": round(found, 4),
           "roofline_insert": {"bound": "hbm", "algorithmic_bytes_per_key": 137, "achieved": round(ins_gbs, 1), "peak": HBM_PEAK_GBS,
                               "unit": "GB/s", "frac": round(ins_gbs / HBM_PEAK_GBS, 4),
                               "note": "the memory moves whole 128-byte lines: counters show 1.7x the algorithmic bytes per insert"},
           "roofline_lookup": {"bound": "hbm", "algorithmic_bytes_per_key": 73, "achieved": round(look_gbs, 1), "peak": HBM_PEAK_GBS,
                               "unit": "GB/s", "frac": round(look_gbs / HBM_PEAK_GBS, 4),
                               "note": "64-byte sectors are algorithmic, 128-byte lines are fetched: 2.0x"}}
    if "atomic_indep_1GiB_Gops" in c:
        out["roofline_insert_ops"] = {"bound": "atomic", "ceiling": 1e3 * c["atomic_indep_1GiB_Gops"], "unit": "M ops/s",
                                      "ceiling_source": "same run: atomic_indep_1GiB_Gops (one compare-swap per key)",
                                      "achieved": round(n / ins_ms / 1e3, 1), "frac": round(n / ins_ms / 1e3 / (1e3 * c["atomic_indep_1GiB_Gops"]), 4)}
    if "randread8_1024MiB_Gops" in c:
        out["roofline_lookup_lines"] = {"bound": "hbm random lines", "ceiling": 1e3 * c["randread8_1024MiB_Gops"], "unit": "M lines/s",
                                        "ceiling_source": "same run: randread8_1024MiB_Gops (random 8-byte reads over 1 GiB)",
                                        "achieved": round(n / look_ms / 1e3, 1), "frac": round(n / look_ms / 1e3 / (1e3 * c["randread8_1024MiB_Gops"]), 4)}
    return out


def extra_bfs(sh, torch, ceilings=None, scale=24, npes=16, wgs=64, nroots=64):
    """Configuration 5: level-synchronous BFS on an R-MAT graph, 64 seeded roots."""
    import numpy as np
    import workgen
    dev = torch.device("cuda:0")
    n = 1 << scale
    row, nbr = workgen.rmat_csr(scale)
    roots = workgen.bfs_roots(row, nroots)
    vpp = n // npes
    seg = ((vpp * 28 + vpp // 8 + (1 << 16)) + 255) // 256 * 256
    heap = torch.zeros(npes * seg, dtype=torch.uint8, device=dev)
    scratch = torch.zeros(sh.scratch_bytes(npes), dtype=torch.uint8, device=dev)
    sh.init(npes, seg, heap, scratch, torch.cuda.current_stream().cuda_stream)
    c = ceilings or {}
    # per search the path streams the adjacency of the reached vertices (4 B per CSR entry), their row offsets,
    # and the (parent, level) records, queue entries and bitmaps: about 2.5 GB at scale 24
    stream_bytes = len(nbr) * 4 + n * 8 + n * (8 + 4 + 4)
    try:
        d_row = torch.from_numpy(row.view(np.int64)).to(dev)
        d_nbr = torch.from_numpy(nbr.view(np.int32)).to(dev)
        g = sh.bfs_create(n, d_row, d_nbr, wgs)
        results = {}
        for name, mode in (("top_down", sh.BFS_TOP_DOWN), ("direction_optimizing", sh.BFS_DIRECTION_OPTIMIZING)):
            sh.bfs_configure(g, mode)
            sh.bfs(g, int(roots[0]))                               # warm-up
            teps, times, levels, probes = [], [], [], []
            level_rows = None
            for r in roots:
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                st = sh.bfs(g, int(r))                             # blocks until the search is complete
                dt = time.perf_counter() - t0
                teps.append(st["edges_traversed"] / dt / 1e9)
                times.append(dt * 1e3)
                levels.append(st["nlevels"])
                probes.append(2 * st["edges_traversed"] / dt / 1e9)     # one bitmap probe per CSR entry of a reached vertex (top-down)
                if level_rows is None:
                    level_rows = [{"level": i, "ms": round(us / 1e3, 4), "bottom_up": bu, "frontier": st["frontier_size"][i]}
                                  for i, (us, bu) in enumerate(sh.bfs_level_times(g))]
            teps = np.array(teps)
            hm = float(len(teps) / (1.0 / teps).sum())
            med_ms = float(np.median(times))
            res = {"GTEPS_harmonic_mean": round(hm, 3),
                   "GTEPS_min": round(float(teps.min()), 3), "GTEPS_median": round(float(np.median(teps)), 3),
                   "GTEPS_max": round(float(teps.max()), 3), "ms_median": round(med_ms, 3),
                   "levels_median": int(np.median(levels)), "levels_of_first_root": level_rows,
                   "roofline_stream": {"bound": "hbm", "algorithmic_bytes_per_search": stream_bytes,
                                       "achieved": round(stream_bytes / med_ms / 1e6, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                       "frac": round(stream_bytes / med_ms / 1e6 / HBM_PEAK_GBS, 4),
                                       "GTEPS_at_peak": round(hm / (stream_bytes / med_ms / 1e6 / HBM_PEAK_GBS), 1)}}
            if name != "top_down":
                res["roofline_stream"]["note"] = ("the bytes are those of the top-down method (every reached vertex's whole row); a bottom-up "
                                                  "level stops at a row's first frontier neighbour, so this is an effective rate, not traffic")
            if name == "top_down" and "randread8_2MiB_Gops" in c:
                pr = float(np.median(probes))
                res["roofline_probes"] = {"bound": "L2 random-probe rate", "ceiling": c["randread8_2MiB_Gops"], "unit": "G probes/s",
                                          "ceiling_source": "same run: randread8_2MiB_Gops (random 8-byte reads of an L2-resident 2 MiB)",
                                          "achieved": round(pr, 1), "frac": round(pr / c["randread8_2MiB_Gops"], 4)}
            results[name] = res
        sh.bfs_destroy(g)
        sh.stream_sync()
    finally:
        sh.finalize()
    out = {"scale": scale, "edge_factor": 16, "npes": npes, "wgs_per_pe": wgs, "roots": nroots,
           "csr_entries": int(len(nbr))}
    out.update(results["top_down"])          # the method as configured: put / fetch_or / fetch_add on every level
    out["direction_optimizing"] = results["direction_optimizing"]
    return out


def run_sweep(path):
    """Configuration 2 in full: contiguous put/get 8 B..64 MiB (plus the paper's 14,336 / 14,352-byte
    MoE message sizes) x 1..256 workgroups per PE, and strided uint32 iput/iget.  Writes one JSON
    record per cell to `path` and prints a one-line summary."""
    import torch
    import paper_2511_15076_amd as sh
    dev = torch.device("cuda:0")
    heap = torch.empty(NPES * SEG, dtype=torch.uint8, device=dev)
    heap.view(torch.int64).random_()
    scratch = torch.zeros(sh.scratch_bytes(NPES), dtype=torch.uint8, device=dev)
    sh.init(NPES, SEG, heap, scratch, torch.cuda.current_stream().cuda_stream)
    base = heap.data_ptr()
    local_sym, remote_sym, window = base, base + SEG // 2, SEG // 2
    cells_out = []

    def time_cell(kind, count, eb, rs, ls, rslot, lslot, nslots, ops, wgs):
        fn = lambda: sh.copy_sweep(kind, remote_sym, local_sym, count, eb, rs, ls, rslot, lslot, nslots, ops, wgs)
        return _median_ms(fn, lambda: None, reps=3, warm=1)

    sizes = sorted([1 << k for k in range(3, 27)] + [14336, 14352])
    for nbytes in sizes:
        print(f"sweep: contiguous {nbytes} B", file=sys.stderr, flush=True)      # progress, so that a long run is seen to be alive
        slot = (nbytes + 255) // 256 * 256
        nslots = max(1, min(window // slot, (1 << 28) // slot))
        ops = max(1, min((1 << 28) // nbytes, 1 << 16))
        for wgs in (1, 2, 4, 8, 16, 32, 64, 128, 256):
            for kind, name in ((sh.OP_PUT, "put"), (sh.OP_GET, "get")):
                ms = time_cell(kind, nbytes, 1, 1, 1, slot, slot, nslots, ops, wgs)
                payload = NPES * ops * nbytes
                cells_out.append({"op": name, "bytes": nbytes, "wgs_per_pe": wgs, "ops_per_pe": ops,
                                  "touched_bytes": 2 * NPES * min(ops, nslots) * nbytes, "ms": round(ms, 4),
                                  "payload_GBs": round(payload / ms / 1e6, 2),
                                  "traffic_GBs": round(2 * payload / ms / 1e6, 2),
                                  "hbm_frac": round(2 * payload / ms / 1e6 / HBM_PEAK_GBS, 4),
                                  "us_per_op": round(ms * 1e3 / ops, 4)})
    # strided: uint32 elements, stride on the local side (gather for iput), the remote side (scatter) or both;
    # payloads from 4 KiB in steps of 4x up to the largest whose spans fit the 512 MiB windows, team sizes 1..256.
    # Traffic is counted in the memory's granularity as the counters show it (profiles/): a strided read side costs
    # min(pitch, 128) bytes per element, a strided written side min(pitch, 32), a unit-stride side 4.
    skipped = []
    for payload_bytes in [4096 << (2 * k) for k in range(9)]:         # 4 KiB .. 256 MiB
        nelems = payload_bytes // 4
        for stride in (2, 4, 8, 16, 32, 64):
            print(f"sweep: strided payload {payload_bytes} B stride {stride}", file=sys.stderr, flush=True)
            for mode, ls, rs in (("local", stride, 1), ("remote", 1, stride), ("both", stride, stride)):
                lspan, rspan = ((nelems - 1) * ls + 1) * 4, ((nelems - 1) * rs + 1) * 4
                lslot, rslot = (lspan + 255) // 256 * 256, (rspan + 255) // 256 * 256
                if max(lslot, rslot) > window:
                    skipped.append({"bytes": payload_bytes, "stride_mode": mode, "stride": stride,
                                    "reason": f"span {max(lspan, rspan)} B exceeds the {window} B window"})
                    continue
                nslots = max(1, min(window // max(lslot, rslot), (1 << 26) // payload_bytes))
                ops = max(1, (1 << 26) // payload_bytes)
                for wgs in (1, 2, 4, 8, 16, 32, 64, 128, 256):
                    for kind, name in ((sh.OP_IPUT, "iput"), (sh.OP_IGET, "iget")):
                        fn = lambda: sh.copy_sweep(kind, remote_sym, local_sym, nelems, 4, rs, ls, rslot, lslot, nslots, ops, wgs)
                        ms = _median_ms(fn, lambda: None, reps=2 if wgs < 8 else 3, warm=1)
                        payload = NPES * ops * payload_bytes
                        # bytes the memory moves per element (profiles/k_copy_sweep_strided_cells_counters.md): reads come
                        # in whole 128-byte lines, writes in 32-byte pieces; a unit-stride side costs its 4 bytes
                        rd = lambda st_: min(st_ * 4, 128) if st_ > 1 else 4
                        wr = lambda st_: min(st_ * 4, 32) if st_ > 1 else 4
                        read_stride, write_stride = (ls, rs) if kind == sh.OP_IPUT else (rs, ls)
                        traffic = NPES * ops * nelems * (rd(read_stride) + wr(write_stride))
                        cells_out.append({"op": name, "bytes": payload_bytes, "stride_mode": mode, "stride": stride,
                                          "wgs_per_pe": wgs, "ops_per_pe": ops, "ms": round(ms, 4),
                                          "payload_GBs": round(payload / ms / 1e6, 2),
                                          "traffic_GBs": round(traffic / ms / 1e6, 2),
                                          "hbm_frac": round(traffic / ms / 1e6 / HBM_PEAK_GBS, 4)})
    sh.stream_sync()
    sh.finalize()
    with open(path, "w") as f:
        json.dump({"npes": NPES, "heap_bytes_per_pe": SEG, "cells": cells_out, "skipped": skipped}, f)
    best = max((c for c in cells_out if c["op"] in ("put", "get") and c["bytes"] >= 1 << 20), key=lambda c: c["hbm_frac"])
    print(json.dumps({"sweep_cells": len(cells_out), "skipped_cells": len(skipped), "file": path, "best_contiguous_ge_1MiB": best}), flush=True)


def run_ceilings():
    """The plain-stream, random-access, atomic and mixed read / write ceilings of THIS box (bench_ceilings, a few seconds)."""
    import subprocess
    exe = os.path.join(ROOT, "bench_ceilings")
    try:
        res = subprocess.run([exe], capture_output=True, text=True, timeout=300)
        return json.loads(res.stdout) if res.returncode == 0 else {"error": (res.stdout + res.stderr)[-300:]}
    except Exception as ex:  # noqa: BLE001
        return {"error": f"{type(ex).__name__}: {ex}"}


def measured_traffic(kernel):
    """HBM bytes per launch of the dominant kernel from rocprofv3 counters: a small tracked file that the profiling
    command writes (bench_profile.py), with the commit it was taken at.  None if there is no such file."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_traffic.json")
    try:
        with open(path) as f:
            d = json.load(f)
        return d["traffic_bytes_per_launch"], {"file": os.path.relpath(path, ROOT), "commit": d.get("commit"),
                                              "fetch_bytes": d.get("fetch_bytes_per_launch"), "write_bytes": d.get("write_bytes_per_launch")}
    except (OSError, KeyError, ValueError):
        return None, None


def profile_cells(which):
    """A few launches of one family of kernels and nothing else, for rocprofv3 (--kernel-trace --stats, --pmc):
    strided  six iput cells of configuration 2 (4 MiB payload, 256 workgroups per PE): gather and scatter at stride 2, 16, 64
    hash     configuration 4 once (2^26 inserts, 2^26 lookups)
    bfs      configuration 5, one root, top-down, then the same root direction-optimising
    Every mode also runs one plain 1 GiB tensor copy, the reference dispatch for scaling FETCH_SIZE / WRITE_SIZE."""
    import numpy as np
    import torch
    import paper_2511_15076_amd as sh
    import workgen
    dev = torch.device("cuda:0")
    cal = torch.empty(2 << 30, dtype=torch.uint8, device=dev)
    cal[1 << 30:].copy_(cal[:1 << 30])                      # plain copy: reads 1 GiB, writes 1 GiB
    torch.cuda.synchronize()
    del cal
    torch.cuda.empty_cache()
    if which == "strided":
        heap = torch.empty(NPES * SEG, dtype=torch.uint8, device=dev)
        heap.view(torch.int64).random_()
        scratch = torch.zeros(sh.scratch_bytes(NPES), dtype=torch.uint8, device=dev)
        sh.init(NPES, SEG, heap, scratch, torch.cuda.current_stream().cuda_stream)
        base = heap.data_ptr()
        nelems, ops = (4 << 20) // 4, 16
        for stride in (2, 16, 64):
            for ls, rs in ((stride, 1), (1, stride)):           # iput: local side strided = gather, remote side strided = scatter
                lslot, rslot = (((nelems - 1) * ls + 1) * 4 + 255) // 256 * 256, (((nelems - 1) * rs + 1) * 4 + 255) // 256 * 256
                nslots = max(1, min((SEG // 2) // max(lslot, rslot), ops))
                sh.copy_sweep(sh.OP_IPUT, base + SEG // 2, base, nelems, 4, rs, ls, rslot, lslot, nslots, ops, 256)
                sh.stream_sync()
        sh.finalize()
        print(json.dumps({"profile_cells": "strided", "launch_order": ["gather s2", "scatter s2", "gather s16", "scatter s16", "gather s64", "scatter s64"],
                          "elements_per_launch": NPES * ops * nelems}), flush=True)
    elif which == "hash":
        print(json.dumps({"profile_cells": "hash", "result": extra_hash(sh, torch)}), flush=True)
    elif which == "bfs":
        print(json.dumps({"profile_cells": "bfs", "result": extra_bfs(sh, torch, nroots=1)}), flush=True)
    else:
        raise SystemExit(f"unknown --profile-cells {which}")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--wgs-per-pe", type=int, default=256)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--extras", default="cfg1,latency,moe,transpose,amo,hash,bfs",
                    help="comma list of the other measurements to run too (cfg1, latency, amo, hash, bfs) or 'none'")
    ap.add_argument("--bfs-scale", type=int, default=24)
    ap.add_argument("--sweep", metavar="FILE", default=None,
                    help="run the whole configuration-2 sweep instead of the headline and write its cells to FILE")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip the plain read / write / copy, random-access, atomic and mixed ceilings of the box "
                         "(they are what the extras' fractions are taken against)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 1 GiB tensor copy (a reference dispatch for scaling rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--profile-cells", metavar="FAMILY", default=None,
                    help="run only a few launches of one kernel family (strided, hash, bfs) for rocprofv3")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (PEs are emulated as workgroup teams on one "
              "MI355X); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2511_15076_amd as sh

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.sweep:
        run_sweep(args.sweep)
        return
    if args.profile_cells:
        profile_cells(args.profile_cells)
        return
    dev = torch.device("cuda:0")
    heap = torch.empty(NPES * SEG, dtype=torch.uint8, device=dev)
    heap.view(torch.int64).random_()                    # synthetic payload, resident in HBM
    scratch = torch.zeros(sh.scratch_bytes(NPES), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()
    sh.init(NPES, SEG, heap, scratch, stream.cuda_stream)
    base = heap.data_ptr()
    local_sym, remote_sym = base, base + (SEG // 2)
    plan = cells(args.wgs_per_pe)

    def launch(c):
        sh.copy_sweep(c["kind"], remote_sym, local_sym, c["nbytes"], 1, 1, 1, c["nbytes"], c["nbytes"],
                      c["nslots"], c["ops"], c["wgs"])

    geometry = sh.copy_sweep_geometry(0, remote_sym, local_sym, SIZES[0], SIZES[0], SIZES[0], plan[0]["nslots"], plan[0]["ops"],
                                      args.wgs_per_pe)
    kernel = {384: "k_copy_sweep_stream", 448: "k_copy_sweep_stream_dyn"}.get(geometry[1], "k_copy_sweep")
    for _ in range(args.warmup):
        for c in plan:
            launch(c)
    torch.cuda.synchronize()
    if args.calibration_copy:
        heap[SEG:2 * SEG].copy_(heap[0:SEG])            # plain copy: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()

    # timed region: exactly `steps` steps; per-launch HIP events on the library's stream
    evs = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        for c in plan:
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            launch(c)
            b.record(stream)
            evs.append((c, a, b))
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    sh.stream_sync()

    per_cell = {}
    kernel_ms = 0.0
    for c, a, b in evs:
        ms = a.elapsed_time(b)
        kernel_ms += ms
        per_cell.setdefault((c["kind"], c["nbytes"]), []).append(ms)
    payload_per_launch = NPES * BYTES_PER_PE_PER_CELL
    payload_per_step = payload_per_launch * len(plan)
    ms_per_step = wall * 1e3 / args.steps
    value = payload_per_step / (wall / args.steps) / 1e9
    avg_launch_ms = kernel_ms / len(evs)
    achieved = 2.0 * payload_per_launch / (avg_launch_ms * 1e-3) / 1e9
    detail = {}
    for (kind, nbytes), v in sorted(per_cell.items()):
        v = sorted(v)
        med = v[len(v) // 2]
        detail[f"{'put' if kind == 0 else 'get'}_{nbytes >> 20}MiB"] = {
            "payload_GBs": round(payload_per_launch / (med * 1e-3) / 1e9, 1),
            "hbm_frac": round(2.0 * payload_per_launch / (med * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "hbm_frac_slowest_launch": round(2.0 * payload_per_launch / (v[-1] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    traffic, traffic_source = measured_traffic(kernel)

    out = {
        "metric": "put/get payload bandwidth, messages >= 1 MiB (config 2 sweep, 8 emulated PEs)",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": "configs[1]: 8 emulated PEs in a ring, contiguous put and get, message sizes "
                               "1/4/16/64 MiB, 256 MiB payload per PE per launch",
                   "npes": NPES, "heap_bytes_per_pe": SEG, "wgs_per_pe": args.wgs_per_pe,
                   "launches_per_step": len(plan), "launch_geometry": {"workgroups": geometry[0], "threads": geometry[1]}},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4),
                     # rocprofv3 FETCH_SIZE + WRITE_SIZE per launch, each scaled by what a plain 1 GiB copy reads
                     "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": kernel, "avg_launch_ms": round(avg_launch_ms, 4),
                     "algorithmic_bytes_per_launch": 2 * payload_per_launch,
                     "target": "north_star: >= 0.80 of HBM peak for messages >= 1 MiB"},
        "cells": detail,
    }
    sh.finalize()
    del heap
    torch.cuda.empty_cache()
    ceilings = {} if args.no_ceilings else run_ceilings()
    if ceilings and "error" not in ceilings:
        paced = ceilings.get("copy_streaming_one_stream_GBs_by_pace_ns", {})
        out["roofline"]["box_copy_ceilings_GBs"] = {
            "read_only_best": max(ceilings.get(f"read_grid{g}_GBs", 0) for g in (256, 1024, 2048, 4096)),
            "write_only_best": max(ceilings.get(f"write_grid{g}_GBs", 0) for g in (256, 1024, 2048, 4096)),
            "plain_copy_best": max([ceilings.get(f"copy_u{u}_grid{g}_GBs", 0) for g in (256, 1024, 2048, 4096) for u in (1, 4)]
                                   + list(ceilings.get("copy_pipelined_grid256_GBs_by_extra_delta_bit", {}).values())),
            "wave_specialised_unpaced_best": ceilings.get("copy_wave_specialised_unpaced_GBs", {}).get("best"),
            "streaming_copy_one_stream_by_pace_ns": paced,
            "source": "same run (bench_ceilings)"}
        best_paced = max([v["median"] for v in paced.values()] or [0])
        if best_paced:
            out["roofline"]["frac_of_box_best_copy"] = round(achieved / best_paced, 4)
    want = [] if args.extras == "none" else args.extras.split(",")
    extras = {}

    def run_extra(key, name, fn, **kw):
        # an extra that fails is reported as such; it never costs the headline line
        if key not in want:
            return
        try:
            extras[name] = fn(sh, torch, **kw)
        except Exception as ex:  # noqa: BLE001
            extras[name] = {"error": f"{type(ex).__name__}: {ex}"}
            try:
                sh.finalize()
            except Exception:  # noqa: BLE001
                pass
        torch.cuda.empty_cache()

    ceil_ok = ceilings if ceilings and "error" not in ceilings else None
    run_extra("cfg1", "config1_optable", extra_config1)
    run_extra("latency", "latency", extra_latency)
    run_extra("moe", "moe_low_latency", extra_moe)
    run_extra("transpose", "transpose_by_gets", extra_transpose)
    run_extra("amo", "config3_amo", extra_amo, ceilings=ceil_ok)
    run_extra("hash", "config4_hash", extra_hash, ceilings=ceil_ok)
    run_extra("bfs", "config5_bfs", extra_bfs, ceilings=ceil_ok, scale=args.bfs_scale)
    if extras:
        out["extras"] = extras
    if ceilings:
        out["stream_ceilings"] = ceilings
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline()
        if extras:
            try:
                out["cpu_baseline_extras"] = cpu_baseline_extras()
            except Exception as ex:  # noqa: BLE001
                out["cpu_baseline_extras"] = {"error": f"{type(ex).__name__}: {ex}"}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
