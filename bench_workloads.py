#!/usr/bin/env python3
"""Timings of the configurations that are not the headline benchmark (bench.py covers that one):

    python bench_workloads.py multihot   # 26 fp16 tables, batch 65,536, hotness 1..100, mean: fwd / dedup / apply
    python bench_workloads.py hashed     # open 2^63 key space, capacity 1e8, dim 64: insert-or-find, fwd, bwd over load factor
    python bench_workloads.py cache      # inference cache, Zipf 1.2, batch 1 / 64 / 1024 / 16384: hit rate, keys/s, p50 latency
    python bench_workloads.py mixed      # headline shape in mixed precision: fp16 table + fp32 master rows, fp16 out / dY
    python bench_workloads.py etc        # training cache staged in host memory: load / train / dump passes of 8 batches
    python bench_workloads.py fwd_probe  # the forward kernel on key patterns of known locality (what bounds it)
    python bench_workloads.py placement  # how much the physical placement of the buffers moves the timings
    python bench_workloads.py speedmap   # fill / copy / random-row gather by the position at which a process is handed its memory
    python bench_workloads.py which_buffer  # the headline step with one buffer replaced at a time (the table's place decides)
    python bench_workloads.py group      # fused group: the 26 DLRM-sized tables with widths 128/64/32/16, dense one-hot input

Each prints one JSON line.  Inputs are synthetic and seeded (datagen/), resident in HBM (the cache's
backing table in pinned host memory) before anything is timed.  The inference-cache configuration
asks for a 5e8-row host table (256 GB); the cache benchmark takes the largest table the machine pins
(1e8 rows = 51 GB on the GPU machine; --host-rows overrides), the cache always holds 10 % of the rows in
32-way sets.  multihot, hashed and cache also carry a roofline object for their dominant kernel, the
oracle timed on the host cores (cpu_baseline) and an oracle check on their timed inputs.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import datagen  # noqa: E402

SEED = datagen.DEFAULT_SEED
DEV = "cuda"
SPACER_GIB = 96.0   # tables are allocated behind this much device memory (see behind_spacer); --spacer-gib 0: the plain way


def timeit(fn, iters=10, warm=2):
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


HBM_PEAK_GBS = 8000.0


def roofline(kernel, algorithmic_bytes, ms, note, bound="hbm", traffic=None):
    """The dominant kernel against the HBM peak: algorithmic bytes of one launch over its duration;
    `traffic` is the profiler's HBM byte count for the launch where profiles/ holds one."""
    gbs = algorithmic_bytes / (ms * 1e-3) / 1e9
    return {"bound": bound, "kernel": kernel, "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": gbs / HBM_PEAK_GBS, "traffic": traffic,
            "measured_frac": None if traffic is None else traffic / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "algorithmic_bytes_per_launch": int(algorithmic_bytes), "avg_launch_ms": ms, "note": note}


def stored_traffic(name):
    """HBM bytes per launch of a kernel from the rocprofv3 --pmc summaries under profiles/ (None if absent)."""
    path = os.path.join(ROOT, "profiles", "other_workloads_hbm_traffic.json")
    try:
        return json.load(open(path))["kernels"][name]["traffic_bytes_per_launch"]
    except Exception:
        return None


def host_copy(table):
    host = np.empty(tuple(table.shape), dtype={torch.float32: np.float32, torch.float16: np.float16}[table.dtype])
    slab = 1 << 22
    for r0 in range(0, table.shape[0], slab):
        r1 = min(table.shape[0], r0 + slab)
        torch.from_numpy(host[r0:r1]).copy_(table[r0:r1])
    return host


def multihot(h, args):
    rows_t = datagen.DLRM_TABLE_ROWS
    S, D, B = 26, 128, 65536
    ro = datagen.row_offsets(rows_t)
    base, total = ro[:-1].copy(), int(ro[-1])
    table = h.allocate_table(total, D, torch.float16, DEV, spacer_gib=SPACER_GIB)
    datagen.fill_table(SEED, table, 1 << 21)
    smp = datagen.make_samplers(rows_t, 1.1, device=DEV)
    offsets = datagen.multihot_offsets(SEED, 7, B * S, 1, 100, device=DEV)
    keys = datagen.multihot_keys(SEED, 7, rows_t, B, 1.1, offsets, device=DEV, samplers=smp)
    del smp
    nnz = keys.numel()
    dY = datagen.normal_grads(SEED, 7, B * S * D, device=DEV).view(B, S, D)
    layer = h.EmbeddingLayer(table, S, h.MEAN, base, rows_t)
    ws = layer.new_workspace(layer.workspace_bytes(B, nnz))
    out = torch.empty((B, S, D), device=DEV)
    f = timeit(lambda: layer.forward(B, keys, offsets, out=out, ws=ws), 10, 3)
    # CPU side first, while the table still holds what the forward read: the oracle's all-cores variant on
    # a dense host copy of the table, over the first quarter of the samples (whole bags), forward +
    # backward; its pooled rows are compared with the timed forward's (parity on timed inputs)
    import oracle
    threads = oracle.hardware_threads()
    host = host_copy(table)
    Bs = B // 4
    nb = Bs * S
    off_h = offsets[:nb + 1].cpu().numpy()
    keys_h = keys[:int(off_h[-1])].cpu().numpy()
    dY_h = dY.view(B * S, D)[:nb].cpu().numpy()
    t0 = time.perf_counter()
    rows_h, bad = oracle.rows_direct(base, rows_t, keys_h, off_h, threads=threads)
    ref = oracle.emb_forward(host, rows_h, off_h, oracle.MEAN, threads=threads)
    t1 = time.perf_counter()
    got = out.view(B * S, D)[:nb].cpu().numpy()
    mag = oracle.emb_forward(np.abs(host), rows_h, off_h, oracle.MEAN, threads=threads)
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    tol = 1e-5 * np.maximum(np.abs(ref.astype(np.float64)), mag.astype(np.float64) / 8)
    assert bad == 0 and (err <= tol).all(), f"multi-hot forward differs from the oracle: max err {err.max():.3e}"
    t2 = time.perf_counter()
    oracle.emb_backward_sgd(host, rows_h, dY_h, 0.01, off_h, oracle.MEAN, threads=threads)
    t3 = time.perf_counter()
    cpu_s = (t1 - t0) + (t3 - t2)
    del host, mag, ref
    d = timeit(lambda: layer.backward_dedup(B, keys, offsets, ws=ws), 10, 3)
    a = timeit(lambda: layer.backward_apply(B, nnz, dY, 0.01, offsets, ws=ws), 10, 3)
    uniq, cnt = layer.dedup_result(B, nnz, ws=ws)
    assert int(cnt.sum()) == nnz and layer.invalid_keys(ws) == 0
    U = int(uniq.numel())
    # the same batch with fp16 pooled output and fp16 upstream gradient (sums still formed in fp32)
    half = h.EmbeddingLayer(table, S, h.MEAN, base, rows_t, io_dtype=torch.float16)
    out16 = torch.empty((B, S, D), dtype=torch.float16, device=DEV)
    dY16 = dY.to(torch.float16)
    f16 = timeit(lambda: half.forward(B, keys, offsets, out=out16, ws=ws), 10, 3)
    half.backward_dedup(B, keys, offsets, ws=ws)
    a16 = timeit(lambda: half.backward_apply(B, nnz, dY16, 0.01, offsets, ws=ws), 10, 3)
    del out16, dY16
    fwd_bytes = nnz * (8 + D * 2) + B * S * (D * 4 + 8)
    apply_bytes = nnz * (8 + D * 4) + U * 2 * D * 2
    compulsory = nnz * 8 + B * S * D * 4 + U * 2 * D * 2      # sorted pairs once, dY once, rows read + written
    tr = stored_traffic("bwd_reduce_windows_multihot")
    return dict(workload="multi-hot: 26 fp16 tables, dim 128, batch 65536, hotness 1..100, Zipf 1.1, mean", keys=nnz,
                distinct_rows=U, forward_ms=f, forward_algorithmic_GBs=fwd_bytes / f / 1e6,
                backward_dedup_ms=d, backward_apply_ms=a, backward_apply_logical_GBs=apply_bytes / a / 1e6,
                fwd_bwd_keys_per_s=nnz / ((f + d + a) * 1e-3),
                metric="embedding keys/s fwd+bwd", value=nnz / ((f + d + a) * 1e-3), unit="keys/s",
                logical_GBs=(fwd_bytes + apply_bytes) / ((f + d + a) * 1e-3) / 1e9,
                compulsory_GBs=(nnz * 8 + U * D * 2 + B * S * (D * 4 + 8) + compulsory) / ((f + d + a) * 1e-3) / 1e9,
                fp16_io=dict(forward_ms=f16, backward_apply_ms=a16, fwd_bwd_keys_per_s=nnz / ((f16 + d + a16) * 1e-3)),
                parity_checked=True, parity=dict(forward_bags_checked=nb, max_abs_err=float(err.max()),
                                                 dedup="occurrence counts add up to the key count"),
                roofline=roofline("bwd_reduce_windows<__half,16,UniformView<__half,float>,false> (+ bwd_carry)",
                                  apply_bytes, a, "algorithmic = a 512-B gradient row and a 16-B sorted pair per "
                                  "occurrence + 512 B per distinct row; compulsory (dY once) is %.2f GB" % (compulsory / 1e9),
                                  traffic=tr),
                cpu_baseline=dict(value=len(keys_h) / cpu_s, unit="keys/s", cores=threads, kind="oracle",
                                  sample=f"the first {Bs} samples of the batch ({len(keys_h)} keys), key -> row + forward + "
                                         "backward/SGD once, dense host copy of the fp16 table, all-cores variant"))


def hashed(h, args):
    S, D, B = 26, 64, 131072
    cap, max_rows = 100_000_000, 80_000_000
    with h.behind_spacer(SPACER_GIB, cap * 16 + max_rows * D * 4):
        ht = h.HashTable(cap, max_rows)
        table = torch.empty((max_rows, D), dtype=torch.float32, device=DEV)
    datagen.fill_table(SEED, table, 1 << 22)
    layer = h.EmbeddingLayer(table, S, h.SUM, hash_table=ht, insert_on_miss=True, reuse_forward_rows=True)
    nnz = B * S
    ws = layer.new_workspace(layer.workspace_bytes(B, nnz))
    out = torch.empty((B, S, D), device=DEV)
    smp = datagen.ZipfSampler(1 << 63, 1.05, device=DEV)
    dY = datagen.normal_grads(SEED, 1, nnz * D, device=DEV).view(B, S, D)
    per_batch = []
    keys = None
    for it in range(args.hash_batches):
        keys = datagen.open_space_keys(SEED, it, S, B, 1.05, device=DEV, sampler=smp)
        torch.cuda.synchronize()
        e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        e[0].record()
        layer.forward(B, keys, out=out, ws=ws)          # insert-or-find + gather
        e[1].record()
        layer.backward_sgd(B, keys, dY, 0.01, ws=ws)    # (rows of the forward) dedup + reduce + SGD
        e[2].record()
        torch.cuda.synchronize()
        per_batch.append((ht.size / cap, e[0].elapsed_time(e[1]), e[1].elapsed_time(e[2])))
    # windows of the load factor reached after the batch; the last window is the saturated regime:
    # the table is at max_rows, new keys are rejected (find + refused inserts)
    trace = []
    edges = [0.0, 0.2, 0.4, 0.6, 0.8 - 1e-9, 1.0]
    names = ["0-0.2", "0.2-0.4", "0.4-0.6", "0.6-0.8", "saturated (0.8)"]
    for lo, hi, name in zip(edges[:-1], edges[1:], names):
        sel = [(f, b) for lf, f, b in per_batch if lo < lf <= hi]
        if sel:
            f, b = float(np.median([x[0] for x in sel])), float(np.median([x[1] for x in sel]))
            trace.append(dict(load_factor=name, batches=len(sel), forward_ms=f, backward_ms=b,
                              keys_per_s=nnz / ((f + b) * 1e-3)))
    rows = torch.empty(nnz, dtype=torch.int64, device=DEV)
    find_ms = timeit(lambda: ht.insert_or_find(keys, False, rows=rows), 10, 2)
    # parity on timed inputs: the rows of the last timed batch in the saturated table, against what the
    # forward of that batch pooled (one key per bag: the pooled row is the table row; a refused key pools
    # zeros), and the table's size
    torch.cuda.synchronize()
    layer.forward(B, keys, out=out, ws=ws)
    torch.cuda.synchronize()
    want = table[rows.clamp(min=0)] * (rows >= 0)[:, None]
    assert torch.equal(out.view(nnz, D), want) and ht.size <= max_rows
    # CPU side: the oracle on the first batches of the same key stream, from an empty table: key -> row by
    # its sequential hash (one thread: first-appearance order is a sequential definition), then forward
    # and backward on all cores over a dense host table of the rows handed out so far
    import oracle
    threads = oracle.hardware_threads()
    ref = oracle.Hash(max_rows)
    n_cpu = 3
    host = np.zeros((n_cpu * nnz, D), dtype=np.float32)
    host[:] = 0.03125
    cpu_s = 0.0
    for it in range(n_cpu):
        k = datagen.open_space_keys(SEED, it, S, B, 1.05, device=DEV, sampler=smp).cpu().numpy()
        g = dY.view(nnz, D).cpu().numpy()
        t0 = time.perf_counter()
        r = ref.insert_or_find(k, True)
        oracle.emb_forward(host, r, threads=threads)
        oracle.emb_backward_sgd(host, r, g, 0.01, threads=threads)
        cpu_s += time.perf_counter() - t0
    mid = [t for t in trace if t["load_factor"] == "0.4-0.6"] or trace
    return dict(workload="hashed open key space: capacity 1e8, max 8e7 rows, dim 64 fp32, 26 one-hot slots, "
                         "batch 131072, Zipf 1.05 over 2^63 ids, insert on miss", keys=nnz, find_only_ms=find_ms,
                find_only_keys_per_s=nnz / find_ms * 1e3, trace=trace,
                metric="embedding keys/s fwd+bwd at load factor 0.4-0.6", value=mid[0]["keys_per_s"], unit="keys/s",
                parity_checked=True, parity=dict(rows_and_pooled_rows_of_last_batch="exact", size=ht.size),
                roofline=roofline("hash_find (find-only call on the saturated table)", nnz * (8 + 128 + 8), find_ms,
                                  "algorithmic = key 8 B + one 128-B bucket + row 8 B per key; random 128-B lines, "
                                  "latency-bound", traffic=stored_traffic("hash_find")),
                cpu_baseline=dict(value=n_cpu * nnz / cpu_s, unit="keys/s", cores=threads, kind="oracle",
                                  sample=f"the first {n_cpu} batches of the key stream from an empty table: insert-or-find by "
                                         "the oracle's sequential hash (one thread), forward + backward/SGD on all cores"))


def pinned_host_table(candidates, D):
    """The largest candidate row count this machine pins in one allocation, filled with the closed form."""
    for host_rows in candidates:
        try:
            host = torch.empty((host_rows, D), dtype=torch.float32, pin_memory=True)
        except RuntimeError:
            continue
        for r0 in range(0, host_rows, 1 << 21):
            r1 = min(host_rows, r0 + (1 << 21))
            host[r0:r1].copy_(datagen.table_rows_at(SEED, torch.arange(r0, r1, device=DEV), D, torch.float32))
        torch.cuda.synchronize()
        return host
    raise RuntimeError("no candidate size of the host table could be pinned")


def cache(h, args):
    import oracle
    import psutil
    D, S, hot, ways = 128, 26, 4, 32
    # the configuration names 5e8 rows (256 GB); the largest table this machine pins is used
    sizes = [args.host_rows] if args.host_rows else [100_000_000, 50_000_000, 20_000_000]
    host = pinned_host_table(sizes, D)
    host_rows = host.shape[0]
    num_sets = host_rows // 10 // ways
    c = h.EmbeddingCache(num_sets, ways, host)
    smp = datagen.ZipfSampler(host_rows, 1.2, DEV)
    big = 16384 * S * hot
    # the first calls go to the oracle's simulation too: parity on the inputs, and its time is the CPU baseline
    ref = oracle.Cache(num_sets, ways, host.numpy())
    n_ref, cpu_s, cpu_keys = 4, 0.0, 0
    call = 0
    for _ in range(30):   # warm up until the hit rate is stationary
        keys = datagen.cache_keys(SEED, call, host_rows, big, 1.2, device=DEV, sampler=smp)
        hm = torch.zeros(big, dtype=torch.uint8, device=DEV)
        o = c.query(16384, S, keys, hit_mask=hm)
        if call < n_ref:
            k = keys.cpu().numpy()
            t0 = time.perf_counter()
            ref_out, ref_hit = ref.query(k, 16384 * S, insert_missing=True)
            cpu_s += time.perf_counter() - t0
            cpu_keys += big
            torch.cuda.synchronize()
            assert np.array_equal(hm.cpu().numpy(), ref_hit) and c.stats == ref.stats.tolist(), "cache differs from the oracle"
            err = np.abs(o.cpu().numpy().reshape(-1, D).astype(np.float64) - ref_out)
            assert err.max() <= 1e-5 * 4 / 16 / 8 + 1e-12, f"pooled rows differ from the oracle: {err.max():.3e}"   # 4 terms of at most 1/16
        call += 1
    torch.cuda.synchronize()
    sweep = []
    side = torch.cuda.Stream()
    for batch in (1, 64, 1024, 16384):
        n = batch * S * hot
        reps = min(args.cache_reps, 1000 if batch < 16384 else 300)
        ks_by_mode = {m: [datagen.cache_keys(SEED, 1000 + 2000 * j + call + i, host_rows, n, 1.2, device=DEV, sampler=smp)
                          for i in range(reps)] for j, m in enumerate(("insert", "lookup_only", "two_phase", "replay_insert", "replay_lookup_only"))}
        o = torch.empty((batch, S, D), device=DEV)
        ws = c.workspace(n)
        hm = torch.zeros(n, dtype=torch.uint8, device=DEV)
        res = {}
        for mode, insert in (("insert", True), ("lookup_only", False)):
            s0 = c.stats
            lat, gpu = [], []
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            for k in ks_by_mode[mode]:   # fresh keys for each mode, so lookup-only sees real misses too
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                e0.record()
                c.query(batch, S, k, None, insert, out=o, hit_mask=hm, ws=ws)
                e1.record()
                torch.cuda.synchronize()
                lat.append((time.perf_counter() - t0) * 1e6)
                gpu.append(e0.elapsed_time(e1) * 1e3)
            s1 = c.stats
            res[mode] = dict(hit_rate=(s1[1] - s0[1]) / (s1[0] - s0[0]), p50_us=float(np.median(lat)),
                             p99_us=float(np.percentile(lat, 99)), gpu_p50_us=float(np.median(gpu)),
                             keys_per_s=n / np.median(lat) * 1e6)
        # two phases: when the hit-only rows are ready (event), and when the whole query is (side stream)
        ready = torch.cuda.Event()
        ready.record()
        t_hits, t_all = [], []
        for k in ks_by_mode["two_phase"]:
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            c.query_hits(batch, S, k, o, hit_mask=hm, ws=ws, ready=ready)
            side.wait_event(ready)
            c.query_complete(batch, S, k, o, insert_missing=True, ws=ws, stream=side)
            ready.synchronize()
            t_hits.append((time.perf_counter() - t0) * 1e6)
            side.synchronize()
            t_all.append((time.perf_counter() - t0) * 1e6)
        res["two_phase"] = dict(hits_ready_p50_us=float(np.median(t_hits)), complete_p50_us=float(np.median(t_all)))
        # the same query captured once in a HIP graph and replayed (small batches: launches dominate)
        if batch <= 1024:
            kbuf = torch.zeros(n, dtype=torch.int64, device=DEV)
            for mode, insert in (("replay_insert", True), ("replay_lookup_only", False)):
                g = torch.cuda.CUDAGraph()
                side.wait_stream(torch.cuda.current_stream())
                with torch.cuda.stream(side):
                    with torch.cuda.graph(g, stream=side):
                        c.query(batch, S, kbuf, None, insert, out=o, hit_mask=hm, ws=ws, stream=side)
                torch.cuda.current_stream().wait_stream(side)
                lat = []
                for k in ks_by_mode[mode]:
                    kbuf.copy_(k)
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                    g.replay()
                    torch.cuda.synchronize()
                    lat.append((time.perf_counter() - t0) * 1e6)
                res[mode] = dict(p50_us=float(np.median(lat)), p99_us=float(np.percentile(lat, 99)))
                del g
        sweep.append(dict(batch=batch, keys=n, queries=reps,
                          **{f"{m}_{k}": v for m, r in res.items() for k, v in r.items()}))
    # CPU baseline on small batches too (the oracle's own, partly warm cache)
    small_cpu = {}
    for batch in (1, 64, 1024):
        n = batch * S * hot
        ks = [datagen.cache_keys(SEED, 9000 + i, host_rows, n, 1.2, sampler=smp, device=DEV).cpu().numpy() for i in range(20)]
        t0 = time.perf_counter()
        for k in ks:
            ref.query(k, batch * S, insert_missing=True)
        small_cpu[str(batch)] = n * len(ks) / (time.perf_counter() - t0)
    last = sweep[-1]
    look_ms = last["lookup_only_gpu_p50_us"] * 1e-3
    n = last["keys"]
    alg = n * (8 + ways * 8 + 4 + 9 + D * 4 + 4) + 16384 * S * D * 4
    return dict(workload=f"inference cache: {host_rows} x 128 fp32 host table ({host_rows * D * 4 / 1e9:.1f} GB pinned; the "
                         f"configuration names 5e8 rows = 256 GB, this machine has {psutil.virtual_memory().total / 2**30:.0f} GiB of "
                         "RAM and pins at most 64 GiB in one allocation), cache 10% in 32-way sets, 26 slots x hotness 4, "
                         "Zipf 1.2; latency = host call + stream sync, gpu = event pair around the call", sweep=sweep,
                host_rows=host_rows, cache_lines=num_sets * ways,
                metric="cache query keys/s at batch 16384, lookup only", value=last["lookup_only_keys_per_s"], unit="keys/s",
                parity_checked=True, parity=dict(calls_compared_with_the_oracle=n_ref, what="hit mask, statistics, pooled rows"),
                roofline=roofline("cache_probe<32> + cache_gather<32,4> (lookup-only call of 16,384 samples)", alg, look_ms,
                                  "algorithmic = per key 8 (key) + 256 (tags of the set) + 4 + 9 (line, mask, flag) + 4 + 512 (row); "
                                  "per bag 512 written; missing rows cross the host link", traffic=stored_traffic("cache_lookup_16384")),
                cpu_baseline=dict(value=cpu_keys / cpu_s, unit="keys/s", cores=1, kind="oracle",
                                  sample=f"the first {n_ref} calls of 16,384 samples ({big} keys each) from a cold cache, query + insertion; "
                                         "the simulation is sequential by definition (one thread)",
                                  small_batches_keys_per_s=small_cpu))


def mixed(h, args):
    rows_t = datagen.DLRM_TABLE_ROWS
    S, D, B = 26, 128, 55296
    ro = datagen.row_offsets(rows_t)
    base, total = ro[:-1].copy(), int(ro[-1])
    with h.behind_spacer(SPACER_GIB, total * D * 6):
        master = torch.empty((total, D), dtype=torch.float32, device=DEV)
        table = torch.empty((total, D), dtype=torch.float16, device=DEV)
    datagen.fill_table(SEED, master, 1 << 21)
    for r0 in range(0, total, 1 << 22):
        table[r0:r0 + (1 << 22)].copy_(master[r0:r0 + (1 << 22)])
    smp = datagen.make_samplers(rows_t, 1.05, device=DEV)
    keys = [datagen.onehot_keys(SEED, b, rows_t, B, 1.05, device=DEV, samplers=smp) for b in range(4)]
    del smp
    nnz = B * S
    dY = datagen.normal_grads(SEED, 5, nnz * D, device=DEV).view(B, S, D).to(torch.float16)
    out = torch.empty((B, S, D), dtype=torch.float16, device=DEV)
    res = {}
    for name, m in (("fp16_table", None), ("fp16_table_fp32_master", master)):
        layer = h.EmbeddingLayer(table, S, h.SUM, base, rows_t, io_dtype=torch.float16, master=m)
        ws = layer.new_workspace(layer.workspace_bytes(B, nnz))
        it = [0]

        def fwd():
            layer.forward(B, keys[it[0] % 4], out=out, ws=ws)
            it[0] += 1

        def bwd():
            layer.backward_sgd(B, keys[it[0] % 4], dY, 0.01, ws=ws)
            it[0] += 1

        f, b = timeit(fwd, 20, 4), timeit(bwd, 20, 4)
        res[name] = dict(forward_ms=f, forward_algorithmic_GBs=nnz * (8 + 2 * D + 2 * D) / f / 1e6, backward_ms=b,
                         fwd_bwd_keys_per_s=nnz / ((f + b) * 1e-3))
    return dict(workload="headline shape in mixed precision: 26 fp16 tables (165,158,233 x 128), fp16 out and dY, "
                         "batch 55296, one-hot, Zipf 1.05, sum", keys=nnz, **res)


def etc(h, args):
    host_rows, D, S, B, per_pass = args.host_rows or 20_000_000, 128, 26, 55296, 8
    host = torch.empty((host_rows, D), dtype=torch.float32, pin_memory=True)
    for r0 in range(0, host_rows, 1 << 20):
        r1 = min(host_rows, r0 + (1 << 20))
        host[r0:r1].copy_(datagen.table_rows_at(SEED, torch.arange(r0, r1, device=DEV), D, torch.float32))
    nnz = B * S
    max_rows = 6_000_000
    cache = h.EmbeddingTrainingCache(host, max_rows, capacity=8_000_000)
    layer = cache.layer(S, h.SUM, reuse_forward_rows=True)
    smp = datagen.ZipfSampler(host_rows, 1.05)
    dY = datagen.normal_grads(SEED, 9, nnz * D, device=DEV).view(B, S, D)
    out = torch.empty((B, S, D), device=DEV)
    ws = layer.new_workspace(layer.workspace_bytes(B, nnz))
    passes = []
    for p in range(args.etc_passes):
        batches = [datagen.cache_keys(SEED, 100 * p + i, host_rows, nnz, 1.05, sampler=smp).cuda() for i in range(per_pass)]
        pass_keys = torch.cat(batches)
        cache.workspace(pass_keys.numel())
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        ev[0].record()
        cache.load(pass_keys)
        ev[1].record()
        for k in batches:
            layer.forward(B, k, out=out, ws=ws)
            layer.backward_sgd(B, k, dY, 0.01, ws=ws)
        ev[2].record()
        cache.dump(evict=True)
        ev[3].record()
        torch.cuda.synchronize()
        st = cache.stats
        rows = st[1] - sum(x["rows"] for x in passes)
        load_ms, train_ms, dump_ms = ev[0].elapsed_time(ev[1]), ev[1].elapsed_time(ev[2]), ev[2].elapsed_time(ev[3])
        passes.append(dict(rows=rows, load_ms=load_ms, load_host_link_GBs=rows * D * 4 / load_ms / 1e6,
                           train_ms_per_batch=train_ms / per_pass, dump_ms=dump_ms,
                           dump_host_link_GBs=rows * D * 4 / dump_ms / 1e6,
                           keys_per_s=per_pass * nnz / ((load_ms + train_ms + dump_ms) * 1e-3)))
    assert cache.stats[2] == 0 and layer.invalid_keys(ws) == 0
    return dict(workload=f"training cache staged in host memory: {host_rows} x 128 fp32 host table (pinned), working "
                         f"table {max_rows} rows, passes of {per_pass} batches of 55296 x 26 one-hot keys, Zipf 1.05, "
                         "load + forward/backward + dump with eviction", keys_per_pass=per_pass * nnz, passes=passes)


def fwd_probe(h, args):
    D, total, nnz = 128, 40_000_000, 55296 * 26
    table = torch.empty((total, D), dtype=torch.float32, device=DEV)
    datagen.fill_table(SEED, table, 1 << 21)
    out = torch.empty((nnz, 1, D), device=DEV)
    layer = h.EmbeddingLayer(table, 1, h.SUM, [0], [total])
    ws = layer.new_workspace(layer.workspace_bytes(nnz, nnz))
    res = []

    def run(name, keys):
        keys = keys.contiguous()
        ms = timeit(lambda: layer.forward(nnz, keys, out=out, ws=ws), 20, 3)
        res.append(dict(pattern=name, us=ms * 1e3, algorithmic_GBs=nnz * (8 + 2 * D * 4) / ms / 1e6))

    run("all keys name one row", torch.zeros(nnz, dtype=torch.int64, device=DEV))
    for hot in (1 << 10, 1 << 14, 1 << 18, 1 << 22):
        idx = torch.randint(0, hot, (nnz,), device=DEV)
        run(f"uniform over {hot} rows spread over the table", idx * (total // hot))
        run(f"uniform over {hot} rows in one stretch of the table", idx)   # same reuse, addresses close together
    run("distinct random rows", torch.randperm(total, device=DEV)[:nnz])
    run("consecutive rows", torch.arange(nnz, device=DEV))
    flat, src = out.view(-1), torch.empty(nnz * D, device=DEV)
    ms = timeit(lambda: flat.copy_(src), 20, 3)
    res.append(dict(pattern="torch device copy of the output size", us=ms * 1e3, read_write_GBs=nnz * D * 8 / ms / 1e6))
    ms = timeit(lambda: flat.fill_(1.5), 20, 3)
    res.append(dict(pattern="torch fill of the output", us=ms * 1e3, write_GBs=nnz * D * 4 / ms / 1e6))
    return dict(workload="forward kernel (one slot, 40,000,000 x 128 fp32 rows, 1,437,696 one-hot keys) on key patterns "
                         "of known locality", patterns=res)


def placement(h, args):
    """How much the physical placement of the buffers matters on this machine: (1) a plain device copy of
    the headline's output size at many distances between source and destination inside one allocation;
    (2) the headline step with the 85 GB table freed and allocated again; (3) the forward with its output
    at many offsets inside one allocation."""
    MB = 1 << 20
    nb = 55296 * 26 * 128 * 4

    def copy_rate(src, dst, n=10):
        ms = timeit(lambda: dst.copy_(src), n, 2)
        return 2 * nb / ms / 1e9                                  # TB/s

    pool = torch.empty(14 * 1024 * MB, dtype=torch.uint8, device=DEV)
    src = pool[0:nb].view(torch.float32)
    by_offset = [(d, copy_rate(src, pool[d * MB:d * MB + nb].view(torch.float32))) for d in range(768, 12 * 1024, 32)]
    del pool, src
    torch.cuda.empty_cache()
    slow = [d for d, r in by_offset if r < 4.8]
    res = dict(copy_TBs_max=max(r for _, r in by_offset), copy_TBs_min=min(r for _, r in by_offset),
               copy_offsets_probed=len(by_offset), copy_slow_offsets_MB=slow[:16],
               copy_slow_offsets_mod_128MB=sorted({d % 128 for d in slow}))
    rows_t = datagen.DLRM_TABLE_ROWS
    S, D, B = 26, 128, 55296
    ro = datagen.row_offsets(rows_t)
    base, total = ro[:-1].copy(), int(ro[-1])
    nnz = B * S
    smp = datagen.make_samplers(rows_t, 1.05)
    keys = [datagen.onehot_keys(SEED, b, rows_t, B, 1.05, samplers=smp).to(DEV) for b in range(8)]
    del smp

    def step_times(table, out, dYs, n=40):
        layer = h.EmbeddingLayer(table, S, h.SUM, base, rows_t)
        ws = layer.new_workspace(layer.workspace_bytes(B, nnz))
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(n)]
        for i in range(n):
            ev[i][0].record()
            layer.forward(B, keys[i % 8], out=out, ws=ws)
            ev[i][1].record()
            layer.backward_sgd(B, keys[i % 8], dYs[i % 2], 1e-6, ws=ws)
            ev[i][2].record()
        torch.cuda.synchronize()
        return (float(np.median([e[0].elapsed_time(e[1]) for e in ev[5:]])) * 1e3,
                float(np.median([e[1].elapsed_time(e[2]) for e in ev[5:]])) * 1e3)

    trials = []
    for trial in range(4):
        table = torch.empty((total, D), dtype=torch.float32, device=DEV)
        table.fill_(0.25)
        dYs = [torch.randn((B, S, D), device=DEV) for _ in range(2)]
        out = torch.empty((B, S, D), device=DEV)
        f, b = step_times(table, out, dYs)
        trials.append(dict(trial=trial, table_at=hex(table.data_ptr()), forward_us=f, backward_us=b))
        if trial == 3:   # the forward alone, output at 64 offsets inside one allocation
            pool = torch.empty(nb + 520 * MB, dtype=torch.uint8, device=DEV)
            layer = h.EmbeddingLayer(table, S, h.SUM, base, rows_t)
            ws = layer.new_workspace(layer.workspace_bytes(B, nnz))
            it = [0]

            def fwd(o):
                layer.forward(B, keys[it[0] % 8], out=o, ws=ws)
                it[0] += 1
            outs = [timeit(lambda: fwd(pool[d * MB:d * MB + nb].view(torch.float32).view(B, S, D)), 16, 4) * 1e3
                    for d in range(0, 512, 8)]
            res["forward_us_over_64_output_offsets"] = [min(outs), max(outs)]
            del pool
        del table, dYs, out
        torch.cuda.empty_cache()
    res["step_after_reallocating_the_table"] = trials
    return dict(workload="placement probes: device copy by source-destination distance; headline step with the table "
                         "allocated again; forward by output offset", **res)


def speedmap(h, args):
    """Speed of plain fills, copies and gathers of random 512-byte rows by the position at which a new
    process is handed its memory: pieces of 8 GiB allocated one after the other, each timed on its own."""
    GiB = 1 << 30
    free, _ = torch.cuda.mem_get_info(DEV)
    n_pieces = int((free - 6 * GiB) // (8 * GiB))
    pieces = [torch.empty(8 * GiB, dtype=torch.uint8, device=DEV) for _ in range(n_pieces)]
    for c in pieces:
        c.fill_(1)
    idx = torch.randint(0, 8 * GiB // 512, (1 << 21,), device=DEV)
    dst = torch.empty((1 << 21, 128), dtype=torch.float32, device=DEV)
    res = []
    for i, c in enumerate(pieces):
        f32 = c.view(torch.float32)
        half = f32.numel() // 2
        rows = f32.view(-1, 128)
        t_fill = timeit(lambda: f32.fill_(2.0), 5, 1) * 1e-3
        t_copy = timeit(lambda: f32[half:].copy_(f32[:half]), 5, 1) * 1e-3
        t_gath = timeit(lambda: torch.index_select(rows, 0, idx, out=dst), 5, 1) * 1e-3
        res.append(dict(piece=i, handed_out_GiB=[8 * i, 8 * i + 8], fill_TBs=8 * GiB / t_fill / 1e12,
                        copy_TBs=8 * GiB / t_copy / 1e12, gather_512B_rows_TBs=2 * (1 << 21) * 512 / t_gath / 1e12))
    return dict(workload="fill, copy (read + write) and torch.index_select of 2 M random 512-byte rows inside pieces of 8 GiB "
                         "allocated one after the other by a new process", pieces=res)


def which_buffer(h, args):
    """Which buffer's placement decides the speed of the headline step: bench.py's allocations in
    bench.py's order with the table allocated the plain way, then one buffer replaced at a time."""
    rows_t = datagen.DLRM_TABLE_ROWS
    S, D, B = 26, 128, 55296
    ro = datagen.row_offsets(rows_t)
    base, total = ro[:-1].copy(), int(ro[-1])
    nnz = B * S
    table = torch.empty((total, D), dtype=torch.float32, device=DEV)
    datagen.fill_table(SEED, table, 1 << 21)
    smp = datagen.make_samplers(rows_t, 1.05)
    keys = [datagen.onehot_keys(SEED, b, rows_t, B, 1.05, samplers=smp).to(DEV) for b in range(8)]
    del smp
    dYs = [datagen.normal_grads(SEED, b, nnz * D, device=DEV).view(B, S, D) for b in range(2)]
    out = torch.empty((B, S, D), dtype=torch.float32, device=DEV)
    layer = h.EmbeddingLayer(table, S, h.SUM, base, rows_t)
    ws = layer.workspace(B, nnz)

    def times(layer, out, dYs, ws, n=40):
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(n)]
        for i in range(n):
            ev[i][0].record()
            layer.forward(B, keys[i % 8], out=out, ws=ws)
            ev[i][1].record()
            layer.backward_sgd(B, keys[i % 8], dYs[i % 2], 1e-6, ws=ws)
            ev[i][2].record()
        torch.cuda.synchronize()
        return dict(forward_us=float(np.median([e[0].elapsed_time(e[1]) for e in ev[5:]])) * 1e3,
                    backward_us=float(np.median([e[1].elapsed_time(e[2]) for e in ev[5:]])) * 1e3)

    res = [dict(what="as bench.py allocates, table first", **times(layer, out, dYs, ws))]
    out2 = torch.empty((B, S, D), dtype=torch.float32, device=DEV)
    res.append(dict(what="new output", **times(layer, out2, dYs, ws)))
    dY2 = [d.clone() for d in dYs]
    res.append(dict(what="new gradients", **times(layer, out, dY2, ws)))
    ws2 = layer.new_workspace(layer.workspace_bytes(B, nnz))
    res.append(dict(what="new workspace", **times(layer, out, dYs, ws2)))
    res.append(dict(what="new output, gradients and workspace", **times(layer, out2, dY2, ws2)))
    MB = 1 << 20
    nb = nnz * D * 4
    pool = torch.empty(nb + 300 * MB, dtype=torch.uint8, device=DEV)
    for d in (0, 4, 16, 36, 64, 100, 128, 200, 256):
        o = pool[d * MB:d * MB + nb].view(torch.float32).view(B, S, D)
        res.append(dict(what=f"output inside a new pool at +{d} MB", **times(layer, o, dYs, ws, n=25)))
    del pool, out2, dY2, ws2
    for trial in range(3):
        del layer, table
        torch.cuda.empty_cache()
        table = torch.empty((total, D), dtype=torch.float32, device=DEV)
        datagen.fill_table(SEED, table, 1 << 21)
        layer = h.EmbeddingLayer(table, S, h.SUM, base, rows_t)
        res.append(dict(what=f"table freed and allocated again ({trial + 1}), other buffers kept", **times(layer, out, dYs, ws)))
    return dict(workload="headline step (forward / backward, medians of 35 steps) with one buffer replaced at a time", probes=res)


def group(h, args):
    rows_t = datagen.DLRM_TABLE_ROWS
    B, L = 55296, len(rows_t)
    dims = [(128, 64, 32, 16)[t % 4] for t in range(L)]
    tables = []
    with h.behind_spacer(SPACER_GIB, sum(int(rows_t[t]) * dims[t] * 4 for t in range(L))):
        for t in range(L):
            tables.append(torch.empty((int(rows_t[t]), dims[t]), dtype=torch.float32, device=DEV))
    for t in range(L):
        datagen.fill_table(SEED + t, tables[t], 1 << 21)
    smp = datagen.make_samplers(rows_t, 1.05, device=DEV)
    keys = [datagen.onehot_keys(SEED, b, rows_t, B, 1.05, device=DEV, samplers=smp) for b in range(4)]
    del smp
    g = h.EmbeddingGroup(tables, [(t, h.SUM, 1) for t in range(L)])
    nnz = B * L
    ws = g.new_workspace(g.workspace_bytes(B, nnz))
    out = torch.empty((B, g.width), device=DEV)
    dY = datagen.normal_grads(SEED, 3, B * g.width, device=DEV).view(B, g.width)
    it = [0]

    def fwd():
        g.forward(B, keys[it[0] % 4], out=out, ws=ws)
        it[0] += 1

    def bwd():
        g.backward_sgd(B, keys[it[0] % 4], dY, 0.01, ws=ws)
        it[0] += 1

    f = timeit(fwd, 20, 4)
    b = timeit(bwd, 20, 4)
    row_bytes = sum(4 * d for d in dims)                       # one sample: every lookup's row once
    fwd_bytes = B * (L * 8 + row_bytes + g.width * 4)          # keys + rows read + output written
    bwd_bytes = B * (L * (8 + 8) + g.width * 4)                # keys + generated offsets + dY read; row updates come on top
    return dict(workload="fused group: 26 fp32 tables of the DLRM sizes with widths 128/64/32/16 (cycling), one lookup "
                         "per table, sum, dense one-hot input, batch 55296, Zipf 1.05", keys=nnz, width=g.width,
                forward_ms=f, forward_algorithmic_GBs=fwd_bytes / f / 1e6, backward_ms=b,
                backward_read_GBs=bwd_bytes / b / 1e6, fwd_bwd_keys_per_s=nnz / ((f + b) * 1e-3))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("workload", choices=["multihot", "hashed", "cache", "group", "mixed", "etc", "fwd_probe", "placement", "speedmap", "which_buffer"])
    ap.add_argument("--etc-passes", type=int, default=4)
    ap.add_argument("--spacer-gib", type=float, default=SPACER_GIB)
    ap.add_argument("--host-rows", type=int, default=0,
                    help="rows of the pinned host table (cache: default = the largest of 1e8 / 5e7 / 2e7 that can be "
                         "pinned; training cache: default 2e7)")
    ap.add_argument("--hash-batches", type=int, default=100)
    ap.add_argument("--cache-reps", type=int, default=1000, help="queries per batch size and mode (fewer under a profiler)")
    args = ap.parse_args()
    if not torch.cuda.is_available():
        print("bench_workloads.py: no GPU visible; the HIP path has no CPU fallback.", file=sys.stderr)
        sys.exit(2)
    import paper_2210_08803_amd as h
    globals()["SPACER_GIB"] = args.spacer_gib
    res = {"multihot": multihot, "hashed": hashed, "cache": cache, "group": group, "mixed": mixed, "etc": etc, "fwd_probe": fwd_probe,
           "placement": placement, "speedmap": speedmap, "which_buffer": which_buffer}[args.workload](h, args)
    res["n_gpus"] = 1
    res["data"] = "synthetic"
    res["tables_behind_spacer_gib"] = args.spacer_gib
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
