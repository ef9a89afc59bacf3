#!/usr/bin/env python3
"""Timings of the configurations that are not the headline benchmark (bench.py covers that one):

    python bench_workloads.py multihot   # 26 fp16 tables, batch 65,536, hotness 1..100, mean: fwd / dedup / apply
    python bench_workloads.py hashed     # open 2^63 key space, capacity 1e8, dim 64: insert-or-find, fwd, bwd over load factor
    python bench_workloads.py cache      # inference cache, Zipf 1.2, batch 1 / 64 / 1024 / 16384: hit rate, keys/s, p50 latency
    python bench_workloads.py mixed      # headline shape in mixed precision: fp16 table + fp32 master rows, fp16 out / dY
    python bench_workloads.py etc        # training cache staged in host memory: load / train / dump passes of 8 batches
    python bench_workloads.py fwd_probe  # the forward kernel on key patterns of known locality (what bounds it)
    python bench_workloads.py group      # fused group: the 26 DLRM-sized tables with widths 128/64/32/16, dense one-hot input

Each prints one JSON line.  Inputs are synthetic and seeded (datagen/), resident in HBM (the cache's
backing table in pinned host memory) before anything is timed.  The inference-cache configuration
asks for a 5e8-row host table (256 GB); --host-rows scales it (default 2e7 rows = 10 GB), the cache
always holds 10 % of the rows in 32-way sets.
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


def multihot(h, args):
    rows_t = datagen.DLRM_TABLE_ROWS
    S, D, B = 26, 128, 65536
    ro = datagen.row_offsets(rows_t)
    base, total = ro[:-1].copy(), int(ro[-1])
    table = torch.empty((total, D), dtype=torch.float16, device=DEV)
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
    f = timeit(lambda: layer.forward(B, keys, offsets, out=out, ws=ws), 5, 1)
    d = timeit(lambda: layer.backward_dedup(B, keys, offsets, ws=ws), 5, 1)
    a = timeit(lambda: layer.backward_apply(B, nnz, dY, 0.01, offsets, ws=ws), 5, 1)
    uniq, _ = layer.dedup_result(B, nnz, ws=ws)
    fwd_bytes = nnz * (8 + D * 2) + B * S * (D * 4 + 8)
    apply_bytes = nnz * (8 + D * 4) + int(uniq.numel()) * 2 * D * 2
    return dict(workload="multi-hot: 26 fp16 tables, dim 128, batch 65536, hotness 1..100, Zipf 1.1, mean", keys=nnz,
                distinct_rows=int(uniq.numel()), forward_ms=f, forward_algorithmic_GBs=fwd_bytes / f / 1e6,
                backward_dedup_ms=d, backward_apply_ms=a, backward_apply_logical_GBs=apply_bytes / a / 1e6,
                fwd_bwd_keys_per_s=nnz / ((f + d + a) * 1e-3))


def hashed(h, args):
    S, D, B = 26, 64, 131072
    cap, max_rows = 100_000_000, 80_000_000
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
    return dict(workload="hashed open key space: capacity 1e8, max 8e7 rows, dim 64 fp32, 26 one-hot slots, "
                         "batch 131072, Zipf 1.05 over 2^63 ids, insert on miss", keys=nnz, find_only_ms=find_ms,
                find_only_keys_per_s=nnz / find_ms * 1e3, trace=trace)


def cache(h, args):
    host_rows, D, S, hot, ways = args.host_rows, 128, 26, 4, 32
    num_sets = host_rows // 10 // ways
    host = torch.empty((host_rows, D), dtype=torch.float32, pin_memory=True)
    for r0 in range(0, host_rows, 1 << 20):
        r1 = min(host_rows, r0 + (1 << 20))
        host[r0:r1].copy_(datagen.table_rows_at(SEED, torch.arange(r0, r1, device=DEV), D, torch.float32))
    c = h.EmbeddingCache(num_sets, ways, host)
    smp = datagen.ZipfSampler(host_rows, 1.2, DEV)
    call = 0
    for _ in range(30):   # warm up until the hit rate is stationary
        keys = datagen.cache_keys(SEED, call, host_rows, 16384 * S * hot, 1.2, device=DEV, sampler=smp)
        call += 1
        c.query(16384, S, keys)
    torch.cuda.synchronize()
    sweep = []
    for batch in (1, 64, 1024, 16384):
        n = batch * S * hot
        reps = 1000
        ks_by_mode = {m: [datagen.cache_keys(SEED, 1000 + 2000 * j + call + i, host_rows, n, 1.2, device=DEV, sampler=smp)
                          for i in range(reps)] for j, m in enumerate(("insert", "lookup_only"))}
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
        sweep.append(dict(batch=batch, keys=n, queries=reps,
                          **{f"{m}_{k}": v for m, r in res.items() for k, v in r.items()}))
    return dict(workload=f"inference cache: {host_rows} x 128 fp32 host table (pinned), cache 10% in 32-way sets, "
                         "26 slots x hotness 4, Zipf 1.2; latency = host call + stream sync, gpu = event pair around the call", sweep=sweep)


def mixed(h, args):
    rows_t = datagen.DLRM_TABLE_ROWS
    S, D, B = 26, 128, 55296
    ro = datagen.row_offsets(rows_t)
    base, total = ro[:-1].copy(), int(ro[-1])
    master = torch.empty((total, D), dtype=torch.float32, device=DEV)
    datagen.fill_table(SEED, master, 1 << 21)
    table = torch.empty((total, D), dtype=torch.float16, device=DEV)
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
    host_rows, D, S, B, per_pass = args.host_rows, 128, 26, 55296, 8
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
        run(f"uniform over {hot} rows spread over the table", torch.randint(0, hot, (nnz,), device=DEV) * (total // hot))
    run("distinct random rows", torch.randperm(total, device=DEV)[:nnz])
    run("consecutive rows", torch.arange(nnz, device=DEV))
    flat, src = out.view(-1), torch.empty(nnz * D, device=DEV)
    ms = timeit(lambda: flat.copy_(src), 20, 3)
    res.append(dict(pattern="torch device copy of the output size", us=ms * 1e3, read_write_GBs=nnz * D * 8 / ms / 1e6))
    ms = timeit(lambda: flat.fill_(1.5), 20, 3)
    res.append(dict(pattern="torch fill of the output", us=ms * 1e3, write_GBs=nnz * D * 4 / ms / 1e6))
    return dict(workload="forward kernel (one slot, 40,000,000 x 128 fp32 rows, 1,437,696 one-hot keys) on key patterns "
                         "of known locality", patterns=res)


def group(h, args):
    rows_t = datagen.DLRM_TABLE_ROWS
    B, L = 55296, len(rows_t)
    dims = [(128, 64, 32, 16)[t % 4] for t in range(L)]
    tables = []
    for t in range(L):
        tab = torch.empty((int(rows_t[t]), dims[t]), dtype=torch.float32, device=DEV)
        datagen.fill_table(SEED + t, tab, 1 << 21)
        tables.append(tab)
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
    ap.add_argument("workload", choices=["multihot", "hashed", "cache", "group", "mixed", "etc", "fwd_probe"])
    ap.add_argument("--etc-passes", type=int, default=4)
    ap.add_argument("--host-rows", type=int, default=20_000_000)
    ap.add_argument("--hash-batches", type=int, default=100)
    args = ap.parse_args()
    if not torch.cuda.is_available():
        print("bench_workloads.py: no GPU visible; the HIP path has no CPU fallback.", file=sys.stderr)
        sys.exit(2)
    import paper_2210_08803_amd as h
    res = {"multihot": multihot, "hashed": hashed, "cache": cache, "group": group, "mixed": mixed, "etc": etc, "fwd_probe": fwd_probe}[args.workload](h, args)
    res["n_gpus"] = 1
    res["data"] = "synthetic"
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
