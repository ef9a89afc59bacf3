#!/usr/bin/env python3
"""Benchmark of the embedding hot path on one MI355X: forward + backward(SGD) keys/s on the
26-slot DLRM-shaped one-hot workload, with the roofline figure of the dominant kernel and the
CPU oracle timed beside it.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--scale F] [--no-cpu-baseline]

A step is one forward and one backward+SGD pass of the whole layer over one batch of 55,296
samples x 26 slots (1,437,696 keys).  Inputs (table, keys, upstream gradients) are resident in HBM
before the timed region starts.  --scale shrinks every table by one factor (for small-memory
debugging only; the reported workload name then says so).
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

BATCH = 55296
DIM = 128
ALPHA = 1.05
LR = 0.01
N_KEY_BATCHES = 8
HBM_PEAK_GBS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_baseline(table_rows, base, keys_batches, seed, budget_s=20.0):
    """The oracle, as it stands, on the host: forward + backward over whole batches of the same
    workload.  The 85 GB table is not copied to the host: the rows a batch touches are generated
    into a compact table (same values, same key -> row structure), which keeps the arithmetic and
    the access pattern per key but makes the host working set smaller than the real one."""
    import oracle
    S = len(table_rows)
    done_keys, spent, batches = 0, 0.0, 0
    for keys in keys_batches:
        k = keys.numpy()
        rows_global = (k.reshape(-1, S) + base[None, :]).reshape(-1)
        uniq, inv = np.unique(rows_global, return_inverse=True)
        compact = datagen.table_rows_at(seed, torch.from_numpy(uniq), DIM, torch.float32).numpy()
        dY = datagen.normal_grads(seed, 1000 + batches, len(k) * DIM).numpy().reshape(len(k), DIM)
        comp_keys = inv.astype(np.int64)
        t0 = time.perf_counter()
        rows, _ = oracle.rows_direct([0] * S, [len(uniq)] * S, comp_keys)
        oracle.emb_forward(compact, rows)
        oracle.emb_backward_sgd(compact, rows, dY, LR)
        spent += time.perf_counter() - t0
        done_keys += len(k)
        batches += 1
        if spent > budget_s:
            break
    return {"value": done_keys / spent, "unit": "keys/s", "cores": 1, "kind": "oracle",
            "sample": f"{batches} full batch(es) of {len(keys_batches[0])} keys, forward+backward, "
                      f"table compacted to the rows each batch touches"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--scale", type=float, default=1.0)
    ap.add_argument("--seed", type=int, default=datagen.DEFAULT_SEED)
    ap.add_argument("--alpha", type=float, default=ALPHA,
                    help="Zipf exponent of the keys (0 = uniform); anything but the default is an experiment")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--schedule", choices=["serial", "overlap", "pipeline"], default="serial",
                    help="how the key-only half of backward is placed in time (see step())")
    ap.add_argument("--graph", action="store_true",
                    help="serial schedule only: capture each key batch's step in a HIP graph and replay it "
                         "(one launch per step; the per-phase event times are then not available)")
    ap.add_argument("--calibrate-gather", action="store_true",
                    help="also run the forward kernel once on all-distinct rows (known bytes, no cache reuse)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain device copy of the pooled-output size (for scaling profiler byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on one GPU only; --gpus must be 1 (no collectives, no sharding).")
        sys.exit(2)
    if not torch.cuda.is_available():
        log("bench.py: no GPU visible; the HIP path has no CPU fallback.")
        sys.exit(2)

    import paper_2210_08803_amd as hctr
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    table_rows = datagen.DLRM_TABLE_ROWS if args.scale == 1.0 else datagen.scaled_table_rows(args.scale)
    S = len(table_rows)
    ro = datagen.row_offsets(table_rows)
    base, total = ro[:-1].copy(), int(ro[-1])
    nnz = BATCH * S

    t0 = time.time()
    table = torch.empty((total, DIM), dtype=torch.float32, device=dev)
    datagen.fill_table(args.seed, table, chunk_rows=1 << 21)
    torch.cuda.synchronize()
    log(f"table {total} x {DIM} fp32 = {total * DIM * 4 / 1e9:.1f} GB filled in {time.time() - t0:.1f}s")

    t0 = time.time()
    samplers = datagen.make_samplers(table_rows, args.alpha) if args.alpha > 0 else None
    keys_cpu = [datagen.onehot_keys(args.seed, b, table_rows, BATCH, args.alpha, samplers=samplers)
                for b in range(N_KEY_BATCHES)]
    del samplers
    keys = [k.to(dev) for k in keys_cpu]
    dYs = [datagen.normal_grads(args.seed, b, nnz * DIM, device=dev).view(BATCH, S, DIM) for b in range(2)]
    out = torch.empty((BATCH, S, DIM), dtype=torch.float32, device=dev)
    uniq_per_batch = [int(torch.unique(k.view(-1, S) + torch.from_numpy(base)).numel()) for k in keys_cpu]
    log(f"inputs generated in {time.time() - t0:.1f}s; distinct rows per batch ~{int(np.mean(uniq_per_batch))}")

    layer = hctr.EmbeddingLayer(table, S, hctr.SUM, base, table_rows)
    ws = layer.workspace(BATCH, nnz)
    stream = torch.cuda.current_stream()

    # One step = forward + backward (dedup + apply) of one batch.  The key-only half of backward
    # (key -> row, sort, run boundaries) depends on nothing but the keys, so it can run on a second
    # stream.  Schedules:
    #   serial    everything on one stream, in order;
    #   overlap   dedup(i) beside forward(i), apply(i) after both;
    #   pipeline  forward(i) alone, then apply(i) beside dedup(i+1) (the next batch's keys are known
    #             ahead of time, as from a prefetching data reader; two workspaces alternate).
    # Every schedule runs exactly one forward, one dedup and one apply per step.
    side = torch.cuda.Stream()
    ws2 = layer.new_workspace(layer.workspace_bytes(BATCH, nnz)) if args.schedule == "pipeline" else None
    wss = [ws, ws2]

    graphs = None

    def step(i, ev=None):
        k = keys[i % N_KEY_BATCHES]
        if graphs is not None:
            if ev:
                ev[0].record(stream)
            graphs[i % N_KEY_BATCHES].replay()
            if ev:
                ev[2].record(stream)
        elif args.schedule == "serial":
            if ev:
                ev[0].record(stream)
            layer.forward(BATCH, k, out=out, ws=ws)
            if ev:
                ev[1].record(stream)
            layer.backward_sgd(BATCH, k, dYs[i % 2], LR, ws=ws)
            if ev:
                ev[2].record(stream)
        elif args.schedule == "overlap":
            side.wait_stream(stream)            # the previous step's apply has finished with ws
            if ev:
                ev[3].record(side)
            layer.backward_dedup(BATCH, k, ws=ws, stream=side)
            if ev:
                ev[4].record(side)
                ev[0].record(stream)
            layer.forward(BATCH, k, out=out, ws=ws)
            if ev:
                ev[1].record(stream)
            stream.wait_stream(side)
            layer.backward_apply(BATCH, nnz, dYs[i % 2], LR, ws=ws)
            if ev:
                ev[2].record(stream)
        else:
            w_cur, w_next = wss[i % 2], wss[(i + 1) % 2]
            if ev:
                ev[0].record(stream)
            layer.forward(BATCH, k, out=out, ws=w_cur)
            if ev:
                ev[1].record(stream)
            side.wait_stream(stream)            # apply(i-1), the last reader of w_next, is done
            if ev:
                ev[3].record(side)
            layer.backward_dedup(BATCH, keys[(i + 1) % N_KEY_BATCHES], ws=w_next, stream=side)
            if ev:
                ev[4].record(side)
            layer.backward_apply(BATCH, nnz, dYs[i % 2], LR, ws=w_cur)   # dedup(i) was ordered before forward(i)
            stream.wait_stream(side)
            if ev:
                ev[2].record(stream)

    if args.graph:
        if args.schedule != "serial":
            log("bench.py: --graph goes with --schedule serial only.")
            sys.exit(2)
        for i in range(2):                       # once eagerly, so that nothing is initialised during capture
            step(i)
        torch.cuda.synchronize()
        captured = []
        side.wait_stream(stream)
        with torch.cuda.stream(side):
            for b in range(N_KEY_BATCHES):       # N_KEY_BATCHES is even: batch b always meets dY buffer b % 2
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=side):
                    layer.forward(BATCH, keys[b], out=out, ws=ws)
                    layer.backward_sgd(BATCH, keys[b], dYs[b % 2], LR, ws=ws)
                captured.append(g)
        stream.wait_stream(side)
        torch.cuda.synchronize()
        graphs = captured

    if args.schedule == "pipeline":             # dedup of the first batch: the pipeline's prologue
        layer.backward_dedup(BATCH, keys[0], ws=wss[0])
        torch.cuda.synchronize()

    if args.calibrate_copy:   # a plain copy of known size: reads and writes out.numel()*4 bytes
        out.copy_(dYs[0])
        torch.cuda.synchronize()
    if args.calibrate_gather:  # the forward kernel on nnz DISTINCT rows: no reuse, so it must fetch
        cal = hctr.EmbeddingLayer(table, 1, hctr.SUM, [0], [total])   # nnz*(8+512) and write nnz*512 bytes
        cal_keys = torch.randperm(total, device=dev)[:nnz].contiguous()
        cal.forward(nnz, cal_keys, out=out.view(nnz, 1, DIM))
        torch.cuda.synchronize()
        del cal, cal_keys
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i, evs[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    if graphs is not None:   # only the whole step is timed; the roofline figure then needs an eager run
        step_ms = np.array([e[0].elapsed_time(e[2]) for e in evs])
        log("bench.py --graph: %.4f ms per step by wall clock, %.4f median / %.4f min by events; run without "
            "--graph for the JSON line with the roofline figure" % (elapsed / args.steps * 1e3,
                                                                     float(np.median(step_ms)), float(step_ms.min())))
        print(json.dumps({"metric": "embedding keys/sec fwd+bwd, 26-slot DLRM shape, step replayed as a HIP graph",
                          "value": nnz / (elapsed / args.steps), "unit": "keys/s", "n_gpus": 1, "steps": args.steps,
                          "warmup": args.warmup, "ms_per_step": elapsed / args.steps * 1e3,
                          "step_ms_median": float(np.median(step_ms)), "data": "synthetic"}), flush=True)
        return
    fwd_ms = np.array([e[0].elapsed_time(e[1]) for e in evs])
    bwd_ms = np.array([e[1].elapsed_time(e[2]) for e in evs])
    dedup_ms = None if args.schedule == "serial" else np.array([e[3].elapsed_time(e[4]) for e in evs])
    assert layer.invalid_keys(ws) == 0

    ms_per_step = elapsed / args.steps * 1e3
    value = nnz / (elapsed / args.steps)

    # Roofline of the dominant kernel, the forward gather (fwd_onehot): one launch per step, and the
    # forward call launches nothing else, so the event pair around the call times exactly that kernel.
    # Algorithmic bytes per key: 8 (key) + 512 (table row read) + 512 (pooled row written).
    fwd_bytes = nnz * (8 + DIM * 4 + DIM * 4)
    fwd_s = float(fwd_ms.mean()) * 1e-3
    achieved = fwd_bytes / fwd_s / 1e9
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "fwd_onehot_dlrm_traffic.json")
    if os.path.exists(tpath) and args.scale == 1.0:
        try:
            traffic = json.load(open(tpath)).get("traffic_bytes_per_launch")
        except Exception:
            traffic = None
    U = float(np.mean(uniq_per_batch))
    bwd_bytes = nnz * 8 + nnz * DIM * 4 + U * 2 * DIM * 4   # keys, dY gather, row read-modify-write (sort excluded)

    res = {
        "metric": "embedding keys/sec fwd+bwd and achieved HBM GB/s (% of peak), 26-slot DLRM shape",
        "value": value, "unit": "keys/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "DLRM-shaped one-hot: 26 fp32 tables, dim 128, %d rows total, batch 55296, "
                               "Zipf %g, sum, fwd + dedup/segmented-reduce bwd + SGD%s"
                               % (total, args.alpha, "" if args.scale == 1.0 else f" (tables scaled x{args.scale})"),
                   "batch": BATCH, "slots": S, "dim": DIM, "keys_per_step": nnz, "distinct_rows_per_step": int(U)},
        "roofline": {"bound": "hbm", "kernel": "fwd_onehot<float,float,32,4>", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "algorithmic_bytes_per_launch": fwd_bytes,
                     # the same with every distinct row read once only (what no cache could go below)
                     "compulsory_bytes_per_launch": nnz * (8 + DIM * 4) + int(U) * DIM * 4,
                     "avg_launch_ms": float(fwd_ms.mean())},
        "phases": {"schedule": args.schedule,
                   # per-step GPU time between the step's first and last event (steps overlap under
                   # the pipelined schedules, so these are meaningful for `serial` only)
                   "step_ms_median": float(np.median(fwd_ms + bwd_ms)) if args.schedule == "serial" else None,
                   "step_ms_min": float((fwd_ms + bwd_ms).min()) if args.schedule == "serial" else None,
                   "forward_ms": float(fwd_ms.mean()), "forward_ms_min": float(fwd_ms.min()),
                   "backward_ms" if args.schedule == "serial" else "backward_apply_ms": float(bwd_ms.mean()),
                   "backward_dedup_ms": None if dedup_ms is None else float(dedup_ms.mean()),
                   "forward_keys_per_s": nnz / fwd_s,
                   "backward_logical_bytes": bwd_bytes,
                   "fwd_bwd_logical_GBs": (fwd_bytes + bwd_bytes) / (elapsed / args.steps) / 1e9},
    }
    if not args.no_cpu_baseline:
        del table
        torch.cuda.empty_cache()
        res["cpu_baseline"] = cpu_baseline(table_rows, base, keys_cpu, args.seed)
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
