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


def host_copy_of(table, log_every_s=5.0):
    """The device table copied into ordinary host memory, a slab at a time."""
    total, D = table.shape
    host = np.empty((total, D), dtype=np.float32)
    slab = 1 << 22                                             # 2 GiB of fp32 rows of 128
    t_last = time.time()
    for r0 in range(0, total, slab):
        r1 = min(total, r0 + slab)
        torch.from_numpy(host[r0:r1]).copy_(table[r0:r1])
        if time.time() - t_last > log_every_s:
            log(f"  host copy of the table: {r1 / total:.0%}")
            t_last = time.time()
    return host


def cpu_baseline(table, table_rows, base, keys_batches, seed, alpha, budget_s=25.0):
    """The oracle's all-cores variant (bit-equal to the single-threaded one, tests/test_oracle_mt.py)
    on the host: key -> row, forward and backward + SGD over whole batches of the same workload.
    The host table is dense, the device table copied to ordinary host memory, when it fits in half
    of the host's RAM; otherwise every table is scaled by one factor (stated in `sample`) and the
    keys are drawn again for the scaled tables.  Median over at least 5 timed batches."""
    import oracle
    import psutil
    S = len(table_rows)
    threads = oracle.hardware_threads()
    ram = psutil.virtual_memory().total
    need = int(table.shape[0]) * DIM * 4
    t0 = time.time()
    if need <= 0.5 * ram:
        host = host_copy_of(table)
        rows_h, base_h, batches, note = list(table_rows), base, [k.numpy() for k in keys_batches], "dense host copy of the full table"
    else:
        f = 0.5 * ram / need
        f = float(f"{f:.1g}") if float(f"{f:.1g}") <= f else float(f"{f:.1g}") / 2
        rows_h = datagen.scaled_table_rows(f)
        ro = datagen.row_offsets(rows_h)
        base_h, total_h = ro[:-1].copy(), int(ro[-1])
        host = np.empty((total_h, DIM), dtype=np.float32)
        for r0 in range(0, total_h, 1 << 21):
            r1 = min(total_h, r0 + (1 << 21))
            host[r0:r1] = datagen.table_rows_at(seed, torch.arange(r0, r1), DIM, torch.float32).numpy()
        smp = datagen.make_samplers(rows_h, alpha) if alpha > 0 else None
        batches = [datagen.onehot_keys(seed, b, rows_h, BATCH, alpha, samplers=smp).numpy() for b in range(len(keys_batches))]
        note = f"every table scaled x{f:g} to fit half of the host's {ram / 2**30:.0f} GiB"
    log(f"cpu baseline: host table {host.shape[0]} x {DIM} ready in {time.time() - t0:.1f}s, {threads} threads")
    times = []
    spent = 0.0
    for b, k in enumerate(batches):
        dY = datagen.normal_grads(seed, 1000 + b, len(k) * DIM).numpy().reshape(len(k), DIM)
        t0 = time.perf_counter()
        rows, _ = oracle.rows_direct(base_h, rows_h, k, threads=threads)
        oracle.emb_forward(host, rows, threads=threads)
        oracle.emb_backward_sgd(host, rows, dY, LR, threads=threads)
        times.append(time.perf_counter() - t0)
        spent += times[-1]
        if spent > budget_s and len(times) >= 5:
            break
    nk = len(batches[0])
    return {"value": nk / float(np.median(times)), "unit": "keys/s", "cores": threads, "kind": "oracle",
            "sample": f"{len(times)} full batches of {nk} keys, key -> row + forward + backward/SGD each, median; "
                      f"{note}; all-cores variant of the oracle",
            "batch_s_median": float(np.median(times)), "batch_s_min": float(min(times))}


def parity_on_timed_batch(layer, table, base, S, keys_cpu, keys_dev, dY, out, ws):
    """One more step on a batch, gradient buffer, output buffer and workspace of the timed region,
    checked against the oracle: pooled rows and dedup result exactly, updated rows within
    1e-5 * max(|ref|, sum|terms| / 8).  The oracle works on the rows the batch touches, read from the
    device table as it stands before the step.  Raises on any difference."""
    import oracle
    threads = oracle.hardware_threads()
    k = keys_cpu.numpy()
    nnz = len(k)
    g_rows = (k.reshape(-1, S) + base[None, :]).reshape(-1)
    uniq, inv = np.unique(g_rows, return_inverse=True)
    u_dev = torch.from_numpy(uniq).to(table.device)
    before = table[u_dev].cpu().numpy()
    dY_h = dY.cpu().numpy().reshape(nnz, DIM)
    ref_out = oracle.emb_forward(before, inv, threads=threads)
    ref_tab = before.copy()
    o_uniq, o_cnt = oracle.emb_backward_sgd(ref_tab, inv, dY_h, LR, threads=threads)
    g_abs = np.zeros(before.shape, dtype=np.float32)
    oracle.emb_backward_sgd(g_abs, inv, np.abs(dY_h), 1.0, threads=threads)
    mag = np.abs(before.astype(np.float64)) + float(np.float32(LR)) * np.abs(g_abs.astype(np.float64))   # sum of |terms|

    layer.forward(BATCH, keys_dev, out=out, ws=ws)
    layer.backward_sgd(BATCH, keys_dev, dY, LR, ws=ws)
    torch.cuda.synchronize()
    got_out = out.cpu().numpy().reshape(nnz, DIM)
    assert np.array_equal(got_out.view(np.uint32), ref_out.view(np.uint32)), "parity: pooled output differs from the oracle"
    d_rows, d_cnt = layer.dedup_result(BATCH, nnz, ws=ws)
    assert np.array_equal(d_rows.cpu().numpy(), uniq), "parity: distinct rows differ from the oracle"
    assert np.array_equal(d_cnt.cpu().numpy(), o_cnt) and np.array_equal(o_uniq, np.arange(len(uniq))), \
        "parity: occurrence counts differ from the oracle"
    got = table[u_dev].cpu().numpy().astype(np.float64)
    ref64 = ref_tab.astype(np.float64)
    err = np.abs(got - ref64)
    tol = 1e-5 * np.maximum(np.abs(ref64), mag / 8.0)
    assert (err <= tol).all(), f"parity: updated rows differ from the oracle, max err {err.max():.3e}"
    return {"keys": int(nnz), "distinct_rows": int(len(uniq)), "max_abs_err_updated_rows": float(err.max())}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--scale", type=float, default=1.0)
    ap.add_argument("--seed", type=int, default=datagen.DEFAULT_SEED)
    ap.add_argument("--alpha", type=float, default=ALPHA,
                    help="Zipf exponent of the keys (0 = uniform); anything but the default is an experiment")
    ap.add_argument("--table-spacer-gib", type=float, default=96.0,
                    help="device memory allocated before the table and freed right after (0: none)")
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
    # behind a spacer: the first tens of gigabytes a process is handed are the slow place for a table
    # (see allocate_table); --table-spacer-gib 0 allocates it the plain way
    table = hctr.allocate_table(total, DIM, torch.float32, dev, spacer_gib=args.table_spacer_gib)
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
    # parity re-asserted on timed inputs: the batch, gradient and buffers the next step would have used
    j = (args.warmup + args.steps) % N_KEY_BATCHES
    parity = parity_on_timed_batch(layer, table, base, S, keys_cpu[j], keys[j], dYs[j % 2], out, ws)
    log(f"parity on a timed batch: {parity}")
    # what the same chip copies at: a device copy of the pooled-output size (read + write), for scale
    cp = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    for it in range(6):
        if it == 1:
            cp[0].record(stream)
        out.copy_(dYs[0])
    cp[1].record(stream)
    torch.cuda.synchronize()
    copy_gbs = 2 * out.numel() * 4 * 5 / (cp[0].elapsed_time(cp[1]) * 1e-3) / 1e9
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
    # HBM bytes per launch by the profiler's counters: a stored figure from profiles/ (the two
    # rocprofv3 --pmc runs cannot happen inside this process), stamped with the commit it was taken on.
    traffic, prof = None, {}
    tpath = os.path.join(ROOT, "profiles", "dlrm_onehot_hbm_traffic.json")
    if os.path.exists(tpath) and args.scale == 1.0 and args.alpha == ALPHA:
        try:
            prof = json.load(open(tpath))
            traffic = prof["kernels"]["fwd_onehot"]["traffic_bytes_per_launch"]
        except Exception:
            traffic, prof = None, {}
    step_traffic = prof.get("step_traffic_bytes")
    # the stored figure belongs to the kernels as they were when it was taken
    import hashlib
    src = os.path.join(ROOT, "paper_2210_08803_amd", "csrc", "emb.hip")
    traffic_current = bool(prof) and hashlib.sha256(open(src, "rb").read()).hexdigest()[:16] == prof.get("emb_hip_sha16")
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
                   "batch": BATCH, "slots": S, "dim": DIM, "keys_per_step": nnz, "distinct_rows_per_step": int(U),
                   "table_allocation": ("first allocation of the process" if args.table_spacer_gib <= 0 else
                                        "behind %g GiB of device memory (pieces of 8 GiB) that are freed again "
                                        "before the other buffers are made" % args.table_spacer_gib)},
        "parity_checked": True, "parity": parity,
        "roofline": {"bound": "hbm", "kernel": "fwd_onehot<float,float,32,16>", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     # achieved / frac count ALGORITHMIC bytes (every key's row, also when L2 serves it);
                     # measured_* count the bytes the profiler saw cross the HBM interface
                     "measured_GBs": None if traffic is None else traffic / fwd_s / 1e9,
                     "measured_frac": None if traffic is None else traffic / fwd_s / 1e9 / HBM_PEAK_GBS,
                     "traffic_source": None if traffic is None else
                     {"file": "profiles/dlrm_onehot_hbm_traffic.json", "kind": "stored rocprofv3 --pmc figure",
                      "measured_on_commit": prof.get("commit"),
                      "kernel_source_unchanged_since": traffic_current},
                     "device_copy_GBs": copy_gbs,
                     "step_traffic": step_traffic,
                     "step_measured_GBs": None if step_traffic is None else step_traffic / (elapsed / args.steps) / 1e9,
                     "step_measured_frac": None if step_traffic is None else
                     step_traffic / (elapsed / args.steps) / 1e9 / HBM_PEAK_GBS,
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
        del layer
        res["cpu_baseline"] = cpu_baseline(table, table_rows, base, keys_cpu, args.seed, args.alpha)
        res["gpu_over_cpu"] = value / res["cpu_baseline"]["value"]
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
