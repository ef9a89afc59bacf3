"""GPU parity at the full sizes of the benchmark configurations.

The oracle cannot hold an 85 GB table, so it works on a compact table: the rows the batch (or
the sampled outputs) touch are regenerated on the host from the closed-form table contents and
keys are renumbered onto that compact table.  Where the whole batch is too much for the oracle
(86 M keys), outputs are sampled and the oracle computes exactly those, plus properties that
hold at any size."""
import numpy as np
import pytest
import torch

import datagen
import oracle
from parity import assert_close, check_table_update, oracle_backward, oracle_forward

pytestmark = pytest.mark.gpu
SEED = datagen.DEFAULT_SEED


def H():
    import paper_2210_08803_amd as h
    return h


def free():
    import gc
    gc.collect()
    torch.cuda.empty_cache()


def test_dlrm_onehot_full_size_in_the_timed_launch_configuration():
    """Config 'DLRM-shaped one-hot': 26 fp32 tables, 165 M rows x 128, batch 55,296, Zipf 1.05,
    run as bench.py runs it (dedup on a second stream, two workspaces), every output checked."""
    h = H()
    rows_t = datagen.DLRM_TABLE_ROWS
    S, D, B = 26, 128, 55296
    ro = datagen.row_offsets(rows_t)
    base, total = ro[:-1].copy(), int(ro[-1])
    nnz = B * S
    table = torch.empty((total, D), dtype=torch.float32, device="cuda")
    datagen.fill_table(SEED, table, chunk_rows=1 << 21)
    smp = datagen.make_samplers(rows_t, 1.05)
    layer = h.EmbeddingLayer(table, S, h.SUM, base, rows_t)
    wss = [layer.new_workspace(layer.workspace_bytes(B, nnz)) for _ in range(2)]
    main, side = torch.cuda.current_stream(), torch.cuda.Stream()
    out = torch.empty((B, S, D), dtype=torch.float32, device="cuda")
    n_steps = 2
    keys = [datagen.onehot_keys(SEED, 100 + i, rows_t, B, 1.05, samplers=smp) for i in range(n_steps + 1)]
    del smp
    dks = [k.cuda() for k in keys]
    layer.backward_dedup(B, dks[0], ws=wss[0])
    rng = np.random.default_rng(1)
    untouched_probe = torch.from_numpy(rng.integers(0, total, 200000))
    for i in range(n_steps):
        dY = datagen.normal_grads(SEED, 100 + i, nnz * D, device="cuda").view(B, S, D)
        # the compact problem for the oracle, from the GPU table as it stands before this step
        k = keys[i].numpy()
        g_rows = (k.reshape(-1, S) + base[None, :]).reshape(-1)
        uniq, inv = np.unique(g_rows, return_inverse=True)
        compact = table[torch.from_numpy(uniq).cuda()].cpu().numpy()
        if i == 0:   # untouched so far: the table is still the closed form
            assert np.array_equal(compact, datagen.table_rows_at(SEED, torch.from_numpy(uniq), D, torch.float32).numpy())
        ref_out, mag_out = oracle_forward(compact, inv, None, 0, nnz)
        ref_tab, mag_tab, o_uniq, o_cnt = oracle_backward(compact, inv, None, 0, nnz, dY.cpu().numpy().reshape(nnz, D), 0.01)

        w_cur, w_next = wss[i % 2], wss[(i + 1) % 2]
        layer.forward(B, dks[i], out=out, ws=w_cur)
        side.wait_stream(main)
        layer.backward_dedup(B, dks[i + 1], ws=w_next, stream=side)
        layer.backward_apply(B, nnz, dY, 0.01, ws=w_cur)
        main.wait_stream(side)
        torch.cuda.synchronize()

        got_out = out.cpu().numpy().reshape(nnz, D)
        assert np.array_equal(got_out.view(np.uint32), ref_out.view(np.uint32)), f"step {i}: forward not bit-exact"
        d_rows, d_cnt = layer.dedup_result(B, nnz, ws=w_cur)
        assert np.array_equal(d_rows.cpu().numpy(), uniq), f"step {i}: unique rows differ"
        assert np.array_equal(d_cnt.cpu().numpy(), o_cnt), f"step {i}: counts differ"
        assert np.array_equal(o_uniq, np.arange(len(uniq)))
        got = table[torch.from_numpy(uniq).cuda()].cpu().numpy()
        check_table_update(got, compact, ref_tab, mag_tab, np.arange(len(uniq)), f"step {i} backward")
        assert layer.invalid_keys(w_cur) == 0
    # rows no step addressed still hold the closed-form contents
    touched = np.unique(np.concatenate([(k.numpy().reshape(-1, S) + base[None, :]).reshape(-1) for k in keys[:n_steps]]))
    probe = untouched_probe[~torch.from_numpy(np.isin(untouched_probe.numpy(), touched))]
    assert torch.equal(table[probe.cuda()].cpu(), datagen.table_rows_at(SEED, probe, D, torch.float32))
    del table, out, layer, wss
    free()


def _close_in_chunks(gpu, ref, mag, what, rows_per_chunk=1 << 18):
    for r0 in range(0, len(ref), rows_per_chunk):
        r1 = min(len(ref), r0 + rows_per_chunk)
        assert_close(gpu[r0:r1], ref[r0:r1], mag[r0:r1], f"{what}, rows {r0}..{r1}")


def test_multihot_fp16_mean_full_size_every_bag_and_every_row():
    """Config 'Multi-hot': the 26 tables in fp16, batch 65,536, hotness 1..100, Zipf 1.1, mean.
    ~86 M keys.  The oracle's all-cores variant (bit-equal to the pinned single-threaded one) works
    on the compact table of the rows the batch touches: EVERY bag of the forward and EVERY touched
    row of the backward is compared, the dedup against torch.unique on everything."""
    h = H()
    rows_t = datagen.DLRM_TABLE_ROWS
    S, D, B = 26, 128, 65536
    ro = datagen.row_offsets(rows_t)
    base, total = ro[:-1].copy(), int(ro[-1])
    n_bags = B * S
    threads = oracle.hardware_threads()
    table = torch.empty((total, D), dtype=torch.float16, device="cuda")
    datagen.fill_table(SEED, table, chunk_rows=1 << 21)
    smp = datagen.make_samplers(rows_t, 1.1, device="cuda")
    offsets = datagen.multihot_offsets(SEED, 7, n_bags, 1, 100, device="cuda")
    keys = datagen.multihot_keys(SEED, 7, rows_t, B, 1.1, offsets, device="cuda", samplers=smp)
    del smp
    free()
    nnz = keys.numel()
    assert 80e6 < nnz < 92e6
    dY = datagen.normal_grads(SEED, 7, n_bags * D, device="cuda").view(B, S, D)
    layer = h.EmbeddingLayer(table, S, h.MEAN, base, rows_t)
    ws = layer.new_workspace(layer.workspace_bytes(B, nnz))
    out = layer.forward(B, keys, offsets, ws=ws)
    torch.cuda.synchronize()

    # the compact problem (plumbing on the GPU: which rows, renumbered keys)
    hot = offsets[1:] - offsets[:-1]
    bag_of_key = torch.repeat_interleave(torch.arange(n_bags, device="cuda"), hot)
    g_rows = keys + torch.from_numpy(base).cuda()[bag_of_key % S]
    del bag_of_key
    uniq_d, inv_d, cnt_d = torch.unique(g_rows, return_inverse=True, return_counts=True)
    del g_rows
    uniq, inv, cnt = uniq_d.cpu().numpy(), inv_d.cpu().numpy(), cnt_d.cpu().numpy()
    del inv_d, cnt_d
    before16 = table[uniq_d].cpu().numpy()
    probe = np.random.default_rng(5).choice(len(uniq), 50000, replace=False)
    assert np.array_equal(before16[probe], datagen.table_rows_at(SEED, torch.from_numpy(uniq[probe]), D, torch.float16).numpy())
    off_np = offsets.cpu().numpy()
    print(f"multi-hot: {nnz} keys, {len(uniq)} distinct rows, oracle on {threads} threads", flush=True)

    # forward, every bag.  fp16 -> fp32 is exact (and numpy's widening equals the oracle's own decoder
    # on every finite pattern, tests/test_oracle_forward.py), so the oracle sums the same values.
    before32 = before16.astype(np.float32)
    ref_out = oracle.emb_forward(before32, inv, off_np, oracle.MEAN, threads=threads)
    mag_out = oracle.emb_forward(np.abs(before32), inv, off_np, oracle.MEAN, threads=threads)
    del before32
    _close_in_chunks(out.cpu().numpy().reshape(n_bags, D), ref_out, mag_out, "forward (all bags)")
    del ref_out, mag_out, out
    print("multi-hot: forward of every bag matches", flush=True)

    # backward, every touched row
    layer.backward_sgd(B, keys, dY, 0.01, offsets, ws=ws)
    torch.cuda.synchronize()
    d_rows, d_cnt = layer.dedup_result(B, nnz, ws=ws)
    assert np.array_equal(d_rows.cpu().numpy(), uniq) and np.array_equal(d_cnt.cpu().numpy(), cnt)
    assert int(d_cnt.sum()) == nnz and layer.invalid_keys(ws) == 0
    dY_h = dY.cpu().numpy().reshape(n_bags, D)
    ref_tab = before16.copy()
    o_uniq, o_cnt = oracle.emb_backward_sgd(ref_tab, inv, dY_h, 0.01, off_np, oracle.MEAN, threads=threads)
    assert np.array_equal(o_uniq, np.arange(len(uniq))) and np.array_equal(o_cnt, cnt)
    g_abs = np.zeros(before16.shape, dtype=np.float32)
    oracle.emb_backward_sgd(g_abs, inv, np.abs(dY_h), 1.0, off_np, oracle.MEAN, threads=threads)
    got = table[uniq_d].cpu().numpy()
    for r0 in range(0, len(uniq), 1 << 18):
        r1 = min(len(uniq), r0 + (1 << 18))
        mag = np.abs(before16[r0:r1].astype(np.float64)) + float(np.float32(0.01)) * np.abs(g_abs[r0:r1].astype(np.float64))
        check_table_update(got[r0:r1], before16[r0:r1], ref_tab[r0:r1], mag, np.arange(r1 - r0), f"backward rows {r0}..{r1}")
    print("multi-hot: every updated row matches", flush=True)
    # rows never addressed keep the closed form
    probe = torch.from_numpy(np.random.default_rng(6).integers(0, total, 100000))
    probe = probe[~torch.from_numpy(np.isin(probe.numpy(), uniq))]
    assert torch.equal(table[probe.cuda()].cpu(), datagen.table_rows_at(SEED, probe, D, torch.float16))
    del table, dY, keys, offsets, layer, ws
    free()


def test_hashed_open_key_space_full_size():
    """Config 'Hashed open key space': capacity 1e8, up to 8e7 rows, dim 64 fp32, 26 one-hot slots,
    batch 131,072, Zipf 1.05 over 2^63 ids, insert on miss; rows compared exactly for every key."""
    h = H()
    S, D, B = 26, 64, 131072
    cap, max_rows = 100_000_000, 80_000_000
    ht = h.HashTable(cap, max_rows)
    ref = oracle.Hash(max_rows)
    table = torch.empty((max_rows, D), dtype=torch.float32, device="cuda")
    datagen.fill_table(SEED, table, chunk_rows=1 << 22)
    layer = h.EmbeddingLayer(table, S, h.SUM, hash_table=ht, insert_on_miss=True)
    nnz = B * S
    ws = layer.new_workspace(layer.workspace_bytes(B, nnz))
    smp = datagen.ZipfSampler(1 << 63, 1.05, device="cuda")
    out = torch.empty((B, S, D), dtype=torch.float32, device="cuda")
    rng = np.random.default_rng(9)
    for it in range(3):
        keys = datagen.open_space_keys(SEED, it, S, B, 1.05, device="cuda", sampler=smp)
        rows_ref = ref.insert_or_find(keys.cpu().numpy(), True)
        layer.forward(B, keys, out=out, ws=ws)
        rows_gpu = ht.insert_or_find(keys, False)             # everything forward inserted is found
        torch.cuda.synchronize()
        assert np.array_equal(rows_gpu.cpu().numpy(), rows_ref), f"batch {it}: key -> row differs"
        assert ht.size == ref.size
        frac_new = ref.size / ((it + 1) * nnz)
        assert 0.15 < frac_new < 0.75                         # Zipf(1.05) over 2^63 ids: most keys of a batch are new
        # forward on sampled bags: one-hot, so the pooled row is the table row, bit for bit
        bags = torch.from_numpy(rng.choice(nnz, 20000, replace=False))
        want = table[torch.from_numpy(rows_ref)[bags].cuda()]
        assert torch.equal(out.view(nnz, D)[bags.cuda()], want)
        # backward on everything the batch touches
        dY = datagen.normal_grads(SEED, 50 + it, nnz * D, device="cuda").view(B, S, D)
        uniq, inv = np.unique(rows_ref, return_inverse=True)
        compact = table[torch.from_numpy(uniq).cuda()].cpu().numpy()
        ref_tab, mag_tab, o_uniq, o_cnt = oracle_backward(compact, inv, None, 0, nnz, dY.cpu().numpy().reshape(nnz, D), 0.01)
        layer.backward_sgd(B, keys, dY, 0.01, ws=ws)
        torch.cuda.synchronize()
        d_rows, d_cnt = layer.dedup_result(B, nnz, ws=ws)
        assert np.array_equal(d_rows.cpu().numpy(), uniq) and np.array_equal(d_cnt.cpu().numpy(), o_cnt)
        got = table[torch.from_numpy(uniq).cuda()].cpu().numpy()
        check_table_update(got, compact, ref_tab, mag_tab, np.arange(len(uniq)), f"hashed backward {it}")
        assert ht.size == ref.size
    del table, out, layer, ws, ht
    free()


def test_hashed_high_load_and_saturation_at_capacity_1e8():
    """Config 'Hashed open key space' where it is hardest: the table of capacity 1e8 is filled to
    load 0.775 on both sides (77.5 M distinct keys, whose rows must come out 0, 1, 2, ...), then
    Zipf batches carry it across max_rows = 8e7 (load 0.8): the batch that hits the limit has some
    new keys accepted and the rest refused, the batches after it only find or refuse.  Every key's
    row, the size, the count of keys without a row, the pooled rows (sampled; one key per bag, so
    bit for bit) and every touched row of the backward are compared with the oracle."""
    h = H()
    S, D, B = 26, 64, 131072
    cap, max_rows, prefill = 100_000_000, 80_000_000, 77_500_000
    ht = h.HashTable(cap, max_rows)
    ref = oracle.Hash(max_rows)
    odd, salt, m63 = 0x5851F42D4C957F2D, 0x1234567, (1 << 63) - 1
    chunk = 1 << 22
    for c0 in range(0, prefill, chunk):
        c1 = min(prefill, c0 + chunk)
        want = torch.arange(c0, c1, dtype=torch.int64, device="cuda")
        keys = (want * odd + salt) & m63                      # odd multiplier: distinct keys
        rows = ht.insert_or_find(keys, True)
        assert torch.equal(rows, want), f"prefill chunk at {c0}: rows are not first-appearance order"
        r_ref = ref.insert_or_find(keys.cpu().numpy(), True)
        assert r_ref[0] == c0 and r_ref[-1] == c1 - 1
        if c0 % (16 * chunk) == 0:
            print(f"hashed prefill {c1}/{prefill}", flush=True)
    assert ht.size == ref.size == prefill

    table = torch.empty((max_rows, D), dtype=torch.float32, device="cuda")
    datagen.fill_table(SEED, table, chunk_rows=1 << 22)
    layer = h.EmbeddingLayer(table, S, h.SUM, hash_table=ht, insert_on_miss=True)
    nnz = B * S
    ws = layer.new_workspace(layer.workspace_bytes(B, nnz))
    smp = datagen.ZipfSampler(1 << 63, 1.05, device="cuda")
    out = torch.empty((B, S, D), dtype=torch.float32, device="cuda")
    rng = np.random.default_rng(19)
    refused_total, sizes = 0, []
    for it in range(5):
        keys = datagen.open_space_keys(SEED, 200 + it, S, B, 1.05, device="cuda", sampler=smp)
        if it == 1:
            keys[::1000] = (torch.arange(0, keys.numel(), 1000, device="cuda") * odd + salt) & m63   # prefilled keys are found
        rows_ref = ref.insert_or_find(keys.cpu().numpy(), True)
        layer.forward(B, keys, out=out, ws=ws)
        rows_gpu = ht.insert_or_find(keys, False)
        torch.cuda.synchronize()
        assert np.array_equal(rows_gpu.cpu().numpy(), rows_ref), f"batch {it}: key -> row differs"
        assert ht.size == ref.size
        sizes.append(ref.size)
        refused = int((rows_ref < 0).sum())
        refused_total += refused
        assert layer.invalid_keys(ws) == refused_total, f"batch {it}: refused keys miscounted"
        bags = torch.from_numpy(rng.choice(nnz, 50000, replace=False))
        r_s = torch.from_numpy(rows_ref)[bags]
        want = table[r_s.clamp(min=0).cuda()] * (r_s >= 0).cuda()[:, None]     # a refused key pools zeros
        assert torch.equal(out.view(nnz, D)[bags.cuda()], want), f"batch {it}: pooled rows differ"
        dY = datagen.normal_grads(SEED, 250 + it, nnz * D, device="cuda").view(B, S, D)
        uniq, inv = np.unique(rows_ref, return_inverse=True)
        if uniq[0] < 0:                                        # refused keys: no row, skipped by backward
            uniq, inv = uniq[1:], inv - 1
        compact = table[torch.from_numpy(uniq).cuda()].cpu().numpy()
        ref_tab, mag_tab, o_uniq, o_cnt = oracle_backward(compact, inv, None, 0, nnz, dY.cpu().numpy().reshape(nnz, D), 0.01)
        layer.backward_sgd(B, keys, dY, 0.01, ws=ws)
        torch.cuda.synchronize()
        refused_total += refused                               # backward meets the same keys without a row
        d_rows, d_cnt = layer.dedup_result(B, nnz, ws=ws)
        assert np.array_equal(d_rows.cpu().numpy(), uniq) and np.array_equal(d_cnt.cpu().numpy(), o_cnt)
        got = table[torch.from_numpy(uniq).cuda()].cpu().numpy()
        check_table_update(got, compact, ref_tab, mag_tab, np.arange(len(uniq)), f"hashed backward at the limit {it}")
        assert ht.size == ref.size
        print(f"hashed batch {it}: size {ref.size}, refused {refused}", flush=True)
    assert sizes[0] < max_rows and sizes[-1] == max_rows and sizes[-2] == max_rows     # crossed, then stayed
    assert refused_total > 0
    del table, out, layer, ws, ht
    free()


def _pinned_host_table(candidates, D):
    """The largest of the candidate row counts that this machine pins in one allocation."""
    for host_rows in candidates:
        try:
            host = torch.empty((host_rows, D), dtype=torch.float32, pin_memory=True)
        except RuntimeError as e:                              # hipHostMalloc refused: try the next size
            print(f"pinning {host_rows} x {D} fp32 refused: {str(e).splitlines()[0]}", flush=True)
            continue
        for r0 in range(0, host_rows, 1 << 21):
            r1 = min(host_rows, r0 + (1 << 21))
            host[r0:r1].copy_(datagen.table_rows_at(SEED, torch.arange(r0, r1, device="cuda"), D, torch.float32))
        torch.cuda.synchronize()
        return host
    raise RuntimeError("no candidate size could be pinned")


def test_inference_cache_batch_sweep_at_scale():
    """Config 'Inference cache' at the largest size the GPU machine allows.  The configuration names a
    5e8-row x 128 fp32 table (256 GB) in pinned host memory; the box has 295 GB of RAM but pins at
    most 64 GiB in one allocation (80 GiB is refused), so the table has 1e8 rows (51.2 GB, scale 1/5;
    5e7 and 1e7 rows are the fall-backs on a smaller machine).  Cache = 10 % of the rows in 32-way sets:
    1e7 lines, 5.12 GB of rows, so line offsets pass 4 GiB.  26 slots x hotness 4, Zipf 1.2, batches
    1 / 64 / 1,024 / 16,384; every call is compared with the oracle's simulation: hit mask, statistics,
    tags and stamps exactly, pooled rows in tolerance; cached rows compared beyond the 4 GiB offset."""
    import psutil
    h = H()
    D, S, hot, ways = 128, 26, 4, 32
    print(f"host RAM {psutil.virtual_memory().total / 2**30:.0f} GiB", flush=True)
    host = _pinned_host_table((100_000_000, 50_000_000, 10_000_000), D)
    host_rows = host.shape[0]
    num_sets = host_rows // 10 // ways
    print(f"inference cache test: host table {host_rows} rows = {host_rows * D * 4 / 1e9:.1f} GB pinned, "
          f"cache {num_sets * ways} lines = {num_sets * ways * D * 4 / 1e9:.2f} GB", flush=True)
    gpu = h.EmbeddingCache(num_sets, ways, host)
    ref = oracle.Cache(num_sets, ways, host.numpy())
    smp = datagen.ZipfSampler(host_rows, 1.2)
    call = 0
    hits = []
    for batch in (16384, 16384, 16384, 1024, 64, 1, 16384, 1, 64, 1024, 16384):
        n_bags = batch * S
        keys = datagen.cache_keys(SEED, call, host_rows, n_bags * hot, 1.2, sampler=smp)
        call += 1
        ref_out, ref_hit = ref.query(keys.numpy(), n_bags, insert_missing=True)
        d_hit = torch.zeros(keys.numel(), dtype=torch.uint8, device="cuda")
        out = gpu.query(batch, S, keys.cuda(), None, True, hit_mask=d_hit)
        torch.cuda.synchronize()
        assert np.array_equal(d_hit.cpu().numpy(), ref_hit), f"call {call}: hit mask differs"
        assert gpu.stats == ref.stats.tolist(), f"call {call}: stats differ"
        mag = np.abs(host.numpy()[keys.numpy()]).astype(np.float64).reshape(n_bags, hot, D).sum(1)
        assert_close(out.cpu().numpy().reshape(n_bags, D), ref_out, mag, f"call {call}: pooled output")
        hits.append(ref_hit.mean())
    tags, stamps = gpu.state()
    rtags, rstamps, rdata = ref.state(with_data=True)
    assert np.array_equal(tags.numpy().view(np.uint64), rtags) and np.array_equal(stamps.numpy().astype(np.uint32), rstamps)
    # the cached rows themselves, where the byte offset of a line passes 4 GiB (line * 512 B)
    live = np.flatnonzero((rtags != oracle.EMPTY_TAG).ravel())
    far = live[live >= (1 << 32) // (D * 4)]
    if host_rows >= 100_000_000:
        assert len(far) > 1000, "no resident line beyond the 4 GiB offset"
    pick = np.concatenate([far[:200000], live[:200000]])
    assert np.array_equal(gpu.data()[torch.from_numpy(pick).cuda()].cpu().numpy(), rdata[pick]), "cached rows differ"
    assert hits[0] == 0.0 and hits[-1] > 0.8                  # cold start, then the Zipf head is resident
    del gpu, host, ref, rdata
    free()
