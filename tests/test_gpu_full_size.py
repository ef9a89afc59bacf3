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


def test_multihot_fp16_mean_full_size_sampled():
    """Config 'Multi-hot': the 26 tables in fp16, batch 65,536, hotness 1..100, Zipf 1.1, mean.
    ~86 M keys: forward is checked on 3,000 sampled bags, backward on 3,000 sampled distinct rows
    (all of their occurrences), dedup against numpy.unique on everything."""
    h = H()
    rows_t = datagen.DLRM_TABLE_ROWS
    S, D, B = 26, 128, 65536
    ro = datagen.row_offsets(rows_t)
    base, total = ro[:-1].copy(), int(ro[-1])
    n_bags = B * S
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

    off_np, keys_np = offsets.cpu().numpy(), keys.cpu().numpy()
    hot = np.diff(off_np)
    bag_of_key = np.repeat(np.arange(n_bags), hot)
    g_rows = keys_np + base[bag_of_key % S]
    rng = np.random.default_rng(5)

    # forward on sampled bags
    bags = np.sort(rng.choice(n_bags, 3000, replace=False))
    sel = np.concatenate([np.arange(off_np[b], off_np[b + 1]) for b in bags])
    u_f, inv_f = np.unique(g_rows[sel], return_inverse=True)
    compact_f = datagen.table_rows_at(SEED, torch.from_numpy(u_f), D, torch.float16).numpy()
    small_off = np.concatenate([[0], np.cumsum(hot[bags])])
    ref_out, mag_out = oracle_forward(compact_f, inv_f, small_off, oracle.MEAN, len(bags))
    got_out = out.view(n_bags, D)[torch.from_numpy(bags).cuda()].cpu().numpy()
    assert_close(got_out, ref_out, mag_out, "sampled forward")

    # backward on sampled distinct rows, all their occurrences, true bag weights
    layer.backward_sgd(B, keys, dY, 0.01, offsets, ws=ws)
    torch.cuda.synchronize()
    uniq, cnt = np.unique(g_rows, return_counts=True)
    d_rows, d_cnt = layer.dedup_result(B, nnz, ws=ws)
    assert np.array_equal(d_rows.cpu().numpy(), uniq) and np.array_equal(d_cnt.cpu().numpy(), cnt)
    assert int(d_cnt.sum()) == nnz and layer.invalid_keys(ws) == 0
    heavy = uniq[np.argsort(cnt)[-20:]]                       # the longest segments are in the sample
    pick = np.unique(np.concatenate([heavy, rng.choice(uniq, 3000, replace=False)]))
    remap = np.full(len(g_rows), -1, dtype=np.int64)
    pos = np.searchsorted(pick, g_rows)
    hit = (pos < len(pick)) & (pick[np.minimum(pos, len(pick) - 1)] == g_rows)
    remap[hit] = pos[hit]
    compact_b = datagen.table_rows_at(SEED, torch.from_numpy(pick), D, torch.float16).numpy()
    ref_tab, mag_tab, o_uniq, o_cnt = oracle_backward(compact_b, remap, off_np, oracle.MEAN, n_bags,
                                                      dY.cpu().numpy().reshape(n_bags, D), 0.01)
    assert np.array_equal(o_cnt, cnt[np.searchsorted(uniq, pick)])
    got = table[torch.from_numpy(pick).cuda()].cpu().numpy()
    check_table_update(got, compact_b, ref_tab, mag_tab, np.arange(len(pick)), "sampled backward")
    # rows never addressed keep the closed form
    probe = torch.from_numpy(rng.integers(0, total, 100000))
    probe = probe[~torch.from_numpy(np.isin(probe.numpy(), uniq))]
    assert torch.equal(table[probe.cuda()].cpu(), datagen.table_rows_at(SEED, probe, D, torch.float16))
    del table, out, dY, keys, offsets, layer, ws
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


def test_inference_cache_batch_sweep_at_scale():
    """Config 'Inference cache', scaled to a 10 M x 128 fp32 table in pinned host memory (5 GB; the
    configuration's 5e8 rows = 256 GB do not fit a test), cache = 10 % of the rows in 32-way sets,
    26 slots x hotness 4, Zipf 1.2, batches 1 / 64 / 1,024 / 16,384; every call is compared with
    the oracle's simulation: hit mask, statistics, tags and stamps exactly, pooled rows in tolerance."""
    h = H()
    host_rows, D, S, hot, ways = 10_000_000, 128, 26, 4, 32
    num_sets = host_rows // 10 // ways
    host = torch.empty((host_rows, D), dtype=torch.float32, pin_memory=True)
    for r0 in range(0, host_rows, 1 << 20):
        r1 = min(host_rows, r0 + (1 << 20))
        host[r0:r1].copy_(datagen.table_rows_at(SEED, torch.arange(r0, r1, device="cuda"), D, torch.float32))
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
    rtags, rstamps = ref.state()
    assert np.array_equal(tags.numpy().view(np.uint64), rtags) and np.array_equal(stamps.numpy().astype(np.uint32), rstamps)
    assert hits[0] == 0.0 and hits[-1] > 0.8                  # cold start, then the Zipf head is resident
    del gpu, host
    free()
