"""GPU: hctr_cache_query_static (the query whose work arrays live in the library's static device
array) against hctr_cache_query with a caller workspace, through the C ABI.  Two caches over the same
host table get the same calls, one through each entry point; outputs, hit masks, tags, stamps, cached
rows and statistics must be equal bit for bit after every call.  The second call is smaller than the
first, so it runs on top of what the first left in the array.  Runs last: a failure here must not hide
the other tests."""
import ctypes as C

import numpy as np
import pytest
import torch

import datagen
import oracle

pytestmark = pytest.mark.gpu
SEED = datagen.DEFAULT_SEED


def H():
    import paper_2210_08803_amd as h
    return h


def pinned_table(rows, dim):
    t = torch.empty((rows, dim), dtype=torch.float32, pin_memory=True)
    t.copy_(datagen.table_rows_at(SEED, torch.arange(rows), dim, torch.float32))
    return t


def both(ws_cache, st_cache, ref, keys, n_bags, insert, what):
    """One call through each entry point, raw ctypes, then everything compared."""
    L = H().lib()
    d_keys = torch.from_numpy(keys).cuda()
    n, dim = len(keys), ws_cache.dim
    outs, hits = [], []
    stream = torch.cuda.current_stream().cuda_stream
    for cache, static in ((ws_cache, False), (st_cache, True)):
        out = torch.full((n_bags, dim), float("nan"), dtype=torch.float32, device="cuda")
        hit = torch.full((n,), 7, dtype=torch.uint8, device="cuda")
        if static:
            st = L.hctr_cache_query_static(cache.handle, n_bags, 1, d_keys.data_ptr(), None, n, int(insert),
                                           out.data_ptr(), hit.data_ptr(), stream)
        else:
            ws = cache.workspace(n)
            st = L.hctr_cache_query(cache.handle, n_bags, 1, d_keys.data_ptr(), None, n, int(insert),
                                    out.data_ptr(), hit.data_ptr(), ws.data_ptr(), ws.numel(), stream)
        assert st == 0, (what, static, L.hctr_last_error().decode())
        outs.append(out)
        hits.append(hit)
    torch.cuda.synchronize()
    assert torch.equal(outs[0], outs[1]), f"{what}: pooled outputs differ"
    assert torch.equal(hits[0], hits[1]), f"{what}: hit masks differ"
    assert ws_cache.stats == st_cache.stats, what
    ta, sa = ws_cache.state()
    tb, sb = st_cache.state()
    assert torch.equal(ta, tb) and torch.equal(sa, sb), f"{what}: tags / stamps differ"
    live = (ta.view(-1) != -1).cuda()
    assert torch.equal(ws_cache.data()[live], st_cache.data()[live]), f"{what}: cached rows differ"
    # and both equal the oracle's simulation of the same call
    ref_out, ref_hit = ref.query(keys, n_bags, insert_missing=insert)
    assert np.array_equal(hits[1].cpu().numpy(), ref_hit), f"{what}: hit mask differs from the oracle"
    assert st_cache.stats == ref.stats.tolist(), what
    err = np.abs(outs[1].cpu().numpy().astype(np.float64) - ref_out)
    assert err.max() <= 1e-5, f"{what}: pooled output off by {err.max():.3e}"   # sums of 4 terms of at most 1/16


@pytest.mark.parametrize("small_limit", [8192, 0], ids=["fused-small", "general"])
def test_static_scratch_query_equals_the_workspace_query(small_limit):
    host_rows, dim, num_sets, ways = 60000, 128, 512, 8
    host = pinned_table(host_rows, dim)
    a = H().EmbeddingCache(num_sets, ways, host)
    b = H().EmbeddingCache(num_sets, ways, host)
    a.set_small_call_limit(small_limit)
    b.set_small_call_limit(small_limit)
    ref = oracle.Cache(num_sets, ways, host.numpy())
    smp = datagen.ZipfSampler(host_rows, 1.2)
    # 64 samples x 26 slots x 4 keys, then 8 samples: the smaller call runs over the larger one's leftovers
    for it, (n_bags, insert) in enumerate([(64 * 26, True), (8 * 26, True), (64 * 26, False), (3 * 26, True)]):
        keys = datagen.cache_keys(SEED, 900 + it, host_rows, n_bags * 4, 1.2, sampler=smp).numpy()
        if it == 1:
            keys[::13] = -5                 # keys without a row
            keys[1::31] = host_rows + 9
        both(a, b, ref, np.ascontiguousarray(keys), n_bags, insert, f"call {it} ({small_limit})")


def test_static_scratch_query_rejects_what_does_not_fit():
    L = H().lib()
    host = pinned_table(1000, 16)
    c = H().EmbeddingCache(16, 4, host)
    n = 8192 + 4
    keys = torch.zeros(n, dtype=torch.int64, device="cuda")
    out = torch.zeros((n // 4, 16), dtype=torch.float32, device="cuda")
    st = L.hctr_cache_query_static(c.handle, n // 4, 1, keys.data_ptr(), None, n, 1, out.data_ptr(), None, None)
    assert st == -4 and b"8192" in L.hctr_last_error()
    assert L.hctr_cache_query_static(None, 1, 1, keys.data_ptr(), None, 4, 1, out.data_ptr(), None, None) == -2
    torch.cuda.synchronize()
    assert c.stats[0] == 0                  # nothing ran
    # rows of 1024 values on the general path: 8192 keys would stage 32 MB
    wide = pinned_table(300, 1024)
    cw = H().EmbeddingCache(8, 4, wide)
    keys = torch.zeros(8192, dtype=torch.int64, device="cuda")
    out = torch.zeros((2048, 1024), dtype=torch.float32, device="cuda")
    st = L.hctr_cache_query_static(cw.handle, 2048, 1, keys.data_ptr(), None, 8192, 1, out.data_ptr(), None, None)
    assert st == -4 and b"static scratch" in L.hctr_last_error()
    torch.cuda.synchronize()
    assert cw.stats[0] == 0
