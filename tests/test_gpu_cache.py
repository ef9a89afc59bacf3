"""GPU parity: hctr_cache_query against the oracle's cache simulation.  Hit masks, tags, stamps
and statistics must match exactly after every call; pooled outputs within the fp32 tolerance."""
import json
import os

import numpy as np
import pytest
import torch

import datagen
import oracle
from parity import assert_close, to_dev

pytestmark = pytest.mark.gpu
SEED = datagen.DEFAULT_SEED
GOLD = os.path.join(os.path.dirname(__file__), "golden", "cache_batch_lru_trace.json")


def H():
    import paper_2210_08803_amd as h
    return h


def pinned_table(rows, dim, seed=SEED):
    t = torch.empty((rows, dim), dtype=torch.float32, pin_memory=True)
    t.copy_(datagen.table_rows_at(seed, torch.arange(rows), dim, torch.float32))
    return t


class Pair:
    def __init__(self, num_sets, ways, host, small_limit=None):
        self.host = host
        self.gpu = H().EmbeddingCache(num_sets, ways, host)
        if small_limit is not None:
            self.gpu.set_small_call_limit(small_limit)
        self.ref = oracle.Cache(num_sets, ways, host.numpy())
        self.num_sets, self.ways = num_sets, ways

    def query(self, keys, n_bags, offsets=None, insert=True, what=""):
        keys = np.ascontiguousarray(keys, dtype=np.int64)
        ref_out, ref_hit = self.ref.query(keys, n_bags, offsets=offsets, insert_missing=insert)
        d_hit = torch.zeros(len(keys), dtype=torch.uint8, device="cuda")
        d_off = None if offsets is None else to_dev(np.ascontiguousarray(offsets, dtype=np.int64))
        out = self.gpu.query(n_bags, 1, to_dev(keys), d_off, insert, hit_mask=d_hit)
        torch.cuda.synchronize()
        assert np.array_equal(d_hit.cpu().numpy(), ref_hit), f"{what}: hit mask differs"
        assert self.gpu.stats == self.ref.stats.tolist(), f"{what}: stats {self.gpu.stats} vs {self.ref.stats.tolist()}"
        tags, stamps = self.gpu.state()
        rtags, rstamps, rdata = self.ref.state(with_data=True)
        assert np.array_equal(tags.numpy().view(np.uint64), rtags), f"{what}: tags differ"
        assert np.array_equal(stamps.numpy().astype(np.uint32), rstamps), f"{what}: stamps differ"
        live = (rtags != oracle.EMPTY_TAG).ravel()
        data = self.gpu.data().cpu().numpy()
        assert np.array_equal(data[live], rdata[live]), f"{what}: cached rows differ"
        # magnitude of the terms: gather-sum of |row| from the host table
        valid = (keys >= 0) & (keys < self.host.shape[0])
        bag = (np.repeat(np.arange(n_bags), np.diff(offsets)) if offsets is not None
               else np.arange(len(keys)) // max(1, len(keys) // n_bags))
        mag = np.zeros((n_bags, self.host.shape[1]))
        np.add.at(mag, bag[valid], np.abs(self.host.numpy()[keys[valid]]).astype(np.float64))
        assert_close(out.cpu().numpy().reshape(n_bags, -1), ref_out, mag, f"{what}: pooled output")
        return ref_hit


def test_hand_worked_trace():
    g = json.load(open(GOLD))
    host = torch.empty((g["host_rows"], g["dim"]), dtype=torch.float32, pin_memory=True)
    host.copy_(torch.arange(g["host_rows"] * g["dim"], dtype=torch.float32).view(g["host_rows"], g["dim"]) / 8)
    gpu = H().EmbeddingCache(g["num_sets"], g["ways"], host)
    for call in g["calls"]:
        keys = torch.tensor(call["keys"], dtype=torch.int64, device="cuda")
        hit = torch.zeros(len(call["keys"]), dtype=torch.uint8, device="cuda")
        gpu.query(call["n_bags"], 1, keys, None, bool(call["insert"]), hit_mask=hit)
        torch.cuda.synchronize()
        tags, stamps = gpu.state()
        assert hit.cpu().tolist() == call["hit"]
        assert tags[0].tolist() == call["tags"] and stamps[0].tolist() == call["stamps"]
        assert gpu.stats == call["stats"]


@pytest.mark.parametrize("small_limit", [0, 8192], ids=["general", "fused-small"])
@pytest.mark.parametrize("num_sets,ways,dim", [(64, 8, 16), (1, 4, 8), (37, 1, 32), (16, 32, 128), (5, 64, 4), (300, 2, 260)])
def test_zipf_traffic_matches_the_simulation(num_sets, ways, dim, small_limit):
    host_rows = 5000
    p = Pair(num_sets, ways, pinned_table(host_rows, dim), small_limit)
    smp = datagen.ZipfSampler(host_rows, 1.2)
    hits = 0
    for it in range(12):
        n_bags, hot = 26 * 9, 4
        keys = datagen.cache_keys(SEED, it, host_rows, n_bags * hot, 1.2, sampler=smp).numpy()
        if it == 5:
            keys[::17] = -3
            keys[1::29] = host_rows + 5                        # outside the host table
        hits += p.query(keys, n_bags, insert=(it % 4 != 3), what=f"call {it}").sum()
    assert hits > 0


@pytest.mark.parametrize("small_limit", [0, 8192], ids=["general", "fused-small"])
def test_call_count_limit_lowers_stamps_like_the_simulation(small_limit):
    """With a limit of 6 the call count and every stamp are lowered by 3 every few calls; ways not
    used for 3 calls collapse to stamp 0.  Tags, stamps, rows and statistics must stay equal to the
    oracle's after each of 40 calls, insert-only calls included."""
    host_rows, dim = 3000, 32
    p = Pair(24, 4, pinned_table(host_rows, dim), small_limit)
    p.gpu.set_epoch_limit(6)
    p.ref.set_epoch_limit(6)
    smp = datagen.ZipfSampler(host_rows, 1.1)
    lowered = 0
    for it in range(40):
        before = p.ref.epoch
        keys = datagen.cache_keys(SEED, 300 + it, host_rows, 60, 1.1, sampler=smp).numpy()
        if it % 7 == 3:
            p.ref.insert(keys)
            p.gpu.insert(to_dev(keys))
            torch.cuda.synchronize()
            _state_equal(p, f"insert {it}")
        else:
            p.query(keys, 20, insert=(it % 5 != 4), what=f"call {it}")
        lowered += p.ref.epoch <= before
        assert p.ref.epoch <= 6
    assert lowered >= 10


@pytest.mark.parametrize("small_limit", [0, 8192], ids=["general", "fused-small"])
def test_csr_bags_and_batch_of_one_key(small_limit):
    host_rows, dim = 800, 64
    p = Pair(32, 4, pinned_table(host_rows, dim), small_limit)
    rng = np.random.default_rng(8)
    for it in range(10):
        h = rng.integers(0, 7, 90)
        offsets = np.concatenate([[0], np.cumsum(h)])
        keys = rng.zipf(1.3, offsets[-1]) % host_rows
        p.query(keys, 90, offsets=offsets, what=f"csr {it}")
    for it in range(30):
        p.query(rng.integers(0, 50, 1), 1, what=f"single {it}")   # classical per-access LRU traffic


@pytest.mark.parametrize("small_limit", [0, 8192], ids=["general", "fused-small"])
@pytest.mark.parametrize("dim", [16, 260], ids=["d16", "d260-never-fused"])
def test_bags_without_keys_still_count_as_a_call(small_limit, dim):
    """A call whose bags are all empty writes zeros, inserts nothing and advances the call count, so the
    stamps of the calls around it come out as in the simulation."""
    p = Pair(8, 4, pinned_table(500, dim), small_limit)
    g = np.random.default_rng(5)
    p.query(g.integers(0, 500, 60), 20, what="before")
    for insert in (True, False):
        p.query(np.zeros(0, dtype=np.int64), 3, offsets=np.zeros(4, dtype=np.int64), insert=insert, what="empty bags")
    p.query(g.integers(0, 500, 60), 20, what="after")


@pytest.mark.parametrize("small_limit", [0, 8192], ids=["general", "fused-small"])
def test_set_overflow_in_one_call_skips_the_surplus(small_limit):
    host_rows, dim = 4096, 8
    p = Pair(2, 4, pinned_table(host_rows, dim), small_limit)
    keys = np.arange(64)                                          # ~32 new keys per set, 4 ways each
    p.query(keys, 64, what="flood")
    assert p.ref.stats[5] > 0
    p.query(keys[::-1].copy(), 64, what="flood again")
    p.query(np.zeros(0, dtype=np.int64), 3, offsets=np.zeros(4, dtype=np.int64), what="empty bags")


def test_paths_switch_back_and_forth_on_one_cache():
    """Calls above and below the small-call limit interleaved on one cache (one workspace)."""
    host_rows, dim = 60000, 64
    p = Pair(128, 16, pinned_table(host_rows, dim))
    smp = datagen.ZipfSampler(host_rows, 1.2)
    for it, batch in enumerate([300, 2, 79, 300, 1, 78, 79, 300]):     # 26*4*78 = 8112 <= 8192 < 26*4*79
        n_bags = batch * 26
        keys = datagen.cache_keys(SEED, 50 + it, host_rows, n_bags * 4, 1.2, sampler=smp).numpy()
        p.query(keys, n_bags, what=f"mixed {it} (batch {batch})")


# ---- manipulation operators ---------------------------------------------------------------------

def _state_equal(p, what):
    tags, stamps = p.gpu.state()
    rtags, rstamps, rdata = p.ref.state(with_data=True)
    assert np.array_equal(tags.numpy().view(np.uint64), rtags), f"{what}: tags differ"
    assert np.array_equal(stamps.numpy().astype(np.uint32), rstamps), f"{what}: stamps differ"
    live = (rtags != oracle.EMPTY_TAG).ravel()
    assert np.array_equal(p.gpu.data().cpu().numpy()[live], rdata[live]), f"{what}: cached rows differ"
    assert p.gpu.stats == p.ref.stats.tolist(), f"{what}: stats differ"


@pytest.mark.parametrize("small_limit", [0, 8192], ids=["general", "fused-small"])
def test_insert_only_calls(small_limit):
    host_rows, dim = 3000, 32
    p = Pair(16, 8, pinned_table(host_rows, dim), small_limit)
    smp = datagen.ZipfSampler(host_rows, 1.2)
    for it in range(6):
        keys = datagen.cache_keys(SEED, 200 + it, host_rows, 700, 1.2, sampler=smp).numpy()
        if it == 3:
            keys[::9] = host_rows + 1
        p.ref.insert(keys)
        p.gpu.insert(to_dev(keys))
        torch.cuda.synchronize()
        _state_equal(p, f"insert {it}")
    p.query(datagen.cache_keys(SEED, 300, host_rows, 400, 1.2, sampler=smp).numpy(), 100, what="query after inserts")


def test_update_then_query_reads_the_new_rows():
    host_rows, dim = 2000, 64
    p = Pair(32, 4, pinned_table(host_rows, dim))
    smp = datagen.ZipfSampler(host_rows, 1.2)
    rng = np.random.default_rng(11)
    for it in range(4):
        p.query(datagen.cache_keys(SEED, 400 + it, host_rows, 600, 1.2, sampler=smp).numpy(), 150, what=f"warm {it}")
    for it in range(3):
        n = [5000, 37, 1][it]
        keys = datagen.cache_keys(SEED, 500 + it, host_rows, n, 1.2, sampler=smp).numpy()   # many repeats
        keys[rng.integers(0, n, max(1, n // 20))] = -7
        rows = rng.standard_normal((n, dim)).astype(np.float32)
        met = p.ref.update(keys, rows)
        p.gpu.update(to_dev(keys), to_dev(rows))
        torch.cuda.synchronize()
        _state_equal(p, f"update {it}")
        assert met > 0 or n == 1
    # a query now mixes updated cached rows (hits) with host rows (misses)
    keys = datagen.cache_keys(SEED, 600, host_rows, 800, 1.2, sampler=smp).numpy()
    ref_out, ref_hit = p.ref.query(keys, 200, insert_missing=False)
    d_hit = torch.zeros(len(keys), dtype=torch.uint8, device="cuda")
    out = p.gpu.query(200, 1, to_dev(keys), None, False, hit_mask=d_hit)
    torch.cuda.synchronize()
    assert np.array_equal(d_hit.cpu().numpy(), ref_hit)
    mag = 4 * np.abs(ref_out) + 1.0
    assert_close(out.cpu().numpy().reshape(200, dim), ref_out, mag, "query after update")


def test_refresh_rereads_the_host_table():
    host_rows, dim = 1500, 16
    host = pinned_table(host_rows, dim)
    p = Pair(20, 4, host)
    smp = datagen.ZipfSampler(host_rows, 1.2)
    for it in range(3):
        p.query(datagen.cache_keys(SEED, 700 + it, host_rows, 500, 1.2, sampler=smp).numpy(), 125, what=f"warm {it}")
    host += 0.25                                   # the level-2 store changes underneath (same memory for both sides)
    p.ref.refresh()
    p.gpu.refresh()
    torch.cuda.synchronize()
    _state_equal(p, "refresh")
    p.query(datagen.cache_keys(SEED, 710, host_rows, 500, 1.2, sampler=smp).numpy(), 125, what="query after refresh")


@pytest.mark.parametrize("small_limit", [0, 8192], ids=["general", "fused-small"])
def test_async_query_signals_results_before_insertion(small_limit):
    host_rows, dim = 4000, 32
    p = Pair(64, 4, pinned_table(host_rows, dim), small_limit)
    keys = datagen.cache_keys(SEED, 800, host_rows, 1040, 1.2).numpy()
    ref_out, ref_hit = p.ref.query(keys, 260, insert_missing=True)
    ready = torch.cuda.Event()
    consumer = torch.cuda.Stream()
    out = p.gpu.query_async(10, 26, to_dev(keys), ready)
    with torch.cuda.stream(consumer):
        consumer.wait_event(ready)
        copy = out.clone()                          # a consumer that only waits for the results
    consumer.synchronize()
    mag = np.abs(p.host.numpy()[keys]).astype(np.float64).reshape(260, 4, dim).sum(1)
    assert_close(copy.cpu().numpy().reshape(260, dim), ref_out, mag, "results seen by the waiting stream")
    torch.cuda.synchronize()
    _state_equal(p, "after async query")


# ---- two-phase query and graph replay -------------------------------------------------------------

def _mag(host, keys, n_bags, offsets=None):
    valid = (keys >= 0) & (keys < host.shape[0])
    bag = (np.repeat(np.arange(n_bags), np.diff(offsets)) if offsets is not None
           else np.arange(len(keys)) // max(1, len(keys) // n_bags))
    mag = np.zeros((n_bags, host.shape[1]))
    np.add.at(mag, bag[valid], np.abs(host.numpy()[keys[valid]]).astype(np.float64))
    return mag


@pytest.mark.parametrize("small_limit", [0, 8192], ids=["general", "fused-small"])
def test_two_phase_query_matches_the_simulation(small_limit):
    """hctr_cache_query_hits + hctr_cache_query_complete against the oracle's pair: after the first
    phase the hit-only pooled rows, the hit mask, the ascending list of missing positions and the
    statistics; after the second (on a side stream that waits for the event) the completed rows and
    the whole cache state; with and without insertion, fixed hotness and CSR bags, keys without a row."""
    host_rows, dim, n_bags, hot = 20000, 64, 26 * 7, 4
    p = Pair(96, 8, pinned_table(host_rows, dim), small_limit)
    smp = datagen.ZipfSampler(host_rows, 1.2)
    side = torch.cuda.Stream()
    ready = torch.cuda.Event()
    ready.record()
    rng = np.random.default_rng(4)
    for it in range(10):
        keys = datagen.cache_keys(SEED, 1200 + it, host_rows, n_bags * hot, 1.2, sampler=smp).numpy()
        if it == 2:
            keys[::15] = -1
            keys[3::40] = host_rows + 11
        offsets = None
        if it % 4 == 3:
            cuts = np.sort(rng.integers(0, len(keys) + 1, n_bags - 1))
            offsets = np.concatenate([[0], cuts, [len(keys)]]).astype(np.int64)
        insert = it % 3 != 2
        d_keys = to_dev(keys)
        d_off = None if offsets is None else to_dev(offsets)
        ref_out, ref_hit, ref_miss = p.ref.query_hits(keys, n_bags, offsets=offsets)
        out = torch.full((n_bags, dim), float("nan"), dtype=torch.float32, device="cuda")
        d_hit = torch.full((len(keys),), 9, dtype=torch.uint8, device="cuda")
        d_miss = torch.full((len(keys),), -1, dtype=torch.int32, device="cuda")
        d_nmiss = torch.full((1,), -1, dtype=torch.int32, device="cuda")
        ws = p.gpu.workspace(len(keys))
        p.gpu.query_hits(n_bags, 1, d_keys, out, d_off, d_hit, d_miss, d_nmiss, ws=ws, ready=ready)
        with torch.cuda.stream(side):
            side.wait_event(ready)
            seen = out.clone()                       # what a consumer sees once the event has fired
        side.synchronize()
        assert np.array_equal(d_hit.cpu().numpy(), ref_hit), f"call {it}: hit mask"
        assert int(d_nmiss.item()) == len(ref_miss), f"call {it}: number of missing positions"
        assert np.array_equal(d_miss.cpu().numpy()[:len(ref_miss)], ref_miss), f"call {it}: missing positions"
        mag = _mag(p.host, keys, n_bags, offsets)
        assert_close(seen.cpu().numpy(), ref_out, mag, f"call {it}: hit-only rows")
        assert p.gpu.stats[:3] == p.ref.stats.tolist()[:3]
        p.ref.query_complete(keys, n_bags, ref_hit, ref_out, offsets=offsets, insert_missing=insert)
        with torch.cuda.stream(side):                # second phase on the side stream, after the event
            p.gpu.query_complete(n_bags, 1, d_keys, out, d_off, insert, ws=ws, stream=side)
        side.synchronize()
        assert_close(out.cpu().numpy(), ref_out, mag, f"call {it}: completed rows")
        no_miss = ~np.isin(np.arange(n_bags), (np.searchsorted(offsets, ref_miss, side="right") - 1) if offsets is not None
                           else ref_miss // hot)
        assert torch.equal(out[torch.from_numpy(no_miss).cuda()], seen[torch.from_numpy(no_miss).cuda()]), \
            f"call {it}: bags without a missing key changed"
        _state_equal(p, f"two-phase call {it}")
    assert p.ref.stats[1] > 0 and p.ref.stats[3] > 0


@pytest.mark.parametrize("small_limit", [0, 8192], ids=["general", "fused-small"])
def test_captured_query_replays_like_eager_calls(small_limit):
    """The call count lives on the device, so a query captured in a HIP graph can be replayed: every
    replay is one more call.  The same graph is replayed on fresh keys (copied into the captured
    buffers between replays, with eager calls and synchronisations in between) and every replay is
    checked against the oracle: hit mask, pooled rows, tags, stamps, cached rows, statistics."""
    host_rows, dim, n_bags, hot = 8000, 32, 26 * 3, 4
    p = Pair(40, 4, pinned_table(host_rows, dim), small_limit)
    smp = datagen.ZipfSampler(host_rows, 1.2)
    n = n_bags * hot
    d_keys = torch.zeros(n, dtype=torch.int64, device="cuda")
    d_hit = torch.zeros(n, dtype=torch.uint8, device="cuda")
    out = torch.zeros((n_bags, dim), dtype=torch.float32, device="cuda")
    ws = p.gpu.workspace(n)

    def fresh(it):
        return datagen.cache_keys(SEED, 1300 + it, host_rows, n, 1.2, sampler=smp).numpy()

    def check(it, keys, what):
        ref_out, ref_hit = p.ref.query(keys, n_bags, insert_missing=True)
        torch.cuda.synchronize()
        assert np.array_equal(d_hit.cpu().numpy(), ref_hit), f"{what} {it}: hit mask"
        assert_close(out.cpu().numpy(), ref_out, _mag(p.host, keys, n_bags), f"{what} {it}: pooled rows")
        _state_equal(p, f"{what} {it}")

    for it in range(2):                              # eagerly first: nothing is set up during capture
        keys = fresh(it)
        d_keys.copy_(torch.from_numpy(keys))
        p.gpu.query(n_bags, 1, d_keys, None, True, out=out, hit_mask=d_hit, ws=ws)
        check(it, keys, "eager")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            p.gpu.query(n_bags, 1, d_keys, None, True, out=out, hit_mask=d_hit, ws=ws, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for it in range(2, 9):
        keys = fresh(it)
        d_keys.copy_(torch.from_numpy(keys))
        if it % 3 == 0:                              # an eager call between replays advances the same count
            p.gpu.query(n_bags, 1, d_keys, None, True, out=out, hit_mask=d_hit, ws=ws)
            check(it, keys, "eager between replays")
            continue
        g.replay()
        check(it, keys, "replay")
    assert p.ref.stats[1] > 0 and p.ref.stats[4] > 0          # hits and evictions happened under replay
