"""Pins for the oracle's inference cache (section 3, "embedding inference cache", "Volatile
database"): a hand-worked trace, the textbook structures it must reduce to (direct-mapped for
one way, classical LRU for one set and one key per call), and state invariants."""
import json
import os
from collections import OrderedDict

import numpy as np

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden", "cache_batch_lru_trace.json")
RNG = np.random.default_rng(77)
M64 = (1 << 64) - 1


def host_table(rows, dim):
    return (np.arange(rows, dtype=np.float32)[:, None] + np.arange(dim, dtype=np.float32)[None, :] / 128).copy()


def set_of(key, num_sets):
    """The frozen set-index rule, in Python integers."""
    x = (key * 0x9E3779B97F4A7C15) & M64
    x ^= x >> 32
    return x % num_sets


def test_hand_worked_trace():
    g = json.load(open(GOLD))
    ht = host_table(g["host_rows"], g["dim"])
    c = oracle.Cache(g["num_sets"], g["ways"], ht)
    for call in g["calls"]:
        keys = np.array(call["keys"], dtype=np.int64)
        out, hit = c.query(keys, call["n_bags"], insert_missing=bool(call["insert"]))
        assert hit.tolist() == call["hit"]
        tags, stamps = c.state()
        assert tags[0].tolist() == call["tags"] and stamps[0].tolist() == call["stamps"]
        assert c.stats.tolist() == call["stats"]
        hot = len(keys) // call["n_bags"]
        ref = ht[keys].astype(np.float64).reshape(call["n_bags"], hot, -1).sum(1).astype(np.float32)
        assert np.array_equal(out, ref)


def test_one_way_is_a_direct_mapped_cache():
    num_sets, ht = 13, host_table(500, 4)
    c = oracle.Cache(num_sets, 1, ht)
    slot = {}                                             # textbook direct-mapped: set -> resident key
    for _ in range(300):
        k = int(RNG.integers(0, 500))
        _, hit = c.query(np.array([k]), 1)
        s = set_of(k, num_sets)
        assert bool(hit[0]) == (slot.get(s) == k)
        slot[s] = k
    tags, _ = c.state()
    for s in range(num_sets):
        assert tags[s, 0] == (slot[s] if s in slot else oracle.EMPTY_TAG)


def test_one_set_one_key_per_call_is_classical_lru():
    ways, ht = 5, host_table(40, 4)
    c = oracle.Cache(1, ways, ht)
    lru = OrderedDict()
    for _ in range(500):
        k = int(RNG.integers(0, 12))
        _, hit = c.query(np.array([k]), 1)
        assert bool(hit[0]) == (k in lru)
        if k in lru:
            lru.move_to_end(k)
        else:
            if len(lru) == ways:
                lru.popitem(last=False)
            lru[k] = True
        tags, _ = c.state()
        assert sorted(t for t in tags[0].tolist() if t != int(oracle.EMPTY_TAG)) == sorted(lru)


def test_big_enough_cache_misses_each_key_exactly_once():
    ht = host_table(300, 8)
    keys_all = RNG.permutation(300)[:64]
    num_sets, ways = 64, 8
    load = np.bincount([set_of(int(k), num_sets) for k in keys_all], minlength=num_sets)
    assert load.max() <= ways                             # no set overflows, so nothing is ever evicted
    c = oracle.Cache(num_sets, ways, ht)
    seen = set()
    for _ in range(20):
        keys = keys_all[RNG.integers(0, 64, 48)]
        out, hit = c.query(keys, 12)
        assert hit.tolist() == [int(k in seen) for k in keys.tolist()]
        seen.update(keys.tolist())
        ref = ht[keys].astype(np.float64).reshape(12, 4, -1).sum(1).astype(np.float32)
        assert np.array_equal(out, ref)                   # output never depends on cache state
    assert c.stats[4] == 0 and c.stats[5] == 0 and c.stats[3] == len(seen)


def test_state_invariants_under_pressure():
    ht = host_table(2000, 4)
    c = oracle.Cache(16, 4, ht)
    offsets = None
    for it in range(30):
        h = RNG.integers(0, 6, 40)
        offsets = np.concatenate([[0], np.cumsum(h)])
        keys = RNG.zipf(1.3, offsets[-1]) % 2000
        keys[RNG.integers(0, len(keys), 2)] = [-5, 2000]  # keys outside the host table: zero rows, never cached
        before_tags, _ = c.state()
        s0 = c.stats
        out, hit = c.query(keys, 40, offsets=offsets, insert_missing=(it % 3 != 2))
        s1 = c.stats
        tags, stamps = c.state()
        assert s1[0] - s0[0] == len(keys) and (s1[1] - s0[1]) + (s1[2] - s0[2]) == len(keys)
        assert s1[1] - s0[1] == hit.sum()
        for s in range(16):
            live = [t for t in tags[s].tolist() if t != int(oracle.EMPTY_TAG)]
            assert len(live) == len(set(live))            # no duplicate tag in a set
            assert all(set_of(t, 16) == s for t in live)  # every tag lives in its own set
            assert all(0 <= t < 2000 for t in live)
        valid = (keys >= 0) & (keys < 2000)
        ref = np.zeros((40, 4))
        np.add.at(ref, np.repeat(np.arange(40), h)[valid], ht[keys[valid]].astype(np.float64))
        assert np.array_equal(out, ref.astype(np.float32))
        if it % 3 == 2:
            assert np.array_equal(tags, before_tags)      # no insertion requested: tags unchanged
        # a key classified as hit was resident at entry; all occurrences of a key agree
        resident = set(before_tags.ravel().tolist())
        assert hit.tolist() == [int(int(k) in resident and k >= 0) for k in keys.tolist()]
        assert s1[3] - s0[3] >= s1[4] - s0[4]


def test_set_index_spreads_scrambled_keys_evenly():
    num_sets = 257
    keys = (np.arange(50000, dtype=np.uint64) * np.uint64(7919)) % np.uint64(10**9)
    cnt = np.bincount([set_of(int(k), num_sets) for k in keys], minlength=num_sets)
    chi2 = ((cnt - 50000 / num_sets) ** 2 / (50000 / num_sets)).sum()
    assert chi2 < 2 * num_sets


# ---- manipulation operators (section 3: "query and manipulation operators", refresh; "Online model
# ---- updating": cached embeddings are replaced when updates arrive)

def test_insert_is_a_query_without_output():
    ht = host_table(400, 4)
    a, b = oracle.Cache(8, 2, ht), oracle.Cache(8, 2, ht)
    for _ in range(12):
        keys = RNG.integers(0, 60, 40)
        a.query(keys, 40)
        b.insert(keys)
        ta, sa = a.state(); tb, sb = b.state()
        assert np.array_equal(ta, tb) and np.array_equal(sa, sb) and np.array_equal(a.stats, b.stats)


def test_update_replaces_resident_rows_only_and_last_row_wins():
    ht = host_table(64, 4)
    c = oracle.Cache(1, 4, ht)
    c.query(np.array([3, 5, 7]), 3)                       # resident: 3, 5, 7 in ways 0, 1, 2
    before_tags, before_stamps = c.state()
    s0 = c.stats.copy()
    rows = np.arange(5 * 4, dtype=np.float32).reshape(5, 4) + 1000
    met = c.update(np.array([5, 9, 3, 5, -1]), rows)      # 9 and -1 are not resident; 5 comes twice
    assert met == 3
    tags, stamps, data = c.state(with_data=True)
    assert np.array_equal(tags, before_tags) and np.array_equal(stamps, before_stamps) and np.array_equal(c.stats, s0)
    assert np.array_equal(data[0], rows[2])               # key 3 <- its only row
    assert np.array_equal(data[1], rows[3])               # key 5 <- the later of its two rows
    assert np.array_equal(data[2], ht[7])                 # key 7 untouched
    out, hit = c.query(np.array([5, 9, 3, 7]), 1, insert_missing=False)   # one bag of four keys
    assert hit.tolist() == [1, 0, 1, 1]
    want = (rows[3].astype(np.float64) + ht[9] + rows[2] + ht[7]).astype(np.float32)
    assert np.array_equal(out[0], want)                   # hits read the cache, the miss reads the host table


def test_refresh_rereads_every_resident_row_from_the_host_table():
    ht = host_table(64, 4)
    c = oracle.Cache(4, 2, ht)
    c.query(np.arange(10), 10)
    tags0, stamps0 = c.state()
    ht[:] += 0.5                                          # the level-2 store changed underneath the cache
    _, _, stale = c.state(with_data=True)
    live = (tags0 != oracle.EMPTY_TAG).ravel()
    assert not np.array_equal(stale[live], ht[tags0.ravel()[live].astype(np.int64)])
    c.refresh()
    tags, stamps, data = c.state(with_data=True)
    assert np.array_equal(tags, tags0) and np.array_equal(stamps, stamps0)
    assert np.array_equal(data[live], ht[tags.ravel()[live].astype(np.int64)])
    assert np.all(data[~live] == 0)                       # empty lines are left alone


def test_epoch_limit_hand_worked():
    """One set of three ways, limit 4: a call that finds the count at 4 first lowers stamps and count
    by 2 (stamps <= 2 become 0).  Expected states worked out by hand; E = empty."""
    E = int(oracle.EMPTY_TAG)
    c = oracle.Cache(1, 3, host_table(10, 4))
    c.set_epoch_limit(4)
    steps = [  # key, hit, tags, stamps, count after the call
        (1, 0, [1, E, E], [1, 0, 0], 1),
        (2, 0, [1, 2, E], [1, 2, 0], 2),
        (2, 1, [1, 2, E], [1, 3, 0], 3),
        (2, 1, [1, 2, E], [1, 4, 0], 4),
        (3, 0, [1, 2, 3], [0, 2, 3], 3),   # lowered first: [0, 2, 0], count 2 -> 3; key 3 takes the empty way
        (4, 0, [4, 2, 3], [4, 2, 3], 4),   # no empty way: the smallest stamp (way 0) goes
        (5, 0, [4, 5, 3], [2, 3, 1], 3),   # lowered first: [2, 0, 1], count 2 -> 3; way 1 goes
        (1, 0, [4, 5, 1], [2, 3, 4], 4),   # way 2 (stamp 1) was the oldest: the order survived the lowering
    ]
    for key, hit, tags, stamps, count in steps:
        _, h = c.query(np.array([key]), 1)
        t, s = c.state()
        assert (int(h[0]), t[0].tolist(), s[0].tolist(), c.epoch) == (hit, tags, stamps, count)


def test_epoch_limit_leaves_classical_lru_intact():
    """The count passes a limit of 64 many times in 600 calls; every resident key was used within the
    last 32 calls (5 ways, 12 keys), so no stamp ever collapses and the cache must still be the
    textbook LRU - it would not be if the lowering lost the order or froze the replacement."""
    ways, ht = 5, host_table(40, 4)
    c = oracle.Cache(1, ways, ht)
    c.set_epoch_limit(64)
    rng = np.random.default_rng(5)
    lru = OrderedDict()
    top = 0
    for _ in range(600):
        k = int(rng.integers(0, 12))
        _, hit = c.query(np.array([k]), 1)
        assert bool(hit[0]) == (k in lru)
        if k in lru:
            lru.move_to_end(k)
        else:
            if len(lru) == ways:
                lru.popitem(last=False)
            lru[k] = True
        tags, stamps = c.state()
        assert sorted(t for t in tags[0].tolist() if t != int(oracle.EMPTY_TAG)) == sorted(lru)
        assert c.epoch <= 64 and stamps.max() <= c.epoch
        top = max(top, c.epoch)
    assert top == 64


# ---- two-phase query: hits first, missing rows added afterwards (oracle_cache_query_hits / _complete)

def _traffic(host_rows, n_calls, n_bags, hot, seed):
    rng = np.random.default_rng(seed)
    for it in range(n_calls):
        keys = np.minimum(rng.zipf(1.3, n_bags * hot) - 1, host_rows + 2).astype(np.int64)   # some outside the table
        keys = (keys * 7919) % (host_rows + 3)
        if it % 3 == 1:
            keys[::11] = -4
        yield it, keys


def test_two_phase_query_leaves_the_state_of_the_single_call():
    """Hits then complete = the one-call query, which the trace and the textbook cases above pin:
    same hit mask, tags, stamps, cached rows, statistics and call count after every call, with and
    without insertion, fixed hotness and CSR bags, also across the lowering of the call count."""
    host_rows, dim = 400, 8
    ht = host_table(host_rows, dim)
    for limit in (None, 7):
        one, two = oracle.Cache(6, 4, ht), oracle.Cache(6, 4, ht)
        if limit:
            one.set_epoch_limit(limit)
            two.set_epoch_limit(limit)
        for it, keys in _traffic(host_rows, 30, 12, 5, 3):
            insert = it % 4 != 2
            offsets = None
            if it % 5 == 4:   # ragged bags, an empty one among them
                cuts = np.sort(np.random.default_rng(it).integers(0, len(keys) + 1, 11))
                offsets = np.concatenate([[0], cuts, [len(keys)]]).astype(np.int64)
            ref_out, ref_hit = one.query(keys, 12, offsets=offsets, insert_missing=insert)
            out, hit, miss = two.query_hits(keys, 12, offsets=offsets)
            assert np.array_equal(hit, ref_hit)
            assert np.array_equal(miss, np.flatnonzero((hit == 0) & (keys >= 0) & (keys < host_rows)))
            assert one.stats[:3].tolist() == two.stats[:3].tolist() and one.epoch == two.epoch
            two.query_complete(keys, 12, hit, out, offsets=offsets, insert_missing=insert)
            for a, b in zip(one.state(with_data=True), two.state(with_data=True)):
                assert np.array_equal(a, b), f"call {it}"
            assert one.stats.tolist() == two.stats.tolist()
            # rows of this table are multiples of 1/128 below 2^9: every sum is exact in fp32, so the
            # two-phase result must equal the one-call result bit for bit
            assert np.array_equal(out, ref_out), f"call {it}"


def test_two_phase_outputs_are_the_sums_over_hits_and_over_misses():
    host_rows, dim, n_bags, hot = 300, 4, 9, 6
    rng = np.random.default_rng(5)
    ht = rng.standard_normal((host_rows, dim)).astype(np.float32)
    c = oracle.Cache(5, 2, ht)
    for it, keys in _traffic(host_rows, 12, n_bags, hot, 9):
        out, hit, miss = c.query_hits(keys, n_bags)
        valid = (keys >= 0) & (keys < host_rows)
        rows = np.where(valid[:, None], ht[np.clip(keys, 0, host_rows - 1)].astype(np.float64), 0.0)
        hits_sum = (rows * (hit == 1)[:, None]).reshape(n_bags, hot, dim).sum(1)
        assert np.array_equal(out, hits_sum.astype(np.float32))           # cached rows are copies of host rows
        miss_sum = (rows * (hit == 0)[:, None]).reshape(n_bags, hot, dim).sum(1)
        phase1 = out.copy()
        c.query_complete(keys, n_bags, hit, out, insert_missing=(it % 2 == 0))
        want = (phase1.astype(np.float64) + miss_sum).astype(np.float32)
        has_miss = ((hit == 0) & valid).reshape(n_bags, hot).any(1)
        assert np.array_equal(out[has_miss], want[has_miss])
        assert np.array_equal(out[~has_miss].view(np.uint32), phase1[~has_miss].view(np.uint32))   # untouched bits
        full = (hits_sum + miss_sum)
        assert np.all(np.abs(out - full) <= 2.0 ** -23 * np.abs(rows).reshape(n_bags, hot, dim).sum(1) + 1e-30)


def test_two_phase_extremes():
    ht = host_table(50, 4)
    c = oracle.Cache(8, 4, ht)
    keys = np.arange(20, dtype=np.int64)
    out, hit, miss = c.query_hits(keys, 5)                    # cold cache: nothing hits
    assert not out.any() and not hit.any() and np.array_equal(miss, np.arange(20))
    c.query_complete(keys, 5, hit, out, insert_missing=True)
    assert np.array_equal(out, ht[keys].reshape(5, 4, 4).sum(1))
    assert c.stats.tolist() == [20, 0, 20, 20, 0, 0]
    out, hit, miss = c.query_hits(keys, 5)                    # warm: everything hits, nothing to complete
    assert hit.all() and len(miss) == 0 and np.array_equal(out, ht[keys].reshape(5, 4, 4).sum(1))
    before = out.copy()
    state = [a.copy() for a in c.state(with_data=True)]
    c.query_complete(keys, 5, hit, out, insert_missing=True)
    assert np.array_equal(out.view(np.uint32), before.view(np.uint32))
    assert all(np.array_equal(a, b) for a, b in zip(state, c.state(with_data=True)))
    assert c.stats.tolist() == [40, 20, 20, 20, 0, 0]
