"""Pins for the oracle's embedding training cache staged in host memory (section 1, "Online
training": subsets of the tables are loaded on demand into the GPU).  The property that matters is
transparency: training through load / train / dump passes leaves the host table exactly as training
on the whole table directly would (checked against the separately pinned backward), plus the
first-appearance row order (against the pinned hash), capacity and range handling by hand."""
import numpy as np

import oracle

RNG = np.random.default_rng(99)


def test_load_rows_follow_first_appearance_and_copy_host_rows():
    host = RNG.standard_normal((50, 8)).astype(np.float32)
    e = oracle.Etc(host, 16)
    keys = np.array([7, 3, 7, 49, 0, 3, 12], dtype=np.int64)
    rows = e.load(keys)
    assert rows.tolist() == [0, 1, 0, 2, 3, 1, 4]                  # by hand
    h = oracle.Hash(16)
    assert np.array_equal(rows, h.insert_or_find(keys, True))     # and as the pinned hash assigns them
    assert np.array_equal(e.work[:5], host[[7, 3, 49, 0, 12]])
    assert e.stats == (5, 5, 0, 0)
    rows2 = e.load([12, 20, 7])                                   # resident keys keep their rows across calls
    assert rows2.tolist() == [4, 5, 0]
    assert e.stats == (6, 6, 0, 0)


def test_capacity_and_range():
    host = RNG.standard_normal((10, 4)).astype(np.float32)
    e = oracle.Etc(host, 3)
    rows = e.load([5, 10, -1, 6, 7, 8, 5, 8, 6])
    assert rows.tolist() == [0, -1, -1, 1, 2, -1, 0, -1, 1]       # 10 and -1 are outside the table; 8 finds no room
    assert e.stats == (3, 3, 2, 2)
    e.dump(evict=True)
    assert e.stats[0] == 0
    assert e.load([8]).tolist() == [0]                            # room again after the eviction


def test_dump_writes_back_and_untouched_rows_keep_their_bits():
    host = RNG.standard_normal((30, 4)).astype(np.float32)
    before = host.copy()
    e = oracle.Etc(host, 8)
    rows = e.load([4, 9, 4, 21])
    e.dump(evict=False)
    assert np.array_equal(host, before)                           # nothing trained: nothing changes
    e.work[rows[1]] += 1.0
    e.dump(evict=True)
    want = before.copy()
    want[9] += 1.0
    assert np.array_equal(host, want)


def test_training_through_the_cache_equals_training_on_the_whole_table():
    host_rows, dim, S, batch = 400, 8, 3, 32
    host = (RNG.standard_normal((host_rows, dim)) * 0.25).astype(np.float32)
    direct = host.copy()
    e = oracle.Etc(host, 300)                                     # room for any pass's distinct keys
    lr = 0.05
    for p in range(5):                                            # passes of 3 batches each
        batches = []
        for _ in range(3):
            h = RNG.integers(0, 4, batch * S)
            offsets = np.concatenate([[0], np.cumsum(h)]).astype(np.int64)
            keys = (RNG.random(offsets[-1]) ** 2 * host_rows).astype(np.int64)
            dY = RNG.standard_normal((batch * S, dim)).astype(np.float32)
            batches.append((keys, offsets, dY))
        e.load(np.concatenate([b[0] for b in batches]))           # the pass's key set
        for keys, offsets, dY in batches:
            rows = e.load(keys)                                   # all resident: plain lookups
            assert (rows >= 0).all()
            oracle.emb_backward_sgd(e.work, rows, dY, lr, offsets, oracle.MEAN)
            oracle.emb_backward_sgd(direct, keys, dY, lr, offsets, oracle.MEAN)
        e.dump(evict=True)
        assert np.array_equal(host, direct), f"pass {p}"
