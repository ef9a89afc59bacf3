"""GPU parity on seeded random call streams: the embedding hash (insert-or-find / find-only calls of
random sizes, repeat rates and key ranges on tables of random capacity, up to and past the row
limit) and the inference cache (random geometry, call sizes on both sides of the fused path's limit,
CSR and fixed-hotness bags, lookup-only and inserting calls, keys outside the host table), each call
compared exactly with the oracle's sequential simulation."""
import os

import numpy as np
import pytest
import torch

from parity import to_dev
from test_gpu_cache import Pair, pinned_table
from test_gpu_hash import both, step

pytestmark = pytest.mark.gpu
SEEDS = range(int(os.environ.get("HCTR_TEST_SEEDS", "8")))   # more seeds for a longer sweep


@pytest.mark.parametrize("seed", SEEDS)
def test_random_hash_stream(seed):
    g = np.random.default_rng(7000 + seed)
    max_rows = int(g.choice([1, 7, 500, 4000, 30000]))
    capacity = int(max(64, max_rows / g.uniform(0.3, 0.8) + 1))   # at least 64 slots, max_rows <= 0.8 * capacity
    gpu, ref = both(capacity, max_rows)
    key_space = int(g.choice([max(2, max_rows // 2), 3 * max_rows + 5, 1 << 62]))
    for call in range(int(g.integers(4, 10))):
        n = int(g.choice([0, 1, 5, 300, 4097, 20000]))
        keys = g.integers(0, key_space, n, dtype=np.int64)
        if n and g.random() < 0.5:      # heavy repeats inside the call
            keys = keys[g.integers(0, max(1, n // 8), n)]
        if n and g.random() < 0.3:
            keys[g.integers(0, n, max(1, n // 50))] = -1 - g.integers(0, 5)   # not keys
        step(gpu, ref, keys, insert=bool(g.random() < 0.75))
    assert gpu.size == ref.size <= max_rows


@pytest.mark.parametrize("seed", SEEDS)
def test_random_cache_stream(seed):
    g = np.random.default_rng(9000 + seed)
    ways = int(g.choice([1, 2, 4, 8, 16, 32, 64]))
    num_sets = int(g.choice([1, 3, 50, 400]))
    dim = int(4 * g.choice([1, 5, 16, 32, 65]))
    host_rows = int(g.choice([10, 700, 6000]))
    small_limit = int(g.choice([0, 300, 8192]))
    p = Pair(num_sets, ways, pinned_table(host_rows, dim), small_limit)
    for call in range(int(g.integers(5, 12))):
        n_bags = int(g.choice([1, 3, 26, 260, 700]))
        if g.random() < 0.5:
            hot = int(g.integers(1, 6))
            offsets, nnz = None, n_bags * hot
        else:
            offsets = np.concatenate([[0], np.cumsum(g.integers(0, 7, n_bags))]).astype(np.int64)
            nnz = int(offsets[-1])
        keys = np.minimum((g.pareto(1.2, nnz) * host_rows / 50).astype(np.int64), host_rows - 1)   # skewed
        if nnz and g.random() < 0.3:
            keys[g.integers(0, nnz, max(1, nnz // 40))] = g.choice([-2, host_rows, host_rows + 9])
        p.query(keys, n_bags, offsets=offsets, insert=bool(g.random() < 0.7), what=f"seed {seed} call {call}")


def _close(got, ref, what):
    # rows may have been replaced by update(): bound the error by the result's own size plus a floor
    err = np.abs(got.astype(np.float64) - ref)
    assert (err <= 1e-5 * (4 * np.abs(ref) + 8.0)).all(), f"{what}: max err {err.max():.3g}"


@pytest.mark.parametrize("seed", SEEDS)
def test_random_cache_operator_stream(seed):
    """One-call queries, two-phase queries, insert-only calls, in-place updates of cached rows and
    refreshes after the host table changed, in random order and sizes (also without any key), on one
    cache; after every operator the tags, stamps, cached rows and statistics equal the simulation's."""
    from test_gpu_cache import _state_equal
    g = np.random.default_rng(11000 + seed)
    ways = int(g.choice([1, 4, 8, 32]))
    num_sets = int(g.choice([2, 31, 200]))
    dim = int(4 * g.choice([2, 16, 32, 65]))
    host_rows = int(g.choice([50, 2000]))
    p = Pair(num_sets, ways, pinned_table(host_rows, dim), int(g.choice([0, 8192])))
    if g.random() < 0.3:
        p.gpu.set_epoch_limit(6)          # stamps are lowered every few calls
        p.ref.set_epoch_limit(6)

    def draw(n):
        k = np.minimum((g.pareto(1.1, n) * host_rows / 40).astype(np.int64), host_rows - 1)
        if n and g.random() < 0.3:
            k[g.integers(0, n, max(1, n // 30))] = g.choice([-4, host_rows, host_rows + 3])
        return k

    for opn in range(int(g.integers(6, 14))):
        op = g.choice(["query", "two_phase", "insert", "update", "refresh"], p=[0.35, 0.25, 0.15, 0.15, 0.10])
        what = f"seed {seed} op {opn} {op}"
        if op in ("query", "two_phase"):
            n_bags = int(g.choice([0, 1, 4, 52, 300]))
            if n_bags and g.random() < 0.5:     # (a call without bags has no hotness: it comes with offsets [0])
                offsets, nnz = None, n_bags * int(g.integers(1, 5))
            else:
                offsets = np.concatenate([[0], np.cumsum(g.integers(0, 5, n_bags))]).astype(np.int64)
                nnz = int(offsets[-1])
            keys = draw(nnz)
            insert = bool(g.random() < 0.7)
            d_keys = to_dev(keys)
            d_off = None if offsets is None else to_dev(offsets)
            d_hit = torch.full((nnz,), 9, dtype=torch.uint8, device="cuda")
            if op == "query":
                ref_out, ref_hit = p.ref.query(keys, n_bags, offsets=offsets, insert_missing=insert)
                out = p.gpu.query(n_bags, 1, d_keys, d_off, insert, hit_mask=d_hit)
                torch.cuda.synchronize()
                assert np.array_equal(d_hit.cpu().numpy(), ref_hit), f"{what}: hit mask"
                _close(out.cpu().numpy().reshape(n_bags, dim), ref_out, what)
            else:
                ref_out, ref_hit, ref_miss = p.ref.query_hits(keys, n_bags, offsets=offsets)
                out = torch.full((n_bags, dim), float("nan"), dtype=torch.float32, device="cuda")
                d_miss = torch.full((max(1, nnz),), -1, dtype=torch.int32, device="cuda")
                d_nmiss = torch.full((1,), -1, dtype=torch.int32, device="cuda")
                ws = p.gpu.workspace(nnz)
                p.gpu.query_hits(n_bags, 1, d_keys, out, d_off, d_hit, d_miss, d_nmiss, ws=ws)
                torch.cuda.synchronize()
                assert np.array_equal(d_hit.cpu().numpy(), ref_hit), f"{what}: hit mask"
                assert int(d_nmiss.item()) == len(ref_miss), f"{what}: number of missing positions"
                assert np.array_equal(d_miss.cpu().numpy()[:len(ref_miss)], ref_miss), f"{what}: missing positions"
                _close(out.cpu().numpy(), ref_out, what + " (hits)")
                p.ref.query_complete(keys, n_bags, ref_hit, ref_out, offsets=offsets, insert_missing=insert)
                p.gpu.query_complete(n_bags, 1, d_keys, out, d_off, insert, ws=ws)
                torch.cuda.synchronize()
                _close(out.cpu().numpy(), ref_out, what + " (completed)")
        elif op == "insert":
            keys = draw(int(g.choice([0, 1, 40, 900, 9000])))
            p.ref.insert(keys)
            p.gpu.insert(to_dev(keys))
        elif op == "update":
            n = int(g.choice([0, 1, 60, 3000]))
            keys = draw(n)
            rows = g.standard_normal((n, dim)).astype(np.float32)
            p.ref.update(keys, rows)
            p.gpu.update(to_dev(keys), to_dev(rows))
        else:
            p.host += 0.125               # the host table changes underneath (one memory for both sides)
            p.ref.refresh()
            p.gpu.refresh()
        torch.cuda.synchronize()
        _state_equal(p, what)


def _hashed_cases(n, seed):
    g = np.random.default_rng(seed)
    out = []
    for i in range(n):
        S = int(g.choice([1, 3, 26]))
        dim = int(4 * g.choice([1, 4, 16, 25, 64]))
        batch = int(g.choice([1, 40, 513, 1500]))
        max_rows = int(g.choice([5, 300, 4000, 30000]))
        capacity = int(max(64, max_rows / g.uniform(0.35, 0.8) + 1))
        out.append(pytest.param(S, dim, batch, capacity, max_rows, bool(g.random() < 0.5), int(g.integers(1, 5)), 13000 + i,
                                float(g.choice([1.05, 1.5])), id=f"{i}-S{S}-D{dim}-B{batch}-rows{max_rows}"))
    return out


@pytest.mark.parametrize("S,dim,batch,capacity,max_rows,reuse,steps,seed,alpha",
                         _hashed_cases(int(os.environ.get("HCTR_TEST_SEEDS", "8")) * 2, 20221011))
def test_random_hashed_layer(S, dim, batch, capacity, max_rows, reuse, steps, seed, alpha):
    """The layer in hashed mode (insert on miss in the forward, the forward's rows reused by the backward
    or looked up again) on random shapes, with tables that fill up during the steps."""
    from test_gpu_hash import check_hashed_layer
    check_hashed_layer(S, dim, batch, capacity, max_rows, reuse, steps, seed, alpha=alpha)


@pytest.mark.parametrize("seed", SEEDS)
def test_random_training_cache_stream(seed):
    """The staged training cache: load calls of random sizes (also empty, with keys outside the host
    table), working rows changed on the device in between, dumps with and without eviction; rows,
    statistics, working table and host table equal the simulation's after every call."""
    import oracle
    import paper_2210_08803_amd as H
    from test_gpu_etc import pinned
    g = np.random.default_rng(15000 + seed)
    host_rows = int(g.choice([9, 400, 7000]))
    dim = int(4 * g.choice([1, 8, 33]))
    max_rows = int(g.choice([1, 50, 3000]))
    host_np = g.standard_normal((host_rows, dim)).astype(np.float32)
    host = pinned(host_np)
    etc = H.EmbeddingTrainingCache(host, max_rows=max_rows)
    ref = oracle.Etc(host_np.copy(), max_rows)
    for call in range(int(g.integers(4, 12))):
        op = g.choice(["load", "load", "load", "touch", "dump", "dump_evict"])
        what = f"seed {seed} call {call} {op}"
        if op == "load":
            n = int(g.choice([0, 1, 30, 700, 5000]))
            keys = (g.random(n) ** 2 * host_rows * 1.05).astype(np.int64)          # a few past the end
            if n and g.random() < 0.4:
                keys[g.integers(0, n, max(1, n // 25))] = g.choice([-1, -2 ** 62, 2 ** 40])
            rows = torch.full((max(1, n),), -7, dtype=torch.int64, device="cuda")
            etc.load(to_dev(keys), rows[:n] if n else None)
            want = ref.load(keys)
            assert np.array_equal(rows.cpu().numpy()[:n], want), what
        elif op == "touch":               # training changes working rows: the same change on both sides
            n = ref.stats[0]
            if n:
                etc.table[:n] += 0.5
                ref.work[:n] += np.float32(0.5)
        else:
            etc.dump(evict=(op == "dump_evict"))
            ref.dump(evict=(op == "dump_evict"))
        torch.cuda.synchronize()
        assert etc.stats == ref.stats, what
        n = ref.stats[0]
        assert np.array_equal(etc.table[:n].cpu().numpy(), ref.work[:n]), what
        assert np.array_equal(host.numpy(), ref.host), what
