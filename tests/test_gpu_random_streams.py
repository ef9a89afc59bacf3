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
