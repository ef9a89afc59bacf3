"""The all-cores variants of the oracle (timed by the benchmark as the CPU baseline) must give the
bits of the single-threaded oracle, which is the one pinned against brute force, torch and numpy
(tests/test_oracle_forward.py, tests/test_oracle_backward.py)."""
import numpy as np
import pytest

import oracle


def problem(seed, n_bags, S, dtype, csr, rows_per_slot=300):
    rng = np.random.default_rng(seed)
    D = 16
    total = S * rows_per_slot
    table = (rng.integers(-2000, 2000, (total, D)) / 1024.0).astype(dtype)
    base = np.arange(S, dtype=np.int64) * rows_per_slot
    num = np.full(S, rows_per_slot, dtype=np.int64)
    if csr:
        hot = rng.integers(0, 9, n_bags)
        offsets = np.concatenate([[0], np.cumsum(hot)]).astype(np.int64)
    else:
        offsets = None
    nnz = int(offsets[-1]) if csr else n_bags
    # skewed keys (long segments), some outside the slot's range
    keys = np.minimum(rng.zipf(1.3, nnz) - 1, rows_per_slot + 3).astype(np.int64)
    keys[rng.random(nnz) < 0.01] = -7
    dY = rng.standard_normal((n_bags, D)).astype(np.float32)
    return table, base, num, keys, offsets, dY


@pytest.mark.parametrize("threads", [2, 3, 8, 37])
@pytest.mark.parametrize("dtype,csr,comb", [(np.float32, False, oracle.SUM), (np.float32, True, oracle.MEAN),
                                            (np.float16, True, oracle.SUM), (np.float16, False, oracle.SUM)])
def test_all_cores_variants_give_the_single_thread_bits(threads, dtype, csr, comb):
    S, n_bags = 5, 5 * 413
    table, base, num, keys, offsets, dY = problem(11 + threads, n_bags, S, dtype, csr)
    r1, bad1 = oracle.rows_direct(base, num, keys, offsets, n_bags)
    rt, badt = oracle.rows_direct(base, num, keys, offsets, n_bags, threads=threads)
    assert bad1 == badt > 0 and np.array_equal(r1, rt)
    o1 = oracle.emb_forward(table, r1, offsets, comb, n_bags)
    ot = oracle.emb_forward(table, r1, offsets, comb, n_bags, threads=threads)
    assert np.array_equal(o1.view(np.uint32), ot.view(np.uint32))
    t1, tt = table.copy(), table.copy()
    u1, c1 = oracle.emb_backward_sgd(t1, r1, dY, 0.05, offsets, comb, n_bags)
    ut, ct = oracle.emb_backward_sgd(tt, r1, dY, 0.05, offsets, comb, n_bags, threads=threads)
    assert np.array_equal(u1, ut) and np.array_equal(c1, ct)
    assert np.array_equal(t1.view(np.uint8), tt.view(np.uint8))
    assert not np.array_equal(t1, table)                       # something was updated


def test_all_cores_variants_on_degenerate_input():
    table = np.ones((4, 8), dtype=np.float32)
    empty = np.zeros(0, dtype=np.int64)
    assert oracle.emb_forward(table, empty, None, oracle.SUM, 0, threads=4).shape == (0, 8)
    u, c = oracle.emb_backward_sgd(table, empty, np.zeros((0, 8), np.float32), 0.1, None, oracle.SUM, 0, threads=4)
    assert len(u) == 0 and len(c) == 0
    # fewer bags than threads
    rows = np.array([1, 1, 3], dtype=np.int64)
    out = oracle.emb_forward(table, rows, None, oracle.SUM, 3, threads=16)
    assert np.array_equal(out, np.ones((3, 8), np.float32))
    assert oracle.hardware_threads() >= 1
