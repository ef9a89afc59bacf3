"""GPU parity of the fused group of lookups (hctr_group_forward / hctr_group_backward_sgd) against
the oracle: tables of different widths, sum and mean, shared tables, sparse (CSR) and dense input,
fp32 and fp16 storage, keys outside their table, hot rows that span many reduction windows."""
import numpy as np
import pytest
import torch

import oracle
import paper_2210_08803_amd as H
from parity import assert_close, to_dev, RTOL

pytestmark = pytest.mark.gpu


def make_group(rng, table_shapes, lookups, dtype):
    tables = [(rng.standard_normal(s) * 0.25).astype(dtype) for s in table_shapes]
    lt = np.array([l[0] for l in lookups], dtype=np.int32)
    lc = np.array([l[1] for l in lookups], dtype=np.int32)
    return tables, lt, lc


def make_keys(rng, table_shapes, lt, batch, offsets, zipf=False, bad=0):
    L = len(lt)
    lens = np.diff(offsets)
    lookup_of_key = np.repeat(np.arange(batch * L) % L, lens)
    rows_of_key = np.array([table_shapes[t][0] for t in lt])[lookup_of_key]
    u = rng.random(len(lookup_of_key))
    if zipf:
        u = u ** 6          # most keys near row 0: rows with thousands of occurrences
    keys = np.minimum((u * rows_of_key).astype(np.int64), rows_of_key - 1)
    if bad:
        pos = rng.choice(len(keys), size=bad, replace=False)
        keys[pos[: bad // 2]] = -1 - rng.integers(0, 5, bad // 2)
        keys[pos[bad // 2:]] = rows_of_key[pos[bad // 2:]] + rng.integers(0, 5, bad - bad // 2)
    return keys


def run_case(rng, table_shapes, lookups, batch, dtype, hmax=None, hot=None, zipf=False, bad=0, lr=0.05):
    tables, lt, lc = make_group(rng, table_shapes, lookups, dtype)
    L = len(lt)
    if hot is not None:     # dense input
        offsets = oracle.dense_offsets(batch, hot)
    else:
        offsets = np.concatenate([[0], np.cumsum(rng.integers(0, hmax + 1, batch * L))]).astype(np.int64)
    keys = make_keys(rng, table_shapes, lt, batch, offsets, zipf, bad)
    width = int(sum(table_shapes[t][1] for t in lt))
    dY = rng.standard_normal((batch, width)).astype(np.float32)

    dev_tables = [to_dev(t) for t in tables]
    spec = [(int(t), int(c), int(hot[i]) if hot is not None else 1) for i, (t, c) in enumerate(zip(lt, lc))]
    g = H.EmbeddingGroup(dev_tables, spec)
    dkeys = to_dev(keys)
    doff = None if hot is not None else to_dev(offsets)

    # forward
    out = g.forward(batch, dkeys, doff).cpu().numpy()
    ref = oracle.group_forward(tables, lt, lc, batch, keys, offsets)
    mag = oracle.group_forward([np.abs(t) for t in tables], lt, lc, batch, keys, offsets)
    assert_close(out, ref, mag, "group forward")
    assert g.invalid_keys() == bad

    # backward
    ref_tables = [t.copy() for t in tables]
    touched = oracle.group_backward_sgd(ref_tables, lt, lc, batch, keys, offsets, dY, lr)
    g_abs = [np.zeros(t.shape, dtype=np.float32) for t in tables]
    oracle.group_backward_sgd(g_abs, lt, lc, batch, keys, offsets, np.abs(dY), -1.0)   # += sum |w dY|
    g.backward_sgd(batch, dkeys, to_dev(dY), lr, doff)
    assert g.invalid_keys() == 2 * bad
    lookup_of_key = np.repeat(np.arange(batch * L) % L, np.diff(offsets))
    n_pairs = 0
    for ti, (t0, tr, ga, dt) in enumerate(zip(tables, ref_tables, g_abs, dev_tables)):
        got = dt.cpu().numpy()
        k = keys[lt[lookup_of_key] == ti]
        named = np.unique(k[(k >= 0) & (k < t0.shape[0])])
        n_pairs += len(named)
        rest = np.setdiff1d(np.arange(t0.shape[0]), named)
        assert np.array_equal(got[rest].view(np.uint8), t0[rest].view(np.uint8)), f"table {ti}: untouched rows changed"
        magn = np.abs(t0[named].astype(np.float64)) + lr * ga[named].astype(np.float64)
        if dtype == np.float16:
            r = tr[named].astype(np.float64)
            ulp = np.spacing(np.abs(tr[named]).astype(np.float16)).astype(np.float64)
            tol = np.maximum(ulp, RTOL * np.maximum(np.abs(r), magn / 8.0))
            assert (np.abs(got[named].astype(np.float64) - r) <= tol).all(), f"table {ti}: fp16 rows off"
        else:
            assert_close(got[named], tr[named], magn, f"group backward, table {ti}")
    assert touched == n_pairs


SHAPES = [(1000, 16), (37, 128), (5000, 64), (300, 8), (64, 256)]
LOOKUPS = [(0, H.SUM), (1, H.MEAN), (2, H.SUM), (1, H.SUM), (3, H.MEAN), (4, H.SUM), (2, H.MEAN)]


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_group_sparse_input_mixed_widths_shared_tables(dtype):
    run_case(np.random.default_rng(11), SHAPES, LOOKUPS, batch=613, dtype=dtype, hmax=9, bad=24)


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_group_dense_input(dtype):
    run_case(np.random.default_rng(12), SHAPES, LOOKUPS, batch=777, dtype=dtype, hot=[1, 3, 1, 2, 5, 1, 4])


def test_group_all_one_hot_dense():
    run_case(np.random.default_rng(13), SHAPES, LOOKUPS, batch=2049, dtype=np.float32, hot=[1] * 7, bad=10)


def test_group_hot_rows_span_many_windows():
    # a few rows collect tens of thousands of occurrences: long carries, both carry kernels
    run_case(np.random.default_rng(14), [(50, 32), (2000, 128), (9, 8)], [(0, H.SUM), (1, H.MEAN), (2, H.SUM), (1, H.SUM)],
             batch=4096, dtype=np.float32, hmax=6, zipf=True)


def test_group_wide_rows_need_column_chunks():
    run_case(np.random.default_rng(15), [(40, 512), (100, 24)], [(0, H.MEAN), (1, H.SUM)], batch=300,
             dtype=np.float32, hmax=4)


def test_group_single_lookup_equals_layer():
    # one table, one lookup: the group and the plain layer must agree bit for bit in forward
    rng = np.random.default_rng(16)
    table = (rng.standard_normal((500, 64)) * 0.25).astype(np.float32)
    keys = rng.integers(0, 500, 1000)
    dt = to_dev(table)
    g = H.EmbeddingGroup([dt], [(0, H.SUM, 1)])
    layer = H.EmbeddingLayer(dt, 1, H.SUM, [0], [500])
    dk = to_dev(keys)
    assert torch.equal(g.forward(1000, dk), layer.forward(1000, dk).view(1000, 64))


def test_group_empty_calls():
    rng = np.random.default_rng(17)
    tables, lt, lc = make_group(rng, SHAPES, LOOKUPS, np.float32)
    g = H.EmbeddingGroup([to_dev(t) for t in tables], [(int(t), int(c), 1) for t, c in zip(lt, lc)])
    empty = torch.empty(0, dtype=torch.int64, device="cuda")
    out = g.forward(0, empty)
    assert out.shape == (0, g.width)
    # samples whose bags are all empty: zeros out, tables untouched
    off = torch.zeros(5 * len(lt) + 1, dtype=torch.int64, device="cuda")
    out = g.forward(5, empty, off)
    assert torch.count_nonzero(out) == 0
    g.backward_sgd(5, empty, torch.ones((5, g.width), device="cuda"), 0.1, off)
    for t, dtab in zip(tables, g.tables):
        assert np.array_equal(dtab.cpu().numpy(), t)


def test_group_is_deterministic():
    rng = np.random.default_rng(18)
    shapes = [(50, 32), (2000, 128), (9, 8)]
    lookups = [(0, H.SUM, 1), (1, H.MEAN, 1), (2, H.SUM, 1), (1, H.SUM, 1)]
    tables = [(rng.standard_normal(s) * 0.25).astype(np.float32) for s in shapes]
    batch, L = 3000, len(lookups)
    offsets = np.concatenate([[0], np.cumsum(rng.integers(0, 7, batch * L))]).astype(np.int64)
    keys = make_keys(rng, shapes, np.array([l[0] for l in lookups]), batch, offsets, zipf=True)
    dY = rng.standard_normal((batch, 32 + 128 + 8 + 128)).astype(np.float32)
    results = []
    for _ in range(2):
        dev = [to_dev(t) for t in tables]
        g = H.EmbeddingGroup(dev, lookups)
        out = g.forward(batch, to_dev(keys), to_dev(offsets))
        g.backward_sgd(batch, to_dev(keys), to_dev(dY), 0.05, to_dev(offsets))
        results.append((out, dev))
    assert torch.equal(results[0][0], results[1][0])
    for a, b in zip(results[0][1], results[1][1]):
        assert torch.equal(a, b)
