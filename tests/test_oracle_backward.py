"""Pins for the oracle's backward + SGD (forward/backward through the embedding: section 1,
"Hybrid sparse embedding"; the SGD rule and dedup come from the benchmark definition).  Checked
against a dense matrix form, torch autograd, numpy.unique and the conservation invariants."""
import numpy as np
import pytest
import torch

import datagen
import oracle

RNG = np.random.default_rng(99)


def _case(total_rows=23, n_bags=17, dim=6, hmax=6, dtype=np.float32):
    table = (RNG.standard_normal((total_rows, dim)) * 0.25).astype(dtype)
    h = RNG.integers(0, hmax + 1, n_bags)
    offsets = np.concatenate([[0], np.cumsum(h)]).astype(np.int64)
    rows = RNG.integers(0, total_rows // 2, offsets[-1])  # upper half of the table stays untouched
    dY = RNG.standard_normal((n_bags, dim)).astype(np.float32)
    return table, offsets, rows, dY


def _dense_M(rows, offsets, n_bags, total_rows, mean):
    M = np.zeros((n_bags, total_rows))
    for bag in range(n_bags):
        h = offsets[bag + 1] - offsets[bag]
        for i in range(offsets[bag], offsets[bag + 1]):
            if 0 <= rows[i] < total_rows:
                M[bag, rows[i]] += (1.0 / h) if mean else 1.0
    return M


@pytest.mark.parametrize("combiner", [oracle.SUM, oracle.MEAN])
def test_backward_equals_dense_form(combiner):
    table, offsets, rows, dY = _case()
    rows = rows.copy(); rows[3] = -1
    lr = np.float32(0.01)
    M = _dense_M(rows, offsets, len(offsets) - 1, len(table), combiner == oracle.MEAN)
    ref = table.astype(np.float64) - float(lr) * (M.T @ dY.astype(np.float64))
    before = table.copy()
    t = table.copy()
    uniq, cnt = oracle.emb_backward_sgd(t, rows, dY, lr, offsets, combiner)
    touched = np.zeros(len(table), bool); touched[uniq] = True
    np.testing.assert_allclose(t[touched], ref[touched], rtol=1e-7, atol=1e-9)
    assert np.array_equal(t[~touched], before[~touched])            # untouched rows: same bits
    assert touched[len(table) // 2:].sum() == 0
    vu, vc = np.unique(rows[rows >= 0], return_counts=True)        # dedup vs numpy
    assert np.array_equal(uniq, vu) and np.array_equal(cnt, vc)


@pytest.mark.parametrize("mode,combiner", [("sum", oracle.SUM), ("mean", oracle.MEAN)])
def test_backward_against_torch_autograd(mode, combiner):
    table, offsets, rows, dY = _case(hmax=5)
    keep = np.diff(offsets) > 0                                     # torch's mean of an empty bag is not ours
    w = torch.from_numpy(table).double().requires_grad_(True)
    out = torch.nn.functional.embedding_bag(torch.from_numpy(rows), w, torch.from_numpy(offsets),
                                            mode=mode, include_last_offset=True)
    out.backward(torch.from_numpy(dY).double() * torch.from_numpy(keep)[:, None])
    ref = (w.detach() - 0.05 * w.grad).numpy()
    t = table.copy()
    oracle.emb_backward_sgd(t, rows, dY, 0.05, offsets, combiner)
    np.testing.assert_allclose(t, ref, rtol=1e-6, atol=1e-7)       # lr=0.05 is inexact in fp32: ~1e-8 rel


@pytest.mark.parametrize("combiner", [oracle.SUM, oracle.MEAN])
def test_gradient_mass_is_conserved(combiner):
    """sum over rows of (T_before - T_after)/lr == sum over bags of (#valid keys * w_bag) * dY[bag]."""
    table, offsets, rows, dY = _case(total_rows=40, n_bags=64, dim=4)
    t64 = table.astype(np.float64)
    t = table.copy()
    lr = np.float32(0.5)  # power of two: the only rounding is the final store
    oracle.emb_backward_sgd(t, rows, dY, lr, offsets, combiner)
    applied = ((t64 - t.astype(np.float64)) / 0.5).sum(0)
    h = np.diff(offsets)
    w = np.where(h > 0, 1.0 / np.maximum(h, 1), 0.0) if combiner == oracle.MEAN else np.ones(len(h))
    scattered = ((h * w)[:, None] * dY.astype(np.float64)).sum(0)
    np.testing.assert_allclose(applied, scattered, rtol=0, atol=40 * 2.0**-24)


def test_identity_cases():
    table, offsets, rows, dY = _case()
    t = table.copy(); oracle.emb_backward_sgd(t, rows, dY, 0.0, offsets)
    assert np.array_equal(t, table)                                  # lr = 0
    t = table.copy(); oracle.emb_backward_sgd(t, rows, np.zeros_like(dY), 0.3, offsets)
    assert np.array_equal(t, table)                                  # dY = 0
    t = table.copy(); u, c = oracle.emb_backward_sgd(t, np.full_like(rows, -1), dY, 0.3, offsets)
    assert np.array_equal(t, table) and len(u) == 0                  # no key has a row
    t = table.copy(); u, c = oracle.emb_backward_sgd(t, np.zeros(0, np.int64), dY[:0], 0.3, np.zeros(1, np.int64))
    assert len(u) == 0                                               # empty batch


def test_repeated_key_in_one_bag_counts_per_occurrence():
    table = np.zeros((4, 2), np.float32)
    rows = np.array([2, 2, 2, 1]); offsets = np.array([0, 3, 4])
    dY = np.array([[1.0, -2.0], [0.5, 0.25]], np.float32)
    t = table.copy(); u, c = oracle.emb_backward_sgd(t, rows, dY, 1.0, offsets, oracle.SUM)
    assert u.tolist() == [1, 2] and c.tolist() == [1, 3]
    assert t.tolist() == [[0, 0], [-0.5, -0.25], [-3.0, 6.0], [0, 0]]
    t = table.copy(); oracle.emb_backward_sgd(t, rows, dY, 1.0, offsets, oracle.MEAN)
    np.testing.assert_allclose(t[2], [-1.0, 2.0], rtol=1e-7)        # 3 occurrences x dY/3


def test_sample_order_does_not_matter():
    table, offsets, rows, dY = _case(n_bags=20)
    h = np.diff(offsets)
    perm = RNG.permutation(20)
    rows_p = np.concatenate([rows[offsets[b]:offsets[b + 1]] for b in perm])
    off_p = np.concatenate([[0], np.cumsum(h[perm])])
    t1 = table.copy(); oracle.emb_backward_sgd(t1, rows, dY, 0.01, offsets)
    t2 = table.copy(); oracle.emb_backward_sgd(t2, rows_p, dY[perm], 0.01, off_p)
    np.testing.assert_allclose(t1, t2, rtol=1e-6, atol=1e-8)


def test_fp16_table_update_rounds_once_to_nearest():
    table, offsets, rows, dY = _case(dtype=np.float16)
    M = _dense_M(rows, offsets, len(offsets) - 1, len(table), False)
    ref = table.astype(np.float64) - float(np.float32(0.01)) * (M.T @ dY.astype(np.float64))
    t = table.copy(); uniq, _ = oracle.emb_backward_sgd(t, rows, dY, 0.01, offsets)
    assert np.array_equal(t[uniq], ref[uniq].astype(np.float16))
    untouched = np.setdiff1d(np.arange(len(table)), uniq)
    assert np.array_equal(t[untouched].view(np.uint16), table[untouched].view(np.uint16))


def test_tiny_config_backward():
    """Tiny configuration: 10,000 x 16 fp32, batch 256 x 4 one-hot slots, lr 0.01, dY ~ N(0,1)."""
    seed = datagen.DEFAULT_SEED
    table = datagen.table_rows_at(seed, torch.arange(10000), 16, torch.float32).numpy()
    keys = datagen.onehot_keys(seed, 0, [10000] * 4, 256, 0.0).numpy()
    dY = datagen.normal_grads(seed, 0, 1024 * 16).numpy().reshape(1024, 16)
    t = table.copy()
    uniq, cnt = oracle.emb_backward_sgd(t, keys, dY, 0.01)
    vu, vc = np.unique(keys, return_counts=True)
    assert np.array_equal(uniq, vu) and np.array_equal(cnt, vc) and cnt.sum() == 1024
    G = np.zeros((10000, 16)); np.add.at(G, keys, dY.astype(np.float64))
    ref = table.astype(np.float64) - float(np.float32(0.01)) * G
    assert np.array_equal(t, ref.astype(np.float32))
