"""Pins for the oracle's forward pass (lookup + intra-slot reduction, section 1 "Localized slot
embedding hash"; FP16 storage, section 1 "Mixed precision training").  None of these re-type the
oracle's loop: they use a dense matrix product, torch's embedding_bag and exact special cases."""
import numpy as np
import pytest
import torch

import datagen
import oracle

RNG = np.random.default_rng(1234)


def _case(n_rows=(7, 5, 9), batch=6, dim=8, hmax=5, dtype=np.float32, empty=True):
    S = len(n_rows)
    ro = datagen.row_offsets(n_rows)
    table = (RNG.standard_normal((ro[-1], dim)) * 0.25).astype(dtype)
    h = RNG.integers(0 if empty else 1, hmax + 1, batch * S)
    offsets = np.concatenate([[0], np.cumsum(h)]).astype(np.int64)
    slot = np.repeat(np.arange(batch * S) % S, h)
    keys = (RNG.random(len(slot)) * np.asarray(n_rows)[slot]).astype(np.int64)
    return ro, table, offsets, keys


def _multiplicity(rows, offsets, n_bags, total_rows):
    M = np.zeros((n_bags, total_rows))
    for bag in range(n_bags):
        for i in range(offsets[bag], offsets[bag + 1]):
            if rows[i] >= 0:
                M[bag, rows[i]] += 1
    return M


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
@pytest.mark.parametrize("combiner", [oracle.SUM, oracle.MEAN])
def test_forward_equals_dense_matrix_product(dtype, combiner):
    ro, table, offsets, keys = _case(dtype=dtype)
    rows, bad = oracle.rows_direct(ro[:-1], np.diff(ro), keys, offsets)
    assert bad == 0
    n_bags = len(offsets) - 1
    M = _multiplicity(rows, offsets, n_bags, ro[-1])
    ref = M @ table.astype(np.float64)
    if combiner == oracle.MEAN:
        h = np.diff(offsets)
        ref = ref / np.maximum(h, 1)[:, None]
    out = oracle.emb_forward(table, rows, offsets, combiner)
    assert np.array_equal(out, ref.astype(np.float32))  # double accumulate, one rounding
    assert np.all(out[np.diff(offsets) == 0] == 0)      # empty bags give zeros, no 0/0


@pytest.mark.parametrize("mode,combiner", [("sum", oracle.SUM), ("mean", oracle.MEAN)])
def test_forward_against_torch_embedding_bag(mode, combiner):
    ro, table, offsets, keys = _case(n_rows=(11, 4), batch=9, dim=12, hmax=7, empty=False)
    rows, _ = oracle.rows_direct(ro[:-1], np.diff(ro), keys, offsets)
    out = oracle.emb_forward(table, rows, offsets, combiner)
    ref = torch.nn.functional.embedding_bag(
        torch.from_numpy(rows), torch.from_numpy(table).double(), torch.from_numpy(offsets),
        mode=mode, include_last_offset=True)
    np.testing.assert_allclose(out, ref.numpy(), rtol=1e-6, atol=1e-7)


def test_rows_direct_slot_offsets_and_range_check():
    # 2 slots with 3 and 4 rows; bag id = b*2 + s, so bags 0,2 use table 0 and bags 1,3 table 1
    ro = np.array([0, 3, 7])
    keys = np.array([2, 3, 0, 4, -1, 1])
    offsets = np.array([0, 1, 2, 4, 6])  # bag2 has keys (0, 4): 4 is outside table 0
    rows, bad = oracle.rows_direct(ro[:-1], np.diff(ro), keys, offsets)
    assert rows.tolist() == [2, 6, 0, -1, -1, 4] and bad == 2
    rows1, bad1 = oracle.rows_direct(ro[:-1], np.diff(ro), np.array([1, 1, 2, 3]))  # one-hot: bag i holds key i
    assert rows1.tolist() == [1, 4, 2, 6] and bad1 == 0


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_one_hot_bag_returns_the_row_bit_for_bit(dtype):
    table = datagen.table_rows_at(5, torch.arange(50), 16, torch.float32 if dtype == np.float32 else torch.float16).numpy()
    rows = RNG.integers(0, 50, 33)
    for comb in (oracle.SUM, oracle.MEAN):
        out = oracle.emb_forward(table, rows, None, comb)
        assert np.array_equal(out, table[rows].astype(np.float32))


def test_linearity_and_invalid_keys():
    table = datagen.table_rows_at(5, torch.arange(20), 8, torch.float32).numpy()
    rows = np.array([3, 3, 7, 7, 7, -1, 9, 25])  # 25 is beyond the table: no row
    offsets = np.array([0, 2, 5, 8])
    out = oracle.emb_forward(table, rows, offsets, oracle.SUM)
    assert np.array_equal(out[0], 2 * table[3])
    assert np.array_equal(out[1], (3 * table[7].astype(np.float64)).astype(np.float32))
    assert np.array_equal(out[2], table[9])
    mean = oracle.emb_forward(table, rows, offsets, oracle.MEAN)
    np.testing.assert_allclose(mean[1], table[7], rtol=2e-7)
    # mean divides by the bag's hotness (3), keys without a row included
    assert np.array_equal(mean[2], (table[9].astype(np.float64) / 3).astype(np.float32))


def test_half_conversions_match_numpy():
    bits = np.arange(0, 1 << 16, dtype=np.uint16)
    h = bits.view(np.float16)
    finite = np.isfinite(h) & (bits != 0x8000)  # 0 + (-0) is +0: a property of the sum, not of the decode
    tab = h[finite].reshape(-1, 1).copy()
    out = oracle.emb_forward(tab, np.arange(len(tab)), None, oracle.SUM)  # fp16 -> double -> fp32
    assert np.array_equal(out.view(np.uint32), tab.astype(np.float32).view(np.uint32))
    # double -> fp16 rounding (nearest even) through the SGD store: T - 1*g with T = 0
    vals = np.concatenate([RNG.standard_normal(4000) * 10.0 ** RNG.integers(-9, 5, 4000),
                           [0.0, 65519.9, 65520.0, 2.0**-24, 2.0**-25, 3 * 2.0**-25, 1.0009765625 + 2.0**-11,
                            1.0 + 2.0**-11, 1.0 + 3 * 2.0**-11, 6.1e-5, 6.0975552e-05]]).astype(np.float32)
    tab = np.zeros((len(vals), 1), dtype=np.float16)
    oracle.emb_backward_sgd(tab, np.arange(len(vals)), -vals.reshape(-1, 1), 1.0)
    with np.errstate(over="ignore"):
        ref = vals.astype(np.float16)
    assert np.array_equal(tab[:, 0].view(np.uint16), ref.view(np.uint16))


def test_tiny_config_three_ways():
    """Tiny configuration: 4 one-hot slots over one 10,000 x 16 table, batch 256, uniform keys."""
    table = datagen.table_rows_at(datagen.DEFAULT_SEED, torch.arange(10000), 16, torch.float32).numpy()
    keys = datagen.onehot_keys(datagen.DEFAULT_SEED, 0, [10000] * 4, 256, 0.0).numpy()
    rows, bad = oracle.rows_direct([0] * 4, [10000] * 4, keys)  # the four slots share the one table
    assert bad == 0 and np.array_equal(rows, keys)
    out = oracle.emb_forward(table, rows, None, oracle.SUM)
    assert np.array_equal(out, table[keys])
    ref = torch.nn.functional.embedding_bag(torch.from_numpy(keys), torch.from_numpy(table),
                                            torch.arange(len(keys) + 1), mode="sum", include_last_offset=True)
    assert np.array_equal(out, ref.numpy())
    M = np.zeros((len(keys), 10000)); M[np.arange(len(keys)), keys] = 1
    assert np.array_equal(out, (M @ table.astype(np.float64)).astype(np.float32))
