"""Pins for the oracle's mixed-precision variants (section 1, "Mixed precision training"): FP16
pooled output, FP16 upstream gradient, FP16 table with an fp32 master copy.  Checked against numpy's
own float64 -> float16 rounding, torch autograd on widened inputs, and the property that gives
master weights their name: the master rows follow exactly the trajectory of an fp32 table."""
import numpy as np
import pytest
import torch

import datagen
import oracle

RNG = np.random.default_rng(777)


def _case(n_rows=(9, 6, 14), batch=8, dim=8, hmax=5, dtype=np.float16):
    S = len(n_rows)
    ro = datagen.row_offsets(n_rows)
    table = (RNG.standard_normal((ro[-1], dim)) * 0.25).astype(dtype)
    h = RNG.integers(0, hmax + 1, batch * S)
    offsets = np.concatenate([[0], np.cumsum(h)]).astype(np.int64)
    slot = np.repeat(np.arange(batch * S) % S, h)
    keys = (RNG.random(len(slot)) * np.asarray(n_rows)[slot]).astype(np.int64)
    rows, _ = oracle.rows_direct(ro[:-1], np.diff(ro), keys, offsets)
    return table, rows, offsets


@pytest.mark.parametrize("tdtype", [np.float32, np.float16])
@pytest.mark.parametrize("combiner", [oracle.SUM, oracle.MEAN])
def test_fp16_output_is_the_double_sum_rounded_once(tdtype, combiner):
    table, rows, offsets = _case(dtype=tdtype)
    n_bags = len(offsets) - 1
    M = np.zeros((n_bags, table.shape[0]))
    for bag in range(n_bags):
        for i in range(offsets[bag], offsets[bag + 1]):
            M[bag, rows[i]] += 1
    ref = M @ table.astype(np.float64)
    if combiner == oracle.MEAN:
        ref = ref / np.maximum(np.diff(offsets), 1)[:, None]
    out = oracle.emb_forward_mixed(table, rows, offsets, combiner)
    assert out.dtype == np.float16
    assert np.array_equal(out.view(np.uint16), ref.astype(np.float16).view(np.uint16))   # numpy's own rounding
    # with fp32 output the mixed entry point is the plain one
    assert np.array_equal(oracle.emb_forward_mixed(table, rows, offsets, combiner, out_dtype=np.float32),
                          oracle.emb_forward(table, rows, offsets, combiner))


def test_fp16_rounding_ties_and_range():
    # one-key bags return the value itself: exercise ties to even, overflow and subnormals through an fp32 table
    vals = np.array([1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 65519.0, 65520.0, 2.0 ** -25, 3 * 2.0 ** -25, -2.0 ** -24,
                     1e-9], dtype=np.float32)
    table = vals.reshape(-1, 1).repeat(4, axis=1).copy()
    out = oracle.emb_forward_mixed(table, np.arange(len(vals)), None, oracle.SUM)
    with np.errstate(over="ignore"):
        want = vals.astype(np.float64).astype(np.float16)
    assert np.array_equal(out[:, 0].view(np.uint16), want.view(np.uint16))
    assert out[0, 0] == np.float16(1.0) and out[1, 0] == np.float16(1.0 + 2.0 ** -9)      # ties to even, both ways
    assert out[2, 0] == np.float16(65504.0) and np.isinf(out[3, 0])
    assert out[4, 0] == 0 and out[5, 0] == np.float16(2.0 ** -23)                          # subnormal ties


@pytest.mark.parametrize("combiner", [oracle.SUM, oracle.MEAN])
def test_fp16_gradient_against_torch_autograd(combiner):
    table, rows, offsets = _case(dtype=np.float32)
    n_bags = len(offsets) - 1
    dY16 = RNG.standard_normal((n_bags, table.shape[1])).astype(np.float16)
    lr = 0.05
    p = torch.from_numpy(table.copy()).double().requires_grad_(True)
    out = torch.nn.functional.embedding_bag(torch.from_numpy(rows), p, torch.from_numpy(offsets),
                                            mode="mean" if combiner == oracle.MEAN else "sum", include_last_offset=True)
    out.backward(torch.from_numpy(dY16.astype(np.float64)))
    want = (p.detach() - lr * p.grad).numpy()
    t = table.copy()
    u = oracle.emb_backward_sgd_mixed(t, rows, dY16, lr, offsets, combiner)
    np.testing.assert_allclose(t, want, rtol=1e-6, atol=1e-7)
    assert u == len(np.unique(rows))
    # widening is exact: the same gradient handed over as fp32 gives the same bits
    t2 = table.copy()
    oracle.emb_backward_sgd_mixed(t2, rows, dY16.astype(np.float32), lr, offsets, combiner)
    assert np.array_equal(t, t2)
    t3 = table.copy()
    oracle.emb_backward_sgd(t3, rows, dY16.astype(np.float32), lr, offsets, combiner)
    assert np.array_equal(t, t3)


def test_master_rows_follow_the_fp32_trajectory():
    table32, rows, offsets = _case(dtype=np.float32)
    n_bags = len(offsets) - 1
    master = table32.copy()
    table16 = master.astype(np.float16)
    start16 = table16.copy()
    plain32 = table32.copy()
    lr = 0.1
    for step in range(4):
        dY = RNG.standard_normal((n_bags, table32.shape[1])).astype(np.float16)
        oracle.emb_backward_sgd_mixed(table16, rows, dY, lr, offsets, oracle.MEAN, master=master)
        oracle.emb_backward_sgd(plain32, rows, dY.astype(np.float32), lr, offsets, oracle.MEAN)   # pinned elsewhere
        assert np.array_equal(master, plain32)                       # the master IS the fp32 table
        touched = np.unique(rows)
        assert np.array_equal(table16[touched].view(np.uint16), master[touched].astype(np.float16).view(np.uint16))
    rest = np.setdiff1d(np.arange(table32.shape[0]), np.unique(rows))
    assert np.array_equal(table16[rest], start16[rest]) and np.array_equal(master[rest], table32[rest])
