"""GPU parity of the mixed-precision variants of the layer (FP16 pooled output, FP16 upstream
gradient, FP16 table with fp32 master rows) against the oracle's mixed functions."""
import numpy as np
import pytest
import torch

import datagen
import oracle
import paper_2210_08803_amd as H
from parity import RTOL, assert_close, to_dev

pytestmark = pytest.mark.gpu
SEED = datagen.DEFAULT_SEED


def half_close(gpu16, ref16, ref_exact, mag, what):
    """fp16 results: within one fp16 ulp of the oracle's rounding, or within the fp32 summation
    tolerance of the exact value (the kernel rounds its fp32 sum, the oracle rounds the double sum)."""
    g, r = gpu16.astype(np.float64), ref16.astype(np.float64)
    ulp = np.spacing(np.abs(ref16)).astype(np.float64)
    tol = np.maximum(ulp, RTOL * np.maximum(np.abs(ref_exact.astype(np.float64)), mag.astype(np.float64) / 8.0))
    bad = np.abs(g - r) > tol
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} fp16 elements more than one ulp off"


def make(table_rows, dim, batch, tdtype, hot, seed=SEED):
    S = len(table_rows)
    ro = datagen.row_offsets(table_rows)
    base, total = ro[:-1].copy(), int(ro[-1])
    num = np.asarray(table_rows, dtype=np.int64)
    table = datagen.table_rows_at(seed, torch.arange(total), dim, tdtype)
    n_bags = batch * S
    if hot is None:
        offsets, keys = None, datagen.onehot_keys(seed, 0, table_rows, batch, 1.05)
    else:
        offsets = datagen.multihot_offsets(seed, 0, n_bags, hot[0], hot[1])
        keys = datagen.multihot_keys(seed, 0, table_rows, batch, 1.05, offsets)
    off_np = None if offsets is None else offsets.numpy()
    rows, _ = oracle.rows_direct(base, num, keys.numpy(), off_np, n_bags=n_bags)
    return S, base, num, table, keys, offsets, off_np, rows, n_bags


@pytest.mark.parametrize("tdtype", [torch.float32, torch.float16])
@pytest.mark.parametrize("hot,combiner", [(None, H.SUM), ((0, 9), H.SUM), ((1, 40), H.MEAN)])
def test_fp16_output(tdtype, hot, combiner):
    check_fp16_output([3000, 17, 800, 12000], 64, 1500, tdtype, hot, combiner)


def check_fp16_output(table_rows, D, batch, tdtype, hot, combiner, seed=SEED):
    S, base, num, table, keys, offsets, off_np, rows, n_bags = make(table_rows, D, batch, tdtype, hot, seed)
    tab = table.numpy()
    ref16 = oracle.emb_forward_mixed(tab, rows, off_np, combiner, n_bags=n_bags)
    ref32 = oracle.emb_forward(tab, rows, off_np, combiner, n_bags=n_bags)
    mag = oracle.emb_forward(np.abs(tab), rows, off_np, combiner, n_bags=n_bags)
    layer = H.EmbeddingLayer(to_dev(table), S, combiner, base, num, io_dtype=torch.float16)
    out = layer.forward(batch, to_dev(keys), None if offsets is None else to_dev(offsets))
    assert out.dtype == torch.float16
    got = out.cpu().numpy().reshape(n_bags, D)
    if hot is None:   # a copy: fp16 rows pass unchanged, fp32 rows are rounded once
        assert np.array_equal(got.view(np.uint16), ref16.view(np.uint16))
    half_close(got, ref16, ref32, mag, "fp16 forward")


@pytest.mark.parametrize("tdtype", [torch.float32, torch.float16])
@pytest.mark.parametrize("hot,combiner", [(None, H.SUM), ((1, 30), H.MEAN)])
def test_fp16_gradient(tdtype, hot, combiner):
    check_fp16_gradient([5000, 9, 600], 32, 4000, tdtype, hot, combiner)


def check_fp16_gradient(table_rows, D, batch, tdtype, hot, combiner, seed=SEED):
    S, base, num, table, keys, offsets, off_np, rows, n_bags = make(table_rows, D, batch, tdtype, hot, seed)
    dY16 = datagen.normal_grads(seed, 2, n_bags * D).view(n_bags, D).to(torch.float16)
    lr = 0.02
    tab = table.numpy()
    ref = tab.copy()
    oracle.emb_backward_sgd_mixed(ref, rows, dY16.numpy(), lr, off_np, combiner, n_bags=n_bags)
    g_abs = np.zeros(tab.shape, dtype=np.float32)
    oracle.emb_backward_sgd(g_abs, rows, np.abs(dY16.numpy().astype(np.float32)), -1.0, off_np, combiner, n_bags=n_bags)
    mag = np.abs(tab.astype(np.float64)) + lr * g_abs
    d_table = to_dev(table)
    layer = H.EmbeddingLayer(d_table, S, combiner, base, num, io_dtype=torch.float16)
    layer.backward_sgd(batch, to_dev(keys), to_dev(dY16), lr, None if offsets is None else to_dev(offsets))
    got = d_table.cpu().numpy()
    touched = np.unique(rows[rows >= 0])
    rest = np.setdiff1d(np.arange(tab.shape[0]), touched)
    assert np.array_equal(got[rest].view(np.uint8), tab[rest].view(np.uint8))
    if tdtype == torch.float16:
        half_close(got[touched], ref[touched], ref[touched], mag[touched], "fp16 table, fp16 gradient")
    else:
        assert_close(got[touched], ref[touched], mag[touched], "fp32 table, fp16 gradient")


@pytest.mark.parametrize("io", [torch.float32, torch.float16])
def test_master_rows(io):
    check_master_rows([4000, 33, 900], 64, 3000, io, (1, 12), H.MEAN)


def check_master_rows(table_rows, D, batch, io, hot, combiner, seed=SEED):
    S, base, num, table32, keys, offsets, off_np, rows, n_bags = make(table_rows, D, batch, torch.float32, hot, seed)
    master0 = table32.numpy().copy()
    table16_0 = master0.astype(np.float16)
    d_master, d_table = to_dev(master0), to_dev(table16_0)
    layer = H.EmbeddingLayer(d_table, S, combiner, base, num, io_dtype=io, master=d_master)
    ref_master, ref_table = master0.copy(), table16_0.copy()
    lr = 0.05
    touched = np.unique(rows[rows >= 0])
    rest = np.setdiff1d(np.arange(master0.shape[0]), touched)
    d_keys, d_off = to_dev(keys), (None if offsets is None else to_dev(offsets))
    for step in range(3):    # errors must not build up: the master is compared after every step
        dY = datagen.normal_grads(seed, 10 + step, n_bags * D).view(n_bags, D).to(io)
        before = ref_master.copy()
        oracle.emb_backward_sgd_mixed(ref_table, rows, dY.numpy(), lr, off_np, combiner, n_bags=n_bags, master=ref_master)
        g_abs = np.zeros(master0.shape, dtype=np.float32)
        oracle.emb_backward_sgd(g_abs, rows, np.abs(dY.numpy().astype(np.float32)), -1.0, off_np, combiner, n_bags=n_bags)
        mag = np.abs(before.astype(np.float64)) + lr * g_abs
        layer.backward_sgd(batch, d_keys, to_dev(dY), lr, d_off)
        got_m, got_t = d_master.cpu().numpy(), d_table.cpu().numpy()
        assert_close(got_m[touched], ref_master[touched], mag[touched], f"master rows, step {step}")
        # the table row is the rounding of the kernel's own master row, bit for bit
        assert np.array_equal(got_t[touched].view(np.uint16), got_m[touched].astype(np.float16).view(np.uint16))
        assert np.array_equal(got_m[rest], master0[rest]) and np.array_equal(got_t[rest].view(np.uint16),
                                                                             table16_0[rest].view(np.uint16))
        half_close(got_t[touched], ref_table[touched], ref_master[touched], mag[touched], f"fp16 rows, step {step}")
        # carry the kernel's master forward in the oracle too, so each step is judged on its own
        ref_master[:] = got_m
        ref_table[:] = got_t
    # forward reads the fp16 table
    out = layer.forward(batch, d_keys, d_off)
    ref = oracle.emb_forward_mixed(d_table.cpu().numpy(), rows, off_np, combiner, n_bags=n_bags,
                                   out_dtype=np.float16 if io == torch.float16 else np.float32)
    ref32 = oracle.emb_forward(d_table.cpu().numpy(), rows, off_np, combiner, n_bags=n_bags)
    mag = oracle.emb_forward(np.abs(d_table.cpu().numpy()), rows, off_np, combiner, n_bags=n_bags)
    got = out.cpu().numpy().reshape(n_bags, D)
    if io == torch.float16:
        half_close(got, ref, ref32, mag, "forward after master updates")
    else:
        assert_close(got, ref, mag, "forward after master updates")
