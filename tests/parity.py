"""Shared helpers of the GPU parity tests: run the oracle and the HIP library on the same seeded
inputs and compare.  Integer results must match exactly.  Floating point must satisfy

    |gpu - ref| <= 1e-5 * max(|ref|, sum_j |term_j| / 8)

per element, where ref is the oracle (double accumulation, one rounding) and the terms are the
addends of that element.  Pure relative error is ill-posed when the addends cancel; the second
operand bounds the error of any fp32 summation order of up to ~1300 terms of one sign pattern
(n * 2^-24 * sum|term| <= 1e-5/8 * sum|term|) and in practice of far longer random sums."""
from __future__ import annotations

import numpy as np
import torch

import oracle

RTOL = 1e-5


def assert_close(gpu: np.ndarray, ref: np.ndarray, term_abs_sum: np.ndarray, what: str) -> None:
    gpu64, ref64 = gpu.astype(np.float64), ref.astype(np.float64)
    tol = RTOL * np.maximum(np.abs(ref64), term_abs_sum.astype(np.float64) / 8.0)
    err = np.abs(gpu64 - ref64)
    bad = err > tol
    if bad.any():
        i = np.unravel_index(np.argmax(err - tol), err.shape)
        raise AssertionError(f"{what}: {bad.sum()} of {bad.size} elements off; worst at {i}: "
                             f"gpu {gpu64[i]!r} ref {ref64[i]!r} err {err[i]:.3e} tol {tol[i]:.3e}")


def oracle_forward(table: np.ndarray, rows: np.ndarray, offsets, combiner: int, n_bags: int):
    """(reference output, per-element sum of |terms|) from the oracle."""
    ref = oracle.emb_forward(table, rows, offsets, combiner, n_bags=n_bags)
    mag = oracle.emb_forward(np.abs(table), rows, offsets, combiner, n_bags=n_bags)
    return ref, mag


def oracle_backward(table: np.ndarray, rows: np.ndarray, offsets, combiner: int, n_bags: int,
                    dY: np.ndarray, lr: float):
    """(updated table, per-element sum of |terms| of the update, unique rows, counts)."""
    t = table.copy()
    uniq, cnt = oracle.emb_backward_sgd(t, rows, dY, lr, offsets, combiner, n_bags=n_bags)
    g_abs = np.zeros(table.shape, dtype=np.float32)
    oracle.emb_backward_sgd(g_abs, rows, np.abs(dY), 1.0, offsets, combiner, n_bags=n_bags)
    mag = np.abs(table.astype(np.float64)) + float(np.float32(lr)) * np.abs(g_abs.astype(np.float64))
    return t, mag, uniq, cnt


def check_table_update(gpu_table: np.ndarray, before: np.ndarray, ref: np.ndarray, mag: np.ndarray,
                       uniq: np.ndarray, what: str) -> None:
    touched = np.zeros(len(before), dtype=bool)
    touched[uniq] = True
    same = gpu_table[~touched].view(np.uint8) == before[~touched].view(np.uint8)
    assert same.all(), f"{what}: rows that no key addressed changed"
    if before.dtype == np.float16:
        # storage rounding: the oracle rounds the exact value once, the kernel rounds its fp32 value;
        # they may land on neighbouring fp16 numbers when the exact value sits next to a tie
        g, r = gpu_table[touched].astype(np.float64), ref[touched].astype(np.float64)
        ulp = np.spacing(np.abs(ref[touched]).astype(np.float16)).astype(np.float64)
        tol = np.maximum(ulp, RTOL * np.maximum(np.abs(r), mag[touched] / 8.0))
        assert (np.abs(g - r) <= tol).all(), f"{what}: fp16 rows more than one ulp from the oracle"
    else:
        assert_close(gpu_table[touched], ref[touched], mag[touched], what)


def to_dev(a, dtype=None) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(a)) if isinstance(a, np.ndarray) else a
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()
