"""Pins for the oracle's fused group of lookups (section 4, "Future Work": tables of different vector
size and combiner fused into one embedding, dense and sparse inputs).  None of these re-type the
oracle's loops: per-lookup torch embedding_bag, torch autograd through the concatenated output
(which also settles how two lookups on one table meet in one update), a dense matrix product per
lookup, and exact special cases."""
import numpy as np
import pytest
import torch

import oracle

RNG = np.random.default_rng(4321)

# tables (rows, dim); lookups (table, combiner): lookups 1 and 3 share table 1
TABLES = [(13, 4), (7, 12), (21, 8), (5, 32)]
LOOKUPS = [(0, oracle.SUM), (1, oracle.MEAN), (2, oracle.SUM), (1, oracle.SUM), (3, oracle.MEAN)]


def _case(batch=7, hmax=5, dtype=np.float32, empty=True, bad_keys=False):
    tables = [(RNG.standard_normal(shape) * 0.25).astype(dtype) for shape in TABLES]
    lt = np.array([t for t, _ in LOOKUPS], dtype=np.int32)
    lc = np.array([c for _, c in LOOKUPS], dtype=np.int32)
    L = len(LOOKUPS)
    h = RNG.integers(0 if empty else 1, hmax + 1, batch * L)
    offsets = np.concatenate([[0], np.cumsum(h)]).astype(np.int64)
    lookup_of_key = np.repeat(np.arange(batch * L) % L, h)
    rows_of_key = np.array([TABLES[t][0] for t in lt])[lookup_of_key]
    keys = (RNG.random(len(lookup_of_key)) * rows_of_key).astype(np.int64)
    if bad_keys and len(keys) > 3:
        keys[1] = -3
        keys[len(keys) // 2] = rows_of_key[len(keys) // 2]      # one past the end
    return tables, lt, lc, batch, keys, offsets


def _torch_forward(tables_t, lt, lc, batch, keys, offsets):
    L = len(lt)
    keys_t, off = torch.from_numpy(keys), torch.from_numpy(offsets)
    cols = []
    for l in range(L):
        # the bags of lookup l, gathered into their own CSR
        starts, ends = off[l::L][:batch], off[l + 1::L][:batch]
        idx = torch.cat([keys_t[s:e] for s, e in zip(starts.tolist(), ends.tolist())] + [keys_t[:0]])
        lens = ends - starts
        o = torch.cat([torch.zeros(1, dtype=torch.int64), torch.cumsum(lens, 0)])
        cols.append(torch.nn.functional.embedding_bag(
            idx, tables_t[lt[l]], o, mode="mean" if lc[l] == oracle.MEAN else "sum", include_last_offset=True))
    return torch.cat(cols, dim=1)


def test_group_forward_against_torch_embedding_bag_per_lookup():
    tables, lt, lc, batch, keys, offsets = _case(empty=True)
    out = oracle.group_forward(tables, lt, lc, batch, keys, offsets)
    ref = _torch_forward([torch.from_numpy(t).double() for t in tables], lt, lc, batch, keys, offsets)
    assert out.shape == (batch, sum(TABLES[t][1] for t in lt))
    np.testing.assert_allclose(out, ref.numpy(), rtol=1e-6, atol=1e-7)


def test_group_forward_fp16_tables_and_column_placement():
    tables, lt, lc, batch, keys, offsets = _case(dtype=np.float16, empty=False)
    out = oracle.group_forward(tables, lt, lc, batch, keys, offsets)
    # lookup l alone, as a group of one lookup, gives exactly the columns it holds in the fused output
    col = 0
    for l in range(len(lt)):
        d = tables[lt[l]].shape[1]
        sel = np.concatenate([np.arange(offsets[b * len(lt) + l], offsets[b * len(lt) + l + 1]) for b in range(batch)])
        lens = np.array([offsets[b * len(lt) + l + 1] - offsets[b * len(lt) + l] for b in range(batch)])
        single = oracle.group_forward([tables[lt[l]]], [0], [lc[l]], batch, keys[sel],
                                      np.concatenate([[0], np.cumsum(lens)]))
        assert np.array_equal(out[:, col:col + d], single)
        col += d
    # and a one-key sum bag returns the fp16 row exactly
    t = tables[0]
    one = oracle.group_forward([t], [0], [oracle.SUM], 3, [2, 0, 5], [0, 1, 2, 3])
    assert np.array_equal(one, t[[2, 0, 5]].astype(np.float32))


def test_group_forward_dense_input_and_bad_keys():
    tables, lt, lc, _, _, _ = _case()
    hot = [1, 3, 2, 1, 4]
    batch = 5
    offsets = oracle.dense_offsets(batch, hot)
    assert offsets[-1] == batch * sum(hot) and np.array_equal(np.diff(offsets)[:5], hot)
    lookup_of_key = np.repeat(np.arange(batch * len(lt)) % len(lt), np.diff(offsets))
    keys = (RNG.random(len(lookup_of_key)) * np.array([TABLES[t][0] for t in lt])[lookup_of_key]).astype(np.int64)
    out = oracle.group_forward(tables, lt, lc, batch, keys, offsets)
    ref = _torch_forward([torch.from_numpy(t).double() for t in tables], lt, lc, batch, keys, offsets)
    np.testing.assert_allclose(out, ref.numpy(), rtol=1e-6, atol=1e-7)
    # a key outside its table adds nothing but still counts in the mean's denominator
    k2 = keys.copy()
    pos = int(offsets[1])            # first key of lookup 1 (mean, hotness 3) of sample 0
    k2[pos] = TABLES[1][0]           # one past the end
    out2 = oracle.group_forward(tables, lt, lc, batch, k2, offsets)
    c0, c1 = TABLES[0][1], TABLES[0][1] + TABLES[1][1]
    want = (tables[1][keys[pos + 1]].astype(np.float64) + tables[1][keys[pos + 2]]) / 3.0
    np.testing.assert_allclose(out2[0, c0:c1], want, rtol=1e-6, atol=1e-7)
    assert np.array_equal(out2[1:], out[1:]) and np.array_equal(out2[0, c1:], out[0, c1:])


@pytest.mark.parametrize("empty", [False, True])
def test_group_backward_against_torch_autograd(empty):
    tables, lt, lc, batch, keys, offsets = _case(empty=empty)
    width = sum(TABLES[t][1] for t in lt)
    dY = RNG.standard_normal((batch, width)).astype(np.float32)
    lr = 0.05
    params = [torch.from_numpy(t.copy()).double().requires_grad_(True) for t in tables]
    out = _torch_forward(params, lt, lc, batch, keys, offsets)
    out.backward(torch.from_numpy(dY).double())
    want = [(p.detach() - lr * (p.grad if p.grad is not None else 0)).numpy() for p in params]
    before = [t.copy() for t in tables]
    touched = oracle.group_backward_sgd(tables, lt, lc, batch, keys, offsets, dY, lr)
    for t, w, b in zip(tables, want, before):
        np.testing.assert_allclose(t, w, rtol=1e-6, atol=1e-7)
    # distinct (table, row) pairs, counted with numpy: lookups 1 and 3 share table 1
    lookup_of_key = np.repeat(np.arange(batch * len(lt)) % len(lt), np.diff(offsets))
    pairs = np.unique(np.stack([lt[lookup_of_key], keys]), axis=1).shape[1]
    assert touched == pairs
    # rows no key names keep their bits
    for ti, (t, b) in enumerate(zip(tables, before)):
        named = np.unique(keys[lt[lookup_of_key] == ti])
        rest = np.setdiff1d(np.arange(t.shape[0]), named)
        assert np.array_equal(t[rest], b[rest])


def test_group_backward_dense_matrix_form_and_conservation():
    tables, lt, lc, batch, keys, offsets = _case(empty=False, bad_keys=True)
    width = sum(TABLES[t][1] for t in lt)
    dY = RNG.standard_normal((batch, width)).astype(np.float32)
    lr = 0.01
    before = [t.astype(np.float64) for t in tables]
    oracle.group_backward_sgd(tables, lt, lc, batch, keys, offsets, dY, lr)
    L = len(lt)
    cols = np.concatenate([[0], np.cumsum([TABLES[t][1] for t in lt])])
    want = [b.copy() for b in before]
    for l in range(L):   # T_t -= lr * M_l^T (w_l * dY_l), M_l the bag x row multiplicity matrix of lookup l
        t = lt[l]
        M = np.zeros((batch, TABLES[t][0]))
        w = np.ones(batch)
        for b in range(batch):
            b0, b1 = offsets[b * L + l], offsets[b * L + l + 1]
            for i in range(b0, b1):
                if 0 <= keys[i] < TABLES[t][0]:
                    M[b, keys[i]] += 1
            if lc[l] == oracle.MEAN and b1 > b0:
                w[b] = 1.0 / (b1 - b0)
        want[t] -= lr * M.T @ (w[:, None] * dY[:, cols[l]:cols[l + 1]].astype(np.float64))
    for t, w_ in zip(tables, want):
        np.testing.assert_allclose(t, w_, rtol=1e-6, atol=1e-7)


def test_group_backward_degenerate_cases():
    tables, lt, lc, batch, keys, offsets = _case()
    width = sum(TABLES[t][1] for t in lt)
    before = [t.copy() for t in tables]
    oracle.group_backward_sgd(tables, lt, lc, batch, keys, offsets, RNG.standard_normal((batch, width)), 0.0)
    assert all(np.array_equal(a, b) for a, b in zip(tables, before))       # lr = 0
    oracle.group_backward_sgd(tables, lt, lc, batch, keys, offsets, np.zeros((batch, width)), 0.3)
    assert all(np.array_equal(a, b) for a, b in zip(tables, before))       # dY = 0
    assert oracle.group_backward_sgd(tables, lt, lc, 0, [], [0], np.zeros((0, width)), 0.3) == 0
