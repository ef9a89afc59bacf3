"""Generators: reproducibility and the closed forms they promise."""
import numpy as np
import torch

import datagen


def test_table_rows_recipe_reproduces_frozen_vector():
    s, rows = datagen.draw_table_rows()
    assert s == datagen.DLRM_TABLE_ROWS_SEED
    assert np.array_equal(rows, datagen.DLRM_TABLE_ROWS)
    assert 1.6e8 <= rows.sum() <= 2.0e8 and len(rows) == 26
    assert rows.min() >= 10 and rows.max() <= 4e7


def test_mix64_matches_python_integers():
    x = torch.tensor([0, 1, -1, 123456789012345, -(1 << 63)], dtype=torch.int64)
    got = datagen.mix64(x).tolist()
    for xi, gi in zip(x.tolist(), got):
        assert (gi & ((1 << 64) - 1)) == datagen._mix64_py(xi & ((1 << 64) - 1))


def test_table_values_exact_and_bounded():
    idx = torch.tensor([0, 5, 10**8, 2**31 + 7], dtype=torch.int64)
    t32 = datagen.table_rows_at(7, idx, 16, torch.float32)
    t16 = datagen.table_rows_at(7, idx, 16, torch.float16)
    assert t32.abs().max() <= 1 / 16 and t16.float().abs().max() <= 1 / 16
    # multiples of 2^-27 (fp32) and 2^-14 (fp16): scaling back gives integers
    assert torch.equal(t32.double() * 2**27, (t32.double() * 2**27).round())
    assert torch.equal(t16.double() * 2**14, (t16.double() * 2**14).round())
    # row content depends on the row index only, not on which other rows were asked for
    again = datagen.table_rows_at(7, idx[[2]], 16, torch.float32)
    assert torch.equal(again[0], t32[2])
    full = torch.empty(40, 16)
    datagen.fill_table(7, full, chunk_rows=16)
    assert torch.equal(full[5], t32[1])


def test_zipf_frequencies_follow_power_law():
    n, alpha, m = 1000, 1.05, 400000
    smp = datagen.ZipfSampler(n, alpha)
    r = smp.ranks(datagen.uniform01(11, 0, m)).numpy()
    assert r.min() >= 1 and r.max() <= n
    p = np.arange(1, n + 1, dtype=np.float64) ** -alpha
    p /= p.sum()
    cnt = np.bincount(r, minlength=n + 1)[1:]
    for k in (1, 2, 3, 10, 100):
        sd = np.sqrt(m * p[k - 1] * (1 - p[k - 1]))
        assert abs(cnt[k - 1] - m * p[k - 1]) < 5 * sd


def test_zipf_open_space_tail_mass():
    smp = datagen.ZipfSampler(1 << 63, 1.05)
    r = smp.ranks(datagen.uniform01(3, 0, 200000))
    assert r.min() >= 1 and int(r.max()) < (1 << 63)
    frac = float((r > 10**8).double().mean())
    assert 0.29 < frac < 0.33  # closed form: 20*(1e8^-0.05 - 2^-3.15) / H ~ 0.31


def test_rank_to_key_is_a_bijection():
    for n in (10, 97, 1000, 4461):
        k = datagen.rank_to_key(torch.arange(1, n + 1), n, 5)
        assert sorted(k.tolist()) == list(range(n))


def test_keys_in_range_and_seeded():
    rows = [10, 1000, 50]
    a = datagen.onehot_keys(1, 0, rows, 64, 1.05)
    b = datagen.onehot_keys(1, 0, rows, 64, 1.05)
    c = datagen.onehot_keys(1, 1, rows, 64, 1.05)
    assert torch.equal(a, b) and not torch.equal(a, c)
    a = a.view(64, 3)
    for s, n in enumerate(rows):
        assert a[:, s].min() >= 0 and a[:, s].max() < n
    off = datagen.multihot_offsets(1, 0, 64 * 3, 1, 100)
    h = off[1:] - off[:-1]
    assert off[0] == 0 and h.min() >= 1 and h.max() <= 100
    k = datagen.multihot_keys(1, 0, rows, 64, 1.1, off)
    assert len(k) == int(off[-1])
    bag = torch.repeat_interleave(torch.arange(64 * 3), h)
    lim = torch.tensor(rows)[bag % 3]
    assert (k >= 0).all() and (k < lim).all()


def test_hotness_mean_and_grad_moments():
    off = datagen.multihot_offsets(2, 0, 200000, 1, 100)
    assert abs(float(off[-1]) / 200000 - 50.5) < 0.3
    g = datagen.normal_grads(2, 0, 500001)
    assert g.dtype == torch.float32 and len(g) == 500001
    assert abs(float(g.mean())) < 0.01 and abs(float(g.std()) - 1) < 0.01
