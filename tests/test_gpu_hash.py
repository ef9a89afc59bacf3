"""GPU parity: hctr_hash_insert_or_find against the oracle (rows must match exactly), and the
hashed mode of the embedding layer."""
import json
import os

import numpy as np
import pytest
import torch

import datagen
import oracle
from parity import assert_close, check_table_update, oracle_backward, oracle_forward, to_dev

pytestmark = pytest.mark.gpu
SEED = datagen.DEFAULT_SEED
GOLD = os.path.join(os.path.dirname(__file__), "golden", "hash_first_appearance.json")


def H():
    import paper_2210_08803_amd as h
    return h


def both(capacity, max_rows):
    return H().HashTable(capacity, max_rows), oracle.Hash(max_rows)


def step(gpu, ref, keys, insert=True):
    keys = np.ascontiguousarray(keys, dtype=np.int64)
    want = ref.insert_or_find(keys, insert)
    got = gpu.insert_or_find(to_dev(keys), insert).cpu().numpy()
    assert np.array_equal(got, want), f"rows differ at {np.nonzero(got != want)[0][:8]}"
    assert gpu.size == ref.size
    return want


def test_hand_worked_traces():
    for case in json.load(open(GOLD))["cases"]:
        gpu = H().HashTable(256, case["max_rows"])
        for call in case["calls"]:
            keys = torch.tensor(call["keys"], dtype=torch.int64)
            rows = gpu.insert_or_find(keys.cuda(), bool(call["insert"])).cpu().tolist()
            assert rows == call["rows"]
            assert gpu.size == call["size"]


def test_zipf_stream_with_growth_to_the_row_limit():
    """Open 2^63 key space, Zipf 1.05, insert on miss until the table is full and beyond."""
    gpu, ref = both(40000, 30000)
    smp = datagen.ZipfSampler(1 << 63, 1.05)
    for it in range(8):
        keys = datagen.open_space_keys(SEED, it, 26, 257, 1.05, sampler=smp).numpy()
        rows = step(gpu, ref, keys, insert=True)
        step(gpu, ref, keys, insert=False)           # everything accepted is now found
        assert (rows >= -1).all() and rows.max() < 30000
    assert ref.size == 30000                           # saturated: later new keys were rejected
    step(gpu, ref, datagen.open_space_keys(SEED, 99, 26, 300, 1.05, sampler=smp).numpy(), insert=True)


def test_adversarial_inputs():
    gpu, ref = both(4096, 3000)
    step(gpu, ref, np.full(5000, 12345))                                  # all keys equal
    step(gpu, ref, np.arange(1000) * 7919 + 1)                            # all distinct
    step(gpu, ref, np.array([], dtype=np.int64))                          # n = 0
    step(gpu, ref, np.array([5]))                                         # n = 1
    step(gpu, ref, np.array([-1, -7, 5, 2**63 - 1, 0, -2**63]))           # negative keys are never stored
    rng = np.random.default_rng(4)
    dup = rng.integers(0, 600, 20000)                                     # heavy duplication among new keys
    step(gpu, ref, dup + 10**12)
    # keys sharing their low bits, a classic failure of weak mixing
    step(gpu, ref, (np.arange(700, dtype=np.int64) << 32) + 99)


def test_exact_fill_then_overflow_by_one():
    gpu, ref = both(64, 51)
    step(gpu, ref, np.arange(100, 151))                                   # exactly fills max_rows
    assert ref.size == 51
    step(gpu, ref, np.array([151, 100, 152, 151]))                        # overflow: -1, found, -1, -1
    gpu2, ref2 = both(64, 51)
    step(gpu2, ref2, np.arange(100, 152))                                 # overflow by one inside one call


def test_split_calls_give_the_same_mapping():
    keys = datagen.open_space_keys(SEED, 5, 26, 400, 1.05).numpy()
    a = H().HashTable(1 << 15, 20000)
    b = H().HashTable(1 << 15, 20000)
    ra = a.insert_or_find(to_dev(keys), True).cpu().numpy()
    rb = np.concatenate([b.insert_or_find(to_dev(keys[:3333]), True).cpu().numpy(),
                         b.insert_or_find(to_dev(keys[3333:]), True).cpu().numpy()])
    assert np.array_equal(ra, rb) and a.size == b.size


@pytest.mark.parametrize("reuse", [False, True], ids=["lookup-twice", "reuse-forward-rows"])
def test_hashed_embedding_forward_backward(reuse):
    """26 one-hot slots over an open key space, dim 64 fp32, insert on miss in forward."""
    check_hashed_layer(26, 64, 513, 16384, 12000, reuse, 3, SEED)


def check_hashed_layer(S, dim, batch, capacity, max_rows, reuse, steps, seed, dtype=torch.float32, alpha=1.05):
    """One-hot slots over an open key space, insert on miss in forward, `steps` forward + backward
    steps (the table may fill up on the way: keys that are refused have no row)."""
    h = H()
    ht, ref_hash = both(capacity, max_rows)
    table = datagen.table_rows_at(seed, torch.arange(max_rows), dim, dtype)
    d_table = to_dev(table)
    layer = h.EmbeddingLayer(d_table, S, h.SUM, hash_table=ht, insert_on_miss=True, reuse_forward_rows=reuse)
    tab_np = table.numpy().copy()
    smp = datagen.ZipfSampler(1 << 63, alpha)
    for it in range(steps):
        keys = datagen.open_space_keys(seed, it, S, batch, alpha, sampler=smp)
        if it == 2:
            keys[::50] = -5                                              # keys that can never get a row
        dY = datagen.normal_grads(seed, it, batch * S * dim).view(batch * S, dim)
        rows = ref_hash.insert_or_find(keys.numpy(), True)
        ref_out, mag = oracle_forward(tab_np, rows, None, 0, batch * S)
        out = layer.forward(batch, to_dev(keys))
        torch.cuda.synchronize()
        assert ht.size == ref_hash.size
        assert layer.invalid_keys() == int((rows < 0).sum())
        layer.reset_invalid_keys()
        out_np = out.cpu().numpy().reshape(batch * S, dim)
        assert np.array_equal(out_np.view(np.uint32), ref_out.view(np.uint32))      # out is fp32: a copy, or an exact widening
        ref_tab, mag_tab, uniq, cnt = oracle_backward(tab_np, rows, None, 0, batch * S, dY.numpy(), 0.01)
        layer.backward_sgd(batch, to_dev(keys), to_dev(dY), 0.01)
        g_rows, g_cnt = layer.dedup_result(batch, keys.numel())
        assert layer.invalid_keys() == int((rows < 0).sum())
        layer.reset_invalid_keys()
        assert np.array_equal(g_rows.cpu().numpy(), uniq) and np.array_equal(g_cnt.cpu().numpy(), cnt)
        check_table_update(d_table.cpu().numpy(), tab_np, ref_tab, mag_tab, uniq, f"hashed backward {it}")
        tab_np = d_table.cpu().numpy().copy()                            # continue from the GPU's table
        assert ht.size == ref_hash.size                                  # backward never inserts
