"""GPU parity of the embedding training cache staged in host memory (hctr_etc_*) against the oracle:
rows and statistics exact, loaded rows bit-identical copies, host table after training passes within
the backward tolerance."""
import numpy as np
import pytest
import torch

import oracle
import paper_2210_08803_amd as H
from parity import assert_close, to_dev

pytestmark = pytest.mark.gpu


def pinned(a: np.ndarray) -> torch.Tensor:
    t = torch.empty(a.shape, dtype=torch.float32, pin_memory=True)
    t.copy_(torch.from_numpy(a))
    return t


def test_load_rows_copies_stats_capacity_and_range():
    rng = np.random.default_rng(5)
    host_np = rng.standard_normal((5000, 32)).astype(np.float32)
    host = pinned(host_np)
    etc = H.EmbeddingTrainingCache(host, max_rows=1500)
    ref = oracle.Etc(host_np.copy(), 1500)
    for call in range(4):     # 4 x 700 draws from 3000 hot keys: the working table fills up and rejects
        keys = (rng.random(700) ** 2 * 3000).astype(np.int64)
        keys[rng.integers(0, 700, 9)] = rng.choice([-1, 5000, 2 ** 40, -2 ** 62], 9)
        rows = torch.empty(700, dtype=torch.int64, device="cuda")
        etc.load(to_dev(keys), rows)
        want = ref.load(keys)
        assert np.array_equal(rows.cpu().numpy(), want), f"call {call}"
        assert etc.stats == ref.stats, f"call {call}"
        n = ref.stats[0]
        assert np.array_equal(etc.table[:n].cpu().numpy(), ref.work[:n])
    assert ref.stats[2] > 0 and ref.stats[3] > 0    # both kinds of refusal happened
    # nothing trained: the dump changes nothing; eviction empties the cache
    etc.dump(evict=True)
    torch.cuda.synchronize()
    assert np.array_equal(host.numpy(), host_np)
    assert etc.stats[0] == 0
    etc.load(to_dev(np.array([7, 7, 3])), rows[:3])
    assert rows[:3].tolist() == [0, 0, 1]


def test_load_without_rows_output_and_empty_calls():
    host = pinned(np.arange(40, dtype=np.float32).reshape(10, 4))
    etc = H.EmbeddingTrainingCache(host, max_rows=8)
    etc.load(to_dev(np.array([3, 9, 3])))              # rows pointer NULL
    etc.load(torch.empty(0, dtype=torch.int64, device="cuda"))
    assert etc.stats == (2, 2, 0, 0)
    assert torch.equal(etc.table[:2].cpu(), host[[3, 9]])


@pytest.mark.parametrize("combiner,hot", [(H.SUM, None), (H.MEAN, (0, 6))])
def test_training_passes_reach_the_host_table(combiner, hot):
    rng = np.random.default_rng(6)
    host_rows, dim, S, batch = 20000, 64, 4, 512
    host_np = (rng.standard_normal((host_rows, dim)) * 0.25).astype(np.float32)
    host = pinned(host_np)
    etc = H.EmbeddingTrainingCache(host, max_rows=16384)
    layer = etc.layer(S, combiner)
    ref_host = host_np.copy()
    ref = oracle.Etc(ref_host, 16384)
    lr = 0.05
    for p in range(3):
        batches = []
        for _ in range(3):
            n_bags = batch * S
            if hot is None:
                offsets = None
                nnz = n_bags
            else:
                h = rng.integers(hot[0], hot[1] + 1, n_bags)
                offsets = np.concatenate([[0], np.cumsum(h)]).astype(np.int64)
                nnz = int(offsets[-1])
            keys = (rng.random(nnz) ** 3 * host_rows).astype(np.int64)
            dY = rng.standard_normal((n_bags, dim)).astype(np.float32)
            batches.append((keys, offsets, dY))
        pass_keys = np.concatenate([b[0] for b in batches])
        etc.load(to_dev(pass_keys))
        ref.load(pass_keys)
        assert etc.stats == ref.stats
        before = ref_host.copy()
        mag = np.abs(before.astype(np.float64))
        for keys, offsets, dY in batches:
            d_off = None if offsets is None else to_dev(offsets)
            out = layer.forward(batch, to_dev(keys), d_off)
            rows = ref.load(keys)
            assert (rows >= 0).all()
            want = oracle.emb_forward(ref.work, rows, offsets, combiner, n_bags=batch * S)
            wmag = oracle.emb_forward(np.abs(ref.work), rows, offsets, combiner, n_bags=batch * S)
            assert_close(out.cpu().numpy().reshape(batch * S, dim), want, wmag, f"forward, pass {p}")
            layer.backward_sgd(batch, to_dev(keys), to_dev(dY), lr, d_off)
            g_abs = np.zeros_like(ref.work)
            oracle.emb_backward_sgd(g_abs, rows, np.abs(dY), -1.0, offsets, combiner, n_bags=batch * S)
            oracle.emb_backward_sgd(ref.work, rows, dY, lr, offsets, combiner, n_bags=batch * S)
            key_of_row = np.zeros(ref.stats[0], dtype=np.int64)
            key_of_row[ref.load(pass_keys)] = pass_keys
            mag[key_of_row] += lr * g_abs[:ref.stats[0]]
            # keep the two working tables together so that every batch is judged on its own
            n = ref.stats[0]
            got_work = etc.table[:n].cpu().numpy()
            assert_close(got_work, ref.work[:n], mag[key_of_row], f"working table, pass {p}")
            ref.work[:n] = got_work
        assert layer.invalid_keys() == 0
        etc.dump(evict=True)
        ref.dump(evict=True)
        torch.cuda.synchronize()
        assert np.array_equal(host.numpy(), ref_host), f"host table after pass {p}"   # same working rows, same copy
        assert np.count_nonzero((host.numpy() != before).any(axis=1)) > 100           # and training did reach it
