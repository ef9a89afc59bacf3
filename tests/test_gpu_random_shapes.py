"""GPU parity on seeded random combinations of the layer's parameters: slot count, table sizes, row
width, storage type, combiner, bag sizes, key skew, keys without a row.  Each case is the full
comparison of tests/test_gpu_emb.py (forward, dedup, backward + SGD, determinism) against the oracle;
the combinations reach paths that the hand-picked cases meet only one at a time (a width that is no
multiple of a wave's columns with bags of several chunks, a mean over bags with keys that have no
row, long runs in narrow rows, ...)."""
import os

import numpy as np
import pytest
import torch

from test_gpu_emb import run_case

pytestmark = pytest.mark.gpu


def _cases(n, seed):
    g = np.random.default_rng(seed)
    out = []
    for i in range(n):
        dtype = torch.float16 if g.random() < 0.5 else torch.float32
        mult = 8 if dtype == torch.float16 else 4
        dim = int(mult * g.choice([1, 2, 3, 4, 8, 13, 16, 25, 32, 48, 64, 96]))
        S = int(g.choice([1, 2, 3, 5, 26, 40]))
        rows = [int(x) for x in np.exp(g.uniform(np.log(2), np.log(20000), S)).astype(np.int64)]
        batch = int(g.choice([1, 7, 64, 130, 517, 1500]))
        kind = g.integers(0, 4)
        hot = None if kind == 0 else [(0, 4), (1, 40), (0, 150)][kind - 1]
        combiner = int(g.integers(0, 2))
        alpha = float(g.choice([0.0, 1.05, 1.4]))
        poison = int(g.choice([0, 0, 3, 40])) if batch * S >= 64 else 0
        out.append(pytest.param(rows, dim, batch, dtype, combiner, alpha, hot, poison, 1000 + i,
                                id=f"{i}-S{S}-D{dim}-{'f16' if dtype == torch.float16 else 'f32'}-B{batch}-"
                                   f"{'onehot' if hot is None else 'hot%d_%d' % hot}-{'mean' if combiner else 'sum'}"))
    return out


@pytest.mark.parametrize("rows,dim,batch,dtype,combiner,alpha,hot,poison,seed", _cases(int(os.environ.get("HCTR_TEST_CASES", "36")), 20221008))
def test_random_layer_configuration(rows, dim, batch, dtype, combiner, alpha, hot, poison, seed):
    run_case(rows, dim, batch, dtype=dtype, combiner=combiner, alpha=alpha, hot=hot, poison=poison, seed=seed)


def _group_cases(n, seed):
    g = np.random.default_rng(seed)
    out = []
    for i in range(n):
        f16 = bool(g.random() < 0.4)
        mult = 8 if f16 else 4
        n_tables = int(g.integers(1, 7))
        shapes = [(int(np.exp(g.uniform(0, np.log(6000)))) + 1, int(mult * g.choice([1, 2, 3, 4, 8, 16, 33, 64, 130])))
                  for _ in range(n_tables)]
        n_lookups = int(g.integers(1, 13))
        lookups = [(int(g.integers(0, n_tables)), int(g.integers(0, 2))) for _ in range(n_lookups)]
        batch = int(g.choice([1, 5, 64, 333, 2100]))
        dense = bool(g.random() < 0.5)
        hot = [int(g.integers(1, 6)) for _ in range(n_lookups)] if dense else None
        hmax = None if dense else int(g.choice([0, 1, 4, 12]))
        bad = int(g.choice([0, 0, 2, 10])) if batch * n_lookups >= 40 and (dense or hmax) else 0
        out.append(pytest.param(shapes, lookups, batch, np.float16 if f16 else np.float32, hmax, hot, bool(g.random() < 0.4),
                                bad, 3000 + i,
                                id=f"{i}-T{n_tables}-L{n_lookups}-B{batch}-{'f16' if f16 else 'f32'}-{'dense' if dense else 'sparse'}"))
    return out


@pytest.mark.parametrize("shapes,lookups,batch,dtype,hmax,hot,zipf,bad,seed",
                         _group_cases(int(os.environ.get("HCTR_TEST_CASES", "24")), 20221009))
def test_random_group_configuration(shapes, lookups, batch, dtype, hmax, hot, zipf, bad, seed):
    from test_gpu_group import run_case as run_group_case
    run_group_case(np.random.default_rng(seed), shapes, lookups, batch=batch, dtype=dtype, hmax=hmax, hot=hot,
                   zipf=zipf, bad=bad)


def _mixed_cases(n, seed):
    g = np.random.default_rng(seed)
    out = []
    for i in range(n):
        S = int(g.choice([1, 2, 4, 26]))
        rows = [int(x) + 1 for x in np.exp(g.uniform(0, np.log(8000), S)).astype(np.int64)]
        dim = int(8 * g.choice([1, 2, 4, 5, 8, 16, 32, 33]))
        batch = int(g.choice([1, 9, 200, 1100]))
        hot = [None, (0, 5), (1, 30), (0, 120)][int(g.integers(0, 4))]
        out.append(pytest.param(int(g.integers(0, 3)), rows, dim, batch, bool(g.random() < 0.5), hot, int(g.integers(0, 2)), 5000 + i,
                                id=f"{i}-S{S}-D{dim}-B{batch}"))
    return out


@pytest.mark.parametrize("kind,rows,dim,batch,half,hot,combiner,seed",
                         _mixed_cases(int(os.environ.get("HCTR_TEST_CASES", "24")), 20221010))
def test_random_mixed_precision_configuration(kind, rows, dim, batch, half, hot, combiner, seed):
    import test_gpu_mixed as m
    if kind == 0:
        m.check_fp16_output(rows, dim, batch, torch.float16 if half else torch.float32, hot, combiner, seed)
    elif kind == 1:
        m.check_fp16_gradient(rows, dim, batch, torch.float16 if half else torch.float32, hot, combiner, seed)
    else:
        m.check_master_rows(rows, dim, batch, torch.float16 if half else torch.float32, hot, combiner, seed)
