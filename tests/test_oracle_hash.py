"""Pins for the oracle's key -> row hash (section 1, the "embedding hash" layers): hand-worked
traces from tests/golden and invariants that hold for any correct insert-or-find."""
import json
import os

import numpy as np

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden", "hash_first_appearance.json")
RNG = np.random.default_rng(5)


def test_hand_worked_traces():
    for case in json.load(open(GOLD))["cases"]:
        h = oracle.Hash(case["max_rows"])
        for call in case["calls"]:
            rows = h.insert_or_find(np.array(call["keys"], dtype=np.int64), bool(call["insert"]))
            assert rows.tolist() == call["rows"]
            assert h.size == call["size"]


def test_invariants_on_random_streams():
    h = oracle.Hash(500)
    seen = {}
    for _ in range(10):
        keys = RNG.integers(0, 400, 300)
        rows = h.insert_or_find(keys, True)
        for k, r in zip(keys.tolist(), rows.tolist()):
            assert seen.setdefault(k, r) == r           # a key never changes row
        vals = sorted(set(seen.values()))
        assert vals == list(range(len(vals))) == list(range(h.size))   # dense and injective
        size = h.size
        assert np.array_equal(h.insert_or_find(keys, True), rows) and h.size == size   # idempotent
        assert np.array_equal(h.insert_or_find(keys, False), rows) and h.size == size  # find-only


def test_first_appearance_order_via_numpy_unique():
    keys = RNG.integers(0, 1 << 62, 2000)
    keys = np.concatenate([keys, keys[RNG.integers(0, 2000, 3000)]])
    RNG.shuffle(keys)
    rows = oracle.Hash(10**6).insert_or_find(keys, True)
    _, first = np.unique(keys, return_index=True)
    order = np.sort(first)                               # positions of first appearances, ascending
    assert np.array_equal(rows[order], np.arange(len(order)))
    # splitting one call in two gives the same mapping (true for first-appearance order only)
    h2 = oracle.Hash(10**6)
    r2 = np.concatenate([h2.insert_or_find(keys[:1234], True), h2.insert_or_find(keys[1234:], True)])
    assert np.array_equal(r2, rows)


def test_exact_fill_and_overflow_by_one():
    h = oracle.Hash(8)
    assert h.insert_or_find(np.arange(100, 108), True).tolist() == list(range(8)) and h.size == 8
    assert h.insert_or_find(np.array([108, 100]), True).tolist() == [-1, 0] and h.size == 8
