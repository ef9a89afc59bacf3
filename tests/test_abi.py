"""CPU-side checks of the C ABI: the library loads, exports every symbol the header declares, and
rejects bad arguments on the host before anything could be launched (no GPU needed)."""
import ctypes as C
import os
import re

import pytest

import paper_2210_08803_amd as H
from paper_2210_08803_amd.binding import EXPORTS, _EmbDesc, _GroupDesc, _GroupLookup, _GroupTable

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    text = open(os.path.join(ROOT, "include", "hctr.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hctr_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = H.lib()
    names = header_functions()
    assert len(names) >= 19
    for n in names:
        assert hasattr(L, n), n
    assert sorted(EXPORTS) == names


def _desc(**kw):
    base = (C.c_int64 * 2)(0, 10)
    num = (C.c_int64 * 2)(10, 5)
    d = _EmbDesc(num_slots=2, dim=8, table_dtype=H.F32, combiner=H.SUM, table=4096, total_rows=15,
                 slot_row_base=base, slot_num_rows=num, hash=None, insert_on_miss=0)
    d._keep = (base, num)
    for k, v in kw.items():
        setattr(d, k, v)
    return d


def _fwd(d, batch=1, keys=4096, offsets=None, nnz=2, out=4096, ws=4096, ws_bytes=1 << 30):
    return H.lib().hctr_emb_forward(C.byref(d), batch, keys, offsets, nnz, out, ws, ws_bytes, None)


def test_forward_argument_errors_are_caught_on_the_host():
    L = H.lib()
    assert L.hctr_emb_forward(None, 1, 4096, None, 2, 4096, 4096, 1 << 30, None) == -2
    assert _fwd(_desc(num_slots=0)) == -1
    assert _fwd(_desc(num_slots=129)) == -1
    assert _fwd(_desc(dim=6)) == -1                       # fp32 rows need a multiple of 4
    assert _fwd(_desc(dim=12, table_dtype=H.F16)) == -1   # fp16 rows need a multiple of 8
    assert _fwd(_desc(table_dtype=7)) == -1
    assert _fwd(_desc(combiner=3)) == -1
    assert _fwd(_desc(io_dtype=2)) == -1
    assert _fwd(_desc(master=8192)) == -1                 # master rows go with an fp16 table only
    assert _fwd(_desc(dim=8, table_dtype=H.F16, master=8196)) == -1   # misaligned master
    assert _fwd(_desc(table=None)) == -2
    assert _fwd(_desc(table=4100)) == -1                  # misaligned table
    assert _fwd(_desc(total_rows=0)) == -4
    assert _fwd(_desc(total_rows=14)) == -1               # slot 1 would leave the table
    assert _fwd(_desc(), nnz=3) == -1                     # one-hot needs nnz == batch*S
    assert _fwd(_desc(), batch=-1) == -1
    assert _fwd(_desc(), keys=None) == -2
    assert _fwd(_desc(), out=None) == -2
    assert _fwd(_desc(), out=4100) == -1
    assert _fwd(_desc(), ws=None) == -3
    assert _fwd(_desc(), ws=4100) == -3
    assert _fwd(_desc(), ws_bytes=16) == -3
    assert b"workspace" in L.hctr_last_error()
    d = _desc()
    assert L.hctr_emb_backward_sgd(C.byref(d), 1, 4096, None, 2, None, 0.1, 4096, 1 << 30, None) == -2
    need = L.hctr_emb_workspace_bytes(C.byref(d), 1, 2)
    assert need > 0 and need % 256 == 0
    assert L.hctr_emb_workspace_bytes(C.byref(d), 1, 1 << 20) > need


def _group(tables=((4096, 10, 8), (8192, 5, 16)), lookups=((0, 0, 1), (1, 1, 2), (0, 1, 1)), dtype=0):
    t = (_GroupTable * len(tables))()
    for i, (ptr, rows, dim) in enumerate(tables):
        t[i].data, t[i].num_rows, t[i].dim = ptr, rows, dim
    l = (_GroupLookup * len(lookups))()
    for i, (tb, comb, hot) in enumerate(lookups):
        l[i].table, l[i].combiner, l[i].hotness = tb, comb, hot
    d = _GroupDesc(num_tables=len(tables), num_lookups=len(lookups), table_dtype=dtype, tables=t, lookups=l)
    d._keep = (t, l)
    return d


def test_group_argument_errors_are_caught_on_the_host():
    L = H.lib()

    def fwd(d, batch=2, keys=4096, offsets=None, nnz=8, out=4096, ws=4096, ws_bytes=1 << 30):
        return L.hctr_group_forward(C.byref(d), batch, keys, offsets, nnz, out, ws, ws_bytes, None)

    assert L.hctr_group_forward(None, 1, 4096, None, 4, 4096, 4096, 1 << 30, None) == -2
    assert fwd(_group(tables=((4096, 10, 6),), lookups=((0, 0, 1),)), nnz=2) == -1       # width not a multiple of 4
    assert fwd(_group(tables=((4096, 10, 12),), lookups=((0, 0, 1),), dtype=1), nnz=2) == -1   # fp16: multiple of 8
    assert fwd(_group(tables=((None, 10, 8),), lookups=((0, 0, 1),)), nnz=2) == -2
    assert fwd(_group(tables=((4100, 10, 8),), lookups=((0, 0, 1),)), nnz=2) == -1       # misaligned table
    assert fwd(_group(tables=((4096, 0, 8),), lookups=((0, 0, 1),)), nnz=2) == -1
    assert fwd(_group(lookups=((2, 0, 1),)), nnz=2) == -1                                # table index out of range
    assert fwd(_group(lookups=((0, 5, 1),)), nnz=2) == -1                                # unknown combiner
    assert fwd(_group(lookups=((0, 0, 0),)), nnz=0) == -1                                # dense input needs hotness >= 1
    assert fwd(_group(), nnz=7) == -1                                                    # dense: nnz = batch * sum(hotness)
    assert fwd(_group(tables=((4096, 1 << 32, 8),), lookups=((0, 0, 1),)), nnz=2) == -4  # too many rows for the dedup
    assert fwd(_group(), keys=None) == -2
    assert fwd(_group(), out=None) == -2
    assert fwd(_group(), ws=None) == -3
    assert fwd(_group(), ws_bytes=64) == -3
    d = _group()
    assert L.hctr_group_backward_sgd(C.byref(d), 2, 4096, None, 8, None, 0.1, 4096, 1 << 30, None) == -2
    need = L.hctr_group_workspace_bytes(C.byref(d), 2, 8)
    assert need > 0 and need % 256 == 0
    assert L.hctr_group_workspace_bytes(C.byref(d), 1000, 8) > need       # room for the dense input's offsets
    assert L.hctr_group_workspace_bytes(None, 2, 8) == 0


def test_hash_and_cache_argument_errors():
    L = H.lib()
    h = C.c_void_p()
    assert L.hctr_hash_storage_bytes(10) == 0
    assert L.hctr_hash_storage_bytes(1024) == 256 + 128 * 128
    assert L.hctr_hash_create(None, 1 << 20, 1024, 100, None, C.byref(h)) == -2
    assert L.hctr_hash_create(4096, 1 << 20, 1024, 900, None, C.byref(h)) == -1   # above 0.8 * capacity
    assert L.hctr_hash_create(4096, 100, 1024, 100, None, C.byref(h)) == -1       # storage too small
    assert L.hctr_hash_create(4100, 1 << 20, 1024, 100, None, C.byref(h)) == -1   # misaligned
    assert L.hctr_hash_insert_or_find(None, 4096, 1, 1, 4096, 4096, 1 << 20, None) == -2
    assert L.hctr_hash_workspace_bytes(1000) % 256 == 0
    assert L.hctr_cache_storage_bytes(8, 3, 16) == 0      # ways must be a power of two
    assert L.hctr_cache_storage_bytes(8, 4, 6) == 0       # dim must be a multiple of 4
    assert L.hctr_cache_storage_bytes(0, 4, 8) == 0
    assert L.hctr_cache_storage_bytes(8, 4, 16) >= 8 * 4 * (8 + 4 + 64)
    c = C.c_void_p()
    assert L.hctr_cache_create(4096, 1 << 20, 8, 3, 16, 4096, 10, None, C.byref(c)) == -1
    assert L.hctr_cache_create(4096, 16, 8, 4, 16, 4096, 10, None, C.byref(c)) == -1
    assert L.hctr_cache_create(4096, 1 << 20, 8, 4, 16, None, 10, None, C.byref(c)) == -2
    assert L.hctr_cache_query(None, 1, 1, 4096, None, 1, 1, 4096, None, 4096, 1 << 20, None) == -2
    assert L.hctr_cache_set_epoch_limit(None, 100) == -2
    assert L.hctr_cache_set_small_call_limit(None, 100) == -2


def test_etc_argument_errors():
    L = H.lib()
    e = C.c_void_p()
    assert L.hctr_etc_storage_bytes(0) == 0
    assert L.hctr_etc_storage_bytes(1000) == 256 + 8192          # header + one key per row, rounded to 256
    assert L.hctr_etc_workspace_bytes(-1) == 0
    assert L.hctr_etc_workspace_bytes(1000) > 16000
    assert L.hctr_etc_create(None, 4096, 8, 4096, 10, 4096, 1 << 20, None, C.byref(e)) == -2
    assert L.hctr_etc_load(None, 4096, 4, None, 4096, 1 << 20, None) == -2
    assert L.hctr_etc_dump(None, 1, None) == -2
    assert L.hctr_etc_stats(None, None, None) == -2
    assert L.hctr_hash_clear(None, None) == -2


def test_workspace_bytes_serve_every_smaller_call():
    """A workspace sized for nnz_max keys must be accepted for every call with fewer keys, also
    where the layout changes with the key count (reduction window at 8 Mi keys, the sort's block
    shapes at 3 Mi and 4 Mi keys): sizes never shrink as nnz_max grows, and the size check that
    every call makes (shown here through hctr_emb_dedup_view, which does pointer arithmetic only)
    accepts the workspace of any larger nnz_max."""
    L = H.lib()
    base = (C.c_int64 * 1)(0)
    num = (C.c_int64 * 1)(1 << 28)
    d = _EmbDesc(num_slots=1, dim=128, table_dtype=H.F32, combiner=H.SUM, table=4096, total_rows=1 << 28,
                 slot_row_base=base, slot_num_rows=num, hash=None, insert_on_miss=0)
    switches = [48 * 16 * 4096, 1024 * 4096, 8 << 20]
    points = sorted({s + k for s in switches for k in (-4097, -1, 0, 1, 4097)} | {1, 1000, 10_000_000, 12_400_000, 90_000_000})
    sizes = [L.hctr_emb_workspace_bytes(C.byref(d), 1, n) for n in points]
    assert all(s > 0 for s in sizes)
    assert all(a <= b for a, b in zip(sizes, sizes[1:])), list(zip(points, sizes))
    for n_max in (10_000_000, 12_400_000, (8 << 20) + 1):
        have = L.hctr_emb_workspace_bytes(C.byref(d), 1, n_max)
        for n in (8 << 20, (8 << 20) - 5, 8_300_000, n_max):
            if n <= n_max:
                a, b, c = C.c_void_p(), C.c_void_p(), C.c_void_p()
                st = L.hctr_emb_dedup_view(C.byref(d), n, n, 4096, have, C.byref(a), C.byref(b), C.byref(c))
                assert st == 0, (n_max, n, L.hctr_last_error())
                assert L.hctr_emb_dedup_view(C.byref(d), n, n, 4096, 4096, C.byref(a), C.byref(b), C.byref(c)) == -3
    g = _group()
    gsizes = [L.hctr_group_workspace_bytes(C.byref(g), 2, n) for n in points]
    assert all(a <= b for a, b in zip(gsizes, gsizes[1:]))


def test_binding_compares_tensor_sizes_with_the_counts_of_the_call():
    """The C calls believe their counts; the binding, which sees the tensors, refuses a call whose
    offsets, output or gradient is shorter than the counts say (it would be read or written past its
    end on the device)."""
    import torch
    from paper_2210_08803_amd.binding import _sizes
    keys = torch.zeros(10, dtype=torch.int64)
    _sizes("ok", 5, keys, torch.zeros(6, dtype=torch.int64), out=(torch.zeros(40), 40), hit_mask=(None, 10))
    with pytest.raises(ValueError, match="offsets has 5 entries"):
        _sizes("short offsets", 5, keys, torch.zeros(5, dtype=torch.int64))
    with pytest.raises(ValueError, match="offsets has 7 entries"):
        _sizes("long offsets", 5, keys, torch.zeros(7, dtype=torch.int64))
    with pytest.raises(ValueError, match="int64"):
        _sizes("int32 keys", 5, keys.to(torch.int32), None)
    with pytest.raises(ValueError, match="int64"):
        _sizes("int32 offsets", 5, keys, torch.zeros(6, dtype=torch.int32))
    with pytest.raises(ValueError, match="out has 39 elements"):
        _sizes("short out", 5, keys, None, out=(torch.zeros(39), 40))
