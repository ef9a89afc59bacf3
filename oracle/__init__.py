"""ctypes access to the CPU oracle (oracle.cpp).  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's cpu_baseline leg import this package; the
product package never does.  All arrays are numpy arrays on the host.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.cpp")
_LIB = os.path.join(_HERE, "liboracle.so")

F32, F16 = 0, 1
SUM, MEAN = 0, 1
EMPTY_TAG = np.uint64(0xFFFFFFFFFFFFFFFF)


def build(force: bool = True) -> str:
    """Compile oracle.cpp with g++ (no GPU toolchain involved).  With HCTR_SANITIZE=1 in the
    environment the library is built with UndefinedBehaviorSanitizer (any finding aborts), so the
    whole test suite can run on an instrumented oracle; AddressSanitizer cannot be loaded into a
    running Python, see sanitize_check() for that."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        extra = []
        if os.environ.get("HCTR_SANITIZE") == "1":
            extra = ["-g", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"]
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-shared", "-fPIC", "-pthread", "-Wall", "-Wextra"] + extra +
                              [_SRC, "-o", _LIB])
    return _LIB


def sanitize_check() -> str:
    """Builds oracle.cpp with sanitize_driver.cpp as one program under AddressSanitizer and
    UndefinedBehaviorSanitizer and runs it: the driver calls every function of the oracle on small
    seeded inputs.  Returns the program's output; raises if it reports anything."""
    out_dir = os.path.join(_HERE, "_build")
    os.makedirs(out_dir, exist_ok=True)
    exe = os.path.join(out_dir, "sanitize_driver")
    subprocess.check_call(["g++", "-O1", "-g", "-std=c++17", "-pthread", "-Wall", "-Wextra",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
                           "-static-libasan", "-static-libubsan",
                           _SRC, os.path.join(_HERE, "sanitize_driver.cpp"), "-o", exe])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    done = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    if done.returncode != 0:
        raise RuntimeError(f"sanitizer run failed ({done.returncode}):\n{done.stdout}\n{done.stderr}")
    return done.stdout


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        build(force=False)
        L = C.CDLL(_LIB)
        p, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
        L.oracle_rows_direct.restype = i64
        L.oracle_rows_direct.argtypes = [i32, p, p, i64, p, p, p]
        L.oracle_emb_forward.restype = None
        L.oracle_emb_forward.argtypes = [i32, i32, i32, p, i64, p, p, i64, p]
        L.oracle_emb_backward_sgd.restype = i64
        L.oracle_emb_backward_sgd.argtypes = [i32, i32, i32, p, i64, p, p, i64, p, f32, p, p]
        L.oracle_hardware_threads.restype = i32
        L.oracle_hardware_threads.argtypes = []
        L.oracle_rows_direct_mt.restype = i64
        L.oracle_rows_direct_mt.argtypes = [i32, i32, p, p, i64, p, p, p]
        L.oracle_emb_forward_mt.restype = None
        L.oracle_emb_forward_mt.argtypes = [i32, i32, i32, i32, p, i64, p, p, i64, p]
        L.oracle_emb_backward_sgd_mt.restype = i64
        L.oracle_emb_backward_sgd_mt.argtypes = [i32, i32, i32, i32, p, i64, p, p, i64, p, f32, p, p]
        L.oracle_emb_forward_mixed.restype = None
        L.oracle_emb_forward_mixed.argtypes = [i32, i32, i32, p, i64, p, p, i64, i32, p]
        L.oracle_emb_backward_sgd_mixed.restype = i64
        L.oracle_emb_backward_sgd_mixed.argtypes = [i32, i32, i32, p, p, i64, p, p, i64, i32, p, f32]
        L.oracle_group_forward.restype = None
        L.oracle_group_forward.argtypes = [i32, p, p, p, i32, i32, p, p, i64, p, p, p]
        L.oracle_group_backward_sgd.restype = i64
        L.oracle_group_backward_sgd.argtypes = [i32, p, p, p, i32, i32, p, p, i64, p, p, p, f32]
        L.oracle_hash_create.restype = p
        L.oracle_hash_create.argtypes = [i64]
        L.oracle_hash_destroy.restype = None
        L.oracle_hash_destroy.argtypes = [p]
        L.oracle_hash_size.restype = i64
        L.oracle_hash_size.argtypes = [p]
        L.oracle_hash_insert_or_find.restype = None
        L.oracle_hash_insert_or_find.argtypes = [p, p, i64, i32, p]
        L.oracle_cache_create.restype = p
        L.oracle_cache_create.argtypes = [i64, i32, i32, p, i64]
        L.oracle_cache_destroy.restype = None
        L.oracle_cache_destroy.argtypes = [p]
        L.oracle_cache_stats.restype = None
        L.oracle_cache_stats.argtypes = [p, p]
        L.oracle_cache_state.restype = None
        L.oracle_cache_state.argtypes = [p, p, p, p]
        L.oracle_cache_set_epoch_limit.restype = None
        L.oracle_cache_set_epoch_limit.argtypes = [p, C.c_uint32]
        L.oracle_cache_epoch.restype = C.c_uint32
        L.oracle_cache_epoch.argtypes = [p]
        L.oracle_cache_insert.restype = None
        L.oracle_cache_insert.argtypes = [p, p, i64]
        L.oracle_cache_update.restype = i64
        L.oracle_cache_update.argtypes = [p, p, p, i64]
        L.oracle_cache_refresh.restype = None
        L.oracle_cache_refresh.argtypes = [p]
        L.oracle_etc_create.restype = p
        L.oracle_etc_create.argtypes = [i64, i32, p, i64, p]
        L.oracle_etc_destroy.restype = None
        L.oracle_etc_destroy.argtypes = [p]
        L.oracle_etc_load.restype = None
        L.oracle_etc_load.argtypes = [p, p, i64, p]
        L.oracle_etc_dump.restype = None
        L.oracle_etc_dump.argtypes = [p, i32]
        L.oracle_etc_stats.restype = None
        L.oracle_etc_stats.argtypes = [p, p]
        L.oracle_cache_query_hits.restype = i64
        L.oracle_cache_query_hits.argtypes = [p, i64, p, p, i64, i64, p, p, p]
        L.oracle_cache_query_complete.restype = None
        L.oracle_cache_query_complete.argtypes = [p, i64, p, p, i64, i64, p, i32, p]
        L.oracle_cache_query.restype = None
        L.oracle_cache_query.argtypes = [p, i64, p, p, i64, i64, i32, p, p]
        _lib = L
    return _lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _i64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int64)


def _dtype_code(table: np.ndarray) -> int:
    if table.dtype == np.float32:
        return F32
    if table.dtype == np.float16:
        return F16
    raise TypeError("table must be float32 or float16")


def hardware_threads() -> int:
    """Threads the all-cores variants may use: the cores this process is allowed to run on."""
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:
        n = int(lib().oracle_hardware_threads())
    env = os.environ.get("OMP_NUM_THREADS", "")
    return max(1, min(n, int(env)) if env.isdigit() and int(env) > 0 else n)


def rows_direct(slot_base, slot_rows, keys, offsets=None, n_bags: Optional[int] = None,
                threads: int = 1) -> Tuple[np.ndarray, int]:
    """Global row per key (direct-index mode) and the number of keys without a row.
    Slot s owns rows [slot_base[s], slot_base[s] + slot_rows[s]) of the fused table.
    threads > 1: the all-cores variant (same result)."""
    slot_base, slot_rows, keys = _i64(slot_base), _i64(slot_rows), _i64(keys)
    S = len(slot_base)
    assert len(slot_rows) == S
    if offsets is not None:
        offsets = _i64(offsets)
        n_bags = len(offsets) - 1
    elif n_bags is None:
        n_bags = len(keys)
    rows = np.empty(len(keys), dtype=np.int64)
    if threads > 1:
        assert n_bags % S == 0
        bad = lib().oracle_rows_direct_mt(threads, S, _ptr(slot_base), _ptr(slot_rows), n_bags, _ptr(keys),
                                          _ptr(offsets), _ptr(rows))
    else:
        bad = lib().oracle_rows_direct(S, _ptr(slot_base), _ptr(slot_rows), n_bags, _ptr(keys),
                                       _ptr(offsets), _ptr(rows))
    return rows, int(bad)


def emb_forward(table: np.ndarray, rows, offsets=None, combiner: int = SUM,
                n_bags: Optional[int] = None, threads: int = 1) -> np.ndarray:
    """Pooled output [n_bags, D] float32.  threads > 1: the all-cores variant (same bits)."""
    assert table.ndim == 2 and table.flags.c_contiguous
    rows = _i64(rows)
    if offsets is not None:
        offsets = _i64(offsets)
        n_bags = len(offsets) - 1
    elif n_bags is None:
        n_bags = len(rows)
    out = np.empty((n_bags, table.shape[1]), dtype=np.float32)
    if threads > 1:
        lib().oracle_emb_forward_mt(threads, table.shape[1], _dtype_code(table), combiner, _ptr(table),
                                    table.shape[0], _ptr(rows), _ptr(offsets), n_bags, _ptr(out))
    else:
        lib().oracle_emb_forward(table.shape[1], _dtype_code(table), combiner, _ptr(table), table.shape[0],
                                 _ptr(rows), _ptr(offsets), n_bags, _ptr(out))
    return out


def emb_backward_sgd(table: np.ndarray, rows, dY: np.ndarray, lr: float, offsets=None,
                     combiner: int = SUM, n_bags: Optional[int] = None, threads: int = 1):
    """Updates `table` in place; returns (unique rows ascending, occurrence counts).
    threads > 1: the all-cores variant (same bits)."""
    assert table.ndim == 2 and table.flags.c_contiguous and table.flags.writeable
    rows = _i64(rows)
    if offsets is not None:
        offsets = _i64(offsets)
        n_bags = len(offsets) - 1
    elif n_bags is None:
        n_bags = len(rows)
    dY = np.ascontiguousarray(dY, dtype=np.float32).reshape(n_bags, table.shape[1])
    uniq = np.empty(max(1, len(rows)), dtype=np.int64)
    cnt = np.empty(max(1, len(rows)), dtype=np.int64)
    if threads > 1:
        u = lib().oracle_emb_backward_sgd_mt(threads, table.shape[1], _dtype_code(table), combiner, _ptr(table),
                                             table.shape[0], _ptr(rows), _ptr(offsets), n_bags, _ptr(dY),
                                             float(np.float32(lr)), _ptr(uniq), _ptr(cnt))
    else:
        u = lib().oracle_emb_backward_sgd(table.shape[1], _dtype_code(table), combiner, _ptr(table),
                                          table.shape[0], _ptr(rows), _ptr(offsets), n_bags, _ptr(dY),
                                          float(np.float32(lr)), _ptr(uniq), _ptr(cnt))
    return uniq[:u].copy(), cnt[:u].copy()


def emb_forward_mixed(table: np.ndarray, rows, offsets=None, combiner: int = SUM, n_bags: Optional[int] = None,
                      out_dtype=np.float16) -> np.ndarray:
    """Pooled output [n_bags, D] in out_dtype (float16: one rounding from the double sum)."""
    assert table.ndim == 2 and table.flags.c_contiguous
    rows = _i64(rows)
    if offsets is not None:
        offsets = _i64(offsets)
        n_bags = len(offsets) - 1
    elif n_bags is None:
        n_bags = len(rows)
    out = np.empty((n_bags, table.shape[1]), dtype=out_dtype)
    lib().oracle_emb_forward_mixed(table.shape[1], _dtype_code(table), combiner, _ptr(table), table.shape[0],
                                   _ptr(rows), _ptr(offsets), n_bags, _dtype_code(out), _ptr(out))
    return out


def emb_backward_sgd_mixed(table: np.ndarray, rows, dY: np.ndarray, lr: float, offsets=None, combiner: int = SUM,
                           n_bags: Optional[int] = None, master: Optional[np.ndarray] = None) -> int:
    """Backward + SGD with dY in its own dtype (float16 or float32) and an optional fp32 master copy
    of an fp16 table; updates table (and master) in place, returns the number of distinct rows."""
    assert table.ndim == 2 and table.flags.c_contiguous and table.flags.writeable
    rows = _i64(rows)
    if offsets is not None:
        offsets = _i64(offsets)
        n_bags = len(offsets) - 1
    elif n_bags is None:
        n_bags = len(rows)
    dY = np.ascontiguousarray(dY).reshape(n_bags, table.shape[1])
    if master is not None:
        assert master.dtype == np.float32 and master.shape == table.shape and master.flags.c_contiguous
        assert table.dtype == np.float16
    return int(lib().oracle_emb_backward_sgd_mixed(table.shape[1], _dtype_code(table), combiner, _ptr(table),
                                                   _ptr(master), table.shape[0], _ptr(rows), _ptr(offsets), n_bags,
                                                   _dtype_code(dY), _ptr(dY), float(np.float32(lr))))


def _group_args(tables, lookup_table, lookup_comb):
    assert len(tables) >= 1 and all(t.ndim == 2 and t.flags.c_contiguous and t.dtype == tables[0].dtype for t in tables)
    ptrs = (C.c_void_p * len(tables))(*[t.ctypes.data for t in tables])
    rows = np.array([t.shape[0] for t in tables], dtype=np.int64)
    dims = np.array([t.shape[1] for t in tables], dtype=np.int32)
    lt = np.ascontiguousarray(lookup_table, dtype=np.int32)
    lc = np.ascontiguousarray(lookup_comb, dtype=np.int32)
    assert len(lt) == len(lc) and lt.min() >= 0 and lt.max() < len(tables)
    width = int(dims[lt].sum())
    return ptrs, rows, dims, lt, lc, width


def dense_offsets(batch: int, hotness) -> np.ndarray:
    """CSR offsets of a dense input: every sample brings hotness[l] keys for lookup l."""
    per_bag = np.tile(np.asarray(hotness, dtype=np.int64), batch)
    return np.concatenate([[0], np.cumsum(per_bag)]).astype(np.int64)


def group_forward(tables, lookup_table, lookup_comb, batch: int, keys, offsets) -> np.ndarray:
    """Fused group of lookups: [batch, sum of the lookups' widths] float32."""
    ptrs, rows, dims, lt, lc, width = _group_args(tables, lookup_table, lookup_comb)
    keys, offsets = _i64(keys), _i64(offsets)
    assert len(offsets) == batch * len(lt) + 1
    out = np.empty((batch, width), dtype=np.float32)
    lib().oracle_group_forward(len(tables), ptrs, _ptr(rows), _ptr(dims), _dtype_code(tables[0]), len(lt),
                               _ptr(lt), _ptr(lc), batch, _ptr(keys), _ptr(offsets), _ptr(out))
    return out


def group_backward_sgd(tables, lookup_table, lookup_comb, batch: int, keys, offsets, dY, lr: float) -> int:
    """Updates the tables in place; returns the number of distinct (table, row) pairs touched."""
    ptrs, rows, dims, lt, lc, width = _group_args(tables, lookup_table, lookup_comb)
    assert all(t.flags.writeable for t in tables)
    keys, offsets = _i64(keys), _i64(offsets)
    assert len(offsets) == batch * len(lt) + 1
    dY = np.ascontiguousarray(dY, dtype=np.float32).reshape(batch, width)
    return int(lib().oracle_group_backward_sgd(len(tables), ptrs, _ptr(rows), _ptr(dims), _dtype_code(tables[0]),
                                               len(lt), _ptr(lt), _ptr(lc), batch, _ptr(keys), _ptr(offsets),
                                               _ptr(dY), float(np.float32(lr))))


class Hash:
    """Key -> dense row id in first-appearance order, capped at max_rows."""

    def __init__(self, max_rows: int):
        self._h = lib().oracle_hash_create(int(max_rows))
        self.max_rows = int(max_rows)

    def __del__(self):
        if getattr(self, "_h", None):
            lib().oracle_hash_destroy(self._h)
            self._h = None

    @property
    def size(self) -> int:
        return int(lib().oracle_hash_size(self._h))

    def insert_or_find(self, keys, insert: bool = True) -> np.ndarray:
        keys = _i64(keys)
        rows = np.empty(len(keys), dtype=np.int64)
        lib().oracle_hash_insert_or_find(self._h, _ptr(keys), len(keys), int(bool(insert)), _ptr(rows))
        return rows


class Cache:
    """Set-associative cache of host_table rows with call-granular LRU."""

    def __init__(self, num_sets: int, ways: int, host_table: np.ndarray):
        assert host_table.dtype == np.float32 and host_table.ndim == 2 and host_table.flags.c_contiguous
        self.host_table = host_table  # keep alive
        self.num_sets, self.ways, self.dim = int(num_sets), int(ways), host_table.shape[1]
        self._c = lib().oracle_cache_create(self.num_sets, self.ways, self.dim, _ptr(host_table),
                                            host_table.shape[0])

    def __del__(self):
        if getattr(self, "_c", None):
            lib().oracle_cache_destroy(self._c)
            self._c = None

    def set_epoch_limit(self, limit: int) -> None:
        """Call count at which stamps and count are lowered by limit / 2 (default 2^32 - 256)."""
        assert 2 <= limit <= 0xFFFFFF00
        lib().oracle_cache_set_epoch_limit(self._c, limit)

    @property
    def epoch(self) -> int:
        return int(lib().oracle_cache_epoch(self._c))

    def query(self, keys, n_bags: int, offsets=None, insert_missing: bool = True):
        """Returns (out [n_bags, D] float32, hit_mask [nnz] uint8)."""
        keys = _i64(keys)
        nnz = len(keys)
        hot = 0
        if offsets is not None:
            offsets = _i64(offsets)
            assert len(offsets) == n_bags + 1 and offsets[-1] == nnz
        else:
            assert n_bags > 0 and nnz % n_bags == 0
            hot = nnz // n_bags
        out = np.empty((n_bags, self.dim), dtype=np.float32)
        hit = np.zeros(nnz, dtype=np.uint8)
        lib().oracle_cache_query(self._c, n_bags, _ptr(keys), _ptr(offsets), hot, nnz,
                                 int(bool(insert_missing)), _ptr(out), _ptr(hit))
        return out, hit

    def _shape(self, keys, n_bags, offsets):
        keys = _i64(keys)
        nnz, hot = len(keys), 0
        if offsets is not None:
            offsets = _i64(offsets)
            assert len(offsets) == n_bags + 1 and offsets[-1] == nnz
        else:
            assert n_bags > 0 and nnz % n_bags == 0
            hot = nnz // n_bags
        return keys, offsets, nnz, hot

    def query_hits(self, keys, n_bags: int, offsets=None):
        """Phase 1 of a two-phase query: (out [n_bags, D] pooled over the hits only, hit_mask [nnz],
        positions of the missing keys inside the host table, ascending)."""
        keys, offsets, nnz, hot = self._shape(keys, n_bags, offsets)
        out = np.empty((n_bags, self.dim), dtype=np.float32)
        hit = np.zeros(nnz, dtype=np.uint8)
        miss = np.empty(max(1, nnz), dtype=np.int64)
        n = lib().oracle_cache_query_hits(self._c, n_bags, _ptr(keys), _ptr(offsets), hot, nnz, _ptr(out), _ptr(hit),
                                          _ptr(miss))
        return out, hit, miss[:n].copy()

    def query_complete(self, keys, n_bags: int, hit_mask: np.ndarray, out: np.ndarray, offsets=None,
                       insert_missing: bool = True) -> np.ndarray:
        """Phase 2: adds the missing keys' host rows into `out` (in place) and inserts them."""
        keys, offsets, nnz, hot = self._shape(keys, n_bags, offsets)
        assert out.dtype == np.float32 and out.shape == (n_bags, self.dim) and out.flags.c_contiguous
        hit_mask = np.ascontiguousarray(hit_mask, dtype=np.uint8)
        assert len(hit_mask) == nnz
        lib().oracle_cache_query_complete(self._c, n_bags, _ptr(keys), _ptr(offsets), hot, nnz, _ptr(hit_mask),
                                          int(bool(insert_missing)), _ptr(out))
        return out

    def insert(self, keys) -> None:
        keys = _i64(keys)
        lib().oracle_cache_insert(self._c, _ptr(keys), len(keys))

    def update(self, keys, rows: np.ndarray) -> int:
        """Overwrite the cached rows of resident keys (last row of a repeated key wins)."""
        keys = _i64(keys)
        rows = np.ascontiguousarray(rows, dtype=np.float32).reshape(len(keys), self.dim)
        return int(lib().oracle_cache_update(self._c, _ptr(keys), _ptr(rows), len(keys)))

    def refresh(self) -> None:
        """Every resident line re-reads its row from the host table (in place, as it is now)."""
        lib().oracle_cache_refresh(self._c)

    @property
    def stats(self) -> np.ndarray:
        """[queries, hits, misses, inserts, evictions, skipped inserts]"""
        s = np.zeros(6, dtype=np.int64)
        lib().oracle_cache_stats(self._c, _ptr(s))
        return s

    def state(self, with_data: bool = False):
        n = self.num_sets * self.ways
        tags = np.empty(n, dtype=np.uint64)
        stamps = np.empty(n, dtype=np.uint32)
        data = np.empty((n, self.dim), dtype=np.float32) if with_data else None
        lib().oracle_cache_state(self._c, _ptr(tags), _ptr(stamps), _ptr(data))
        tags = tags.reshape(self.num_sets, self.ways)
        stamps = stamps.reshape(self.num_sets, self.ways)
        return (tags, stamps, data) if with_data else (tags, stamps)


class Etc:
    """Embedding training cache staged in host memory: `host` [host_rows, D] float32 is the model (written
    by dump), `work` [max_rows, D] float32 is the working table training addresses through load's rows."""

    def __init__(self, host: np.ndarray, max_rows: int):
        assert host.dtype == np.float32 and host.ndim == 2 and host.flags.c_contiguous and host.flags.writeable
        self.host = host
        self.work = np.zeros((max_rows, host.shape[1]), dtype=np.float32)
        self._e = lib().oracle_etc_create(int(max_rows), host.shape[1], _ptr(host), host.shape[0], _ptr(self.work))

    def __del__(self):
        if getattr(self, "_e", None):
            lib().oracle_etc_destroy(self._e)
            self._e = None

    def load(self, keys) -> np.ndarray:
        keys = _i64(keys)
        rows = np.empty(len(keys), dtype=np.int64)
        lib().oracle_etc_load(self._e, _ptr(keys), len(keys), _ptr(rows))
        return rows

    def dump(self, evict: bool = True) -> None:
        lib().oracle_etc_dump(self._e, int(evict))

    @property
    def stats(self) -> Tuple[int, int, int, int]:
        """(resident keys, rows loaded, rejected key occurrences, occurrences outside the host table)."""
        out = np.zeros(4, dtype=np.int64)
        lib().oracle_etc_stats(self._e, _ptr(out))
        return tuple(int(x) for x in out)
