"""ctypes binding of libhctr.so.  Names follow include/hctr.h; no arithmetic happens here."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
# HCTR_LIB points at another build of the same library (e.g. to compare two builds in one run)
_LIB_PATH = os.environ.get("HCTR_LIB") or os.path.join(HERE, "libhctr.so")

F32, F16 = 0, 1
SUM, MEAN = 0, 1
MAX_SLOTS = 128


class HctrError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"hctr status {status}: {text}")
        self.status = status


class _EmbDesc(C.Structure):
    _fields_ = [
        ("num_slots", C.c_int32), ("dim", C.c_int32), ("table_dtype", C.c_int32), ("combiner", C.c_int32),
        ("table", C.c_void_p), ("total_rows", C.c_int64),
        ("slot_row_base", C.POINTER(C.c_int64)), ("slot_num_rows", C.POINTER(C.c_int64)),
        ("hash", C.c_void_p), ("insert_on_miss", C.c_int32), ("io_dtype", C.c_int32),
        ("reuse_forward_rows", C.c_int32), ("master", C.c_void_p),
    ]


class _GroupTable(C.Structure):
    _fields_ = [("data", C.c_void_p), ("num_rows", C.c_int64), ("dim", C.c_int32), ("reserved", C.c_int32)]


class _GroupLookup(C.Structure):
    _fields_ = [("table", C.c_int32), ("combiner", C.c_int32), ("hotness", C.c_int32), ("reserved", C.c_int32)]


class _GroupDesc(C.Structure):
    _fields_ = [("num_tables", C.c_int32), ("num_lookups", C.c_int32), ("table_dtype", C.c_int32),
                ("reserved", C.c_int32), ("tables", C.POINTER(_GroupTable)), ("lookups", C.POINTER(_GroupLookup))]


_lib = None


def lib_path() -> str:
    return _LIB_PATH


def lib() -> C.CDLL:
    """Loads the built library; builds it first only when no library exists.  There is no other
    implementation to fall back to: a missing toolchain or library is an error."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from . import build as _build
        _build.build()
    L = C.CDLL(_LIB_PATH)
    p, i32, i64, sz, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t, C.c_float
    dp = C.POINTER(_EmbDesc)
    gp = C.POINTER(_GroupDesc)
    sig = {
        "hctr_group_workspace_bytes": (sz, [gp, i64, i64]),
        "hctr_group_forward": (i32, [gp, i64, p, p, i64, p, p, sz, p]),
        "hctr_group_backward_sgd": (i32, [gp, i64, p, p, i64, p, f32, p, sz, p]),
        "hctr_emb_workspace_bytes": (sz, [dp, i64, i64]),
        "hctr_emb_workspace_init": (i32, [p, sz, p]),
        "hctr_emb_forward": (i32, [dp, i64, p, p, i64, p, p, sz, p]),
        "hctr_emb_backward_sgd": (i32, [dp, i64, p, p, i64, p, f32, p, sz, p]),
        "hctr_emb_backward_dedup": (i32, [dp, i64, p, p, i64, p, sz, p]),
        "hctr_emb_backward_apply": (i32, [dp, i64, p, i64, p, f32, p, sz, p]),
        "hctr_emb_dedup_view": (i32, [dp, i64, i64, p, sz, C.POINTER(p), C.POINTER(p), C.POINTER(p)]),
        "hctr_emb_invalid_keys": (i32, [p, sz, p, C.POINTER(i64)]),
        "hctr_check_offsets": (i32, [p, i64, i64, p, sz, p]),
        "hctr_hash_storage_bytes": (sz, [i64]),
        "hctr_hash_create": (i32, [p, sz, i64, i64, p, C.POINTER(p)]),
        "hctr_hash_workspace_bytes": (sz, [i64]),
        "hctr_hash_insert_or_find": (i32, [p, p, i64, i32, p, p, sz, p]),
        "hctr_hash_size": (i32, [p, p, C.POINTER(i64)]),
        "hctr_hash_destroy": (None, [p]),
        "hctr_hash_clear": (i32, [p, p]),
        "hctr_etc_storage_bytes": (sz, [i64]),
        "hctr_etc_workspace_bytes": (sz, [i64]),
        "hctr_etc_create": (i32, [p, p, i32, p, i64, p, sz, p, C.POINTER(p)]),
        "hctr_etc_load": (i32, [p, p, i64, p, p, sz, p]),
        "hctr_etc_dump": (i32, [p, i32, p]),
        "hctr_etc_stats": (i32, [p, p, C.POINTER(i64)]),
        "hctr_etc_destroy": (None, [p]),
        "hctr_cache_storage_bytes": (sz, [i64, i32, i32]),
        "hctr_cache_create": (i32, [p, sz, i64, i32, i32, p, i64, p, C.POINTER(p)]),
        "hctr_cache_workspace_bytes": (sz, [p, i64]),
        "hctr_cache_set_small_call_limit": (i32, [p, i64]),
        "hctr_cache_set_epoch_limit": (i32, [p, i64]),
        "hctr_cache_query": (i32, [p, i64, i32, p, p, i64, i32, p, p, p, sz, p]),
        "hctr_cache_query_async": (i32, [p, i64, i32, p, p, i64, i32, p, p, p, sz, p, p]),
        "hctr_cache_query_static": (i32, [p, i64, i32, p, p, i64, i32, p, p, p]),
        "hctr_cache_query_hits": (i32, [p, i64, i32, p, p, i64, p, p, p, p, p, sz, p, p]),
        "hctr_cache_query_complete": (i32, [p, i64, i32, p, p, i64, i32, p, p, sz, p]),
        "hctr_cache_insert": (i32, [p, p, i64, p, sz, p]),
        "hctr_cache_update": (i32, [p, p, p, i64, p, sz, p]),
        "hctr_cache_refresh": (i32, [p, p]),
        "hctr_cache_stats": (i32, [p, p, C.POINTER(i64)]),
        "hctr_cache_state_view": (i32, [p, C.POINTER(p), C.POINTER(p), C.POINTER(p)]),
        "hctr_cache_destroy": (None, [p]),
        "hctr_last_error": (C.c_char_p, []),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype, fn.argtypes = res, args
    _lib = L
    return L


EXPORTS = [
    "hctr_emb_workspace_bytes", "hctr_emb_workspace_init", "hctr_emb_forward", "hctr_emb_backward_sgd", "hctr_emb_backward_dedup",
    "hctr_emb_backward_apply", "hctr_emb_dedup_view",
    "hctr_emb_invalid_keys", "hctr_check_offsets", "hctr_group_workspace_bytes", "hctr_group_forward", "hctr_group_backward_sgd",
    "hctr_hash_storage_bytes", "hctr_hash_create", "hctr_hash_workspace_bytes",
    "hctr_hash_insert_or_find", "hctr_hash_size", "hctr_hash_destroy", "hctr_hash_clear", "hctr_etc_storage_bytes",
    "hctr_etc_workspace_bytes", "hctr_etc_create", "hctr_etc_load", "hctr_etc_dump", "hctr_etc_stats",
    "hctr_etc_destroy", "hctr_cache_storage_bytes",
    "hctr_cache_create", "hctr_cache_workspace_bytes", "hctr_cache_set_small_call_limit", "hctr_cache_set_epoch_limit", "hctr_cache_query",
    "hctr_cache_query_async", "hctr_cache_query_static", "hctr_cache_query_hits",
    "hctr_cache_query_complete", "hctr_cache_insert", "hctr_cache_update", "hctr_cache_refresh", "hctr_cache_stats",
    "hctr_cache_state_view", "hctr_cache_destroy", "hctr_last_error",
]


def _check(status: int) -> None:
    if status != 0:
        raise HctrError(status, lib().hctr_last_error().decode())


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream: Optional[torch.cuda.Stream]) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream


def _ws(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(256, nbytes), dtype=torch.uint8, device=device)


def _sizes(what: str, n_bags: int, keys: Optional[torch.Tensor] = None, offsets: Optional[torch.Tensor] = None,
           **arrays) -> None:
    """The C calls take bare pointers and believe the counts they are given: a tensor shorter than the
    call says is read or written past its end on the device.  The tensors know their sizes, so the
    binding compares them before it hands the pointers over.  arrays: name=(tensor or None, least
    number of elements)."""
    if offsets is not None and offsets.numel() != n_bags + 1:
        raise ValueError(f"{what}: offsets has {offsets.numel()} entries, {n_bags} bags need {n_bags + 1}")
    if offsets is not None and offsets.dtype != torch.int64:
        raise ValueError(f"{what}: offsets must be int64")
    if keys is not None and keys.dtype != torch.int64:
        raise ValueError(f"{what}: keys must be int64")
    for name, (t, least) in arrays.items():
        if t is not None and t.numel() < least:
            raise ValueError(f"{what}: {name} has {t.numel()} elements, the call needs {least}")


def check_offsets(offsets: torch.Tensor, nnz: int, stream=None) -> None:
    """hctr_check_offsets: raises HctrError unless offsets is a valid CSR offset array for nnz keys."""
    ws = torch.empty(1, dtype=torch.int64, device=offsets.device)
    _check(lib().hctr_check_offsets(_ptr(offsets), offsets.numel() - 1, int(nnz), _ptr(ws), 8, _stream(stream)))


class behind_spacer:
    """Context manager: what is allocated inside lands behind `gib` GiB of device memory, which are
    given back on exit (later, smaller buffers may land there).

    Why: on MI355X the first 88 GiB of device memory that a process is handed in pieces of 8 GiB
    serve random row reads about 8 % slower than the memory handed out after them, while fills and
    copies run at the same rate everywhere (a gather of random 512-byte rows out of 8 GiB pieces
    allocated one after the other: 3.70 TB/s in pieces 0 to 10, 4.00 TB/s in all later ones, on
    every box looked at).  With the 85 GB table of the DLRM-shaped workload: forward / backward
    218 / 290 us with the table as the first allocation, 200 / 274 us behind the spacer, whatever
    the other buffers of the step are and wherever they lie (the 22 GB of the hashed workload and
    the tables of the fused group, allocated first, showed no difference).  A process that
    allocates a large table first therefore puts it in the slow place.  The spacer is allocated
    in pieces of 8 GiB because that is the request size for which the order in which the driver
    hands out its memory was seen to repeat: behind one 96 GiB allocation the table came to lie
    in the fast place on one day's boxes and in the slow place on another's.  This is a property
    of the machine, not of the kernels; it only pays for the first allocations of a process, and
    the spacer is skipped when less than `gib` + `room_for` bytes + 1 GiB are free."""

    PIECE = 8 << 30

    def __init__(self, gib: float = 96.0, room_for: int = 0, device="cuda"):
        self.gib, self.room_for, self.device, self._spacer = gib, int(room_for), device, None

    def __enter__(self):
        if self.gib > 0:
            free, _ = torch.cuda.mem_get_info(self.device)
            want = int(self.gib * (1 << 30))
            if free > self.room_for + want + (1 << 30):
                self._spacer = [torch.empty(min(self.PIECE, want - at), dtype=torch.uint8, device=self.device)
                                for at in range(0, want, self.PIECE)]
        return self

    def __exit__(self, *exc):
        if self._spacer is not None:
            self._spacer = None
            torch.cuda.empty_cache()
        return False


def allocate_table(num_rows: int, dim: int, dtype: torch.dtype = torch.float32, device="cuda",
                   spacer_gib: float = 96.0) -> torch.Tensor:
    """An uninitialised [num_rows, dim] device tensor for a large table, placed behind a spacer (see
    behind_spacer; spacer_gib 0: allocated the plain way)."""
    nbytes = int(num_rows) * int(dim) * torch.empty((), dtype=dtype).element_size()
    with behind_spacer(spacer_gib, nbytes, device):
        return torch.empty((int(num_rows), int(dim)), dtype=dtype, device=device)


class HashTable:
    """hctr_hash_*: key -> dense row id, rows assigned in first-appearance order."""

    def __init__(self, capacity: int, max_rows: int, device="cuda"):
        L = lib()
        nbytes = L.hctr_hash_storage_bytes(capacity)
        if nbytes == 0:
            raise HctrError(-1, "capacity out of range")
        self.storage = torch.empty(nbytes, dtype=torch.uint8, device=device)
        self.capacity, self.max_rows, self.device = capacity, max_rows, device
        h = C.c_void_p()
        _check(L.hctr_hash_create(self.storage.data_ptr(), nbytes, capacity, max_rows, _stream(None), C.byref(h)))
        self.handle = h
        self._wsbuf = None

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:   # at interpreter exit the module may be gone
            _lib.hctr_hash_destroy(self.handle)
            self.handle = None

    def workspace(self, n: int) -> torch.Tensor:
        need = lib().hctr_hash_workspace_bytes(n)
        if self._wsbuf is None or self._wsbuf.numel() < need:
            self._wsbuf = _ws(need, self.device)
        return self._wsbuf

    def insert_or_find(self, keys: torch.Tensor, insert: bool = True, rows: Optional[torch.Tensor] = None,
                       ws: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
        n = keys.numel()
        if rows is None:
            rows = torch.empty(n, dtype=torch.int64, device=keys.device)
        if ws is None:
            ws = self.workspace(n)
        _check(lib().hctr_hash_insert_or_find(self.handle, _ptr(keys), n, int(insert), _ptr(rows), _ptr(ws),
                                              ws.numel(), _stream(stream)))
        return rows

    @property
    def size(self) -> int:
        v = C.c_int64()
        _check(lib().hctr_hash_size(self.handle, _stream(None), C.byref(v)))
        return v.value

    def clear(self, stream=None) -> None:
        _check(lib().hctr_hash_clear(self.handle, _stream(stream)))


class EmbeddingLayer:
    """hctr_emb_*: fused multi-slot embedding over one table tensor [total_rows, dim]."""

    def __init__(self, table: torch.Tensor, num_slots: int, combiner: int = SUM,
                 slot_row_base: Optional[Sequence[int]] = None, slot_num_rows: Optional[Sequence[int]] = None,
                 hash_table: Optional[HashTable] = None, insert_on_miss: bool = True,
                 io_dtype: torch.dtype = torch.float32, master: Optional[torch.Tensor] = None,
                 reuse_forward_rows: bool = False):
        assert table.is_cuda and table.is_contiguous() and table.dim() == 2
        assert io_dtype in (torch.float32, torch.float16)
        if master is not None:
            assert master.is_cuda and master.is_contiguous() and master.dtype == torch.float32
            assert master.shape == table.shape
        self.io_dtype, self.master = io_dtype, master
        self.table, self.num_slots, self.combiner = table, num_slots, combiner
        self.hash_table = hash_table
        d = _EmbDesc()
        d.num_slots, d.dim = num_slots, table.shape[1]
        d.table_dtype = F32 if table.dtype == torch.float32 else F16
        assert table.dtype in (torch.float32, torch.float16)
        d.combiner = combiner
        d.table, d.total_rows = table.data_ptr(), table.shape[0]
        if hash_table is None:
            self._base = (C.c_int64 * num_slots)(*[int(x) for x in slot_row_base])
            self._num = (C.c_int64 * num_slots)(*[int(x) for x in slot_num_rows])
            d.slot_row_base, d.slot_num_rows = self._base, self._num
            d.hash = None
        else:
            d.hash = hash_table.handle
        d.insert_on_miss = int(insert_on_miss)
        d.io_dtype = F32 if io_dtype == torch.float32 else F16
        d.master = None if master is None else master.data_ptr()
        d.reuse_forward_rows = int(reuse_forward_rows)
        self.desc = d
        self._wsbuf = None
        self._invalid_carry = 0   # keys without a row counted on earlier, smaller workspaces of the layer

    def workspace_bytes(self, batch: int, nnz: int) -> int:
        return lib().hctr_emb_workspace_bytes(C.byref(self.desc), batch, nnz)

    def workspace(self, batch: int, nnz: int, stream=None) -> torch.Tensor:
        """The layer's own workspace, grown when a call needs more.  Growing replaces the buffer: the
        count of keys without a row seen so far is carried over (invalid_keys() keeps adding up), but
        the rows a forward left for a reuse_forward_rows backward would be lost, so that case raises."""
        need = self.workspace_bytes(batch, nnz)
        if self._wsbuf is None or self._wsbuf.numel() < need:
            if self._wsbuf is not None:
                if self.desc.reuse_forward_rows:
                    raise HctrError(-3, "the layer's workspace would have to grow between a forward and the "
                                        "backward that reuses its rows; size it for the largest call first")
                self._invalid_carry += self.invalid_keys(self._wsbuf)   # explicit buffer: its own count only
            self._wsbuf = self.new_workspace(need, stream)
        return self._wsbuf

    def new_workspace(self, nbytes: int, stream=None) -> torch.Tensor:
        """A fresh workspace, initialised on `stream` (the stream its first call will use)."""
        ws = _ws(nbytes, self.table.device)
        _check(lib().hctr_emb_workspace_init(_ptr(ws), ws.numel(), _stream(stream)))
        return ws

    def reset_invalid_keys(self, ws: Optional[torch.Tensor] = None, stream=None) -> None:
        if ws is None:
            ws, self._invalid_carry = self._wsbuf, 0
        _check(lib().hctr_emb_workspace_init(_ptr(ws), ws.numel(), _stream(stream)))

    def forward(self, batch: int, keys: torch.Tensor, offsets: Optional[torch.Tensor] = None,
                out: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
        nnz = keys.numel()
        if out is None:
            out = torch.empty((batch, self.num_slots, self.table.shape[1]), dtype=self.io_dtype,
                              device=self.table.device)
        assert out.dtype == self.io_dtype
        n_bags = batch * self.num_slots
        _sizes("forward", n_bags, keys, offsets, out=(out, n_bags * self.table.shape[1]))
        if ws is None:
            ws = self.workspace(batch, nnz, stream)
        _check(lib().hctr_emb_forward(C.byref(self.desc), batch, _ptr(keys), _ptr(offsets), nnz, _ptr(out),
                                      _ptr(ws), ws.numel(), _stream(stream)))
        return out

    def backward_sgd(self, batch: int, keys: torch.Tensor, dY: torch.Tensor, lr: float,
                     offsets: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None, stream=None) -> None:
        nnz = keys.numel()
        assert dY.dtype == self.io_dtype and dY.is_contiguous()
        n_bags = batch * self.num_slots
        _sizes("backward_sgd", n_bags, keys, offsets, dY=(dY, n_bags * self.table.shape[1]))
        if ws is None:
            ws = self.workspace(batch, nnz, stream)
        _check(lib().hctr_emb_backward_sgd(C.byref(self.desc), batch, _ptr(keys), _ptr(offsets), nnz, _ptr(dY),
                                           float(lr), _ptr(ws), ws.numel(), _stream(stream)))

    def backward_dedup(self, batch: int, keys: torch.Tensor, offsets: Optional[torch.Tensor] = None,
                       ws: Optional[torch.Tensor] = None, stream=None) -> None:
        nnz = keys.numel()
        _sizes("backward_dedup", batch * self.num_slots, keys, offsets)
        if ws is None:
            ws = self.workspace(batch, nnz, stream)
        _check(lib().hctr_emb_backward_dedup(C.byref(self.desc), batch, _ptr(keys), _ptr(offsets), nnz,
                                             _ptr(ws), ws.numel(), _stream(stream)))

    def backward_apply(self, batch: int, nnz: int, dY: torch.Tensor, lr: float,
                       offsets: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None,
                       stream=None) -> None:
        assert dY.dtype == self.io_dtype and dY.is_contiguous()
        n_bags = batch * self.num_slots
        _sizes("backward_apply", n_bags, None, offsets, dY=(dY, n_bags * self.table.shape[1]))
        if ws is None:
            ws = self.workspace(batch, nnz, stream)
        _check(lib().hctr_emb_backward_apply(C.byref(self.desc), batch, _ptr(offsets), nnz, _ptr(dY),
                                             float(lr), _ptr(ws), ws.numel(), _stream(stream)))

    def dedup_result(self, batch: int, nnz: int, ws: Optional[torch.Tensor] = None):
        """(unique rows uint32-as-int64 [U], occurrence counts [U]) of the last backward on ws."""
        ws = ws if ws is not None else self._wsbuf
        pu, pr, ps = C.c_void_p(), C.c_void_p(), C.c_void_p()
        _check(lib().hctr_emb_dedup_view(C.byref(self.desc), batch, nnz, _ptr(ws), ws.numel(),
                                         C.byref(pu), C.byref(pr), C.byref(ps)))
        torch.cuda.synchronize()
        base = ws.data_ptr()
        u = int(ws[pu.value - base: pu.value - base + 8].view(torch.int64).item())
        rows = ws[pr.value - base: pr.value - base + 4 * u].view(torch.int32).to(torch.int64) & 0xFFFFFFFF
        seg = ws[ps.value - base: ps.value - base + 4 * (u + 1)].view(torch.int32).to(torch.int64) & 0xFFFFFFFF
        return rows, seg[1:] - seg[:-1]

    def invalid_keys(self, ws: Optional[torch.Tensor] = None) -> int:
        """Keys without a row counted on `ws`; for the layer's own workspace (ws None) the total over
        all the buffers it has had."""
        carry = self._invalid_carry if ws is None else 0
        ws = ws if ws is not None else self._wsbuf
        v = C.c_int64()
        _check(lib().hctr_emb_invalid_keys(_ptr(ws), ws.numel(), _stream(None), C.byref(v)))
        return v.value + carry


class EmbeddingGroup:
    """hctr_group_*: fused lookups over tables of different widths.  `tables`: 2-D device tensors of one
    dtype; `lookups`: (table index, combiner[, hotness]) per lookup.  Dense input = offsets None."""

    def __init__(self, tables: Sequence[torch.Tensor], lookups: Sequence[Sequence[int]]):
        assert len(tables) >= 1 and all(t.is_cuda and t.is_contiguous() and t.dim() == 2 for t in tables)
        assert all(t.dtype == tables[0].dtype for t in tables) and tables[0].dtype in (torch.float32, torch.float16)
        self.tables = list(tables)
        self.lookups = [tuple(l) + (1,) * (3 - len(l)) for l in lookups]
        self._t = (_GroupTable * len(tables))()
        for i, t in enumerate(tables):
            self._t[i].data, self._t[i].num_rows, self._t[i].dim = t.data_ptr(), t.shape[0], t.shape[1]
        self._l = (_GroupLookup * len(self.lookups))()
        for i, (t, c, h) in enumerate(self.lookups):
            self._l[i].table, self._l[i].combiner, self._l[i].hotness = int(t), int(c), int(h)
        d = _GroupDesc()
        d.num_tables, d.num_lookups = len(tables), len(self.lookups)
        d.table_dtype = F32 if tables[0].dtype == torch.float32 else F16
        d.tables, d.lookups = self._t, self._l
        self.desc = d
        self.width = sum(tables[t].shape[1] for t, _, _ in self.lookups)
        self.device = tables[0].device
        self._wsbuf = None

    def workspace_bytes(self, batch: int, nnz: int) -> int:
        return lib().hctr_group_workspace_bytes(C.byref(self.desc), batch, nnz)

    def new_workspace(self, nbytes: int) -> torch.Tensor:
        ws = _ws(nbytes, self.device)
        _check(lib().hctr_emb_workspace_init(_ptr(ws), ws.numel(), _stream(None)))
        return ws

    def workspace(self, batch: int, nnz: int) -> torch.Tensor:
        need = self.workspace_bytes(batch, nnz)
        if self._wsbuf is None or self._wsbuf.numel() < need:
            self._wsbuf = self.new_workspace(need)
        return self._wsbuf

    def forward(self, batch: int, keys: torch.Tensor, offsets: Optional[torch.Tensor] = None,
                out: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
        nnz = keys.numel()
        if out is None:
            out = torch.empty((batch, self.width), dtype=torch.float32, device=self.device)
        _sizes("group forward", batch * len(self.lookups), keys, offsets, out=(out, batch * self.width))
        if ws is None:
            ws = self.workspace(batch, nnz)
        _check(lib().hctr_group_forward(C.byref(self.desc), batch, _ptr(keys), _ptr(offsets), nnz, _ptr(out),
                                        _ptr(ws), ws.numel(), _stream(stream)))
        return out

    def backward_sgd(self, batch: int, keys: torch.Tensor, dY: torch.Tensor, lr: float,
                     offsets: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None, stream=None) -> None:
        nnz = keys.numel()
        _sizes("group backward_sgd", batch * len(self.lookups), keys, offsets, dY=(dY, batch * self.width))
        if ws is None:
            ws = self.workspace(batch, nnz)
        _check(lib().hctr_group_backward_sgd(C.byref(self.desc), batch, _ptr(keys), _ptr(offsets), nnz, _ptr(dY),
                                             float(lr), _ptr(ws), ws.numel(), _stream(stream)))

    def invalid_keys(self, ws: Optional[torch.Tensor] = None) -> int:
        ws = ws if ws is not None else self._wsbuf
        v = C.c_int64()
        _check(lib().hctr_emb_invalid_keys(_ptr(ws), ws.numel(), _stream(None), C.byref(v)))
        return v.value


class EmbeddingTrainingCache:
    """hctr_etc_*: the model in pinned host memory, the rows of a pass in a working table on the GPU.
    `layer(...)` gives the hashed-mode layer that trains on the working table."""

    def __init__(self, host_table: torch.Tensor, max_rows: int, capacity: Optional[int] = None, device="cuda"):
        assert host_table.is_pinned() and host_table.dtype == torch.float32 and host_table.is_contiguous()
        L = lib()
        self.host_table, self.max_rows, self.device = host_table, max_rows, device
        self.hash_table = HashTable(capacity if capacity is not None else max(64, int(max_rows / 0.75) + 8), max_rows,
                                    device)
        self.table = torch.zeros((max_rows, host_table.shape[1]), dtype=torch.float32, device=device)
        nbytes = L.hctr_etc_storage_bytes(max_rows)
        self.storage = torch.empty(nbytes, dtype=torch.uint8, device=device)
        h = C.c_void_p()
        _check(L.hctr_etc_create(self.hash_table.handle, self.table.data_ptr(), host_table.shape[1],
                                 host_table.data_ptr(), host_table.shape[0], self.storage.data_ptr(), nbytes,
                                 _stream(None), C.byref(h)))
        self.handle = h
        self._wsbuf = None

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:   # at interpreter exit the module may be gone
            _lib.hctr_etc_destroy(self.handle)
            self.handle = None

    def workspace(self, n: int) -> torch.Tensor:
        need = lib().hctr_etc_workspace_bytes(n)
        if self._wsbuf is None or self._wsbuf.numel() < need:
            self._wsbuf = _ws(need, self.device)
        return self._wsbuf

    def load(self, keys: torch.Tensor, rows: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None,
             stream=None) -> Optional[torch.Tensor]:
        n = keys.numel()
        if ws is None:
            ws = self.workspace(n)
        _check(lib().hctr_etc_load(self.handle, _ptr(keys), n, _ptr(rows), _ptr(ws), ws.numel(), _stream(stream)))
        return rows

    def dump(self, evict: bool = True, stream=None) -> None:
        _check(lib().hctr_etc_dump(self.handle, int(evict), _stream(stream)))

    def layer(self, num_slots: int, combiner: int = SUM, reuse_forward_rows: bool = False) -> "EmbeddingLayer":
        return EmbeddingLayer(self.table, num_slots, combiner, hash_table=self.hash_table, insert_on_miss=False,
                              reuse_forward_rows=reuse_forward_rows)

    @property
    def stats(self):
        out = (C.c_int64 * 4)()
        _check(lib().hctr_etc_stats(self.handle, _stream(None), out))
        return tuple(out)


class EmbeddingCache:
    """hctr_cache_*: set-associative GPU cache over a pinned host table [host_rows, dim] fp32."""

    def __init__(self, num_sets: int, ways: int, host_table: torch.Tensor, device="cuda"):
        assert host_table.dtype == torch.float32 and host_table.dim() == 2 and host_table.is_contiguous()
        assert host_table.is_pinned(), "host_table must be pinned (device-mapped) host memory"
        L = lib()
        self.host_table, self.device = host_table, device
        self.num_sets, self.ways, self.dim = num_sets, ways, host_table.shape[1]
        nbytes = L.hctr_cache_storage_bytes(num_sets, ways, self.dim)
        if nbytes == 0:
            raise HctrError(-1, "cache shape out of range")
        self.storage = torch.empty(nbytes, dtype=torch.uint8, device=device)
        h = C.c_void_p()
        _check(L.hctr_cache_create(self.storage.data_ptr(), nbytes, num_sets, ways, self.dim,
                                   host_table.data_ptr(), host_table.shape[0], _stream(None), C.byref(h)))
        self.handle = h
        self._wsbuf = None

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:   # at interpreter exit the module may be gone
            _lib.hctr_cache_destroy(self.handle)
            self.handle = None

    def set_small_call_limit(self, max_keys: int) -> None:
        _check(lib().hctr_cache_set_small_call_limit(self.handle, max_keys))

    def set_epoch_limit(self, limit: int) -> None:
        _check(lib().hctr_cache_set_epoch_limit(self.handle, limit))

    def workspace(self, nnz: int) -> torch.Tensor:
        need = lib().hctr_cache_workspace_bytes(self.handle, nnz)
        if self._wsbuf is None or self._wsbuf.numel() < need:
            self._wsbuf = _ws(need, self.device)
        return self._wsbuf

    def query(self, batch: int, num_slots: int, keys: torch.Tensor, offsets: Optional[torch.Tensor] = None,
              insert_missing: bool = True, out: Optional[torch.Tensor] = None,
              hit_mask: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None, stream=None):
        nnz = keys.numel()
        if out is None:
            out = torch.empty((batch, num_slots, self.dim), dtype=torch.float32, device=self.device)
        _sizes("cache query", batch * num_slots, keys, offsets, out=(out, batch * num_slots * self.dim),
               hit_mask=(hit_mask, nnz))
        if ws is None:
            ws = self.workspace(nnz)
        _check(lib().hctr_cache_query(self.handle, batch, num_slots, _ptr(keys), _ptr(offsets), nnz,
                                      int(insert_missing), _ptr(out), _ptr(hit_mask), _ptr(ws), ws.numel(),
                                      _stream(stream)))
        return out

    def query_static(self, batch: int, num_slots: int, keys: torch.Tensor, out: torch.Tensor,
                     offsets: Optional[torch.Tensor] = None, insert_missing: bool = True,
                     hit_mask: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
        """hctr_cache_query_static: the query without a workspace argument; the caller brings `out`."""
        _sizes("cache query_static", batch * num_slots, keys, offsets, out=(out, batch * num_slots * self.dim),
               hit_mask=(hit_mask, keys.numel()))
        _check(lib().hctr_cache_query_static(self.handle, batch, num_slots, _ptr(keys), _ptr(offsets), keys.numel(),
                                             int(insert_missing), _ptr(out), _ptr(hit_mask), _stream(stream)))
        return out

    def query_hits(self, batch: int, num_slots: int, keys: torch.Tensor, out: torch.Tensor,
                   offsets: Optional[torch.Tensor] = None, hit_mask: Optional[torch.Tensor] = None,
                   miss_positions: Optional[torch.Tensor] = None, n_missing: Optional[torch.Tensor] = None,
                   ws: Optional[torch.Tensor] = None, stream=None, ready: Optional[torch.cuda.Event] = None):
        """hctr_cache_query_hits: first phase, pools the hits only.  `ready` must be an event that has been
        recorded once already (torch creates the underlying event on the first record)."""
        nnz = keys.numel()
        _sizes("cache query_hits", batch * num_slots, keys, offsets, out=(out, batch * num_slots * self.dim),
               hit_mask=(hit_mask, nnz), miss_positions=(miss_positions, nnz), n_missing=(n_missing, 1))
        if ws is None:
            ws = self.workspace(nnz)
        _check(lib().hctr_cache_query_hits(self.handle, batch, num_slots, _ptr(keys), _ptr(offsets), nnz, _ptr(out),
                                           _ptr(hit_mask), _ptr(miss_positions), _ptr(n_missing), _ptr(ws), ws.numel(),
                                           _stream(stream), None if ready is None else ready.cuda_event))
        return out

    def query_complete(self, batch: int, num_slots: int, keys: torch.Tensor, out: torch.Tensor,
                       offsets: Optional[torch.Tensor] = None, insert_missing: bool = True,
                       ws: Optional[torch.Tensor] = None, stream=None):
        """hctr_cache_query_complete: second phase, adds the missing rows into `out` and inserts them."""
        nnz = keys.numel()
        _sizes("cache query_complete", batch * num_slots, keys, offsets, out=(out, batch * num_slots * self.dim))
        if ws is None:
            ws = self.workspace(nnz)
        _check(lib().hctr_cache_query_complete(self.handle, batch, num_slots, _ptr(keys), _ptr(offsets), nnz,
                                               int(insert_missing), _ptr(out), _ptr(ws), ws.numel(), _stream(stream)))
        return out

    def query_async(self, batch: int, num_slots: int, keys: torch.Tensor, ready: torch.cuda.Event,
                    offsets: Optional[torch.Tensor] = None, insert_missing: bool = True,
                    out: Optional[torch.Tensor] = None, hit_mask: Optional[torch.Tensor] = None,
                    ws: Optional[torch.Tensor] = None, stream=None):
        """As query(); `ready` (a torch.cuda.Event) fires when out / hit_mask are complete."""
        nnz = keys.numel()
        if out is None:
            out = torch.empty((batch, num_slots, self.dim), dtype=torch.float32, device=self.device)
        _sizes("cache query_async", batch * num_slots, keys, offsets, out=(out, batch * num_slots * self.dim),
               hit_mask=(hit_mask, nnz))
        if ws is None:
            ws = self.workspace(nnz)
        if not ready.cuda_event:   # torch creates the underlying event on its first record
            ready.record(torch.cuda.current_stream() if stream is None else stream)
        _check(lib().hctr_cache_query_async(self.handle, batch, num_slots, _ptr(keys), _ptr(offsets), nnz,
                                            int(insert_missing), _ptr(out), _ptr(hit_mask), _ptr(ws),
                                            ws.numel(), _stream(stream), ready.cuda_event))
        return out

    def insert(self, keys: torch.Tensor, ws: Optional[torch.Tensor] = None, stream=None) -> None:
        if ws is None:
            ws = self.workspace(keys.numel())
        _check(lib().hctr_cache_insert(self.handle, _ptr(keys), keys.numel(), _ptr(ws), ws.numel(), _stream(stream)))

    def update(self, keys: torch.Tensor, rows: torch.Tensor, ws: Optional[torch.Tensor] = None, stream=None) -> None:
        assert rows.dtype == torch.float32 and rows.is_contiguous() and rows.shape == (keys.numel(), self.dim)
        if ws is None:
            ws = self.workspace(keys.numel())
        _check(lib().hctr_cache_update(self.handle, _ptr(keys), _ptr(rows), keys.numel(), _ptr(ws), ws.numel(),
                                       _stream(stream)))

    def refresh(self, stream=None) -> None:
        _check(lib().hctr_cache_refresh(self.handle, _stream(stream)))

    @property
    def stats(self):
        arr = (C.c_int64 * 6)()
        _check(lib().hctr_cache_stats(self.handle, _stream(None), arr))
        return list(arr)

    def state(self):
        """(tags [num_sets, ways] int64 bit patterns, stamps [num_sets, ways] int64) copied to host."""
        pt, ps, pd = C.c_void_p(), C.c_void_p(), C.c_void_p()
        _check(lib().hctr_cache_state_view(self.handle, C.byref(pt), C.byref(ps), C.byref(pd)))
        torch.cuda.synchronize()
        base, n = self.storage.data_ptr(), self.num_sets * self.ways
        tags = self.storage[pt.value - base: pt.value - base + 8 * n].view(torch.int64).view(self.num_sets, self.ways)
        stamps = self.storage[ps.value - base: ps.value - base + 4 * n].view(torch.int32).view(self.num_sets, self.ways)
        return tags.cpu(), stamps.cpu().to(torch.int64) & 0xFFFFFFFF

    def data(self) -> torch.Tensor:
        pt, ps, pd = C.c_void_p(), C.c_void_p(), C.c_void_p()
        _check(lib().hctr_cache_state_view(self.handle, C.byref(pt), C.byref(ps), C.byref(pd)))
        base, n = self.storage.data_ptr(), self.num_sets * self.ways
        off = pd.value - base
        return self.storage[off: off + 4 * n * self.dim].view(torch.float32).view(n, self.dim)
