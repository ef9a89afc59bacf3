"""Seeded synthetic input generators (shared by the CPU oracle's tests and the HIP path's tests).

This module produces INPUTS only: table sizes, table contents, categorical keys, CSR offsets and
upstream gradients with the shapes of a 26-slot DLRM-like recommender (the paper's training
benchmark is MLPerf DLRM on Criteo Terabyte, which is a dataset this repository does not ship;
these generators stand in for it).  It holds none of the embedding method's arithmetic: no lookup,
no pooling, no dedup, no update, no hashing of keys into tables or cache sets.

Everything is a pure function of an explicit 64-bit seed.  Random bits come from a counter-based
generator (the public-domain splitmix64 output function applied to seed/stream/counter), written
with integer tensor ops so the same code runs on CPU and GPU tensors and gives identical bits.
Floating-point post-processing (Zipf inversion, Box-Muller) may differ in the last ulp between
devices, so a test generates an input once, on one device, and copies it to the other side.
"""
from __future__ import annotations

import math
from typing import Optional, Sequence, Tuple

import numpy as np
import torch

DEFAULT_SEED = 20221008

_M64 = (1 << 64) - 1


def _s64(x: int) -> int:
    """Two's-complement reinterpretation of a 64-bit pattern as a signed Python int."""
    x &= _M64
    return x - (1 << 64) if x >= (1 << 63) else x


_GOLDEN = _s64(0x9E3779B97F4A7C15)
_MUL1 = _s64(0xBF58476D1CE4E5B9)
_MUL2 = _s64(0x94D049BB133111EB)


def _lsr(x: torch.Tensor, k: int) -> torch.Tensor:
    """Logical right shift of int64 lanes (torch's >> is arithmetic)."""
    return (x >> k) & ((1 << (64 - k)) - 1)


def mix64(x: torch.Tensor) -> torch.Tensor:
    """splitmix64 output function on int64 lanes (wrapping arithmetic)."""
    z = x + _GOLDEN
    z = (z ^ _lsr(z, 30)) * _MUL1
    z = (z ^ _lsr(z, 27)) * _MUL2
    return z ^ _lsr(z, 31)


def _mix64_py(x: int) -> int:
    z = (x + 0x9E3779B97F4A7C15) & _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


def stream_key(seed: int, *tags: int) -> int:
    """Derive a 64-bit sub-stream key from a seed and integer tags (host-side, Python ints)."""
    k = _mix64_py(seed & _M64)
    for t in tags:
        k = _mix64_py(k ^ ((t * 0xD1342543DE82EF95) & _M64))
    return _s64(k)


def random_bits(key: int, start: int, n: int, device="cpu") -> torch.Tensor:
    """n 64-bit random words: word i = mix64(key + GOLDEN * (start + i))."""
    ctr = torch.arange(start, start + n, dtype=torch.int64, device=device)
    return mix64(ctr * _GOLDEN + key)


def uniform01(key: int, start: int, n: int, device="cpu") -> torch.Tensor:
    """n float64 uniforms in [0,1) with 53 random bits each."""
    return _lsr(random_bits(key, start, n, device), 11).to(torch.float64) * (2.0 ** -53)


# ----------------------------------------------------------------------------------------------
# Table sizes
# ----------------------------------------------------------------------------------------------

def draw_table_rows(n_tables: int = 26, lo: float = 10.0, hi: float = 4e7,
                    total_lo: float = 1.6e8, total_hi: float = 2.0e8,
                    max_tries: int = 100000) -> Tuple[int, np.ndarray]:
    """Recipe behind DLRM_TABLE_ROWS: rows_t = floor(exp(U(ln lo, ln hi))), U from
    numpy.random.default_rng(s) for s = 0, 1, 2, ... until the total lands in [total_lo, total_hi]
    (a plain log-uniform draw averages ~2.6e6 rows per table, i.e. well under the ~1.8e8 total the
    benchmark configuration quotes, hence the search).  Returns (s, rows)."""
    for s in range(max_tries):
        rng = np.random.default_rng(s)
        rows = np.floor(np.exp(rng.uniform(math.log(lo), math.log(hi), n_tables))).astype(np.int64)
        if total_lo <= rows.sum() <= total_hi:
            return s, rows
    raise RuntimeError("no seed found")


# Frozen output of draw_table_rows() (numpy seed recorded next to it); tests re-derive it.
DLRM_TABLE_ROWS_SEED = 75
DLRM_TABLE_ROWS = np.array([
    255, 102, 242896, 329609, 14481293, 914917, 13158335, 17948250, 5278618, 12, 5355, 2715153, 14,
    82, 32373152, 36373277, 2649033, 3693173, 4461, 253767, 3373987, 31353342, 216, 2048, 6736, 150,
], dtype=np.int64)  # 165,158,233 rows in total


def scaled_table_rows(scale: float) -> np.ndarray:
    """DLRM_TABLE_ROWS with every table scaled by one factor (never below 4 rows)."""
    return np.maximum(4, np.floor(DLRM_TABLE_ROWS * scale)).astype(np.int64)


def row_offsets(table_rows: Sequence[int]) -> np.ndarray:
    """[S+1] exclusive prefix of per-slot row counts."""
    out = np.zeros(len(table_rows) + 1, dtype=np.int64)
    np.cumsum(np.asarray(table_rows, dtype=np.int64), out=out[1:])
    return out


# ----------------------------------------------------------------------------------------------
# Table contents: closed form in (seed, global row, column)
# ----------------------------------------------------------------------------------------------

def table_rows_at(seed: int, rows: torch.Tensor, dim: int, dtype: torch.dtype) -> torch.Tensor:
    """Contents of the given global rows of the fused table, [len(rows), dim].

    v = mix64(mix64(key + row) + GOLDEN*col).  fp32: ((v >>> 40) - 2^23) * 2^-27, a 24-bit integer
    times a power of two, so exact in fp32 and within +-1/16.  fp16: ((v >>> 53) - 2^10) * 2^-14,
    an 11-bit integer times a power of two, exact in fp16, same range."""
    key = stream_key(seed, 0x7AB1E)
    base = mix64(rows.to(torch.int64) + key)
    col = torch.arange(dim, dtype=torch.int64, device=rows.device) * _GOLDEN
    v = mix64(base[:, None] + col[None, :])
    if dtype == torch.float32:
        return ((_lsr(v, 40) - (1 << 23)).to(torch.float32)) * (2.0 ** -27)
    if dtype == torch.float16:
        return ((_lsr(v, 53) - (1 << 10)).to(torch.float32) * (2.0 ** -14)).to(torch.float16)
    raise ValueError("dtype must be float32 or float16")


def fill_table(seed: int, table: torch.Tensor, chunk_rows: int = 1 << 20) -> None:
    """Fill table[total_rows, dim] in place with table_rows_at(), chunk by chunk."""
    total, dim = table.shape
    for r0 in range(0, total, chunk_rows):
        r1 = min(total, r0 + chunk_rows)
        idx = torch.arange(r0, r1, dtype=torch.int64, device=table.device)
        table[r0:r1] = table_rows_at(seed, idx, dim, table.dtype)


# ----------------------------------------------------------------------------------------------
# Zipf ranks and keys
# ----------------------------------------------------------------------------------------------

class ZipfSampler:
    """Rank r in {1..n} with P(r) proportional to r^-alpha.

    n <= 2^27: exact inverse CDF on the float64 cumulative table.  Larger n (the open 2^63 id
    space): the first 2^20 ranks keep their exact weights and the tail uses the continuous
    approximation weight(r) = integral of x^-alpha over [r-1/2, r+1/2], inverted in closed form."""

    HEAD = 1 << 20

    def __init__(self, n: int, alpha: float, device="cpu"):
        self.n, self.alpha, self.device = int(n), float(alpha), device
        head = self.n if self.n <= (1 << 27) else self.HEAD
        k = torch.arange(1, head + 1, dtype=torch.float64, device=device)
        self.cdf = torch.cumsum(k.pow(-alpha), 0)
        self.head = head
        self.head_mass = float(self.cdf[-1])
        if head < self.n:
            a = alpha
            self.x0 = head + 0.5
            self.tail_mass = (self.x0 ** (1 - a) - (self.n + 0.5) ** (1 - a)) / (a - 1)
        else:
            self.tail_mass = 0.0
        self.total = self.head_mass + self.tail_mass

    def ranks(self, u: torch.Tensor) -> torch.Tensor:
        """Map uniforms in [0,1) to int64 ranks in [1, n]."""
        t = u.to(self.device) * self.total
        r = torch.searchsorted(self.cdf, t, right=True).clamp_(max=self.head - 1) + 1
        if self.tail_mass > 0.0:
            a = self.alpha
            tt = (t - self.head_mass).clamp_(min=0.0)
            x = (self.x0 ** (1 - a) - tt * (a - 1)).clamp_(min=(self.n + 0.5) ** (1 - a)).pow(1.0 / (1 - a))
            xr = torch.round(x).clamp_(min=self.head + 1, max=float(self.n - 2048))
            r = torch.where(t >= self.head_mass, xr.to(torch.int64), r)
        return r


def _coprime_multiplier(n: int) -> int:
    a = max(1, int(n * 0.6180339887498949))
    while math.gcd(a, n) != 1:
        a += 1
    return a


def rank_to_key(rank: torch.Tensor, n_rows: int, salt: int) -> torch.Tensor:
    """Bijection {1..n_rows} -> [0, n_rows): key = (A*(rank-1) + c) mod n_rows, gcd(A, n_rows) = 1,
    so that popular rows are spread over the table instead of sitting next to each other."""
    a = _coprime_multiplier(n_rows)
    c = (_mix64_py(salt & _M64) % n_rows)
    return ((rank - 1) * a + c) % n_rows


def onehot_keys(seed: int, batch_index: int, table_rows: Sequence[int], batch: int, alpha: float,
                device="cpu", samplers: Optional[list] = None) -> torch.Tensor:
    """int64 keys [batch * S], bag-major (bag id = b*S + s), one key per bag, key in [0, rows_s).
    alpha <= 0 selects uniform keys."""
    S = len(table_rows)
    out = torch.empty((batch, S), dtype=torch.int64, device=device)
    for s, n in enumerate(table_rows):
        u = uniform01(stream_key(seed, 0x6B6579, batch_index, s), 0, batch, device)
        if alpha <= 0:
            out[:, s] = (u * int(n)).to(torch.int64).clamp_(max=int(n) - 1)
        else:
            smp = samplers[s] if samplers is not None else ZipfSampler(int(n), alpha, device)
            out[:, s] = rank_to_key(smp.ranks(u), int(n), seed + s)
    return out.reshape(-1)


def make_samplers(table_rows: Sequence[int], alpha: float, device="cpu") -> list:
    return [ZipfSampler(int(n), alpha, device) for n in table_rows]


def multihot_offsets(seed: int, batch_index: int, n_bags: int, h_lo: int, h_hi: int,
                     device="cpu") -> torch.Tensor:
    """int64 CSR offsets [n_bags+1]; hotness per bag uniform on {h_lo..h_hi} (h_lo may be 0)."""
    u = uniform01(stream_key(seed, 0x686F74, batch_index), 0, n_bags, device)
    h = (u * (h_hi - h_lo + 1)).to(torch.int64).clamp_(max=h_hi - h_lo) + h_lo
    off = torch.zeros(n_bags + 1, dtype=torch.int64, device=device)
    torch.cumsum(h, 0, out=off[1:])
    return off


def multihot_keys(seed: int, batch_index: int, table_rows: Sequence[int], batch: int, alpha: float,
                  offsets: torch.Tensor, device="cpu", samplers: Optional[list] = None) -> torch.Tensor:
    """int64 keys [nnz] for CSR offsets [batch*S+1]; the keys of bag (b, s) index table s."""
    S = len(table_rows)
    nnz = int(offsets[-1])
    h = (offsets[1:] - offsets[:-1]).to(device)
    bag = torch.repeat_interleave(torch.arange(batch * S, dtype=torch.int64, device=device), h)
    slot = bag % S
    u = uniform01(stream_key(seed, 0x6D686B, batch_index), 0, nnz, device)
    keys = torch.empty(nnz, dtype=torch.int64, device=device)
    for s, n in enumerate(table_rows):
        m = slot == s
        us = u[m]
        if alpha <= 0:
            keys[m] = (us * int(n)).to(torch.int64).clamp_(max=int(n) - 1)
        else:
            smp = samplers[s] if samplers is not None else ZipfSampler(int(n), alpha, device)
            keys[m] = rank_to_key(smp.ranks(us), int(n), seed + s)
    return keys


_ODD63 = 0x2545F4914F6CDD1D  # odd => multiplication by it is a bijection modulo 2^63


def open_space_keys(seed: int, batch_index: int, n_slots: int, batch: int, alpha: float,
                    device="cpu", sampler: Optional[ZipfSampler] = None) -> torch.Tensor:
    """int64 keys [batch * n_slots] in [0, 2^63): Zipf rank over a 2^63 id space, then
    key = (rank * ODD + salt_slot) mod 2^63, a bijection that salts every slot differently."""
    smp = sampler if sampler is not None else ZipfSampler(1 << 63, alpha, device)
    out = torch.empty((batch, n_slots), dtype=torch.int64, device=device)
    for s in range(n_slots):
        u = uniform01(stream_key(seed, 0x6F70656E, batch_index, s), 0, batch, device)
        salt = _mix64_py((seed + 977 * s) & _M64) & ((1 << 63) - 1)
        out[:, s] = (smp.ranks(u) * _s64(_ODD63) + _s64(salt)) & ((1 << 63) - 1)
    return out.reshape(-1)


def cache_keys(seed: int, batch_index: int, host_rows: int, n: int, alpha: float, device="cpu",
               sampler: Optional[ZipfSampler] = None) -> torch.Tensor:
    """int64 keys [n] in [0, host_rows) for the inference cache: Zipf ranks, scrambled."""
    smp = sampler if sampler is not None else ZipfSampler(host_rows, alpha, device)
    u = uniform01(stream_key(seed, 0x63616368, batch_index), 0, n, device)
    return rank_to_key(smp.ranks(u), host_rows, seed)


def normal_grads(seed: int, batch_index: int, n: int, device="cpu") -> torch.Tensor:
    """n float32 samples of N(0,1) by Box-Muller on the counter-based uniforms."""
    key = stream_key(seed, 0x6479, batch_index)
    m = (n + 1) // 2
    u1 = 1.0 - uniform01(key, 0, m, device)          # (0, 1]
    u2 = uniform01(key, m, m, device)
    r = torch.sqrt(-2.0 * torch.log(u1))
    z = torch.cat([r * torch.cos(2 * math.pi * u2), r * torch.sin(2 * math.pi * u2)])[:n]
    return z.to(torch.float32)
