"""Seeded synthetic inputs for the embedding-lookup hot path.

This module only *makes inputs*: table shapes, table values, bag lengths, lookup
indices and the table-to-rank assignment of each named workload.  It holds none
of the method's arithmetic (no bucketing, pooling, packing or ring logic) and is
the one module that both the CPU oracle's tests and the HIP path's tests use, so
that both sides see byte-identical inputs.

Everything random comes from one counter-based generator (the public splitmix64
finaliser applied to ``key + counter * golden``) written with torch int64 ops, so
the same integers come out on the CPU and on a GPU and any single element can be
recomputed without materialising the rest: a 40 GB table is filled on the device
and the oracle recomputes just the rows it touches.  The only exception is the
Gaussian tables of the two small workloads, drawn with numpy on the host.

Workloads stand in for the paper's datasets (Experimental Setup: Criteo
Mini-Kaggle with 26 sparse features and one index per table, Ali-CCP with 23; the
heterogeneous synthetic setting with a random number of vectors per table), which
are not available here; shapes follow the five benchmark configurations.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np
import torch

SEED_BASE = 251219342

_M64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_MUL1 = 0xBF58476D1CE4E5B9
_MUL2 = 0x94D049BB133111EB


def _s64(x: int) -> int:
    """Two's-complement reinterpretation of a u64 python int as an int64 value."""
    x &= _M64
    return x - (1 << 64) if x >= (1 << 63) else x


def _mix_py(x: int) -> int:
    x &= _M64
    x = ((x ^ (x >> 30)) * _MUL1) & _M64
    x = ((x ^ (x >> 27)) * _MUL2) & _M64
    return x ^ (x >> 31)


def stream_key(*parts: int) -> int:
    """Fold integers (seed, purpose, table, iteration, ...) into one u64 stream key."""
    k = 0x243F6A8885A308D3
    for p in parts:
        k = _mix_py(k ^ ((int(p) + _GOLDEN) & _M64))
    return k


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical right shift of int64 (torch's >> is arithmetic)."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def hash_u64(key: int, counter: torch.Tensor) -> torch.Tensor:
    """splitmix64 output for state ``key + (counter+1)*golden`` as int64 bit patterns."""
    z = counter * _s64(_GOLDEN) + _s64(key + _GOLDEN)
    z = (z ^ _lsr(z, 30)) * _s64(_MUL1)
    z = (z ^ _lsr(z, 27)) * _s64(_MUL2)
    return z ^ _lsr(z, 31)


def hash_u64_py(key: int, counter: int) -> int:
    """Pure-python twin of :func:`hash_u64` for one counter (used by tests)."""
    return _mix_py((key + (counter + 1) * _GOLDEN) & _M64)


def uniform01(key: int, counter: torch.Tensor) -> torch.Tensor:
    """float64 uniforms in [0,1) from the top 53 bits of the hash."""
    return _lsr(hash_u64(key, counter), 11).to(torch.float64) * (2.0 ** -53)


def randint(key: int, counter: torch.Tensor, n: int) -> torch.Tensor:
    """Integers in [0,n) (plain modulo of a 63-bit value; the bias is < 2^-30)."""
    return _lsr(hash_u64(key, counter), 1) % n


# purposes
_P_TABLE, _P_LEN, _P_IDX, _P_ROWS = 1, 2, 3, 4


@dataclass
class Workload:
    name: str
    cfg: int
    P: int
    T: int
    D: int
    k: int
    B: int
    table_dtype: str            # "fp32" | "fp16" | "u8rq" / "f8rq" (8-bit integer / E4M3 codes, scale and bias per row)
    part_kind: int              # 0 table-wise, 1 row-wise block
    rows: List[int]
    table_owner: List[int]      # table-wise only (zeros for row-wise)
    values: str                 # "gauss" | "grid"
    bag: Tuple                  # ("fixed", L) | ("uniform", lo, hi)
    index_dist: Tuple           # ("uniform",) | ("zipf", alpha)
    seed: int
    _cdf_cache: dict = field(default_factory=dict, repr=False)

    @property
    def K(self) -> int:
        return max(self.k, 1)

    @property
    def F(self) -> int:
        return self.P if self.part_kind == 1 else 1

    @property
    def dtype_code(self) -> int:
        """Storage code shared by the library's and the oracle's interfaces."""
        return {"fp32": 0, "fp16": 1, "u8rq": 2, "f8rq": 3}[self.table_dtype]

    @property
    def row_bytes(self) -> int:
        """Bytes from one table row to the next."""
        if self.table_dtype in ("u8rq", "f8rq"):
            return rowq_stride(self.D)
        return self.D * (2 if self.table_dtype == "fp16" else 4)

    @property
    def row_width(self) -> int:
        """Second dimension of a table tensor (elements; bytes for row-quantised tables)."""
        return rowq_stride(self.D) if self.table_dtype in ("u8rq", "f8rq") else self.D

    @property
    def torch_dtype(self):
        return {"fp32": torch.float32, "fp16": torch.float16, "u8rq": torch.uint8, "f8rq": torch.uint8}[self.table_dtype]

    def mean_bag(self) -> float:
        return float(self.bag[1]) if self.bag[0] == "fixed" else 0.5 * (self.bag[1] + self.bag[2])

    def table_bytes(self) -> int:
        return sum(self.rows) * self.row_bytes


def rowq_stride(D: int) -> int:
    """Row-quantised storage: D one-byte codes, fp32 scale, fp32 bias, padded to 16 bytes."""
    return (D + 8 + 15) // 16 * 16


# ----------------------------------------------------------------------------- partitions

def owners_round_robin(T: int, P: int) -> List[int]:
    return [t % P for t in range(T)]


def owners_balanced_by_rows(rows: List[int], P: int) -> List[int]:
    """Largest table first, each to the rank with the fewest rows so far (ties: lower id)."""
    order = sorted(range(len(rows)), key=lambda t: (-rows[t], t))
    load = [0] * P
    own = [0] * len(rows)
    for t in order:
        d = min(range(P), key=lambda r: (load[r], r))
        own[t] = d
        load[d] += rows[t]
    return own


def owners_hot_on_rank0(rows: List[int], P: int, n_hot: int) -> List[int]:
    """The n_hot largest tables all on rank 0, the rest round-robin over ranks 1..P-1."""
    hot = set(sorted(range(len(rows)), key=lambda t: (-rows[t], t))[:n_hot])
    own, nxt = [], 0
    for t in range(len(rows)):
        if t in hot or P == 1:
            own.append(0)
        else:
            own.append(1 + nxt % (P - 1))
            nxt += 1
    return own


# ----------------------------------------------------------------------------- workloads

def _rows_loguniform(seed: int, T: int, lo_exp: float, hi_exp: float) -> List[int]:
    u = uniform01(stream_key(seed, _P_ROWS), torch.arange(T, dtype=torch.int64))
    return [int(math.floor(10.0 ** (lo_exp + (hi_exp - lo_exp) * float(x)))) for x in u]


def workload(cfg: int, size: str = "full") -> Workload:
    """The five benchmark workloads (1..5) and the paper's own heterogeneous setting (6), at
    full size or as reduced twins (``size="small"``).

    The reduced twins keep every structural feature (partition kind, ragged last
    shard, bag-length law, index law, dtype, ring depth) at sizes a CPU oracle
    finishes in seconds.
    """
    seed = SEED_BASE * 10 + cfg
    small = size == "small"
    if size not in ("full", "small"):
        raise ValueError("size must be 'full' or 'small'")
    if cfg == 1:
        T, P = 8, 2
        rows = [10_000] * T
        return Workload("cfg1", 1, P, T, 16, 1, 128, "fp32", 0, rows, owners_round_robin(T, P),
                        "gauss", ("fixed", 1), ("uniform",), seed)
    if cfg == 2:
        T, P = 26, 4
        rows = _rows_loguniform(seed, T, 3.0, 5.0)
        return Workload("cfg2", 2, P, T, 64, 1, 2048, "fp32", 0, rows, owners_balanced_by_rows(rows, P),
                        "gauss", ("fixed", 1), ("uniform",), seed)
    if cfg == 3:
        T, P = 26, 8
        rows = [10_007 if small else 1_000_000] * T
        B = 256 if small else 8192
        return Workload("cfg3" + ("s" if small else ""), 3, P, T, 128, 2, B, "fp32", 1, rows, [0] * T,
                        "grid", ("uniform", 1, 40), ("zipf", 1.05), seed)
    if cfg == 4:
        T, P = 64, 8
        top = 4e4 if small else 4e7
        floor_rows = 50 if small else 1000
        rows = [max(floor_rows, int(math.floor(top / (t + 1) ** 1.7))) for t in range(T)]
        B = 512 if small else 16384
        return Workload("cfg4" + ("s" if small else ""), 4, P, T, 128, 4, B, "fp32", 0, rows,
                        owners_hot_on_rank0(rows, P, 8),
                        "grid", ("uniform", 1, 64), ("zipf", 1.2), seed)
    if cfg == 5:
        T, P = 8, 8
        rows = [20_011 if small else 20_000_000] * T
        B = 1024 if small else 65536
        return Workload("cfg5" + ("s" if small else ""), 5, P, T, 128, 4, B, "fp16", 1, rows, [0] * T,
                        "grid", ("fixed", 32), ("zipf", 1.05), seed)
    if cfg == 6:
        # the paper's heterogeneous synthetic setting (Synthetic DLRM benchmarks, Setting 1): a random
        # number of vectors per table from 1 to 100, with the shapes of its dataset runs (26 tables,
        # largest about a million rows, batch 512, 8 processes) at embedding dimension 64
        T, P = 26, 8
        rows = [max(1000, r // (20 if small else 1)) for r in _rows_loguniform(seed, T, 3.0, 6.0)]
        return Workload("cfg6" + ("s" if small else ""), 6, P, T, 64, 2, 128 if small else 512, "fp32", 0, rows,
                        owners_balanced_by_rows(rows, P), "grid", ("uniform", 1, 100), ("uniform",), seed)
    raise ValueError("cfg must be 1..6")


def custom(name: str, *, P: int, T: int, D: int, k: int, B: int, rows: List[int], part_kind: int,
           table_owner: Optional[List[int]] = None, table_dtype: str = "fp32", values: str = "grid",
           bag: Tuple = ("uniform", 0, 5), index_dist: Tuple = ("uniform",), seed: int = 7) -> Workload:
    """A free-form workload for edge-case tests (empty bags, P not dividing B, odd D, ...)."""
    if table_owner is None:
        table_owner = owners_round_robin(T, P) if part_kind == 0 else [0] * T
    return Workload(name, 0, P, T, D, k, B, table_dtype, part_kind, list(rows), list(table_owner),
                    values, bag, index_dist, seed)


# ----------------------------------------------------------------------------- table values

def grid_rows(w: Workload, t: int, row_ids: torch.Tensor) -> torch.Tensor:
    """Rows ``row_ids`` of table t on the exact grid, as float32 ``[n, D]`` on row_ids' device.

    element = (b0+b1+b2+b3 - 510) * 2^-14 with b* four bytes of hash(table key, row*D+col):
    a sum of four uniform bytes (bell-shaped, sigma ~ 0.009).  Every value, and every
    sum of up to 2^10 of them, is exact in fp32 and every value is exact in fp16, so
    any summation order gives the same bits.
    """
    key = stream_key(w.seed, _P_TABLE, t)
    cols = torch.arange(w.D, dtype=torch.int64, device=row_ids.device)
    ctr = row_ids.to(torch.int64)[:, None] * w.D + cols[None, :]
    h = hash_u64(key, ctr)
    s = (h & 255) + ((h >> 8) & 255) + ((h >> 16) & 255) + ((h >> 24) & 255) - 510
    return s.to(torch.float32) * (2.0 ** -14)


def rowq_rows(w: Workload, t: int, row_ids: torch.Tensor) -> torch.Tensor:
    """Rows ``row_ids`` of row-quantised table t as stored: uint8 ``[n, rowq_stride(D)]``.

    Codes are hash bytes; for E4M3 codes ("f8rq") the two NaN patterns are replaced by the
    largest finite code of the same sign, and "grid" tables keep the exponent field below 8
    (|value| < 2, a multiple of 2^-9).  "grid" values: scale in {2^-8, 2^-9, 2^-10} and bias a multiple of
    2^-10 in [-1/16, 1/16), so every element and every sum of up to 2^10 of them is exact in
    fp32 in any order.  Otherwise scale and bias are arbitrary floats (scale in (1e-4, 1e-2),
    bias in (-0.5, 0.5)), which makes the roundings of the decoding and of the sum visible.
    Padding bytes are zero.
    """
    dev = row_ids.device
    n, stride = row_ids.numel(), rowq_stride(w.D)
    key = stream_key(w.seed, _P_TABLE, t)
    ids = row_ids.to(torch.int64)
    out = torch.zeros((n, stride), dtype=torch.uint8, device=dev)
    cols = torch.arange(w.D, dtype=torch.int64, device=dev)
    codes = hash_u64(key, ids[:, None] * w.D + cols[None, :]) & 255
    if w.table_dtype == "f8rq":
        if w.values == "grid":
            codes = codes & 0xBF                                  # exponent field 0..7
        codes = torch.where((codes & 0x7F) == 0x7F, codes - 1, codes)
    out[:, :w.D] = codes.to(torch.uint8)
    hk = stream_key(w.seed, _P_TABLE, t, 1)
    if w.values == "grid":
        h = hash_u64(hk, ids)
        scale = torch.pow(2.0, -(8.0 + (h % 3).to(torch.float32))).to(torch.float32)
        bias = (((h >> 8) & 127) - 64).to(torch.float32) * (2.0 ** -10)
    else:
        scale = (1e-4 + 9.9e-3 * uniform01(hk, 2 * ids)).to(torch.float32)
        bias = (uniform01(hk, 2 * ids + 1) - 0.5).to(torch.float32)
    out[:, w.D:w.D + 4] = scale.contiguous().view(torch.uint8).reshape(n, 4)
    out[:, w.D + 4:w.D + 8] = bias.contiguous().view(torch.uint8).reshape(n, 4)
    return out


def make_table(w: Workload, t: int, device="cpu", chunk_rows: Optional[int] = None) -> torch.Tensor:
    """Full table t in the workload's storage on ``device``: ``[rows_t, D]``, or uint8
    ``[rows_t, rowq_stride(D)]`` for row-quantised storage."""
    rows = w.rows[t]
    if w.table_dtype in ("u8rq", "f8rq"):
        out = torch.empty((rows, rowq_stride(w.D)), dtype=torch.uint8, device=device)
        if chunk_rows is None:
            chunk_rows = max(1, (1 << 24) // w.D)
        for r0 in range(0, rows, chunk_rows):
            r1 = min(rows, r0 + chunk_rows)
            out[r0:r1] = rowq_rows(w, t, torch.arange(r0, r1, dtype=torch.int64, device=device))
        return out
    if w.values == "gauss":
        rng = np.random.Generator(np.random.PCG64([w.seed, _P_TABLE, t]))
        a = rng.normal(0.0, 0.01, size=(rows, w.D)).astype(np.float32)
        return torch.from_numpy(a).to(w.torch_dtype).to(device)
    out = torch.empty((rows, w.D), dtype=w.torch_dtype, device=device)
    if chunk_rows is None:
        chunk_rows = max(1, (1 << 25) // w.D)
    for r0 in range(0, rows, chunk_rows):
        r1 = min(rows, r0 + chunk_rows)
        ids = torch.arange(r0, r1, dtype=torch.int64, device=device)
        out[r0:r1] = grid_rows(w, t, ids).to(w.torch_dtype)
    return out


def table_rows(w: Workload, t: int, row_ids: torch.Tensor, table: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Selected rows of table t as float32 on the CPU (recomputed for grid tables).
    Not for row-quantised tables, whose stored rows come from ``rowq_rows``."""
    assert w.table_dtype not in ("u8rq", "f8rq")
    if w.values == "grid":
        return grid_rows(w, t, row_ids.cpu()).to(w.torch_dtype).to(torch.float32)
    if table is None:
        table = make_table(w, t, "cpu")
    return table.cpu()[row_ids.cpu()].to(torch.float32)


# ----------------------------------------------------------------------------- batches

def _coprime_multiplier(rows: int) -> int:
    a = max(1, int(math.ceil(0.618 * rows)))
    while math.gcd(a, rows) != 1:
        a += 1
    return a


def _zipf_cdf(w: Workload, t: int, device) -> torch.Tensor:
    key = (w.rows[t], str(device))
    cdf = w._cdf_cache.get(key)
    if cdf is None:
        z = torch.arange(1, w.rows[t] + 1, dtype=torch.float64, device=device)
        cdf = torch.cumsum(z.pow_(-float(w.index_dist[1])), 0)
        w._cdf_cache[key] = cdf
    return cdf


def bag_lengths(w: Workload, t: int, it: int, device="cpu") -> torch.Tensor:
    b = torch.arange(w.B, dtype=torch.int64, device=device)
    if w.bag[0] == "fixed":
        return torch.full((w.B,), int(w.bag[1]), dtype=torch.int64, device=device)
    lo, hi = int(w.bag[1]), int(w.bag[2])
    return lo + randint(stream_key(w.seed, _P_LEN, t, it), b, hi - lo + 1)


def make_batch(w: Workload, it: int, device="cpu") -> Tuple[torch.Tensor, torch.Tensor]:
    """One iteration's sparse input: ``(indices[nnz], offsets[T*B+1])``, int64, table-major.

    Bag g = t*B + b holds lookups ``offsets[g] .. offsets[g+1]-1`` into table t (global
    row ids).  Zipf ranks are drawn by exact inverse CDF (float64 cumulative sum and a
    binary search) and scattered over the table by ``row = rank * A_t mod rows_t`` with
    A_t coprime to rows_t, so that hot rows fall in every shard.
    """
    lens, idx = [], []
    for t in range(w.T):
        ln = bag_lengths(w, t, it, device)
        n = int(ln.sum().item())
        c = torch.arange(n, dtype=torch.int64, device=device)
        key = stream_key(w.seed, _P_IDX, t, it)
        if w.index_dist[0] == "uniform":
            ix = randint(key, c, w.rows[t])
        else:
            cdf = _zipf_cdf(w, t, device)
            u = uniform01(key, c) * cdf[-1]
            z0 = torch.searchsorted(cdf, u, right=True).clamp_(max=w.rows[t] - 1)
            ix = (z0 * _coprime_multiplier(w.rows[t])) % w.rows[t]
        lens.append(ln)
        idx.append(ix)
    offsets = torch.zeros(w.T * w.B + 1, dtype=torch.int64, device=device)
    torch.cumsum(torch.cat(lens), 0, out=offsets[1:])
    indices = torch.cat(idx) if idx else torch.zeros(0, dtype=torch.int64, device=device)
    return indices, offsets


# ----------------------------------------------------------------------------- dense part of the model

_P_DENSE, _P_MLP = 5, 6
N_DENSE = 13                      # dense features per sample of the click-log datasets the paper uses


def _bell(key: int, n: int, device="cpu") -> torch.Tensor:
    """n values with mean 0 and variance 1, bell-shaped: a centred, scaled sum of four hash bytes."""
    h = hash_u64(key, torch.arange(n, dtype=torch.int64, device=device))
    s = (h & 255) + ((h >> 8) & 255) + ((h >> 16) & 255) + ((h >> 24) & 255) - 510
    return s.to(torch.float32) * (1.0 / 147.8)               # sd of a uniform byte is 73.9; four of them: 147.8


def dense_features(w: Workload, it: int, device="cpu") -> torch.Tensor:
    """Dense inputs of iteration ``it``: ``[B, N_DENSE]`` fp32 uniforms in [0, 1)."""
    u = uniform01(stream_key(w.seed, _P_DENSE, it), torch.arange(w.B * N_DENSE, dtype=torch.int64, device=device))
    return u.to(torch.float32).reshape(w.B, N_DENSE)


def mlp_sizes(w: Workload, size: str = "full") -> Tuple[List[int], List[int]]:
    """Layer widths (bottom, top).  The paper builds on the reference recommendation model and
    gives no widths; "full" takes that model's large configuration around the workload's D and T
    (bottom 13-512-256-D, top z-1024-1024-512-256-1 with z = D + T(T+1)/2), "small" a narrow
    stack for tests the CPU oracle finishes quickly."""
    zdim = w.D + w.T * (w.T + 1) // 2
    if size == "full":
        return [N_DENSE, 512, 256, w.D], [zdim, 1024, 1024, 512, 256, 1]
    return [N_DENSE, 40, w.D], [zdim, 72, 24, 1]


def mlp_weights(w: Workload, sizes: List[int], which: int, device="cpu"):
    """Seeded layers ``[(W [N, K], bias [N]), ...]`` for widths ``sizes``: W ~ N(0, 2/(K+N)),
    bias ~ N(0, 1/N) (the reference model's initialisation), values from the hash."""
    layers = []
    for i, (K, N) in enumerate(zip(sizes[:-1], sizes[1:])):
        W = _bell(stream_key(w.seed, _P_MLP, which, i, 0), N * K, device).reshape(N, K) * math.sqrt(2.0 / (K + N))
        b = _bell(stream_key(w.seed, _P_MLP, which, i, 1), N, device) * math.sqrt(1.0 / N)
        layers.append((W.contiguous(), b.contiguous()))
    return layers
