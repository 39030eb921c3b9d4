"""CPU oracle for the embedding-lookup path.  TEST INFRASTRUCTURE ONLY.

Thin numpy/ctypes wrapper over ``bls_oracle.c`` (plain single-threaded C written from
the paper's description) plus a host model of the bounded-lag ring.  Only ``tests/``,
the smoke check and the benchmark's ``cpu_baseline`` leg may import this package; the
product library never does, and this package imports nothing from the product.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bls_oracle.c")
_LIB = os.path.join(_HERE, "libbls_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with the host compiler (no fused multiply-add contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-std=c99", "-Wall", "-Wextra",
                               "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _i64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int64))


class OracleError(RuntimeError):
    def __init__(self, fn: str, code: int):
        super().__init__(f"{fn} failed with code {code}")
        self.code = code


def _chk(fn: str, rc: int):
    if rc != 0:
        raise OracleError(fn, rc)


@dataclass
class Case:
    """Shape of one problem: P ranks, T tables, vector length D, global batch B,
    partition kind (0 table-wise with ``owner[t]``, 1 row-wise block), rows per table,
    storage dtype (0 fp32, 1 fp16, 2 / 3 row-quantised 8-bit with integer / E4M3 codes:
    ``rowq_stride(D)`` bytes per row, D codes, fp32 scale, fp32 bias, padding)."""
    P: int
    T: int
    D: int
    B: int
    part_kind: int
    rows: Sequence[int]
    owner: Sequence[int]
    dtype: int = 0

    def __post_init__(self):
        self._rows = _i64(self.rows)
        self._owner = np.ascontiguousarray(np.asarray(self.owner, dtype=np.int32))
        assert len(self._rows) == self.T and len(self._owner) == self.T

    @property
    def F(self) -> int:
        return self.P if self.part_kind == 1 else 1

    @property
    def n_vec(self) -> int:
        """Pooled vectors in flight per iteration."""
        return self.F * self.T * self.B


def rowq_stride(D: int) -> int:
    """Bytes per row of a row-quantised table: D codes + scale + bias, padded to 16."""
    return (D + 8 + 15) // 16 * 16


def e4m3_table() -> np.ndarray:
    """The 256 E4M3 codes decoded to float32."""
    out = np.zeros(256, np.float32)
    _chk("orc_e4m3_table", _load().orc_e4m3_table(_p(out)))
    return out


def _table_ptrs(case: Case, tables: List[np.ndarray]):
    want = {0: np.float32, 1: np.float16, 2: np.uint8, 3: np.uint8}[case.dtype]
    width = rowq_stride(case.D) if case.dtype in (2, 3) else case.D
    keep = []
    for t, a in enumerate(tables):
        assert a.dtype == want and a.flags.c_contiguous and a.shape == (case.rows[t], width), (t, a.dtype, a.shape)
        keep.append(a)
    arr = (C.c_void_p * case.T)(*[a.ctypes.data for a in keep])
    return arr, keep


def plan(case: Case, indices, offsets, want_perm: bool = True, weights=None) -> dict:
    indices, offsets = _i64(indices), _i64(offsets)
    if weights is not None:
        weights = np.ascontiguousarray(weights, dtype=np.float32)
    assert offsets.shape[0] == case.T * case.B + 1
    nnz = int(offsets[-1]) if offsets[-1] >= 0 else 0
    assert indices.shape[0] >= nnz
    pp = case.P * case.P
    out = {k: np.zeros(pp, np.int64) for k in ("sendcounts", "sdispls", "recvcounts", "rdispls")}
    out["ridx"] = np.zeros(nnz, np.int64)
    out["segoff"] = np.zeros(case.n_vec + 1, np.int64)
    out["perm"] = np.zeros(nnz, np.int64) if want_perm else None
    out["rweights"] = np.zeros(nnz, np.float32) if weights is not None else None
    rc = _load().orc_plan_weighted(C.c_int(case.P), C.c_int(case.T), C.c_int64(case.B), C.c_int(case.part_kind),
                                   _p(case._rows), _p(case._owner), _p(indices), _p(offsets), _p(weights),
                                   _p(out["sendcounts"]), _p(out["sdispls"]), _p(out["recvcounts"]), _p(out["rdispls"]),
                                   _p(out["ridx"]), _p(out["rweights"]), _p(out["segoff"]), _p(out["perm"]))
    _chk("orc_plan", rc)
    return out


def embbag_plain(case: Case, tables: List[np.ndarray], indices, offsets, want64=True, want32=True,
                 weights=None, mean: bool = False):
    """The plain definition: Out[b][t][:] in float64 and in ordered float32 (optionally with
    per-sample weights, or as the mean over the bag)."""
    indices, offsets = _i64(indices), _i64(offsets)
    if weights is not None:
        weights = np.ascontiguousarray(weights, dtype=np.float32)
    ptrs, _keep = _table_ptrs(case, tables)
    o64 = np.zeros((case.B, case.T, case.D), np.float64) if want64 else None
    o32 = np.zeros((case.B, case.T, case.D), np.float32) if want32 else None
    rc = _load().orc_embbag_plain_ex(C.c_int(case.T), C.c_int(case.D), C.c_int64(case.B), C.c_int(case.dtype),
                                     _p(case._rows), ptrs, _p(indices), _p(offsets), _p(weights),
                                     C.c_int(1 if mean else 0), _p(o64), _p(o32))
    _chk("orc_embbag_plain", rc)
    return o64, o32


def embbag_absmass(case: Case, tables: List[np.ndarray], indices, offsets) -> np.ndarray:
    indices, offsets = _i64(indices), _i64(offsets)
    ptrs, _keep = _table_ptrs(case, tables)
    m = np.zeros((case.B, case.T, case.D), np.float64)
    _chk("orc_embbag_absmass",
         _load().orc_embbag_absmass(C.c_int(case.T), C.c_int(case.D), C.c_int64(case.B), C.c_int(case.dtype),
                                    ptrs, _p(indices), _p(offsets), _p(m)))
    return m


def pool(case: Case, tables: List[np.ndarray], ridx, segoff, rweights=None) -> np.ndarray:
    ridx, segoff = _i64(ridx), _i64(segoff)
    if rweights is not None:
        rweights = np.ascontiguousarray(rweights, dtype=np.float32)
    ptrs, _keep = _table_ptrs(case, tables)
    Y = np.zeros(case.n_vec * case.D, np.float32)
    _chk("orc_pool",
         _load().orc_pool_weighted(C.c_int(case.P), C.c_int(case.T), C.c_int(case.D), C.c_int64(case.B),
                                   C.c_int(case.part_kind), _p(case._rows), _p(case._owner), C.c_int(case.dtype),
                                   ptrs, _p(ridx), _p(rweights), _p(segoff), _p(Y)))
    return Y


def pooled_counts(case: Case) -> dict:
    pp = case.P * case.P
    out = {k: np.zeros(pp, np.int64) for k in ("pcount", "psdispl", "prcount", "prdispl")}
    out["psbase"] = np.zeros(case.P, np.int64)
    out["prbase"] = np.zeros(case.P, np.int64)
    _chk("orc_pooled_counts",
         _load().orc_pooled_counts(C.c_int(case.P), C.c_int(case.T), C.c_int(case.D), C.c_int64(case.B),
                                   C.c_int(case.part_kind), _p(case._owner),
                                   _p(out["pcount"]), _p(out["psdispl"]), _p(out["prcount"]), _p(out["prdispl"]),
                                   _p(out["psbase"]), _p(out["prbase"])))
    return out


def pack(case: Case, Y: np.ndarray) -> np.ndarray:
    Y = np.ascontiguousarray(Y, dtype=np.float32).reshape(-1)
    assert Y.size == case.n_vec * case.D
    S = np.zeros_like(Y)
    _chk("orc_pack", _load().orc_pack(C.c_int(case.P), C.c_int(case.T), C.c_int(case.D), C.c_int64(case.B),
                                      C.c_int(case.part_kind), _p(case._owner), _p(Y), _p(S)))
    return S


def alltoallv(P: int, send: np.ndarray, sbase, sendcounts, sdispls, rbase, recvcounts, rdispls,
              recv_size: int) -> np.ndarray:
    send = np.ascontiguousarray(send, dtype=np.float32).reshape(-1)
    recv = np.zeros(recv_size, np.float32)
    a = [_i64(x) for x in (sbase, sendcounts, sdispls, rbase, recvcounts, rdispls)]
    _chk("orc_alltoallv_f32",
         _load().orc_alltoallv_f32(C.c_int(P), _p(send), _p(a[0]), _p(a[1]), _p(a[2]), _p(recv),
                                   _p(a[3]), _p(a[4]), _p(a[5])))
    return recv


def exchange(case: Case, S: np.ndarray) -> np.ndarray:
    """The pooled-vector alltoallv with the closed-form counts of :func:`pooled_counts`."""
    pc = pooled_counts(case)
    return alltoallv(case.P, S, pc["psbase"], pc["pcount"], pc["psdispl"],
                     pc["prbase"], pc["prcount"], pc["prdispl"], case.n_vec * case.D)


def unpack(case: Case, R: np.ndarray, mean_offsets=None) -> np.ndarray:
    """Completion copy-out; with ``mean_offsets`` (the batch's offsets) also the division by the bag length."""
    R = np.ascontiguousarray(R, dtype=np.float32).reshape(-1)
    assert R.size == case.n_vec * case.D
    out = np.zeros((case.B, case.T, case.D), np.float32)
    off = None if mean_offsets is None else _i64(mean_offsets)
    _chk("orc_unpack", _load().orc_unpack_mean(C.c_int(case.P), C.c_int(case.T), C.c_int(case.D), C.c_int64(case.B),
                                               C.c_int(case.part_kind), _p(case._owner), _p(R), _p(off), _p(out)))
    return out


def bag_sum(rows_nd: np.ndarray):
    rows_nd = np.ascontiguousarray(rows_nd, dtype=np.float32)
    n, D = rows_nd.shape
    o32, o64 = np.zeros(D, np.float32), np.zeros(D, np.float64)
    _chk("orc_bag_sum", _load().orc_bag_sum(C.c_int(D), C.c_int64(n), _p(rows_nd), _p(o32), _p(o64)))
    return o32, o64


def pipeline(case: Case, tables: List[np.ndarray], indices, offsets, weights=None, mean: bool = False) -> dict:
    """Every stage in path order: plan, pool, pack, exchange, unpack."""
    r = plan(case, indices, offsets, weights=weights)
    r["Y"] = pool(case, tables, r["ridx"], r["segoff"], r["rweights"])
    r["S"] = pack(case, r["Y"])
    r["R"] = exchange(case, r["S"])
    r["Out"] = unpack(case, r["R"], offsets if mean else None)
    return r


# ----------------------------------------------------------------------------- dense layers

def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def mlp_layer(x, W, bias, act: int, err_in=None, want_err: bool = True):
    """act(x @ W.T + bias) in double; x [M, K] (any float dtype), W [N, K] fp32, bias [N] fp32 or None.
    Returns (y [M, N] float64, err [M, N] float64 bound for an fp32 implementation, or None)."""
    x = _f64(x)
    W = np.ascontiguousarray(W, dtype=np.float32)
    M, K = x.shape
    N = W.shape[0]
    assert W.shape == (N, K)
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
        assert bias.shape == (N,)
    if err_in is not None:
        err_in = _f64(err_in)
        assert err_in.shape == x.shape
    y = np.zeros((M, N), np.float64)
    err = np.zeros((M, N), np.float64) if want_err else None
    _chk("orc_mlp_layer", _load().orc_mlp_layer(C.c_int64(M), C.c_int(K), C.c_int(N), _p(x), _p(W), _p(bias),
                                                C.c_int(act), _p(err_in), _p(y), _p(err)))
    return y, err


def mlp(x, layers, err_in=None):
    """A stack of layers [(W, bias, act), ...]; returns the last output and its error bound."""
    y, err = _f64(x), err_in
    for W, bias, act in layers:
        y, err = mlp_layer(y, W, bias, act, err)
    return y, err


def interact(x, emb, err_x=None, want_err: bool = True):
    """x [B, D] (double), emb [B, T, D] fp32 -> z [B, D + T(T+1)/2] double and its error bound."""
    x = _f64(x)
    emb = np.ascontiguousarray(emb, dtype=np.float32)
    B, T, D = emb.shape
    assert x.shape == (B, D)
    if err_x is not None:
        err_x = _f64(err_x)
    Wd = D + T * (T + 1) // 2
    z = np.zeros((B, Wd), np.float64)
    err = np.zeros((B, Wd), np.float64) if want_err else None
    _chk("orc_interact", _load().orc_interact(C.c_int64(B), C.c_int(T), C.c_int(D), _p(x), _p(emb), _p(err_x),
                                              _p(z), _p(err)))
    return z, err


# ----------------------------------------------------------------------------- ring model

class RingFull(RuntimeError):
    pass


class RingEmpty(RuntimeError):
    pass


class RingOrder(RuntimeError):
    pass


class RingModel:
    """Host model of the k-deep ring of in-flight iterations.

    Alltoallv initiation: iteration j writes receive buffers R(*, j mod k).  Bound
    section and its figure: k buffers per process; a process that has issued k
    iterations must complete the oldest before issuing the next, after which that
    buffer is reused.  Backend section: wait() completes the tail (oldest) request and
    pops it.  Reading for k = 0 (semantically synchronous, but j mod 0 is undefined):
    one slot.
    """

    def __init__(self, k: int):
        if k < 0:
            raise ValueError("k must be >= 0")
        self.K = max(k, 1)
        self.next_iter = 0
        self.in_flight: List[int] = []

    def acquire(self):
        if len(self.in_flight) == self.K:
            raise RingFull()
        j = self.next_iter
        self.next_iter += 1
        self.in_flight.append(j)
        return j, j % self.K

    def retire(self, j: int) -> int:
        if not self.in_flight:
            raise RingEmpty()
        if self.in_flight[0] != j:
            raise RingOrder()
        self.in_flight.pop(0)
        return j % self.K

    def drain(self):
        """Listing 2's final loop: retire everything outstanding, oldest first."""
        out = []
        while self.in_flight:
            j = self.in_flight[0]
            out.append((j, self.retire(j)))
        return out


def ring_bytes_per_bound(s: int, b: int, n_tables: int) -> int:
    """Extra memory per unit of the bound k, the paper's Experimental Setup formula
    s*b*|tables| + s^2 + b (the worked example gives about 860 KB for b=512, s=64, 26 tables)."""
    return s * b * n_tables + s * s + b
