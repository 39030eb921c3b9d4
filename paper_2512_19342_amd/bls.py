"""ctypes binding of libbls.so: argument marshalling only.

Function names and argument order follow include/bls.h.  Device buffers are torch
tensors (used for their memory and for the current stream, nothing else); the binding
passes ``data_ptr()`` and sizes through.  If the library has not been built the import
of a symbol raises - there is no CPU or PyTorch fallback for any step.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch

BLS_OK, BLS_EINVAL, BLS_ERANGE, BLS_ENOSPC = 0, -1, -2, -3
BLS_ERING_FULL, BLS_ERING_EMPTY, BLS_EORDER, BLS_EHIP = -4, -5, -6, -7
BLS_FP32, BLS_FP16, BLS_U8_ROWQ, BLS_F8_ROWQ = 0, 1, 2, 3
BLS_ACT_NONE, BLS_ACT_RELU, BLS_ACT_SIGMOID = 0, 1, 2
BLS_TABLE_WISE, BLS_ROW_WISE = 0, 1

EXPORTS = [
    "bls_create", "bls_destroy", "bls_set_shard", "bls_shard_range", "bls_desc_bytes", "bls_commit", "bls_set_hot_rows", "bls_set_pool_tuning", "bls_set_plan_tuning", "bls_sizes", "bls_pooled_counts", "bls_plan", "bls_plan_noalloc", "bls_plan_weighted", "bls_step_tablewise",
    "bls_embbag_pool", "bls_embbag_pool_weighted", "bls_embbag_pool_put", "bls_embbag_pool_put_weighted", "bls_pack",
    "bls_set_ring", "bls_ring_advance", "bls_alltoallv_local", "bls_unpack", "bls_unpack_mean", "bls_ring_state",
    "bls_rank_put", "bls_rank_complete", "bls_rank_delay", "bls_mlp_layer", "bls_interact", "bls_unpack_interact", "bls_check", "bls_last_error",
]

_HERE = os.path.dirname(os.path.abspath(__file__))
_lib = None


class bls_config(C.Structure):
    _fields_ = [("P", C.c_int32), ("T", C.c_int32), ("D", C.c_int32), ("k", C.c_int32),
                ("B", C.c_int64), ("table_dtype", C.c_int32), ("part_kind", C.c_int32),
                ("rows", C.POINTER(C.c_int64)), ("table_owner", C.POINTER(C.c_int32))]


def lib_path() -> str:
    return os.path.join(_HERE, "libbls.so")


def lib() -> C.CDLL:
    """The loaded library.  Raises if it has not been built (python -m paper_2512_19342_amd.build)."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            raise RuntimeError(f"{path} is missing: build it with `python -m paper_2512_19342_amd.build` "
                               "(there is no fallback path)")
        L = C.CDLL(path)
        vp, i64p = C.c_void_p, C.c_void_p
        L.bls_create.argtypes = [C.POINTER(bls_config), C.POINTER(vp)]
        L.bls_destroy.argtypes = [vp]
        L.bls_set_shard.argtypes = [vp, C.c_int32, C.c_int32, vp, C.c_int64]
        L.bls_shard_range.argtypes = [vp, C.c_int32, C.c_int32, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
        L.bls_desc_bytes.argtypes = [vp, C.POINTER(C.c_size_t)]
        L.bls_commit.argtypes = [vp, vp, C.c_size_t, vp]
        L.bls_set_hot_rows.argtypes = [vp, C.c_int32, C.c_int32, C.POINTER(C.c_int64), C.c_int32]
        L.bls_set_pool_tuning.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32, C.c_int32]
        L.bls_set_plan_tuning.argtypes = [vp, C.c_int32]
        L.bls_sizes.argtypes = [vp, C.c_int64] + [C.POINTER(C.c_size_t)] * 4
        L.bls_pooled_counts.argtypes = [vp] + [C.POINTER(C.c_int64)] * 4
        L.bls_plan.argtypes = [vp, i64p, i64p, C.c_int64, i64p, i64p, i64p, i64p, i64p, i64p, i64p, vp, C.c_size_t, vp]
        L.bls_plan_noalloc.argtypes = [vp, i64p, i64p, C.c_int64, i64p, i64p, i64p, i64p, i64p, i64p, i64p, vp]
        L.bls_step_tablewise.argtypes = [vp, i64p, i64p, C.c_int64, i64p, i64p, i64p, i64p, i64p, i64p, i64p, vp, vp, vp,
                                         C.POINTER(C.c_int64), vp]
        L.bls_plan_weighted.argtypes = [vp, i64p, i64p, vp, C.c_int64, i64p, i64p, i64p, i64p, i64p, vp, i64p, i64p, vp,
                                        C.c_size_t, vp]
        L.bls_embbag_pool.argtypes = [vp, i64p, i64p, C.c_int64, vp, vp]
        L.bls_embbag_pool_weighted.argtypes = [vp, i64p, vp, i64p, C.c_int64, vp, vp]
        L.bls_embbag_pool_put_weighted.argtypes = [vp, i64p, vp, i64p, C.c_int64, C.c_int32, vp]
        L.bls_unpack_mean.argtypes = [vp, C.c_int64, i64p, vp, vp]
        L.bls_rank_put.argtypes = [vp, C.c_int32, i64p, vp, i64p, C.c_int64, C.c_int64, vp]
        L.bls_rank_complete.argtypes = [vp, C.c_int32, C.c_int64, i64p, vp, vp]
        L.bls_rank_delay.argtypes = [vp, C.c_uint32, vp]
        L.bls_embbag_pool_put.argtypes = [vp, i64p, i64p, C.c_int64, C.c_int32, vp]
        L.bls_pack.argtypes = [vp, vp, vp, vp]
        L.bls_set_ring.argtypes = [vp, vp, C.c_size_t]
        L.bls_ring_advance.argtypes = [vp, C.POINTER(C.c_int64), C.POINTER(C.c_int32), vp]
        L.bls_alltoallv_local.argtypes = [vp, vp, C.c_int32, vp]
        L.bls_unpack.argtypes = [vp, C.c_int64, vp, vp]
        L.bls_ring_state.argtypes = [vp, C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.POINTER(C.c_int32)]
        L.bls_mlp_layer.argtypes = [vp, vp, C.c_int64, C.c_int32, vp, vp, C.c_int32, C.c_int32, vp, vp]
        L.bls_interact.argtypes = [vp, vp, vp, vp, C.c_int64, C.c_int64, vp]
        L.bls_unpack_interact.argtypes = [vp, C.c_int64, vp, vp, vp]
        L.bls_check.argtypes = [vp, vp]
        L.bls_last_error.argtypes = [vp]
        L.bls_last_error.restype = C.c_char_p
        for name in EXPORTS:
            if name != "bls_last_error":
                getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


class BlsError(RuntimeError):
    def __init__(self, fn: str, code: int, text: str = ""):
        super().__init__(f"{fn} -> {code}: {text}")
        self.code = code


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


class Context:
    """One bls_ctx.  Methods carry the names of the C entry points."""

    def __init__(self, P: int, T: int, D: int, k: int, B: int, rows: Sequence[int], table_owner: Sequence[int],
                 table_dtype: int = BLS_FP32, part_kind: int = BLS_TABLE_WISE):
        self._h = C.c_void_p()
        rows_a = (C.c_int64 * T)(*[int(x) for x in rows])
        own_a = (C.c_int32 * T)(*[int(x) for x in table_owner])
        cfg = bls_config(P, T, D, k, B, table_dtype, part_kind, rows_a, own_a)
        rc = lib().bls_create(C.byref(cfg), C.byref(self._h))
        if rc != BLS_OK:
            self._h = C.c_void_p()
            raise BlsError("bls_create", rc, "invalid configuration")
        self.P, self.T, self.D, self.k, self.B = P, T, D, k, B
        self.K = max(k, 1)
        self.F = P if part_kind == BLS_ROW_WISE else 1
        self.part_kind, self.table_dtype = part_kind, table_dtype
        self.n_vec = self.F * T * B
        self._keep = []

    # -- plumbing
    def _call(self, name: str, *args) -> int:
        rc = getattr(lib(), name)(self._h, *args)
        if rc != BLS_OK:
            raise BlsError(name, rc, self.bls_last_error())
        return rc

    def bls_last_error(self) -> str:
        return lib().bls_last_error(self._h).decode()

    def bls_destroy(self):
        if self._h:
            lib().bls_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.bls_destroy()
        except Exception:
            pass

    # -- set-up
    def bls_set_shard(self, t: int, rank: int, rows_tensor: Optional[torch.Tensor], rows_in_shard: Optional[int] = None):
        n = int(rows_tensor.shape[0]) if rows_in_shard is None else int(rows_in_shard)
        if rows_tensor is not None:
            assert rows_tensor.is_contiguous()
            self._keep.append(rows_tensor)
        self._call("bls_set_shard", t, rank, _ptr(rows_tensor), n)

    def bls_shard_range(self, t: int, rank: int):
        lo, n = C.c_int64(), C.c_int64()
        self._call("bls_shard_range", int(t), int(rank), C.byref(lo), C.byref(n))
        return lo.value, n.value

    def bls_desc_bytes(self) -> int:
        n = C.c_size_t()
        self._call("bls_desc_bytes", C.byref(n))
        return n.value

    def bls_commit(self, desc: torch.Tensor, stream=None):
        self._keep.append(desc)
        self._call("bls_commit", _ptr(desc), desc.numel() * desc.element_size(), _stream(stream))

    def bls_set_hot_rows(self, t: int, rank: int, rows: Sequence[int]):
        a = (C.c_int64 * max(len(rows), 1))(*[int(x) for x in rows])
        self._call("bls_set_hot_rows", int(t), int(rank), a, len(rows))

    def bls_set_plan_tuning(self, scan_while_placing=-1):
        self._call("bls_set_plan_tuning", int(scan_while_placing))

    def bls_set_pool_tuning(self, lane_bytes=0, segments_per_group=0, xcd_map=-1, wide_positions=-1):
        self._call("bls_set_pool_tuning", int(lane_bytes), int(segments_per_group), int(xcd_map), int(wide_positions))

    def bls_sizes(self, max_nnz: int):
        a = [C.c_size_t() for _ in range(4)]
        self._call("bls_sizes", max_nnz, *[C.byref(x) for x in a])
        return dict(zip(("plan_ws_bytes", "pooled_bytes", "send_bytes", "slot_bytes"), (x.value for x in a)))

    def bls_pooled_counts(self):
        pp = self.P * self.P
        a = [(C.c_int64 * pp)() for _ in range(4)]
        self._call("bls_pooled_counts", *a)
        return dict(zip(("pcount", "psdispl", "prcount", "prdispl"), (list(x) for x in a)))

    def bls_set_ring(self, slots: torch.Tensor):
        self._keep.append(slots)
        self._call("bls_set_ring", _ptr(slots), slots.numel() * slots.element_size())

    # -- the path
    def bls_plan(self, indices, offsets, nnz, sendcounts, sdispls, recvcounts, rdispls, ridx, segoff, perm, ws, stream=None):
        self._call("bls_plan", _ptr(indices), _ptr(offsets), int(nnz), _ptr(sendcounts), _ptr(sdispls), _ptr(recvcounts),
                   _ptr(rdispls), _ptr(ridx), _ptr(segoff), _ptr(perm), _ptr(ws), ws.numel() * ws.element_size(),
                   _stream(stream))

    def bls_plan_noalloc(self, indices, offsets, nnz, sendcounts, sdispls, recvcounts, rdispls, ridx, segoff, perm, stream=None):
        self._call("bls_plan_noalloc", _ptr(indices), _ptr(offsets), int(nnz), _ptr(sendcounts), _ptr(sdispls),
                   _ptr(recvcounts), _ptr(rdispls), _ptr(ridx), _ptr(segoff), _ptr(perm), _stream(stream))

    def bls_step_tablewise(self, indices, offsets, nnz, sendcounts, sdispls, recvcounts, rdispls, ridx, segoff, perm,
                           pooled, send, out, stream=None) -> int:
        it = C.c_int64()
        self._call("bls_step_tablewise", _ptr(indices), _ptr(offsets), int(nnz), _ptr(sendcounts), _ptr(sdispls),
                   _ptr(recvcounts), _ptr(rdispls), _ptr(ridx), _ptr(segoff), _ptr(perm), _ptr(pooled), _ptr(send), _ptr(out),
                   C.byref(it), _stream(stream))
        return it.value

    def bls_plan_weighted(self, indices, offsets, weights, nnz, sendcounts, sdispls, recvcounts, rdispls, ridx, rweights,
                          segoff, perm, ws, stream=None):
        self._call("bls_plan_weighted", _ptr(indices), _ptr(offsets), _ptr(weights), int(nnz), _ptr(sendcounts),
                   _ptr(sdispls), _ptr(recvcounts), _ptr(rdispls), _ptr(ridx), _ptr(rweights), _ptr(segoff), _ptr(perm),
                   _ptr(ws), ws.numel() * ws.element_size(), _stream(stream))

    def bls_embbag_pool_weighted(self, ridx, rweights, segoff, nnz, pooled, stream=None):
        self._call("bls_embbag_pool_weighted", _ptr(ridx), _ptr(rweights), _ptr(segoff), int(nnz), _ptr(pooled),
                   _stream(stream))

    def bls_embbag_pool_put_weighted(self, ridx, rweights, segoff, nnz, slot, stream=None):
        self._call("bls_embbag_pool_put_weighted", _ptr(ridx), _ptr(rweights), _ptr(segoff), int(nnz), int(slot),
                   _stream(stream))

    def bls_unpack_mean(self, it, offsets, out, stream=None):
        self._call("bls_unpack_mean", int(it), _ptr(offsets), _ptr(out), _stream(stream))

    def bls_embbag_pool(self, ridx, segoff, nnz, pooled, stream=None):
        self._call("bls_embbag_pool", _ptr(ridx), _ptr(segoff), int(nnz), _ptr(pooled), _stream(stream))

    def bls_embbag_pool_put(self, ridx, segoff, nnz, slot, stream=None):
        self._call("bls_embbag_pool_put", _ptr(ridx), _ptr(segoff), int(nnz), int(slot), _stream(stream))

    def bls_pack(self, pooled, send, stream=None):
        self._call("bls_pack", _ptr(pooled), _ptr(send), _stream(stream))

    def bls_ring_advance(self, stream=None):
        it, slot = C.c_int64(), C.c_int32()
        self._call("bls_ring_advance", C.byref(it), C.byref(slot), _stream(stream))
        return it.value, slot.value

    def bls_alltoallv_local(self, send, slot, stream=None):
        self._call("bls_alltoallv_local", _ptr(send), int(slot), _stream(stream))

    def bls_unpack(self, it, out, stream=None):
        self._call("bls_unpack", int(it), _ptr(out), _stream(stream))

    def bls_rank_put(self, rank, ridx, rweights, segoff, nnz, it, stream=None):
        self._call("bls_rank_put", int(rank), _ptr(ridx), _ptr(rweights), _ptr(segoff), int(nnz), int(it), _stream(stream))

    def bls_rank_complete(self, rank, it, mean_offsets, out, stream=None):
        self._call("bls_rank_complete", int(rank), int(it), _ptr(mean_offsets), _ptr(out), _stream(stream))

    def bls_rank_delay(self, microseconds, stream=None):
        self._call("bls_rank_delay", int(microseconds), _stream(stream))

    def bls_mlp_layer(self, x, W, bias, act, y, stream=None):
        """y[M, N] = act(x[M, K] @ W[N, K].T + bias); shapes are taken from the tensors."""
        M, K = x.shape
        N = W.shape[0]
        assert W.shape == (N, K) and y.shape == (M, N) and x.is_contiguous() and W.is_contiguous() and y.is_contiguous()
        assert x.dtype == W.dtype == y.dtype == torch.float32 and (bias is None or bias.shape == (N,))
        self._call("bls_mlp_layer", _ptr(x), int(M), int(K), _ptr(W), _ptr(bias), int(N), int(act), _ptr(y), _stream(stream))

    def bls_interact(self, x, emb, z, b0=0, bn=None, stream=None):
        self._call("bls_interact", _ptr(x), _ptr(emb), _ptr(z), int(b0), int(self.B - b0 if bn is None else bn),
                   _stream(stream))

    def bls_unpack_interact(self, it, x, z, stream=None):
        self._call("bls_unpack_interact", int(it), _ptr(x), _ptr(z), _stream(stream))

    def bls_ring_state(self):
        h, t, k = C.c_int64(), C.c_int64(), C.c_int32()
        self._call("bls_ring_state", C.byref(h), C.byref(t), C.byref(k))
        return h.value, t.value, k.value

    def bls_check(self, stream=None):
        self._call("bls_check", _stream(stream))
