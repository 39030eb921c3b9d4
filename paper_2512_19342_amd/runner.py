"""Buffer plumbing around one libbls context: allocates the device buffers the C entry
points need (torch is used for memory and streams only) and issues the calls of one
iteration in path order.  No arithmetic happens here."""
from __future__ import annotations

from typing import List, Optional

import torch

from . import bls


class Pipeline:
    """Device buffers + one Context for a fixed problem shape.

    ``w`` is any object with P, T, D, k, B, rows, table_owner, table_dtype ("fp32" / "fp16" / "u8rq" / "f8rq")
    and part_kind; ``tables`` are the T full tables (global row numbering) on the GPU.
    Row-wise shards are views into those tables.
    """

    def __init__(self, w, tables: List[torch.Tensor], max_nnz: int, want_perm: bool = False):
        dev = tables[0].device
        assert dev.type == "cuda", "the hot path runs on the GPU only"
        self.w, self.dev, self.max_nnz = w, dev, int(max_nnz)
        dt = {"fp32": bls.BLS_FP32, "fp16": bls.BLS_FP16, "u8rq": bls.BLS_U8_ROWQ, "f8rq": bls.BLS_F8_ROWQ}[w.table_dtype]
        width = (w.D + 8 + 15) // 16 * 16 if dt in (bls.BLS_U8_ROWQ, bls.BLS_F8_ROWQ) else w.D   # bytes per row-quantised row
        self.ctx = bls.Context(w.P, w.T, w.D, w.k, w.B, w.rows, w.table_owner, dt, w.part_kind)
        c = self.ctx
        for t, tab in enumerate(tables):
            assert tab.is_contiguous() and tab.shape == (w.rows[t], width)
            if w.part_kind == bls.BLS_TABLE_WISE:
                c.bls_set_shard(t, w.table_owner[t], tab)
            else:
                for d in range(w.P):
                    lo, n = c.bls_shard_range(t, d)     # the partition rule is the library's
                    if n == 0:
                        continue                        # empty shard: nothing to hand over
                    shard = tab[lo:lo + n]
                    if shard.data_ptr() % 16:
                        shard = shard.clone()
                    c.bls_set_shard(t, d, shard)
        self.desc = torch.empty(c.bls_desc_bytes(), dtype=torch.uint8, device=dev)
        c.bls_commit(self.desc)
        sz = c.bls_sizes(self.max_nnz)
        pp = w.P * w.P
        i64 = dict(dtype=torch.int64, device=dev)
        self.sendcounts, self.sdispls = torch.zeros(pp, **i64), torch.zeros(pp, **i64)
        self.recvcounts, self.rdispls = torch.zeros(pp, **i64), torch.zeros(pp, **i64)
        self.ridx = torch.zeros(max(self.max_nnz, 1), **i64)
        self.segoff = torch.zeros(c.n_vec + 1, **i64)
        self.perm = torch.zeros(max(self.max_nnz, 1), **i64) if want_perm else None
        self.rweights = None                                   # allocated on first weighted call
        self.ws = torch.zeros((sz["plan_ws_bytes"] + 7) // 8, **i64)
        nfl = c.n_vec * w.D
        self.pooled = torch.zeros(nfl, dtype=torch.float32, device=dev)
        self.send = torch.zeros(nfl, dtype=torch.float32, device=dev)
        self.slots = torch.zeros(c.K * nfl, dtype=torch.float32, device=dev)
        c.bls_set_ring(self.slots)
        self.n_floats = nfl

    def set_hot_rows(self, lists):
        """Name popular rows: ``lists`` maps (table, rank) to local row numbers of that shard, most
        popular first (bls_set_hot_rows); the descriptor tables are committed again."""
        c = self.ctx
        for (t, rank), rows in lists.items():
            c.bls_set_hot_rows(t, rank, rows)
        self.desc = torch.empty(c.bls_desc_bytes(), dtype=torch.uint8, device=self.dev)
        c.bls_commit(self.desc)

    def hot_rows_from_batch(self, indices: torch.Tensor, offsets: torch.Tensor, per_shard: int):
        """The ``per_shard`` most looked-up rows of every shard in one batch (counted with torch on the
        batch's device): what a caller would take from its own traffic statistics."""
        w, c = self.w, self.ctx
        lists = {}
        for t in range(w.T):
            ix = indices[int(offsets[t * w.B]):int(offsets[(t + 1) * w.B])]
            if ix.numel() == 0:
                continue
            rows, counts = torch.unique(ix, return_counts=True)
            ranks = range(w.P) if w.part_kind == bls.BLS_ROW_WISE else [w.table_owner[t]]
            for d in ranks:
                lo, n = c.bls_shard_range(t, d)
                sel = (rows >= lo) & (rows < lo + n)
                r, k = rows[sel], counts[sel]
                if r.numel() == 0:
                    continue
                top = torch.topk(k, min(per_shard, r.numel())).indices
                lists[(t, d)] = (r[top] - lo).tolist()
        return lists

    def new_out(self) -> torch.Tensor:
        return torch.empty((self.w.B, self.w.T, self.w.D), dtype=torch.float32, device=self.dev)

    # one iteration, split where the ring allows other iterations in between
    def issue(self, indices: torch.Tensor, offsets: torch.Tensor, nnz: int, stream=None):
        """plan, pool, pack, take a ring slot, exchange.  Returns (iteration, slot)."""
        c = self.ctx
        assert nnz <= self.max_nnz
        c.bls_plan(indices, offsets, nnz, self.sendcounts, self.sdispls, self.recvcounts, self.rdispls,
                   self.ridx, self.segoff, self.perm, self.ws, stream)
        c.bls_embbag_pool(self.ridx, self.segoff, nnz, self.pooled, stream)
        c.bls_pack(self.pooled, self.send, stream)
        it, slot = c.bls_ring_advance(stream)
        c.bls_alltoallv_local(self.send, slot, stream)
        return it, slot

    def issue_fused(self, indices: torch.Tensor, offsets: torch.Tensor, nnz: int, stream=None):
        """plan, take a ring slot, pool straight into it (no pooled or send buffer)."""
        c = self.ctx
        assert nnz <= self.max_nnz
        c.bls_plan(indices, offsets, nnz, self.sendcounts, self.sdispls, self.recvcounts, self.rdispls,
                   self.ridx, self.segoff, self.perm, self.ws, stream)
        it, slot = c.bls_ring_advance(stream)
        c.bls_embbag_pool_put(self.ridx, self.segoff, nnz, slot, stream)
        return it, slot

    def issue_weighted(self, indices, offsets, weights, nnz: int, fused: bool = False, stream=None):
        """As issue / issue_fused with per-sample weights (float32, input order)."""
        c = self.ctx
        assert nnz <= self.max_nnz
        if self.rweights is None:
            self.rweights = torch.zeros(max(self.max_nnz, 1), dtype=torch.float32, device=self.dev)
        c.bls_plan_weighted(indices, offsets, weights, nnz, self.sendcounts, self.sdispls, self.recvcounts, self.rdispls,
                            self.ridx, self.rweights, self.segoff, self.perm, self.ws, stream)
        if fused:
            it, slot = c.bls_ring_advance(stream)
            c.bls_embbag_pool_put_weighted(self.ridx, self.rweights, self.segoff, nnz, slot, stream)
            return it, slot
        c.bls_embbag_pool_weighted(self.ridx, self.rweights, self.segoff, nnz, self.pooled, stream)
        c.bls_pack(self.pooled, self.send, stream)
        it, slot = c.bls_ring_advance(stream)
        c.bls_alltoallv_local(self.send, slot, stream)
        return it, slot

    def complete(self, it: int, out: torch.Tensor, stream=None, mean_offsets: Optional[torch.Tensor] = None):
        if mean_offsets is not None:
            self.ctx.bls_unpack_mean(it, mean_offsets, out, stream)
        else:
            self.ctx.bls_unpack(it, out, stream)

    def step(self, indices, offsets, nnz, out, stream=None):
        it, _ = self.issue(indices, offsets, nnz, stream)
        self.complete(it, out, stream)

    def step_one_launch(self, indices, offsets, nnz, out, stream=None) -> int:
        """The whole iteration in one launch (table-wise partitions, nothing in flight): bls_step_tablewise.
        Returns the iteration number; its receive regions are in slot ``iteration % K``."""
        assert nnz <= self.max_nnz
        return self.ctx.bls_step_tablewise(indices, offsets, nnz, self.sendcounts, self.sdispls, self.recvcounts, self.rdispls,
                                           self.ridx, self.segoff, self.perm, self.pooled, self.send, out, stream)

    def slot_view(self, slot: int) -> torch.Tensor:
        return self.slots[slot * self.n_floats:(slot + 1) * self.n_floats]


class DenseModel:
    """Bottom MLP, dot interaction and top MLP around a Pipeline's lookups (Listings 1 and 2:
    apply_mlp, interact_features): layer weights and activation buffers on the GPU, every
    step a call into the library.  ``bottom`` / ``top`` are lists of (W [N, K], bias [N])
    float32 tensors; ReLU between layers, a sigmoid after the last top layer."""

    def __init__(self, ctx: "bls.Context", bottom, top, batch: int):
        self.ctx, self.B = ctx, int(batch)
        dev = bottom[0][0].device
        assert dev.type == "cuda", "the dense layers run on the GPU only"
        self.bottom = [(W.contiguous(), b.contiguous()) for W, b in bottom]
        self.top = [(W.contiguous(), b.contiguous()) for W, b in top]
        zdim = ctx.D + ctx.T * (ctx.T + 1) // 2
        assert self.bottom[-1][0].shape[0] == ctx.D and self.top[0][0].shape[1] == zdim
        f32 = dict(dtype=torch.float32, device=dev)
        self.bot_act = [torch.empty((self.B, W.shape[0]), **f32) for W, _ in self.bottom]
        self.z = torch.empty((self.B, zdim), **f32)
        self.top_act = [torch.empty((self.B, W.shape[0]), **f32) for W, _ in self.top]

    def apply_bottom(self, dense: torch.Tensor, x_out: Optional[torch.Tensor] = None, stream=None,
                     rows: Optional[tuple] = None) -> torch.Tensor:
        """x = bottom MLP of the dense features ``[B, n_dense]``, written to ``x_out`` [B, D]
        (default: the model's own buffer, overwritten by the next call).  ``rows = (b0, bn)``
        restricts the work to those samples (one rank's mini-batch); every tensor is the full one."""
        lo, hi = (0, self.B) if rows is None else (rows[0], rows[0] + rows[1])
        a = dense[lo:hi]
        for i, ((W, b), y) in enumerate(zip(self.bottom, self.bot_act)):
            if x_out is not None and i == len(self.bottom) - 1:
                y = x_out
            self.ctx.bls_mlp_layer(a, W, b, bls.BLS_ACT_RELU, y[lo:hi], stream)
            a = y[lo:hi]
        return y

    def compute_ctr(self, x: torch.Tensor, emb, p_out: Optional[torch.Tensor] = None, stream=None,
                    rows: Optional[tuple] = None) -> torch.Tensor:
        """The prediction [B, 1] from the bottom MLP's output and the completed lookup [B, T, D].
        ``emb`` may instead be the number of the oldest iteration in flight: its completion is then
        folded into the interaction (bls_unpack_interact; whole batch only)."""
        lo, hi = (0, self.B) if rows is None else (rows[0], rows[0] + rows[1])
        if isinstance(emb, int):
            assert rows is None
            self.ctx.bls_unpack_interact(emb, x, self.z, stream)
        else:
            self.ctx.bls_interact(x, emb, self.z, lo, hi - lo, stream)
        a = self.z[lo:hi]
        for i, ((W, b), y) in enumerate(zip(self.top, self.top_act)):
            last = i == len(self.top) - 1
            if last and p_out is not None:
                y = p_out
            self.ctx.bls_mlp_layer(a, W, b, bls.BLS_ACT_SIGMOID if last else bls.BLS_ACT_RELU, y[lo:hi], stream)
            a = y[lo:hi]
        return y


class BlsDlrm:
    """The forward loop of Listing 2 on one stream: every call issues one iteration's lookup
    (plan, pool straight into the ring slot) and its bottom MLP, and completes the oldest
    iteration (unpack, interaction, top MLP) once more than ``bound`` are unfinished; the last
    batch drains the ring.  Results do not depend on the bound; only how far completion lags.

    The ring has K = max(bound, 1) slots, so with bound >= 1 the oldest iteration is completed
    before the one that would reuse its slot is issued (Fig. "bound": the process blocks on
    iteration 0 before it may start iteration k)."""

    def __init__(self, pipe: Pipeline, model: DenseModel, fused_completion: bool = False, lookup_stream=None):
        self.pipe, self.model, self.fused_completion = pipe, model, fused_completion
        # With a lookup stream the sparse side (plan, pool into the slot) runs there and the dense side
        # (MLPs, completion, interaction) on the caller's stream: the library's slot events order the
        # two, and the gather-bound pooling of one iteration overlaps the matrix work of another.
        self.lookup_stream = lookup_stream
        self.bound = pipe.w.k
        n = pipe.ctx.K + 1
        f32 = dict(dtype=torch.float32, device=pipe.dev)
        self.x_list = [torch.empty((pipe.w.B, pipe.w.D), **f32) for _ in range(n)]   # the listing's x-list
        self.emb = pipe.new_out()
        self.unfinished: List[int] = []

    def _finish_tail(self, stream=None):
        it = self.unfinished.pop(0)
        p = torch.empty((self.pipe.w.B, 1), dtype=torch.float32, device=self.pipe.dev)
        if self.fused_completion:                               # no [B, T, D] copy-out: the interaction reads the slot
            self.model.compute_ctr(self.x_list[it % len(self.x_list)], it, p, stream)
        else:
            self.pipe.complete(it, self.emb, stream)
            self.model.compute_ctr(self.x_list[it % len(self.x_list)], self.emb, p, stream)
        return it, p

    def forward(self, dense, indices, offsets, nnz: int, last_batch: bool = False, stream=None):
        """Returns the (iteration, prediction) pairs completed by this call, oldest first."""
        done = []
        if self.bound > 0 and len(self.unfinished) == self.pipe.ctx.K:
            done.append(self._finish_tail(stream))
        it, _ = self.pipe.issue_fused(indices, offsets, nnz, self.lookup_stream if self.lookup_stream is not None else stream)
        self.unfinished.append(it)
        self.model.apply_bottom(dense, self.x_list[it % len(self.x_list)], stream)
        if len(self.unfinished) > self.bound:
            done.append(self._finish_tail(stream))
        if last_batch:
            while self.unfinished:
                done.append(self._finish_tail(stream))
        return done


class BlsDlrmRanks:
    """Listing 2 run by every simulated rank on a stream of its own.  ``issue(rank, ...)`` is the
    rank's part of an iteration's start - its puts into the ring slot (owner side) and the bottom
    MLP of its mini-batch; ``finish(rank, it)`` completes the rank's oldest iteration - copy-out
    of its samples, interaction, top MLP.  The caller keeps every rank within K iterations of its
    own completions (the library refuses a put into a slot a requester has not been asked to
    release) and may run the ranks in any order; ranks never wait for each other on the host."""

    def __init__(self, pipe: Pipeline, model: DenseModel, streams):
        assert len(streams) == pipe.w.P
        self.pipe, self.model, self.streams = pipe, model, streams
        K, w = pipe.ctx.K, pipe.w
        f32 = dict(dtype=torch.float32, device=pipe.dev)
        self.first = [s * (w.B // w.P) + min(s, w.B % w.P) for s in range(w.P + 1)]
        self.x_list = [torch.empty((w.B, w.D), **f32) for _ in range(K + 1)]
        self.emb = [pipe.new_out() for _ in range(K)]
        self.pred = [torch.empty((w.B, 1), **f32) for _ in range(K)]

    def rows(self, rank: int) -> tuple:
        return self.first[rank], self.first[rank + 1] - self.first[rank]

    def issue(self, rank: int, it: int, ridx, segoff, nnz: int, dense, delay_us: int = 0):
        c, st = self.pipe.ctx, self.streams[rank]
        if delay_us:
            c.bls_rank_delay(int(delay_us), st)
        c.bls_rank_put(rank, ridx, None, segoff, nnz, it, st)
        self.model.apply_bottom(dense, self.x_list[it % len(self.x_list)], st, self.rows(rank))

    def finish(self, rank: int, it: int) -> torch.Tensor:
        """Returns the prediction buffer of iteration ``it`` (valid for this rank's samples once
        its stream has run; reused K iterations later)."""
        c, st, K = self.pipe.ctx, self.streams[rank], self.pipe.ctx.K
        c.bls_rank_complete(rank, it, None, self.emb[it % K], st)
        self.model.compute_ctr(self.x_list[it % len(self.x_list)], self.emb[it % K], self.pred[it % K], st, self.rows(rank))
        return self.pred[it % K]
