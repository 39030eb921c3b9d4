"""Parity at the full benchmark sizes, in the launch configuration bench.py times.

Tables (13-41 GB) are generated on the device; the oracle cannot hold them, so
  - the integer outputs of bls_plan are compared in full with the oracle's plan, and
  - pooled vectors are checked on sampled bags: the oracle sums the bag's rows, recomputed
    on the host from the table generator, and the result must sit, bit for bit, at the
    closed-form address of that bag in the pooled buffer, the send buffer, the receive slot
    and the output (addresses computed here from the layout definitions, not by the library).
Table values of these workloads lie on an exact grid, so every summation order gives the
same bits and the row-wise partial sums can be checked the same way.
"""
import numpy as np
import pytest
import torch

import oracle
import synth

pytestmark = pytest.mark.gpu


def layout(w):
    P, T, B = w.P, w.T, w.B
    first = [s * (B // P) + min(s, B % P) for s in range(P + 1)]
    if w.part_kind == 0:
        n_loc = [sum(1 for t in range(T) if w.table_owner[t] == d) for d in range(P)]
        loc = [sum(1 for u in range(t) if w.table_owner[u] == w.table_owner[t]) for t in range(T)]
    else:
        n_loc, loc = [T] * P, list(range(T))
    nsum = np.concatenate([[0], np.cumsum(n_loc)])
    return first, n_loc, loc, nsum


def bag_sum32(w, t, idx):
    """fp32 sum, in order, of rows idx of table t: the rows are regenerated on the host and handed
    to the oracle (as a little table of their own when the storage is row-quantised)."""
    ids = torch.from_numpy(np.ascontiguousarray(idx))
    if w.table_dtype in ("u8rq", "f8rq"):
        n = len(idx)
        if n == 0:
            return np.zeros(w.D, np.float32)
        mini = oracle.Case(1, 1, w.D, 1, 0, [n], [0], w.dtype_code)
        _, o32 = oracle.embbag_plain(mini, [synth.rowq_rows(w, t, ids).numpy()], np.arange(n, dtype=np.int64),
                                     np.array([0, n], np.int64))
        return o32.reshape(w.D)
    return oracle.bag_sum(synth.table_rows(w, t, ids).numpy().reshape(-1, w.D))[0]


@pytest.mark.parametrize("cfg,storage", [(3, None), (4, None), (5, None), (4, "u8rq"), (4, "f8rq"), (6, None)])
def test_full_size(cfg, storage):
    from paper_2512_19342_amd.runner import Pipeline
    w = synth.workload(cfg, "full")
    if storage:
        w.table_dtype = storage
    dev = torch.device("cuda:0")
    print(f"full-size parity {w.name}: generating {w.table_bytes() / 1e9:.1f} GB of tables", flush=True)
    tabs = [synth.make_table(w, t, dev) for t in range(w.T)]
    ix, off = synth.make_batch(w, 3, dev)
    w._cdf_cache.clear()
    nnz = int(off[-1].item())
    pipe = Pipeline(w, tabs, nnz, want_perm=True)
    out = pipe.new_out()
    it, slot = pipe.issue(ix, off, nnz)
    Y, S, R = pipe.pooled, pipe.send, pipe.slot_view(slot)
    pipe.complete(it, out)
    pipe.ctx.bls_check()
    print(f"  {nnz} lookups through the path; comparing the plan in full", flush=True)

    ix_h, off_h = ix.cpu().numpy(), off.cpu().numpy()
    case = oracle.Case(w.P, w.T, w.D, w.B, w.part_kind, w.rows, w.table_owner, w.dtype_code)
    ref = oracle.plan(case, ix_h, off_h)
    assert ref["sendcounts"].sum() == nnz
    for name, got in (("sendcounts", pipe.sendcounts), ("sdispls", pipe.sdispls), ("recvcounts", pipe.recvcounts),
                      ("rdispls", pipe.rdispls), ("segoff", pipe.segoff), ("ridx", pipe.ridx[:nnz]), ("perm", pipe.perm[:nnz])):
        assert np.array_equal(got.cpu().numpy(), ref[name]), name
    del ref

    P, T, B, D = w.P, w.T, w.B, w.D
    first, n_loc, loc, nsum = layout(w)
    rng = np.random.default_rng(cfg)
    n_samples = 1200
    ts, bs = rng.integers(0, T, n_samples), rng.integers(0, B, n_samples)
    ts[:4], bs[:4] = [0, 0, T - 1, T - 1], [0, B - 1, 0, B - 1]
    Yv, Sv, Rv = (x.view(-1, D) for x in (Y, S, R))
    for t, b in zip(ts.tolist(), bs.tolist()):
        g = t * B + b
        idx = ix_h[off_h[g]:off_h[g + 1]]
        s = next(r for r in range(P) if b < first[r + 1])
        b_loc, n = b - first[s], first[s + 1] - first[s]
        whole32 = bag_sum32(w, t, idx)
        assert np.array_equal(out[b, t].cpu().numpy().view(np.uint32), whole32.view(np.uint32)), (t, b)
        owners = [w.table_owner[t]] if w.part_kind == 0 else range(P)
        for d in owners:
            if w.part_kind == 0:
                part32 = whole32
            else:
                rps = -(-w.rows[t] // P)
                part32 = bag_sum32(w, t, idx[idx // rps == d])
            q = int(nsum[d]) + loc[t]
            sigma = int(nsum[d]) * B + n_loc[d] * first[s] + loc[t] * n + b_loc
            rho = w.F * T * first[s] + q * n + b_loc
            for name, buf, at in (("Y", Yv, q * B + b), ("S", Sv, sigma), ("R", Rv, rho)):
                assert np.array_equal(buf[at].cpu().numpy().view(np.uint32), part32.view(np.uint32)), (name, t, b, d)
    print(f"  {n_samples} sampled bags match in Y, S, R and Out", flush=True)


def test_dense_model_full_size():
    """The dense model at the benchmark's batch (16384 samples, D = 128, T = 64; layer widths as
    bench.py times them): every kernel runs on the whole batch, the oracle recomputes sampled
    samples of every kernel's output from the inputs that kernel received."""
    import paper_2512_19342_amd as A
    from paper_2512_19342_amd.runner import DenseModel
    w = synth.workload(4, "full")
    dev = torch.device("cuda:0")
    c = A.Context(w.P, w.T, w.D, w.k, w.B, w.rows, w.table_owner)
    bs, ts = synth.mlp_sizes(w, "full")
    bot, top = synth.mlp_weights(w, bs, 0), synth.mlp_weights(w, ts, 1)
    model = DenseModel(c, [(W.to(dev), b.to(dev)) for W, b in bot], [(W.to(dev), b.to(dev)) for W, b in top], w.B)
    dense = synth.dense_features(w, 2, dev)
    gen = torch.Generator(device="cpu").manual_seed(11)
    emb = (torch.randn((w.B, w.T, w.D), generator=gen) * 0.05).to(dev)       # stands in for the completed lookup
    print(f"dense model at full size: batch {w.B}, bottom {bs}, top {ts}", flush=True)
    x = model.apply_bottom(dense)
    p = model.compute_ctr(x, emb)
    c.bls_check()

    rng = np.random.default_rng(4)
    rows = np.unique(np.concatenate([[0, 127, 128, w.B - 1], rng.integers(0, w.B, 44)]))   # tile edges and random samples
    pick = torch.from_numpy(rows).to(dev)
    a = dense[pick].cpu().numpy()
    for (W, b), y in zip(bot, model.bot_act):
        ref, err = oracle.mlp_layer(a, W.numpy(), b.numpy(), 1)
        a = y[pick].cpu().numpy()
        assert np.all(np.abs(a - ref) <= err), ("bottom", W.shape)
    ref, err = oracle.interact(a, emb[pick].cpu().numpy())
    a = model.z[pick].cpu().numpy()
    assert np.all(np.abs(a - ref) <= err), "interaction"
    for i, ((W, b), y) in enumerate(zip(top, model.top_act)):
        ref, err = oracle.mlp_layer(a, W.numpy(), b.numpy(), 2 if i == len(top) - 1 else 1)
        a = y[pick].cpu().numpy()
        assert np.all(np.abs(a - ref) <= err), ("top", W.shape)
    got = p[pick].cpu().numpy()
    assert np.array_equal(got, a) and np.all((got > 0) & (got < 1))
    print(f"  {len(rows)} sampled samples match through {len(bot) + len(top)} layers and the interaction", flush=True)


@pytest.mark.parametrize("cfg", [4, 3])
def test_full_size_weighted(cfg):
    """Per-sample weights at full size (the weighted kernels in the launch shape bench.py uses), with
    mean pooling at completion for the table-wise workload: sampled bags recomputed by the oracle
    from regenerated rows - per shard in bag order, shards added in rank order."""
    from paper_2512_19342_amd.runner import Pipeline
    w = synth.workload(cfg, "full")
    dev = torch.device("cuda:0")
    mean = w.part_kind == 0
    print(f"full-size weighted parity {w.name}: generating {w.table_bytes() / 1e9:.1f} GB of tables", flush=True)
    tabs = [synth.make_table(w, t, dev) for t in range(w.T)]
    ix, off = synth.make_batch(w, 5, dev)
    w._cdf_cache.clear()
    nnz = int(off[-1].item())
    gen = torch.Generator(device="cpu").manual_seed(cfg)
    wts = torch.rand(nnz, generator=gen) * 4 - 2
    pipe = Pipeline(w, tabs, nnz)
    out = pipe.new_out()
    it, _ = pipe.issue_weighted(ix, off, wts.to(dev), nnz)
    pipe.complete(it, out, mean_offsets=off if mean else None)
    pipe.ctx.bls_check()
    ix_h, off_h, wts_h = ix.cpu().numpy(), off.cpu().numpy(), wts.numpy()
    rng = np.random.default_rng(10 + cfg)
    n_samples = 600
    ts, bs = rng.integers(0, w.T, n_samples), rng.integers(0, w.B, n_samples)
    for t, b in zip(ts.tolist(), bs.tolist()):
        g = t * w.B + b
        idx, wt = ix_h[off_h[g]:off_h[g + 1]], wts_h[off_h[g]:off_h[g + 1]]
        rows = synth.table_rows(w, t, torch.from_numpy(idx)).numpy().reshape(-1, w.D)
        if w.part_kind == 0:
            mini = oracle.Case(1, 1, w.D, 1, 0, [max(len(idx), 1)], [0], 0)
            tab = rows if len(idx) else np.zeros((1, w.D), np.float32)
            _, want = oracle.embbag_plain(mini, [np.ascontiguousarray(tab)], np.arange(len(idx)), np.array([0, len(idx)]),
                                          weights=wt, mean=mean)
            want = want.reshape(w.D)
        else:
            rps = -(-w.rows[t] // w.P)
            parts = np.zeros((w.P, w.D), np.float32)
            for d in range(w.P):
                sel = idx // rps == d
                m = int(sel.sum())
                if m:
                    mini = oracle.Case(1, 1, w.D, 1, 0, [m], [0], 0)
                    _, p32 = oracle.embbag_plain(mini, [np.ascontiguousarray(rows[sel])], np.arange(m), np.array([0, m]),
                                                 weights=wt[sel])
                    parts[d] = p32.reshape(w.D)
            want, _ = oracle.bag_sum(parts)
        assert np.array_equal(out[b, t].cpu().numpy().view(np.uint32), want.view(np.uint32)), (t, b)
    print(f"  {n_samples} sampled weighted bags match", flush=True)


@pytest.mark.parametrize("part_kind,L", [(0, 600), (1, 1100), (1, 2100)], ids=["tablewise-2.5e9", "rowwise-2.3e9", "rowwise-4.4e9"])
def test_more_than_two_to_the_31_lookups(part_kind, L):
    """A batch of 2.3e9 to 4.4e9 lookups (the last one beyond 2^32, where the row-wise plan scans in 64 bits): positions, counts and displacements beyond 32 bits.  The expected values
    are worked out with torch on the device from the definitions: owner-side order is (owner, requester,
    table, sample, position), which for these two shapes is the input order (table-wise, one table per
    rank) or the input order filtered by owner (row-wise, one table); table values are small integers, so
    every bag sum is exact in fp32 whatever the order."""
    from paper_2512_19342_amd.runner import Pipeline
    dev = torch.device("cuda:0")
    B, D = 1 << 21, 4
    if part_kind == 0:
        P, T, rows = 2, 2, [1000, 777]
    else:
        P, T, rows = 4, 1, [100003]
    nnz = T * B * L
    assert nnz > 1 << 31
    w = synth.custom("huge", P=P, T=T, D=D, B=B, k=1, part_kind=part_kind, rows=rows, bag=("fixed", L))
    print(f"large batch, part_kind {part_kind}: {nnz} lookups", flush=True)
    g = torch.Generator(device=dev)
    g.manual_seed(20250 + L)
    ix = torch.cat([torch.randint(0, rows[t], (B * L,), generator=g, device=dev, dtype=torch.int64) for t in range(T)])
    off = torch.arange(T * B + 1, device=dev, dtype=torch.int64) * L
    tabs = [((torch.arange(r, device=dev) % 7).to(torch.float32)[:, None] + torch.arange(D, device=dev, dtype=torch.float32)[None, :]).contiguous()
            for r in rows]
    pipe = Pipeline(w, tabs, nnz)
    out = pipe.new_out()
    it, slot = pipe.issue(ix, off, nnz)
    pipe.complete(it, out)
    pipe.ctx.bls_check()
    torch.cuda.synchronize()

    rps = [(r + P - 1) // P for r in rows]
    if part_kind == 0:
        assert torch.equal(pipe.ridx[:nnz], ix)
        assert torch.equal(pipe.segoff, off)
        sc = pipe.sendcounts.view(P, P).cpu().numpy()
        first = [s * (B // P) + min(s, B % P) for s in range(P + 1)]
        for s in range(P):
            for d in range(P):
                assert sc[s, d] == (first[s + 1] - first[s]) * L      # rank d owns table d
    else:
        owner = torch.div(ix, rps[0], rounding_mode="floor").to(torch.int8)
        per_bag = [(owner == d).view(B, L).sum(1) for d in range(P)]
        totals = [int(c.sum()) for c in per_bag]
        assert sum(totals) == nnz
        at = [sum(totals[:d]) for d in range(P)]                      # start of owner d's block; then the next free place
        step = 1 << 28                                                # masked selection in pieces torch can index
        for c0 in range(0, nnz, step):
            ixc, ownc = ix[c0:c0 + step], owner[c0:c0 + step]
            for d in range(P):
                want = ixc[ownc == d] - d * rps[0]
                assert torch.equal(pipe.ridx[at[d]:at[d] + want.numel()], want), f"ridx of owner {d}, lookups from {c0}"
                at[d] += want.numel()
        assert at == [sum(totals[:d + 1]) for d in range(P)]
        counts = torch.stack(per_bag).reshape(-1)                     # (owner, bag): segment lengths in segment order
        want_seg = torch.zeros(P * B + 1, dtype=torch.int64, device=dev)
        torch.cumsum(counts, 0, out=want_seg[1:])
        assert torch.equal(pipe.segoff, want_seg)
        rc = pipe.recvcounts.view(P, P)
        first = [s * (B // P) + min(s, B % P) for s in range(P + 1)]
        for d in range(P):
            for s in range(P):
                assert int(rc[d, s]) == int(per_bag[d][first[s]:first[s + 1]].sum())
        del owner
    # bag sums: exact integers
    for t in range(T):
        vals = (ix[t * B * L:(t + 1) * B * L] % rows[t] % 7).to(torch.float32).view(B, L).sum(1)   # row value is row % 7 (+ column)
        want = vals[:, None] + L * torch.arange(D, device=dev, dtype=torch.float32)[None, :]
        assert torch.equal(out[:, t, :], want), f"table {t}"
