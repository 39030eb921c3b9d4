"""Pins for the CPU oracle: everything here runs without a GPU and checks the oracle
against things other than itself - brute force on tiny inputs (python's stable sort,
dictionaries, numpy.array_split), closed forms, invariants, library routines
(numpy.take, torch embedding_bag) and the values the paper prints."""
import itertools
import os
from collections import Counter

import numpy as np
import pytest
import torch

import oracle
import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------- helpers

def np_tables(w, device="cpu"):
    return [synth.make_table(w, t, "cpu").numpy() for t in range(w.T)]


def case_of(w):
    return oracle.Case(w.P, w.T, w.D, w.B, w.part_kind, w.rows, w.table_owner, w.dtype_code)


def brute(w, tables, indices, offsets):
    """Everything from first principles in python: no scans, python's stable sort."""
    P, T, B, D = w.P, w.T, w.B, w.D
    blocks = np.array_split(np.arange(B), P)          # first B mod P ranks get one extra
    s_of_b = np.empty(B, int)
    bloc_of_b = np.empty(B, int)
    for s, blk in enumerate(blocks):
        s_of_b[blk] = s
        bloc_of_b[blk] = np.arange(len(blk))
    if w.part_kind == 0:
        n_loc = [sum(1 for t in range(T) if w.table_owner[t] == d) for d in range(P)]
        loc = [sum(1 for u in range(t) if w.table_owner[u] == w.table_owner[t]) for t in range(T)]
    else:
        n_loc, loc = [T] * P, list(range(T))
    rec = []
    for t in range(T):
        for b in range(B):
            g = t * B + b
            for l in range(offsets[g], offsets[g + 1]):
                idx = int(indices[l])
                if w.part_kind == 1:
                    rps = -(-w.rows[t] // P)
                    d, r = idx // rps, idx % rps
                else:
                    d, r = w.table_owner[t], idx
                rec.append(dict(l=l, t=t, b=b, s=int(s_of_b[b]), d=d, r=r))
    nnz = len(rec)
    send_order = sorted(range(nnz), key=lambda i: (rec[i]["s"], rec[i]["d"]))
    recv_order = sorted(range(nnz), key=lambda i: (rec[i]["d"], rec[i]["s"]))
    perm = np.empty(nnz, np.int64)
    for pos, i in enumerate(send_order):
        perm[i] = pos
    ridx = np.array([rec[i]["r"] for i in recv_order], np.int64)
    cnt = Counter((x["s"], x["d"]) for x in rec)
    sendcounts = np.array([[cnt[(s, d)] for d in range(P)] for s in range(P)], np.int64)
    # segments in (d, s, t_loc, b_loc) order
    segcnt = Counter((x["d"], x["s"], loc[x["t"]], int(bloc_of_b[x["b"]])) for x in rec)
    seglen = []
    for d in range(P):
        for s in range(P):
            for tl in range(n_loc[d]):
                for bl in range(len(blocks[s])):
                    seglen.append(segcnt[(d, s, tl, bl)])
    segoff = np.concatenate([[0], np.cumsum(seglen)]).astype(np.int64)
    out = np.zeros((B, T, D), np.float32)
    for x in rec:
        row = tables[x["t"]][int(indices[x["l"]])].astype(np.float32)
        out[x["b"], x["t"]] = out[x["b"], x["t"]] + row
    return dict(perm=perm, ridx=ridx, sendcounts=sendcounts, segoff=segoff, out=out,
                n_loc=n_loc, loc=loc, blocks=blocks, rec=rec)


TINY = [
    dict(P=2, T=3, D=4, B=4, part_kind=0, rows=[7, 5, 9], bag=("uniform", 0, 3)),
    dict(P=3, T=4, D=4, B=7, part_kind=0, rows=[11, 3, 8, 20], bag=("uniform", 0, 4)),     # P does not divide B
    dict(P=3, T=2, D=8, B=5, part_kind=1, rows=[10, 4], bag=("uniform", 0, 6)),             # ragged last shard
    dict(P=4, T=3, D=4, B=8, part_kind=1, rows=[3, 17, 1], bag=("uniform", 1, 5)),          # empty shards (rows < P)
    dict(P=1, T=2, D=4, B=3, part_kind=0, rows=[5, 6], bag=("fixed", 2)),
]


def tiny_workload(spec, seed=11, values="gauss"):
    return synth.custom("tiny", k=1, values=values, seed=seed, **spec)


@pytest.mark.parametrize("spec", TINY)
@pytest.mark.parametrize("seed", [3, 4])
def test_plan_matches_brute_force(spec, seed):
    w = tiny_workload(spec, seed)
    ix, off = (x.numpy() for x in synth.make_batch(w, 0))
    tabs = np_tables(w)
    ref = brute(w, tabs, ix, off)
    got = oracle.plan(case_of(w), ix, off)
    P = w.P
    assert np.array_equal(got["sendcounts"].reshape(P, P), ref["sendcounts"])
    assert np.array_equal(got["recvcounts"].reshape(P, P), ref["sendcounts"].T)
    assert np.array_equal(got["perm"], ref["perm"])
    assert np.array_equal(got["ridx"], ref["ridx"])
    assert np.array_equal(got["segoff"], ref["segoff"])
    sd = np.cumsum(ref["sendcounts"], axis=1) - ref["sendcounts"]
    rd = np.cumsum(ref["sendcounts"].T, axis=1) - ref["sendcounts"].T
    assert np.array_equal(got["sdispls"].reshape(P, P), sd)
    assert np.array_equal(got["rdispls"].reshape(P, P), rd)


@pytest.mark.parametrize("spec", TINY)
def test_pipeline_out_matches_brute_force_and_plain(spec):
    w = tiny_workload(spec, 5)
    ix, off = (x.numpy() for x in synth.make_batch(w, 0))
    tabs = np_tables(w)
    ref = brute(w, tabs, ix, off)
    c = case_of(w)
    o64, o32 = oracle.embbag_plain(c, tabs, ix, off)
    assert np.array_equal(o32.view(np.uint32), ref["out"].view(np.uint32))
    full = oracle.pipeline(c, tabs, ix, off)
    if w.part_kind == 0:
        assert np.array_equal(full["Out"].view(np.uint32), o32.view(np.uint32))
    mass = oracle.embbag_absmass(c, tabs, ix, off)
    assert np.all(np.abs(full["Out"].astype(np.float64) - o64) <= 1e-6 * mass + 1e-300)
    # fp64 definition against numpy's own float64 accumulation
    for x in (0, w.B - 1):
        for t in range(w.T):
            g = t * w.B + x
            rows = tabs[t][ix[off[g]:off[g + 1]]].astype(np.float64)
            assert np.allclose(o64[x, t], rows.sum(axis=0), rtol=1e-14, atol=1e-300)


def test_closed_form_counts_cfg1_cfg2():
    w = synth.workload(1)
    ix, off = (x.numpy() for x in synth.make_batch(w, 0))
    p = oracle.plan(case_of(w), ix, off)
    assert np.all(p["sendcounts"] == 64 * 4) and p["sendcounts"].sum() == 1024
    assert np.array_equal(p["ridx"].reshape(2, 2, 4, 64)[0, 1, 2], ix.reshape(8, 128)[4, 64:128])
    w = synth.workload(2)
    ix, off = (x.numpy() for x in synth.make_batch(w, 0))
    p = oracle.plan(case_of(w), ix, off)
    n_loc = np.bincount(w.table_owner, minlength=4)
    assert np.array_equal(p["sendcounts"].reshape(4, 4), np.tile(512 * n_loc, (4, 1)))
    assert p["sendcounts"].sum() == 53248
    # balanced-by-rows partition: no rank is more than one largest table above the lightest
    load = np.bincount(w.table_owner, weights=w.rows, minlength=4)
    assert load.max() - load.min() <= max(w.rows)


@pytest.mark.parametrize("cfg", [3, 4, 5])
def test_plan_invariants_small_twins(cfg):
    w = synth.workload(cfg, "small")
    ix, off = (x.numpy() for x in synth.make_batch(w, 0))
    P, T, B = w.P, w.T, w.B
    p = oracle.plan(case_of(w), ix, off)
    nnz = int(off[-1])
    sc, rc = p["sendcounts"].reshape(P, P), p["recvcounts"].reshape(P, P)
    assert sc.sum() == nnz and np.array_equal(rc, sc.T)
    for cnt, dsp in ((sc, p["sdispls"].reshape(P, P)), (rc, p["rdispls"].reshape(P, P))):
        assert np.all(dsp[:, 0] == 0)
        assert np.array_equal(dsp[:, 1:] - dsp[:, :-1], cnt[:, :-1])
    if cfg == 5:
        assert np.all(sc.sum(axis=1) == T * (B // P) * 32)
    # perm is a bijection; keys read through it are sorted; equal keys keep input order
    perm = p["perm"]
    assert np.array_equal(np.sort(perm), np.arange(nnz))
    lens = np.diff(off)
    bag_of_l = np.repeat(np.arange(T * B), lens)
    t_of_l, b_of_l = bag_of_l // B, bag_of_l % B
    s_of_l = b_of_l // (B // P)
    if w.part_kind == 1:
        rps = -(-np.array(w.rows)[t_of_l] // P)
        d_of_l, r_of_l = ix // rps, ix % rps
    else:
        d_of_l, r_of_l = np.array(w.table_owner)[t_of_l], ix
    key = s_of_l * P + d_of_l
    inv = np.empty(nnz, np.int64)
    inv[perm] = np.arange(nnz)
    assert np.all(np.diff(key[inv]) >= 0)
    same = np.diff(key[inv]) == 0
    assert np.all(np.diff(inv)[same] > 0)
    # numpy's stable argsort is the unique stable permutation
    assert np.array_equal(inv, np.argsort(key, kind="stable"))
    rkey = d_of_l * P + s_of_l
    assert np.array_equal(p["ridx"], r_of_l[np.argsort(rkey, kind="stable")])
    # segoff: starts at 0, ends at nnz, non-decreasing, block boundaries give recvcounts
    so = p["segoff"]
    assert so[0] == 0 and so[-1] == nnz and np.all(np.diff(so) >= 0)
    n_loc = np.bincount(w.table_owner, minlength=P) if w.part_kind == 0 else np.full(P, T)
    edge = 0
    for d in range(P):
        for s in range(P):
            n = n_loc[d] * (B // P)
            assert so[edge + n] - so[edge] == rc[d, s]
            edge += n


def test_pooling_one_is_a_row_copy_and_integer_tables():
    w = synth.workload(2)
    ix, off = (x.numpy() for x in synth.make_batch(w, 0))
    tabs = np_tables(w)
    c = case_of(w)
    o64, o32 = oracle.embbag_plain(c, tabs, ix, off)
    res = oracle.pipeline(c, tabs, ix, off)
    for t in range(w.T):
        take = np.take(tabs[t], ix[t * w.B:(t + 1) * w.B], axis=0)
        take = take + np.float32(0.0)               # accumulator starts at +0: -0.0 rows become +0.0
        assert np.array_equal(o32[:, t].view(np.uint32), take.view(np.uint32))
        assert np.array_equal(res["Out"][:, t].view(np.uint32), take.view(np.uint32))
    # W[i][c] = i  =>  pooled = sum of the bag's indices; all-ones => bag length
    w = synth.custom("ints", P=3, T=3, D=4, k=1, B=9, rows=[50, 60, 70], part_kind=1, bag=("uniform", 0, 9))
    ix, off = (x.numpy() for x in synth.make_batch(w, 1))
    c = case_of(w)
    tabs = [np.repeat(np.arange(r, dtype=np.float32)[:, None], 4, axis=1).copy() for r in w.rows]
    out = oracle.pipeline(c, tabs, ix, off)["Out"]
    ones = oracle.pipeline(c, [np.ones((r, 4), np.float32) for r in w.rows], ix, off)["Out"]
    for t in range(3):
        for b in range(9):
            g = t * 9 + b
            assert np.all(out[b, t] == ix[off[g]:off[g + 1]].sum())
            assert np.all(ones[b, t] == off[g + 1] - off[g])


@pytest.mark.parametrize("cfg,size", [(1, "full"), (2, "full"), (3, "small"), (5, "small")])
def test_against_torch_embedding_bag(cfg, size):
    w = synth.workload(cfg, size)
    if cfg == 3:
        w.values = "gauss"                          # order-sensitive values for the row-wise path
    ix, off = synth.make_batch(w, 0)
    tabs_t = [synth.make_table(w, t, "cpu") for t in range(w.T)]
    tabs = [x.numpy() for x in tabs_t]
    c = case_of(w)
    o64, o32 = oracle.embbag_plain(c, tabs, ix.numpy(), off.numpy())
    out = oracle.pipeline(c, tabs, ix.numpy(), off.numpy())["Out"]
    mass = oracle.embbag_absmass(c, tabs, ix.numpy(), off.numpy())
    tol = 1e-3 if w.table_dtype == "fp16" else 1e-6
    for t in range(w.T):
        o = off[t * w.B:(t + 1) * w.B + 1]
        sub = ix[o[0]:o[-1]]
        ref64 = torch.nn.functional.embedding_bag(sub, tabs_t[t].double(), o[:-1] - o[0], mode="sum").numpy()
        ref32 = torch.nn.functional.embedding_bag(sub, tabs_t[t].float(), o[:-1] - o[0], mode="sum").numpy()
        assert np.allclose(o64[:, t], ref64, rtol=1e-13, atol=1e-300)
        assert np.all(np.abs(o32[:, t] - ref64) <= tol * mass[:, t])
        assert np.all(np.abs(out[:, t] - ref64) <= tol * mass[:, t])
        assert np.all(np.abs(ref32 - ref64) <= tol * mass[:, t])     # the library itself meets the bound
    if w.values == "grid":                           # exact grid: every order gives the same bits
        assert np.array_equal(out.view(np.uint32), o32.view(np.uint32))
        assert np.array_equal(out.astype(np.float64), o64)


def test_half_conversion_all_bit_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    tab = bits.view(np.float16).reshape(65536, 1).copy()
    c = oracle.Case(1, 1, 1, 65536, 0, [65536], [0], dtype=1)
    ix, off = np.arange(65536), np.arange(65537)
    _, o32 = oracle.embbag_plain(c, [tab], ix, off, want64=False)
    with np.errstate(invalid="ignore"):
        ref = tab.astype(np.float32).reshape(-1) + np.float32(0.0)
    ok = ~np.isnan(ref)
    assert np.array_equal(o32.reshape(-1)[ok].view(np.uint32), ref[ok].view(np.uint32))
    assert np.all(np.isnan(o32.reshape(-1)[~ok]))


def _address_tag_Y(w, n_loc):
    Y = []
    for d in range(w.P):
        y = np.zeros((n_loc[d], w.B, w.D), np.float32)
        y[:, :, 0] = (d * 64 + np.arange(n_loc[d]))[:, None]
        y[:, :, 1] = np.arange(w.B)[None, :]
        y[:, :, 2:] = np.random.default_rng(d).integers(-8, 8, size=y[:, :, 2:].shape)
        Y.append(y)
    return Y


@pytest.mark.parametrize("spec", TINY[:4])
def test_pack_exchange_unpack_addresses(spec):
    """Every pooled vector carries its own (owner, local table, sample) and must land at the
    closed-form address in the send regions, the receive regions and the output."""
    w = tiny_workload(spec)
    P, T, B, D = w.P, w.T, w.B, w.D
    c = case_of(w)
    blocks = np.array_split(np.arange(B), P)
    if w.part_kind == 0:
        n_loc = [sum(1 for t in range(T) if w.table_owner[t] == d) for d in range(P)]
        tabs_of = [[t for t in range(T) if w.table_owner[t] == d] for d in range(P)]
    else:
        n_loc, tabs_of = [T] * P, [list(range(T))] * P
    Yl = _address_tag_Y(w, n_loc)
    Y = np.concatenate([y.reshape(-1) for y in Yl])
    S = oracle.pack(c, Y)
    R = oracle.exchange(c, S)
    Out = oracle.unpack(c, R)
    # S: owner regions one after another, each [s][t_loc][b_loc]
    exp_S = np.concatenate([Yl[d][:, blocks[s]].reshape(-1) for d in range(P) for s in range(P)])
    assert np.array_equal(S, exp_S)
    # R: requester regions one after another, each [d][t_loc][b_loc]
    exp_R = np.concatenate([Yl[d][:, blocks[s]].reshape(-1) for s in range(P) for d in range(P)])
    assert np.array_equal(R, exp_R)
    pc = oracle.pooled_counts(c)
    assert np.array_equal(pc["pcount"].reshape(P, P),
                          np.array([[n_loc[d] * len(blocks[s]) * D for s in range(P)] for d in range(P)]))
    assert pc["pcount"].sum() == c.n_vec * D
    # Out built directly from Y
    exp = np.zeros((B, T, D), np.float32)
    for d in range(P):
        for tl, t in enumerate(tabs_of[d]):
            exp[:, t] += Yl[d][tl]
    assert np.array_equal(Out, exp)
    if w.part_kind == 0:
        for d in range(P):
            for tl, t in enumerate(tabs_of[d]):
                assert np.all(Out[:, t, 0] == d * 64 + tl) and np.array_equal(Out[:, t, 1], np.arange(B))


def test_alltoallv_textbook_irregular():
    rng = np.random.default_rng(0)
    P = 4
    counts = rng.integers(0, 6, size=(P, P))
    counts[1, 2] = 0
    send_blocks = [[rng.normal(size=counts[s, d]).astype(np.float32) for d in range(P)] for s in range(P)]
    send = np.concatenate([np.concatenate(send_blocks[s]) if counts[s].sum() else np.zeros(0, np.float32) for s in range(P)])
    sdis = np.cumsum(counts, axis=1) - counts
    rcnt = counts.T.copy()
    rdis = np.cumsum(rcnt, axis=1) - rcnt
    sbase = np.cumsum(counts.sum(axis=1)) - counts.sum(axis=1)
    rbase = np.cumsum(rcnt.sum(axis=1)) - rcnt.sum(axis=1)
    recv = oracle.alltoallv(P, send, sbase, counts.reshape(-1), sdis.reshape(-1), rbase, rcnt.reshape(-1),
                            rdis.reshape(-1), int(counts.sum()))
    exp = np.concatenate([send_blocks[s][d] for d in range(P) for s in range(P)])
    assert np.array_equal(recv, exp)
    bad = rcnt.copy()
    bad[0, 1] += 1
    with pytest.raises(oracle.OracleError):
        oracle.alltoallv(P, send, sbase, counts.reshape(-1), sdis.reshape(-1), rbase, bad.reshape(-1),
                         rdis.reshape(-1), int(counts.sum()))


def test_errors_are_raised():
    w = tiny_workload(TINY[0])
    ix, off = (x.numpy().copy() for x in synth.make_batch(w, 0))
    c = case_of(w)
    bad = ix.copy()
    bad[0] = w.rows[0]
    with pytest.raises(oracle.OracleError) as e:
        oracle.plan(c, bad, off)
    assert e.value.code == -2
    bad[0] = -1
    with pytest.raises(oracle.OracleError):
        oracle.plan(c, bad, off)
    boff = off.copy()
    boff[2], boff[3] = boff[3] + 1, boff[2]
    if boff[3] < boff[2]:
        with pytest.raises(oracle.OracleError):
            oracle.plan(c, ix, boff)


# ----------------------------------------------------------------------------- ring

def test_ring_figure_scenario():
    lines = [x.strip() for x in open(os.path.join(GOLD, "bound_figure_scenario.txt")) if x.strip() and not x.startswith("#")]
    ring = oracle.RingModel(int(lines[0].split()[1]))
    for ln in lines[1:]:
        lhs, rhs = [x.strip() for x in ln.split("->")]
        if lhs == "acquire":
            if rhs == "FULL":
                with pytest.raises(oracle.RingFull):
                    ring.acquire()
            else:
                assert list(ring.acquire()) == [int(x) for x in rhs.split()]
        else:
            assert ring.retire(int(lhs.split()[1])) == int(rhs)


def test_ring_memory_example():
    for ln in open(os.path.join(GOLD, "ring_memory_example.txt")):
        if ln.startswith("#") or not ln.strip():
            continue
        b, s, nt, nbytes, kb = (int(x) for x in ln.split())
        assert oracle.ring_bytes_per_bound(s, b, nt) == nbytes
        assert round(nbytes / 1000, -1) == kb     # "about 860 KB"


def test_ring_fifo_and_slots():
    for k in (0, 1, 2, 4):
        ring = oracle.RingModel(k)
        K = max(k, 1)
        assert ring.K == K
        with pytest.raises(oracle.RingEmpty):
            ring.retire(0)
        seen = []
        for j in range(3 * K + 1):
            if len(ring.in_flight) == K:
                with pytest.raises(oracle.RingFull):
                    ring.acquire()
                tail = ring.in_flight[0]
                if K > 1:
                    with pytest.raises(oracle.RingOrder):
                        ring.retire(ring.in_flight[1])
                assert ring.retire(tail) == tail % K
            it, slot = ring.acquire()
            assert it == j and slot == j % K
            seen.append(slot)
        pending = list(ring.in_flight)
        assert [j for j, _ in ring.drain()] == pending and [s for _, s in []] == []
        assert ring.in_flight == []
    # two iterations in flight never share a slot
    ring = oracle.RingModel(4)
    for _ in range(4):
        ring.acquire()
    assert len({j % 4 for j in ring.in_flight}) == 4


def test_results_do_not_depend_on_k():
    """Abstract / Related Work: results are unchanged by the bound.  The ring only chooses
    where an iteration's receive region lives; replaying N iterations through ring models of
    different depth, with completion deferred as long as the ring allows, returns the same
    outputs in the same order."""
    w = synth.workload(3, "small")
    c = case_of(w)
    tabs = np_tables(w)
    N = 5
    batches = [tuple(x.numpy() for x in synth.make_batch(w, it)) for it in range(N)]
    direct = [oracle.embbag_plain(c, tabs, ix, off, want64=False)[1] for ix, off in batches]
    for k in (0, 1, 2, 4):
        ring = oracle.RingModel(k)
        slots = [None] * ring.K
        outs = []
        for it, (ix, off) in enumerate(batches):
            if len(ring.in_flight) == ring.K:
                j = ring.in_flight[0]
                outs.append(oracle.unpack(c, slots[ring.retire(j)]))
            j, slot = ring.acquire()
            r = oracle.pipeline(c, tabs, ix, off)
            slots[slot] = r["R"]
        for j, slot in ring.drain():
            outs.append(oracle.unpack(c, slots[slot]))
        assert len(outs) == N
        for a, b in zip(outs, direct):
            assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


# ----------------------------------------------------------------------------- generators

def test_generator_statistics_and_determinism():
    w = synth.workload(4, "small")
    a = synth.make_batch(w, 0)
    b = synth.make_batch(w, 0)
    c = synth.make_batch(w, 1)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1]) and not torch.equal(a[0][:100], c[0][:100])
    lens = np.diff(a[1].numpy())
    assert lens.min() == 1 and lens.max() == 64 and abs(lens.mean() - 32.5) < 0.5
    tab = synth.make_table(w, 3)
    assert tab.dtype == torch.float32 and abs(float(tab.std()) - 0.009) < 0.001
    assert float(tab.abs().max()) <= 510 * 2.0 ** -14
    assert torch.equal(synth.table_rows(w, 3, torch.tensor([0, 17, 99])), tab[[0, 17, 99]])
    w5 = synth.workload(5, "small")
    t5 = synth.make_table(w5, 0)
    assert t5.dtype == torch.float16 and torch.equal(t5.float(), synth.grid_rows(w5, 0, torch.arange(w5.rows[0])))
    # Zipf head: the most popular row takes the closed-form share 1 / H(rows, alpha)
    w3 = synth.workload(3, "small")
    ix, off = synth.make_batch(w3, 0)
    n0 = int(off[w3.B])
    top = np.bincount(ix[:n0].numpy(), minlength=w3.rows[0]).max() / n0
    share = 1.0 / np.sum(np.arange(1, w3.rows[0] + 1, dtype=np.float64) ** -1.05)
    assert abs(top - share) < 0.02
    full = synth.workload(4)
    assert sum(full.rows) == 79_079_336 and full.table_owner[:8] == [0] * 8 and set(full.table_owner[8:]) == set(range(1, 8))


# ----------------------------------------------------------------------------- weights, mean

def _weights_for(nnz, seed=5):
    rng = np.random.default_rng(seed)
    return rng.uniform(-2.0, 2.0, size=nnz).astype(np.float32)


@pytest.mark.parametrize("spec", TINY)
def test_weighted_and_mean_match_brute_force(spec):
    w = tiny_workload(spec, 9)
    ix, off = (x.numpy() for x in synth.make_batch(w, 0))
    tabs = np_tables(w)
    wts = _weights_for(len(ix))
    c = case_of(w)
    exp_w = np.zeros((w.B, w.T, w.D), np.float32)
    exp_m = np.zeros((w.B, w.T, w.D), np.float32)
    for t in range(w.T):
        for b in range(w.B):
            g = t * w.B + b
            for l in range(off[g], off[g + 1]):
                row = tabs[t][ix[l]].astype(np.float32)
                exp_w[b, t] = exp_w[b, t] + (np.float32(wts[l]) * row).astype(np.float32)
                exp_m[b, t] = exp_m[b, t] + row
            if off[g + 1] > off[g]:
                exp_m[b, t] = exp_m[b, t] / np.float32(off[g + 1] - off[g])
    _, o32w = oracle.embbag_plain(c, tabs, ix, off, want64=False, weights=wts)
    _, o32m = oracle.embbag_plain(c, tabs, ix, off, want64=False, mean=True)
    assert np.array_equal(o32w.view(np.uint32), exp_w.view(np.uint32))
    assert np.array_equal(o32m.view(np.uint32), exp_m.view(np.uint32))
    if w.part_kind == 0:      # table-wise: the staged path reproduces the definition bit for bit
        assert np.array_equal(oracle.pipeline(c, tabs, ix, off, weights=wts)["Out"].view(np.uint32), exp_w.view(np.uint32))
        assert np.array_equal(oracle.pipeline(c, tabs, ix, off, mean=True)["Out"].view(np.uint32), exp_m.view(np.uint32))


@pytest.mark.parametrize("cfg", [3, 4, 5])
def test_weighted_and_mean_against_torch(cfg):
    w = synth.workload(cfg, "small")
    w.values = "gauss" if cfg != 5 else w.values
    ix, off = synth.make_batch(w, 0)
    tabs_t = [synth.make_table(w, t, "cpu") for t in range(w.T)]
    tabs = [x.numpy() for x in tabs_t]
    wts = torch.from_numpy(_weights_for(ix.numel()))
    c = case_of(w)
    o64w, o32w = oracle.embbag_plain(c, tabs, ix.numpy(), off.numpy(), weights=wts.numpy())
    o64m, o32m = oracle.embbag_plain(c, tabs, ix.numpy(), off.numpy(), mean=True)
    out_w = oracle.pipeline(c, tabs, ix.numpy(), off.numpy(), weights=wts.numpy())
    out_m = oracle.pipeline(c, tabs, ix.numpy(), off.numpy(), mean=True)["Out"]
    mass = oracle.embbag_absmass(c, tabs, ix.numpy(), off.numpy())
    tol = 1e-3 if w.table_dtype == "fp16" else 1e-6
    lens = np.maximum(np.diff(off.numpy()), 1).reshape(w.T, w.B).T[:, :, None]
    for t in range(w.T):
        o = off[t * w.B:(t + 1) * w.B + 1]
        sub, sw = ix[o[0]:o[-1]], wts[o[0]:o[-1]]
        ref_w = torch.nn.functional.embedding_bag(sub, tabs_t[t].double(), o[:-1] - o[0], mode="sum",
                                                  per_sample_weights=sw.double()).numpy()
        ref_m = torch.nn.functional.embedding_bag(sub, tabs_t[t].double(), o[:-1] - o[0], mode="mean").numpy()
        assert np.allclose(o64w[:, t], ref_w, rtol=1e-12, atol=1e-300)
        assert np.allclose(o64m[:, t], ref_m, rtol=1e-12, atol=1e-300)
        for got in (o32w[:, t], out_w["Out"][:, t]):       # |w| <= 2: twice the mass bounds the terms
            assert np.all(np.abs(got - ref_w) <= 2 * 2 * tol * mass[:, t] + 1e-30)
        for got in (o32m[:, t], out_m[:, t]):
            assert np.all(np.abs(got - ref_m) <= 2 * tol * mass[:, t] / lens[:, t] + 1e-30)
    # the weight of every lookup travels with its row number
    P, T, B = w.P, w.T, w.B
    bag = np.repeat(np.arange(T * B), np.diff(off.numpy()))
    t_of, s_of = bag // B, (bag % B) // (B // P)
    d_of = ix.numpy() // (-(-np.array(w.rows)[t_of] // P)) if w.part_kind == 1 else np.array(w.table_owner)[t_of]
    order = np.argsort(d_of * P + s_of, kind="stable")
    assert np.array_equal(out_w["rweights"], wts.numpy()[order])


def test_weights_exact_cases():
    """Weights of one change nothing; power-of-two weights on integer tables stay exact."""
    w = synth.custom("ints", P=3, T=3, D=4, k=1, B=9, rows=[50, 60, 70], part_kind=1, bag=("uniform", 0, 9))
    ix, off = (x.numpy() for x in synth.make_batch(w, 1))
    c = case_of(w)
    tabs = [np.repeat(np.arange(r, dtype=np.float32)[:, None], 4, axis=1).copy() for r in w.rows]
    ones = np.ones(len(ix), np.float32)
    a = oracle.pipeline(c, tabs, ix, off)
    b = oracle.pipeline(c, tabs, ix, off, weights=ones)
    for k in ("Y", "S", "R", "Out"):
        assert np.array_equal(a[k].view(np.uint32), b[k].view(np.uint32))
    rng = np.random.default_rng(3)
    pw = (2.0 ** rng.integers(-3, 4, size=len(ix))).astype(np.float32) * rng.choice([-1, 1], size=len(ix)).astype(np.float32)
    out = oracle.pipeline(c, tabs, ix, off, weights=pw)["Out"]
    for t in range(3):
        for bb in range(9):
            g = t * 9 + bb
            sl = slice(off[g], off[g + 1])
            assert np.all(out[bb, t] == np.sum(pw[sl].astype(np.float64) * ix[sl]))
    m = oracle.pipeline(c, [np.ones((r, 4), np.float32) for r in w.rows], ix, off, mean=True)["Out"]
    lens = np.diff(off).reshape(3, 9).T
    assert np.array_equal(m[:, :, 0], (lens > 0).astype(np.float32))


# ----------------------------------------------------------------------------- row-quantised tables

def _rowq_table(D, rows):
    """Bytes of a row-quantised table written out by hand: rows = [(codes, scale, bias), ...]."""
    import struct
    stride = (D + 8 + 15) // 16 * 16
    buf = bytearray(stride * len(rows))
    for r, (codes, scale, bias) in enumerate(rows):
        assert len(codes) == D
        buf[r * stride:r * stride + D] = bytes(codes)
        buf[r * stride + D:r * stride + D + 8] = struct.pack("<ff", scale, bias)
    return np.frombuffer(bytes(buf), dtype=np.uint8).reshape(len(rows), stride).copy()


def test_rowq_worked_example():
    """Four rows written byte by byte, sums worked out by hand (all exact in fp32)."""
    D = 4
    tab = _rowq_table(D, [([0, 1, 2, 255], 0.5, -1.0),       # -1, -0.5, 0, 126.5
                          ([10, 20, 30, 40], 0.25, 3.0),     # 5.5, 8, 10.5, 13
                          ([1, 1, 1, 1], 2.0, 0.0),          # 2, 2, 2, 2
                          ([128, 64, 32, 16], 0.125, -16.0)])  # 0, -8, -12, -14
    assert tab.shape == (4, 16)
    case = oracle.Case(1, 1, D, 3, 0, [4], [0], 2)
    indices = np.array([0, 1, 3, 2, 2, 2], np.int64)         # bags: {0,1,3}, {}, {2,2,2}
    offsets = np.array([0, 3, 3, 6], np.int64)
    o64, o32 = oracle.embbag_plain(case, [tab], indices, offsets)
    want = np.array([[[4.5, -0.5, -1.5, 125.5]], [[0, 0, 0, 0]], [[6, 6, 6, 6]]])
    assert np.array_equal(o64, want) and np.array_equal(o32, want.astype(np.float32))
    # the whole path moves these vectors unchanged (P = 1: one owner, one requester)
    res = oracle.pipeline(case, [tab], indices, offsets)
    assert np.array_equal(res["Out"], want.astype(np.float32))


def test_rowq_stride_and_padding():
    """Row r starts r * stride bytes in, stride = D + 8 rounded up to 16; padding is ignored."""
    for D in (1, 7, 8, 9, 24, 40, 128):
        stride = oracle.rowq_stride(D)
        assert stride % 16 == 0 and D + 8 <= stride < D + 8 + 16 and stride == synth.rowq_stride(D)
        rng = np.random.default_rng(D)
        rows = [(list(rng.integers(0, 256, D)), float(2.0 ** -int(rng.integers(1, 6))), float(rng.integers(-8, 8)))
                for _ in range(5)]
        tab = _rowq_table(D, rows)
        junk = tab.copy()
        junk[:, D + 8:] = 0xA5                                # padding bytes must not matter
        case = oracle.Case(1, 1, D, 5, 0, [5], [0], 2)
        idx, off = np.arange(5, dtype=np.int64), np.arange(6, dtype=np.int64)
        a64, _ = oracle.embbag_plain(case, [tab], idx, off)
        b64, _ = oracle.embbag_plain(case, [junk], idx, off)
        want = np.array([[np.array(c, np.float64) * s + b] for c, s, b in rows])
        assert np.array_equal(a64, want) and np.array_equal(b64, want)


def test_rowq_decoding_rounds_twice_in_fp32():
    """value = fl32(fl32(code * scale) + bias): compared with numpy's float32 arithmetic, on
    rows where a single rounding (as a fused multiply-add would do) gives other bits."""
    D, n = 64, 400
    w = synth.custom("rowq", P=1, T=1, D=D, B=n, k=0, part_kind=0, rows=[n], table_dtype="u8rq", values="gauss", seed=41)
    tab = synth.make_table(w, 0).numpy()
    codes = tab[:, :D].astype(np.float32)
    scale = tab[:, D:D + 4].copy().view(np.float32)          # [n, 1]
    bias = tab[:, D + 4:D + 8].copy().view(np.float32)
    twice = (codes * scale).astype(np.float32) + bias         # numpy rounds each step to float32
    once = (codes.astype(np.float64) * scale.astype(np.float64) + bias.astype(np.float64)).astype(np.float32)
    assert twice.dtype == np.float32 and np.count_nonzero(twice != once) > 50
    case = oracle.Case(1, 1, D, n, 0, [n], [0], 2)
    idx, off = np.arange(n, dtype=np.int64), np.arange(n + 1, dtype=np.int64)
    o64, o32 = oracle.embbag_plain(case, [tab], idx, off)
    assert np.array_equal(o32[:, 0, :], twice) and np.array_equal(o64[:, 0, :], twice.astype(np.float64))


@pytest.mark.parametrize("part_kind", [0, 1])
def test_rowq_pipeline_against_decoded_fp32_tables(part_kind):
    """The path over a row-quantised table equals the path over the fp32 table of its decoded
    values (decoded here with numpy), step by step: only the element decoding differs."""
    w = synth.custom("rowq", P=3, T=4, D=24, B=10, k=1, part_kind=part_kind, rows=[30, 7, 19, 64],
                     table_dtype="u8rq", values="gauss", seed=43, bag=("uniform", 0, 6))
    tabs = np_tables(w)
    dec = []
    for tab in tabs:
        s = tab[:, w.D:w.D + 4].copy().view(np.float32)
        b = tab[:, w.D + 4:w.D + 8].copy().view(np.float32)
        dec.append(np.ascontiguousarray((tab[:, :w.D].astype(np.float32) * s).astype(np.float32) + b))
    ix, off = synth.make_batch(w, 0)
    ix, off = ix.numpy(), off.numpy()
    q = oracle.pipeline(case_of(w), tabs, ix, off)
    f = oracle.pipeline(oracle.Case(w.P, w.T, w.D, w.B, w.part_kind, w.rows, w.table_owner, 0), dec, ix, off)
    for key in ("Y", "S", "R", "Out", "ridx", "segoff"):
        assert np.array_equal(q[key], f[key]), key


def test_rowq_grid_tables_are_exact():
    """Grid-valued row-quantised tables: fp32 and fp64 bag sums agree bit for bit."""
    w = synth.custom("rowq", P=2, T=3, D=16, B=32, k=0, part_kind=1, rows=[50, 11, 200],
                     table_dtype="u8rq", values="grid", seed=47, bag=("uniform", 0, 40))
    tabs = np_tables(w)
    ix, off = synth.make_batch(w, 0)
    o64, o32 = oracle.embbag_plain(case_of(w), tabs, ix.numpy(), off.numpy())
    assert np.array_equal(o64, o32.astype(np.float64)) and np.abs(o64).max() > 1.0
    res = oracle.pipeline(case_of(w), tabs, ix.numpy(), off.numpy())
    assert np.array_equal(res["Out"], o32)


# ----------------------------------------------------------------------------- dense layers and interaction

def test_mlp_layer_brute_force_and_closed_forms():
    rng = np.random.default_rng(5)
    M, K, N = 4, 6, 3
    x = rng.normal(size=(M, K))
    W = rng.normal(size=(N, K)).astype(np.float32)
    b = rng.normal(size=N).astype(np.float32)
    for act in (0, 1, 2):
        y, _ = oracle.mlp_layer(x, W, b, act)
        for m in range(M):
            for n in range(N):
                v = float(b[n]) + sum(x[m, k] * float(W[n, k]) for k in range(K))
                want = v if act == 0 else max(v, 0.0) if act == 1 else 1.0 / (1.0 + np.exp(-v))
                assert abs(y[m, n] - want) <= 1e-14 * max(1.0, abs(want)), (act, m, n)
    # identity weights: the layer is act(x + b); a one-hot row of W picks a column of x
    eye = np.eye(K, dtype=np.float32)
    bb = np.arange(K, dtype=np.float32) - 2
    y, _ = oracle.mlp_layer(x, eye, bb, 1)
    assert np.array_equal(y, np.maximum(x + bb, 0.0))
    pick = np.zeros((2, K), np.float32)
    pick[0, 4], pick[1, 1] = 1.0, -2.0
    y, _ = oracle.mlp_layer(x, pick, None, 0)
    assert np.array_equal(y[:, 0], x[:, 4]) and np.array_equal(y[:, 1], -2.0 * x[:, 1])
    assert oracle.mlp_layer(np.zeros((3, K)), W, b, 2)[0][0, 0] == 1.0 / (1.0 + np.exp(-float(b[0])))


@pytest.mark.parametrize("act", [0, 1, 2])
def test_mlp_layer_against_torch_linear(act):
    rng = np.random.default_rng(6)
    M, K, N = 33, 29, 17
    x = rng.normal(size=(M, K))
    W = rng.normal(size=(N, K)).astype(np.float32)
    b = rng.normal(size=N).astype(np.float32)
    y, _ = oracle.mlp_layer(x, W, b, act)
    ref = torch.nn.functional.linear(torch.from_numpy(x), torch.from_numpy(W).double(), torch.from_numpy(b).double())
    ref = ref if act == 0 else torch.relu(ref) if act == 1 else torch.sigmoid(ref)
    assert np.allclose(y, ref.numpy(), rtol=1e-13, atol=1e-13)


def test_interact_brute_force_order_and_torch():
    rng = np.random.default_rng(7)
    B, T, D = 3, 5, 4
    x = rng.normal(size=(B, D))
    emb = rng.normal(size=(B, T, D)).astype(np.float32)
    z, _ = oracle.interact(x, emb)
    assert z.shape == (B, D + T * (T + 1) // 2)
    for b in range(B):
        Z = [x[b]] + [emb[b, t].astype(np.float64) for t in range(T)]
        want = list(x[b])
        for i in range(T + 1):
            for j in range(i):                                # i > j, ordered by i then j, no diagonal
                want.append(float(np.dot(Z[i], Z[j])))
        assert np.allclose(z[b], want, rtol=1e-14, atol=1e-14)
    # library route: batched Gram matrix and the strictly lower triangle in row-major order
    Zt = torch.cat([torch.from_numpy(x)[:, None, :], torch.from_numpy(emb).double()], dim=1)
    G = torch.bmm(Zt, Zt.transpose(1, 2))
    li, lj = torch.tril_indices(T + 1, T + 1, offset=-1)
    ref = torch.cat([torch.from_numpy(x), G[:, li, lj]], dim=1)
    assert np.allclose(z, ref.numpy(), rtol=1e-13, atol=1e-13)
    # every pair is told apart: Z_i = a_i * e_0 with a = 1 and distinct primes, so Z_i . Z_j = a_i a_j
    a = [1.0, 2.0, 3.0, 5.0, 7.0, 11.0, 13.0]
    Zc = np.zeros((len(a), 3))
    Zc[:, 0] = a
    zz, _ = oracle.interact(Zc[None, 0], Zc[None, 1:].astype(np.float32))
    want = [a[i] * a[j] for i in range(1, len(a)) for j in range(i)]
    assert len(set(want)) == len(want) and list(zz[0, 3:]) == want


def test_dense_error_bounds_hold_for_an_fp32_implementation():
    """The bound the GPU tests rely on: a plain fp32 evaluation (numpy, any summation order numpy
    picks) stays inside it, through a chain of layers and the interaction; and it is not vacuous."""
    w = synth.custom("dense", P=2, T=5, D=16, B=48, k=1, part_kind=0, rows=[10] * 5, seed=3)
    bot, top = synth.mlp_sizes(w, "small")
    Lb = [(W.numpy(), b.numpy(), 1) for W, b in synth.mlp_weights(w, bot, 0)]
    Lt = [(W.numpy(), b.numpy(), 1) for W, b in synth.mlp_weights(w, top, 1)]
    Lt[-1] = (Lt[-1][0], Lt[-1][1], 2)
    dense = synth.dense_features(w, 0).numpy()
    emb = np.random.default_rng(1).normal(0, 0.3, size=(w.B, w.T, w.D)).astype(np.float32)
    x, ex = oracle.mlp(dense, Lb)
    z, ez = oracle.interact(x, emb, ex)
    p, ep = oracle.mlp(z, Lt, ez)

    def f32_layer(a, W, b, act):
        v = (a.astype(np.float32) @ W.T.astype(np.float32) + b).astype(np.float32)
        return np.maximum(v, 0) if act == 1 else (1 / (1 + np.exp(-v))).astype(np.float32) if act == 2 else v
    a = dense
    for W, b, act in Lb:
        a = f32_layer(a, W, b, act)
    assert np.all(np.abs(a - x) <= ex) and ex.max() < 1e-4 * max(1.0, np.abs(x).max())
    Z = np.concatenate([a[:, None, :], emb], axis=1)
    G = np.einsum("bid,bjd->bij", Z, Z).astype(np.float32)
    li, lj = np.tril_indices(w.T + 1, -1)
    zf = np.concatenate([a, G[:, li, lj]], axis=1)
    assert np.all(np.abs(zf - z) <= ez)
    for W, b, act in Lt:
        zf = f32_layer(zf, W, b, act)
    assert np.all(np.abs(zf - p) <= ep) and ep.max() < 2e-3      # worst case carried through six layers
    # one layer on exact inputs: the bound is (K + 3) roundings on the sum of magnitudes, a few 1e-6
    y1, e1 = oracle.mlp_layer(z, Lt[0][0], Lt[0][1], 1)
    assert np.all(np.abs(f32_layer(z.astype(np.float32), *Lt[0]) - oracle.mlp_layer(z.astype(np.float32), Lt[0][0], Lt[0][1], 1)[0]) <= e1)
    assert e1.max() < 2e-5 * max(1.0, np.abs(y1).max())
    assert p.shape == (w.B, 1) and np.all((p > 0) & (p < 1)) and p.std() > 1e-3


# ----------------------------------------------------------------------------- E4M3 codes

def test_e4m3_decoder_all_codes():
    """All 256 codes against torch's float8_e4m3fn conversion and against the format's definition
    (sign, 4 exponent bits with bias 7, 3 mantissa bits, subnormals, NaN only at 0x7f / 0xff)."""
    got = oracle.e4m3_table()
    ref = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float32).numpy()
    nan = np.isnan(ref)
    assert list(np.flatnonzero(nan)) == [0x7F, 0xFF] and np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), ref[~nan].view(np.uint32))
    for v in range(256):
        e, m, sgn = (v >> 3) & 15, v & 7, -1.0 if v & 0x80 else 1.0
        if e == 15 and m == 7:
            continue
        want = sgn * (m * 2.0 ** -9 if e == 0 else (1 + m / 8) * 2.0 ** (e - 7))
        assert got[v] == want and np.signbit(got[v]) == bool(v & 0x80), v
    assert got[0x7E] == 448.0 and got[0x08] == 2.0 ** -6 and got[0x01] == 2.0 ** -9


def test_f8rq_worked_example_and_decoded_tables():
    """A row written by hand, and the path over an E4M3-coded table against the path over the fp32
    table of its decoded values (decoded here through torch's float8 type and numpy float32)."""
    D = 4
    tab = _rowq_table(D, [([0x38, 0x40, 0xB8, 0x01], 2.0, 1.0),      # codes 1, 2, -1, 2^-9 -> 3, 5, -1, 1 + 2^-8
                          ([0x30, 0x34, 0x00, 0x7E], 4.0, 0.0)])     # 0.5, 0.75, 0, 448 -> 2, 3, 0, 1792
    case = oracle.Case(1, 1, D, 2, 0, [2], [0], 3)
    o64, o32 = oracle.embbag_plain(case, [tab], np.array([0, 1, 1], np.int64), np.array([0, 1, 3], np.int64))
    want = np.array([[[3.0, 5.0, -1.0, 1.0 + 2.0 ** -8]], [[4.0, 6.0, 0.0, 3584.0]]])
    assert np.array_equal(o64, want) and np.array_equal(o32, want.astype(np.float32))

    w = synth.custom("f8", P=3, T=3, D=24, B=11, k=1, part_kind=1, rows=[30, 7, 64],
                     table_dtype="f8rq", values="gauss", seed=59, bag=("uniform", 0, 6))
    tabs = np_tables(w)
    dec = []
    for t in tabs:
        codes = torch.from_numpy(t[:, :w.D].copy()).view(torch.float8_e4m3fn).to(torch.float32).numpy()
        assert np.all(np.isfinite(codes))
        s = t[:, w.D:w.D + 4].copy().view(np.float32)
        b = t[:, w.D + 4:w.D + 8].copy().view(np.float32)
        dec.append(np.ascontiguousarray((codes * s).astype(np.float32) + b))
    ix, off = synth.make_batch(w, 0)
    q = oracle.pipeline(case_of(w), tabs, ix.numpy(), off.numpy())
    f = oracle.pipeline(oracle.Case(w.P, w.T, w.D, w.B, w.part_kind, w.rows, w.table_owner, 0), dec, ix.numpy(), off.numpy())
    for key in ("Y", "S", "R", "Out"):
        assert np.array_equal(q[key], f[key]), key
    # grid tables are exact
    wg = synth.custom("f8", P=2, T=2, D=16, B=20, k=0, part_kind=0, rows=[50, 200], table_dtype="f8rq", values="grid",
                      seed=61, bag=("uniform", 0, 40))
    tg = np_tables(wg)
    ix, off = synth.make_batch(wg, 0)
    o64, o32 = oracle.embbag_plain(case_of(wg), tg, ix.numpy(), off.numpy())
    assert np.array_equal(o64, o32.astype(np.float64)) and np.abs(o64).max() > 0.1


# ----------------------------------------------------------------------------- single-bag sum and the tolerance scale

def _ordered_fp32_sum(rows):
    """One fp32 accumulator from +0, rows added in order: spelled out with numpy scalars."""
    acc = np.zeros(rows.shape[1], np.float32)
    for r in rows:
        acc = (acc + r.astype(np.float32)).astype(np.float32)
    return acc


@pytest.mark.parametrize("n", [0, 1, 2, 70])
def test_bag_sum_is_the_ordered_fp32_sum(n):
    """orc_bag_sum stands in for the whole-table oracle at sizes the host cannot hold (Listing 1,
    apply_emb on one bag): bit for bit an ordered numpy fp32 loop, bit for bit orc_embbag_plain on
    the same rows, float64 output = numpy's float64 sum; Gaussian values, so that a reordered,
    pairwise or double-accumulated sum would show in the last bit."""
    rng = np.random.default_rng(40 + n)
    D = 12
    rows = (rng.normal(0.0, 0.01, size=(n, D)) * rng.choice([1.0, 64.0, 1 / 64.0], size=(n, 1))).astype(np.float32)
    o32, o64 = oracle.bag_sum(rows)
    want = _ordered_fp32_sum(rows)
    assert np.array_equal(o32.view(np.uint32), want.view(np.uint32))
    assert np.allclose(o64, rows.astype(np.float64).sum(axis=0), rtol=1e-15, atol=1e-300)
    if n == 0:
        assert not o32.any() and not np.signbit(o32).any() and not o64.any()
    else:
        mini = oracle.Case(1, 1, D, 1, 0, [n], [0], 0)
        p64, p32 = oracle.embbag_plain(mini, [rows], np.arange(n), np.array([0, n]))
        assert np.array_equal(p32.reshape(D).view(np.uint32), o32.view(np.uint32))
        assert np.array_equal(p64.reshape(D), o64)
    if n == 70:                                     # the values are order-sensitive: another order gives other bits
        assert not np.array_equal(_ordered_fp32_sum(rows[::-1]).view(np.uint32), want.view(np.uint32))
        assert not np.array_equal(o64.astype(np.float32).view(np.uint32), want.view(np.uint32))
    # column c of the result depends on column c of the rows only, and on every row
    if n >= 2:
        probe = rows.copy()
        probe[n // 2, 3] += np.float32(1.0)
        q32, _ = oracle.bag_sum(probe)
        changed = q32.view(np.uint32) != o32.view(np.uint32)
        assert changed[3] and not np.delete(changed, 3).any()


def test_bag_sum_signed_zero_and_exact_cases():
    """A bag of -0.0 rows gives +0.0 (the accumulator starts at +0); powers of two add exactly;
    a large term followed by small ones loses them in fp32 but not in float64."""
    z = np.full((3, 2), -0.0, np.float32)
    o32, o64 = oracle.bag_sum(z)
    assert not np.signbit(o32).any() and not o32.any()
    rows = np.array([[2.0 ** -3], [2.0 ** -5], [2.0 ** 4]], np.float32)
    o32, o64 = oracle.bag_sum(rows)
    assert o32[0] == 16.15625 and o64[0] == 16.15625
    rows = np.array([[1.0]] + [[2.0 ** -25]] * 8, np.float32)
    o32, o64 = oracle.bag_sum(rows)
    assert o32[0] == 1.0 and o64[0] == 1.0 + 8 * 2.0 ** -25           # in order: every small term is rounded away
    o32r, _ = oracle.bag_sum(rows[::-1].copy())
    assert o32r[0] == np.float32(1.0 + 2.0 ** -22)                    # small terms first: they survive


@pytest.mark.parametrize("spec", TINY)
@pytest.mark.parametrize("dtype", ["fp32", "fp16"])
def test_absmass_is_the_sum_of_magnitudes(spec, dtype):
    """orc_embbag_absmass scales every tolerance assertion (|x - exact| <= tol * sum |terms|): it must
    EQUAL numpy's float64 sum of |row| over exactly the bag's lookups - a mass summed over a wider
    range, or over the wrong table or column, would make every such assertion pass too easily."""
    w = synth.custom("tiny", k=1, values="gauss", seed=17, table_dtype=dtype, **spec)
    ix, off = (x.numpy() for x in synth.make_batch(w, 0))
    tabs = np_tables(w)
    mass = oracle.embbag_absmass(case_of(w), tabs, ix, off)
    assert mass.shape == (w.B, w.T, w.D) and mass.dtype == np.float64
    for t in range(w.T):
        for b in range(w.B):
            g = t * w.B + b
            rows = tabs[t][ix[off[g]:off[g + 1]]].astype(np.float64).reshape(-1, w.D)
            want = np.abs(rows).sum(axis=0)
            assert np.allclose(mass[b, t], want, rtol=1e-15, atol=0.0), (t, b)
            if off[g + 1] == off[g]:
                assert not mass[b, t].any()
    # duplicates count as often as they occur; signs do not cancel
    c1 = oracle.Case(1, 1, 2, 2, 0, [3], [0], 0)
    tab = np.array([[1.0, -2.0], [-4.0, 8.0], [0.5, 0.25]], np.float32)
    m = oracle.embbag_absmass(c1, [tab], np.array([0, 1, 1, 2]), np.array([0, 3, 4]))
    assert np.array_equal(m, np.array([[[9.0, 18.0]], [[0.5, 0.25]]]))
    o64, _ = oracle.embbag_plain(c1, [tab], np.array([0, 1, 1, 2]), np.array([0, 3, 4]))
    assert np.array_equal(o64, np.array([[[-7.0, 14.0]], [[0.5, 0.25]]]))


def test_absmass_bounds_the_plain_sums_tightly():
    """|sum| <= mass with equality for one-signed bags; and mass is no more than that: for bags of
    non-negative values mass == the float64 sum itself."""
    w = synth.custom("pos", P=2, T=2, D=4, k=1, B=6, rows=[9, 5], part_kind=0, bag=("uniform", 0, 7), seed=3)
    ix, off = (x.numpy() for x in synth.make_batch(w, 2))
    rng = np.random.default_rng(8)
    tabs = [np.abs(rng.normal(0, 1, size=(r, 4))).astype(np.float32) for r in w.rows]
    c = case_of(w)
    o64, _ = oracle.embbag_plain(c, tabs, ix, off)
    assert np.array_equal(oracle.embbag_absmass(c, tabs, ix, off), o64)
    neg = [-t for t in tabs]
    o64n, _ = oracle.embbag_plain(c, neg, ix, off)
    assert np.array_equal(oracle.embbag_absmass(c, neg, ix, off), -o64n)
