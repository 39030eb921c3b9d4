"""Parity of the HIP path against the CPU oracle, element by element, through the C ABI.

Integer outputs (counts, displacements, ridx, segoff, perm) and every fp32 buffer (pooled,
send, receive slot, output) must equal the oracle's bit for bit: both sides add a segment's
rows in segment order from +0 and, for row-wise partitions, the P partial vectors in
increasing owner rank.  Against the plain float64 definition the bound is
|x - exact| <= tol * sum|terms| with tol = 1e-6 for fp32 tables and 1e-3 for fp16 storage; row-quantised 8-bit tables decode to
fp32 numbers (the same two roundings on both sides) and are held to the fp32 bound.
"""
import numpy as np
import pytest
import torch

import oracle
import synth

pytestmark = pytest.mark.gpu

TOL = {"fp32": 1e-6, "fp16": 1e-3, "u8rq": 1e-6, "f8rq": 1e-6}


def case_of(w):
    return oracle.Case(w.P, w.T, w.D, w.B, w.part_kind, w.rows, w.table_owner, w.dtype_code)


def bits(a):
    a = np.ascontiguousarray(a)
    return a.view(np.uint32) if a.dtype == np.float32 else a


def run_gpu(w, tabs_cpu, batches, want_perm=True, tuning=None, plan_scan=None):
    from paper_2512_19342_amd.runner import Pipeline
    dev = torch.device("cuda:0")
    tabs = [t.to(dev) for t in tabs_cpu]
    max_nnz = max(int(off[-1]) for _, off in batches)
    pipe = Pipeline(w, tabs, max_nnz, want_perm=want_perm)
    if tuning:
        pipe.ctx.bls_set_pool_tuning(**tuning)
    if plan_scan is not None:
        pipe.ctx.bls_set_plan_tuning(plan_scan)
    res = []
    for ix, off in batches:
        nnz = int(off[-1])
        out = pipe.new_out()
        it, slot = pipe.issue(ix.to(dev), off.to(dev), nnz)
        r = dict(sendcounts=pipe.sendcounts.cpu().numpy(), sdispls=pipe.sdispls.cpu().numpy(),
                 recvcounts=pipe.recvcounts.cpu().numpy(), rdispls=pipe.rdispls.cpu().numpy(),
                 ridx=pipe.ridx[:nnz].cpu().numpy(), segoff=pipe.segoff.cpu().numpy(),
                 perm=pipe.perm[:nnz].cpu().numpy() if want_perm else None,
                 Y=pipe.pooled.cpu().numpy(), S=pipe.send.cpu().numpy(), R=pipe.slot_view(slot).cpu().numpy())
        pipe.complete(it, out)
        pipe.ctx.bls_check()
        r["Out"] = out.cpu().numpy()
        res.append(r)
    return res, pipe


def check_against_oracle(w, tabs_cpu, batches, got):
    c = case_of(w)
    tabs_np = [t.numpy() for t in tabs_cpu]
    for (ix, off), g in zip(batches, got):
        ref = oracle.pipeline(c, tabs_np, ix.numpy(), off.numpy())
        for k in ("sendcounts", "sdispls", "recvcounts", "rdispls", "ridx", "segoff", "perm"):
            assert np.array_equal(g[k], ref[k]), k
        for k in ("Y", "S", "R", "Out"):
            assert np.array_equal(bits(g[k]), bits(ref[k])), k
        o64, _ = oracle.embbag_plain(c, tabs_np, ix.numpy(), off.numpy(), want32=False)
        mass = oracle.embbag_absmass(c, tabs_np, ix.numpy(), off.numpy())
        assert np.all(np.abs(g["Out"].astype(np.float64) - o64) <= TOL[w.table_dtype] * mass)


WORKLOADS = [(1, "full"), (2, "full"), (3, "small"), (4, "small"), (5, "small"), (6, "small")]


@pytest.mark.parametrize("cfg,size", WORKLOADS)
def test_benchmark_workloads_match_oracle(cfg, size):
    w = synth.workload(cfg, size)
    tabs = [synth.make_table(w, t) for t in range(w.T)]
    batches = [synth.make_batch(w, it) for it in range(2)]
    got, _ = run_gpu(w, tabs, batches)
    check_against_oracle(w, tabs, batches, got)


def test_order_sensitive_values_rowwise_and_tablewise():
    """Gaussian values make every reassociation visible in the last bit."""
    for cfg in (3, 4):
        w = synth.workload(cfg, "small")
        w.values = "gauss"
        tabs = [synth.make_table(w, t) for t in range(w.T)]
        batches = [synth.make_batch(w, 7)]
        got, _ = run_gpu(w, tabs, batches)
        check_against_oracle(w, tabs, batches, got)


EDGE = [
    dict(P=1, T=2, D=4, B=3, part_kind=0, rows=[5, 6], bag=("fixed", 2)),
    dict(P=2, T=3, D=4, B=4, part_kind=0, rows=[7, 5, 9], bag=("uniform", 0, 3)),            # empty bags
    dict(P=3, T=4, D=8, B=7, part_kind=0, rows=[11, 3, 8, 20], bag=("uniform", 0, 4)),       # P does not divide B
    dict(P=3, T=2, D=8, B=5, part_kind=1, rows=[10, 4], bag=("uniform", 0, 6)),              # ragged last shard
    dict(P=4, T=3, D=4, B=8, part_kind=1, rows=[3, 17, 1], bag=("uniform", 1, 5)),           # empty shards
    dict(P=3, T=5, D=7, B=50, part_kind=0, rows=[100, 30, 77, 5, 64], bag=("uniform", 0, 9)),   # odd D: scalar paths
    dict(P=4, T=3, D=5, B=33, part_kind=1, rows=[101, 64, 9], bag=("uniform", 0, 70)),       # odd D, bags > 64
    dict(P=2, T=3, D=24, B=70, part_kind=0, rows=[300, 200, 100], bag=("uniform", 0, 150)),  # 6 of 8 lanes, long bags
    dict(P=2, T=2, D=320, B=40, part_kind=1, rows=[500, 333], bag=("uniform", 0, 20)),       # rows > 1 KB
    dict(P=8, T=2, D=128, B=300, part_kind=1, rows=[4097, 1000], bag=("uniform", 0, 200)),   # long bags over 8 owners
    dict(P=64, T=2, D=8, B=130, part_kind=1, rows=[5000, 129], bag=("uniform", 0, 90)),      # maximum P
    dict(P=5, T=7, D=64, B=5000, part_kind=0, rows=[1000] * 7, bag=("uniform", 0, 3)),       # several scan tiles, one workgroup
    dict(P=4, T=16, D=8, B=2000, part_kind=1, rows=[300] * 16, bag=("uniform", 0, 3)),       # 32 scan tiles: multi-block scan
    dict(P=3, T=40, D=4, B=3001, part_kind=0, rows=[64] * 40, bag=("uniform", 0, 2)),        # 30 scan tiles, table-wise
    dict(P=16, T=200, D=4, B=64, part_kind=1, rows=[50] * 200, bag=("uniform", 0, 3)),       # 51200 tile counts: multi-block scan
    dict(P=3, T=2, D=4, B=600, part_kind=1, rows=[5000, 77], bag=("uniform", 0, 200)),       # tiles of several chunks, several tiles per run
    dict(P=2, T=1, D=4, B=128, part_kind=1, rows=[1000], bag=("fixed", 64)),                 # tiles of exactly one full chunk
    dict(P=9, T=3, D=4, B=400, part_kind=1, rows=[900, 10, 4000], bag=("uniform", 0, 30)),   # more than eight owners: two ranking passes
    dict(P=8, T=300, D=4, B=64, part_kind=1, rows=[40] * 300, bag=("uniform", 0, 3)),        # 19200 tile counts over eight owners: too many for every workgroup to add up
]


@pytest.mark.parametrize("spec", EDGE)
@pytest.mark.parametrize("dtype", ["fp32", "fp16", "u8rq"])
def test_edge_shapes(spec, dtype):
    w = synth.custom("edge", k=1, values="gauss", table_dtype=dtype, seed=23,
                     index_dist=("zipf", 1.1), **spec)
    tabs = [synth.make_table(w, t) for t in range(w.T)]
    batches = [synth.make_batch(w, it) for it in range(2)]
    got, _ = run_gpu(w, tabs, batches)
    check_against_oracle(w, tabs, batches, got)


ROWQ = [
    dict(P=2, T=3, D=16, B=90, part_kind=0, rows=[300, 17, 1000], bag=("uniform", 0, 40)),    # one lane per row
    dict(P=3, T=2, D=32, B=100, part_kind=1, rows=[4000, 50], bag=("uniform", 0, 30)),        # two lanes
    dict(P=4, T=4, D=64, B=257, part_kind=0, rows=[5000, 64, 900, 33], bag=("uniform", 0, 60)),   # four lanes, streams
    dict(P=8, T=3, D=128, B=1000, part_kind=1, rows=[20000, 3000, 129], bag=("uniform", 1, 64)),  # the benchmark's row
    dict(P=2, T=2, D=20, B=64, part_kind=0, rows=[100, 200], bag=("uniform", 0, 12)),         # 4 bytes per lane, 5 of 8 lanes
    dict(P=2, T=2, D=1024, B=24, part_kind=1, rows=[300, 77], bag=("uniform", 0, 9)),         # a whole wavefront per row
    dict(P=2, T=2, D=2048, B=12, part_kind=0, rows=[50, 60], bag=("uniform", 0, 5)),          # longer than 64 lanes cover
]


@pytest.mark.parametrize("spec", ROWQ, ids=lambda s: f"D{s['D']}-P{s['P']}-part{s['part_kind']}")
@pytest.mark.parametrize("values", ["gauss", "grid"])
@pytest.mark.parametrize("storage", ["u8rq", "f8rq"])
def test_row_quantised_tables(spec, values, storage):
    """8-bit codes (integers or E4M3 floats) with a scale and a bias per row: decoding (two fp32
    roundings) and the ordered sum must give the oracle's bits for every row length the kernels
    treat differently."""
    w = synth.custom("rowq", k=2, values=values, table_dtype=storage, seed=37, index_dist=("zipf", 1.05), **spec)
    tabs = [synth.make_table(w, t) for t in range(w.T)]
    batches = [synth.make_batch(w, it) for it in range(2)]
    got, _ = run_gpu(w, tabs, batches)
    check_against_oracle(w, tabs, batches, got)
    if values == "grid":                                      # exact values: fp64 definition, bit for bit
        o64, _ = oracle.embbag_plain(case_of(w), [t.numpy() for t in tabs], batches[0][0].numpy(),
                                     batches[0][1].numpy(), want32=False)
        assert np.array_equal(got[0]["Out"].astype(np.float64), o64)


def test_e4m3_codes_all_values_on_the_device():
    """Every finite E4M3 code through the pooling kernel with scale 1 and bias 0 (bags of one row):
    the hardware conversion must agree with the oracle's decoder, subnormals and signed zeros included."""
    D = 256
    codes = np.arange(256, dtype=np.uint8)
    codes[[0x7F, 0xFF]] = [0x7E, 0xFE]                          # the two NaN patterns are left out
    stride = synth.rowq_stride(D)
    tab = np.zeros((3, stride), np.uint8)
    for r, perm in enumerate((codes, codes[::-1], np.roll(codes, 37))):
        tab[r, :D] = perm
        tab[r, D:D + 8] = np.array([1.0, 0.0], np.float32).view(np.uint8)
    w = synth.custom("codes", P=1, T=1, D=D, B=3, k=1, part_kind=0, rows=[3], table_dtype="f8rq", bag=("fixed", 1))
    ix, off = torch.tensor([0, 1, 2]), torch.tensor([0, 1, 2, 3])
    got, _ = run_gpu(w, [torch.from_numpy(tab)], [(ix, off)])
    ref = oracle.pipeline(case_of(w), [tab], ix.numpy(), off.numpy())
    assert np.array_equal(bits(got[0]["Out"]), bits(ref["Out"]))
    want = oracle.e4m3_table()[codes] + np.float32(0.0)         # the sum starts from +0: -0 becomes +0
    assert np.array_equal(got[0]["Out"][0, 0].view(np.uint32), want.view(np.uint32))


def test_rowwise_plan_chunk_edges():
    """Hand-made offsets for the row-wise placement: a tile whose lookups fill a chunk exactly and whose
    remaining bags are empty (they start where the chunk ends), a bag longer than two chunks, empty bags
    in front, and a run without any lookup."""
    P, T, B, D = 2, 2, 64, 4
    lens = np.zeros((T, B), np.int64)
    lens[0, 0] = 2048                                        # run (0, 0): one full chunk, then 31 empty bags
    lens[0, 40] = 4096 + 5                                   # run (0, 1): empty bags, a long bag, empty bags
    lens[1, 3], lens[1, 31] = 2047, 1                        # run (1, 0): ends one short of a chunk, then a single lookup
    # exact-grid values: a bag of 4101 lookups summed in fp32 is then still exact, as the 1e-6 bound needs
    w = synth.custom("chunks", P=P, T=T, D=D, B=B, k=1, part_kind=1, rows=[777, 10], values="grid", bag=("fixed", 0))
    off = np.concatenate([[0], np.cumsum(lens.reshape(-1))])
    rng = np.random.default_rng(5)
    ix = np.concatenate([rng.integers(0, w.rows[t], int(lens[t].sum())) for t in range(T)])
    tabs = [synth.make_table(w, t) for t in range(T)]
    batches = [(torch.from_numpy(ix), torch.from_numpy(off))]
    got, _ = run_gpu(w, tabs, batches)
    check_against_oracle(w, tabs, batches, got)


ROWWISE_EDGE = [spec for spec in EDGE if spec["part_kind"] == 1]


@pytest.mark.parametrize("spec", ROWWISE_EDGE, ids=lambda s: f"P{s['P']}-T{s['T']}-B{s['B']}")
@pytest.mark.parametrize("want_perm", [True, False])
def test_rowwise_plan_in_three_launches(spec, want_perm):
    """bls_plan leaves the scan to the placing workgroups for a row-wise partition where it can (the
    default, which every other test runs); the three-launch form (count, scan, place) must give the
    same plan."""
    w = synth.custom("edge3", k=1, values="grid", seed=29, index_dist=("zipf", 1.1), **spec)
    tabs = [synth.make_table(w, t) for t in range(w.T)]
    batches = [synth.make_batch(w, it) for it in range(2)]
    got, _ = run_gpu(w, tabs, batches, want_perm=want_perm, plan_scan=0)
    c = case_of(w)
    tabs_np = [t.numpy() for t in tabs]
    for (ix, off), g in zip(batches, got):
        ref = oracle.pipeline(c, tabs_np, ix.numpy(), off.numpy())
        for k in ("sendcounts", "sdispls", "recvcounts", "rdispls", "ridx", "segoff") + (("perm",) if want_perm else ()):
            assert np.array_equal(g[k], ref[k]), k
        assert np.array_equal(bits(g["Out"]), bits(ref["Out"]))


TABLEWISE_EDGE = [spec for spec in EDGE if spec["part_kind"] == 0]


@pytest.mark.parametrize("spec", TABLEWISE_EDGE, ids=lambda s: f"P{s['P']}-T{s['T']}-B{s['B']}")
def test_tablewise_plan_in_three_launches(spec):
    """bls_plan takes one launch for a small table-wise batch (up to 2048 runs and 2^22 lookups: the default,
    which every other test here runs); the three-launch form (count, scan, place) must give the same plan."""
    w = synth.custom("edge3t", k=1, values="grid", seed=31, index_dist=("zipf", 1.1), **spec)
    tabs = [synth.make_table(w, t) for t in range(w.T)]
    batches = [synth.make_batch(w, it) for it in range(2)]
    got, _ = run_gpu(w, tabs, batches, plan_scan=0)
    check_against_oracle(w, tabs, batches, got)


def test_tablewise_plan_with_more_runs_than_one_launch_takes():
    """P * Q = 2112 runs: beyond what the one-launch form scans in LDS, so the three launches serve."""
    w = synth.custom("manyruns", P=64, T=33, D=4, B=128, k=1, part_kind=0, rows=[50 + 3 * t for t in range(33)],
                     values="grid", bag=("uniform", 0, 4), seed=41)
    tabs = [synth.make_table(w, t) for t in range(w.T)]
    batches = [synth.make_batch(w, it) for it in range(2)]
    got, _ = run_gpu(w, tabs, batches)
    check_against_oracle(w, tabs, batches, got)


@pytest.mark.parametrize("cfg", [3, 4, 5, 6])
@pytest.mark.parametrize("scan_while_placing", [0, 1])
def test_workloads_in_either_plan_form(cfg, scan_while_placing):
    w = synth.workload(cfg, "small")
    tabs = [synth.make_table(w, t) for t in range(w.T)]
    batches = [synth.make_batch(w, it) for it in range(3)]
    got, _ = run_gpu(w, tabs, batches, plan_scan=scan_while_placing)
    check_against_oracle(w, tabs, batches, got)


def test_all_bags_empty():
    w = synth.custom("empty", P=2, T=3, D=8, k=1, B=6, rows=[4, 5, 6], part_kind=1, bag=("fixed", 0))
    tabs = [synth.make_table(w, t) for t in range(w.T)]
    batches = [synth.make_batch(w, 0)]
    assert int(batches[0][1][-1]) == 0
    got, _ = run_gpu(w, tabs, batches)
    check_against_oracle(w, tabs, batches, got)
    assert not got[0]["Out"].any() and not np.signbit(got[0]["Out"]).any()


@pytest.mark.parametrize("k", [0, 1, 2, 4])
@pytest.mark.parametrize("cfg", [3, 4])
def test_ring_deferred_completion(k, cfg):
    """Completion deferred as long as the ring allows, on a second stream; every iteration
    must still come out right (a slot overwritten too early would show) and in FIFO order."""
    import paper_2512_19342_amd as B
    from paper_2512_19342_amd.runner import Pipeline
    w = synth.workload(cfg, "small")
    w.k = k
    dev = torch.device("cuda:0")
    tabs_cpu = [synth.make_table(w, t) for t in range(w.T)]
    tabs = [t.to(dev) for t in tabs_cpu]
    N = 7
    batches = [synth.make_batch(w, it) for it in range(N)]
    pipe = Pipeline(w, tabs, max(int(o[-1]) for _, o in batches))
    c = case_of(w)
    tabs_np = [t.numpy() for t in tabs_cpu]
    model = oracle.RingModel(k)
    side = torch.cuda.Stream()
    outs, pending = {}, []
    for it, (ix, off) in enumerate(batches):
        if len(model.in_flight) == model.K:
            with pytest.raises(B.BlsError) as e:
                pipe.ctx.bls_ring_advance()
            assert e.value.code == B.BLS_ERING_FULL
            if model.K > 1:
                with pytest.raises(B.BlsError) as e:
                    pipe.complete(pending[1], pipe.new_out())
                assert e.value.code == B.BLS_EORDER
            j = pending.pop(0)
            model.retire(j)
            outs[j] = pipe.new_out()
            pipe.complete(j, outs[j], side)
        j, slot = pipe.issue(ix.to(dev), off.to(dev), int(off[-1]))
        assert (j, slot) == model.acquire()
        pending.append(j)
    for j, _ in model.drain():
        assert pending.pop(0) == j
        outs[j] = pipe.new_out()
        pipe.complete(j, outs[j], side)
    with pytest.raises(B.BlsError) as e:
        pipe.complete(N, pipe.new_out())
    assert e.value.code == B.BLS_ERING_EMPTY
    torch.cuda.synchronize()
    pipe.ctx.bls_check()
    for it, (ix, off) in enumerate(batches):
        ref = oracle.pipeline(c, tabs_np, ix.numpy(), off.numpy())["Out"]
        assert np.array_equal(bits(outs[it].cpu().numpy()), bits(ref)), (k, it)


def test_bad_inputs_are_flagged_not_faulted():
    import paper_2512_19342_amd as B
    from paper_2512_19342_amd.runner import Pipeline
    for cfg in (3, 4):
        w = synth.workload(cfg, "small")
        dev = torch.device("cuda:0")
        tabs = [synth.make_table(w, t).to(dev) for t in range(w.T)]
        ix, off = synth.make_batch(w, 0)
        nnz = int(off[-1])
        pipe = Pipeline(w, tabs, nnz)
        for how in ("index_high", "index_negative", "offsets_decrease", "offsets_past_end"):
            bix, boff = ix.clone(), off.clone()
            if how == "index_high":
                bix[nnz // 2] = w.rows[0] + 10 ** 12
            elif how == "index_negative":
                bix[5] = -3
            elif how == "offsets_decrease":
                boff[10] = boff[12] + 5
            else:
                boff[-1] = nnz + 1000
            bad_out = pipe.new_out()
            pipe.step(bix.to(dev), boff.to(dev), nnz, bad_out)
            with pytest.raises(B.BlsError) as e:
                pipe.ctx.bls_check()
            assert e.value.code == B.BLS_ERANGE, how
            if how.startswith("index"):
                # the bad lookup adds nothing to its bag: the output is that of the batch without it
                at = nnz // 2 if how == "index_high" else 5
                gix = np.delete(ix.numpy(), at)
                goff = off.numpy().copy()
                goff[goff > at] -= 1
                want = oracle.pipeline(case_of(w), [t.cpu().numpy() for t in tabs], gix, goff)["Out"]
                assert np.array_equal(bits(bad_out.cpu().numpy()), bits(want)), (cfg, how)
        # and the context still works afterwards
        out = pipe.new_out()
        pipe.step(ix.to(dev), off.to(dev), nnz, out)
        pipe.ctx.bls_check()
        c = case_of(w)
        ref = oracle.pipeline(c, [t.cpu().numpy() for t in tabs], ix.numpy(), off.numpy())["Out"]
        assert np.array_equal(bits(out.cpu().numpy()), bits(ref))


def test_host_side_argument_errors():
    import paper_2512_19342_amd as B
    with pytest.raises(B.BlsError):
        B.Context(0, 1, 4, 1, 4, [5], [0])
    with pytest.raises(B.BlsError):
        B.Context(2, 1, 4, 1, 1, [5], [0])               # B < P
    with pytest.raises(B.BlsError):
        B.Context(2, 1, 4, 1, 4, [5], [2])               # owner out of range
    c = B.Context(2, 2, 4, 1, 4, [5, 6], [0, 1])
    t0 = torch.zeros(5, 4, device="cuda")
    with pytest.raises(B.BlsError):
        c.bls_set_shard(0, 1, t0)                         # wrong owner
    with pytest.raises(B.BlsError):
        c.bls_set_shard(1, 1, t0)                         # wrong row count
    c.bls_set_shard(0, 0, t0)
    z = torch.zeros(64, dtype=torch.int64, device="cuda")
    y = torch.zeros(64, device="cuda")
    with pytest.raises(B.BlsError) as e:                  # shard of table 1 never set
        c.bls_embbag_pool(z, z, 0, y)
    assert e.value.code == B.BLS_EINVAL
    c.bls_set_shard(1, 1, torch.zeros(6, 4, device="cuda"))
    with pytest.raises(B.BlsError) as e:                  # every shard set, but the tables are not on the device yet
        c.bls_embbag_pool(z, z, 0, y)
    assert e.value.code == B.BLS_EINVAL and "bls_commit" in c.bls_last_error()
    with pytest.raises(B.BlsError) as e:
        c.bls_commit(torch.zeros(8, dtype=torch.uint8, device="cuda"))
    assert e.value.code == B.BLS_ENOSPC
    desc = torch.empty(c.bls_desc_bytes(), dtype=torch.uint8, device="cuda")
    c.bls_commit(desc)
    c.bls_embbag_pool(z, z, 0, y)
    c.bls_set_shard(1, 1, torch.zeros(6, 4, device="cuda"))   # a shard replaced: commit again
    with pytest.raises(B.BlsError) as e:
        c.bls_embbag_pool(z, z, 0, y)
    assert e.value.code == B.BLS_EINVAL
    c.bls_commit(desc)
    c.bls_embbag_pool(z, z, 0, y)
    c.bls_check()
    with pytest.raises(B.BlsError) as e:
        c.bls_set_ring(torch.zeros(3, device="cuda"))
    assert e.value.code == B.BLS_ENOSPC
    with pytest.raises(B.BlsError) as e:
        c.bls_alltoallv_local(y, 0)                       # no ring yet
    assert e.value.code == B.BLS_EINVAL


@pytest.mark.parametrize("vb,nb,xcd", [(16, 1, 0), (16, 3, 1), (16, 16, 0), (8, 0, 1), (8, 7, 0), (4, 0, 0), (4, 2, 1)])
def test_pool_launch_variants(vb, nb, xcd):
    """bls_set_pool_tuning picks other lane widths, segments per group, grid mappings and row-position
    widths; every variant must give the same bits."""
    tuning = dict(lane_bytes=vb, segments_per_group=nb, xcd_map=xcd, wide_positions=1 - xcd)
    works = [synth.workload(c, "small") for c in (3, 4, 5)]
    for w in works[:2]:
        w.values = "gauss"
    works.append(synth.custom("long", P=3, T=4, D=64, k=1, B=100, rows=[500, 40, 7, 1000], part_kind=0,
                              bag=("uniform", 0, 150), values="gauss", index_dist=("zipf", 1.1)))
    works.append(synth.custom("sparse", P=4, T=3, D=32, k=1, B=203, rows=[50, 3000, 9], part_kind=1,
                              bag=("uniform", 0, 2), values="gauss", table_dtype="fp16"))
    for w in works:
        tabs = [synth.make_table(w, t) for t in range(w.T)]
        batches = [synth.make_batch(w, 5)]
        got, _ = run_gpu(w, tabs, batches, want_perm=False, tuning=tuning)
        c = case_of(w)
        ref = oracle.pipeline(c, [t.numpy() for t in tabs], batches[0][0].numpy(), batches[0][1].numpy())
        for k in ("Y", "Out"):
            assert np.array_equal(bits(got[0][k]), bits(ref[k])), (w.name, k)


HOT = [(3, "small", None), (4, "small", None), (5, "small", None), (4, "small", "u8rq"), (6, "small", None)]


@pytest.mark.parametrize("cfg,size,storage", HOT)
def test_hot_row_lists_change_nothing(cfg, size, storage):
    """Popular rows named by the caller are served from LDS by workgroups that stay: whatever the lists
    name (the batch's truly popular rows, rows never looked up, repeats, lists for some shards only),
    every buffer equals the oracle's bit for bit, through the staged and the fused owner side, with
    and without per-sample weights."""
    from paper_2512_19342_amd.runner import Pipeline
    w = synth.workload(cfg, size)
    if storage:
        w.table_dtype = storage
    if w.table_dtype == "fp32":
        w.values = "gauss"
    dev = torch.device("cuda:0")
    tabs_cpu = [synth.make_table(w, t) for t in range(w.T)]
    batches = [synth.make_batch(w, it) for it in range(2)]
    pipe = Pipeline(w, [t.to(dev) for t in tabs_cpu], max(int(o[-1]) for _, o in batches))
    c, ctx = case_of(w), pipe.ctx
    tabs_np = [t.numpy() for t in tabs_cpu]
    rng = np.random.default_rng(cfg)
    true_hot = pipe.hot_rows_from_batch(batches[0][0], batches[0][1], 300)       # more than the library keeps
    junk = {}
    for t in range(w.T):
        for d in (range(w.P) if w.part_kind == 1 else [w.table_owner[t]]):
            lo, n = ctx.bls_shard_range(t, d)
            if n and rng.random() < 0.7:                                          # some shards get no list
                r = rng.integers(0, n, int(rng.integers(1, 40))).tolist()
                junk[(t, d)] = r + r[:3]                                          # with repeats
    for lists in (true_hot, junk):
        pipe.set_hot_rows(lists)
        for ix, off in batches:
            nnz = int(off[-1])
            ref = oracle.pipeline(c, tabs_np, ix.numpy(), off.numpy())
            out = pipe.new_out()
            it, slot = pipe.issue(ix.to(dev), off.to(dev), nnz)
            assert np.array_equal(bits(pipe.pooled.cpu().numpy()), bits(ref["Y"]))
            pipe.complete(it, out)
            assert np.array_equal(bits(out.cpu().numpy()), bits(ref["Out"]))
            it, slot = pipe.issue_fused(ix.to(dev), off.to(dev), nnz)
            assert np.array_equal(bits(pipe.slot_view(slot).cpu().numpy()), bits(ref["R"]))
            pipe.complete(it, out)
        ix, off = batches[1]
        nnz = int(off[-1])
        wts = torch.from_numpy(rng.uniform(-2.0, 2.0, size=nnz).astype(np.float32))
        ref = oracle.pipeline(c, tabs_np, ix.numpy(), off.numpy(), weights=wts.numpy())
        out = pipe.new_out()
        it, _ = pipe.issue_weighted(ix.to(dev), off.to(dev), wts.to(dev), nnz)
        pipe.complete(it, out)
        assert np.array_equal(bits(out.cpu().numpy()), bits(ref["Out"]))
        ctx.bls_check()
    import paper_2512_19342_amd as B
    with pytest.raises(B.BlsError) as e:                                          # a row outside the shard
        t0 = 0
        d0 = 0 if w.part_kind == 1 else w.table_owner[0]
        ctx.bls_set_hot_rows(t0, d0, [ctx.bls_shard_range(t0, d0)[1]])
    assert e.value.code == B.BLS_EINVAL


FUSED = [synth.workload(1), synth.workload(2), synth.workload(3, "small"), synth.workload(4, "small"),
         synth.workload(5, "small")] + [
    synth.custom("edge", k=2, values="gauss", table_dtype=dt, seed=29, index_dist=("zipf", 1.1), **EDGE[i])
    for i in (2, 4, 5, 6, 7, 8, 10) for dt in ("fp32", "fp16")] + [
    synth.custom("edge", k=2, values="gauss", table_dtype="u8rq", seed=29, index_dist=("zipf", 1.1), **EDGE[i])
    for i in (5, 7, 9)]


@pytest.mark.parametrize("w", FUSED, ids=lambda w: f"{w.name}-{w.table_dtype}-D{w.D}-P{w.P}")
def test_pool_put_equals_staged_path(w):
    """bls_embbag_pool_put (pool straight into the ring slot) must leave the receive regions and
    the output exactly as pool + pack + alltoallv do, and as the oracle says."""
    from paper_2512_19342_amd.runner import Pipeline
    if w.name in ("cfg3s", "cfg4s"):
        w.values = "gauss"
    dev = torch.device("cuda:0")
    tabs_cpu = [synth.make_table(w, t) for t in range(w.T)]
    pipe = Pipeline(w, [t.to(dev) for t in tabs_cpu], 1 << 21)
    c = case_of(w)
    tabs_np = [t.numpy() for t in tabs_cpu]
    pending = []
    for it in range(3):
        ix, off = synth.make_batch(w, it)
        nnz = int(off[-1])
        if len(pending) == pipe.ctx.K:
            j, out, ref = pending.pop(0)
            pipe.complete(j, out)
            assert np.array_equal(bits(out.cpu().numpy()), bits(ref["Out"])), (w.name, j)
        j, slot = pipe.issue_fused(ix.to(dev), off.to(dev), nnz)
        ref = oracle.pipeline(c, tabs_np, ix.numpy(), off.numpy())
        assert np.array_equal(bits(pipe.slot_view(slot).cpu().numpy()), bits(ref["R"])), (w.name, it)
        pending.append((j, pipe.new_out(), ref))
    for j, out, ref in pending:
        pipe.complete(j, out)
        assert np.array_equal(bits(out.cpu().numpy()), bits(ref["Out"])), (w.name, j)
    pipe.ctx.bls_check()


ONE_LAUNCH = [synth.workload(1), synth.workload(2), synth.workload(4, "small"), synth.workload(6, "small")] + [
    synth.custom("edge", k=k, values="gauss", table_dtype=dt, seed=41, index_dist=("zipf", 1.1), **EDGE[i])
    for i, k in ((0, 0), (1, 1), (2, 3), (7, 2), (11, 1), (13, 2)) for dt in ("fp32", "fp16", "u8rq")
    if (EDGE[i]["D"] * {"fp32": 4, "fp16": 2, "u8rq": 1}[dt]) % 16 == 0]


@pytest.mark.parametrize("w", ONE_LAUNCH, ids=lambda w: f"{w.name}-{w.table_dtype}-D{w.D}-P{w.P}-B{w.B}-k{w.k}")
def test_one_launch_step_equals_staged_path(w):
    """bls_step_tablewise writes every output of the staged calls in one launch: counts, displacements,
    ridx, segoff, perm, the pooled, send and receive buffers and the output, all equal to the oracle's,
    iteration after iteration (the ring slot rotates), and mixes with the staged calls on one context."""
    from paper_2512_19342_amd.runner import Pipeline
    if w.name in ("cfg4s", "cfg6s"):
        w.values = "gauss"
    dev = torch.device("cuda:0")
    tabs_cpu = [synth.make_table(w, t) for t in range(w.T)]
    pipe = Pipeline(w, [t.to(dev) for t in tabs_cpu], 1 << 21, want_perm=True)
    c = case_of(w)
    tabs_np = [t.numpy() for t in tabs_cpu]
    for it in range(4):
        ix, off = synth.make_batch(w, it)
        nnz = int(off[-1])
        ref = oracle.pipeline(c, tabs_np, ix.numpy(), off.numpy())
        out = pipe.new_out().fill_(float("nan"))
        for buf in (pipe.ridx, pipe.perm, pipe.segoff, pipe.sendcounts, pipe.sdispls, pipe.recvcounts, pipe.rdispls):
            buf.fill_(-7)
        if it == 2:                                               # a staged iteration in between
            pipe.step(ix.to(dev), off.to(dev), nnz, out)
            j = it
        else:
            j = pipe.step_one_launch(ix.to(dev), off.to(dev), nnz, out)
        assert j == it
        pipe.ctx.bls_check()
        for k in ("sendcounts", "sdispls", "recvcounts", "rdispls", "segoff"):
            assert np.array_equal(getattr(pipe, k).cpu().numpy(), ref[k]), (k, it)
        assert np.array_equal(pipe.ridx[:nnz].cpu().numpy(), ref["ridx"]), it
        assert np.array_equal(pipe.perm[:nnz].cpu().numpy(), ref["perm"]), it
        for k, buf in (("Y", pipe.pooled), ("S", pipe.send), ("R", pipe.slot_view(j % pipe.ctx.K)), ("Out", out)):
            assert np.array_equal(bits(buf.cpu().numpy().reshape(-1)), bits(ref[k].reshape(-1))), (k, it)
    head, tail, _ = pipe.ctx.bls_ring_state()
    assert head == tail == 4


def test_one_launch_step_flags_bad_inputs():
    """Bad indices and offsets through the one-launch step: flagged, never a fault; a bad index adds
    nothing to its bag, as in the staged calls."""
    import paper_2512_19342_amd as B
    from paper_2512_19342_amd.runner import Pipeline
    w = synth.workload(4, "small")
    dev = torch.device("cuda:0")
    tabs = [synth.make_table(w, t).to(dev) for t in range(w.T)]
    ix, off = synth.make_batch(w, 0)
    nnz = int(off[-1])
    pipe = Pipeline(w, tabs, nnz, want_perm=True)
    for how in ("index_high", "index_negative", "offsets_decrease", "offsets_past_end", "run_edge_negative"):
        bix, boff = ix.clone(), off.clone()
        if how == "index_high":
            bix[nnz // 2] = 10 ** 12
        elif how == "index_negative":
            bix[5] = -3
        elif how == "offsets_decrease":
            boff[10] = boff[12] + 5
        elif how == "offsets_past_end":
            boff[-1] = nnz + 1000
        else:
            boff[w.B] = -4                                         # the first bag of the second table
        out = pipe.new_out()
        pipe.step_one_launch(bix.to(dev), boff.to(dev), nnz, out)
        with pytest.raises(B.BlsError) as e:
            pipe.ctx.bls_check()
        assert e.value.code == B.BLS_ERANGE, how
        if how.startswith("index"):
            at = nnz // 2 if how == "index_high" else 5
            goff = off.numpy().copy()
            goff[goff > at] -= 1
            want = oracle.pipeline(case_of(w), [t.cpu().numpy() for t in tabs], np.delete(ix.numpy(), at), goff)["Out"]
            assert np.array_equal(bits(out.cpu().numpy()), bits(want)), how
    out = pipe.new_out()
    pipe.step_one_launch(ix.to(dev), off.to(dev), nnz, out)
    pipe.ctx.bls_check()
    ref = oracle.pipeline(case_of(w), [t.cpu().numpy() for t in tabs], ix.numpy(), off.numpy())["Out"]
    assert np.array_equal(bits(out.cpu().numpy()), bits(ref))


def test_one_launch_step_refusals():
    import paper_2512_19342_amd as B
    from paper_2512_19342_amd.runner import Pipeline
    dev = torch.device("cuda:0")
    w = synth.workload(3, "small")                                # row-wise
    pipe = Pipeline(w, [synth.make_table(w, t).to(dev) for t in range(w.T)], 1 << 20)
    ix, off = synth.make_batch(w, 0)
    with pytest.raises(B.BlsError) as e:
        pipe.step_one_launch(ix.to(dev), off.to(dev), int(off[-1]), pipe.new_out())
    assert e.value.code == B.BLS_EINVAL and "row-wise" in pipe.ctx.bls_last_error()
    w = synth.custom("odd", P=2, T=2, D=7, k=2, B=8, rows=[9, 9], part_kind=0)   # 28-byte rows
    pipe = Pipeline(w, [synth.make_table(w, t).to(dev) for t in range(w.T)], 1 << 10)
    ix, off = synth.make_batch(w, 0)
    with pytest.raises(B.BlsError) as e:
        pipe.step_one_launch(ix.to(dev), off.to(dev), int(off[-1]), pipe.new_out())
    assert e.value.code == B.BLS_EINVAL
    w = synth.workload(4, "small")
    pipe = Pipeline(w, [synth.make_table(w, t).to(dev) for t in range(w.T)], 1 << 21)
    ix, off = synth.make_batch(w, 0)
    j, _ = pipe.issue(ix.to(dev), off.to(dev), int(off[-1]))      # an iteration in flight
    with pytest.raises(B.BlsError) as e:
        pipe.step_one_launch(ix.to(dev), off.to(dev), int(off[-1]), pipe.new_out())
    assert e.value.code == B.BLS_EORDER
    pipe.complete(j, pipe.new_out())
    pipe.step_one_launch(ix.to(dev), off.to(dev), int(off[-1]), pipe.new_out())
    pipe.ctx.bls_check()


def test_pool_put_needs_the_current_slot():
    import paper_2512_19342_amd as B
    from paper_2512_19342_amd.runner import Pipeline
    w = synth.workload(4, "small")
    dev = torch.device("cuda:0")
    pipe = Pipeline(w, [synth.make_table(w, t).to(dev) for t in range(w.T)], 1 << 21)
    ix, off = synth.make_batch(w, 0)
    nnz = int(off[-1])
    with pytest.raises(B.BlsError) as e:                  # no iteration started
        pipe.ctx.bls_embbag_pool_put(pipe.ridx, pipe.segoff, 0, 0)
    assert e.value.code == B.BLS_EORDER
    j, slot = pipe.issue_fused(ix.to(dev), off.to(dev), nnz)
    with pytest.raises(B.BlsError) as e:                  # slot already filled
        pipe.ctx.bls_embbag_pool_put(pipe.ridx, pipe.segoff, nnz, slot)
    assert e.value.code == B.BLS_EORDER
    with pytest.raises(B.BlsError) as e:
        pipe.ctx.bls_embbag_pool_put(pipe.ridx, pipe.segoff, nnz, 99)
    assert e.value.code == B.BLS_EINVAL
    pipe.complete(j, pipe.new_out())
    pipe.ctx.bls_check()


WEIGHTED = [synth.workload(2), synth.workload(3, "small"), synth.workload(4, "small"), synth.workload(5, "small"),
            synth.workload(6, "small")] + [
    synth.custom("edge", k=1, values="gauss", table_dtype=dt, seed=31, index_dist=("zipf", 1.1), **EDGE[i])
    for i in (1, 2, 4, 5, 6, 7, 8, 10) for dt in ("fp32", "fp16")] + [
    synth.custom("edge", k=1, values="gauss", table_dtype=dt, seed=31, index_dist=("zipf", 1.1), **EDGE[i])
    for i in (4, 6, 7, 9, 10) for dt in ("u8rq", "f8rq")]


@pytest.mark.parametrize("w", WEIGHTED, ids=lambda w: f"{w.name}-{w.table_dtype}-D{w.D}-P{w.P}-part{w.part_kind}")
def test_weighted_and_mean_pooling(w):
    """Per-sample weights (every product rounded, then added) through the staged and the fused
    owner side, and mean pooling at completion, bit for bit against the oracle."""
    from paper_2512_19342_amd.runner import Pipeline
    if w.name in ("cfg3s", "cfg4s", "cfg6s"):
        w.values = "gauss"
    dev = torch.device("cuda:0")
    tabs_cpu = [synth.make_table(w, t) for t in range(w.T)]
    pipe = Pipeline(w, [t.to(dev) for t in tabs_cpu], 1 << 21)
    c = case_of(w)
    tabs_np = [t.numpy() for t in tabs_cpu]
    ix, off = synth.make_batch(w, 4)
    nnz = int(off[-1])
    rng = np.random.default_rng(nnz)
    wts = torch.from_numpy(rng.uniform(-2.0, 2.0, size=nnz).astype(np.float32))
    ref = oracle.pipeline(c, tabs_np, ix.numpy(), off.numpy(), weights=wts.numpy())
    d_ix, d_off, d_w = ix.to(dev), off.to(dev), wts.to(dev)
    for fused in (False, True):
        out = pipe.new_out()
        j, slot = pipe.issue_weighted(d_ix, d_off, d_w, nnz, fused=fused)
        assert np.array_equal(pipe.ridx[:nnz].cpu().numpy(), ref["ridx"])
        assert np.array_equal(bits(pipe.rweights[:nnz].cpu().numpy()), bits(ref["rweights"]))
        if not fused:
            assert np.array_equal(bits(pipe.pooled.cpu().numpy()), bits(ref["Y"]))
        assert np.array_equal(bits(pipe.slot_view(slot).cpu().numpy()), bits(ref["R"])), fused
        pipe.complete(j, out)
        assert np.array_equal(bits(out.cpu().numpy()), bits(ref["Out"])), fused
    o64, _ = oracle.embbag_plain(c, tabs_np, ix.numpy(), off.numpy(), want32=False, weights=wts.numpy())
    mass = oracle.embbag_absmass(c, tabs_np, ix.numpy(), off.numpy())
    assert np.all(np.abs(out.cpu().numpy().astype(np.float64) - o64) <= 4 * TOL[w.table_dtype] * mass + 1e-30)
    # mean pooling
    refm = oracle.pipeline(c, tabs_np, ix.numpy(), off.numpy(), mean=True)["Out"]
    for fused in (False, True):
        out = pipe.new_out()
        j, slot = (pipe.issue_fused if fused else pipe.issue)(d_ix, d_off, nnz)
        pipe.complete(j, out, mean_offsets=d_off)
        assert np.array_equal(bits(out.cpu().numpy()), bits(refm)), fused
    pipe.ctx.bls_check()


@pytest.mark.parametrize("k", [0, 2, 4])
@pytest.mark.parametrize("cfg", [3, 4, 6])
def test_per_rank_issue_and_completion(k, cfg):
    """Every simulated rank on its own stream, ranks served in a scrambled order, stragglers
    delayed on the device: whatever the interleaving within the bound, every iteration's
    output is the oracle's, bit for bit; the ring refuses what the bound forbids."""
    import paper_2512_19342_amd as B
    from paper_2512_19342_amd.runner import Pipeline
    w = synth.workload(cfg, "small")
    w.k = k
    w.values = "gauss"
    dev = torch.device("cuda:0")
    tabs_cpu = [synth.make_table(w, t) for t in range(w.T)]
    pipe = Pipeline(w, [t.to(dev) for t in tabs_cpu], 1 << 21)
    c, ctx, P, K = case_of(w), pipe.ctx, w.P, max(k, 1)
    tabs_np = [t.numpy() for t in tabs_cpu]
    N = 6
    rng = np.random.default_rng(100 * cfg + k)
    streams = [torch.cuda.Stream() for _ in range(P)]
    plans, refs, outs = [], [], []
    for it in range(N):                               # plans are prepared up front, one buffer set each
        ix, off = synth.make_batch(w, it)
        nnz = int(off[-1])
        ctx.bls_plan(ix.to(dev), off.to(dev), nnz, pipe.sendcounts, pipe.sdispls, pipe.recvcounts, pipe.rdispls,
                     pipe.ridx, pipe.segoff, None, pipe.ws)
        plans.append((pipe.ridx[:max(nnz, 1)].clone(), pipe.segoff.clone(), nnz))
        refs.append(oracle.pipeline(c, tabs_np, ix.numpy(), off.numpy())["Out"])
        outs.append(pipe.new_out())
    torch.cuda.synchronize()
    with pytest.raises(B.BlsError) as e:
        ctx.bls_rank_complete(0, 0, None, outs[0], streams[0])
    assert e.value.code == B.BLS_ERING_EMPTY
    done = [0] * P
    for it in range(N):
        if it >= K:                                   # the slot must be released by every requester first
            with pytest.raises(B.BlsError) as e:
                ctx.bls_rank_put(0, plans[it][0], None, plans[it][1], plans[it][2], it, streams[0])
            assert e.value.code == B.BLS_ERING_FULL
            for s in rng.permutation(P):
                ctx.bls_rank_complete(int(s), it - K, None, outs[it - K], streams[s])
                done[s] += 1
        order = rng.permutation(P)
        if it == 0:
            ctx.bls_rank_put(int(order[0]), plans[0][0], None, plans[0][1], plans[0][2], 0, streams[order[0]])
            with pytest.raises(B.BlsError) as e:      # not every owner has issued iteration 0 yet
                ctx.bls_rank_complete(0, 0, None, outs[0], streams[0])
            assert e.value.code == B.BLS_EORDER
            with pytest.raises(B.BlsError) as e:      # an owner cannot skip ahead
                ctx.bls_rank_put(int(order[0]), plans[0][0], None, plans[0][1], plans[0][2], 2, streams[order[0]])
            assert e.value.code == B.BLS_EORDER
            order = order[1:]
        for d in order:
            if rng.random() < 0.4:
                ctx.bls_rank_delay(int(rng.integers(50, 400)), streams[d])
            ctx.bls_rank_put(int(d), plans[it][0], None, plans[it][1], plans[it][2], it, streams[d])
    for it in range(max(N - K, 0), N):
        for s in rng.permutation(P):
            ctx.bls_rank_complete(int(s), it, None, outs[it], streams[s])
    torch.cuda.synchronize()
    ctx.bls_check()
    for it in range(N):
        assert np.array_equal(bits(outs[it].cpu().numpy()), bits(refs[it])), (cfg, k, it)
    # back to whole-batch calls on the same context once everything has drained
    ix, off = synth.make_batch(w, 0)
    out = pipe.new_out()
    pipe.step(ix.to(dev), off.to(dev), int(off[-1]), out)
    assert np.array_equal(bits(out.cpu().numpy()), bits(refs[0]))


@pytest.mark.parametrize("part_kind", [0, 1])
def test_per_rank_weighted_and_mean(part_kind):
    """The per-rank calls with per-sample weights in the puts and mean pooling at completion."""
    from paper_2512_19342_amd.runner import Pipeline
    w = synth.custom("rankw", P=3, T=4, D=24, B=31, k=2, part_kind=part_kind, rows=[300, 17, 1000, 64], values="gauss",
                     bag=("uniform", 0, 9), index_dist=("zipf", 1.1), seed=63)
    dev = torch.device("cuda:0")
    tabs_cpu = [synth.make_table(w, t) for t in range(w.T)]
    pipe = Pipeline(w, [t.to(dev) for t in tabs_cpu], 4096)
    c, ctx = case_of(w), pipe.ctx
    streams = [torch.cuda.Stream() for _ in range(w.P)]
    rng = np.random.default_rng(7)
    for mean in (False, True):
        runs = []
        for j in range(2):                                      # two iterations in flight (K = 2)
            it = (2 if mean else 0) + j
            ix, off = synth.make_batch(w, it)
            nnz = int(off[-1])
            wts = torch.from_numpy(rng.uniform(-2, 2, nnz).astype(np.float32))
            rweights = torch.zeros(max(nnz, 1), dtype=torch.float32, device=dev)
            ctx.bls_plan_weighted(ix.to(dev), off.to(dev), wts.to(dev), nnz, pipe.sendcounts, pipe.sdispls, pipe.recvcounts,
                                  pipe.rdispls, pipe.ridx, rweights, pipe.segoff, None, pipe.ws)
            ridx, segoff, off_d = pipe.ridx[:max(nnz, 1)].clone(), pipe.segoff.clone(), off.to(dev)
            torch.cuda.synchronize()
            for d in rng.permutation(w.P):
                ctx.bls_rank_put(int(d), ridx, rweights, segoff, nnz, it, streams[d])
            ref = oracle.pipeline(c, [t.numpy() for t in tabs_cpu], ix.numpy(), off.numpy(), weights=wts.numpy(), mean=mean)["Out"]
            runs.append((it, off_d, ref, pipe.new_out()))
        for it, off_d, ref, out in runs:
            for s in rng.permutation(w.P):
                ctx.bls_rank_complete(int(s), it, off_d if mean else None, out, streams[s])
        torch.cuda.synchronize()
        ctx.bls_check()
        for it, off_d, ref, out in runs:
            assert np.array_equal(bits(out.cpu().numpy()), bits(ref)), (mean, it)


@pytest.mark.parametrize("cfg,size", [(2, "full"), (5, "small")], ids=["tablewise", "rowwise"])
def test_step_can_be_captured_in_a_graph_and_replayed(cfg, size):
    """The whole staged step recorded once into a HIP graph (the calls allocate nothing and clear
    nothing with memsets) and replayed on new batches written into the same input buffers, with
    eager work and synchronisations between the replays: every replay equals the oracle.  Both
    partitions: the plan has a form of its own for each."""
    from paper_2512_19342_amd.runner import Pipeline
    w = synth.workload(cfg, size)                               # bags of a fixed length: every batch has the same number of lookups
    dev = torch.device("cuda:0")
    tabs_cpu = [synth.make_table(w, t) for t in range(w.T)]
    batches = [synth.make_batch(w, it) for it in range(4)]
    nnz = int(batches[0][1][-1])
    assert all(int(off[-1]) == nnz for _, off in batches)
    pipe = Pipeline(w, [t.to(dev) for t in tabs_cpu], nnz)
    out = pipe.new_out()
    s_ix, s_off = batches[0][0].to(dev).clone(), batches[0][1].to(dev).clone()
    torch.cuda.synchronize()                                    # no eager step first: no call allocates or uploads
    graph, st = torch.cuda.CUDAGraph(), torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(st):
        with torch.cuda.graph(graph, stream=st):
            pipe.step(s_ix, s_off, nnz, out, stream=st)
    torch.cuda.synchronize()
    c = case_of(w)
    tabs_np = [t.numpy() for t in tabs_cpu]
    for ix, off in batches[1:] + batches[:1]:
        s_ix.copy_(ix.to(dev))
        s_off.copy_(off.to(dev))
        out.fill_(float("nan"))
        torch.randn(4096, device=dev).sum().item()              # unrelated eager work and a synchronisation
        graph.replay()
        torch.cuda.synchronize()
        ref = oracle.pipeline(c, tabs_np, ix.numpy(), off.numpy())
        assert np.array_equal(bits(out.cpu().numpy()), bits(ref["Out"]))
        assert np.array_equal(pipe.sendcounts.cpu().numpy(), ref["sendcounts"])
        assert np.array_equal(pipe.ridx[:nnz].cpu().numpy(), ref["ridx"])
    pipe.ctx.bls_check()
    head, tail, _ = pipe.ctx.bls_ring_state()
    assert head == tail                                          # the recorded step left nothing in flight


def _random_spec(rng):
    P = int(rng.integers(1, 10))
    T = int(rng.integers(1, 8))
    D = int(rng.choice([1, 2, 3, 4, 6, 8, 12, 16, 20, 24, 32, 40, 64, 128, int(rng.integers(1, 70))]))
    B = int(rng.integers(P, 90))
    rows = [int(rng.choice([1, 2, int(rng.integers(1, 50)), int(rng.integers(50, 5000))])) for _ in range(T)]
    lo = int(rng.integers(0, 3))
    bag = ("uniform", lo, lo + int(rng.integers(0, 40))) if rng.random() < 0.8 else ("fixed", int(rng.integers(0, 5)))
    return dict(P=P, T=T, D=D, B=B, part_kind=int(rng.integers(0, 2)), rows=rows, bag=bag,
                k=int(rng.integers(0, 4)), table_dtype=str(rng.choice(["fp32", "fp16", "u8rq", "f8rq"])),
                index_dist=("zipf", 1.1) if rng.random() < 0.5 else ("uniform",))


@pytest.mark.parametrize("seed", range(40))
def test_random_shapes(seed):
    """Shapes drawn at random (ranks, tables, vector lengths incl. odd ones, ragged batches, one-row
    tables, empty bags, every storage type, both partitions): the staged path, the fused owner side
    with weights, and mean pooling, all against the oracle bit for bit."""
    from paper_2512_19342_amd.runner import Pipeline
    rng = np.random.default_rng(1000 + seed)
    spec = _random_spec(rng)
    w = synth.custom(f"rand{seed}", values="gauss", seed=100 + seed, **spec)
    tabs = [synth.make_table(w, t) for t in range(w.T)]
    batches = [synth.make_batch(w, it) for it in range(2)]
    got, pipe = run_gpu(w, tabs, batches)
    check_against_oracle(w, tabs, batches, got)
    dev, c = torch.device("cuda:0"), case_of(w)
    ix, off = batches[1]
    nnz = int(off[-1])
    wts = torch.from_numpy(rng.uniform(-2, 2, max(nnz, 1)).astype(np.float32))[:nnz]
    out = pipe.new_out()
    it, _ = pipe.issue_weighted(ix.to(dev), off.to(dev), wts.to(dev), nnz, fused=True)
    pipe.complete(it, out, mean_offsets=off.to(dev))
    pipe.ctx.bls_check()
    ref = oracle.pipeline(c, [t.numpy() for t in tabs], ix.numpy(), off.numpy(), weights=wts.numpy(), mean=True)["Out"]
    assert np.array_equal(bits(out.cpu().numpy()), bits(ref)), spec
