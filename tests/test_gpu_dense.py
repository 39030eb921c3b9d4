"""Parity of the dense kernels (bls_mlp_layer, bls_interact) against the CPU oracle, through the
C ABI.  The oracle evaluates in double; the fp32 matrix-core result must lie within the bound
the oracle derives from the arithmetic for the same fp32 inputs: (K + 3) roundings of 2^-24 on
|bias| + sum |x||w| for a layer (a few more for the sigmoid), (D + 2) on sum |u||v| for a dot
product of the interaction.  Each kernel is checked on the inputs it really received; the whole
chain is also compared with the oracle's chain under the bound carried from layer to layer."""
import numpy as np
import pytest
import torch

import oracle
import synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def ctx_for(T=2, D=4, B=4):
    import paper_2512_19342_amd as A
    return A.Context(1, T, D, 0, B, [4] * T, [0] * T)


LAYERS = [
    # M, K, N, act, bias
    (1, 1, 1, 0, True), (5, 13, 7, 1, True), (130, 13, 512, 1, True), (257, 512, 256, 1, True),
    (128, 256, 128, 0, False), (300, 276, 100, 1, True), (64, 100, 1, 2, True), (200, 17, 33, 2, True),
    (384, 64, 1024, 1, True), (129, 130, 129, 1, False), (1000, 16, 16, 0, True), (3, 2208, 40, 1, True),
]


@pytest.mark.parametrize("M,K,N,act,has_bias", LAYERS)
def test_mlp_layer_matches_oracle(M, K, N, act, has_bias):
    c = ctx_for()
    rng = np.random.default_rng(M * 7 + K * 3 + N)
    x = rng.normal(0, 1, size=(M, K)).astype(np.float32)
    W = (rng.normal(0, 1, size=(N, K)) / np.sqrt(K)).astype(np.float32)
    b = rng.normal(0, 1, size=N).astype(np.float32) if has_bias else None
    y = torch.full((M, N), float("nan"), device=DEV)
    c.bls_mlp_layer(torch.from_numpy(x).to(DEV), torch.from_numpy(W).to(DEV),
                    None if b is None else torch.from_numpy(b).to(DEV), act, y)
    c.bls_check()
    ref, err = oracle.mlp_layer(x, W, b, act)
    got = y.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got)) and np.all(np.abs(got - ref) <= err)
    # the worst case grows with K; rounding errors behave like a random walk, so in practice the
    # result is within a few sqrt(K) roundings (the sigmoid's own few units included)
    assert np.all(np.abs(got - ref) <= 4.0 * err / np.sqrt(K + 3) + (8 * 2.0 ** -24 if act == 2 else 0.0))
    assert err.max() <= 2e-3 * max(1.0, np.abs(ref).max())


def test_mlp_layer_unaligned_rows_and_empty():
    """A view that starts 4 bytes into an allocation takes the scalar-load path; M = 0 is a no-op."""
    c = ctx_for()
    rng = np.random.default_rng(9)
    M, K, N = 70, 24, 50
    x = rng.normal(size=(M, K)).astype(np.float32)
    W = rng.normal(size=(N, K)).astype(np.float32)
    xb = torch.zeros(M * K + 1, device=DEV)
    xb[1:] = torch.from_numpy(x).reshape(-1).to(DEV)
    xv = xb[1:].view(M, K)
    assert xv.data_ptr() % 16 == 4
    y = torch.empty((M, N), device=DEV)
    c.bls_mlp_layer(xv, torch.from_numpy(W).to(DEV), None, 1, y)
    ref, err = oracle.mlp_layer(x, W, None, 1)
    assert np.all(np.abs(y.cpu().numpy() - ref) <= err)
    c.bls_mlp_layer(torch.empty((0, K), device=DEV), torch.from_numpy(W).to(DEV), None, 1, torch.empty((0, N), device=DEV))
    c.bls_check()


INTERACT = [(1, 4, 3), (3, 5, 6), (8, 16, 9), (26, 64, 20), (64, 128, 12), (33, 20, 7), (70, 32, 5), (32, 7, 4), (2, 1, 3)]


@pytest.mark.parametrize("T,D,B", INTERACT)
def test_interact_matches_oracle(T, D, B):
    c = ctx_for(T, D, B)
    rng = np.random.default_rng(T * 5 + D)
    x = rng.normal(size=(B, D)).astype(np.float32)
    emb = rng.normal(size=(B, T, D)).astype(np.float32)
    Wz = D + T * (T + 1) // 2
    z = torch.full((B, Wz), float("nan"), device=DEV)
    c.bls_interact(torch.from_numpy(x).to(DEV), torch.from_numpy(emb).to(DEV), z)
    c.bls_check()
    ref, err = oracle.interact(x, emb)
    got = z.cpu().numpy()
    assert np.array_equal(got[:, :D], x)                      # the dense vector is copied
    assert np.all(np.abs(got - ref) <= err)
    # a range of samples leaves the others alone
    if B >= 3:
        z2 = torch.full((B, Wz), -7.0, device=DEV)
        c.bls_interact(torch.from_numpy(x).to(DEV), torch.from_numpy(emb).to(DEV), z2, 1, B - 2)
        g2 = z2.cpu().numpy()
        assert np.all(g2[0] == -7.0) and np.all(g2[-1] == -7.0) and np.array_equal(g2[1:-1], got[1:-1])


def test_dense_bad_arguments():
    import paper_2512_19342_amd as A
    c = ctx_for(2, 4, 4)
    t = torch.zeros((4, 4), device=DEV)
    with pytest.raises(A.BlsError) as e:
        c.bls_mlp_layer(t, t, None, 7, torch.zeros((4, 4), device=DEV))
    assert e.value.code == A.BLS_EINVAL
    with pytest.raises(A.BlsError):
        c.bls_interact(t, torch.zeros((4, 2, 4), device=DEV), torch.zeros((4, 7), device=DEV), 2, 3)   # 2 + 3 > B
    big = ctx_for(64, 512, 4)                                  # 64 vectors of 512 floats: 128 KB
    with pytest.raises(A.BlsError) as e:
        big.bls_interact(torch.zeros((4, 512), device=DEV), torch.zeros((4, 64, 512), device=DEV),
                         torch.zeros((4, 512 + 2080), device=DEV))
    assert e.value.code == A.BLS_EINVAL


@pytest.mark.parametrize("cfg", [2, 4])
def test_model_around_the_lookup(cfg):
    """Bottom MLP, the lookup through the path, interaction, top MLP -> prediction, on a workload's
    reduced twin: every kernel against the oracle on the inputs it received, and the prediction
    against the oracle's own chain."""
    from paper_2512_19342_amd.runner import DenseModel, Pipeline
    w = synth.workload(cfg, "small") if cfg != 2 else synth.workload(2)
    tabs = [synth.make_table(w, t) for t in range(w.T)]
    ix, off = synth.make_batch(w, 1)
    nnz = int(off[-1])
    pipe = Pipeline(w, [t.to(DEV) for t in tabs], nnz)
    bot_sizes, top_sizes = synth.mlp_sizes(w, "small")
    bot, top = synth.mlp_weights(w, bot_sizes, 0), synth.mlp_weights(w, top_sizes, 1)
    model = DenseModel(pipe.ctx, [(W.to(DEV), b.to(DEV)) for W, b in bot], [(W.to(DEV), b.to(DEV)) for W, b in top], w.B)
    dense = synth.dense_features(w, 1)

    out = pipe.new_out()
    it, _ = pipe.issue_fused(ix.to(DEV), off.to(DEV), nnz)
    x = model.apply_bottom(dense.to(DEV))
    pipe.complete(it, out)
    p = model.compute_ctr(x, out)
    pipe.ctx.bls_check()

    case = oracle.Case(w.P, w.T, w.D, w.B, w.part_kind, w.rows, w.table_owner, w.dtype_code)
    emb = oracle.pipeline(case, [t.numpy() for t in tabs], ix.numpy(), off.numpy())["Out"]
    assert np.array_equal(out.cpu().numpy(), emb)
    # kernel by kernel, each on what it was given
    a = dense.numpy()
    for (W, b), y in zip(bot, model.bot_act):
        ref, err = oracle.mlp_layer(a, W.numpy(), b.numpy(), 1)
        a = y.cpu().numpy()
        assert np.all(np.abs(a - ref) <= err)
    ref, err = oracle.interact(a, emb)
    a = model.z.cpu().numpy()
    assert np.all(np.abs(a - ref) <= err)
    for i, ((W, b), y) in enumerate(zip(top, model.top_act)):
        ref, err = oracle.mlp_layer(a, W.numpy(), b.numpy(), 2 if i == len(top) - 1 else 1)
        a = y.cpu().numpy()
        assert np.all(np.abs(a - ref) <= err)
    # the whole chain in double, with the bound carried along
    Lb = [(W.numpy(), b.numpy(), 1) for W, b in bot]
    Lt = [(W.numpy(), b.numpy(), 1) for W, b in top]
    Lt[-1] = (Lt[-1][0], Lt[-1][1], 2)
    x64, ex = oracle.mlp(dense.numpy(), Lb)
    z64, ez = oracle.interact(x64, emb, ex)
    p64, ep = oracle.mlp(z64, Lt, ez)
    got = p.cpu().numpy()
    assert got.shape == (w.B, 1) and np.all(np.abs(got - p64) <= ep)
    # the carried worst case is loose after six layers (about 1e-2); the prediction, a probability,
    # is in fact within a few fp32 units of the double-precision chain
    assert np.abs(got - p64).max() < 1e-6


@pytest.mark.parametrize("part_kind", [0, 1])
def test_bls_dlrm_loop_does_not_depend_on_the_bound(part_kind):
    """Listing 2's loop for bounds 0, 1 and 3: every iteration's prediction is the same bits
    whatever the bound, arrives in order, lags by at most the bound, and matches the oracle."""
    from paper_2512_19342_amd.runner import BlsDlrm, DenseModel, Pipeline
    n_iter = 6
    ref_bits, base = None, None
    for k, folded, second_stream in ((0, False, False), (1, False, False), (3, False, False), (3, True, False), (2, True, True)):
        w = synth.custom("loop", P=4, T=6, D=32, B=96, k=k, part_kind=part_kind, rows=[500, 64, 3000, 17, 256, 999],
                         bag=("uniform", 0, 12), index_dist=("zipf", 1.1), values="gauss", seed=51)
        tabs = [synth.make_table(w, t) for t in range(w.T)]
        batches = [synth.make_batch(w, it) for it in range(n_iter)]
        dense = [synth.dense_features(w, it) for it in range(n_iter)]
        pipe = Pipeline(w, [t.to(DEV) for t in tabs], max(int(o[-1]) for _, o in batches))
        bs, ts = synth.mlp_sizes(w, "small")
        bot, top = synth.mlp_weights(w, bs, 0), synth.mlp_weights(w, ts, 1)
        model = DenseModel(pipe.ctx, [(W.to(DEV), b.to(DEV)) for W, b in bot], [(W.to(DEV), b.to(DEV)) for W, b in top], w.B)
        # completion folded into the interaction, and the sparse side on a stream of its own, change nothing
        loop = BlsDlrm(pipe, model, fused_completion=folded, lookup_stream=torch.cuda.Stream() if second_stream else None)
        got = {}
        staged = [(dense[it].to(DEV), batches[it][0].to(DEV), batches[it][1].to(DEV)) for it in range(n_iter)]
        torch.cuda.synchronize()                                # inputs are in place before any stream reads them
        for it in range(n_iter):
            dn, ixd, offd = staged[it]
            for j, p in loop.forward(dn, ixd, offd, int(batches[it][1][-1]), last_batch=it == n_iter - 1):
                assert j == len(got) and it - j <= max(k, 0)  # FIFO, lag within the bound
                got[j] = p.cpu().numpy()
            if it < n_iter - 1:
                assert len(loop.unfinished) == min(k, it + 1)
        pipe.ctx.bls_check()
        assert sorted(got) == list(range(n_iter))
        bits = [got[j].view(np.uint32) for j in range(n_iter)]
        if ref_bits is None:
            ref_bits, base = bits, (w, tabs, batches, dense, bot, top)
        else:
            assert all(np.array_equal(a, b) for a, b in zip(bits, ref_bits)), k
    w, tabs, batches, dense, bot, top = base
    case = oracle.Case(w.P, w.T, w.D, w.B, w.part_kind, w.rows, w.table_owner, w.dtype_code)
    Lb = [(W.numpy(), b.numpy(), 1) for W, b in bot]
    Lt = [(W.numpy(), b.numpy(), 1) for W, b in top]
    Lt[-1] = (Lt[-1][0], Lt[-1][1], 2)
    for it in (0, n_iter - 1):
        emb = oracle.pipeline(case, [t.numpy() for t in tabs], batches[it][0].numpy(), batches[it][1].numpy())["Out"]
        x64, ex = oracle.mlp(dense[it].numpy(), Lb)
        z64, ez = oracle.interact(x64, emb, ex)
        p64, ep = oracle.mlp(z64, Lt, ez)
        p = ref_bits[it].view(np.float32)
        assert np.all(np.abs(p - p64) <= ep) and np.abs(p - p64).max() < 1e-6


@pytest.mark.parametrize("k", [1, 3])
def test_per_rank_model_loop_matches_the_whole_batch_loop(k):
    """Every simulated rank on its own stream (puts + bottom MLP of its mini-batch, later copy-out,
    interaction and top MLP), ranks visited in a scrambled order with device-side delays: the
    predictions are the bits the single-stream loop gives."""
    from paper_2512_19342_amd.runner import BlsDlrm, BlsDlrmRanks, DenseModel, Pipeline
    n_iter = 7
    w = synth.custom("ranks", P=4, T=5, D=32, B=90, k=k, part_kind=0, rows=[400, 64, 3000, 17, 256],
                     bag=("uniform", 0, 10), index_dist=("zipf", 1.1), values="gauss", seed=53)   # 90 = 23+23+22+22
    tabs = [synth.make_table(w, t).to(DEV) for t in range(w.T)]
    batches = [synth.make_batch(w, it) for it in range(n_iter)]
    dense = [synth.dense_features(w, it).to(DEV) for it in range(n_iter)]
    bs, ts = synth.mlp_sizes(w, "small")
    bot = [(W.to(DEV), b.to(DEV)) for W, b in synth.mlp_weights(w, bs, 0)]
    top = [(W.to(DEV), b.to(DEV)) for W, b in synth.mlp_weights(w, ts, 1)]
    max_nnz = max(int(o[-1]) for _, o in batches)

    pipe = Pipeline(w, tabs, max_nnz)
    loop = BlsDlrm(pipe, DenseModel(pipe.ctx, bot, top, w.B))
    want = {}
    for it in range(n_iter):
        ix, off = batches[it]
        for j, p in loop.forward(dense[it], ix.to(DEV), off.to(DEV), int(off[-1]), last_batch=it == n_iter - 1):
            want[j] = p.cpu().numpy()
    pipe.ctx.bls_check()

    pipe2 = Pipeline(w, tabs, max_nnz)
    c, K, P = pipe2.ctx, pipe2.ctx.K, w.P
    plans = []
    for ix, off in batches:
        nnz = int(off[-1])
        c.bls_plan(ix.to(DEV), off.to(DEV), nnz, pipe2.sendcounts, pipe2.sdispls, pipe2.recvcounts, pipe2.rdispls,
                   pipe2.ridx, pipe2.segoff, None, pipe2.ws)
        plans.append((pipe2.ridx[:max(nnz, 1)].clone(), pipe2.segoff.clone(), nnz))
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream() for _ in range(P)]
    ranks = BlsDlrmRanks(pipe2, DenseModel(c, bot, top, w.B), streams)
    rng = np.random.default_rng(k)
    got = {}

    def finish_all(it):
        parts = []
        for s in rng.permutation(P):
            pred = ranks.finish(int(s), it)
            lo, n = ranks.rows(int(s))
            with torch.cuda.stream(streams[s]):
                parts.append((lo, n, pred[lo:lo + n].clone()))       # the buffer is reused K iterations later
        got[it] = parts

    for it in range(n_iter):
        if it >= K:
            finish_all(it - K)
        for d in rng.permutation(P):
            ranks.issue(int(d), it, *plans[it], dense[it], delay_us=int(rng.integers(0, 300)))
    for it in range(max(n_iter - K, 0), n_iter):
        finish_all(it)
    torch.cuda.synchronize()
    c.bls_check()
    for it in range(n_iter):
        full = np.empty((w.B, 1), np.float32)
        for lo, n, part in got[it]:
            full[lo:lo + n] = part.cpu().numpy()
        assert np.array_equal(full.view(np.uint32), want[it].view(np.uint32)), it


FOLDED = [
    dict(P=3, T=5, D=32, B=50, part_kind=0, rows=[400, 64, 3000, 17, 256]),        # table-wise, P does not divide B
    dict(P=4, T=6, D=24, B=37, part_kind=1, rows=[500, 64, 3000, 17, 256, 999]),   # row-wise: partial vectors summed on the way
    dict(P=2, T=33, D=7, B=9, part_kind=1, rows=[40] * 33),                       # odd D (scalar copies), two tile rows
    dict(P=8, T=64, D=128, B=64, part_kind=0, rows=[300] * 64),                   # the benchmark's shape
]


@pytest.mark.parametrize("spec", FOLDED, ids=lambda s: f"T{s['T']}-D{s['D']}-P{s['P']}-part{s['part_kind']}")
def test_completion_folded_into_the_interaction(spec):
    """bls_unpack_interact gives the bits of bls_unpack followed by bls_interact, retires the slot,
    and keeps the ring's FIFO rule."""
    import paper_2512_19342_amd as A
    from paper_2512_19342_amd.runner import Pipeline
    w = synth.custom("folded", k=2, values="gauss", bag=("uniform", 0, 9), index_dist=("zipf", 1.1), seed=57, **spec)
    tabs = [synth.make_table(w, t).to(DEV) for t in range(w.T)]
    batches = [synth.make_batch(w, it) for it in range(3)]
    pipe = Pipeline(w, tabs, max(int(o[-1]) for _, o in batches))
    c = pipe.ctx
    Wz = w.D + w.T * (w.T + 1) // 2
    xs = [torch.randn((w.B, w.D), device=DEV) for _ in range(3)]
    want = []
    for (ix, off), x in zip(batches, xs):                       # staged: copy-out, then interaction
        out, z = pipe.new_out(), torch.empty((w.B, Wz), device=DEV)
        it, _ = pipe.issue_fused(ix.to(DEV), off.to(DEV), int(off[-1]))
        pipe.complete(it, out)
        c.bls_interact(x, out, z)
        want.append(z.cpu().numpy())
    its = []
    for ix, off in batches[:2]:                                 # two iterations in flight
        its.append(pipe.issue_fused(ix.to(DEV), off.to(DEV), int(off[-1]))[0])
    z = torch.full((w.B, Wz), float("nan"), device=DEV)
    with pytest.raises(A.BlsError) as e:
        c.bls_unpack_interact(its[1], xs[1], z)                 # not the oldest
    assert e.value.code == A.BLS_EORDER
    c.bls_unpack_interact(its[0], xs[0], z)
    assert np.array_equal(z.cpu().numpy().view(np.uint32), want[0].view(np.uint32))
    it2, _ = pipe.issue_fused(batches[2][0].to(DEV), batches[2][1].to(DEV), int(batches[2][1][-1]))   # the slot is free again
    for it, k in ((its[1], 1), (it2, 2)):
        c.bls_unpack_interact(it, xs[k], z)
        assert np.array_equal(z.cpu().numpy().view(np.uint32), want[k].view(np.uint32)), k
    assert c.bls_ring_state()[0] == c.bls_ring_state()[1]       # nothing left in flight
    with pytest.raises(A.BlsError) as e:
        c.bls_unpack_interact(it2 + 1, xs[0], z)
    assert e.value.code == A.BLS_ERING_EMPTY
    c.bls_check()


@pytest.mark.parametrize("seed", range(20))
def test_random_dense_shapes(seed):
    """Layer and interaction shapes drawn at random (tile edges, K not a multiple of 4 or 16, N = 1)."""
    rng = np.random.default_rng(500 + seed)
    M, K, N = int(rng.integers(1, 400)), int(rng.choice([1, 3, 13, 16, 17, 64, 100, 128, 260])), int(rng.choice([1, 2, 31, 64, 127, 128, 129, 300]))
    act = int(rng.integers(0, 3))
    c = ctx_for()
    x = rng.normal(size=(M, K)).astype(np.float32)
    W = (rng.normal(size=(N, K)) / np.sqrt(K)).astype(np.float32)
    b = rng.normal(size=N).astype(np.float32)
    y = torch.full((M, N), float("nan"), device=DEV)
    c.bls_mlp_layer(torch.from_numpy(x).to(DEV), torch.from_numpy(W).to(DEV), torch.from_numpy(b).to(DEV), act, y)
    ref, err = oracle.mlp_layer(x, W, b, act)
    assert np.all(np.abs(y.cpu().numpy() - ref) <= err), (M, K, N, act)
    T, D, B = int(rng.integers(1, 70)), int(rng.choice([1, 4, 5, 16, 24, 33, 64])), int(rng.integers(1, 12))
    ci = ctx_for(T, D, B)
    xe = rng.normal(size=(B, D)).astype(np.float32)
    emb = rng.normal(size=(B, T, D)).astype(np.float32)
    z = torch.full((B, D + T * (T + 1) // 2), float("nan"), device=DEV)
    ci.bls_interact(torch.from_numpy(xe).to(DEV), torch.from_numpy(emb).to(DEV), z)
    ci.bls_check()
    ref, err = oracle.interact(xe, emb)
    assert np.all(np.abs(z.cpu().numpy() - ref) <= err), (T, D, B)
