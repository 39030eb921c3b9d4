"""bls_plan_noalloc (the plan with its scratch in a static device array, for callers that cannot
allocate) against bls_plan, through the C ABI: every output equal bit for bit on two calls in a
row, the second on a smaller input, so that anything the first call left in the shared array
would show."""
import numpy as np
import pytest
import torch

import synth

pytestmark = pytest.mark.gpu

NAMES = ("sendcounts", "sdispls", "recvcounts", "rdispls", "ridx", "segoff", "perm")


def _plan_both(w, it, keep):
    from paper_2512_19342_amd.runner import Pipeline
    dev = torch.device("cuda:0")
    tabs = [synth.make_table(w, t).to(dev) for t in range(w.T)]
    ix, off = (x.to(dev) for x in synth.make_batch(w, it))
    nnz = int(off[-1].item())
    pipe = Pipeline(w, tabs, nnz, want_perm=True)
    c = pipe.ctx
    outs = []
    for which in ("ws", "static"):
        bufs = [torch.full_like(getattr(pipe, n), -7) for n in NAMES]      # poisoned: every word must be written
        if which == "ws":
            c.bls_plan(ix, off, nnz, *bufs, pipe.ws)
        else:
            c.bls_plan_noalloc(ix, off, nnz, *bufs)
        c.bls_check()
        outs.append([b.cpu().numpy() for b in bufs])
    keep.append((pipe, tabs))
    return nnz, outs


def test_plan_noalloc_equals_plan_on_two_calls_in_a_row():
    keep = []
    big = synth.workload(3, "small")                      # row-wise, 8 ranks, ragged bags: several scan tiles
    small = synth.custom("small", P=3, T=2, D=8, k=1, B=7, rows=[40, 9], part_kind=1, bag=("uniform", 0, 4))
    tw = synth.workload(4, "small")                       # table-wise
    sizes = []
    for w, it in ((big, 0), (small, 1), (tw, 2), (small, 3)):
        nnz, (ref, got) = _plan_both(w, it, keep)
        sizes.append(nnz)
        for name, a, b in zip(NAMES, ref, got):
            n = nnz if name in ("ridx", "perm") else a.size
            assert np.array_equal(a[:n], b[:n]), (w.name, name)
            assert not (b[:n] == -7).all() or n == 0
    assert sizes[1] < sizes[0] and sizes[3] < sizes[2]   # the second call of each pair is the smaller one


def test_plan_noalloc_refuses_what_does_not_fit():
    import paper_2512_19342_amd as B
    T, P, Bt = 4096, 8, 1 << 15                           # F*T*B = 2^30 segments: 2 MiB of block sums
    c = B.Context(P, T, 4, 1, Bt, [8] * T, [0] * T, part_kind=B.BLS_ROW_WISE)
    assert c.bls_sizes(0)["plan_ws_bytes"] > (1 << 20)
    z = torch.zeros(64, dtype=torch.int64, device="cuda")
    with pytest.raises(B.BlsError) as e:
        c.bls_plan_noalloc(z, z, 0, z, z, z, z, z, z, None)
    assert e.value.code == B.BLS_ENOSPC and "1 MiB" in c.bls_last_error()
