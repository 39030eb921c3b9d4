#!/usr/bin/env python3
"""Benchmark of the embedding-lookup hot path on one MI355X.

One step = one pass of the whole path (plan, EmbeddingBag pool, pack, ring slot, local
alltoallv, unpack) over one synthetic batch that is already resident in HBM.  Prints one
JSON line: lookups/s for the whole path, the HBM roofline of the dominant kernel (the
pool) from HIP events recorded inside the timed region, and the CPU oracle timed on a
bounded sample of the same workload on this machine's host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBPS = 8000.0          # MI355X published HBM3E peak
PEAK_L1_GBPS = 256 * 64 * 2.4   # vector L1 path: 256 compute units x 64 B per clock x 2.4 GHz

WORKLOAD_TEXT = {
    1: "cfg1: 8 tables x 10000 rows x dim 16 fp32, batch 128, pooling 1, uniform, P=2 table-wise round-robin, k=1",
    2: "cfg2: 26 tables rows log-uniform [1e3,1e5], dim 64 fp32, batch 2048, pooling 1, uniform, P=4 table-wise balanced, k=1",
    3: "cfg3: 26 tables x 1e6 rows x dim 128 fp32, batch 8192, bags U[1,40], Zipf 1.05, P=8 row-wise, k=2",
    4: "cfg4: 64 tables rows power-law [1e3,4e7] (40.5 GB fp32, dim 128), batch 16384, bags U[1,64], Zipf 1.2, "
       "8 largest tables on rank 0 of P=8 table-wise, k=4",
    6: "cfg6: the paper's heterogeneous synthetic setting: 26 tables rows log-uniform [1e3,1e6], dim 64 fp32, batch 512, "
       "bags U[1,100], uniform indices, P=8 table-wise balanced, k=2",
    5: "cfg5: 8 tables x 2e7 rows x dim 128 fp16 storage / fp32 accumulate, batch 65536, pooling 32, Zipf 1.05, "
       "P=8 row-wise, k=4",
}


def stage_bytes(w, nnz: int) -> dict:
    """Algorithmic bytes per launch of every stage (what the stage must read and write)."""
    nvec = w.F * w.T * w.B
    pv = nvec * w.D * 4
    out = w.T * w.B * w.D * 4
    seg = 8 * nvec
    return {
        "plan": 8 * nnz + 8 * (w.T * w.B + 1) + 8 * nnz + seg,
        "pool": 8 * nnz + seg + nnz * w.row_bytes + pv,
        "pack": 2 * pv,
        "exchange": 2 * pv,
        "unpack": pv + out,
    }


def recorded_traffic(cfg: int, uniform: bool = False):
    """(HBM bytes per pool launch, file) from the committed rocprofv3 counter summary of this workload
    (FETCH_SIZE and WRITE_SIZE scaled by a plain copy's readings), or None if there is none."""
    name = f"pool_stream_cfg{cfg}{'_uniform' if uniform else ''}_pmc.txt"
    try:
        m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(os.path.join(ROOT, "profiles", name)).read(), re.M)
        return (float(m.group(1)), "profiles/" + name) if m else None
    except OSError:
        return None


def pool_roofline(algorithmic_bytes: int, ms: dict, recorded) -> dict:
    """Roofline entry of the pool kernel.  achieved = algorithmic bytes per launch over the mean
    launch time between two HIP events.  When that rate is above what HBM can deliver the rows
    are coming out of the caches, and the ceiling that applies is the vector L1 path (64 B per
    clock per compute unit); the HBM side is then given by the counter traffic alone."""
    achieved = algorithmic_bytes / (ms["mean"] * 1e-3) / 1e9
    cached = achieved > PEAK_HBM_GBPS
    peak = PEAK_L1_GBPS if cached else PEAK_HBM_GBPS
    traffic, src = recorded if recorded else (None, None)
    r = {"bound": "l1" if cached else "hbm", "kernel": "pool_stream (bls_embbag_pool)", "achieved": achieved, "peak": peak,
         "unit": "GB/s", "frac": achieved / peak, "traffic": traffic, "traffic_source": src,
         "algorithmic_bytes_per_launch": algorithmic_bytes, "avg_launch_ms": ms["mean"],
         "median_launch_ms": ms["median"], "min_launch_ms": ms["min"],
         "peak_note": ("vector L1 path: 256 compute units x 64 B per clock x 2.4 GHz; the algorithmic rate is above the "
                       "8 TB/s HBM peak because popular rows are served by L1 and L2") if cached else "MI355X HBM3E peak"}
    if traffic is not None:
        r["hbm_traffic_gbps"] = traffic / (ms["mean"] * 1e-3) / 1e9
        r["hbm_traffic_frac_of_peak"] = r["hbm_traffic_gbps"] / PEAK_HBM_GBPS
        r["algorithmic_over_traffic"] = algorithmic_bytes / traffic
    return r


def cpu_baseline(w, tabs_gpu, batches, budget_s: float) -> dict:
    """The oracle, as it stands and single-threaded, over whole batches of the same workload
    (all tables at full size, copied to the host) until about `budget_s` seconds are spent."""
    import oracle
    tabs = [t.cpu().numpy() for t in tabs_gpu]
    case = oracle.Case(w.P, w.T, w.D, w.B, w.part_kind, w.rows, w.table_owner, w.dtype_code)
    spent, nnz, n = 0.0, 0, 0
    while spent < budget_s and n < 64:
        ix, off = (x.cpu().numpy() for x in batches[n % len(batches)])
        t0 = time.perf_counter()
        oracle.pipeline(case, tabs, ix, off)
        spent += time.perf_counter() - t0
        nnz += int(off[-1])
        n += 1
    return {"value": nnz / spent, "unit": "lookups/s", "cores": 1, "kind": "oracle", "seconds": round(spent, 3),
            "sample": f"{n} whole batches ({nnz} lookups) through the oracle's plan, pool, pack, alltoallv and "
                      f"unpack, all {w.T} tables at full size on the host"}


def dense_section(args, w, pipe, batches, nnzs, note) -> dict:
    """The model around the lookup (bottom MLP, dot interaction, top MLP) at the workload's batch:
    every kernel timed with events, then Listing 2's loop (lookup + model per iteration)."""
    import torch

    import synth
    from paper_2512_19342_amd.runner import BlsDlrm, DenseModel
    dev = pipe.dev
    bs, ts = synth.mlp_sizes(w, "full")
    bot = [(W.to(dev), b.to(dev)) for W, b in synth.mlp_weights(w, bs, 0)]
    top = [(W.to(dev), b.to(dev)) for W, b in synth.mlp_weights(w, ts, 1)]
    model = DenseModel(pipe.ctx, bot, top, w.B)
    dense = [synth.dense_features(w, i, dev) for i in range(2)]
    emb = pipe.new_out().normal_(0.0, 0.1)
    c = pipe.ctx
    names = [f"bottom {K}->{N}" for K, N in zip(bs[:-1], bs[1:])] + ["interact"] + [f"top {K}->{N}" for K, N in zip(ts[:-1], ts[1:])]
    flops = [2.0 * w.B * K * N for K, N in zip(bs[:-1], bs[1:])] + [2.0 * w.B * w.D * w.T * (w.T + 1) / 2] + \
            [2.0 * w.B * K * N for K, N in zip(ts[:-1], ts[1:])]

    def model_step(i: int, ev=None):
        a, k = dense[i % 2], 0
        for (W, b), y in zip(model.bottom, model.bot_act):
            if ev: ev[k].record()
            c.bls_mlp_layer(a, W, b, 1, y)
            a, k = y, k + 1
        if ev: ev[k].record()
        c.bls_interact(a, emb, model.z)
        a, k = model.z, k + 1
        for j, ((W, b), y) in enumerate(zip(model.top, model.top_act)):
            if ev: ev[k].record()
            c.bls_mlp_layer(a, W, b, 2 if j == len(model.top) - 1 else 1, y)
            a, k = y, k + 1
        if ev: ev[k].record()

    for i in range(args.warmup):
        model_step(i)
    n = len(names)
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(n + 1)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    for i in range(args.steps):
        model_step(i, events[i])
    torch.cuda.synchronize()
    ms = [sum(e[k].elapsed_time(e[k + 1]) for e in events) / args.steps for k in range(n)]
    kernels = {nm: {"ms": m, "tflops": f / (m * 1e-3) / 1e12} for nm, m, f in zip(names, ms, flops)}
    big = max(range(n), key=lambda k: flops[k] if names[k] != "interact" else 0.0)
    note(f"dense model: {sum(ms):.3f} ms per batch; {names[big]}: {ms[big]:.3f} ms, {kernels[names[big]]['tflops']:.1f} TFLOP/s")

    # the vendor library's fp32 GEMM on the largest layer's shape (no bias, no activation), for scale
    Wb, xb = model.top[big - len(bs)][0] if big >= len(bs) else model.bottom[big][0], None
    xb = model.z if big == len(bs) else (model.top_act[big - len(bs) - 1] if big > len(bs) else dense[0])
    lib_ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    yb = torch.empty((xb.shape[0], Wb.shape[0]), dtype=torch.float32, device=dev)
    for _ in range(2):
        torch.mm(xb, Wb.t(), out=yb)
    lib_ev[0].record()
    for _ in range(5):
        torch.mm(xb, Wb.t(), out=yb)
    lib_ev[1].record()
    torch.cuda.synchronize()
    lib_tflops = flops[big] / (lib_ev[0].elapsed_time(lib_ev[1]) / 5 * 1e-3) / 1e12
    note(f"torch.mm (rocBLAS / hipBLASLt) on the same shape: {lib_tflops:.1f} TFLOP/s")

    # Listing 2's loop: lookup (fused owner side) + bottom MLP per call, completion + prediction k calls later
    loops = {}
    side = torch.cuda.Stream()
    for fused_completion, two_streams in ((False, False), (True, False), (True, True)):
        loop = BlsDlrm(pipe, model, fused_completion=fused_completion, lookup_stream=side if two_streams else None)
        torch.cuda.synchronize()
        for i in range(args.warmup):
            loop.forward(dense[i % 2], *batches[i % len(batches)], nnzs[i % len(batches)], last_batch=i == args.warmup - 1)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        done = 0
        for i in range(args.steps):
            done += len(loop.forward(dense[i % 2], *batches[i % len(batches)], nnzs[i % len(batches)], last_batch=i == args.steps - 1))
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        c.bls_check()
        assert done == args.steps
        what = "completion folded into the interaction" if fused_completion else "copy-out, then interaction"
        what += ", lookups on a second stream" if two_streams else ""
        note(f"{args.steps} iterations of the model loop ({what}): {dt / args.steps * 1e3:.3f} ms per iteration")
        loops[("folded_completion_two_streams" if two_streams else "folded_completion") if fused_completion else "staged_completion"] = {
            "ms_per_iteration": dt / args.steps * 1e3, "samples_per_s": w.B * args.steps / dt}
    mm = [k for k in range(n) if names[k] != "interact"]
    return {"layers": {"bottom": bs, "top": ts}, "kernels": kernels, "dense_ms_per_batch": sum(ms),
            "library_gemm_tflops_same_shape": lib_tflops,
            "mlp_tflops": sum(flops[k] for k in mm) / (sum(ms[k] for k in mm) * 1e-3) / 1e12,
            "mfma_roofline": {"bound": "mfma", "kernel": f"mlp_gemm ({names[big]})", "achieved": kernels[names[big]]["tflops"],
                              "peak": 157.3, "unit": "TFLOP/s", "frac": kernels[names[big]]["tflops"] / 157.3},
            "loop": {"entry_points": "bls_plan + bls_embbag_pool_put + bls_mlp_layer x3 | bls_unpack + bls_interact "
                                     "(or bls_unpack_interact) + bls_mlp_layer x5", "bound": w.k, **loops}}


def alltoallv_demo(args) -> int:
    """The paper's two alltoallv microbenchmarks (Results, Alltoallv benchmarks) for the device-local
    exchange with k = 0: (a) one collective (slot acquire, exchange, completion copy-out) for equal
    message sizes per rank from 32 B to 256 MiB, (b) 1 .. 100 000 collectives in sequence at 32 KiB per
    rank.  P = 8 ranks, one table per rank, so a rank sends B*D*4 bytes in all."""
    import torch

    import paper_2512_19342_amd as A
    dev = torch.device("cuda:0")
    P = 8

    def make(per_rank_bytes: int):
        D = 128 if per_rank_bytes >= 4096 else 1
        B = max(P, per_rank_bytes // (4 * D))
        c = A.Context(P, P, D, 0, B, [1] * P, list(range(P)))
        tabs = [torch.zeros((1, D), dtype=torch.float32, device=dev) for _ in range(P)]
        for t in range(P):
            c.bls_set_shard(t, t, tabs[t])
        c.bls_commit(torch.empty(c.bls_desc_bytes(), dtype=torch.uint8, device=dev))
        n = P * B * D
        send = torch.rand(n, dtype=torch.float32, device=dev)
        slot = torch.empty(n, dtype=torch.float32, device=dev)
        out = torch.empty((B, P, D), dtype=torch.float32, device=dev)
        c.bls_set_ring(slot)
        return c, send, out, B * D * 4, tabs

    def collective(c, send, out):
        it, slot = c.bls_ring_advance()
        c.bls_alltoallv_local(send, slot)
        c.bls_unpack(it, out)

    sizes, rows_a = [32 << i for i in range(0, 24)], []          # 32 B .. 256 MiB per rank
    for sz in sizes:
        c, send, out, actual, _keep = make(sz)
        for _ in range(3):
            collective(c, send, out)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        reps = 20
        torch.cuda.synchronize()
        ev[0].record()
        for _ in range(reps):
            collective(c, send, out)
        ev[1].record()
        torch.cuda.synchronize()
        c.bls_check()
        us = ev[0].elapsed_time(ev[1]) / reps * 1e3
        # bytes moved: exchange reads and writes all P messages, the copy-out reads and writes them again
        rows_a.append({"bytes_per_rank": actual, "us_per_collective": us, "GBps_moved": 4 * P * actual / (us * 1e-6) / 1e9})
        print(f"[a2a] {actual:>10d} B per rank: {us:9.2f} us", file=sys.stderr, flush=True)
        del c, send, out, _keep

    rows_b = []
    c, send, out, actual, _keep = make(32 * 1024)
    for _ in range(10):
        collective(c, send, out)
    torch.cuda.synchronize()
    for reps in (1, 10, 100, 1000, 10000, 100000):
        t0 = time.perf_counter()
        for _ in range(reps):
            collective(c, send, out)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        c.bls_check()
        rows_b.append({"collectives": reps, "seconds": dt, "us_per_collective": dt / reps * 1e6})
        print(f"[a2a] {reps:>6d} collectives of {actual} B per rank: {dt:.4f} s ({dt / reps * 1e6:.2f} us each)",
              file=sys.stderr, flush=True)
    print(json.dumps({"experiment": "device-local alltoallv microbenchmarks, k = 0 (the paper's message-size and repetition sweeps)",
                      "ranks": P, "entry_points": "bls_ring_advance + bls_alltoallv_local + bls_unpack",
                      "message_size_sweep": rows_a, "repetition_sweep_32KiB_per_rank": rows_b}))
    return 0


def lag_demo(args) -> int:
    """The paper's Setting 2 on one GPU: every simulated rank on its own stream, a uniformly random
    delay before each rank's work in every iteration, bound k swept.  With k = 0 every iteration
    costs the slowest rank's delay; with k > 0 ranks run ahead and the delays average out."""
    import numpy as np
    import torch

    import synth
    from paper_2512_19342_amd.runner import BlsDlrmRanks, DenseModel, Pipeline
    dev = torch.device("cuda:0")
    base = synth.workload(args.config, args.size)
    tabs = [synth.make_table(base, t, dev) for t in range(base.T)]
    N, P = args.steps, base.P
    if args.with_model:                                    # the dense model around every rank's lookup
        bs, ts = synth.mlp_sizes(base, "full")
        bot = [(W.to(dev), b.to(dev)) for W, b in synth.mlp_weights(base, bs, 0)]
        top = [(W.to(dev), b.to(dev)) for W, b in synth.mlp_weights(base, ts, 1)]
        dense = [synth.dense_features(base, i, dev) for i in range(4)]
    batches = [synth.make_batch(base, it, dev) for it in range(N)]
    nnzs = [int(off[-1].item()) for _, off in batches]
    delays = np.random.default_rng(2512).integers(0, args.max_delay_us + 1, size=(N, P))
    rows = []
    for n_cfg, k in enumerate([args.bounds[0]] + list(args.bounds)):   # the first pass only warms the device up
        w = synth.workload(args.config, args.size)
        w.k = k
        pipe = Pipeline(w, tabs, max(nnzs))
        c, K = pipe.ctx, max(k, 1)
        plans = []
        for (ix, off), nnz in zip(batches, nnzs):          # data and plans are prepared before timing
            c.bls_plan(ix, off, nnz, pipe.sendcounts, pipe.sdispls, pipe.recvcounts, pipe.rdispls,
                       pipe.ridx, pipe.segoff, None, pipe.ws)
            plans.append((pipe.ridx[:max(nnz, 1)].clone(), pipe.segoff.clone(), nnz))
        outs = [pipe.new_out() for _ in range(K)]
        streams = [torch.cuda.Stream() for _ in range(P)]
        ranks = BlsDlrmRanks(pipe, DenseModel(c, bot, top, w.B), streams) if args.with_model else None
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(P)]
        for with_delay in (None, False, True):           # None: an untimed warm-up pass without delays
            torch.cuda.synchronize()
            for r in range(P):
                ev[r][0].record(streams[r])
            t0 = time.perf_counter()
            first = getattr(pipe, "_lag_iter", 0)       # per-rank iteration numbers keep counting
            for j in range(N):
                it = first + j
                if j >= K:
                    for s in range(P):
                        if ranks: ranks.finish(s, it - K)
                        else: c.bls_rank_complete(s, it - K, None, outs[(it - K) % K], streams[s])
                for d in range(P):
                    dly = int(delays[j, d]) if with_delay else 0
                    if ranks:
                        ranks.issue(d, it, *plans[j], dense[j % 4], delay_us=dly)
                        continue
                    if dly:
                        c.bls_rank_delay(dly, streams[d])
                    c.bls_rank_put(d, plans[j][0], None, plans[j][1], plans[j][2], it, streams[d])
            for j in range(max(N - K, 0), N):
                for s in range(P):
                    if ranks: ranks.finish(s, first + j)
                    else: c.bls_rank_complete(s, first + j, None, outs[(first + j) % K], streams[s])
            t_host = time.perf_counter() - t0
            for r in range(P):
                ev[r][1].record(streams[r])
            torch.cuda.synchronize()
            pipe._lag_iter = first + N
            c.bls_check()
            per_rank = [ev[r][0].elapsed_time(ev[r][1]) / N for r in range(P)]
            if with_delay is None or n_cfg == 0:
                continue
            rows.append({"k": k, "delays": with_delay, "latency_ms_per_iteration_mean_over_ranks": sum(per_rank) / P,
                         "iterations_per_s_sum_over_ranks": sum(1e3 / x for x in per_rank),
                         "host_enqueue_ms_per_iteration": t_host / N * 1e3})
            print(f"[lag] k={k} delays={'U(0,%d us)' % args.max_delay_us if with_delay else 'none'}: "
                  f"{rows[-1]['latency_ms_per_iteration_mean_over_ranks']:.4f} ms per iteration per rank "
                  f"(host enqueue {rows[-1]['host_enqueue_ms_per_iteration']:.4f})", file=sys.stderr, flush=True)
        del pipe
    print(json.dumps({"experiment": "per-rank streams with injected delays (the paper's Setting 2 on one GPU)",
                      "workload": WORKLOAD_TEXT[args.config], "iterations": N, "ranks": P,
                      "model": "bottom MLP, interaction and top MLP per rank (Listing 2)" if args.with_model else "lookup only",
                      "max_delay_us": args.max_delay_us, "mean_delay_ms": args.max_delay_us / 2e3,
                      "expected_max_of_P_delays_ms": args.max_delay_us * P / (P + 1) / 1e3, "results": rows}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=4, help="benchmark workload 1..6 (default 4, the target)")
    ap.add_argument("--size", default="full", choices=["full", "small"])
    ap.add_argument("--batches", type=int, default=16, help="distinct pre-generated batches, rotated")
    ap.add_argument("--no-uniform-control", action="store_true", help="skip the uniform-index control run")
    ap.add_argument("--flat-control", action=argparse.BooleanOptionalAction, default=True,
                    help="with the uniform-index control: also the run with equal-size tables (regenerates the tables)")
    ap.add_argument("--hot-rows", type=int, default=0,
                    help="name this many popular rows per shard (counted on a batch that is not among the timed ones): "
                         "the pooling kernels keep them in LDS (bls_set_hot_rows)")
    ap.add_argument("--flat-rows", action="store_true",
                    help="experiment: every table gets the same number of rows (same total), so that uniform indices leave "
                         "no small table for the caches to hold")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="CPU time to spend on the oracle baseline")
    ap.add_argument("--index-dist", default=None, choices=[None, "uniform"],
                    help="cache-defeating control: uniform indices instead of the workload's law")
    ap.add_argument("--timed-only", action="store_true",
                    help="only the warm-up and the timed staged steps (for profiler runs: no fused, ring or copy sections)")
    ap.add_argument("--lag-demo", action="store_true",
                    help="instead of the benchmark: per-rank streams with random delays, bound k swept "
                         "(use a workload with P <= 4, e.g. --config 2: a process has 4 hardware queues here, "
                         "more streams than that share queues and serialise)")
    ap.add_argument("--alltoallv-demo", action="store_true",
                    help="instead of the benchmark: the paper's alltoallv microbenchmarks for the device-local exchange")
    ap.add_argument("--with-model", action="store_true",
                    help="with --lag-demo: every rank also runs the bottom MLP, the interaction and the top MLP of its mini-batch")
    ap.add_argument("--max-delay-us", type=int, default=1000)
    ap.add_argument("--bounds", type=int, nargs="+", default=[0, 1, 2, 4, 8])
    ap.add_argument("--table-dtype", default=None, choices=[None, "fp32", "fp16", "u8rq", "f8rq"],
                    help="variant: store the tables this way instead of the workload's own dtype")
    ap.add_argument("--dense", action="store_true", help="with --timed-only: also time the dense model around the lookup")
    ap.add_argument("--rows-cap", type=int, default=0, help="experiment: no table has more rows than this")
    ap.add_argument("--bag-fixed", type=int, default=0, help="experiment: every bag has this many lookups")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs the path on one GPU (P simulated ranks live in its memory); "
              "--gpus above 1 is not supported", file=sys.stderr)
        return 2

    import torch

    import synth
    from paper_2512_19342_amd.runner import Pipeline

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    if args.lag_demo:
        return lag_demo(args)
    if args.alltoallv_demo:
        return alltoallv_demo(args)
    dev = torch.device("cuda:0")
    w = synth.workload(args.config, args.size)
    if args.index_dist == "uniform":
        w.index_dist = ("uniform",)
    if args.bag_fixed:
        w.bag = ("fixed", args.bag_fixed)
    if args.table_dtype:
        w.table_dtype = args.table_dtype
    if args.rows_cap:
        w.rows = [min(r, args.rows_cap) for r in w.rows]
    if args.flat_rows:
        w.rows = [sum(w.rows) // w.T] * w.T
    def note(msg: str):
        print(f"[bench] {msg}", file=sys.stderr, flush=True)

    t_setup = time.perf_counter()
    tabs = [synth.make_table(w, t, dev) for t in range(w.T)]
    torch.cuda.synchronize()
    note(f"{w.T} tables ({w.table_bytes() / 1e9:.1f} GB) generated on the device")
    batches = [synth.make_batch(w, it, dev) for it in range(args.batches)]
    torch.cuda.synchronize()
    note(f"{args.batches} batches generated")
    w._cdf_cache.clear()
    nnzs = [int(off[-1].item()) for _, off in batches]
    pipe = Pipeline(w, tabs, max(nnzs))
    out = pipe.new_out()
    if args.hot_rows:                                      # traffic statistics from a batch of its own
        sx, so = synth.make_batch(w, args.batches + 1000, dev)
        pipe.set_hot_rows(pipe.hot_rows_from_batch(sx, so.cpu(), args.hot_rows))
        del sx, so
        w._cdf_cache.clear()
    torch.cuda.synchronize()
    t_setup = time.perf_counter() - t_setup
    c = pipe.ctx
    names = ["plan", "pool", "pack", "exchange", "unpack"]

    def timed_run(bts, nz, steps: int, warmup: int, pipe=pipe, out=out) -> dict:
        """`warmup` untimed and `steps` timed staged steps over the batches `bts`, with HIP events on the
        launch stream around the pool launch of every timed step (the roofline's launch duration); then the
        same steps once more with events around every stage, for the per-stage figures.  Six events per step
        cost the step 23 us on workload 4, which is why the timed steps carry only two."""
        c = pipe.ctx

        def one_step(i: int, ev=None, pool_ev=None):
            ix, off = bts[i % len(bts)]
            nnz = nz[i % len(bts)]
            if ev: ev[0].record()
            c.bls_plan(ix, off, nnz, pipe.sendcounts, pipe.sdispls, pipe.recvcounts, pipe.rdispls,
                       pipe.ridx, pipe.segoff, None, pipe.ws)
            if ev: ev[1].record()
            if pool_ev: pool_ev[0].record()
            c.bls_embbag_pool(pipe.ridx, pipe.segoff, nnz, pipe.pooled)
            if pool_ev: pool_ev[1].record()
            if ev: ev[2].record()
            c.bls_pack(pipe.pooled, pipe.send)
            if ev: ev[3].record()
            it, slot = c.bls_ring_advance()
            c.bls_alltoallv_local(pipe.send, slot)
            if ev: ev[4].record()
            c.bls_unpack(it, out)
            if ev: ev[5].record()
            return nnz

        for i in range(warmup):
            one_step(i)
        c.bls_check()
        pool_events = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        lookups = 0
        for i in range(steps):
            lookups += one_step(warmup + i, None, pool_events[i])
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        c.bls_check()
        events = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(steps)]
        for i in range(steps):
            one_step(warmup + i, events[i])
        torch.cuda.synchronize()
        c.bls_check()
        per_stage = {n: [e[k].elapsed_time(e[k + 1]) for e in events] for k, n in enumerate(names)}
        per_stage["pool"] = [e[0].elapsed_time(e[1]) for e in pool_events]      # from the timed steps themselves
        per_step = [e[0].elapsed_time(e[5]) for e in events]
        stat = lambda v: {"mean": statistics.fmean(v), "median": statistics.median(v), "min": min(v)}
        return {"dt": dt, "lookups": lookups, "stage_ms": {n: statistics.fmean(v) for n, v in per_stage.items()},
                "stage_ms_stats": {n: stat(v) for n, v in per_stage.items()}, "step_ms_stats": stat(per_step)}

    run = timed_run(batches, nnzs, args.steps, args.warmup)
    dt, lookups = run["dt"], run["lookups"]
    note(f"{args.steps} timed steps: {dt / args.steps * 1e3:.3f} ms per step")

    def one_step(i: int):
        ix, off = batches[i % len(batches)]
        nnz = nnzs[i % len(batches)]
        c.bls_plan(ix, off, nnz, pipe.sendcounts, pipe.sdispls, pipe.recvcounts, pipe.rdispls,
                   pipe.ridx, pipe.segoff, None, pipe.ws)
        c.bls_embbag_pool(pipe.ridx, pipe.segoff, nnz, pipe.pooled)
        c.bls_pack(pipe.pooled, pipe.send)
        it, slot = c.bls_ring_advance()
        c.bls_alltoallv_local(pipe.send, slot)
        c.bls_unpack(it, out)
        return nnz

    copy_gbps = dtf = dtr = fused_lookups = None
    if not args.timed_only:
        # achievable ceiling for the permute stages: a plain device copy of one pooled buffer
        cp = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        pipe.send.copy_(pipe.pooled)
        cp[0].record()
        for _ in range(10):
            pipe.send.copy_(pipe.pooled)
        cp[1].record()
        torch.cuda.synchronize()
        copy_gbps = 2 * pipe.pooled.numel() * 4 / (cp[0].elapsed_time(cp[1]) / 10 * 1e-3) / 1e9

        # the same work with the owner side fused (bls_embbag_pool_put: no pooled or send buffer);
        # reported beside the staged path, never as `value`
        def fused_step(i: int):
            ix, off = batches[i % len(batches)]
            nnz = nnzs[i % len(batches)]
            c.bls_plan(ix, off, nnz, pipe.sendcounts, pipe.sdispls, pipe.recvcounts, pipe.rdispls,
                       pipe.ridx, pipe.segoff, None, pipe.ws)
            it, slot = c.bls_ring_advance()
            c.bls_embbag_pool_put(pipe.ridx, pipe.segoff, nnz, slot)
            c.bls_unpack(it, out)
            return nnz

        for i in range(args.warmup):
            fused_step(i)
        torch.cuda.synchronize()
        tf = time.perf_counter()
        fused_lookups = 0
        for i in range(args.steps):
            fused_lookups += fused_step(args.warmup + i)
        torch.cuda.synchronize()
        dtf = time.perf_counter() - tf
        c.bls_check()
        note(f"{args.steps} fused steps: {dtf / args.steps * 1e3:.3f} ms per step")

        # the ring at work: K-1 iterations stay in flight, completion runs on a second stream
        side = torch.cuda.Stream()
        outs = [pipe.new_out() for _ in range(c.K)]

        def issue(i: int):
            ix, off = batches[i % len(batches)]
            nnz = nnzs[i % len(batches)]
            c.bls_plan(ix, off, nnz, pipe.sendcounts, pipe.sdispls, pipe.recvcounts, pipe.rdispls,
                       pipe.ridx, pipe.segoff, None, pipe.ws)
            c.bls_embbag_pool(pipe.ridx, pipe.segoff, nnz, pipe.pooled)
            c.bls_pack(pipe.pooled, pipe.send)
            it, slot = c.bls_ring_advance()
            c.bls_alltoallv_local(pipe.send, slot)
            return it

        torch.cuda.synchronize()
        tr = time.perf_counter()
        flying = []
        for i in range(args.steps):
            if len(flying) == c.K:
                j = flying.pop(0)
                c.bls_unpack(j, outs[j % c.K], side)
            flying.append(issue(i))
        for j in flying:
            c.bls_unpack(j, outs[j % c.K], side)
        torch.cuda.synchronize()
        dtr = time.perf_counter() - tr
        c.bls_check()
        note(f"{args.steps} steps with up to {c.K} iterations in flight: {dtr / args.steps * 1e3:.3f} ms per step")

    # table-wise partitions: the whole iteration in one launch (bls_step_tablewise); beside `value`, never in it
    one = None
    if w.part_kind == 0 and not args.timed_only:
        try:
            for i in range(args.warmup):
                pipe.step_one_launch(*batches[i % len(batches)], nnzs[i % len(batches)], out)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            done = 0
            for i in range(args.steps):
                k = (args.warmup + i) % len(batches)
                pipe.step_one_launch(*batches[k], nnzs[k], out)
                done += nnzs[k]
            torch.cuda.synchronize()
            d1 = time.perf_counter() - t1
            c.bls_check()
            one = {"entry_point": "bls_step_tablewise", "ms_per_step": d1 / args.steps * 1e3, "lookups_per_s": done / d1}
            note(f"{args.steps} one-launch steps: {one['ms_per_step']:.4f} ms per step")
        except Exception as e:                              # a shape the one-launch kernel does not take
            one = {"entry_point": "bls_step_tablewise", "refused": str(e)}

    dlrm = None
    if not args.timed_only or args.dense:
        dlrm = dense_section(args, w, pipe, batches, nnzs, note)

    stage_ms = run["stage_ms"]
    mean_nnz = lookups / args.steps
    sb = stage_bytes(w, int(mean_nnz))
    a_staged = sum(sb.values())
    pool_pack_gbps = (sb["pool"] + sb["pack"]) / ((stage_ms["pool"] + stage_ms["pack"]) * 1e-3) / 1e9
    plain = args.size == "full" and not args.table_dtype and not args.bag_fixed and not args.rows_cap and not args.flat_rows and not args.hot_rows
    roofline = pool_roofline(sb["pool"], run["stage_ms_stats"]["pool"],
                             recorded_traffic(args.config, uniform=bool(args.index_dist)) if plain else None)

    # the rows one batch touches at least once: what an infinite cache would still have to fetch
    if not args.timed_only:
        ix0, off0 = batches[0]
        distinct = 0
        for t in range(w.T):
            distinct += int(torch.unique(ix0[int(off0[t * w.B]):int(off0[(t + 1) * w.B])]).numel())
        row_bytes = w.row_bytes
        roofline["distinct_rows_per_batch"] = distinct
        roofline["compulsory_row_bytes"] = distinct * row_bytes
        roofline["compulsory_over_row_bytes"] = distinct / max(1, nnzs[0])

    # cache-defeating control: the same tables and bag lengths with uniform indices, the same staged step
    control = None
    if w.index_dist[0] == "zipf" and not args.timed_only and not args.no_uniform_control:
        wu = synth.workload(args.config, args.size)
        wu.rows, wu.table_dtype, wu.bag, wu.index_dist = w.rows, w.table_dtype, w.bag, ("uniform",)
        ub = [synth.make_batch(wu, it, dev) for it in range(args.batches)]
        un = [int(off[-1].item()) for _, off in ub]
        urun = timed_run(ub, un, args.steps, args.warmup)
        usb = stage_bytes(w, int(urun["lookups"] / args.steps))
        ums = urun["stage_ms"]
        control = {
            "what": "the same tables, bag lengths and staged step with uniform indices: no popular rows for the caches to hold",
            "ms_per_step": urun["dt"] / args.steps * 1e3, "lookups_per_s": urun["lookups"] / urun["dt"],
            "stage_ms": ums, "stage_ms_stats": urun["stage_ms_stats"],
            "roofline": pool_roofline(usb["pool"], urun["stage_ms_stats"]["pool"],
                                      recorded_traffic(args.config, uniform=True) if plain else None),
            "pool_plus_pack_gbps": (usb["pool"] + usb["pack"]) / ((ums["pool"] + ums["pack"]) * 1e-3) / 1e9,
        }
        control["pool_plus_pack_frac_of_hbm_peak"] = control["pool_plus_pack_gbps"] / PEAK_HBM_GBPS
        note(f"uniform-index control: {control['ms_per_step']:.3f} ms per step, pool {ums['pool']:.3f} ms = "
             f"{control['roofline']['achieved']:.0f} GB/s of algorithmic bytes")
        del ub
        # the same again with every table the same size (same total): under uniform indices no table is
        # then small enough for L2 or the memory-side cache to hold, every row comes from HBM
        if args.flat_control and plain and len(set(w.rows)) > 1:
            wf = synth.workload(args.config, args.size)
            wf.rows, wf.index_dist = [sum(w.rows) // w.T] * w.T, ("uniform",)
            ftabs = [synth.make_table(wf, t, dev) for t in range(wf.T)]
            fb = [synth.make_batch(wf, it, dev) for it in range(min(args.batches, 8))]
            fn = [int(off[-1].item()) for _, off in fb]
            fpipe = Pipeline(wf, ftabs, max(fn))
            frun = timed_run(fb, fn, args.steps, args.warmup, fpipe, fpipe.new_out())
            fsb = stage_bytes(wf, int(frun["lookups"] / args.steps))
            fms = frun["stage_ms"]
            control["equal_tables"] = {
                "what": f"{wf.T} tables of {wf.rows[0]} rows each ({wf.table_bytes() / 1e9:.1f} GB), uniform indices: every row from HBM",
                "ms_per_step": frun["dt"] / args.steps * 1e3, "stage_ms": fms,
                "roofline": pool_roofline(fsb["pool"], frun["stage_ms_stats"]["pool"], None),
                "pool_plus_pack_gbps": (fsb["pool"] + fsb["pack"]) / ((fms["pool"] + fms["pack"]) * 1e-3) / 1e9,
            }
            control["equal_tables"]["pool_plus_pack_frac_of_hbm_peak"] = control["equal_tables"]["pool_plus_pack_gbps"] / PEAK_HBM_GBPS
            note(f"equal-size tables, uniform indices: pool {fms['pool']:.3f} ms = "
                 f"{control['equal_tables']['roofline']['achieved']:.0f} GB/s of algorithmic bytes")
            del fpipe, ftabs, fb

    # the other end: the same bags over tables of sixteen rows each, which every compute unit's L1 holds whole.
    # What the pooling kernel reaches there is the rate of the vector memory path for its load shape, measured:
    # the ceiling that applies when popular rows are served by the caches.
    if w.index_dist[0] == "zipf" and not args.timed_only and not args.no_uniform_control and plain:
        wl = synth.workload(args.config, args.size)
        wl.rows = [16] * w.T
        ltabs = [synth.make_table(wl, t, dev) for t in range(wl.T)]
        lb = [synth.make_batch(wl, it, dev) for it in range(min(args.batches, 8))]
        ln = [int(off[-1].item()) for _, off in lb]
        lpipe = Pipeline(wl, ltabs, max(ln))
        lrun = timed_run(lb, ln, args.steps, args.warmup, lpipe, lpipe.new_out())
        lsb = stage_bytes(wl, int(lrun["lookups"] / args.steps))
        lms = lrun["stage_ms_stats"]["pool"]
        roofline["l1_resident_control"] = {
            "what": f"the same bags over {wl.T} tables of 16 rows: every row in every compute unit's L1",
            "pool_ms": lms["mean"], "pool_ms_median": lms["median"], "pool_ms_min": lms["min"],
            "achieved": lsb["pool"] / (lms["mean"] * 1e-3) / 1e9, "unit": "GB/s",
        }
        roofline["frac_of_l1_resident_rate"] = roofline["achieved"] / roofline["l1_resident_control"]["achieved"]
        note(f"L1-resident control: pool {lms['mean']:.3f} ms = {roofline['l1_resident_control']['achieved']:.0f} GB/s of algorithmic bytes; "
             f"the workload's pool runs at {roofline['frac_of_l1_resident_rate']:.2f} of that")
        del lpipe, ltabs, lb

    res = {
        "metric": "embedding lookups/sec + achieved HBM GB/s (bucket+pool+pack), 1 MI355X",
        "value": lookups / dt, "unit": "lookups/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt / args.steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"fp32": "f32", "fp16": "f16 storage, f32 accumulate",
                  "u8rq": "u8 row-quantised storage, f32 accumulate",
                  "f8rq": "e4m3 row-quantised storage, f32 accumulate"}[w.table_dtype], "data": "synthetic",
        "config": {"workload": WORKLOAD_TEXT[args.config] + ("" if args.size == "full" else " [reduced twin]")
                   + (" [uniform-index control]" if args.index_dist else "")
                   + (f" [every bag {args.bag_fixed} lookups]" if args.bag_fixed else "")
                   + (f" [tables capped at {args.rows_cap} rows]" if args.rows_cap else "")
                   + (" [all tables the same size]" if args.flat_rows else "")
                   + (f" [{args.hot_rows} popular rows per shard named]" if args.hot_rows else "")
                   + (f" [tables stored as {args.table_dtype}]" if args.table_dtype else ""),
                   "P": w.P, "T": w.T, "D": w.D, "B": w.B, "k": w.k, "lookups_per_step": mean_nnz,
                   "table_bytes": w.table_bytes(), "distinct_batches": args.batches},
        "roofline": roofline,
        "uniform_control": control,
        "step_ms_stats": run["step_ms_stats"],
        "hbm_gbps": {"note": "algorithmic bytes over time; above the HBM peak when popular rows are served by L1 / L2",
                     "whole_path_staged": a_staged / (dt / args.steps) / 1e9, "pool_plus_pack": pool_pack_gbps,
                     "pool_plus_pack_over_hbm_peak": pool_pack_gbps / PEAK_HBM_GBPS},
        "stage_ms": stage_ms,
        "stage_ms_stats": run["stage_ms_stats"],
        "stage_gbps": {n: sb[n] / (stage_ms[n] * 1e-3) / 1e9 for n in names},
        "fused_owner_side": None if dtf is None else {
            "entry_point": "bls_plan + bls_embbag_pool_put + bls_unpack", "ms_per_step": dtf / args.steps * 1e3,
            "lookups_per_s": fused_lookups / dtf},
        "one_launch_step": one,
        "ring_in_flight": None if dtr is None else {
            "K": c.K, "ms_per_step": dtr / args.steps * 1e3,
            "note": "staged path, completion deferred K-1 iterations on a second stream"},
        "dlrm_model": dlrm,
        "bucket_pool_pack": {"ms": stage_ms["plan"] + stage_ms["pool"] + stage_ms["pack"],
                             "lookups_per_s": mean_nnz / ((stage_ms["plan"] + stage_ms["pool"] + stage_ms["pack"]) * 1e-3)},
        "plain_copy_gbps": copy_gbps,
        "setup_s": round(t_setup, 2),
    }
    if not args.no_cpu_baseline:
        note("timing the CPU oracle on the host")
        res["cpu_baseline"] = cpu_baseline(w, tabs, batches, args.cpu_seconds)
    print(json.dumps(res))
    return 0


if __name__ == "__main__":
    sys.exit(main())
