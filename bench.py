#!/usr/bin/env python3
"""Benchmark of the GNND build on one MI355X.

Workload: n = 1,000,000 float32 vectors, d = 128, SIFT-shaped synthetic mixture
(a stand-in for SIFT1M, which is not available), k = 32, p = 32, squared L2.
A step is one complete build: random initial graph plus T iterations of
sampling, cross-matching and list update, where T is the first iteration after
which Recall@10 (on a seeded sample of nodes, against exhaustive search) is at
least 0.95; T is found in an untimed calibration build, then K builds are timed
with the vectors resident in HBM.  Prints one JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0
PEAK_FP32_TFLOPS = 157.3
PEAK_INT8_TOPS = 5000.0

# HBM-side traffic of the join kernel on the default workload, from rocprofv3
# --pmc FETCH_SIZE / WRITE_SIZE (profiles/gnnd_build_sift1m_d128_k32.md): raw counter
# MiB of every launch of one build (iteration 1, 2, ...), and the factors by which the
# same counters misread a 1 GiB device copy.  Keyed by (workload, n, d, k, p, join
# kernel): any other run reports "traffic": null.  A build of T iterations takes the
# mean of the first T entries; T beyond the table also gives null.
JOIN_TRAFFIC = {
    ("sift1m", 1_000_000, 128, 32, 32, "k_join_mfma", "selective"): {
        "fetch_raw_mib": [3930.8, 4592.3, 5184.2, 5013.2, 5055.2, 4731.6, 4191.9],
        "write_raw_mib": [577.5, 478.0, 740.7, 591.7, 446.0, 250.8, 140.9],
        "fetch_scale": 2.0, "write_scale": 1.0},
}


def join_traffic(key, T):
    rec = JOIN_TRAFFIC.get(key)
    if rec is None or T > len(rec["fetch_raw_mib"]) or T > len(rec["write_raw_mib"]):
        return None, None
    f = sum(rec["fetch_raw_mib"][:T]) / T
    w = sum(rec["write_raw_mib"][:T]) / T
    return ((f * rec["fetch_scale"] + w * rec["write_scale"]) * 2 ** 20, (f + w) * 2 ** 20)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--n", type=int, default=None, help="default: the workload's size")
    ap.add_argument("--d", type=int, default=None)
    ap.add_argument("--k", type=int, default=32)
    ap.add_argument("--p", type=int, default=32)
    ap.add_argument("--max-iters", type=int, default=12)
    ap.add_argument("--target", type=float, default=0.95)
    ap.add_argument("--eval-nodes", type=int, default=2000)
    ap.add_argument("--join", choices=["auto", "valu", "mfma", "gram"], default="auto")
    ap.add_argument("--update", choices=["selective", "all-pairs"], default="selective",
                    help="all-pairs: the ablation variant that proposes every evaluated pair "
                         "(runs with the valu join; ~100 KB of workspace per node at p = 32)")
    ap.add_argument("--lists", choices=["plain", "segmented"], default="plain",
                    help="segmented: the k-NN list as k/32 segments of 32, object v in segment "
                         "v %% (k/32) (the paper's multiple-spinlock layout; k = 64, 96, 128)")
    ap.add_argument("--cpu-sample-n", type=int, default=None,
                    help="rows of the oracle's timed sample (default 200000; 30000 at d = 960)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-one-thread-n", type=int, default=None,
                    help="rows of the oracle's one-thread timing (default 30000; 2000 at d = 960)")
    ap.add_argument("--no-valu-line", action="store_true",
                    help="skip the extra timing of the same workload through the float32 join")
    ap.add_argument("--workload", choices=["sift1m", "gist1m", "deep10m", "sharded"],
                    default="sift1m",
                    help="sift1m is the metric's workload; gist1m (960-d, squared L2) and deep10m "
                         "(96-d unit vectors, angular) are the paper's other float shapes, extra "
                         "lines through the general float join; sharded is the merge workload")
    ap.add_argument("--shards", type=int, default=4)
    ap.add_argument("--store", choices=["memory", "files"], default="memory",
                    help="sharded workload: keep collection and graph in pinned host memory, or "
                         "in files under --store-dir behind one pinned staging buffer")
    ap.add_argument("--store-dir", default=None)
    ap.add_argument("--staging-mib", type=int, default=256)
    ap.add_argument("--build-iters", type=int, default=8)
    ap.add_argument("--merge-iters", type=int, default=4)
    ap.add_argument("--copy-calib-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB (a dispatch of known "
                         "size to scale rocprofv3's FETCH_SIZE / WRITE_SIZE counters with)")
    args = ap.parse_args()
    n, d = {"sift1m": (1_000_000, 128), "gist1m": (1_000_000, 960), "deep10m": (10_000_000, 96),
            "sharded": (100_000_000, 128)}[args.workload]
    args.n = args.n or n
    args.d = args.d or d
    args.cpu_sample_n = args.cpu_sample_n or (30_000 if args.d > 512 else 200_000)
    args.cpu_one_thread_n = args.cpu_one_thread_n or (2_000 if args.d > 512 else 30_000)
    return args


def float_workload(args, W, amd_or_og):
    """Generator, metric and description of the float workloads."""
    name = args.workload
    if name == "gist1m":
        return (lambda n: W.gist_like_f32(n, args.d), amd_or_og.L2SQ_F32,
                "gist-shaped L1-normalised mixture", "squared L2")
    if name == "deep10m":
        return (lambda n: W.deep_like_f32(n, args.d), amd_or_og.ANGULAR_F32,
                "deep-shaped unit-length mixture", "angular (1 - dot)")
    return (lambda n: W.sift_like_f32(n, args.d, seed=1002), amd_or_og.L2SQ_F32,
            "sift-shaped GMM", "squared L2")


def time_oracle(args, iters, n, threads):
    """One oracle build (random initial graph + `iters` iterations) of the first n
    rows of the workload's generator on `threads` host threads."""
    import oracle as og
    import workloads as W

    og.set_threads(threads)
    gen, metric, _, _ = float_workload(args, W, og)
    x = gen(n)
    t0 = time.perf_counter()
    seg = args.lists == "segmented"
    g = og.init_random(x, args.k, metric, W.ALGO_SEED, segmented=seg)
    evals = 0
    for it in range(1, iters + 1):
        evals += og.iterate(x, metric, g, args.p, W.ALGO_SEED, it, segmented=seg)["dist_evals"]
    dt = time.perf_counter() - t0
    return evals, dt


def cpu_baseline(args, iters):
    """The oracle as it stands, timed on this host's cores on cuts of the same
    generator (same d, k, p, same number of iterations): all cores on the larger
    cut (the reported value) and one thread on a smaller one (the paper's own
    baseline is a single thread)."""
    cores = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "16")))
    n = min(args.cpu_sample_n, args.n)
    evals, dt = time_oracle(args, iters, n, cores)
    n1 = min(args.cpu_one_thread_n, args.n)
    evals1, dt1 = time_oracle(args, iters, n1, 1)
    what = f"d={args.d}, k={args.k}, p={args.p}, {iters} iterations, init + all stages"
    return {"value": evals / dt, "unit": "dist_evals/s", "cores": cores, "kind": "oracle",
            "build_s_on_sample": dt,
            "sample": f"n={n} cut of the same generator, {what}",
            "one_thread": {"value": evals1 / dt1, "unit": "dist_evals/s", "cores": 1,
                           "build_s_on_sample": dt1,
                           "sample": f"n={n1} cut of the same generator, {what}"}}


def sharded(args, torch, amd, W, dev):
    """The merge workload: uint8 vectors, d = 128, SIFT-shaped 64-component
    mixture; graphs of `--shards` equal shards are built one at a time and merged
    pairwise with GGM, the collection staying in pinned host memory (only two
    shards resident).  Not the headline metric: an extra line for that path."""
    n, d, k, p = args.n, args.d, args.k, args.p
    g = torch.Generator(device=dev).manual_seed(1005)
    centres = torch.rand((64, d), generator=g, device=dev) * 128.0
    xh = torch.empty((n, d), dtype=torch.uint8, pin_memory=True)
    xd = torch.empty((n, d), dtype=torch.uint8, device=dev)  # for the ground truth only
    step = 1 << 21
    for lo in range(0, n, step):
        hi = min(n, lo + step)
        comp = torch.randint(0, 64, (hi - lo,), generator=g, device=dev)
        v = centres[comp] + 20.0 * torch.randn((hi - lo, d), generator=g, device=dev)
        xd[lo:hi] = v.clamp_(0.0, 255.0).round_().to(torch.uint8)
        xh[lo:hi].copy_(xd[lo:hi])
    torch.cuda.synchronize()
    q = torch.from_numpy(W.sample_nodes(n, args.eval_nodes)).to(dev)
    _, tdist = amd.exact_knn(xd, q, 10, amd.L2SQ_U8)
    del xd
    torch.cuda.empty_cache()
    where = "pinned host memory"
    if args.store == "files":
        import tempfile

        import numpy as np
        folder = tempfile.mkdtemp(prefix="gnnd_shards_", dir=args.store_dir)
        paths = [os.path.join(folder, f) for f in ("vectors.u8", "ids.i32", "dist.i32")]
        xh.numpy().tofile(paths[0])
        del xh
        t0 = time.perf_counter()
        st = amd.gnnd_build_sharded_files(paths[0], n, d, args.shards, k, p, paths[1], paths[2],
                                          amd.L2SQ_U8, W.ALGO_SEED, args.build_iters,
                                          args.merge_iters, staging_bytes=args.staging_mib << 20)
        wall = time.perf_counter() - t0
        dist = torch.from_numpy(np.memmap(paths[2], dtype=np.int32, mode="r", shape=(n, k))[
            q.cpu().numpy()].copy())
        rec = amd.recall_at(dist.to(dev), tdist, 10)
        for f in paths:
            os.remove(f)
        os.rmdir(folder)
        where = f"files behind a {args.staging_mib} MiB pinned staging buffer"
    else:
        t0 = time.perf_counter()
        ids, dist, st = amd.gnnd_build_sharded(xh, args.shards, k, p, amd.L2SQ_U8, W.ALGO_SEED,
                                               args.build_iters, args.merge_iters)
        wall = time.perf_counter() - t0
        rec = amd.recall_at(dist[q.cpu().long()].to(dev), tdist, 10)
    out = {"metric": "sharded_build_seconds", "value": st["ms_total"] / 1e3, "unit": "s",
           "n_gpus": 1, "steps": 1, "warmup": 0, "ms_per_step": st["ms_total"],
           "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "i8",
           "data": "synthetic",
           "config": {"workload": f"uint8 sift-shaped GMM n={n} d={d}, {args.shards} shards in "
                                  f"{where}, k={k} p={p}, {args.build_iters} build + "
                                  f"{args.merge_iters} merge iterations, all pairs merged once"},
           "recall_at_10": rec, "stats": st, "wall_s_including_arena_alloc": wall}
    print(json.dumps(out))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding or collectives); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch

    import paper_2103_15386_amd as amd
    import workloads as W

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.workload == "sharded":
        return sharded(args, torch, amd, W, dev)
    gen, metric, shape_name, metric_name = float_workload(args, W, amd)
    x = gen(args.n)
    xd = torch.from_numpy(x).to(dev)
    del x
    if args.copy_calib_mib:
        src = torch.empty(args.copy_calib_mib << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    join_path = {"auto": amd.JOIN_AUTO, "valu": amd.JOIN_VALU, "mfma": amd.JOIN_MFMA,
                 "gram": amd.JOIN_GRAM}[args.join]
    seed = W.ALGO_SEED

    # ground truth for the recall evaluation: exhaustive search on sampled nodes
    q = torch.from_numpy(W.sample_nodes(args.n, args.eval_nodes)).to(dev)
    _, tdist = amd.exact_knn(xd, q, 10, metric)
    ql = q.long()

    update_mode = amd.UPDATE_ALL_PAIRS if args.update == "all-pairs" else amd.UPDATE_SELECTIVE
    list_mode = amd.LISTS_SEGMENTED if args.lists == "segmented" else amd.LISTS_PLAIN
    ctx = amd.Gnnd(xd, args.k, args.p, metric, seed, join_path, update_mode, list_mode)

    # calibration build (untimed): recall and per-stage times after every iteration
    ctx.init_random()
    trace, T = [], None
    for it in range(1, args.max_iters + 1):
        st = ctx.iterate()
        _, dist = ctx.graph()
        st["recall_at_10"] = amd.recall_at(dist[ql], tdist, 10)
        trace.append(st)
        if T is None and st["recall_at_10"] >= args.target:
            T = it
            break
    reached = T is not None
    if not reached:
        T = args.max_iters
    best = max(t["recall_at_10"] for t in trace)

    stream = torch.cuda.current_stream(dev)
    mfma = ctx.join_path() == amd.JOIN_MFMA
    gram = ctx.join_path() == amd.JOIN_GRAM

    def timed_builds(c, steps, warmup):
        """`steps` builds of T iterations on context c after `warmup` untimed ones: seconds
        per build by the host clock around the whole loop, and per-build stage milliseconds
        from HIP events recorded on the stream inside those same builds (a window sized
        for all of them, created before the clock starts; nothing synchronises in the loop)."""
        for _ in range(warmup):
            c.build(T, want_stats=False)
        c.set_profiling(max(1, T * steps))
        stream.synchronize()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            c.build(T, want_stats=False)
        stream.synchronize()
        torch.cuda.synchronize()
        per_build = (time.perf_counter() - t0) / steps
        n_rec, missed, sample_ms, join_ms, handout_ms, update_ms = c.stage_ms()
        c.set_profiling(0)
        builds_rec = n_rec / T if n_rec else float("nan")
        # "join" is the cross-matching kernel alone; "handout" the pass behind it that moves
        # staged results into the destinations' segments (~0 where the join hands them on itself)
        stages = {"sample": sample_ms / builds_rec, "join": join_ms / builds_rec,
                  "handout": handout_ms / builds_rec, "update": update_ms / builds_rec}
        return per_build, stages, {"recorded": n_rec, "missed": missed, "expected": T * steps}

    build_s, stage, stage_records = timed_builds(ctx, args.steps, args.warmup)
    sample_ms, join_ms, update_ms = stage["sample"], stage["join"], stage["update"]

    total_evals = sum(t["dist_evals"] for t in trace[:T])

    # Roofline of the dominant kernel, the cross-matching join; one launch = one
    # iteration.  Algorithmic bytes per launch: every sampled vector is read once
    # per joined node (d elements of e bytes: e = 1 for the int8 copy the
    # matrix-core kernel reads, 4 for float32) plus its 4-byte id.
    # Algorithmic operations: 3 per dimension and evaluated pair in the direct
    # form (subtract, multiply, add), 2 in the Gram form.
    elem = 1 if mfma else 4
    drow = ((args.d + 31) // 32 * 32) if mfma else args.d
    vectors = sum(t["sum_new"] + t["sum_old"] for t in trace[:T]) / T
    alg_bytes = vectors * (drow * elem + 4)
    avg_join_s = join_ms / T / 1e3
    hbm = {"bound": "hbm", "achieved": alg_bytes / avg_join_s / 1e9, "peak": PEAK_HBM_GBS,
           "unit": "GB/s", "traffic": None}
    kernel_name = "k_join_mfma" if mfma else "k_join_gram" if gram else (
        "k_join_long" if args.p > 32 else "k_join_valu")
    hbm["traffic"], hbm["traffic_raw"] = join_traffic(
        (args.workload, args.n, args.d, args.k, args.p, kernel_name, args.update), T) \
        if args.lists == "plain" else (None, None)
    hbm["frac"] = hbm["achieved"] / hbm["peak"]
    if mfma:
        ops = total_evals / T * args.d * 2
        other = {"bound": "mfma", "achieved": ops / avg_join_s / 1e12, "peak": PEAK_INT8_TOPS,
                 "unit": "TOP/s"}
    elif gram:  # float32 matrix instructions: the same peak as the vector units'
        ops = total_evals / T * args.d * 2
        other = {"bound": "mfma", "achieved": ops / avg_join_s / 1e12, "peak": PEAK_FP32_TFLOPS,
                 "unit": "TFLOP/s"}
    else:
        ops = total_evals / T * args.d * (2 if metric == amd.ANGULAR_F32 else 3)
        other = {"bound": "alu", "achieved": ops / avg_join_s / 1e12, "peak": PEAK_FP32_TFLOPS,
                 "unit": "TFLOP/s"}
    other["frac"] = other["achieved"] / other["peak"]
    roof = dict(hbm)
    if other["frac"] > hbm["frac"]:
        roof = dict(other)
        roof["traffic"] = None
        roof["other_bound"] = hbm
    else:
        roof["other_bound"] = other
    roof["kernel"] = kernel_name
    if gram:  # one launch per class of nodes; the figures are per iteration, all seven together
        roof["launches_per_iteration"] = 7
    elif kernel_name == "k_join_mfma" and args.n <= (1 << 20):
        # staged hand-out: one build per shape of node (<= 32 OLD samples, <= 32 NEW samples,
        # the rest); the figures are per iteration, the three launches together
        roof["launches_per_iteration"] = 3
    roof["avg_launch_ms"] = avg_join_s * 1e3
    roof["algorithmic_bytes_per_launch"] = alg_bytes

    out = {
        "metric": "build_seconds_to_recall@10>=%.2f" % args.target,
        "value": build_s, "unit": "s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": build_s * 1e3, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "i8" if mfma else "f32",
        "data": "synthetic",
        "config": {"workload": f"{shape_name} n={args.n} d={args.d} f32, k={args.k} "
                               f"p={args.p}, {metric_name}, random init + {T} iterations",
                   "join_path": "mfma_i8" if mfma else "gram_f32" if gram else "valu",
                   "update": args.update,
                   "lists": args.lists,
                   "eval_nodes": args.eval_nodes},
        "reached_target": reached, "iterations": T, "recall_at_10": trace[T - 1]["recall_at_10"],
        "best_recall_at_10": best,
        "dist_evals": total_evals, "dist_evals_per_s": total_evals / build_s,
        "join_dist_evals_per_s": total_evals / (join_ms / 1e3),
        "stage_ms": stage,
        "stage_records": stage_records,
        "per_iteration": [{k: (round(v, 4) if isinstance(v, float) else v) for k, v in t.items()}
                          for t in trace],
        "roofline": roof,
    }
    if mfma and not args.no_valu_line:
        # the same workload through the two float32 joins, same T, as extra figures: the
        # paper's arithmetic (one fused multiply-add per dimension and pair) for every pair,
        # and the matrix-core form that spends it on the possible nearest partners only
        ctx.close()
        del ctx
        for key, path, kernel, per_dim in (("f32_gram_join", amd.JOIN_GRAM, "k_join_gram", 2),
                                           ("f32_valu_join", amd.JOIN_VALU, "k_join_valu", 3)):
            vctx = amd.Gnnd(xd, args.k, args.p, metric, seed, path, update_mode, list_mode)
            v_s, v_stage, v_rec = timed_builds(vctx, min(args.steps, 3), 1)
            v_bytes = vectors * (args.d * 4 + 4)
            v_join_s = v_stage["join"] / T / 1e3
            out[key] = {
                "build_s": v_s, "stage_ms": v_stage, "stage_records": v_rec, "dtype": "f32",
                "kernel": kernel, "avg_launch_ms": v_join_s * 1e3,
                "hbm_frac": v_bytes / v_join_s / 1e9 / PEAK_HBM_GBS,
                "alu_frac": total_evals / T * args.d * per_dim / v_join_s / 1e12 / PEAK_FP32_TFLOPS}
            vctx.close()
    if not args.no_cpu_baseline:
        try:
            out["cpu_baseline"] = cpu_baseline(args, T)
        except Exception as exc:  # the line is printed whatever happens to the baseline leg
            out["cpu_baseline"] = {"value": None, "unit": "dist_evals/s", "cores": 0,
                                   "kind": "oracle", "sample": f"failed: {exc!r}"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
