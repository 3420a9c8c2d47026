#!/usr/bin/env python3
"""Benchmark of one S3GD-MV step (encode -> majority vote -> update) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C5]

A "step" is one pass of the whole hot path over one batch of synthetic gradients on a resident
[M, N] fp32 tensor.  Inputs are generated on the host from the seeded recipes in
paper_2302_07475_amd/datagen.py and are resident in HBM before the timed region starts.
Prints ONE JSON line:

  value        M*N / t   gradient elements per second through one step of the fused call s3gd_step
  three_calls  the same step as the three public calls (s3gd_topk_sign_encode, s3gd_majority_vote
               with int8 votes, s3gd_apply_update) enqueued back to back, timed in the same run
  roofline     the dominant kernel's algorithmic bytes per launch over its mean duration, measured
               with HIP events on the launch stream inside the timed region, against 8 TB/s
  cpu_baseline the CPU oracle timed on this machine's host cores on a bounded sample of the workload,
               single-threaded and with the rows spread over threads
"""
import argparse
import dataclasses
import json
import os
import statistics
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK = 8.0e12  # bytes/s, MI355X published peak

# HBM bytes per launch (read + written) of a workload's dominant kernel, from rocprofv3 FETCH_SIZE / WRITE_SIZE
# runs of this same command, scaled by the factors a plain copy of known size gives (2.0 for FETCH_SIZE, 1.0 for
# WRITE_SIZE).  Counter figures cannot be taken inside this run; they are quoted with the file they come from.
PROFILED_TRAFFIC = {  # (workload, variant, dominant kernel): bytes read + bytes written per launch
    ("C5", "", "filter"): (19.2003e9 + 0.0652e9, "profiles/s3gd_step_C5_hbm_traffic.md"),
    ("C5", "three-calls", "filter"): (19.2003e9 + 0.0653e9, "profiles/s3gd_three_calls_C5_hbm_traffic.md"),
    ("C4", "", "filter"): (3.9688e9 + 0.0885e9, "profiles/s3gd_step_C4_hbm_traffic.md"),
    ("C3", "", "filter"): (3.2792e9 + 0.0166e9, "profiles/s3gd_step_C3_hbm_traffic.md"),
    ("C2", "", "filter"): (0.7181e9 + 0.0187e9, "profiles/s3gd_step_C2_hbm_traffic.md"),
    ("C4", "sparsity 0.1", "filter"): (3.9688e9 + 0.5586e9, "profiles/s3gd_step_C4_gamma0.1_hbm_traffic.md"),
    ("C5", "memory", "filter_mem"): (38.4211e9 + 21.3004e9, "profiles/s3gd_step_ec_C5_hbm_traffic.md"),
    ("C4", "memory sparsity 0.1", "filter_mem"): (7.9416e9 + 4.9787e9, "profiles/s3gd_step_ec_C4_gamma0.1_hbm_traffic.md"),
    ("C4", "memory-acc sparsity 0.1", "filter_mem"): (3.9698e9 + 4.0843e9, "profiles/s3gd_step_acc_C4_gamma0.1_hbm_traffic.md"),
    ("C5", "memory-acc", "filter"): (19.2003e9 + 0.0649e9, "profiles/s3gd_step_acc_C5_hbm_traffic.md"),
    ("C5", "momentum", "filter"): (19.2004e9 + 0.0652e9, "profiles/s3gd_step_momentum_C5_hbm_traffic.md"),
    ("C5", "momentum dense-state", "vote_momentum"): (9.6932e9 + 9.6008e9, "profiles/s3gd_step_momentum_dense_C5_hbm_traffic.md"),
    ("C5", "wire", "filter"): (19.2004e9 + 0.0653e9, "profiles/s3gd_wire_format_C5_hbm_traffic.md"),
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(cfg, datagen):
    """The oracle, as it stands, on a bounded sample: all M workers, the first N_s coordinates, K scaled to
    keep K/N.  Timed twice: on one thread (t_cpu1) and with the rows' selections spread over min(M, cores)
    threads (t_cpuP; the vote and the update stay serial).  Sorting is O(N log N), so the per-element rate
    at the full N is lower; the full configuration would take minutes to hours and is not run."""
    from concurrent.futures import ThreadPoolExecutor

    from oracle import s3gd_oracle as O
    n_s = min(cfg.N, max(1 << 16, (120_000_000 // cfg.M)))
    k_s = max(1, round(cfg.K * n_s / cfg.N))
    small = cfg.scaled(N=n_s, K=k_s)
    G = datagen.gradients(small)
    x = datagen.params(small)
    lr = datagen.lr32(small)
    t0 = time.perf_counter()
    one = O.step(G, small.K, x, lr)
    t_cpu1 = time.perf_counter() - t0
    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    threads = max(1, min(cfg.M, cores, 16))
    t0 = time.perf_counter()
    with ThreadPoolExecutor(threads) as pool:
        rows = list(pool.map(lambda m: O.encode_row(G[m], small.K), range(cfg.M)))
    words = np.full((cfg.M, small.K), O.PAD, dtype=np.uint32)
    counts = np.zeros(cfg.M, dtype=np.uint32)
    for m, (w, c) in enumerate(rows):
        words[m], counts[m] = w, c
    tally, votes = O.majority_vote(words, counts, n_s)
    xp = O.apply_update(x, votes, lr)
    t_cpup = time.perf_counter() - t0
    assert np.array_equal(xp.view(np.uint32), one["x"].view(np.uint32))
    return {"value": cfg.M * n_s / t_cpup, "unit": "gradient elements/s", "cores": threads, "kind": "oracle",
            "single_thread_value": cfg.M * n_s / t_cpu1, "t_cpu1_s": round(t_cpu1, 2), "t_cpuP_s": round(t_cpup, 2),
            "host_cores_available": cores, "cpu_model": cpu_model(), "sample_fraction": n_s / cfg.N,
            "sample": f"all {cfg.M} workers, first {n_s} of {cfg.N} coordinates of {cfg.name} ({100.0 * n_s / cfg.N:.1f} %), "
                      f"K={k_s}, one step; 1 thread {t_cpu1:.1f} s, {threads} threads over the rows {t_cpup:.1f} s"}


def kernel_bytes(name, M, N, K, rows, n_voted, dense_state, tally_out, votes_out, mem_pass_bytes=12.0):
    """Algorithmic bytes one launch of a kernel moves: what the step needs from that pass, not what the
    hardware counters saw.  `rows` = rows of G the pass actually reads."""
    if name in ("filter", "hist_rows_0", "hist_rows_1", "hist_rows_2", "tile_count", "emit_rows"):
        return 4.0 * N * rows
    if name == "filter_mem":  # reads g~ and e, writes the new memory (8 bytes an entry when it rewrites the one buffer that holds g)
        return mem_pass_bytes * N * rows
    if name == "plain_read":
        return 4.0 * M * N
    if name == "randk":  # K gathered gradient entries and K words per row
        return 8.0 * M * K
    if name == "vote_sparse":  # the words, and a read and a write of every voted parameter
        return 4.0 * M * K + 8.0 * n_voted
    if name == "vote_dense":
        out = (4.0 * N if tally_out else 0.0) + (1.0 * N if votes_out else 0.0)
        return 4.0 * M * K + (out if out else 8.0 * n_voted)
    if name == "apply_update":  # the votes, and a read and a write of every voted parameter
        return 1.0 * N + 8.0 * n_voted
    if name == "vote_momentum":
        return 4.0 * M * K + (16.0 * N if dense_state else 4.0 * N + 16.0 * n_voted)
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C5", choices=["C1", "C2", "C3", "C4", "C5"])
    ap.add_argument("--three-calls", action="store_true",
                    help="make the three separate calls the timed entry (they are always timed as a second record)")
    ap.add_argument("--memory", action="store_true",
                    help="time s3gd_step_ec: the step with the error-compensation memory (eta = 1), a second "
                         "[M, N] fp32 tensor read and rewritten every step (not the headline workload)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", type=float, default=0.0, metavar="GiB",
                    help="instead of the benchmark, run three plain device copies of this size; run it under "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE to get the factor between counter units and bytes")
    ap.add_argument("--calibrate-read", type=float, default=0.0, metavar="GiB",
                    help="instead of the benchmark, time a plain non-temporal read of this size with the launch shape "
                         "of the selection pass (s3gd_calibrate_read): the practical read ceiling of the memory system")
    ap.add_argument("--calibrate-rmw", type=float, default=0.0, metavar="GiB",
                    help="instead of the benchmark, time b <- a + b over two buffers of this size with the launch shape of the "
                         "selection pass with a memory (s3gd_calibrate_rmw): the practical ceiling of a two-reads-one-write stream")
    ap.add_argument("--wire", action="store_true",
                    help="time encode -> pack -> unpack -> vote+update: the step with the messages passed through the "
                         "compact wire format, as they would be around an exchange (not the headline workload)")
    ap.add_argument("--randk", action="store_true",
                    help="time s3gd_step_randk (Algorithm 2: random-K instead of top-K; not the headline workload)")
    ap.add_argument("--graph", action="store_true",
                    help="capture the step into a HIP graph once and time replays (the same kernels, fewer launch gaps)")
    ap.add_argument("--momentum", action="store_true",
                    help="time s3gd_step_momentum (mu = 0.9): the update streams a momentum vector (not the headline workload)")
    ap.add_argument("--memory-acc", action="store_true",
                    help="time s3gd_step_acc: the error-compensation memory already holds g~ + e when the step starts (the "
                         "gradients were accumulated into it), so the step reads one tensor (not the headline workload)")
    ap.add_argument("--dense-state", action="store_true",
                    help="with --momentum: start from a momentum vector without zeros, as it is after some hundred "
                         "steps of training (every coordinate is then read, updated and written each step); without "
                         "this flag the vector starts at zero, as in the first steps, and stays as sparse as the votes")
    ap.add_argument("--sparsity", type=float, default=0.0, metavar="GAMMA",
                    help="override K with GAMMA * N on the chosen workload (the paper sweeps K/N from 1 down to 0.001; "
                         "not the headline workload)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build measures one GPU only (all M workers are rows of one tensor); --gpus must be 1")
        sys.exit(2)

    import torch

    from paper_2302_07475_amd import costs, datagen, s3gd

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        sys.exit(3)
    dev = torch.device("cuda:0")
    if args.calibrate_copy > 0:
        n = int(args.calibrate_copy * (1 << 30)) // 4
        src = torch.ones(n, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "plain copy", "bytes_read_per_copy": 4 * n, "bytes_written_per_copy": 4 * n}))
        return
    if args.calibrate_read > 0:
        n = (int(args.calibrate_read * (1 << 30)) // 4) // 1024 * 1024
        buf = torch.ones(n, dtype=torch.float32, device=dev)
        ctx = s3gd.Context(4, min(n, s3gd.N_LIMIT), 1, device=0)
        for _ in range(2):
            ctx.calibrate_read(buf)
        ctx.profile_enable(2)
        reps = 10
        for _ in range(reps):
            ctx.calibrate_read(buf)
        ms, cnt = ctx.profile_read()["plain_read"]
        print(json.dumps({"calibration": "plain non-temporal read, launch shape of the selection pass", "bytes_per_launch": 4 * n,
                          "launches": cnt, "ms_avg": ms / cnt, "GB_per_s": 4.0 * n / (ms / cnt * 1e-3) / 1e9,
                          "fraction_of_8TB_per_s": 4.0 * n / (ms / cnt * 1e-3) / HBM_PEAK}))
        return
    if args.calibrate_rmw > 0:
        n = (int(args.calibrate_rmw * (1 << 30)) // 4) // 8192 * 8192
        a = torch.ones(n, dtype=torch.float32, device=dev)
        b = torch.zeros(n, dtype=torch.float32, device=dev)
        ctx = s3gd.Context(4, min(n, s3gd.N_LIMIT), 1, device=0)
        for _ in range(2):
            ctx.calibrate_rmw(a, b)
        ctx.profile_enable(2)
        reps = 10
        for _ in range(reps):
            ctx.calibrate_rmw(a, b)
        ms, cnt = ctx.profile_read()["plain_rmw"]
        torch.cuda.synchronize()
        if not bool((b == float(reps + 2)).all()):
            log("bench.py: the calibration stream did not add up")
            sys.exit(1)
        print(json.dumps({"calibration": "plain b <- a + b, launch shape of the selection pass with a memory", "bytes_per_launch": 12 * n,
                          "launches": cnt, "ms_avg": ms / cnt, "GB_per_s": 12.0 * n / (ms / cnt * 1e-3) / 1e9,
                          "fraction_of_8TB_per_s": 12.0 * n / (ms / cnt * 1e-3) / HBM_PEAK}))
        return
    cfg = datagen.CONFIGS[args.workload]
    t0 = time.perf_counter()
    g, x = datagen.to_device(cfg, device="cuda:0")
    log(f"[bench] {cfg.name}: M={cfg.M} N={cfg.N} K={cfg.K} generated and uploaded in {time.perf_counter() - t0:.1f} s")
    # what the input was: SHA-256 of the first chunk (2^22 coordinates) of worker 0's gradients and of x^0, as generated on the host
    import hashlib
    input_sha256 = {"g[0] first chunk": hashlib.sha256(datagen.grad_chunk(cfg, 0, 0, 0).tobytes()).hexdigest(),
                    "x0 first chunk": hashlib.sha256(datagen.x0_chunk(cfg, 0).tobytes()).hexdigest()}
    log(f"[bench] input sha256: {input_sha256}")
    M, N, K = cfg.M, cfg.N, cfg.K
    if args.sparsity > 0:
        K = max(1, min(N, int(round(args.sparsity * N))))
        cfg = dataclasses.replace(cfg, K=K)
    lr = float(datagen.lr32(cfg))
    ctx = s3gd.Context(M, N, K, device=0)
    words = torch.empty((M, K), dtype=torch.int32, device=dev)
    counts = torch.empty((M,), dtype=torch.int32, device=dev)
    votes = torch.empty((N,), dtype=torch.int8, device=dev)
    err = torch.zeros((M, N), dtype=torch.float32, device=dev) if args.memory else None

    mom = torch.zeros((N,), dtype=torch.float32, device=dev) if args.momentum else None
    if args.momentum and args.dense_state:
        gen = torch.Generator(device=dev)
        gen.manual_seed(1234)
        mom.normal_(0.0, 1.0, generator=gen)
        mom[mom == 0] = 1.0

    packed = w2 = c2 = None
    if args.wire:
        packed = torch.empty((M, s3gd.packed_row_words(N, K)), dtype=torch.int32, device=dev)
        w2, c2 = torch.empty_like(words), torch.empty_like(counts)

    step_no = [0]

    def three_calls_step():
        ctx.topk_sign_encode(g, K, words, counts)
        ctx.majority_vote(words, counts, N, None, votes)
        ctx.apply_update(x, votes, lr)

    def fused_step():
        ctx.step(g, K, x, lr, words, counts, None, None)

    def variant_step():
        if args.randk:
            ctx.step_randk(g, K, 0x5EED, step_no[0], x, lr, words, counts, None, None)
            step_no[0] += 1
        elif args.wire:
            ctx.topk_sign_encode(g, K, words, counts)
            ctx.pack_messages(words, counts, N, packed)
            ctx.unpack_messages(packed, N, K, w2, c2)
            ctx.vote_update(w2, c2, N, x, lr)
        elif args.momentum:
            ctx.step_momentum(g, K, x, mom, lr, 0.9, words, counts, err=err, eta=1.0)
        elif args.memory_acc:
            ctx.step_acc(acc, K, x, lr, words, counts, None, None)
        elif args.memory:
            ctx.step_ec(g, err, 1.0, K, x, lr, words, counts, None, None)
        else:
            raise AssertionError

    # s3gd_step_acc finds g~ + e in the memory: the producer of the gradients accumulates them there.  Here that is an
    # addition before every step, outside the step's event pair (the step's time is then the mean of the event times).
    acc = g.clone() if args.memory_acc else None
    before_step = (lambda: acc.add_(g)) if args.memory_acc else None

    is_variant = args.randk or args.wire or args.momentum or args.memory_acc or args.memory
    headline = variant_step if is_variant else (three_calls_step if args.three_calls else fused_step)

    def measure(eager_step, steps, warmup, use_graph=False, pre=None):
        """W untimed steps, then exactly `steps` steps between two synchronisations.  Returns the mean wall
        time per step, the median of the per-step times between HIP events recorded on the launch stream,
        and the per-kernel figures (a breakdown pass with an event pair around every launch, run before the
        timed region; the dominant passes carry their own event pair inside it)."""
        one_step = eager_step
        if pre is not None:
            def one_step():
                pre()
                eager_step()
        if use_graph:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                eager_step()
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                eager_step()
            one_step = graph.replay
        for _ in range(warmup):
            one_step()
        torch.cuda.synchronize()
        assert ctx.last_async_status() == 0
        routes = ctx.last_encode_routes()
        ctx.profile_enable(1)
        for _ in range(3):
            one_step() if pre is not None else eager_step()
        prof = ctx.profile_read()
        kern = {k: {"ms_avg": v[0] / v[1], "launches_per_step": v[1] / 3} for k, v in prof.items()}
        ctx.profile_enable(0 if use_graph else 2)
        torch.cuda.synchronize()
        if pre is None:
            # the timed region: exactly `steps` steps between two synchronisations; the only events on the stream are the
            # pair around the dominant pass (profile mode 2: about 9 us per step)
            t0 = time.perf_counter()
            for i in range(steps):
                one_step()
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            live = {} if use_graph else ctx.profile_read()
            ctx.profile_enable(0)
            # the same again with an event after every step, for the spread (each event costs the stream a few
            # microseconds, which is why the timed region has none): a step runs from the end of the one before it
            ends = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
            ends[0].record()
            for i in range(steps):
                one_step()
                ends[i + 1].record()
            torch.cuda.synchronize()
            per_step = [ends[i].elapsed_time(ends[i + 1]) for i in range(steps)]
        else:  # the producer's work before each step lies outside the step's event pair
            starts = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
            ends = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
            for i in range(steps):
                pre()
                starts[i].record()
                eager_step()
                ends[i].record()
            torch.cuda.synchronize()
            live = {} if use_graph else ctx.profile_read()
            ctx.profile_enable(0)
            per_step = [starts[i].elapsed_time(ends[i]) for i in range(steps)]
            dt = sum(per_step) * 1e-3
        for k, v in live.items():  # measured inside the timed region: these replace the figures of the breakdown pass
            kern[k] = {"ms_avg": v[0] / v[1], "launches_per_step": v[1] / steps}
        return dt * 1e3 / steps, statistics.median(per_step), kern, set(live), routes

    ms_step, ms_median, kern, live, routes = measure(headline, args.steps, args.warmup, args.graph, pre=before_step)
    log(f"[bench] timed {args.steps} steps: mean {ms_step:.4f} ms, median of per-step event times {ms_median:.4f} ms")
    for k, v in sorted(kern.items(), key=lambda kv: -kv[1]["ms_avg"] * kv[1]["launches_per_step"]):
        log(f"[bench]   {k:14s} {v['ms_avg']:9.4f} ms x {v['launches_per_step']:.0f}" + ("  (timed region)" if k in live else ""))

    # the support of the vote: coordinates that received a message (what the update has to touch at most)
    seen = torch.zeros((N,), dtype=torch.bool, device=dev)
    for m in range(M if K > 0 else 0):
        w = words[m, : int(counts[m].item())].to(torch.int64) & 0xFFFFFFFF
        seen[w >> 1] = True
    n_voted = int(seen.sum().item())
    del seen
    n_rows, general, _wide, row_pass, skipped = routes
    # s3gd_step_acc takes the pass in chunks, over the one buffer, from K = N/32 on
    rewrite = args.memory_acc and K * 32 >= N
    plan = ctx.encode_plan_info(M, N, K, with_memory=args.memory or rewrite)
    mem_pass_bytes = 8.0 if rewrite else 12.0
    # rows of G each pass reads (the kernels of routes no row takes are enqueued and return at once)
    rows_read = {"filter": (M - skipped) if plan["candidates"] and not plan["chunks"] else 0,
                 "filter_mem": M if plan["candidates"] and plan["chunks"] else 0,
                 "hist_rows_0": general, "hist_rows_1": general, "hist_rows_2": general,
                 "tile_count": general + row_pass, "emit_rows": general + row_pass}
    if args.randk:
        rows_read = {}

    def alg_bytes(name, tally_out=False, votes_out=False):
        return kernel_bytes(name, M, N, K, rows_read.get(name, M), n_voted, args.dense_state, tally_out, votes_out, mem_pass_bytes)

    def fractions(kern_, votes_out):
        out = {}
        for k, v in kern_.items():
            b = alg_bytes(k, votes_out=votes_out)
            if b and v["ms_avg"] > 0:
                out[k] = {"ms": round(v["ms_avg"] * v["launches_per_step"], 5), "alg_GB": round(b / 1e9, 4),
                          "frac_of_peak": round(b * v["launches_per_step"] / (v["ms_avg"] * v["launches_per_step"] * 1e-3) / HBM_PEAK, 4)}
        return out

    votes_in_headline = args.three_calls and not is_variant
    dom = max(kern, key=lambda k: kern[k]["ms_avg"] * kern[k]["launches_per_step"])
    dom_bytes = alg_bytes(dom, votes_out=votes_in_headline) or 0.0
    achieved = dom_bytes / (kern[dom]["ms_avg"] * 1e-3)
    # bytes of G the step reads as built, plus the words written and read; the floor is one read of G, the words,
    # and a read and a write of every voted parameter (the fused step never moves an unvoted one)
    per_pass = {"filter_mem": mem_pass_bytes}
    g_bytes = sum(per_pass.get(k, 4.0) * N * r for k, r in rows_read.items() if k in kern)
    as_built = g_bytes + 8.0 * M * K + 8.0 * n_voted
    floor_bytes = (12.0 if args.memory else 4.0) * M * N + 8.0 * M * K + 8.0 * n_voted
    if args.randk:
        as_built = floor_bytes = 16.0 * M * K + 8.0 * n_voted
    variant = " ".join(name for name, on in (("three-calls", args.three_calls), ("memory", args.memory), ("memory-acc", args.memory_acc),
                                             ("momentum", args.momentum), ("dense-state", args.dense_state), ("wire", args.wire),
                                             ("randk", args.randk), (f"sparsity {args.sparsity:g}", args.sparsity > 0)) if on)
    traffic = PROFILED_TRAFFIC.get((cfg.name, variant, dom))
    entry = ("s3gd_step_randk (Algorithm 2)" if args.randk else
             "encode, pack, unpack, vote_update (messages through the wire format)" if args.wire else
             ("s3gd_step_momentum (mu=0.9" + (", with memory" if args.memory else "") +
              (", dense momentum state)" if args.dense_state else ", momentum starts at zero)")) if args.momentum else
             "s3gd_step_acc (fused, the memory already holds the compensated gradients)" if args.memory_acc else
             "s3gd_step_ec (fused, with error-compensation memory, eta=1)" if args.memory else
             ("s3gd_topk_sign_encode + s3gd_majority_vote (int8 votes) + s3gd_apply_update" if args.three_calls
              else "s3gd_step (fused, vote not materialised)"))
    out = {
        "metric": "gradient elements/sec per S3GD-MV step (M*N/t)",
        "value": M * N / (ms_step * 1e-3),
        "unit": "gradient elements/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "ms_per_step_median_of_event_times": ms_median,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32 keys of fp32 gradients, int32 tally, fp32 update", "data": "synthetic", "input_sha256": input_sha256,
        "config": {"workload": f"{cfg.name}: M={M} workers, N={N} fp32 coords, K={K}", "recipe": cfg.recipe, "entry": entry,
                   "rows": {"general_route": general, "wide_radix_select": _wide, "row_passes_known_threshold": row_pass,
                            "skipped_single_pass": skipped},
                   "launch": "HIP graph replay" if args.graph else "eager",
                   "timing": ("mean of per-step HIP event times; before each step the gradients are accumulated into the memory "
                              "(acc += g, the producer's work), outside the step's event pair") if args.memory_acc else
                             "wall clock over the timed steps between two synchronisations; the median of per-step event times comes "
                             "from a second run of as many steps with an event after each"},
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": achieved / 1e9, "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK, "algorithmic_bytes_per_launch": dom_bytes,
                     "duration_from": "HIP events inside the timed region" if dom in live else "HIP events, eager pass before the timed region",
                     "traffic": traffic[0] if traffic else None, "traffic_from": traffic[1] if traffic else None},
        "step_roofline": {"reads_of_G_per_step": g_bytes / (4.0 * M * N),
                          "voted_coordinates": n_voted,
                          "floor_bytes": floor_bytes, "f_alg": floor_bytes / (ms_step * 1e-3) / HBM_PEAK,
                          "step_bytes_as_built": as_built, "f_step": as_built / (ms_step * 1e-3) / HBM_PEAK},
        "kernels_ms": {k: round(v["ms_avg"] * v["launches_per_step"], 5) for k, v in kern.items()},
        "kernel_fractions": fractions(kern, votes_in_headline),
        "paper_bits_per_step": {"s3gd_uplink": costs.s3gd_uplink(M, N, K), "s3gd_total": costs.s3gd_mv(M, N, K),
                                "signsgd": costs.signsgd_mv(M, N), "packed_words": costs.packed_words_bits(M, K)},
    }
    if not is_variant and not args.graph:
        # the same step as the other entry: the three public calls beside the fused one (or the reverse)
        other = fused_step if args.three_calls else three_calls_step
        ms2, med2, kern2, live2, _ = measure(other, args.steps, args.warmup)
        log(f"[bench] {'fused' if args.three_calls else 'three calls'}: mean {ms2:.4f} ms, median {med2:.4f} ms")
        rec = {"entry": "s3gd_step (fused, vote not materialised)" if args.three_calls
               else "s3gd_topk_sign_encode + s3gd_majority_vote (int8 votes) + s3gd_apply_update",
               "ms_per_step": ms2, "ms_per_step_median_of_event_times": med2, "value": M * N / (ms2 * 1e-3),
               "unit": "gradient elements/s", "steps": args.steps, "warmup": args.warmup,
               "kernels_ms": {k: round(v["ms_avg"] * v["launches_per_step"], 5) for k, v in kern2.items()},
               "kernel_fractions": fractions(kern2, not args.three_calls)}
        b3 = g_bytes + 8.0 * M * K + 2.0 * N + 8.0 * n_voted  # + the int8 votes written and read
        if not args.three_calls:
            rec["step_bytes_as_built"] = b3
            rec["f_step"] = b3 / (ms2 * 1e-3) / HBM_PEAK
        out["fused" if args.three_calls else "three_calls"] = rec
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, datagen)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
