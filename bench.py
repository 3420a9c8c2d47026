#!/usr/bin/env python3
"""Benchmark of one S3GD-MV step (encode -> majority vote -> update) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C5]

A "step" is one pass of the whole hot path over one batch of synthetic gradients: the fused
C-ABI call s3gd_step on a resident [M, N] fp32 tensor.  Inputs are generated on the host from
the seeded recipes in paper_2302_07475_amd/datagen.py and are resident in HBM before the timed
region starts.  Prints ONE JSON line:

  value        M*N / t   gradient elements per second through one step
  roofline     the dominant kernel's algorithmic bytes per launch over its mean duration, measured
               with HIP events on the launch stream inside the timed region, against 8 TB/s
  cpu_baseline the CPU oracle timed on this machine's host cores on a bounded sample of the workload
"""
import argparse
import dataclasses
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK = 8.0e12  # bytes/s, MI355X published peak

# HBM bytes per launch (read + written) from rocprofv3 FETCH_SIZE / WRITE_SIZE, scaled by the factors a
# plain copy of known size gives (2.0 for FETCH_SIZE, 1.0 for WRITE_SIZE); figures and commands are in
# profiles/s3gd_step_C5_hbm_traffic.md.  Reported only for the workload and kernel they were taken on.
MEASURED_TRAFFIC_BYTES = {("C5", "filter"): 19.2000e9 + 0.0620e9}

# algorithmic bytes one launch of a kernel moves, per gradient element (4 = one fp32 read of G)
FULL_READ_KERNELS = {"hist_rows_0", "hist_rows_1", "hist_rows_2", "tile_count", "emit_rows", "filter"}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_baseline(cfg, datagen):
    """The oracle, as it stands, on a bounded sample: all M workers, the first N_s coordinates,
    K scaled to keep K/N.  Sorting is O(N log N), so the per-element rate at the full N is lower."""
    from oracle import s3gd_oracle as O
    n_s = min(cfg.N, max(1 << 16, (120_000_000 // cfg.M)))
    k_s = max(1, round(cfg.K * n_s / cfg.N))
    small = cfg.scaled(N=n_s, K=k_s)
    G = datagen.gradients(small)
    x = datagen.params(small)
    t0 = time.perf_counter()
    O.step(G, small.K, x, datagen.lr32(small))
    dt = time.perf_counter() - t0
    return {"value": cfg.M * n_s / dt, "unit": "gradient elements/s", "cores": 1, "kind": "oracle",
            "sample": f"all {cfg.M} workers, first {n_s} coordinates of {cfg.name}, K={k_s}, one step, {dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="C5", choices=["C1", "C2", "C3", "C4", "C5"])
    ap.add_argument("--three-calls", action="store_true", help="time encode, vote, update as separate calls")
    ap.add_argument("--memory", action="store_true",
                    help="time s3gd_step_ec: the step with the error-compensation memory (eta = 1), a second "
                         "[M, N] fp32 tensor read and rewritten every step (not the headline workload)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", type=float, default=0.0, metavar="GiB",
                    help="instead of the benchmark, run three plain device copies of this size; run it under "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE to get the factor between counter units and bytes")
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
    if args.calibrate_copy > 0:
        n = int(args.calibrate_copy * (1 << 30)) // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "plain copy", "bytes_read_per_copy": 4 * n, "bytes_written_per_copy": 4 * n}))
        return
    cfg = datagen.CONFIGS[args.workload]
    dev = torch.device("cuda:0")
    t0 = time.perf_counter()
    g, x = datagen.to_device(cfg, device="cuda:0")
    log(f"[bench] {cfg.name}: M={cfg.M} N={cfg.N} K={cfg.K} generated and uploaded in {time.perf_counter() - t0:.1f} s")
    M, N, K = cfg.M, cfg.N, cfg.K
    if args.sparsity > 0:
        K = max(1, min(N, int(round(args.sparsity * N))))
        cfg = dataclasses.replace(cfg, K=K)
    lr = float(datagen.lr32(cfg))
    ctx = s3gd.Context(M, N, K, device=0)
    words = torch.empty((M, K), dtype=torch.int32, device=dev)
    counts = torch.empty((M,), dtype=torch.int32, device=dev)
    tally = votes = None
    if args.three_calls:
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

    def one_step():
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
            ctx.step_acc(g, K, x, lr, words, counts, None, None)  # g plays the memory: each step's zeros stay in it
        elif args.memory:
            ctx.step_ec(g, err, 1.0, K, x, lr, words, counts, None, None)
        elif args.three_calls:
            ctx.topk_sign_encode(g, K, words, counts)
            ctx.majority_vote(words, counts, N, None, votes)
            ctx.apply_update(x, votes, lr)
        else:
            ctx.step(g, K, x, lr, words, counts, None, None)

    eager_step = one_step
    if args.graph:
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
    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    assert ctx.last_async_status() == 0
    general_rows = ctx.last_encode_info()[1]
    # per-kernel breakdown from a short eager pass with an event pair around every launch (not timed: the
    # hundred events per step it records cost a few per cent)
    ctx.profile_enable(1)
    for _ in range(3):
        eager_step()
    prof = ctx.profile_read()
    kern = {k: {"ms_avg": v[0] / v[1], "launches_per_step": v[1] / 3} for k, v in prof.items()}
    # timed region: only the selection pass (the dominant kernel) carries an event pair
    ctx.profile_enable(0 if args.graph else 2)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    live = {} if args.graph else ctx.profile_read()
    ctx.profile_enable(0)
    log(f"[bench] timed {args.steps} steps in {dt * 1e3:.2f} ms")
    for k, v in live.items():  # measured inside the timed region: these replace the figures of the breakdown pass
        kern[k] = {"ms_avg": v[0] / v[1], "launches_per_step": v[1] / args.steps}

    ms_step = dt * 1e3 / args.steps
    for k, v in sorted(kern.items(), key=lambda kv: -kv[1]["ms_avg"] * kv[1]["launches_per_step"]):
        log(f"[bench]   {k:14s} {v['ms_avg']:9.4f} ms x {v['launches_per_step']:.0f}" + ("  (timed region)" if k in live else ""))
    dom = max(kern, key=lambda k: kern[k]["ms_avg"])
    if dom == "randk":  # K gathered gradient entries and K words per row; nothing else of G is touched
        alg_bytes = 8.0 * M * K
    elif dom == "filter_mem":  # reads g~ and e, writes the new memory
        alg_bytes = 12.0 * M * N
    elif dom in FULL_READ_KERNELS:
        alg_bytes = 4.0 * M * N
    elif dom == "vote_momentum":
        # the momentum is read in full; where it is non-zero (everywhere, in the dense state) it is written back and
        # the parameter is read and written too
        alg_bytes = 4.0 * M * K + (16.0 * N if args.dense_state else 4.0 * N)
    else:  # the vote kernel dominates only when the gradient passes are cheaper than it
        alg_bytes = 8.0 * M * K + 8.0 * N
    achieved = alg_bytes / (kern[dom]["ms_avg"] * 1e-3)
    per_pass = 12.0 if args.memory else 4.0  # with the memory a pass reads g~ and e and writes e
    floor_bytes = per_pass * M * N + 8.0 * M * K + 8.0 * N
    # the general route's kernels are always enqueued and return at once unless a row needs them
    full_reads = sum(v["launches_per_step"] for k, v in kern.items()
                     if k in ("filter", "filter_mem") or (k in FULL_READ_KERNELS and general_rows > 0))
    out = {
        "metric": "gradient elements/sec per S3GD-MV step (M*N/t)",
        "value": M * N / (ms_step * 1e-3),
        "unit": "gradient elements/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32 keys of fp32 gradients, int32 tally, fp32 update", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: M={M} workers, N={N} fp32 coords, K={K}", "recipe": cfg.recipe,
                   "entry": "s3gd_step_randk (Algorithm 2)" if args.randk else
                            "encode, pack, unpack, vote_update (messages through the wire format)" if args.wire else
                            ("s3gd_step_momentum (mu=0.9" + (", with memory" if args.memory else "") +
                             (", dense momentum state)" if args.dense_state else ", momentum starts at zero)")) if args.momentum else
                            "s3gd_step_acc (fused, the memory already holds the compensated gradients)" if args.memory_acc else
                            "s3gd_step_ec (fused, with error-compensation memory, eta=1)" if args.memory else
                            ("three calls" if args.three_calls else "s3gd_step (fused, vote not materialised)"),
                   "rows_on_general_path": general_rows, "launch": "HIP graph replay" if args.graph else "eager"},
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": achieved / 1e9, "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK,
                     "duration_from": "HIP events inside the timed region" if dom in live else "HIP events, eager pass before the timed region",
                     "traffic": MEASURED_TRAFFIC_BYTES.get((cfg.name, dom)) if not (args.three_calls or args.memory or args.memory_acc or args.momentum or args.wire or args.randk) else None},
        "step_roofline": {"full_reads_of_G_per_step": full_reads,
                          "f_alg": floor_bytes / (ms_step * 1e-3) / HBM_PEAK,
                          "floor_bytes": floor_bytes,
                          "step_bytes_as_built": per_pass * M * N * full_reads + 8.0 * M * K,
                          "f_step": (per_pass * M * N * full_reads + 8.0 * M * K) / (ms_step * 1e-3) / HBM_PEAK},
        "kernels_ms": {k: round(v["ms_avg"] * v["launches_per_step"], 5) for k, v in kern.items()},
        "paper_bits_per_step": {"s3gd_uplink": costs.s3gd_uplink(M, N, K), "s3gd_total": costs.s3gd_mv(M, N, K),
                                "signsgd": costs.signsgd_mv(M, N), "packed_words": costs.packed_words_bits(M, K)},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, datagen)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
