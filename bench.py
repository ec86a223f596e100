#!/usr/bin/env python3
"""Benchmark of the broadcast hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]
                    [--algo chain|direct|binomial|fanout|auto] [--chunk BYTES] [--lanes N] [--stages N] [--trip BYTES] [--block THREADS]
                    [--rank-stride BYTES]

A "step" is one whole broadcast (every chunk over every hop) of the workload's
message to all P virtual ranks, with all buffers already resident in HBM.
The default workload is the top of the message-size sweep: 64 MiB to P=8.
Prints ONE JSON line.  `value` is the effective bandwidth 2(P-1)M / t of the
pipelined chain in GB/s (algorithmic bytes: each delivered byte is read once
from the left neighbour and written once); `ms_per_step` is the latency.
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

KiB, MiB, GiB = 1 << 10, 1 << 20, 1 << 30
HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E peak

# name -> (P, root, message bytes, seed, what it stands for)
WORKLOADS = {
    "cfg1": (4, 0, 1 * MiB, 0, "1 MiB fp32 uniform[-1,1), P=4"),
    "cfg2": (8, 0, 64 * MiB, 1, "64 MiB random bytes, P=8 (top of the message-size sweep)"),
    "cfg3": (16, 0, 553430176, 2, "VGG-16 parameters packed (138M fp32, N(0,0.01)), P=16"),
    "cfg4": (32, 0, 512 * MiB, 3, "512 MiB random bytes, P=32"),
    "cfg5": (64, 17, 1 * GiB, 4, "1 GiB random bytes, P=64, root 17"),
    "cfg5b": (64, 17, 4 * KiB, 4, "4 KiB random bytes back to back, P=64, root 17 (use --steps 1000)"),
}

# HBM traffic per launch of the dominant kernel, measured with rocprofv3 --pmc
# FETCH_SIZE and --pmc WRITE_SIZE (KiB per dispatch; summaries under profiles/).
# FETCH_SIZE is scaled by the factor a plain copy of known size shows in the same
# run (a 64 MiB copy reads 32786.9 KiB on the counter: factor 1.999); WRITE_SIZE
# reads the true size (factor 1.000).  Workloads without a profile report null.
# The chain's traffic is BELOW its algorithmic bytes: part of what a wave reads
# back inside a stage is served by the CU's vector L1 and never reaches the fabric.
MEASURED_TRAFFIC_BYTES = {
    ("cfg2", "chain"): int((138361.4 * (65536.0 / 32787.3) + 459264.0) * 1024),
    ("cfg2", "direct"): int((32785.0 * (65536.0 / 32786.9) + 65536.0) * 1024),
    ("cfg3", "chain"): int((1022961.4 * (540459.2 / 270254.7) + 8112519.3) * 1024),
    ("cfg4", "chain"): int((1598370.7 * (524288.0 / 262166.7) + 16258400.0) * 1024),
    ("cfg5", "chain"): int((5878015.7 * (1048576.0 / 524315.7) + 66071232.0) * 1024),
    # the chain reduction (--op reduce): (P + 3) M with two stages -- every contribution read once, the running
    # sum written to and read from the scratch buffer once, the result written once
    ("cfg2", "reduce"): int((295938.8 * (65536.0 / 32787.3) + 131584.0) * 1024),
    ("cfg4", "reduce"): int((8656715.8 * (524288.0 / 262166.7) + 1052672.0) * 1024),
}


def make_message(name, seed, nbytes, custom=False):
    from paper_1707_09414_amd import inputs

    if custom:
        return inputs.random_bytes(seed, nbytes)
    if name == "cfg1":
        return inputs.uniform_fp32_message(seed, nbytes // 4)
    if name == "cfg3":
        return inputs.vgg16_packed_message(seed)[0]
    return inputs.random_bytes(seed, nbytes)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg2", choices=sorted(WORKLOADS))
    ap.add_argument("--algo", default="chain", choices=["chain", "direct", "binomial", "fanout", "auto"])
    ap.add_argument("--chunk", type=int, default=0, help="chain chunk bytes (0 = tuned table / built-in rule)")
    ap.add_argument("--lanes", type=int, default=0, help="wavefronts per chain hop (0 = automatic)")
    ap.add_argument("--stages", type=int, default=0, help="chain stages (0 = tuned table / built-in rule)")
    ap.add_argument("--op", choices=["bcast", "reduce"], default="bcast",
                    help="reduce: the chain reduction (fp32 sum to the root) at the workload's P and size instead of the broadcast")
    ap.add_argument("--rank-stride", type=int, default=0,
                    help="place the rank buffers in one allocation this many bytes apart (>= message bytes, multiple of 256; "
                         "0 = one allocation per rank)")
    ap.add_argument("--block", type=int, default=0, help="chain workgroup size, 64, 128 or 256 (0 = default)")
    ap.add_argument("--trip", type=int, default=0, help="chain trip bytes, 3072 or 4096 (0 = tuned table / 4096)")
    ap.add_argument("--ranks", type=int, default=0, help="override the workload's P (experiments)")
    ap.add_argument("--bytes", type=int, default=0, help="override the workload's message size (experiments)")
    ap.add_argument("--no-sweep", action="store_true", help="skip the per-message-size latency table (cfg2 only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-verify", action="store_true")
    args = ap.parse_args()

    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (P virtual ranks are buffers in one GPU's HBM); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_1707_09414_amd import binding as B
    from paper_1707_09414_amd import inputs
    from paper_1707_09414_amd import tuned

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    P, root, M, seed, what = WORKLOADS[args.workload]
    if args.ranks or args.bytes:
        P = args.ranks or P
        M = args.bytes or M
        root = root % P
        what = "custom: %d random bytes, P=%d" % (M, P)
    algo = {"chain": B.BCAST_ALGO_CHAIN, "direct": B.BCAST_ALGO_DIRECT, "binomial": B.BCAST_ALGO_BINOMIAL,
            "fanout": B.BCAST_ALGO_FANOUT, "auto": B.BCAST_ALGO_AUTO}[args.algo]

    table = tuned.load_default_table()  # installs the shipped MI355X table if present
    if args.op == "reduce":
        return bench_reduce(args, B, torch, P, root, M, seed, what)

    msg = make_message(args.workload, seed, M, custom=bool(args.ranks or args.bytes))
    assert msg.nbytes == M
    d_msg = torch.from_numpy(msg).cuda()
    bufs = []
    arena = None
    if args.rank_stride:
        if args.rank_stride < M or args.rank_stride % 256:
            print("bench.py: --rank-stride must be >= the message size and a multiple of 256", file=sys.stderr)
            return 2
        arena = torch.empty(args.rank_stride * (P - 1) + M, dtype=torch.uint8, device="cuda")
    for r in range(P):
        t = arena[r * args.rank_stride: r * args.rank_stride + M] if arena is not None else torch.empty(M, dtype=torch.uint8, device="cuda")
        if r == root:
            t.copy_(d_msg)
        else:
            t.fill_(inputs.FILL_BYTE)
        bufs.append(t)
    del d_msg

    plan = B.bcast_plan_create(P, M, args.chunk, algo)
    if args.lanes:
        B.bcast_plan_set_lanes(plan, args.lanes)
    if args.stages:
        B.bcast_plan_set_stages(plan, args.stages)
    if args.trip:
        B.bcast_plan_set_trip(plan, args.trip)
    if args.block:
        B.bcast_plan_set_block_threads(plan, args.block)
    info = B.bcast_plan_info(plan, M, bufs)
    stream = torch.cuda.current_stream()
    ptrs = B.RankPointers(bufs)  # marshalled once: at small sizes building the pointer array costs more than the broadcast

    for _ in range(args.warmup):
        B.bcast_run(plan, ptrs, root, M, stream)
    torch.cuda.synchronize()

    # timed region: exactly --steps broadcasts back to back, bracketed by
    # synchronize + wall clock (the whole-job figure) and by one pair of HIP
    # events recorded on the launch stream (torch's current stream is the stream
    # we launch on): elapsed / steps is the average launch duration, gaps between
    # consecutive launches included
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record(stream)
    for _ in range(args.steps):
        B.bcast_run(plan, ptrs, root, M, stream)
    e1.record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    status, detail = B.bcast_plan_status(plan)
    if status != B.BCAST_OK:
        print("bench.py: plan status %d detail %x" % (status, detail), file=sys.stderr)
        return 1
    wall_ms = (t1 - t0) * 1e3 / args.steps
    avg_launch_ms = e0.elapsed_time(e1) / args.steps

    # every rank must now hold the root's message: one rank at a time over PCIe
    verified = None
    if not args.no_verify:
        verified = True
        for r in range(P):
            if not np.array_equal(bufs[r].cpu().numpy(), msg):
                verified = False
                print("bench.py: rank %d does not hold the root's message" % r, file=sys.stderr)
        if not verified:
            return 1

    algorithmic = int(info["algorithmic_bytes"])
    value = algorithmic / (wall_ms * 1e-3) / 1e9
    achieved = algorithmic / (avg_launch_ms * 1e-3) / 1e9
    custom = bool(args.ranks or args.bytes or args.chunk or args.lanes or args.stages or args.trip or args.block or args.rank_stride)
    traffic = None if custom else MEASURED_TRAFFIC_BYTES.get((args.workload, args.algo))

    sweep = None
    if args.workload == "cfg2" and not custom and not args.no_sweep:
        sweep = size_sweep(B, torch, bufs, P, root, M, stream)

    per_tensor = None
    if args.workload == "cfg3" and not custom and not args.no_sweep:
        per_tensor = vgg_tensor_by_tensor(B, torch, bufs, P, root, stream)

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(P, root, M, int(info["chunk_bytes"]) or M, msg)

    out = {
        "metric": "broadcast effective HBM bandwidth 2(P-1)M/t (GB/s) at the stated message size and P; latency in ms_per_step",
        "value": round(value, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(wall_ms, 5),
        "latency_us": round(wall_ms * 1e3, 2),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u8",
        "data": "synthetic",
        "config": {
            "workload": "%s: %s, root %d" % (args.workload, what, root),
            "P": P, "message_bytes": M, "algo": B.ALGO_NAMES[info["algo"]],
            "chunk_bytes": int(info["chunk_bytes"]), "nchunks": int(info["nchunks"]), "stages": info["stages"], "hops_per_stage": info["hops_per_stage"], "trip_bytes": info["trip_bytes"], "block_threads": info["block_threads"], "rank_stride": args.rank_stride,
            "lanes": info["lanes"],
            "grid_blocks": info["grid_blocks"], "vec_bytes": info["vec_bytes"], "launches_per_step": info["launches"],
            "tuning_table": table,
        },
        "delivered_GBps": round((P - 1) * M / (wall_ms * 1e-3) / 1e9, 2),
        "verified_bit_exact": verified,
        "roofline": {
            "bound": "hbm",
            "achieved": round(achieved, 2),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4),
            "traffic": traffic,
            # the same counters as a rate: fabric bytes per launch / launch duration, and against the HBM peak
            "traffic_GBps": round(traffic / (avg_launch_ms * 1e-3) / 1e9, 2) if traffic else None,
            "traffic_frac": round(traffic / (avg_launch_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4) if traffic else None,
            "kernel": ("bcast::chain_kernel<%d, %d, %s>" % (info["vec_bytes"], info["trip_bytes"] // 1024, "true" if M <= (2 << 20) else "false"))
            if info["algo"] == B.BCAST_ALGO_CHAIN else B.ALGO_NAMES[info["algo"]],
            "algorithmic_bytes_per_launch": algorithmic,
            "avg_launch_ms": round(avg_launch_ms, 5),
        },
        "cpu_baseline": cpu,
        "sweep": sweep,
        "per_tensor": per_tensor,
    }
    print(json.dumps(out))
    plan.destroy()
    return 0


def bench_reduce(args, B, torch, P, root, M, seed, what):
    """The pipelined chain reduction (fp32 sum to the root) at the workload's rank
    count and message size: every rank contributes M bytes of N(0, 0.01) values
    (one seeded draw, shifted and rescaled per rank).  Algorithmic bytes: every
    input read once, the result written once, (P + 1) M."""
    import numpy as np

    import oracle

    count = M // 4
    rng = np.random.default_rng(seed)
    base = rng.normal(0.0, 0.01, size=count).astype(np.float32)
    d_base = torch.from_numpy(base).cuda()
    send = [torch.roll(d_base, 4099 * r) * (1.0 + r / 64.0) for r in range(P)]
    recv = torch.empty(count, dtype=torch.float32, device="cuda")
    plan = B.bcast_plan_create(P, count * 4, args.chunk, B.BCAST_ALGO_CHAIN)
    if args.lanes:
        B.bcast_plan_set_lanes(plan, args.lanes)
    if args.stages:
        B.bcast_plan_set_stages(plan, args.stages)
    info = B.bcast_reduce_info(plan, count)
    stream = torch.cuda.current_stream()
    ptrs = B.RankPointers(send)
    for _ in range(max(1, args.warmup)):
        B.bcast_reduce_sum_f32(plan, ptrs, recv, root, count, stream)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record(stream)
    for _ in range(args.steps):
        B.bcast_reduce_sum_f32(plan, ptrs, recv, root, count, stream)
    e1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    avg_launch_ms = e0.elapsed_time(e1) / args.steps
    st, detail = B.bcast_plan_status(plan)
    if st != B.BCAST_OK:
        print("bench.py: plan status %d (detail %#x)" % (st, detail), file=sys.stderr)
        return 1

    # bit-exact against the oracle on a prefix (a sum is element-wise, so a prefix stands alone)
    sample = min(count, 4 << 20)
    host = np.stack([s[:sample].cpu().numpy() for s in send])
    verified = None
    if not args.no_verify:
        want, _ = oracle.chain_reduce_f32(host, P, root, sample, max(1, int(info["chunk_bytes"]) // 4))
        verified = bool(np.array_equal(recv[:sample].cpu().numpy().view(np.uint32), want.view(np.uint32)))
        if not verified:
            print("bench.py: the reduction differs from the oracle", file=sys.stderr)
            return 1
    cpu = None
    if not args.no_cpu_baseline:
        reps, t = 0, 0.0
        while t < 10.0 or reps < 3:
            c0 = time.perf_counter()
            oracle.chain_reduce_f32(host, P, root, sample, max(1, int(info["chunk_bytes"]) // 4))
            t += time.perf_counter() - c0
            reps += 1
        cpu = {"value": round((P + 1) * sample * 4 / (t / reps) / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": "oracle.chain_reduce_f32, P=%d, first %d elements, %d reps, %.1f ms each" % (P, sample, reps, 1e3 * t / reps)}
    algorithmic = (P + 1) * count * 4
    custom = bool(args.ranks or args.bytes or args.chunk or args.lanes or args.stages)
    traffic = None if custom else MEASURED_TRAFFIC_BYTES.get((args.workload, "reduce"))
    out = {
        "metric": "chain reduction (fp32 sum to the root) effective HBM bandwidth (P+1)M/t (GB/s); latency in ms_per_step",
        "value": round(algorithmic / (wall_ms * 1e-3) / 1e9, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(wall_ms, 5), "latency_us": round(wall_ms * 1e3, 2), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s as a reduction: P=%d contributions of %d fp32 values N(0, 0.01), root %d" % (args.workload, P, count, root),
                   "P": P, "message_bytes": count * 4, "algo": "chain_reduce", "chunk_bytes": int(info["chunk_bytes"]),
                   "nchunks": int(info["nchunks"]), "stages": info["stages"], "lanes": info["lanes"], "grid_blocks": info["grid_blocks"]},
        "verified_bit_exact": verified,
        "roofline": {"bound": "hbm", "achieved": round(algorithmic / (avg_launch_ms * 1e-3) / 1e9, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(algorithmic / (avg_launch_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4), "traffic": traffic,
                     "traffic_GBps": round(traffic / (avg_launch_ms * 1e-3) / 1e9, 2) if traffic else None,
                     "traffic_frac": round(traffic / (avg_launch_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4) if traffic else None,
                     "kernel": "bcast::reduce_kernel<1, 16>" if count * 4 <= (2 << 20) else "bcast::reduce_kernel<4, 4>", "algorithmic_bytes_per_launch": algorithmic, "avg_launch_ms": round(avg_launch_ms, 5)},
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))
    plan.destroy()
    return 0


def vgg_tensor_by_tensor(B, torch, bufs, P, root, stream):
    """The same VGG-16 parameters broadcast as 32 messages, one per tensor, each
    with the tuned choice (AUTO), back to back: the alternative to packing them
    into one message.  Mean of a few passes between two HIP events."""
    from paper_1707_09414_amd import inputs

    spans, off = [], 0
    for n in inputs.vgg16_tensor_bytes():
        spans.append((off, n))
        off += n
    plan = B.bcast_plan_create(P, max(n for _, n in spans), 0, B.BCAST_ALGO_AUTO)
    views = [(B.RankPointers([b[o: o + n] for b in bufs]), n) for o, n in spans]
    algos = {}
    for ptrs, n in views:
        name = B.ALGO_NAMES[B.bcast_plan_info(plan, n, ptrs)["algo"]]
        algos[name] = algos.get(name, 0) + 1
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    passes = 5
    for it in range(passes + 1):
        if it == 1:
            e0.record(stream)
        for ptrs, n in views:
            B.bcast_run(plan, ptrs, root, n, stream)
    e1.record(stream)
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / passes
    plan.destroy()
    total = sum(n for _, n in spans)
    return {"tensors": len(spans), "ms_per_pass": round(ms, 4), "algorithms": algos,
            "GBps": round(2 * (P - 1) * total / (ms * 1e-3) / 1e9, 1)}


def size_sweep(B, torch, bufs, P, root, max_bytes, stream):
    """Latency per message size (4 B .. the workload's size, powers of two) at the
    workload's P, measured live: the tuned choice (AUTO) and the chain, each as
    the mean of a batch of back-to-back runs between two HIP events."""
    rows = []
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ptrs = B.RankPointers(bufs)

    def time_plan(plan, M):
        reps = 200 if M <= (1 << 20) else 20
        for _ in range(3):
            B.bcast_run(plan, ptrs, root, M, stream)
        e0.record(stream)
        for _ in range(reps):
            B.bcast_run(plan, ptrs, root, M, stream)
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / reps  # microseconds

    M = 4
    while M <= max_bytes:
        auto = B.bcast_plan_create(P, M, 0, B.BCAST_ALGO_AUTO)
        chain = B.bcast_plan_create(P, M, 0, B.BCAST_ALGO_CHAIN)
        ai = B.bcast_plan_info(auto, M, bufs)
        ci = B.bcast_plan_info(chain, M, bufs)
        a_us, c_us = time_plan(auto, M), time_plan(chain, M)
        rows.append({
            "bytes": M, "auto_algo": B.ALGO_NAMES[ai["algo"]], "auto_us": round(a_us, 2),
            "chain_us": round(c_us, 2), "chain_chunk_bytes": int(ci["chunk_bytes"]), "chain_stages": ci["stages"],
            "chain_GBps": round(2 * (P - 1) * M / c_us / 1e3, 1),
            "chain_frac_of_peak": round(2 * (P - 1) * M / c_us / 1e3 / HBM_PEAK_GBS, 4),
        })
        auto.destroy()
        chain.destroy()
        M *= 2
    return rows


def cpu_baseline(P, root, M, C, msg):
    """The CPU oracle's chain simulation, as it stands, timed on this host on a
    bounded sample: the same P and chunk size, the message cut to at most 64 MiB,
    repeated for about ten seconds."""
    import numpy as np

    import oracle

    sample = min(M, 64 * MiB)
    host = np.full((P, sample), 0xFF, dtype=np.uint8)
    host[root] = msg[:sample]
    oracle.chain_bcast(host, P, root, sample, C)  # touch pages once
    reps = 0
    t0 = time.perf_counter()
    while True:
        oracle.chain_bcast(host, P, root, sample, C)
        reps += 1
        dt = time.perf_counter() - t0
        if dt > 10.0 and reps >= 3:
            break
    sec = dt / reps
    return {
        "value": round(2 * (P - 1) * sample / sec / 1e9, 3),
        "unit": "GB/s",
        "cores": 1,
        "kind": "oracle",
        "sample": "oracle.chain_bcast, P=%d, first %d bytes of the message, C=%d, %d reps, %.1f ms each"
                  % (P, sample, C, reps, sec * 1e3),
    }


if __name__ == "__main__":
    sys.exit(main())
