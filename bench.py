#!/usr/bin/env python3
"""Benchmark of the broadcast hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workloads cfg1,cfg2,...]
                    [--no-cpu-baseline] [--no-verify] [--quick]
    python bench.py --leg WORKLOAD:VARIANT [--steps K]      (one variant only: the target of rocprofv3 runs)

A "step" is one whole broadcast (every chunk over every hop) of a workload's
message to all P virtual ranks, with all buffers already resident in HBM.  The
default run measures every benchmark configuration and prints ONE JSON line:

  * headline (`value`, `ms_per_step`, `config`, `roofline`): the largest one,
    cfg5a -- 1 GiB to P = 64 ranks, root 17 -- with the tuned pipelined chain;
    exactly --steps broadcasts back to back between two synchronisations.
  * `configs`: one row per configuration (cfg1, cfg2, cfg3, cfg4, cfg5a, cfg5b),
    each with its variants -- the tuned chain (whichever chain kernel the table
    holds), the chain with one wavefront per rank (the literal Sec. IV-B picture),
    the chain with one wavefront per stage, the chain with one stage per hop and
    every hand-off through a flag in memory, direct (Eq. 1), the one-die fan-out
    -- timed run by run with HIP events: median, min and mean latency,
    algorithmic GB/s (2(P-1)M/t), the fraction of the 8 TB/s HBM peak that the
    kernel's own minimum of HBM bytes ((P-1)M written + one read of M per stage)
    needs at that time (`floor_frac`, <= 1 by construction), and the rocprofv3
    counter traffic of the same launch configuration read from profiles/
    (`traffic_frac`); cold-cache rows, the message-size sweep, VGG-16 tensor by
    tensor, the 1000 x 4 KiB bursts, and the chain reduction.
  * `cpu_baseline`: the CPU oracle's chain simulation, as it stands, on one host
    core and on all cores, on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

KiB, MiB, GiB = 1 << 10, 1 << 20, 1 << 30
HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E peak

# name -> (P, root, message bytes, seed, what it stands for)
WORKLOADS = {
    "cfg1": (4, 0, 1 * MiB, 0, "1 MiB fp32 uniform[-1,1), P=4, 64 KiB chunks"),
    "cfg2": (8, 0, 64 * MiB, 1, "64 MiB random bytes, P=8 (top of the message-size sweep)"),
    "cfg3": (16, 0, 553430176, 2, "VGG-16 parameters packed (138M fp32, N(0,0.01)), P=16"),
    "cfg4": (32, 0, 512 * MiB, 3, "512 MiB random bytes, P=32"),
    "cfg5a": (64, 17, 1 * GiB, 4, "1 GiB random bytes, P=64, root 17"),
    "cfg5b": (64, 17, 4 * KiB, 4, "1000 back-to-back 4 KiB broadcasts, P=64, root 17"),
}
HEADLINE = "cfg5a"
VARIANTS = {
    "cfg1": ["chain", "auto"],
    "cfg2": ["chain", "chain_wave_per_rank", "chain_wave_per_stage", "chain_stage_per_hop", "direct", "fanout"],
    "cfg3": ["chain", "chain_wave_per_rank", "chain_wave_per_stage", "direct"],
    "cfg4": ["chain", "chain_wave_per_rank", "chain_wave_per_stage", "chain_stage_per_hop", "direct", "fanout"],
    "cfg5a": ["chain", "chain_wave_per_rank", "chain_wave_per_stage", "chain_stage_per_hop", "direct", "fanout"],
    "cfg5b": ["auto", "chain", "chain_wave_per_rank"],
}
PROFILE_DIR = os.path.join(ROOT, "profiles")


# ---------------------------------------------------------------------------
# rocprofv3 summaries under profiles/: HBM-side traffic per launch
# ---------------------------------------------------------------------------
def parse_profile(path):
    """One profiles/*.txt summary -> dict, or None if it is not one of ours.

    The file carries a line `# leg: {json}` (the workload, variant and launch
    geometry of the run it was made from: what `bench.py --leg` printed), the
    per-kernel duration table of `rocprofv3 --kernel-trace --stats` and the
    FETCH_SIZE / WRITE_SIZE tables of two `--pmc` runs (KiB per dispatch).  The
    counters are calibrated against the runtime's own copy of the message in
    the same run (`__amd_rocclr_copyBuffer`, reads and writes `message_bytes`).
    """
    leg, section, rows = None, None, {"stats": {}, "FETCH_SIZE": {}, "WRITE_SIZE": {}}
    for line in open(path):
        if line.startswith("# leg:"):
            leg = json.loads(line[len("# leg:"):])
        elif line.startswith("## kernel-trace"):
            section = "stats"
        elif line.startswith("## --pmc FETCH_SIZE"):
            section = "FETCH_SIZE"
        elif line.startswith("## --pmc WRITE_SIZE"):
            section = "WRITE_SIZE"
        elif section and line.strip() and not line.startswith(("#", "kernel ")):
            if section == "stats":
                m = re.match(r"(.*?)\s+(\d+)\s+(\d+)\s+(\d+)\s+(\d+)\s+(\d+)\s*$", line)
                if m:
                    rows["stats"][m.group(1).strip()] = {"calls": int(m.group(2)), "avg_ns": float(m.group(4))}
            else:
                m = re.match(r"(.*?)\s+(FETCH_SIZE|WRITE_SIZE)\s+(\d+)\s+([\d.]+)\s+([\d.]+)\s+([\d.]+)\s*$", line)
                if m:
                    rows[section][m.group(1).strip()] = {"calls": int(m.group(3)), "avg_kib": float(m.group(4))}
    if leg is None:
        return None
    return {"leg": leg, "rows": rows, "path": os.path.basename(path)}


def profile_traffic(prof):
    """(bytes per launch, avg kernel ns, calibration factors) of a parsed summary."""
    leg, rows = prof["leg"], prof["rows"]
    kernel = leg["kernel"]
    msg_kib = leg["calibration_copy_bytes"] / 1024.0

    def pick(table, name):
        hits = [v for k, v in table.items() if name in k]
        if len(hits) != 1:
            raise ValueError("%s: %d rows match %r" % (prof["path"], len(hits), name))
        return hits[0]

    if leg["calibration_copy_bytes"] >= MiB:
        f_cal = msg_kib / pick(rows["FETCH_SIZE"], "__amd_rocclr_copyBuffer")["avg_kib"]
        w_cal = msg_kib / pick(rows["WRITE_SIZE"], "__amd_rocclr_copyBuffer")["avg_kib"]
    else:
        # a copy of a few KiB is lost in the counters' fixed overheads: use what every large copy shows
        # (FETCH_SIZE reads half the bytes, WRITE_SIZE all of them)
        f_cal, w_cal = 2.0, 1.0
    fetch = pick(rows["FETCH_SIZE"], kernel)["avg_kib"] * f_cal
    write = pick(rows["WRITE_SIZE"], kernel)["avg_kib"] * w_cal
    launches = leg.get("launches_per_step", 1)
    return {
        "bytes": int((fetch + write) * 1024 * launches), "fetch_bytes": int(fetch * 1024 * launches),
        "write_bytes": int(write * 1024 * launches), "avg_kernel_ns": pick(rows["stats"], kernel)["avg_ns"],
        "fetch_factor": round(f_cal, 4), "write_factor": round(w_cal, 4), "file": prof["path"],
    }


def load_profiles():
    out = {}
    if os.path.isdir(PROFILE_DIR):
        for name in sorted(os.listdir(PROFILE_DIR)):
            if name.endswith(".txt"):
                p = parse_profile(os.path.join(PROFILE_DIR, name))
                if p:
                    out[(p["leg"]["workload"], p["leg"]["variant"])] = p
    return out


def traffic_for(profiles, workload, variant, geometry):
    """Counter traffic of this launch configuration, or None with the reason."""
    prof = profiles.get((workload, variant))
    if prof is None:
        return None, "no profile"
    if prof["leg"]["geometry"] != geometry:
        return None, "profile %s was made with another launch geometry" % prof["path"]
    try:
        return profile_traffic(prof), None
    except (ValueError, KeyError, ZeroDivisionError) as e:
        return None, str(e)


# ---------------------------------------------------------------------------
# workloads and variants
# ---------------------------------------------------------------------------
def make_message(name, seed, nbytes):
    from paper_1707_09414_amd import inputs

    if name == "cfg1":
        return inputs.uniform_fp32_message(seed, nbytes // 4)
    if name == "cfg3":
        return inputs.vgg16_packed_message(seed)[0]
    return inputs.random_bytes(seed, nbytes)


def make_plan(B, name, variant, P, M):
    """The plan of one variant: what is requested, everything else is the
    library's choice (tuning table, else its rules)."""
    if variant == "auto":
        return B.bcast_plan_create(P, M, 0, B.BCAST_ALGO_AUTO)
    if variant == "direct":
        return B.bcast_plan_create(P, M, 0, B.BCAST_ALGO_DIRECT)
    if variant == "fanout":
        return B.bcast_plan_create(P, M, 0, B.BCAST_ALGO_FANOUT)
    if variant == "binomial":
        return B.bcast_plan_create(P, M, 0, B.BCAST_ALGO_BINOMIAL)
    if variant == "chain":
        # cfg1 fixes its chunk size (64 KiB: 16 chunks)
        return B.bcast_plan_create(P, M, 64 * KiB if name == "cfg1" else 0, B.BCAST_ALGO_CHAIN)
    if variant == "chain_wave_per_rank":
        plan = B.bcast_plan_create(P, M, 0, B.BCAST_ALGO_CHAIN)
        B.bcast_plan_set_chain_waves(plan, B.BCAST_CHAIN_WAVE_PER_RANK)
        return plan
    if variant == "chain_wave_per_stage":
        plan = B.bcast_plan_create(P, M, 0, B.BCAST_ALGO_CHAIN)
        B.bcast_plan_set_chain_waves(plan, B.BCAST_CHAIN_WAVE_PER_STAGE)
        return plan
    if variant == "chain_stage_per_hop":
        # one stage per receiving rank, every hand-off through a flag in memory, 4 MiB chunks
        plan = B.bcast_plan_create(P, M, min(4 * MiB, max(16, (M + 15) // 16 * 16)), B.BCAST_ALGO_CHAIN)
        B.bcast_plan_set_chain_waves(plan, B.BCAST_CHAIN_WAVE_PER_STAGE)
        B.bcast_plan_set_stages(plan, P - 1)
        B.bcast_plan_set_trip(plan, 4096)
        return plan
    raise ValueError(variant)


def geometry_of(B, info):
    return {"algo": B.ALGO_NAMES[info["algo"]], "chunk_bytes": int(info["chunk_bytes"]), "nchunks": int(info["nchunks"]),
            "stages": info["stages"], "hops_per_stage": info["hops_per_stage"], "lanes": info["lanes"], "trip_bytes": info["trip_bytes"],
            "rank_waves": info["rank_waves"], "grid_blocks": info["grid_blocks"], "block_threads": info["block_threads"],
            "vec_bytes": info["vec_bytes"], "launches": info["launches"]}


def kernel_name(info, B):
    if info["algo"] == B.BCAST_ALGO_CHAIN:
        if info["rank_waves"]:
            return "bcast::rank_chain_kernel<%d, %d>" % (info["vec_bytes"], info["trip_bytes"] // 1024)
        # third parameter: in-stage stores written through (0) or back (1); bench.py sets no cache policies of its own
        return "bcast::chain_kernel<%d, %d, %d>" % (info["vec_bytes"], info["trip_bytes"] // 1024, int(info["stage_store"] == B.BCAST_STORE_BACK))
    return {B.BCAST_ALGO_DIRECT: "bcast::pair_copy_kernel<%d>", B.BCAST_ALGO_BINOMIAL: "bcast::pair_copy_kernel<%d>",
            B.BCAST_ALGO_FANOUT: "bcast::fanout_kernel<%d>", B.BCAST_ALGO_KNOMIAL_PIPELINED: "bcast::tree_kernel<%d>",
            B.BCAST_ALGO_KNOMIAL: "bcast::ranged_copy_kernel<%d>", B.BCAST_ALGO_SCATTER_ALLGATHER: "bcast::ranged_copy_kernel<%d>"}[info["algo"]] % info["vec_bytes"]


def floor_bytes(B, info, P, M):
    """The least HBM traffic the variant's schedule needs on one die: every
    receiving rank's buffer written once, plus what has to be read out of memory
    rather than out of the compute unit that wrote it -- the message once per
    stage for the chain (stage 1 reads the root, every later stage what the stage
    before it stored), once per launch for the copy algorithms."""
    if info["algo"] == B.BCAST_ALGO_CHAIN:
        return (P - 1) * M + info["stages"] * M
    if info["algo"] == B.BCAST_ALGO_FANOUT:
        return P * M
    return 2 * (P - 1) * M


def stats_us(samples_ms):
    s = sorted(samples_ms)
    n = len(s)
    med = s[n // 2] if n % 2 else 0.5 * (s[n // 2 - 1] + s[n // 2])
    return {"median_us": round(med * 1e3, 3), "min_us": round(s[0] * 1e3, 3), "mean_us": round(sum(s) / n * 1e3, 3), "reps": n}


def time_runs(torch, run, stream, warmup, reps, before_each=None):
    """`reps` runs, each between its own pair of HIP events on `stream` (torch's
    current stream, the one the library launches on); milliseconds per run."""
    for _ in range(warmup):
        run()
    torch.cuda.synchronize()
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for e0, e1 in pairs:
        if before_each is not None:
            before_each()
        e0.record(stream)
        run()
        e1.record(stream)
    torch.cuda.synchronize()
    return [e0.elapsed_time(e1) for e0, e1 in pairs]


def reps_for(M, quick):
    if quick:
        return 5
    return 200 if M < MiB else 20


PLACED_NAMES = {0: "a slab was taken where it fell", 1: "one label only: nothing to tell apart", 2: "placed, confirmed by measurement"}
PLACE_MIN_BYTES = 8 * MiB  # smaller rank buffers are allocated plainly: their broadcasts are bound by latency, not by memory


class _DeviceSpan:
    """Device memory the library allocated, described the way torch reads foreign device arrays."""

    def __init__(self, ptr, nbytes):
        self.__cuda_array_interface__ = {"shape": (int(nbytes),), "typestr": "|u1", "data": (int(ptr), False), "version": 2}


def tensor_at(torch, ptr, nbytes):
    return torch.as_tensor(_DeviceSpan(ptr, nbytes), device="cuda")


class Placed:
    """Device buffers from bcast_buffers_alloc (library=True) or from torch."""

    def __init__(self, B, torch, sizes, regions, library):
        self.B, self.ptrs = B, None
        if library:
            self.ptrs, verdict = B.bcast_buffers_alloc(sizes, regions)
            self.bufs = [tensor_at(torch, p, n) for p, n in zip(self.ptrs, sizes)]
            self.how = {"by": "bcast_buffers_alloc", "verdict": PLACED_NAMES[verdict]}
        else:
            self.bufs = [torch.empty(n, dtype=torch.uint8, device="cuda") for n in sizes]
            self.how = {"by": "torch.empty (plain allocations)", "verdict": None}

    def free(self):
        self.bufs = None
        if self.ptrs is not None:
            self.B.bcast_buffers_free(self.ptrs)
            self.ptrs = None


class Ranks:
    """P rank buffers of M bytes in HBM: the root's holds the message, the others 0xFF.
    With library=True they come from bcast_buffers_alloc, the first half of the
    chain (positions 0 .. P/2-1, the root among them) under one region label and the
    second half under another: the library places the two in different regions of
    the device's memory."""

    def __init__(self, B, torch, inputs, P, root, M, msg, library):
        self.P, self.root, self.M = P, root, M
        self.msg = msg
        d_msg = torch.from_numpy(msg).cuda()
        library = library and M >= PLACE_MIN_BYTES
        regions = [0 if (r - root) % P < P // 2 else 1 for r in range(P)]
        self.mem = Placed(B, torch, [M] * P, regions, library)
        self.allocation = dict(self.mem.how)
        if library:
            self.allocation["layout"] = "chain positions 0..%d under one region label, %d..%d under another" % (P // 2 - 1, P // 2, P - 1)
        self.bufs = self.mem.bufs
        for r in range(P):
            if r == root:
                # the runtime's device-to-device copy of the whole message (M bytes read, M written): in a
                # profiled run this plain copy of known size calibrates FETCH_SIZE / WRITE_SIZE
                self.bufs[r].copy_(d_msg)
            else:
                self.bufs[r].fill_(inputs.FILL_BYTE)
        self.fill = inputs.FILL_BYTE

    def free(self):
        self.bufs = None
        self.mem.free()

    def clear(self):
        for r in range(self.P):
            if r != self.root:
                self.bufs[r].fill_(self.fill)

    def verify(self, torch, np, full_ranks):
        """Every rank against the root's buffer on the device, and `full_ranks`
        byte for byte against the host copy of the message over PCIe."""
        for r in range(self.P):
            if not torch.equal(self.bufs[r], self.bufs[self.root]):
                return "rank %d differs from the root's buffer" % r
        for r in full_ranks:
            if not np.array_equal(self.bufs[r].cpu().numpy(), self.msg):
                return "rank %d does not hold the message" % r
        return None


def measure_variant(B, torch, ranks, name, variant, stream, warmup, reps, profiles, no_verify, np, before_each=None):
    P, root, M = ranks.P, ranks.root, ranks.M
    plan = make_plan(B, name, variant, P, M)
    info = B.bcast_plan_info(plan, M, ranks.bufs)
    ptrs = B.RankPointers(ranks.bufs)
    if not no_verify:
        ranks.clear()
    ms = time_runs(torch, lambda: B.bcast_run(plan, ptrs, root, M, stream), stream, warmup, reps, before_each)
    status, detail = B.bcast_plan_status(plan)
    plan.destroy()
    if status != B.BCAST_OK:
        raise RuntimeError("%s %s: plan status %d detail %x" % (name, variant, status, detail))
    verified = None
    if not no_verify:
        err = ranks.verify(torch, np, sorted({(root + 1) % P, (root + P // 2) % P, (root + P - 1) % P} - {root}))
        if err:
            raise RuntimeError("%s %s: %s" % (name, variant, err))
        verified = True
    row = stats_us(ms)
    med_s = row["median_us"] * 1e-6
    geometry = geometry_of(B, info)
    algorithmic = int(info["algorithmic_bytes"])
    fl = floor_bytes(B, info, P, M)
    row.update({
        "algorithmic_bytes": algorithmic, "algorithmic_GBps": round(algorithmic / med_s / 1e9, 1),
        "delivered_GBps": round((P - 1) * M / med_s / 1e9, 1),
        "floor_bytes": fl, "floor_GBps": round(fl / med_s / 1e9, 1), "floor_frac": round(fl / med_s / 1e9 / HBM_PEAK_GBS, 4),
        "kernel": kernel_name(info, B), "geometry": geometry, "verified_bit_exact": verified,
    })
    if info["algo"] == B.BCAST_ALGO_CHAIN:
        row["stage_store"] = "write-back" if info["stage_store"] == B.BCAST_STORE_BACK else "write-through"
        if info["rank_waves"]:
            row["rank_handoff"] = "LDS" if info["rank_handoff"] == B.BCAST_HANDOFF_LDS else "cache"
    traffic, why = traffic_for(profiles, name, variant, geometry)
    if traffic:
        row.update({"traffic_bytes": traffic["bytes"], "traffic_fetch_bytes": traffic["fetch_bytes"], "traffic_write_bytes": traffic["write_bytes"],
                    "traffic_GBps": round(traffic["bytes"] / med_s / 1e9, 1), "traffic_frac": round(traffic["bytes"] / med_s / 1e9 / HBM_PEAK_GBS, 4),
                    "traffic_over_floor": round(traffic["bytes"] / fl, 3), "profile": traffic["file"],
                    "profile_kernel_us": round(traffic["avg_kernel_ns"] * 1e-3, 3)})
    else:
        row.update({"traffic_bytes": None, "traffic_note": why})
    return row, ms


# ---------------------------------------------------------------------------
# extra legs
# ---------------------------------------------------------------------------
def size_sweep(B, torch, bufs, P, root, max_bytes, stream, quick):
    """Latency per message size (4 B .. the workload's size, powers of two) at the
    workload's P, run by run with HIP events: the tuned choice (AUTO) and the
    tuned chain; median and min."""
    rows = []
    ptrs = B.RankPointers(bufs)
    M = 4
    while M <= max_bytes:
        row = {"bytes": M}
        for tag, algo in (("auto", B.BCAST_ALGO_AUTO), ("chain", B.BCAST_ALGO_CHAIN)):
            plan = B.bcast_plan_create(P, M, 0, algo)
            info = B.bcast_plan_info(plan, M, bufs)
            ms = time_runs(torch, lambda: B.bcast_run(plan, ptrs, root, M, stream), stream, 5, reps_for(M, quick))
            plan.destroy()
            st = stats_us(ms)
            row[tag + "_algo"] = B.ALGO_NAMES[info["algo"]]
            row[tag + "_median_us"], row[tag + "_min_us"] = st["median_us"], st["min_us"]
            if tag == "chain":
                row["chain_chunk_bytes"], row["chain_stages"], row["chain_rank_waves"] = int(info["chunk_bytes"]), info["stages"], info["rank_waves"]
                row["chain_algorithmic_GBps"] = round(2 * (P - 1) * M / st["median_us"] / 1e3, 1)
                row["chain_floor_frac"] = round(((P - 1) * M + info["stages"] * M) / st["median_us"] / 1e3 / HBM_PEAK_GBS, 4)
        rows.append(row)
        M *= 2
    return rows


def cold_rows(B, torch, bufs, P, root, sizes, stream, quick):
    """The same broadcasts with the memory-side cache emptied before every timed
    run: a 1 GiB scratch buffer is overwritten on the launch stream, so neither
    the message nor the rank buffers of the run before survive in the 256 MiB
    Infinity Cache.  Beside it the warm figure (runs back to back)."""
    scratch = torch.empty(GiB, dtype=torch.uint8, device="cuda")
    ptrs = B.RankPointers(bufs)
    rows = []
    for M in sizes:
        plan = B.bcast_plan_create(P, M, 0, B.BCAST_ALGO_CHAIN)
        info = B.bcast_plan_info(plan, M, bufs)
        reps = 5 if quick else 20
        warm = stats_us(time_runs(torch, lambda: B.bcast_run(plan, ptrs, root, M, stream), stream, 5, reps))
        cold = stats_us(time_runs(torch, lambda: B.bcast_run(plan, ptrs, root, M, stream), stream, 2, reps, before_each=lambda: scratch.fill_(0x5A)))
        plan.destroy()
        fl = (P - 1) * M + info["stages"] * M
        rows.append({"bytes": M, "warm_median_us": warm["median_us"], "warm_min_us": warm["min_us"], "cold_median_us": cold["median_us"],
                     "cold_min_us": cold["min_us"], "warm_algorithmic_GBps": round(2 * (P - 1) * M / warm["median_us"] / 1e3, 1),
                     "cold_algorithmic_GBps": round(2 * (P - 1) * M / cold["median_us"] / 1e3, 1),
                     "warm_floor_frac": round(fl / warm["median_us"] / 1e3 / HBM_PEAK_GBS, 4), "cold_floor_frac": round(fl / cold["median_us"] / 1e3 / HBM_PEAK_GBS, 4)})
    del scratch
    return rows


def record_graph(torch, enqueue):
    """What enqueue(stream) launches, recorded during stream capture."""
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        enqueue(torch.cuda.current_stream())
    return graph


def vgg_tensor_by_tensor(B, torch, bufs, P, root, stream, quick):
    """The same VGG-16 parameters broadcast as 32 messages, one per tensor, each
    with the tuned choice (AUTO), back to back: the alternative to packing them
    into one message.  Each pass between two HIP events."""
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

    def one_pass(on_stream=stream):
        for ptrs, n in views:
            B.bcast_run(plan, ptrs, root, n, on_stream)

    reps = 5 if quick else 20
    st = stats_us(time_runs(torch, one_pass, stream, 2, reps))
    # the same pass recorded once during stream capture and replayed as a graph (what a training loop
    # that repeats it every iteration would do): the plan keeps its run counter on the device for that
    B.bcast_plan_set_replayable(plan, True)
    one_pass()
    torch.cuda.synchronize()
    graph = record_graph(torch, one_pass)
    replayed = stats_us(time_runs(torch, graph.replay, stream, 2, reps))
    del graph
    plan.destroy()
    total = sum(n for _, n in spans)
    st.update({"tensors": len(spans), "algorithms": algos, "algorithmic_GBps": round(2 * (P - 1) * total / st["median_us"] / 1e3, 1),
               "graph_replay_median_us": replayed["median_us"], "graph_replay_min_us": replayed["min_us"]})
    return st


def burst(B, torch, inputs, np, P, root, M, stream, variant, n_runs, no_verify, profiles):
    """n_runs back-to-back broadcasts of M bytes between two HIP events: what a
    small broadcast costs when launches queue up behind each other."""
    msg = inputs.random_bytes(4, M)
    ranks = Ranks(B, torch, inputs, P, root, M, msg, False)
    plan = make_plan(B, "cfg5b", variant, P, M)
    info = B.bcast_plan_info(plan, M, ranks.bufs)
    ptrs = B.RankPointers(ranks.bufs)
    samples = []
    for it in range(6):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(n_runs):
            B.bcast_run(plan, ptrs, root, M, stream)
        e1.record(stream)
        torch.cuda.synchronize()
        if it:
            samples.append(e0.elapsed_time(e1) / n_runs)
    # the same burst recorded once and replayed as a graph, on a replayable plan
    B.bcast_plan_set_replayable(plan, True)
    B.bcast_run(plan, ptrs, root, M, stream)
    torch.cuda.synchronize()
    ranks.clear()

    def many(on_stream):
        for _ in range(n_runs):
            B.bcast_run(plan, ptrs, root, M, on_stream)

    graph = record_graph(torch, many)
    replayed = stats_us([t / n_runs for t in time_runs(torch, graph.replay, stream, 1, 5)])
    del graph
    status, _ = B.bcast_plan_status(plan)
    plan.destroy()
    if status != B.BCAST_OK:
        raise RuntimeError("cfg5b %s: plan status %d" % (variant, status))
    if not no_verify:
        err = ranks.verify(torch, np, [r for r in range(P) if r != root])
        if err:
            raise RuntimeError("cfg5b %s: %s" % (variant, err))
    row = stats_us(samples)
    row.update({"graph_replay_median_us": replayed["median_us"], "graph_replay_min_us": replayed["min_us"]})
    geometry = geometry_of(B, info)
    row.update({"runs_per_sample": n_runs, "algo": B.ALGO_NAMES[info["algo"]], "kernel": kernel_name(info, B), "geometry": geometry,
                "algorithmic_GBps": round(2 * (P - 1) * M / row["median_us"] / 1e3, 2), "verified_bit_exact": None if no_verify else True})
    traffic, why = traffic_for(profiles, "cfg5b", variant, geometry)
    if traffic:
        row.update({"traffic_bytes": traffic["bytes"], "traffic_GBps": round(traffic["bytes"] / row["median_us"] / 1e3, 2), "profile": traffic["file"],
                    "profile_kernel_us": round(traffic["avg_kernel_ns"] * 1e-3, 3)})
    else:
        row.update({"traffic_bytes": None, "traffic_note": why})
    return row


def reduce_row(B, torch, np, P, root, M, seed, stream, profiles, name, quick, no_verify, library=True):
    """The pipelined chain reduction (fp32 sum to the root) at the workload's rank
    count and message size: every rank contributes M bytes of N(0, 0.01) values
    (one seeded draw, shifted and rescaled per rank).  Algorithmic bytes: every
    input read once, the result written once, (P + 1) M.  With library=True the
    buffers come from bcast_buffers_alloc: the contributions in one region of the
    device's memory, the result in the next."""
    import oracle

    count = M // 4
    rng = np.random.default_rng(seed)
    base = rng.normal(0.0, 0.01, size=count).astype(np.float32)
    d_base = torch.from_numpy(base).cuda()
    calib = torch.empty_like(d_base)
    calib.copy_(d_base)  # a plain device-to-device copy of count * 4 bytes: calibrates the counters in a profiled run
    del calib
    mem = Placed(B, torch, [count * 4] * (P + 1), [0] * P + [1], library)
    send = [b.view(torch.float32) for b in mem.bufs[:P]]
    recv = mem.bufs[P].view(torch.float32)
    for r in range(P):
        send[r].copy_(torch.roll(d_base, 4099 * r) * (1.0 + r / 64.0))
    plan = B.bcast_plan_create(P, count * 4, 0, B.BCAST_ALGO_CHAIN)
    B.bcast_plan_reserve_reduce(plan, count, 2)
    info = B.bcast_reduce_info(plan, count)
    ptrs = B.RankPointers(send)
    ms = time_runs(torch, lambda: B.bcast_reduce_sum_f32(plan, ptrs, recv, root, count, stream), stream, 3, 5 if quick else 20)
    st, detail = B.bcast_plan_status(plan)
    plan.destroy()
    if st != B.BCAST_OK:
        raise RuntimeError("reduce %s: plan status %d (detail %#x)" % (name, st, detail))
    verified = None
    if not no_verify:
        # bit-exact against the oracle on a prefix (a sum is element-wise, so a prefix stands alone)
        sample = min(count, 1 << 20)
        host = np.stack([s[:sample].cpu().numpy() for s in send])
        want, _ = oracle.chain_reduce_f32(host, P, root, sample, max(1, int(info["chunk_bytes"]) // 4))
        verified = bool(np.array_equal(recv[:sample].cpu().numpy().view(np.uint32), want.view(np.uint32)))
        if not verified:
            raise RuntimeError("reduce %s: differs from the oracle" % name)
    n = count * 4 // 4096 * 4096
    # (the measurement kernel overwrites the result buffer, which has been checked by now)
    load_ms = stats_us(time_runs(torch, lambda: B.bcast_debug_load_pattern(send, n, recv, False, stream), stream, 2, 5 if quick else 10))
    both_ms = stats_us(time_runs(torch, lambda: B.bcast_debug_load_pattern(send, n, recv, True, stream), stream, 2, 5 if quick else 10))
    del send, recv
    mem.free()
    row = stats_us(ms)
    row["allocation"] = dict(mem.how, layout="the contributions under one region label, the result under another") if library else dict(mem.how)
    # the same P buffers only read, and read with the fold written out, by the library's dependency-free
    # measurement kernel: what this memory system gives the reduction's access pattern
    row["ceilings"] = {"load_only_median_us": load_ms["median_us"], "load_only_GBps": round(P * n / load_ms["median_us"] / 1e3, 1),
                       "load_and_store_result_median_us": both_ms["median_us"],
                       "load_and_store_result_GBps": round((P + 1) * n / both_ms["median_us"] / 1e3, 1)}
    med_s = row["median_us"] * 1e-6
    algorithmic = (P + 1) * count * 4
    fl = algorithmic + 2 * (info["stages"] - 1) * count * 4  # + the running sum through memory at every stage boundary
    geometry = geometry_of(B, info)
    row.update({"algorithmic_bytes": algorithmic, "algorithmic_GBps": round(algorithmic / med_s / 1e9, 1),
                "algorithmic_frac": round(algorithmic / med_s / 1e9 / HBM_PEAK_GBS, 4), "floor_bytes": fl,
                "floor_frac": round(fl / med_s / 1e9 / HBM_PEAK_GBS, 4),
                "kernel": "bcast::reduce_kernel<1, 16>" if count * 4 <= (2 << 20) else "bcast::reduce_kernel<4, 4>",
                "geometry": geometry, "verified_bit_exact": verified})
    traffic, why = traffic_for(profiles, name, "reduce", geometry)
    if traffic:
        row.update({"traffic_bytes": traffic["bytes"], "traffic_GBps": round(traffic["bytes"] / med_s / 1e9, 1),
                    "traffic_frac": round(traffic["bytes"] / med_s / 1e9 / HBM_PEAK_GBS, 4), "profile": traffic["file"]})
    else:
        row.update({"traffic_bytes": None, "traffic_note": why})
    return row


def ceilings(B, torch, bufs, root, M, stream, quick):
    """What the device's memory gives the broadcast's write set with no
    dependencies at all: the P-1 receiving buffers overwritten tile by tile by
    the library's measurement kernel (bcast_debug_store_pattern).  No broadcast
    to P-1 ranks on one die can finish sooner."""
    targets = [b for r, b in enumerate(bufs) if r != root]
    n = M // 4096 * 4096
    if n == 0:
        return None
    ms = time_runs(torch, lambda: B.bcast_debug_store_pattern(targets, n, stream), stream, 2, 5 if quick else 10)
    st = stats_us(ms)
    return {"store_only_median_us": st["median_us"], "store_only_min_us": st["min_us"], "store_only_bytes": len(targets) * n,
            "store_only_GBps": round(len(targets) * n / st["median_us"] / 1e3, 1),
            "store_only_frac_of_peak": round(len(targets) * n / st["median_us"] / 1e3 / HBM_PEAK_GBS, 4)}


def cpu_baseline(P, root, M, C, msg, budget_s=5.0):
    """The CPU oracle's chain simulation, as it stands, timed on this host on a
    bounded sample of the headline workload -- the same P, root and chunk size,
    the message cut down so that one pass takes well under a second -- on one
    core, and on all cores as one independent instance of the same simulation
    per core (the oracle itself is single-threaded), each for about budget_s."""
    import numpy as np

    import oracle

    sample = min(M, max(C, (256 * MiB // P) // C * C))
    cores = max(1, min(len(os.sched_getaffinity(0)), 16))

    def instance():
        host = np.full((P, sample), 0xFF, dtype=np.uint8)
        host[root] = msg[:sample]
        return host

    host = instance()
    oracle.chain_bcast(host, P, root, sample, C)  # touch pages once
    reps, t0 = 0, time.perf_counter()
    while True:
        oracle.chain_bcast(host, P, root, sample, C)
        reps += 1
        dt = time.perf_counter() - t0
        if dt > budget_s and reps >= 2:
            break
    one = {"value": round(2 * (P - 1) * sample * reps / dt / 1e9, 3), "reps": reps, "ms_each": round(dt / reps * 1e3, 2)}

    hosts = [host] + [instance() for _ in range(cores - 1)]
    counts = [0] * cores
    stop = time.perf_counter() + budget_s

    def worker(i):
        oracle.chain_bcast(hosts[i], P, root, sample, C)
        while time.perf_counter() < stop:
            oracle.chain_bcast(hosts[i], P, root, sample, C)  # the C call runs without the interpreter lock
            counts[i] += 1

    t0 = time.perf_counter()
    threads = [threading.Thread(target=worker, args=(i,)) for i in range(cores)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    dt_all = time.perf_counter() - t0
    allc = round(2 * (P - 1) * sample * sum(counts) / dt_all / 1e9, 3) if sum(counts) else None
    return {
        "value": one["value"], "unit": "GB/s", "cores": 1, "kind": "oracle",
        "sample": "oracle.chain_bcast, P=%d, root %d, first %d bytes of the message, C=%d, %d reps, %.1f ms each; rate = 2(P-1) x sample bytes / time"
                  % (P, root, sample, C, one["reps"], one["ms_each"]),
        "all_cores": {"value": allc, "unit": "GB/s", "cores": cores, "nproc": os.cpu_count(),
                      "sample": "%d concurrent instances of the same simulation, one thread each, %d passes in %.1f s" % (cores, sum(counts), dt_all)},
    }


# ---------------------------------------------------------------------------
def run_leg(args, B, torch, np, inputs):
    """One variant of one workload, --steps runs: what rocprofv3 wraps.  Prints a
    JSON line with the leg's launch geometry (the `# leg:` line of a profile)."""
    name, variant = args.leg.split(":")
    P, root, M, seed, what = WORKLOADS[name]
    stream = torch.cuda.current_stream()
    if variant == "reduce":
        row = reduce_row(B, torch, np, P, root, M, seed, stream, {}, name, True, True, args.allocation == "library")
        leg = {"workload": name, "variant": variant, "kernel": row["kernel"].split("<")[0], "geometry": row["geometry"], "launches_per_step": 1,
               "calibration_copy_bytes": (M // 4) * 4, "median_us": row["median_us"]}
        print(json.dumps(leg))
        return 0
    msg = make_message(name, seed, M)
    ranks = Ranks(B, torch, inputs, P, root, M, msg, args.allocation == "library")
    plan = make_plan(B, name, variant, P, M)
    info = B.bcast_plan_info(plan, M, ranks.bufs)
    ptrs = B.RankPointers(ranks.bufs)
    ms = time_runs(torch, lambda: B.bcast_run(plan, ptrs, root, M, stream), stream, 2, args.steps)
    st, _ = B.bcast_plan_status(plan)
    plan.destroy()
    leg = {"workload": name, "variant": variant, "kernel": kernel_name(info, B).split("<")[0], "geometry": geometry_of(B, info),
           "launches_per_step": info["launches"], "calibration_copy_bytes": M, "median_us": stats_us(ms)["median_us"], "status": st,
           "allocation": ranks.allocation}
    ranks.free()
    print(json.dumps(leg))
    return 0 if st == B.BCAST_OK else 1


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workloads", default=",".join(WORKLOADS), help="comma-separated subset of " + ",".join(WORKLOADS))
    ap.add_argument("--leg", default=None, help="WORKLOAD:VARIANT -- run only this variant, --steps times (for rocprofv3)")
    ap.add_argument("--quick", action="store_true", help="5 timed runs per variant instead of 20 / 200")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-verify", action="store_true")
    ap.add_argument("--allocation", choices=("library", "plain"), default="library",
                    help="rank buffers from bcast_buffers_alloc (placed by region of the device's memory) or from torch.empty")
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
    table = tuned.load_default_table()  # installs the shipped MI355X table if present
    if args.leg:
        return run_leg(args, B, torch, np, inputs)

    wanted = [w for w in args.workloads.split(",") if w]
    for w in wanted:
        if w not in WORKLOADS:
            print("bench.py: unknown workload %r" % w, file=sys.stderr)
            return 2
    if HEADLINE not in wanted:
        wanted.append(HEADLINE)
    profiles = load_profiles()
    stream = torch.cuda.current_stream()
    configs, headline, cpu = [], None, None
    t_start = time.perf_counter()

    library = args.allocation == "library"
    # The reductions first (their placement -- all contributions in one region, the result in another -- is the
    # one that allocating and freeing before it spoils), then the headline, then the rest.
    reduce_rows = {}
    for name in ("cfg4", "cfg2"):
        if name not in wanted:
            continue
        P, root, M, seed, what = WORKLOADS[name]
        try:
            reduce_rows[name] = reduce_row(B, torch, np, P, root, M, seed, stream, profiles, name, args.quick, args.no_verify, library)
        except RuntimeError as e:
            print("bench.py: %s" % e, file=sys.stderr)
            return 1
        torch.cuda.empty_cache()
    for name in [HEADLINE] + [w for w in WORKLOADS if w in wanted and w != HEADLINE]:
        P, root, M, seed, what = WORKLOADS[name]
        row = {"workload": name, "what": what, "P": P, "root": root, "message_bytes": M, "variants": {}}
        if name == "cfg5b":
            n = 200 if args.quick else 1000
            for variant in VARIANTS[name]:
                row["variants"][variant] = burst(B, torch, inputs, np, P, root, M, stream, variant, n, args.no_verify, profiles)
            configs.append(row)
            continue
        msg = make_message(name, seed, M)
        assert msg.nbytes == M
        ranks = Ranks(B, torch, inputs, P, root, M, msg, library)
        row["allocation"] = ranks.allocation
        for variant in VARIANTS[name]:
            reps = 5 if args.quick else max(20, reps_for(M, False))
            if name == HEADLINE and variant == "chain":
                # the contract's timed region: exactly --steps broadcasts back to back between two
                # synchronisations (wall clock), and between one pair of HIP events on the launch stream
                plan = make_plan(B, name, variant, P, M)
                ptrs = B.RankPointers(ranks.bufs)
                for _ in range(args.warmup):
                    B.bcast_run(plan, ptrs, root, M, stream)
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                t0 = time.perf_counter()
                e0.record(stream)
                for _ in range(args.steps):
                    B.bcast_run(plan, ptrs, root, M, stream)
                e1.record(stream)
                torch.cuda.synchronize()
                t1 = time.perf_counter()
                status, detail = B.bcast_plan_status(plan)
                plan.destroy()
                if status != B.BCAST_OK:
                    print("bench.py: plan status %d detail %x" % (status, detail), file=sys.stderr)
                    return 1
                headline = {"wall_ms": (t1 - t0) * 1e3 / args.steps, "avg_launch_ms": e0.elapsed_time(e1) / args.steps}
            try:
                row["variants"][variant], _ = measure_variant(B, torch, ranks, name, variant, stream, args.warmup, reps, profiles,
                                                               args.no_verify, np)
            except RuntimeError as e:
                print("bench.py: %s" % e, file=sys.stderr)
                return 1
        if name == "cfg2":
            row["sweep"] = size_sweep(B, torch, ranks.bufs, P, root, M, stream, args.quick)
            row["cold"] = cold_rows(B, torch, ranks.bufs, P, root, [8 * MiB, 16 * MiB, 32 * MiB, 64 * MiB], stream, args.quick)
        if name == "cfg3":
            row["per_tensor"] = vgg_tensor_by_tensor(B, torch, ranks.bufs, P, root, stream, args.quick)
        if M >= MiB:
            row["ceilings"] = ceilings(B, torch, ranks.bufs, root, M, stream, args.quick)
            for v in row["variants"].values():
                v["of_store_only_rate"] = round(row["ceilings"]["store_only_median_us"] / v["median_us"], 4)
        if name == HEADLINE and not args.no_cpu_baseline:
            C = row["variants"]["chain"]["geometry"]["chunk_bytes"] or M
            cpu = cpu_baseline(P, root, M, C, msg)
        ranks.free()
        del ranks, msg
        torch.cuda.empty_cache()
        if name in reduce_rows:
            row["reduce"] = reduce_rows[name]
        configs.append(row)
    configs.sort(key=lambda c: list(WORKLOADS).index(c["workload"]))

    P, root, M, seed, what = WORKLOADS[HEADLINE]
    head_cfg = next(c for c in configs if c["workload"] == HEADLINE)
    head = head_cfg["variants"]["chain"]
    head_ceiling = head_cfg.get("ceilings")
    g = head["geometry"]
    algorithmic = head["algorithmic_bytes"]
    wall_ms, avg_launch_ms = headline["wall_ms"], headline["avg_launch_ms"]
    launch_s = avg_launch_ms * 1e-3
    fl = head["floor_bytes"]
    traffic = head.get("traffic_bytes")
    out = {
        "metric": "broadcast effective HBM bandwidth 2(P-1)M/t (GB/s) at the stated message size and P; latency in ms_per_step",
        "value": round(algorithmic / (wall_ms * 1e-3) / 1e9, 2),
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
        "config": {"workload": "%s: %s" % (HEADLINE, what), "P": P, "root": root, "message_bytes": M, "variant": "tuned pipelined chain",
                   "tuning_table": table, "allocation": head_cfg.get("allocation"), "stage_store": head.get("stage_store"), **g},
        "delivered_GBps": round((P - 1) * M / (wall_ms * 1e-3) / 1e9, 2),
        "median_us": head["median_us"], "min_us": head["min_us"],
        "verified_bit_exact": head["verified_bit_exact"],
        "roofline": {
            "bound": "hbm",
            # the kernel's own minimum of HBM bytes per launch -- (P-1) M written, M read per stage -- over the
            # average launch duration measured here with HIP events on the launch stream
            "achieved": round(fl / launch_s / 1e9, 2),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(fl / launch_s / 1e9 / HBM_PEAK_GBS, 4),
            "floor_bytes": fl,
            # L2 <-> fabric bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, read from profiles/
            "traffic": traffic,
            "traffic_GBps": round(traffic / launch_s / 1e9, 2) if traffic else None,
            "traffic_frac": round(traffic / launch_s / 1e9 / HBM_PEAK_GBS, 4) if traffic else None,
            "traffic_note": head.get("traffic_note"),
            "profile": head.get("profile"),
            # 2 (P-1) M over the same time: what the ranks' buffers exchanged, most of it inside compute units
            "algorithmic_bytes_per_launch": algorithmic,
            "algorithmic_GBps": round(algorithmic / launch_s / 1e9, 2),
            "kernel": head["kernel"],
            "avg_launch_ms": round(avg_launch_ms, 5),
            # the same P-1 buffers only written, with no dependencies (bcast_debug_store_pattern), in this run:
            # the rate this device's memory gives the broadcast's write set, and the chain's time relative to it
            "store_only_GBps": head_ceiling["store_only_GBps"] if head_ceiling else None,
            "store_only_ms": round(head_ceiling["store_only_median_us"] * 1e-3, 5) if head_ceiling else None,
            "of_store_only_rate": head.get("of_store_only_rate"),
        },
        "cpu_baseline": cpu,
        "configs": configs,
        "bench_seconds": round(time.perf_counter() - t_start, 1),
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
