"""The pipelined chain with one wavefront per rank (Sec. IV-B read literally:
every rank receives from its left neighbour, stores, and tells its right
neighbour) against the CPU oracle, byte for byte, guard bands included.

A stage is a workgroup of up to 16 wavefronts, one per consecutive rank, whose
hand-offs go through LDS counters and the payload through LDS trip slots or the
compute unit's cache (every test runs both ways); between stages
chunks are handed over through the ready flags in memory.  Covered: every rank
count up to 64, stage counts from the fewest possible to one rank per workgroup,
every trip size, ragged sizes, misaligned pointers, empty and short messages,
forced wait-limit expiry inside a workgroup and between workgroups, bursts of
changing messages, the wrap of the run counter, alternation with the
wave-per-stage kernel on one plan, a seeded sweep."""
import numpy as np
import pytest
import torch

import oracle
from paper_1707_09414_amd import binding as B
from paper_1707_09414_amd import inputs
import gpu_harness
from gpu_harness import RankBuffers, run_and_check, FILL

pytestmark = pytest.mark.gpu
KiB, MiB = inputs.KiB, inputs.MiB
RANK = B.BCAST_CHAIN_WAVE_PER_RANK
STAGE = B.BCAST_CHAIN_WAVE_PER_STAGE


@pytest.fixture(scope="module")
def noise():
    return inputs.random_bytes(7, 8 * MiB + 64)


@pytest.fixture(autouse=True, params=[B.BCAST_HANDOFF_CACHE, gpu_harness.PREFER_LDS], ids=["cache", "lds"])
def handoff(request):
    """Every test of this module twice: trips between the ranks of a workgroup
    through the compute unit's cache, and through LDS wherever the slots fit."""
    gpu_harness.RANK_HANDOFF = request.param
    yield request.param
    gpu_harness.RANK_HANDOFF = B.BCAST_HANDOFF_AUTO


def fewest_stages(P):
    return -(-(P - 1) // 16)


@pytest.mark.parametrize("P", [2, 3, 4, 8, 9, 10, 17, 18, 33, 34, 50, 64])
@pytest.mark.parametrize("M,C", [(1, 16), (15, 16), (17, 16), (1000, 112), (4096, 0), (65536 + 3, 8192), (MiB + 17, 64 * KiB),
                                 (5 * MiB + 4096 + 5, 0), (3 * MiB, 4 * MiB)])
def test_sizes_and_ranks(noise, P, M, C):
    info = run_and_check(P, (5 * P) // 7 % P, M, C, B.BCAST_ALGO_CHAIN, noise, waves=RANK)
    assert info["rank_waves"] == 1 and info["launches"] == 1
    # automatic stages: at most 8 ranks per workgroup; a workgroup per (stage, lane)
    assert info["stages"] == -(-(P - 1) // 8) and info["hops_per_stage"] == -(-(P - 1) // info["stages"])
    assert info["block_threads"] == 64 * info["hops_per_stage"] and info["grid_blocks"] == info["stages"] * info["lanes"]


@pytest.mark.parametrize("P,stages", [(2, 1), (5, 1), (5, 2), (5, 4), (8, 1), (8, 3), (17, 1), (17, 2), (17, 16), (18, 1), (18, 2), (33, 2), (33, 3),
                                      (64, 1), (64, 4), (64, 5), (64, 8), (64, 9), (64, 63), (64, 100)])
@pytest.mark.parametrize("M,C,lanes", [(7, 16, 0), (70000, 8192, 0), (3 * MiB + 5, 256 * KiB, 0), (MiB + 1, 48 * KiB, 3)])
def test_stage_counts(noise, P, stages, M, C, lanes):
    """From every rank of the chain in one workgroup (up to 16) to one rank per
    workgroup (every hand-off through memory)."""
    info = run_and_check(P, P // 3, M, C, B.BCAST_ALGO_CHAIN, noise, stages=stages, lanes=lanes, waves=RANK)
    want = max(min(stages, P - 1), fewest_stages(P))
    assert info["stages"] == want and info["hops_per_stage"] == -(-(P - 1) // want) <= 16
    if lanes:
        assert info["lanes"] == lanes


@pytest.mark.parametrize("trip", [1024, 2048, 3072, 4096, 6144, 8192])
@pytest.mark.parametrize("offsets", [None, [4] * 9, [1, 0, 3, 16, 8, 2, 5, 7, 12]])
@pytest.mark.parametrize("stages,M,C", [(1, 3072, 3072), (2, 8193, 8192), (3, 70000, 6144), (8, 3 * MiB + 5, 96 * KiB), (2, 5 * MiB + 1000, 768 * KiB)])
def test_trip_sizes_and_alignments(noise, trip, offsets, stages, M, C):
    info = run_and_check(9, 2, M, C, B.BCAST_ALGO_CHAIN, noise, stages=stages, trip=trip, offsets=offsets, waves=RANK)
    assert info["trip_bytes"] == trip and info["slice_bytes"] % trip == 0
    assert info["vec_bytes"] == (16 if offsets is None or len(set(offsets)) == 1 else 1)


@pytest.mark.parametrize("offsets_kind", ["same4", "same1", "mixed4", "mixed1", "mixed8"])
@pytest.mark.parametrize("M", [5, 16, 4099, 300 * KiB + 7])
def test_misaligned_pointers(noise, offsets_kind, M):
    P = 5
    offsets = {"same4": [4] * P, "same1": [1] * P, "mixed4": [0, 4, 8, 12, 20], "mixed1": [0, 1, 2, 3, 5], "mixed8": [0, 8, 16, 24, 40]}[offsets_kind]
    info = run_and_check(P, 2, M, 64 * KiB, B.BCAST_ALGO_CHAIN, noise, offsets=offsets, waves=RANK)
    assert info["vec_bytes"] == {"same4": 16, "same1": 16, "mixed4": 4, "mixed1": 1, "mixed8": 8}[offsets_kind]


def test_degenerate_cases(noise):
    run_and_check(1, 0, 4096, 4096, B.BCAST_ALGO_CHAIN, noise, waves=RANK)
    run_and_check(4, 2, 0, 4096, B.BCAST_ALGO_CHAIN, noise, cap=4096, waves=RANK)
    run_and_check(4, 2, 1000, 4096, B.BCAST_ALGO_CHAIN, noise, cap=1 * MiB, waves=RANK)
    run_and_check(64, 63, 1, 0, B.BCAST_ALGO_CHAIN, noise, waves=RANK)
    # the write-back default of small messages and the write-through one of large ones, and both forced
    for pol in [(-1, -1, -1, -1), (16, 16, 0, 0), (16, 16, 0, 16), (0, 16, 0, 16), (16, 16, 16, 16)]:
        plan = B.bcast_plan_create(12, 3 * MiB, 0, B.BCAST_ALGO_CHAIN)
        B.bcast_plan_set_cache_policy(plan, *pol)
        run_and_check(12, 5, 3 * MiB - 9, 0, B.BCAST_ALGO_CHAIN, noise, plan=plan, cap=3 * MiB, waves=RANK)
        run_and_check(12, 6, 100 * KiB, 0, B.BCAST_ALGO_CHAIN, noise, plan=plan, cap=3 * MiB, waves=RANK)
        plan.destroy()


@pytest.mark.parametrize("mute,stages", [(2, 1), (4, 2), (3, 2), (1, 5)])
def test_wait_limit_inside_and_between_workgroups(noise, mute, stages):
    """Position `mute` stores its pieces but never tells its right neighbour
    (forced from the host), with a tiny wait limit: the neighbour gives up, every
    wave exits, the plan reports which position gave up, and works again after.
    P = 6: with 1 stage every hand-off is inside the workgroup; with 2 stages
    (hops 1-3 | 4-5) position 3 -> 4 crosses workgroups; with 5 every one does."""
    P, M = 6, 256 * KiB
    rb = RankBuffers(P, M)
    rb.reset(0, noise[:M])
    plan = B.bcast_plan_create(P, M, 16 * KiB, B.BCAST_ALGO_CHAIN)
    B.bcast_plan_set_chain_waves(plan, RANK)
    B.bcast_plan_set_stages(plan, stages)
    gpu_harness.set_rank_handoff(plan, M)
    B.bcast_plan_set_debug(plan, 200000, mute)  # 2 ms of the 100 MHz clock
    B.bcast_run(plan, rb.ptrs(), 0, M)
    torch.cuda.synchronize()
    st, detail = B.bcast_plan_status(plan)
    assert st == B.BCAST_ERR_TIMEOUT
    # every position behind the silent one starts waiting for its first trip (chunk 0) at the same moment; the
    # silent one itself waits, two trips on, for its right neighbour's reading (reported under that neighbour's
    # position), and the stall spreads upstream two trips per position (position q - 1 waits for position q's
    # reading of trip 2 (mute - q + 2), again reported under q).  The waits begin within microseconds of each
    # other and the limit is looked at every 64 polls, so any of them may be the first to see it pass.
    pos, chunk = detail >> 32, detail & 0xFFFFFFFF
    assert 2 <= pos <= P - 1 and chunk <= (2 if pos > mute else 2 * (mute - pos + 2)), hex(detail)
    got = rb.to_host()
    # every position up to the silent one got at least its first trip (a rank may run two
    # trips ahead of its right neighbour's reading; after that the stall spreads upstream)
    for r in range(1, mute + 1):
        assert np.array_equal(got[r][rb.start(r): rb.start(r) + 8192], noise[:8192]), r
    for r in range(mute + 1, P):   # nothing reached the positions behind it
        assert (got[r] == FILL).all(), r
    B.bcast_plan_clear_status(plan)
    B.bcast_plan_set_debug(plan, 0, 0)
    rb.reset(0, noise[7: 7 + M])
    B.bcast_run(plan, rb.ptrs(), 0, M)
    got = rb.to_host()
    assert B.bcast_plan_status(plan)[0] == B.BCAST_OK
    for r in range(P):
        assert np.array_equal(got[r][rb.start(r): rb.start(r) + M], noise[7: 7 + M]), r
    plan.destroy()


def test_burst_of_small_broadcasts_reuses_flags_and_counters():
    """500 back-to-back 4 KiB broadcasts at P=64, root 17, a different message
    each time, alternating between the two chain kernels on ONE plan (they share
    its flags and run counter): a stale flag would forward an earlier message."""
    P, root, M, N = 64, 17, 4 * KiB, 500
    msgs = inputs.random_bytes(5, N * M).reshape(N, M)
    d_msgs = torch.from_numpy(msgs).cuda()
    rb = RankBuffers(P, M)
    rb.reset(root, msgs[0])
    watch = [(root + k) % P for k in (1, 8, 9, 31, 63)]
    outs = [torch.empty((N, M), dtype=torch.uint8, device="cuda") for _ in watch]
    plan = B.bcast_plan_create(P, M, 0, B.BCAST_ALGO_CHAIN)
    B.bcast_plan_set_chain_waves(plan, RANK)
    gpu_harness.set_rank_handoff(plan, M)
    ptrs = rb.ptrs()
    s0 = rb.start(root)
    stream = torch.cuda.current_stream()
    for i in range(N):
        B.bcast_plan_set_chain_waves(plan, STAGE if i % 5 == 4 else RANK)
        rb.raw[root][s0: s0 + M].copy_(d_msgs[i])
        B.bcast_run(plan, ptrs, root, M, stream)
        for o, r in zip(outs, watch):
            o[i].copy_(rb.raw[r][rb.start(r): rb.start(r) + M])
    torch.cuda.synchronize()
    assert B.bcast_plan_status(plan)[0] == B.BCAST_OK
    for o, r in zip(outs, watch):
        assert np.array_equal(o.cpu().numpy(), msgs), r
    plan.destroy()


def test_run_counter_wrap(noise):
    P, root, M = 20, 4, 200 * KiB + 8
    plan = B.bcast_plan_create(P, M, 24 * KiB, B.BCAST_ALGO_CHAIN)
    B.bcast_plan_set_stages(plan, 3)
    run_and_check(P, root, M, 24 * KiB, B.BCAST_ALGO_CHAIN, noise, plan=plan, waves=RANK)
    B.bcast_plan_debug_set_epoch(plan, (1 << 32) - 6)
    for i in range(10):
        run_and_check(P, (root + i) % P, M - 16 * i, 24 * KiB, B.BCAST_ALGO_CHAIN, noise[1000 * i:], plan=plan, waves=RANK)
    plan.destroy()


def test_pipeline_really_overlaps_ranks():
    """One lane, 15 ranks in one workgroup, 64 trips: if the ranks ran one after
    the other the kernel would take 15 x the time of one rank's pass; pipelined,
    it takes about (64 + 14) trip times.  Compared on device time against the
    same shape with 2 ranks (one hop)."""
    M, trip = 64 * 8192, 8192
    times = {}
    for P in (2, 16):
        bufs = [torch.full((M,), 0xFF, dtype=torch.uint8, device="cuda") for _ in range(P)]
        bufs[0].random_(0, 256)
        plan = B.bcast_plan_create(P, M, M, B.BCAST_ALGO_CHAIN)
        B.bcast_plan_set_chain_waves(plan, RANK)
        B.bcast_plan_set_stages(plan, 1)
        B.bcast_plan_set_lanes(plan, 1)
        B.bcast_plan_set_trip(plan, trip)
        gpu_harness.set_rank_handoff(plan, M)
        ptrs = B.RankPointers(bufs)
        stream = torch.cuda.current_stream()
        best = 1e9
        for _ in range(5):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            B.bcast_run(plan, ptrs, 0, M, stream)
            e1.record(stream)
            torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1))
        assert all(torch.equal(b, bufs[0]) for b in bufs)
        times[P] = best
        plan.destroy()
    # 15 hops, serial: >= 15 x; pipelined: (64 + 14) / 64 = 1.2 x plus hand-off costs
    assert times[16] < 6 * times[2], times


@pytest.mark.parametrize("seed", [21, 22])
def test_random_configurations(noise, seed):
    rng = np.random.default_rng(seed)
    for case in range(70):
        P = int(rng.integers(2, 65))
        root = int(rng.integers(0, P))
        M = int(rng.choice([1, 17, 4096, 70001, int(rng.integers(1, 3 * MiB))]))
        C = int(rng.choice([0, 16, 4096, 65536, 1 << 20])) if rng.random() < 0.8 else 16 * int(rng.integers(1, 20000))
        stages = int(rng.integers(0, 70))
        lanes = int(rng.choice([0, 0, 1, 3, 32]))
        trip = int(rng.choice([0, 1024, 2048, 3072, 4096, 6144, 8192]))
        offsets = None if rng.random() < 0.6 else [int(x) for x in rng.integers(0, 64, size=P)]
        try:
            run_and_check(P, root, M, C, B.BCAST_ALGO_CHAIN, noise, stages=stages, lanes=lanes, trip=trip, offsets=offsets, waves=RANK)
        except Exception as e:
            raise AssertionError("case %d: P=%d root=%d M=%d C=%d stages=%d lanes=%d trip=%d offsets=%s: %s"
                                 % (case, P, root, M, C, stages, lanes, trip, offsets, e))


def test_handoff_knob(noise, handoff):
    """What the plan reports and refuses: LDS needs two trip slots per wavefront
    of the workgroup (9 ranks in one workgroup at 4 KiB trips: 64 KiB; 17 ranks at
    8 KiB trips: 256 KiB, more than a workgroup can have); AUTO takes LDS where it
    fits and the message is longer than 2 MiB; a workgroup of one rank has nothing to hand over; ragged trips go
    through the cache in either mode (covered by every ragged size above)."""
    P, M = 10, 2 * MiB + 16
    plan = B.bcast_plan_create(P, M, 0, B.BCAST_ALGO_CHAIN)
    B.bcast_plan_set_chain_waves(plan, RANK)
    B.bcast_plan_set_stages(plan, 1)
    B.bcast_plan_set_trip(plan, 4096)
    for mode, want in ((B.BCAST_HANDOFF_AUTO, B.BCAST_HANDOFF_LDS), (B.BCAST_HANDOFF_LDS, B.BCAST_HANDOFF_LDS),
                       (B.BCAST_HANDOFF_CACHE, B.BCAST_HANDOFF_CACHE)):
        B.bcast_plan_set_rank_handoff(plan, mode)
        gpu_harness.RANK_HANDOFF = mode
        info = run_and_check(P, 3, M, 0, B.BCAST_ALGO_CHAIN, noise, plan=plan, waves=RANK)
        assert info["rank_handoff"] == want and info["hops_per_stage"] == 9
    with pytest.raises(B.BcastError):
        B.bcast_plan_set_rank_handoff(plan, 3)
    # left to the library, messages up to 2 MiB go through the cache (the faster way there), longer ones through LDS
    B.bcast_plan_set_rank_handoff(plan, B.BCAST_HANDOFF_AUTO)
    assert B.bcast_plan_info(plan, 2 * MiB)["rank_handoff"] == B.BCAST_HANDOFF_CACHE
    assert B.bcast_plan_info(plan, 2 * MiB + 16)["rank_handoff"] == B.BCAST_HANDOFF_LDS
    B.bcast_plan_set_rank_handoff(plan, B.BCAST_HANDOFF_LDS)
    assert B.bcast_plan_info(plan, 4096)["rank_handoff"] == B.BCAST_HANDOFF_LDS
    plan.destroy()
    gpu_harness.RANK_HANDOFF = handoff
    # 16 ranks per workgroup at 8 KiB trips: 256 KiB of slots
    plan = B.bcast_plan_create(17, M, 0, B.BCAST_ALGO_CHAIN)
    B.bcast_plan_set_chain_waves(plan, RANK)
    B.bcast_plan_set_stages(plan, 1)
    B.bcast_plan_set_trip(plan, 8192)
    B.bcast_plan_set_rank_handoff(plan, B.BCAST_HANDOFF_AUTO)
    assert B.bcast_plan_info(plan, M)["rank_handoff"] == B.BCAST_HANDOFF_CACHE
    B.bcast_plan_set_rank_handoff(plan, B.BCAST_HANDOFF_LDS)
    with pytest.raises(B.BcastError):
        B.bcast_plan_info(plan, M)
    rb = RankBuffers(17, M)
    rb.reset(0, noise[:M])
    with pytest.raises(B.BcastError):
        B.bcast_run(plan, rb.ptrs(), 0, M)
    assert all((t == FILL).all() for t in rb.to_host()[1:])  # nothing was launched
    plan.destroy()
    # one rank per workgroup: nothing to hand over inside it
    plan = B.bcast_plan_create(5, M, 0, B.BCAST_ALGO_CHAIN)
    B.bcast_plan_set_chain_waves(plan, RANK)
    B.bcast_plan_set_stages(plan, 4)
    assert B.bcast_plan_info(plan, M)["rank_handoff"] == B.BCAST_HANDOFF_CACHE
    plan.destroy()
    # the wave-per-stage chain has no such hand-off
    plan = B.bcast_plan_create(5, M, 0, B.BCAST_ALGO_CHAIN)
    B.bcast_plan_set_chain_waves(plan, STAGE)
    assert B.bcast_plan_info(plan, M)["rank_handoff"] == 0
    plan.destroy()
