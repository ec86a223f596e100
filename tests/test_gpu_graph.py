"""Replayable plans: runs recorded during stream capture and replayed as a graph.

A deep-learning step repeats the same broadcasts every iteration (Sec. I), so a
caller records them once and replays the graph.  A replay re-issues the recorded
kernel arguments unchanged; a replayable plan therefore keeps its run counter
(the epoch in the ready flags of Sec. IV-B's hand-off) in device memory, where a
small kernel ahead of each run advances it.  Every replay is compared byte for
byte with the CPU oracle on a message that changes from replay to replay, with
directly issued runs of the same plan in between; a forced wait-limit expiry
proves that each replay really gets an epoch later than every flag left behind
(a stale epoch would find those flags and not wait at all).  All kernels exit
normally in every case.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_1707_09414_amd import binding as B
from paper_1707_09414_amd import inputs
from gpu_harness import RankBuffers, assert_same, expected_with_oracle

pytestmark = pytest.mark.gpu
KiB, MiB = inputs.KiB, inputs.MiB


def capture(fn):
    """Record what fn(stream) enqueues into a graph; returns the graph."""
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        fn(torch.cuda.current_stream())
    return g


def oracle_end_state(info, before, starts, P, root, M):
    if info["algo"] == B.BCAST_ALGO_KNOMIAL_PIPELINED:
        schedule = lambda a: oracle.knomial_pipeline_bcast(a, P, root, M, max(16, info["chunk_bytes"]), max(2, info["stages"]))
    elif info["algo"] == B.BCAST_ALGO_CHAIN:
        schedule = lambda a: oracle.chain_bcast(a, P, root, M, max(1, info["chunk_bytes"]))
    elif info["algo"] == B.BCAST_ALGO_DIRECT:
        schedule = lambda a: oracle.direct_bcast(a, P, root, M)
    else:
        schedule = lambda a: oracle.binomial_bcast(a, P, root, M)
    exp, _ = expected_with_oracle(before, starts, root, M, schedule)
    return exp


VARIANTS = [
    ("chain, a wavefront per stage", B.BCAST_ALGO_CHAIN, dict(stages=3, waves=B.BCAST_CHAIN_WAVE_PER_STAGE)),
    ("chain, a wavefront per rank", B.BCAST_ALGO_CHAIN, dict(stages=2, waves=B.BCAST_CHAIN_WAVE_PER_RANK)),
    ("chain, one stage (no flags)", B.BCAST_ALGO_CHAIN, dict(stages=1, waves=B.BCAST_CHAIN_WAVE_PER_STAGE)),
    ("pipelined k-nomial tree", B.BCAST_ALGO_KNOMIAL_PIPELINED, dict(radix=2)),
    ("direct", B.BCAST_ALGO_DIRECT, dict()),
    ("binomial", B.BCAST_ALGO_BINOMIAL, dict()),
]


@pytest.mark.parametrize("name,algo,knobs", VARIANTS, ids=[v[0] for v in VARIANTS])
def test_replays_of_a_captured_broadcast(name, algo, knobs):
    P, root, M, C = 8, 5, 3 * MiB // 2 + 13, 64 * KiB
    draw = inputs.random_bytes(61, 6 * M)
    rb = RankBuffers(P, M)
    plan = B.bcast_plan_create(P, M, C, algo)
    if "stages" in knobs:
        B.bcast_plan_set_stages(plan, knobs["stages"])
    if "waves" in knobs:
        B.bcast_plan_set_chain_waves(plan, knobs["waves"])
    if "radix" in knobs:
        B.bcast_plan_set_radix(plan, knobs["radix"])
    B.bcast_plan_set_replayable(plan, True)
    ptrs = rb.ptrs()
    info = B.bcast_plan_info(plan, M, rb.ptrs())
    starts = [rb.start(r) for r in range(P)]

    # once directly (loads the kernels), then recorded
    rb.reset(root, draw[:M])
    B.bcast_run(plan, ptrs, root, M, torch.cuda.current_stream())
    torch.cuda.synchronize()
    graph = capture(lambda s: B.bcast_run(plan, ptrs, root, M, s))

    for rep in range(4):
        message = draw[(rep + 1) * M: (rep + 2) * M]
        rb.reset(root, message)
        before = rb.to_host()
        graph.replay()
        got = rb.to_host()
        assert B.bcast_plan_status(plan)[0] == B.BCAST_OK
        assert_same(got, oracle_end_state(info, before, starts, P, root, M), "%s, replay %d" % (name, rep))
        # a directly issued run of the same plan from another root in between
        other = (root + 3) % P
        rb.reset(other, draw[:M])
        before = rb.to_host()
        B.bcast_run(plan, ptrs, other, M, torch.cuda.current_stream())
        got = rb.to_host()
        assert_same(got, oracle_end_state(info, before, starts, P, other, M), "%s, direct run after replay %d" % (name, rep))
    plan.destroy()


def test_every_replay_gets_a_later_epoch_than_the_flags_left_behind():
    """Two graphs on one plan: a normal broadcast, and the same broadcast with one
    position muted and a tiny wait limit.  After the normal one has raised every
    flag, the muted one must still run into the wait limit, on every replay."""
    P, root, M = 8, 0, 256 * KiB
    rb = RankBuffers(P, M)
    message = inputs.random_bytes(62, M)
    for waves in (B.BCAST_CHAIN_WAVE_PER_STAGE, B.BCAST_CHAIN_WAVE_PER_RANK):
        plan = B.bcast_plan_create(P, M, 32 * KiB, B.BCAST_ALGO_CHAIN)
        B.bcast_plan_set_stages(plan, 7 if waves == B.BCAST_CHAIN_WAVE_PER_STAGE else 2)
        B.bcast_plan_set_chain_waves(plan, waves)
        B.bcast_plan_set_replayable(plan, True)
        ptrs = rb.ptrs()
        rb.reset(root, message)
        B.bcast_run(plan, ptrs, root, M, torch.cuda.current_stream())
        torch.cuda.synchronize()
        good = capture(lambda s: B.bcast_run(plan, ptrs, root, M, s))
        B.bcast_plan_set_debug(plan, 200000, 4)  # 2 ms of the 100 MHz clock; position 4 stores but never publishes
        muted = capture(lambda s: B.bcast_run(plan, ptrs, root, M, s))
        B.bcast_plan_set_debug(plan, 0, 0)
        for rep in range(3):
            good.replay()
            torch.cuda.synchronize()
            assert B.bcast_plan_status(plan)[0] == B.BCAST_OK
            muted.replay()
            torch.cuda.synchronize()
            st, detail = B.bcast_plan_status(plan)
            assert st == B.BCAST_ERR_TIMEOUT, "replay %d of the muted run found flags of an earlier run" % rep
            assert 4 < (detail >> 32) <= P - 1
            B.bcast_plan_clear_status(plan)
        # and the plan still broadcasts correctly afterwards
        rb.reset(root, message)
        before = rb.to_host()
        good.replay()
        got = rb.to_host()
        info = B.bcast_plan_info(plan, M, rb.ptrs())
        assert_same(got, oracle_end_state(info, before, [rb.start(r) for r in range(P)], P, root, M), "after the muted replays")
        assert B.bcast_plan_status(plan)[0] == B.BCAST_OK
        plan.destroy()


def contributions(seed, P, count):
    rng = np.random.default_rng(seed)
    x = rng.normal(0.0, 0.01, size=(P, count)).astype(np.float32)
    x[:, 0] = np.float32(1e30) * rng.choice([-1.0, 1.0], size=P)
    return x


@pytest.mark.parametrize("entry", ["plan", "static"])
def test_replays_of_a_captured_reduction_and_allreduce(entry):
    P, root, count = 8, 2, 300001
    plan = B.bcast_plan_create(P, count * 4, 64 * KiB, B.BCAST_ALGO_CHAIN)
    B.bcast_plan_set_stages(plan, 2)
    B.bcast_plan_reserve_reduce(plan, count, 2)
    B.bcast_plan_set_replayable(plan, True)
    send = [torch.zeros(count, dtype=torch.float32, device="cuda") for _ in range(P)]
    recv = [torch.zeros(count, dtype=torch.float32, device="cuda") for _ in range(P)]
    reduce = B.bcast_reduce_sum_f32 if entry == "plan" else B.bcast_reduce_sum_f32_static
    assert B.bcast_reduce_info(plan, count)["stages"] == 2

    def step(s):
        # MPI_Allreduce as the two chains: the reduction to the root, then its result down the broadcast chain
        reduce(plan, send, recv[root], root, count, s)
        B.bcast_run(plan, recv, root, count * 4, s)

    step(torch.cuda.current_stream())
    torch.cuda.synchronize()
    graph = capture(step)
    for rep in range(4):
        x = contributions(70 + rep, P, count)
        for r in range(P):
            send[r].copy_(torch.from_numpy(x[r]))
            recv[r].fill_(-1.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert B.bcast_plan_status(plan)[0] == B.BCAST_OK
        want, _ = oracle.chain_reduce_f32(np.ascontiguousarray(x), P, root, count, 16 * KiB)
        for r in range(P):
            assert np.array_equal(recv[r].cpu().numpy().view(np.uint32), want.view(np.uint32)), "%s entry, replay %d, rank %d" % (entry, rep, r)
        # the static array is shared: a direct call from another plan in between must not disturb the next replay
        if entry == "static":
            other = B.bcast_plan_create(4, 4096 * 4, 0, B.BCAST_ALGO_CHAIN)
            B.bcast_plan_set_stages(other, 3)
            o_send = [torch.full((4096,), float(r + 1), dtype=torch.float32, device="cuda") for r in range(4)]
            o_recv = torch.zeros(4096, dtype=torch.float32, device="cuda")
            B.bcast_reduce_sum_f32_static(other, o_send, o_recv, 1, 4096, torch.cuda.current_stream())
            torch.cuda.synchronize()
            assert (o_recv == 10.0).all()
            other.destroy()
    plan.destroy()


def test_the_epoch_wraps_on_the_device_between_replays():
    """2^32 - 2 runs exhaust the 32-bit count in the flag words: the kernel that
    advances the count then clears the flags first.  Reached here by setting the
    count close to the limit; the replays before, at and after the wrap all
    deliver, and a muted run after the wrap still runs into the wait limit."""
    P, root, M = 6, 1, 200 * KiB + 5
    rb = RankBuffers(P, M)
    draw = inputs.random_bytes(63, 8 * M)
    plan = B.bcast_plan_create(P, M, 16 * KiB, B.BCAST_ALGO_CHAIN)
    B.bcast_plan_set_stages(plan, 5)
    B.bcast_plan_set_replayable(plan, True)
    ptrs = rb.ptrs()
    info = B.bcast_plan_info(plan, M, rb.ptrs())
    starts = [rb.start(r) for r in range(P)]
    rb.reset(root, draw[:M])
    B.bcast_run(plan, ptrs, root, M, torch.cuda.current_stream())
    torch.cuda.synchronize()
    good = capture(lambda s: B.bcast_run(plan, ptrs, root, M, s))
    B.bcast_plan_set_debug(plan, 200000, 2)
    muted = capture(lambda s: B.bcast_run(plan, ptrs, root, M, s))
    B.bcast_plan_set_debug(plan, 0, 0)
    B.bcast_plan_debug_set_epoch(plan, (1 << 32) - 5)
    for rep in range(6):  # epochs 2^32-4, -3, -2, then 1, 2, 3 after the wrap
        message = draw[(rep + 1) * M: (rep + 2) * M]
        rb.reset(root, message)
        before = rb.to_host()
        good.replay()
        got = rb.to_host()
        assert B.bcast_plan_status(plan)[0] == B.BCAST_OK
        assert_same(got, oracle_end_state(info, before, starts, P, root, M), "replay %d across the wrap" % rep)
    muted.replay()
    torch.cuda.synchronize()
    assert B.bcast_plan_status(plan)[0] == B.BCAST_ERR_TIMEOUT
    B.bcast_plan_clear_status(plan)
    # back to the host's count: it continues from the device's
    B.bcast_plan_set_replayable(plan, False)
    with pytest.raises(B.BcastError):
        B.bcast_plan_debug_set_epoch(plan, 2)  # below the count the device reached
    rb.reset(root, draw[:M])
    before = rb.to_host()
    B.bcast_run(plan, ptrs, root, M, torch.cuda.current_stream())
    got = rb.to_host()
    assert_same(got, oracle_end_state(info, before, starts, P, root, M), "host-counted run after the replays")
    B.bcast_plan_set_debug(plan, 200000, 2)
    B.bcast_run(plan, ptrs, root, M, torch.cuda.current_stream())
    torch.cuda.synchronize()
    assert B.bcast_plan_status(plan)[0] == B.BCAST_ERR_TIMEOUT, "the host's count fell behind the flags the replays left"
    plan.destroy()
