"""Chain reduction (fp32 sum) on the GPU against the CPU oracle, bit for bit.

Both sides add in the same order (own contribution + running sum from the right
neighbour, position P-1 first) and in fp32, so the 32-bit patterns must agree:
ragged counts, several chunks, every stage count, non-zero roots, in place at
the root, denormals, signed zeros, values whose sum depends on the order."""
import numpy as np
import pytest
import torch

import oracle
from paper_1707_09414_amd import binding as B
from paper_1707_09414_amd import inputs

pytestmark = pytest.mark.gpu
KiB, MiB = inputs.KiB, inputs.MiB
GUARD = 64  # floats before and after every buffer, kept at a canary value
CANARY = np.float32(-123456.0)


def contributions(seed, P, count):
    """N(0, 0.01) like the gradients of a network, salted with the values that
    make fp32 sums interesting: denormals, signed zeros, exact integers around
    2^24, huge magnitudes that cancel."""
    rng = np.random.default_rng(seed)
    x = rng.normal(0.0, 0.01, size=(P, count)).astype(np.float32)
    if count >= 8:
        x[:, 0] = np.float32(1e-40) * rng.integers(-5, 6, size=P)        # denormals
        x[:, 1] = np.where(rng.random(P) < 0.5, np.float32(0.0), np.float32(-0.0))
        x[:, 2] = rng.integers(-3, 4, size=P).astype(np.float32)
        x[:, 2][rng.integers(0, P)] = np.float32(2.0 ** 24)
        x[:, 3] = np.float32(1e30) * rng.choice([-1.0, 1.0], size=P)
        x[:, 4] = rng.integers(-(1 << 20), 1 << 20, size=P).astype(np.float32)
        x[:, 5] = np.float32(3.0e-39)                                     # sums of denormals that become normal
    return x


def reduce_and_check(P, root, count, C, seed=0, stages=0, lanes=0, in_place=False, values=None, plan=None, cap=None):
    send = contributions(seed, P, count) if values is None else values
    cap = count if cap is None else cap
    dev = []
    for r in range(P):
        t = torch.full((cap + 2 * GUARD,), float(CANARY), dtype=torch.float32, device="cuda")
        t[GUARD: GUARD + count].copy_(torch.from_numpy(send[r]))
        dev.append(t)
    recv_t = dev[root] if in_place else torch.full((cap + 2 * GUARD,), float(CANARY), dtype=torch.float32, device="cuda")
    ptrs = [t.data_ptr() + 4 * GUARD for t in dev]
    own = plan is None
    if own:
        plan = B.bcast_plan_create(P, cap * 4, C, B.BCAST_ALGO_CHAIN)
    try:
        if stages:
            B.bcast_plan_set_stages(plan, stages)
        if lanes:
            B.bcast_plan_set_lanes(plan, lanes)
        # staging memory for the running sums between stages: reserved up front, the run path never allocates
        B.bcast_plan_reserve_reduce(plan, cap, max(2, stages))
        info = B.bcast_reduce_info(plan, count)
        B.bcast_reduce_sum_f32(plan, ptrs, recv_t.data_ptr() + 4 * GUARD, root, count, torch.cuda.current_stream())
        torch.cuda.synchronize()
        st, detail = B.bcast_plan_status(plan)
        assert st == B.BCAST_OK, "plan status %d detail %x" % (st, detail)
    finally:
        if own:
            plan.destroy()
    want, res = oracle.chain_reduce_f32(np.ascontiguousarray(send), P, root, count, max(1, info["chunk_bytes"] // 4) if count else 1)
    got = recv_t.cpu().numpy()
    what = "P=%d root=%d count=%d C=%d stages=%d lanes=%d in_place=%s" % (P, root, count, C, stages, lanes, in_place)
    bad = np.nonzero(got[GUARD: GUARD + count].view(np.uint32) != want.view(np.uint32))[0]
    assert bad.size == 0, "%s: %d elements differ, first at %d: got %r want %r" % (what, bad.size, bad[0], got[GUARD + bad[0]], want[bad[0]])
    assert (got[:GUARD] == CANARY).all() and (got[GUARD + count:] == CANARY).all(), what + ": wrote outside the result"
    for r in range(P):
        if in_place and r == root:
            continue
        h = dev[r].cpu().numpy()
        assert np.array_equal(h[GUARD: GUARD + count].view(np.uint32), send[r].view(np.uint32)), what + ": contribution %d changed" % r
        assert (h[:GUARD] == CANARY).all() and (h[GUARD + count:] == CANARY).all()
    if P > 1 and count > 0:
        assert res.steps == info["nchunks"] + P - 2
        assert info["algorithmic_bytes"] == (P + 1) * count * 4
    return info


def test_hand_worked_rounding_cases():
    """The fixtures that pin the oracle's order of additions, on the GPU."""
    import os

    path = os.path.join(os.path.dirname(__file__), "golden", "reduce_order.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    for row in rows:
        P, root = int(row[0]), int(row[1])
        vals = np.repeat(np.array([[float(v)] for v in row[2:2 + P]], dtype=np.float32), 37, axis=1).copy()
        reduce_and_check(P, root, 37, 64, values=vals, stages=1)
        reduce_and_check(P, root, 37, 64, values=vals, stages=max(1, P - 1))


@pytest.mark.parametrize("P", [1, 2, 3, 5, 8, 17, 64])
@pytest.mark.parametrize("count,C", [(1, 16), (3, 16), (4, 16), (5, 4096), (1023, 1024), (70001, 32 * KiB), (MiB // 4 + 3, 0), (3 * MiB // 4, 256 * KiB)])
def test_counts_and_ranks(P, count, C):
    reduce_and_check(P, P // 3, count, C, seed=P * 1000 + count)


@pytest.mark.parametrize("P,stages", [(2, 1), (5, 1), (5, 2), (5, 4), (8, 2), (8, 3), (9, 8), (17, 4), (64, 1), (64, 2), (64, 9), (64, 63), (64, 100)])
@pytest.mark.parametrize("count,C,lanes", [(7, 16, 0), (50001, 8 * KiB, 3), (MiB + 5, 128 * KiB, 0)])
def test_stage_counts(P, stages, count, C, lanes):
    info = reduce_and_check(P, P - 1, count, C, seed=stages, stages=stages, lanes=lanes)
    assert info["stages"] == min(stages, P - 1)


@pytest.mark.parametrize("P,root", [(2, 0), (2, 1), (4, 3), (16, 5)])
def test_in_place_at_the_root(P, root):
    reduce_and_check(P, root, 300001, 64 * KiB, seed=9, in_place=True)
    reduce_and_check(P, root, 17, 16, seed=10, in_place=True, stages=1)


def test_degenerate_and_repeated_runs():
    reduce_and_check(4, 2, 0, 4096, cap=1024)
    reduce_and_check(1, 0, 1000, 4096)
    reduce_and_check(1, 0, 1000, 4096, in_place=True)
    # one plan, many runs: growing stage counts re-reserve the staging memory, sizes change, flags are reused
    P, cap = 9, 200000
    plan = B.bcast_plan_create(P, cap * 4, 16 * KiB, B.BCAST_ALGO_CHAIN)
    for i, (stages, count) in enumerate([(1, 1000), (2, cap), (5, 77777), (8, 12345), (2, cap), (3, 4)]):
        reduce_and_check(P, i % P, count, 16 * KiB, seed=100 + i, stages=stages, plan=plan, cap=cap)
    # a broadcast on the same plan in between shares the flags and the epoch
    from gpu_harness import run_and_check

    noise = inputs.random_bytes(3, cap * 4)
    B.bcast_plan_set_stages(plan, 3)
    run_and_check(P, 4, cap * 4 - 12, 16 * KiB, B.BCAST_ALGO_CHAIN, noise, plan=plan, cap=cap * 4)
    reduce_and_check(P, 4, cap, 16 * KiB, seed=200, stages=3, plan=plan, cap=cap)
    plan.destroy()


def test_argument_errors_launch_nothing():
    P, count = 4, 1024
    send = [torch.zeros(count + 8, dtype=torch.float32, device="cuda") for _ in range(P)]
    recv = torch.full((count + 8,), 7.0, dtype=torch.float32, device="cuda")
    ptrs = [t.data_ptr() for t in send]
    plan = B.bcast_plan_create(P, count * 4, 4096, B.BCAST_ALGO_CHAIN)
    E = B.BCAST_ERR_ARG
    assert B.bcast_reduce_status(plan, ptrs, recv.data_ptr(), P, count) == E           # root out of range
    assert B.bcast_reduce_status(plan, ptrs, recv.data_ptr(), 0, count + 1) == E       # longer than the plan
    assert B.bcast_reduce_status(plan, ptrs, recv.data_ptr() + 4, 0, 16) == E          # misaligned result
    assert B.bcast_reduce_status(plan, [ptrs[0] + 8, ptrs[1], ptrs[2], ptrs[3]], recv.data_ptr(), 0, 16) == E  # misaligned input
    assert B.bcast_reduce_status(plan, [ptrs[0], ptrs[0], ptrs[2], ptrs[3]], recv.data_ptr(), 0, count) == E   # duplicate
    assert B.bcast_reduce_status(plan, [ptrs[0], ptrs[0] + 64, ptrs[2], ptrs[3]], recv.data_ptr(), 0, count) == E  # overlap
    assert B.bcast_reduce_status(plan, ptrs, ptrs[1], 0, count) == E                   # result on another rank's contribution
    assert B.bcast_reduce_status(plan, [ptrs[0], 0, ptrs[2], ptrs[3]], recv.data_ptr(), 0, count) == E
    torch.cuda.synchronize()
    assert bool((recv == 7.0).all())
    plan.destroy()


def test_wait_limit_in_the_reduction():
    """Stage 1 of 3 never publishes: stage 2 gives up after the (tiny) wait
    limit, every wave exits, the plan reports it and works again afterwards."""
    P, count = 7, 100000
    send = contributions(1, P, count)
    dev = [torch.from_numpy(send[r]).cuda() for r in range(P)]
    recv = torch.zeros(count, dtype=torch.float32, device="cuda")
    plan = B.bcast_plan_create(P, count * 4, 16 * KiB, B.BCAST_ALGO_CHAIN)
    B.bcast_plan_set_stages(plan, 3)       # hops 1-2, 3-4, 5-6
    B.bcast_plan_reserve_reduce(plan, count, 3)
    B.bcast_plan_set_debug(plan, 200000, 3)  # the stage that plays hop 3 stays silent; 2 ms limit
    B.bcast_reduce_sum_f32(plan, dev, recv, 0, count)
    torch.cuda.synchronize()
    st, detail = B.bcast_plan_status(plan)
    assert st == B.BCAST_ERR_TIMEOUT and detail >> 32 == 5 and (detail & 0xFFFFFFFF) == 0, hex(detail)
    B.bcast_plan_clear_status(plan)
    B.bcast_plan_set_debug(plan, 0, 0)
    B.bcast_reduce_sum_f32(plan, dev, recv, 0, count)
    torch.cuda.synchronize()
    assert B.bcast_plan_status(plan)[0] == B.BCAST_OK
    want, _ = oracle.chain_reduce_f32(send, P, 0, count, 4 * KiB)
    assert np.array_equal(recv.cpu().numpy().view(np.uint32), want.view(np.uint32))
    plan.destroy()


def test_vgg16_gradient_sized_reduction_p16():
    """The VGG-16 parameter count (138M fp32, N(0, 0.01)) summed over 16 ranks:
    the full result is compared with the oracle's; then the same as an allreduce,
    every rank's full result compared."""
    P, root = 16, 0
    count = sum(inputs.vgg16_tensor_bytes()) // 4
    base = inputs.vgg16_packed_message(2)[0].view(np.float32)   # one N(0, 0.01) draw of the right size
    assert base.size == count
    dev, host = [], np.empty((P, count), dtype=np.float32)
    for r in range(P):
        # every rank its own values: the draw, shifted by a few thousand elements and rescaled
        host[r] = np.roll(base, 4099 * r) * np.float32(1.0 + r / 64.0)
        dev.append(torch.from_numpy(host[r]).cuda())
    recv = torch.empty(count, dtype=torch.float32, device="cuda")
    plan = B.bcast_plan_create(P, count * 4, 0, B.BCAST_ALGO_CHAIN)
    B.bcast_plan_reserve_reduce(plan, count, 2)
    info = B.bcast_reduce_info(plan, count)
    B.bcast_reduce_sum_f32(plan, dev, recv, root, count, torch.cuda.current_stream())
    torch.cuda.synchronize()
    assert B.bcast_plan_status(plan)[0] == B.BCAST_OK
    plan.destroy()
    want, res = oracle.chain_reduce_f32(host, P, root, count, info["chunk_bytes"] // 4)
    assert res.steps == info["nchunks"] + P - 2
    assert np.array_equal(recv.cpu().numpy().view(np.uint32), want.view(np.uint32))
    del recv
    # the same size as an allreduce, in place: every rank must end with exactly these bits
    plan = B.bcast_plan_create(P, count * 4, 0, B.BCAST_ALGO_CHAIN)
    B.bcast_allreduce_sum_f32(plan, dev, dev, root, count, torch.cuda.current_stream())
    torch.cuda.synchronize()
    assert B.bcast_plan_status(plan)[0] == B.BCAST_OK
    plan.destroy()
    for r in range(P):
        assert np.array_equal(dev[r].cpu().numpy().view(np.uint32), want.view(np.uint32)), "rank %d" % r


@pytest.mark.parametrize("P,root,count,in_place", [(2, 1, 5, False), (4, 0, 70001, True), (8, 5, 1 << 20, False), (16, 3, 300000, True), (64, 17, 65536, False)])
def test_allreduce_is_reduce_then_broadcast(P, root, count, in_place):
    """Every rank ends with the bits the chain reduction defines."""
    send = contributions(P + count, P, count)
    dev = [torch.from_numpy(send[r]).cuda() for r in range(P)]
    recv = dev if in_place else [torch.full((count,), float(CANARY), dtype=torch.float32, device="cuda") for _ in range(P)]
    plan = B.bcast_plan_create(P, count * 4, 64 * KiB, B.BCAST_ALGO_CHAIN)
    if P % 2 == 0 and count > 5:
        B.bcast_plan_reserve_reduce(plan, count, 2)   # else: no staging memory, the reduction runs in one stage
    B.bcast_allreduce_sum_f32(plan, dev, recv, root, count, torch.cuda.current_stream())
    torch.cuda.synchronize()
    assert B.bcast_plan_status(plan)[0] == B.BCAST_OK
    want, _ = oracle.chain_reduce_f32(send, P, root, count, 16 * KiB)
    for r in range(P):
        assert np.array_equal(recv[r].cpu().numpy().view(np.uint32), want.view(np.uint32)), r
        if not in_place:
            assert np.array_equal(dev[r].cpu().numpy().view(np.uint32), send[r].view(np.uint32)), r
    # a result placed on another rank's contribution is refused
    if not in_place:
        with pytest.raises(B.BcastError):
            B.bcast_allreduce_sum_f32(plan, dev, [dev[(r + 1) % P] for r in range(P)], root, count)
    plan.destroy()


def test_staging_memory_is_reserved_never_allocated_by_a_run():
    """Without a reservation the library's own choice is one stage (no staging
    memory needed); a stage count the caller asks for beyond the reservation is
    refused and launches nothing; the reservation grows on request."""
    P, count = 6, 50000
    send = contributions(5, P, count)
    dev = [torch.from_numpy(send[r]).cuda() for r in range(P)]
    recv = torch.full((count,), 7.0, dtype=torch.float32, device="cuda")
    want, _ = oracle.chain_reduce_f32(send, P, 2, count, 4 * KiB)
    plan = B.bcast_plan_create(P, count * 4, 16 * KiB, B.BCAST_ALGO_CHAIN)
    assert B.bcast_reduce_info(plan, count)["stages"] == 1
    B.bcast_reduce_sum_f32(plan, dev, recv, 2, count)
    torch.cuda.synchronize()
    assert np.array_equal(recv.cpu().numpy().view(np.uint32), want.view(np.uint32))
    recv.fill_(7.0)
    B.bcast_plan_set_stages(plan, 3)
    assert B.bcast_reduce_status(plan, dev, recv, 2, count) == B.BCAST_ERR_CAPACITY
    B.bcast_plan_reserve_reduce(plan, count // 2, 3)          # enough for half the size only
    assert B.bcast_reduce_status(plan, dev, recv, 2, count) == B.BCAST_ERR_CAPACITY
    torch.cuda.synchronize()
    assert bool((recv == 7.0).all())
    B.bcast_reduce_sum_f32(plan, dev, recv, 2, count // 2)
    torch.cuda.synchronize()
    assert np.array_equal(recv[: count // 2].cpu().numpy().view(np.uint32), want[: count // 2].view(np.uint32))
    assert bool((recv[count // 2:] == 7.0).all())
    B.bcast_plan_reserve_reduce(plan, count, 3)
    assert B.bcast_reduce_info(plan, count)["stages"] == 3
    B.bcast_reduce_sum_f32(plan, dev, recv, 2, count)
    torch.cuda.synchronize()
    assert np.array_equal(recv.cpu().numpy().view(np.uint32), want.view(np.uint32))
    with pytest.raises(B.BcastError):
        B.bcast_plan_reserve_reduce(plan, count + 1, 2)       # beyond the plan's size
    with pytest.raises(B.BcastError):
        B.bcast_plan_reserve_reduce(plan, count, -1)
    B.bcast_plan_reserve_reduce(plan, count, 0)               # 0 = the library's own choice for this size
    plan.destroy()


def test_reduction_table_entries_shape_the_run():
    """What a plan leaves open (chunk 0, no stage request) comes from the
    reduction's tuning table: stage count, chunk and trip size; the reservation
    with stages = 0 follows it; a plan that fixes its chunk ignores it."""
    P, count = 6, 300000
    send = contributions(8, P, count)
    dev = [torch.from_numpy(send[r]).cuda() for r in range(P)]
    recv = torch.zeros(count, dtype=torch.float32, device="cuda")
    want, _ = oracle.chain_reduce_f32(send, P, 1, count, 4 * KiB)
    B.bcast_tune_clear()
    try:
        with pytest.raises(B.BcastError):
            B.bcast_tune_reduce_get(P, count * 4)
        B.bcast_tune_reduce_put(P, 1 << 20, chunk_bytes=96 * KiB, stages=3, trip_bytes=1024, usec=5.0)
        for bad in (dict(chunk_bytes=0, stages=1, trip_bytes=4096), dict(chunk_bytes=24, stages=1, trip_bytes=4096),
                    dict(chunk_bytes=4096, stages=0, trip_bytes=4096), dict(chunk_bytes=4096, stages=1, trip_bytes=2048)):
            with pytest.raises(B.BcastError):
                B.bcast_tune_reduce_put(P, 1 << 20, **bad)
        assert B.bcast_tune_reduce_get(P, count * 4)["stages"] == 3
        plan = B.bcast_plan_create(P, count * 4, 0, B.BCAST_ALGO_CHAIN)
        # nothing reserved yet: the entry's three stages do not fit, the choice shrinks to one and the entry's chunk is not used
        assert B.bcast_reduce_info(plan, count)["stages"] == 1
        B.bcast_plan_reserve_reduce(plan, count, 0)
        info = B.bcast_reduce_info(plan, count)
        assert (info["stages"], info["chunk_bytes"], info["trip_bytes"]) == (3, 96 * KiB, 1024)
        B.bcast_reduce_sum_f32(plan, dev, recv, 1, count)
        torch.cuda.synchronize()
        assert np.array_equal(recv.cpu().numpy().view(np.uint32), want.view(np.uint32))
        plan.destroy()
        fixed = B.bcast_plan_create(P, count * 4, 64 * KiB, B.BCAST_ALGO_CHAIN)
        B.bcast_plan_reserve_reduce(fixed, count, 2)
        info = B.bcast_reduce_info(fixed, count)
        assert (info["stages"], info["chunk_bytes"]) == (2, 64 * KiB)
        fixed.destroy()
    finally:
        B.bcast_tune_clear()


def test_tune_reduce_installs_measured_entries(tmp_path):
    """The sweep itself, small: entries for every size, saved and loaded with the
    broadcast's in one file; the tuned shape gives the oracle's bits."""
    P = 5
    B.bcast_tune_clear()
    try:
        path = str(tmp_path / "table.txt")
        B.bcast_tune_set(P, 1 << 16, B.BCAST_ALGO_DIRECT, 0, 3.0)
        B.bcast_tune_reduce(P, 1 << 14, 1 << 18, torch.cuda.current_stream(), None)
        entries = {b: B.bcast_tune_reduce_get(P, 1 << b) for b in range(14, 19)}
        assert all(1 <= e["stages"] <= 4 and e["usec"] > 0 and e["trip_bytes"] in (1024, 4096) for e in entries.values())
        B.bcast_tune_save(path)
        B.bcast_tune_clear()
        B.bcast_tune_load(path)
        assert B.bcast_tune_lookup(P, 1 << 16)[0] == B.BCAST_ALGO_DIRECT
        for b, e in entries.items():
            got = B.bcast_tune_reduce_get(P, 1 << b)
            assert (got["stages"], got["chunk_bytes"], got["trip_bytes"]) == (e["stages"], e["chunk_bytes"], e["trip_bytes"])
        count = (1 << 16) + 5
        plan = B.bcast_plan_create(P, count * 4, 0, B.BCAST_ALGO_CHAIN)
        B.bcast_plan_reserve_reduce(plan, count, 0)
        assert B.bcast_reduce_info(plan, count)["stages"] == B.bcast_tune_reduce_get(P, count * 4)["stages"]
        reduce_and_check(P, 3, count, 0, seed=77, plan=plan, cap=count)
        plan.destroy()
    finally:
        B.bcast_tune_clear()


@pytest.mark.parametrize("seed", [11, 12])
def test_random_reduction_configurations(seed):
    """Seeded sweep: ranks, root, count, chunk size, stage and lane counts, in
    place or not."""
    rng = np.random.default_rng(seed)
    for case in range(60):
        P = int(rng.integers(1, 65)) if case % 3 else int(rng.integers(1, 9))
        root = int(rng.integers(0, P))
        count = int(rng.choice([0, 1, 2, 3, 4, 7, 1024, 4097, 100003, int(rng.integers(1, 400000))]))
        C = int(rng.choice([0, 16, 112, 4096, 65536, 1 << 20])) if rng.random() < 0.8 else 16 * int(rng.integers(1, 20000))
        stages = int(rng.integers(0, 70))
        lanes = int(rng.choice([0, 0, 1, 3, 32, 100]))
        in_place = bool(rng.integers(0, 2))
        try:
            reduce_and_check(P, root, count, C, seed=1000 * seed + case, stages=stages, lanes=lanes, in_place=in_place)
        except Exception as e:
            raise AssertionError("case %d: P=%d root=%d count=%d C=%d stages=%d lanes=%d in_place=%s: %s"
                                 % (case, P, root, count, C, stages, lanes, in_place, e))
