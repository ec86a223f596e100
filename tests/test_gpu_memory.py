"""bcast_buffers_alloc: buffers placed by region of the device's memory.

The method's result does not depend on where its buffers lie, its speed on this
device does: the tests check that the placed buffers are sound (distinct,
aligned, every byte usable, usable by every entry point, results bit-exact
against the oracle), that the verdict the call reports agrees with a
measurement taken here, that buffers can be given back in any order, and the
error paths.  Nothing is assumed about the state the device's memory is in.
"""
import gc

import numpy as np
import pytest
import torch

import oracle
from paper_1707_09414_amd import binding as B
from paper_1707_09414_amd import inputs
from gpu_harness import tensor_at

pytestmark = pytest.mark.gpu
KiB, MiB, GiB = inputs.KiB, inputs.MiB, 1 << 30
SLACK = 64 * MiB  # what the runtime itself may allocate meanwhile (code objects, events)


def used_bytes():
    gc.collect()
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    free, total = torch.cuda.mem_get_info()
    return total - free


def store_rate(ptrs, nbytes):
    """GB/s of the dependency-free store pattern over nbytes of each buffer."""
    s = torch.cuda.current_stream()
    best = 0.0
    B.bcast_debug_store_pattern(ptrs, nbytes, s)
    for _ in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(s)
        B.bcast_debug_store_pattern(ptrs, nbytes, s)
        e1.record(s)
        torch.cuda.synchronize()
        best = max(best, len(ptrs) * nbytes / e0.elapsed_time(e1) / 1e6)
    return best


def spread_measured(pa, pb, nbytes):
    """Whether writes to both groups together run clearly faster than to the slower
    group alone, or at the rate of a write set spread over regions.  A pass over a
    few GiB takes a fraction of a millisecond, so one disturbed pass is not a verdict:
    up to three attempts.  Returns (yes, together, slower) of the last attempt."""
    for attempt in range(3):
        together = store_rate(pa + pb, nbytes)
        slower = min(store_rate(pa, nbytes), store_rate(pb, nbytes))
        if together / slower > 1.05 or together > 6300.0:
            return True, together, slower
    return False, together, slower


def test_regions_of_the_device():
    n, each = B.bcast_memory_regions()
    _, total = torch.cuda.mem_get_info()
    assert n == 3 and each == total // 3


def test_broadcast_buffers_spread_over_two_regions():
    P, M, root = 16, 256 * MiB, 3
    before = used_bytes()
    ptrs, placed = B.bcast_buffers_alloc([M] * P, [0] * (P // 2) + [1] * (P // 2))
    try:
        assert len(set(ptrs)) == P and all(p and p % (2 * MiB) == 0 for p in ptrs)
        order = sorted(ptrs)
        assert all(b - a >= M for a, b in zip(order, order[1:])), "buffers overlap"
        assert placed in (B.BCAST_PLACED_NO, B.BCAST_PLACED_MEASURED)
        # the verdict against a measurement taken here: both halves together vs the slower half alone
        yes, together, slower = spread_measured(ptrs[: P // 2], ptrs[P // 2:], M)
        print("verdict %d, %.2f GiB in use before; store-only GB/s: slower half %.0f, together %.0f" % (placed, before / GiB, slower, together))
        if placed == B.BCAST_PLACED_MEASURED:
            assert yes, "reported as measured-spread, but writes to both halves run at %.0f GB/s, %.2fx the slower half alone" % (
                together, together / slower)
        # the buffers serve as rank buffers: a broadcast of the whole size, every rank against the root on the
        # device, and a prefix of every rank against the oracle's end state
        message = inputs.random_bytes(81, M)
        views = [tensor_at(p, M) for p in ptrs]
        for r in range(P):
            views[r].fill_(inputs.FILL_BYTE)
        views[root].copy_(torch.from_numpy(message))
        plan = B.bcast_plan_create(P, M, 0, B.BCAST_ALGO_CHAIN)
        B.bcast_run(plan, ptrs, root, M, torch.cuda.current_stream())
        torch.cuda.synchronize()
        assert B.bcast_plan_status(plan)[0] == B.BCAST_OK
        plan.destroy()
        for r in range(P):
            assert torch.equal(views[r], views[root]), "rank %d" % r
        n = 1 * MiB + 5
        state = np.full((P, n), inputs.FILL_BYTE, np.uint8)
        state[root] = message[:n]
        oracle.chain_bcast(state, P, root, n, 64 * KiB)
        for r in range(P):
            assert np.array_equal(views[r][:n].cpu().numpy(), state[r]), "rank %d differs from the oracle" % r
        del views
    finally:
        B.bcast_buffers_free(ptrs)


def test_reduction_buffers_result_in_another_region():
    P, root, count = 8, 5, 8 * MiB + 3
    nbytes = (count * 4 + 255) // 256 * 256
    ptrs, placed = B.bcast_buffers_alloc([nbytes] * (P + 1), [0] * P + [1])
    try:
        assert placed in (B.BCAST_PLACED_NO, B.BCAST_PLACED_MEASURED)
        rng = np.random.default_rng(82)
        x = rng.normal(0.0, 0.01, size=(P, count)).astype(np.float32)
        views = [tensor_at(p, nbytes) for p in ptrs]
        for r in range(P):
            views[r][: count * 4].copy_(torch.from_numpy(x[r].view(np.uint8)))
        views[P].fill_(0xEE)
        plan = B.bcast_plan_create(P, count * 4, 0, B.BCAST_ALGO_CHAIN)
        B.bcast_reduce_sum_f32(plan, ptrs[:P], ptrs[P], root, count, torch.cuda.current_stream())
        torch.cuda.synchronize()
        assert B.bcast_plan_status(plan)[0] == B.BCAST_OK
        plan.destroy()
        got = views[P].cpu().numpy()
        want, _ = oracle.chain_reduce_f32(np.ascontiguousarray(x), P, root, count, 16 * KiB)
        assert np.array_equal(got[: count * 4].view(np.uint32), want.view(np.uint32))
        assert (got[count * 4:] == 0xEE).all(), "wrote beyond the result"
        del views
    finally:
        B.bcast_buffers_free(ptrs)


def check_sound(ptrs, sizes):
    assert len(set(ptrs)) == len(ptrs) and all(p and p % 256 == 0 for p in ptrs)
    spans = sorted(zip(ptrs, sizes))
    assert all(a + n <= b for (a, n), (b, _) in zip(spans, spans[1:])), "buffers overlap"
    # every byte of every buffer is usable: write a pattern through the whole length, read it back
    for p, n in zip(ptrs, sizes):
        t = tensor_at(p, n)
        t.fill_(p >> 21 & 0xFF)
    torch.cuda.synchronize()
    for p, n in zip(ptrs, sizes):
        t = tensor_at(p, n)
        assert int(t[0]) == int(t[n - 1]) == int(t[n // 2]) == (p >> 21 & 0xFF)


def test_three_labels_large_groups_and_memory_mostly_in_use():
    """Groups under all three labels; a group larger than one slab; then the
    same with most of the device's memory in use, where a slab may have to be
    taken where it falls."""
    sizes = [256 * MiB] * 12
    ptrs, placed = B.bcast_buffers_alloc(sizes, [0] * 4 + [1] * 4 + [2] * 4)
    try:
        assert placed in (B.BCAST_PLACED_NO, B.BCAST_PLACED_MEASURED)
        check_sound(ptrs, sizes)
        if placed == B.BCAST_PLACED_MEASURED:
            # any two groups together are faster than the slower of them alone, or at the spread rate
            for a, b in ((0, 1), (0, 2), (1, 2)):
                pa, pb = ptrs[4 * a: 4 * a + 4], ptrs[4 * b: 4 * b + 4]
                yes, together, slower = spread_measured(pa, pb, 256 * MiB)
                assert yes, (a, b, together, slower)
    finally:
        B.bcast_buffers_free(ptrs)
    # 40 GiB under one label (three slabs) and 3 GiB under another
    sizes = [GiB] * 40 + [GiB] * 3
    ptrs, placed = B.bcast_buffers_alloc(sizes, [0] * 40 + [1] * 3)
    try:
        assert placed in (B.BCAST_PLACED_NO, B.BCAST_PLACED_MEASURED)
        check_sound(ptrs, sizes)
    finally:
        # given back in two parts, out of order
        B.bcast_buffers_free(ptrs[1::2])
        B.bcast_buffers_free(ptrs[0::2][::-1])
    in_use = used_bytes()
    _, total = torch.cuda.mem_get_info()
    if in_use > 16 * GiB:
        pytest.skip("the device's memory is in use by something else")
    ballast = [torch.empty(GiB, dtype=torch.uint8, device="cuda") for _ in range((total - in_use - 40 * GiB) // GiB)]
    sizes = [GiB] * 16
    ptrs, placed = B.bcast_buffers_alloc(sizes, [0] * 8 + [1] * 8)
    try:
        assert placed in (B.BCAST_PLACED_NO, B.BCAST_PLACED_MEASURED)
        check_sound(ptrs, sizes)
        yes, together, slower = spread_measured(ptrs[:8], ptrs[8:], GiB)
        print("verdict %d with %.0f GiB in use; store-only GB/s: together %.0f, slower half %.0f" % (placed, (in_use + len(ballast) * GiB) / GiB, together, slower))
        if placed == B.BCAST_PLACED_MEASURED:
            assert yes, (together, slower)
    finally:
        B.bcast_buffers_free(ptrs)
        del ballast


def test_errors_and_requests_beyond_the_memory():
    before = used_bytes()
    E = B.BCAST_ERR_ARG
    for sizes, regions in ([[], []], [[0], [0]], [[4096], [3]], [[4096], [-1]]):
        with pytest.raises(B.BcastError) as err:
            B.bcast_buffers_alloc(sizes, regions)
        assert err.value.status == E
    with pytest.raises(B.BcastError):
        B.bcast_buffers_alloc([4096, 4096], [0])
    assert abs(used_bytes() - before) <= SLACK, "a refused request left memory allocated"
    # one label only: nothing to tell apart; a tiny buffer still gets a slab of its own
    ptrs, placed = B.bcast_buffers_alloc([4096, 100], [1, 1])
    assert placed == B.BCAST_PLACED_BY_ORDER and ptrs[1] - ptrs[0] == 2 * MiB
    check_sound(ptrs, [4096, 100])
    # only what the library handed out can be given back, and only once
    with pytest.raises(B.BcastError) as err:
        B.bcast_buffers_free([ptrs[0] + 4096])
    assert err.value.status == E
    B.bcast_buffers_free([ptrs[1]])
    with pytest.raises(B.BcastError):
        B.bcast_buffers_free([ptrs[1], ptrs[0]])  # the second one is still freed
    with pytest.raises(B.BcastError):
        B.bcast_buffers_free([ptrs[0]])
    assert abs(used_bytes() - before) <= SLACK
    # more memory than the device has: nothing stays allocated
    _, each = B.bcast_memory_regions()
    with pytest.raises(B.BcastError) as err:
        B.bcast_buffers_alloc([each, each, each, each], [0, 0, 1, 1])
    assert err.value.status == B.BCAST_ERR_NOMEM
    assert abs(used_bytes() - before) <= SLACK
