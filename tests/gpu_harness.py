"""Shared helpers for the GPU parity tests: allocate P rank buffers with guard
bands, run the library through its C ABI (via the ctypes binding), and build the
expected end state with the CPU oracle on the same seeded inputs."""
import numpy as np
import torch

import oracle
from paper_1707_09414_amd import binding as B
from paper_1707_09414_amd import inputs

GUARD = 256  # bytes of 0xFF kept before and after every rank buffer
FILL = inputs.FILL_BYTE
# How run_and_check asks the wave-per-rank chain to hand trips over inside a workgroup
# (a test module sets it for all its cases): one of the library's modes, or PREFER_LDS =
# LDS wherever the slots fit the device (whatever the message size), else the library's choice.
PREFER_LDS = -1
RANK_HANDOFF = B.BCAST_HANDOFF_AUTO


def set_rank_handoff(plan, M, ptrs=None):
    """Apply RANK_HANDOFF to a plan that runs the wave-per-rank chain on M bytes."""
    if RANK_HANDOFF != PREFER_LDS:
        B.bcast_plan_set_rank_handoff(plan, RANK_HANDOFF)
        return
    B.bcast_plan_set_rank_handoff(plan, B.BCAST_HANDOFF_LDS)
    try:
        B.bcast_plan_info(plan, M, ptrs)
    except B.BcastError:
        B.bcast_plan_set_rank_handoff(plan, B.BCAST_HANDOFF_AUTO)  # the slots do not fit this shape


class RankBuffers:
    """P device allocations of GUARD + offset_r + cap + GUARD bytes, all 0xFF;
    rank r's buffer starts at GUARD + offset_r."""

    def __init__(self, P, cap, offsets=None, device="cuda:0"):
        self.P = P
        self.cap = cap
        self.offsets = list(offsets) if offsets is not None else [0] * P
        assert len(self.offsets) == P and all(0 <= o < 64 for o in self.offsets)
        self.total = GUARD + 64 + cap + GUARD
        self.raw = [torch.full((self.total,), FILL, dtype=torch.uint8, device=device) for _ in range(P)]

    def start(self, r):
        return GUARD + self.offsets[r]

    def ptrs(self):
        return [self.raw[r].data_ptr() + self.start(r) for r in range(self.P)]

    def reset(self, root, message):
        for r in range(self.P):
            self.raw[r].fill_(FILL)
        self.set_message(root, message)

    def set_message(self, root, message):
        m = torch.from_numpy(np.ascontiguousarray(message))
        self.raw[root][self.start(root): self.start(root) + m.numel()].copy_(m)

    def to_host(self):
        torch.cuda.synchronize()
        return [t.cpu().numpy() for t in self.raw]


def expected_with_oracle(bufs_host, starts, root, M, schedule):
    """Apply `schedule` (a function over a [P, M] uint8 array) with the oracle to
    the message region of each host buffer; everything else must stay as it was."""
    P = len(bufs_host)
    region = np.stack([bufs_host[r][starts[r]: starts[r] + M] for r in range(P)]) if M else np.zeros((P, 0), np.uint8)
    region = np.ascontiguousarray(region)
    res = schedule(region)
    exp = [b.copy() for b in bufs_host]
    for r in range(P):
        exp[r][starts[r]: starts[r] + M] = region[r]
    return exp, res


def oracle_schedule(algo, P, root, M, C):
    if algo == B.BCAST_ALGO_CHAIN:
        return lambda a: oracle.chain_bcast(a, P, root, M, max(1, C))
    if algo == B.BCAST_ALGO_DIRECT:
        return lambda a: oracle.direct_bcast(a, P, root, M)
    if algo == B.BCAST_ALGO_BINOMIAL:
        return lambda a: oracle.binomial_bcast(a, P, root, M)
    if algo == B.BCAST_ALGO_SCATTER_ALLGATHER:
        return lambda a: oracle.scatter_allgather_bcast(a, P, root, M)
    if algo == B.BCAST_ALGO_FANOUT:
        # the fan-out has no schedule of its own in the paper: its result is the definition
        return lambda a: oracle.naive_bcast(a, root, M)
    raise ValueError(algo)


def assert_same(got, exp, what):
    for r, (g, e) in enumerate(zip(got, exp)):
        if not np.array_equal(g, e):
            bad = np.flatnonzero(g != e)
            raise AssertionError("%s: rank %d differs at %d bytes, first at allocation offset %d (got %d, want %d)"
                                 % (what, r, bad.size, bad[0], g[bad[0]], e[bad[0]]))


def run_and_check(P, root, M, C, algo, message, offsets=None, cap=None, lanes=0, stream=None, plan=None, stages=0, radix=0, trip=0, block=0,
                  waves=0):
    """One broadcast on the GPU, compared byte for byte (guards included) with
    the oracle's end state.  Returns the plan info used."""
    cap = M if cap is None else cap
    rb = RankBuffers(P, max(cap, 1), offsets)
    rb.reset(root, message[:M])
    before = rb.to_host()
    own = plan is None
    if own:
        plan = B.bcast_plan_create(P, cap, C, algo)
    try:
        if lanes:
            B.bcast_plan_set_lanes(plan, lanes)
        if stages:
            B.bcast_plan_set_stages(plan, stages)
        if radix:
            B.bcast_plan_set_radix(plan, radix)
        if trip:
            B.bcast_plan_set_trip(plan, trip)
        if block:
            B.bcast_plan_set_block_threads(plan, block)
        if waves:
            B.bcast_plan_set_chain_waves(plan, waves)
        if waves == B.BCAST_CHAIN_WAVE_PER_RANK:
            set_rank_handoff(plan, M, rb.ptrs())
        info = B.bcast_plan_info(plan, M, rb.ptrs())
        B.bcast_run(plan, rb.ptrs(), root, M, stream)
        got = rb.to_host()
        st, detail = B.bcast_plan_status(plan)
        assert st == B.BCAST_OK, "plan status %d detail %x" % (st, detail)
    finally:
        if own:
            plan.destroy()
    starts = [rb.start(r) for r in range(P)]
    if info["algo"] == B.BCAST_ALGO_KNOMIAL:
        schedule = lambda a: oracle.knomial_bcast(a, P, root, M, max(2, info["stages"]))
    elif info["algo"] == B.BCAST_ALGO_KNOMIAL_PIPELINED:
        schedule = lambda a: oracle.knomial_pipeline_bcast(a, P, root, M, max(16, info["chunk_bytes"]), max(2, info["stages"]))
    else:
        schedule = oracle_schedule(info["algo"], P, root, M, info["chunk_bytes"])
    exp, res = expected_with_oracle(before, starts, root, M, schedule)
    if info["algo"] == B.BCAST_ALGO_KNOMIAL and P > 1 and M > 0:
        assert info["launches"] == res.steps, "one launch per k-nomial round"
    assert_same(got, exp, "P=%d root=%d M=%d C=%d algo=%d offsets=%s" % (P, root, M, C, algo, offsets))
    return info


class _DeviceSpan:
    """`nbytes` bytes of device memory at `ptr`, described the way torch reads foreign device arrays."""

    def __init__(self, ptr, nbytes):
        self.__cuda_array_interface__ = {"shape": (int(nbytes),), "typestr": "|u1", "data": (int(ptr), False), "version": 2}


def tensor_at(ptr, nbytes):
    """A uint8 tensor over device memory the library allocated (no copy, no ownership)."""
    return torch.as_tensor(_DeviceSpan(ptr, nbytes), device="cuda")
