"""The five benchmark configurations at their full sizes, on the GPU, through
the C ABI, in the launch configuration bench.py uses (tuned table installed).

A broadcast is exact data movement, so the oracle's end state for every rank is
the root's message.  Where P*M fits comfortably in host memory the oracle's
payload simulation is run at full size and compared row by row; for the two
largest configurations the oracle runs its schedule at full scale (step count)
and its payload simulation at full P on a prefix of the message, and the GPU
buffers are compared with the message itself: three ranks completely, every
other rank on seeded 1 MiB windows copied back to the host, plus a device-side
whole-buffer comparison."""
import numpy as np
import pytest
import torch

import oracle
from paper_1707_09414_amd import binding as B
from paper_1707_09414_amd import inputs, tuned

pytestmark = pytest.mark.gpu
KiB, MiB, GiB = inputs.KiB, inputs.MiB, inputs.GiB
FILL = inputs.FILL_BYTE


@pytest.fixture(scope="module", autouse=True)
def shipped_table():
    B.bcast_tune_clear()
    assert tuned.load_default_table() is not None, "the shipped MI355X tuning table is missing"
    yield
    B.bcast_tune_clear()


def device_buffers(P, M, root, msg, slack=0):
    bufs = [torch.full((M + slack,), FILL, dtype=torch.uint8, device="cuda") for _ in range(P)]
    bufs[root][:M].copy_(torch.from_numpy(msg))
    return bufs


def check_against_message(bufs, msg, M, root, full_ranks, windows=64, seed=0):
    d_msg = torch.from_numpy(msg).cuda()
    rng = np.random.default_rng(seed)
    for r, t in enumerate(bufs):
        assert torch.equal(t[:M], d_msg), "rank %d differs from the message (device compare)" % r
        assert bool((t[M:] == FILL).all()), "rank %d: bytes beyond the message were written" % r
        if r in full_ranks:
            assert np.array_equal(t[:M].cpu().numpy(), msg), "rank %d differs from the message" % r
        else:
            starts = [0, max(0, M - MiB)] + [int(x) for x in rng.integers(0, max(1, M - MiB), size=windows)]
            for s in starts:
                e = min(M, s + MiB)
                assert np.array_equal(t[s:e].cpu().numpy(), msg[s:e]), "rank %d differs in [%d, %d)" % (r, s, e)


def oracle_prefix_check(P, root, msg, C, prefix):
    """Full-P payload simulation on a prefix of the message + full-scale schedule."""
    host = np.full((P, prefix), FILL, dtype=np.uint8)
    host[root] = msg[:prefix]
    res = oracle.chain_bcast(host, P, root, prefix, C)
    assert (host == msg[:prefix][None, :]).all()
    assert res.steps == -(-prefix // C) + P - 2
    full = oracle.chain_bcast(None, P, root, msg.nbytes, C)
    assert full.steps == -(-msg.nbytes // C) + P - 2 and full.bytes_copied == (P - 1) * msg.nbytes


def test_config2_message_size_sweep_p8():
    """4 B .. 64 MiB in powers of two, P=8, root 0: chain (tuned chunk and one
    swept chunk), direct and binomial against the oracle's full simulation."""
    P, root = 8, 0
    draw = inputs.random_bytes(1, 64 * MiB)
    sizes = inputs.sweep_message_sizes(4, 64 * MiB)
    assert len(sizes) == 25
    chunks = inputs.sweep_chunk_sizes()
    assert chunks[0] == 8 * KiB and chunks[-1] == 4 * MiB and len(chunks) == 10
    stream = torch.cuda.current_stream()
    for i, M in enumerate(sizes):
        msg = draw[:M]
        want = np.full((P, M), FILL, dtype=np.uint8)
        want[root] = msg
        swept = chunks[i % len(chunks)]
        steps = oracle.chain_bcast(want, P, root, M, swept).steps
        assert steps == -(-M // swept) + P - 2
        for algo, C in [(B.BCAST_ALGO_CHAIN, 0), (B.BCAST_ALGO_CHAIN, swept), (B.BCAST_ALGO_DIRECT, 0),
                        (B.BCAST_ALGO_BINOMIAL, 0), (B.BCAST_ALGO_AUTO, 0)]:
            bufs = device_buffers(P, M, root, msg, slack=64)
            plan = B.bcast_plan_create(P, M, C, algo)
            B.bcast_run(plan, bufs, root, M, stream)
            torch.cuda.synchronize()
            assert B.bcast_plan_status(plan)[0] == B.BCAST_OK
            plan.destroy()
            for r in range(P):
                got = bufs[r].cpu().numpy()
                assert np.array_equal(got[:M], want[r]), (M, algo, C, r)
                assert (got[M:] == FILL).all(), (M, algo, C, r)
            del bufs


def test_config3_vgg16_per_tensor_and_packed_p16():
    """138M fp32 VGG-16 parameters, N(0, 0.01), seed 2, P=16, root 0: one
    broadcast per tensor (32 runs, AUTO from the tuning table) and one packed."""
    P, root = 16, 0
    msg, spans = inputs.vgg16_packed_message(2)
    M = msg.nbytes
    assert M == 553430176 and len(spans) == 32
    stream = torch.cuda.current_stream()

    # tensor by tensor, each tensor in its own set of P buffers carved out of one allocation per rank
    bufs = device_buffers(P, M, root, msg)
    plan = B.bcast_plan_create(P, max(n for _, n in spans), 0, B.BCAST_ALGO_AUTO)
    algos = set()
    for off, n in spans:
        views = [b[off: off + n] for b in bufs]
        algos.add(B.bcast_plan_info(plan, n, views)["algo"])
        B.bcast_run(plan, views, root, n, stream)
    torch.cuda.synchronize()
    assert B.bcast_plan_status(plan)[0] == B.BCAST_OK
    plan.destroy()
    assert len(algos) >= 2, "the message mix should exercise more than one algorithm"
    check_against_message(bufs, msg, M, root, full_ranks={1, 8, 15}, seed=3)

    # packed into one buffer, chain
    for b in bufs[1:]:
        b.fill_(FILL)
    plan = B.bcast_plan_create(P, M, 0, B.BCAST_ALGO_CHAIN)
    info = B.bcast_plan_info(plan, M, bufs)
    B.bcast_run(plan, bufs, root, M, stream)
    torch.cuda.synchronize()
    assert B.bcast_plan_status(plan)[0] == B.BCAST_OK
    plan.destroy()
    check_against_message(bufs, msg, M, root, full_ranks={1, 8, 15}, seed=4)
    oracle_prefix_check(P, root, msg, int(info["chunk_bytes"]), 32 * MiB)


def test_config4_512mib_p32():
    P, root, M = 32, 0, 512 * MiB
    msg = inputs.random_bytes(3, M)
    bufs = device_buffers(P, M, root, msg)
    plan = B.bcast_plan_create(P, M, 0, B.BCAST_ALGO_CHAIN)
    info = B.bcast_plan_info(plan, M, bufs)
    B.bcast_run(plan, bufs, root, M, torch.cuda.current_stream())
    torch.cuda.synchronize()
    assert B.bcast_plan_status(plan)[0] == B.BCAST_OK
    plan.destroy()
    check_against_message(bufs, msg, M, root, full_ranks={1, 16, 31}, seed=5)
    oracle_prefix_check(P, root, msg, int(info["chunk_bytes"]), 8 * MiB)


def test_config5_1gib_p64_root17():
    P, root, M = 64, 17, 1 * GiB
    msg = inputs.random_bytes(4, M)
    bufs = device_buffers(P, M, root, msg, slack=4096)
    for algo in (B.BCAST_ALGO_CHAIN, B.BCAST_ALGO_AUTO):
        for r in range(P):
            if r != root:
                bufs[r].fill_(FILL)
        plan = B.bcast_plan_create(P, M, 0, algo)
        info = B.bcast_plan_info(plan, M, bufs)
        B.bcast_run(plan, bufs, root, M, torch.cuda.current_stream())
        torch.cuda.synchronize()
        assert B.bcast_plan_status(plan)[0] == B.BCAST_OK
        plan.destroy()
        # chain positions 1, 32 and 63 (the last: rank root - 1) completely
        full = {(root + 1) % P, (root + 32) % P, (root + P - 1) % P}
        check_against_message(bufs, msg, M, root, full_ranks=full, seed=6)
    oracle_prefix_check(P, root, msg, int(info["chunk_bytes"]) if info["algo"] == B.BCAST_ALGO_CHAIN else 4 * MiB, 4 * MiB)


@pytest.mark.parametrize("P", [3, 6, 12, 24, 48, 63])
def test_auto_for_rank_counts_the_table_does_not_hold(P):
    """The shipped table is measured for P in {2, 4, 8, 16, 32, 64}; any other
    rank count borrows the closest one's entries, with stage counts and radices
    cut down to what P allows.  Small, medium and large messages, bit-exact."""
    from gpu_harness import run_and_check

    noise = inputs.random_bytes(11, 24 * MiB + 64)
    for M in (24, 4 * KiB, 300 * KiB + 8, 24 * MiB + 16):
        info = run_and_check(P, P // 2, M, 0, B.BCAST_ALGO_AUTO, noise)
        assert info["algo"] in (B.BCAST_ALGO_CHAIN, B.BCAST_ALGO_KNOMIAL_PIPELINED, B.BCAST_ALGO_KNOMIAL,
                                B.BCAST_ALGO_BINOMIAL, B.BCAST_ALGO_DIRECT)
        if info["algo"] == B.BCAST_ALGO_CHAIN:
            assert 1 <= info["stages"] <= P - 1
