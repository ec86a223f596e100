"""The five benchmark configurations at their full sizes, on the GPU, through
the C ABI, in the launch configuration bench.py uses (tuned table installed).

A broadcast is exact data movement, so the oracle's end state for every rank is
the root's message.  Where P*M fits comfortably in host memory the oracle's
payload simulation is run at full size and compared row by row; for the two
largest configurations the oracle runs its schedule at full scale (step count)
and its payload simulation at full P on a prefix of the message, and the GPU
buffers are compared with the message itself: three ranks completely, every
other rank on seeded 1 MiB windows copied back to the host, plus a device-side
whole-buffer comparison.  Every rank buffer sits between two 256-byte guard
bands of 0xFF that are compared after every run."""
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


GUARD = 256  # bytes of 0xFF kept before and after every rank buffer, compared after every run


def device_buffers(P, M, root, msg):
    """P allocations of GUARD + M + GUARD bytes of 0xFF; rank r's buffer is the
    middle M bytes.  Returns (rank buffers, whole allocations)."""
    raws = [torch.full((GUARD + M + GUARD,), FILL, dtype=torch.uint8, device="cuda") for _ in range(P)]
    bufs = [t[GUARD: GUARD + M] for t in raws]
    bufs[root].copy_(torch.from_numpy(msg))
    return bufs, raws


def check_against_message(bufs, raws, msg, M, root, full_ranks, windows=64, seed=0):
    d_msg = torch.from_numpy(msg).cuda()
    rng = np.random.default_rng(seed)
    for r, t in enumerate(bufs):
        assert torch.equal(t, d_msg), "rank %d differs from the message (device compare)" % r
        assert bool((raws[r][:GUARD] == FILL).all()), "rank %d: bytes before the buffer were written" % r
        assert bool((raws[r][GUARD + M:] == FILL).all()), "rank %d: bytes beyond the message were written" % r
        if r in full_ranks:
            assert np.array_equal(t.cpu().numpy(), msg), "rank %d differs from the message" % r
        else:
            starts = [0, max(0, M - MiB)] + [int(x) for x in rng.integers(0, max(1, M - MiB), size=windows)]
            for s in starts:
                e = min(M, s + MiB)
                assert np.array_equal(t[s:e].cpu().numpy(), msg[s:e]), "rank %d differs in [%d, %d)" % (r, s, e)


def refill(bufs, root):
    for r, b in enumerate(bufs):
        if r != root:
            b.fill_(FILL)


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
    """4 B .. 64 MiB in powers of two, P=8, root 0: chain (tuned, and one swept
    chunk with a wavefront per stage and per rank), direct, binomial and AUTO
    against the oracle's full simulation."""
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
        for algo, C, waves in [(B.BCAST_ALGO_CHAIN, 0, 0), (B.BCAST_ALGO_CHAIN, swept, B.BCAST_CHAIN_WAVE_PER_STAGE),
                               (B.BCAST_ALGO_CHAIN, swept, B.BCAST_CHAIN_WAVE_PER_RANK), (B.BCAST_ALGO_DIRECT, 0, 0),
                               (B.BCAST_ALGO_BINOMIAL, 0, 0), (B.BCAST_ALGO_AUTO, 0, 0)]:
            bufs, raws = device_buffers(P, M, root, msg)
            plan = B.bcast_plan_create(P, M, C, algo)
            if waves:
                B.bcast_plan_set_chain_waves(plan, waves)
            B.bcast_run(plan, bufs, root, M, stream)
            torch.cuda.synchronize()
            assert B.bcast_plan_status(plan)[0] == B.BCAST_OK
            plan.destroy()
            for r in range(P):
                got = raws[r].cpu().numpy()
                assert np.array_equal(got[GUARD: GUARD + M], want[r]), (M, algo, C, waves, r)
                assert (got[:GUARD] == FILL).all() and (got[GUARD + M:] == FILL).all(), (M, algo, C, waves, r)
            del bufs, raws


def test_config3_vgg16_per_tensor_and_packed_p16():
    """138M fp32 VGG-16 parameters, N(0, 0.01), seed 2, P=16, root 0: one
    broadcast per tensor (32 runs, AUTO from the tuning table) and one packed."""
    P, root = 16, 0
    msg, spans = inputs.vgg16_packed_message(2)
    M = msg.nbytes
    assert M == 553430176 and len(spans) == 32
    stream = torch.cuda.current_stream()

    # tensor by tensor, each tensor in its own set of P buffers carved out of one allocation per rank
    bufs, raws = device_buffers(P, M, root, msg)
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
    check_against_message(bufs, raws, msg, M, root, full_ranks={1, 8, 15}, seed=3)

    # packed into one buffer: the tuned chain, and the chain with a wavefront per stage and per rank
    for waves in (B.BCAST_CHAIN_AUTO, B.BCAST_CHAIN_WAVE_PER_STAGE, B.BCAST_CHAIN_WAVE_PER_RANK):
        refill(bufs, root)
        plan = B.bcast_plan_create(P, M, 0, B.BCAST_ALGO_CHAIN)
        B.bcast_plan_set_chain_waves(plan, waves)
        info = B.bcast_plan_info(plan, M, bufs)
        B.bcast_run(plan, bufs, root, M, stream)
        torch.cuda.synchronize()
        assert B.bcast_plan_status(plan)[0] == B.BCAST_OK
        plan.destroy()
        check_against_message(bufs, raws, msg, M, root, full_ranks={1, 8, 15} if waves == B.BCAST_CHAIN_AUTO else {15}, seed=4 + waves)
    oracle_prefix_check(P, root, msg, int(info["chunk_bytes"]), 32 * MiB)


def test_config4_512mib_p32():
    P, root, M = 32, 0, 512 * MiB
    msg = inputs.random_bytes(3, M)
    bufs, raws = device_buffers(P, M, root, msg)
    for waves in (B.BCAST_CHAIN_AUTO, B.BCAST_CHAIN_WAVE_PER_STAGE, B.BCAST_CHAIN_WAVE_PER_RANK):
        refill(bufs, root)
        plan = B.bcast_plan_create(P, M, 0, B.BCAST_ALGO_CHAIN)
        B.bcast_plan_set_chain_waves(plan, waves)
        info = B.bcast_plan_info(plan, M, bufs)
        B.bcast_run(plan, bufs, root, M, torch.cuda.current_stream())
        torch.cuda.synchronize()
        assert B.bcast_plan_status(plan)[0] == B.BCAST_OK
        plan.destroy()
        check_against_message(bufs, raws, msg, M, root, full_ranks={1, 16, 31} if waves == B.BCAST_CHAIN_AUTO else {31}, seed=5 + waves)
        oracle_prefix_check(P, root, msg, int(info["chunk_bytes"]), 8 * MiB)


def test_config5_1gib_p64_root17():
    P, root, M = 64, 17, 1 * GiB
    msg = inputs.random_bytes(4, M)
    bufs, raws = device_buffers(P, M, root, msg)
    for algo, waves in ((B.BCAST_ALGO_CHAIN, B.BCAST_CHAIN_AUTO), (B.BCAST_ALGO_CHAIN, B.BCAST_CHAIN_WAVE_PER_RANK), (B.BCAST_ALGO_AUTO, B.BCAST_CHAIN_AUTO)):
        refill(bufs, root)
        plan = B.bcast_plan_create(P, M, 0, algo)
        B.bcast_plan_set_chain_waves(plan, waves)
        info = B.bcast_plan_info(plan, M, bufs)
        B.bcast_run(plan, bufs, root, M, torch.cuda.current_stream())
        torch.cuda.synchronize()
        assert B.bcast_plan_status(plan)[0] == B.BCAST_OK
        plan.destroy()
        # chain positions 1, 32 and 63 (the last: rank root - 1) completely
        full = {(root + 1) % P, (root + 32) % P, (root + P - 1) % P} if waves == B.BCAST_CHAIN_AUTO and algo == B.BCAST_ALGO_CHAIN else {(root + P - 1) % P}
        check_against_message(bufs, raws, msg, M, root, full_ranks=full, seed=6 + waves + algo)
    oracle_prefix_check(P, root, msg, int(info["chunk_bytes"]) if info["algo"] == B.BCAST_ALGO_CHAIN else 4 * MiB, 4 * MiB)


@pytest.mark.parametrize("algo", [B.BCAST_ALGO_AUTO, B.BCAST_ALGO_CHAIN])
def test_config5_burst_of_1000_small_broadcasts(algo):
    """1000 back-to-back 4 KiB broadcasts at P=64, root 17, with the shipped
    table (AUTO: the pipelined tree; CHAIN: the tuned chain), a distinct message
    in every run and no flag reset in between: chain positions 1, 32 and 63 are
    captured after every run, so a stale flag that let a wave forward an earlier
    run's bytes would show."""
    P, root, M, N = 64, 17, 4 * KiB, 1000
    msgs = inputs.random_bytes(4, N * M).reshape(N, M)
    d_msgs = torch.from_numpy(msgs).cuda()
    bufs, raws = device_buffers(P, M, root, msgs[0])
    watch = [(root + k) % P for k in (1, 32, 63)]
    outs = [torch.empty((N, M), dtype=torch.uint8, device="cuda") for _ in watch]
    plan = B.bcast_plan_create(P, M, 0, algo)
    info = B.bcast_plan_info(plan, M, bufs)
    assert info["algo"] == (B.bcast_tune_lookup(P, M)[0] if algo == B.BCAST_ALGO_AUTO else B.BCAST_ALGO_CHAIN)
    ptrs = B.RankPointers(bufs)
    stream = torch.cuda.current_stream()
    for i in range(N):
        bufs[root].copy_(d_msgs[i])
        B.bcast_run(plan, ptrs, root, M, stream)
        for o, r in zip(outs, watch):
            o[i].copy_(bufs[r])
    torch.cuda.synchronize()
    assert B.bcast_plan_status(plan)[0] == B.BCAST_OK
    plan.destroy()
    for o, r in zip(outs, watch):
        assert np.array_equal(o.cpu().numpy(), msgs), "rank %d saw a stale or wrong message in some run" % r
    for r in range(P):
        got = raws[r].cpu().numpy()
        assert np.array_equal(got[GUARD: GUARD + M], msgs[N - 1]), r
        assert (got[:GUARD] == FILL).all() and (got[GUARD + M:] == FILL).all(), r


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
