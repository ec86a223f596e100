"""GPU parity: the HIP library, called through its C ABI, against the CPU
oracle on the same seeded inputs -- byte for byte, guard bands included.
Integer/byte work: the bar is bit-exact equality, nothing less."""
import numpy as np
import pytest
import torch

import oracle
from paper_1707_09414_amd import binding as B
from paper_1707_09414_amd import inputs
from gpu_harness import RankBuffers, run_and_check, assert_same, expected_with_oracle, oracle_schedule, FILL

pytestmark = pytest.mark.gpu

KiB, MiB = inputs.KiB, inputs.MiB
ALGOS = [B.BCAST_ALGO_CHAIN, B.BCAST_ALGO_DIRECT, B.BCAST_ALGO_BINOMIAL, B.BCAST_ALGO_FANOUT,
         B.BCAST_ALGO_SCATTER_ALLGATHER, B.BCAST_ALGO_KNOMIAL, B.BCAST_ALGO_KNOMIAL_PIPELINED]


@pytest.fixture(scope="module")
def noise():
    return inputs.random_bytes(1, 8 * MiB + 64)


def test_config1_chain_1mib_p4_c64k():
    """1 MiB of fp32 uniform[-1,1) from seed 0, P=4, root 0, 64 KiB chunks."""
    msg = inputs.uniform_fp32_message(0, 262144)
    assert msg.nbytes == MiB
    info = run_and_check(4, 0, MiB, 64 * KiB, B.BCAST_ALGO_CHAIN, msg)
    assert info["nchunks"] == 16 and info["algo"] == B.BCAST_ALGO_CHAIN
    # the oracle's schedule for this case takes chunks + P - 2 = 18 steps (Eq. 5)
    assert oracle.chain_bcast(None, 4, 0, MiB, 64 * KiB).steps == 18


@pytest.mark.parametrize("P", [2, 3, 8, 17, 64])
@pytest.mark.parametrize("M,C", [
    (1, 16), (4, 16), (12, 16), (15, 16), (16, 16), (17, 16), (33, 16), (1000, 112), (4096, 8192),
    (65536 + 3, 8192), (MiB + 17, 64 * KiB), (5 * MiB + 4096 + 5, 256 * KiB), (3 * MiB, 4 * MiB),
])
def test_chain_sizes_and_ranks(noise, P, M, C):
    run_and_check(P, (5 * P) // 7 % P, M, C, B.BCAST_ALGO_CHAIN, noise)


@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("offsets_kind", ["same4", "same1", "mixed4", "mixed1", "mixed8"])
@pytest.mark.parametrize("M", [5, 16, 4099, 300 * KiB + 7])
def test_misaligned_pointers(noise, algo, offsets_kind, M):
    P = 5
    offsets = {
        "same4": [4] * P, "same1": [1] * P, "mixed4": [0, 4, 8, 12, 20],
        "mixed1": [0, 1, 2, 3, 5], "mixed8": [0, 8, 16, 24, 40],
    }[offsets_kind]
    info = run_and_check(P, 2, M, 64 * KiB, algo, noise, offsets=offsets)
    assert info["vec_bytes"] == {"same4": 16, "same1": 16, "mixed4": 4, "mixed1": 1, "mixed8": 8}[offsets_kind]


@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("P,root,M", [(2, 1, 100), (4, 3, 70000), (7, 0, 2 * MiB + 1), (9, 4, 12345), (33, 32, 8192), (64, 17, 64 * KiB + 16)])
def test_every_algorithm_matches_its_oracle_schedule(noise, algo, P, root, M):
    run_and_check(P, root, M, 32 * KiB, algo, noise)


@pytest.mark.parametrize("lanes", [1, 2, 3, 7, 64])
def test_chain_lane_counts(noise, lanes):
    """Slices per chunk that do not divide the chunk evenly, including empty ones."""
    info = run_and_check(6, 1, 200 * KiB + 3, 16 * KiB, B.BCAST_ALGO_CHAIN, noise, lanes=lanes)
    assert info["lanes"] == lanes


@pytest.mark.parametrize("P,stages", [(2, 1), (5, 1), (5, 2), (5, 3), (8, 2), (9, 3), (10, 4), (17, 4), (33, 5), (64, 1), (64, 2), (64, 8), (64, 9),
                                      (64, 10), (64, 62), (64, 63), (64, 100)])
@pytest.mark.parametrize("M,C", [(7, 16), (70000, 8192), (3 * MiB + 5, 256 * KiB)])
def test_chain_stages(noise, P, stages, M, C):
    """A stage's wavefront plays several consecutive ranks in turn; every rank's
    buffer must still end up with the root's bytes, whatever the grouping."""
    info = run_and_check(P, P // 3, M, C, B.BCAST_ALGO_CHAIN, noise, stages=stages)
    want = min(stages, P - 1)
    assert info["stages"] == want and info["hops_per_stage"] == -(-(P - 1) // want)


@pytest.mark.parametrize("mode", [0, B.BCAST_MODE_FIXED_SPANS, B.BCAST_MODE_ROTATE_SPANS])
@pytest.mark.parametrize("P,stages", [(4, 2), (6, 2), (8, 2), (8, 3), (10, 4), (17, 3), (33, 2), (64, 2), (64, 5), (64, 40)])
def test_chain_rotating_and_fixed_spans(noise, P, stages, mode):
    """Stages of unequal length: the longer ones either stay where they are or
    move on by one stage per chunk.  Enough chunks for several full turns, a
    ragged last chunk, several trips per lane."""
    M, C = 40 * 24 * KiB + 4100, 24 * KiB
    plan = B.bcast_plan_create(P, M, C, B.BCAST_ALGO_CHAIN)
    B.bcast_plan_set_mode(plan, mode)
    info = run_and_check(P, 1, M, C, B.BCAST_ALGO_CHAIN, noise, stages=stages, lanes=2, plan=plan)
    hops = P - 1
    auto = hops % stages != 0 and hops // stages < 4
    want = {0: auto, B.BCAST_MODE_FIXED_SPANS: False, B.BCAST_MODE_ROTATE_SPANS: True}[mode]
    assert info["rotating_spans"] == int(want) and info["nchunks"] == 41
    with pytest.raises(B.BcastError):
        B.bcast_plan_set_mode(plan, B.BCAST_MODE_FIXED_SPANS | B.BCAST_MODE_ROTATE_SPANS)
    plan.destroy()


@pytest.mark.parametrize("P", [2, 3, 5, 8, 13, 64])
@pytest.mark.parametrize("M", [1, 3, 63, 64, 65, 1000, 64 * KiB + 1, 2 * MiB + 77])
def test_scatter_allgather_piece_edges(noise, P, M):
    """Pieces of ceil(M/P) bytes: short last pieces, empty pieces (M < P), odd sizes."""
    info = run_and_check(P, P - 1, M, 0, B.BCAST_ALGO_SCATTER_ALLGATHER, noise)
    rounds = (P - 1).bit_length()
    assert info["launches"] == rounds + P - 1 and info["chunk_bytes"] == -(-M // P)
    # the traffic the library accounts for equals what the oracle's schedule moves
    assert info["algorithmic_bytes"] == 2 * oracle.scatter_allgather_bcast(None, P, P - 1, M).bytes_copied


@pytest.mark.parametrize("offsets", [None, [4] * 9, [1, 0, 3, 16, 8, 2, 5, 7, 12]])
@pytest.mark.parametrize("stages,M,C", [(1, 3072, 3072), (2, 3073, 3072), (3, 70000, 6144), (8, 3 * MiB + 5, 96 * KiB),
                                        (2, 5 * MiB + 1000, 768 * KiB), (4, 100000, 1 << 20)])
def test_chain_three_kib_trips(noise, stages, M, C, offsets):
    """The 3 KiB-trip build of the chain kernel: chunk sizes that are and are
    not whole trips, ragged tails, pointers of every alignment."""
    info = run_and_check(9, 2, M, C, B.BCAST_ALGO_CHAIN, noise, stages=stages, trip=3072, offsets=offsets)
    assert info["trip_bytes"] == 3072 and info["slice_bytes"] % 3072 == 0


@pytest.mark.parametrize("policy", [None, (16, 16, 0, 16), (16, 16, 0, 0), (0, 16, 0, 16), (16, 16, 16, 16), (18, 16, 2, 16), (16, 18, 0, 18)])
@pytest.mark.parametrize("trip", [2048, 3072, 4096, 6144])
@pytest.mark.parametrize("P,stages", [(5, 4), (9, 2), (12, 3)])
@pytest.mark.parametrize("tail", [0, 5])
def test_chain_trip_paths_and_cache_policies(noise, policy, trip, P, stages, tail):
    """The chain kernel's two ways through a trip and its three policy builds.
    Chunks of two trips and three vectors: a chunk's last trip is short but made
    of whole vectors (the short way: the descriptors end with the trip); with
    `tail` the message's last trip has a ragged end (the general way).  The
    policy sets the library chooses by itself (None, and the two written out) are
    built into the kernel, every other one is read from the arguments at each
    hop; one hop per stage (first = last) and several."""
    C = 2 * trip + 48
    M = 5 * C + 16 * 7 + tail
    plan = B.bcast_plan_create(P, M, C, B.BCAST_ALGO_CHAIN)
    if policy is not None:
        B.bcast_plan_set_cache_policy(plan, *policy)
    info = run_and_check(P, 1, M, C, B.BCAST_ALGO_CHAIN, noise, stages=stages, trip=trip, lanes=2, plan=plan)
    assert info["trip_bytes"] == trip and info["stages"] == stages and info["rank_waves"] == 0
    plan.destroy()


@pytest.mark.parametrize("block", [64, 128, 256])
@pytest.mark.parametrize("P,stages,lanes,M,C", [(2, 1, 1, 5, 16), (5, 4, 3, 70001, 8192), (9, 3, 7, MiB + 3, 64 * KiB),
                                                (64, 2, 0, 3 * MiB + 5, 384 * KiB), (64, 63, 5, 100000, 4096)])
def test_chain_workgroup_sizes(noise, block, P, stages, lanes, M, C):
    """Workgroups of 1, 2 and 4 wavefronts, also where the last one is only
    partly used (odd stage x lane products)."""
    info = run_and_check(P, P - 1, M, C, B.BCAST_ALGO_CHAIN, noise, stages=stages, lanes=lanes, block=block)
    assert info["block_threads"] == block
    assert info["grid_blocks"] == -(-info["stages"] * info["lanes"] // (block // 64))


@pytest.mark.parametrize("store", [B.BCAST_STORE_THROUGH, B.BCAST_STORE_BACK])
@pytest.mark.parametrize("waves", [B.BCAST_CHAIN_WAVE_PER_STAGE, B.BCAST_CHAIN_WAVE_PER_RANK])
@pytest.mark.parametrize("P,stages,M,C", [(5, 4, 300 * KiB + 3, 16 * KiB), (8, 2, 6 * MiB + 77, 256 * KiB), (16, 3, 9 * MiB, MiB),
                                          (64, 4, 5 * MiB + 16, 0), (33, 4, 3000, 1024)])
def test_stage_store_modes(noise, store, waves, P, stages, M, C):
    """The stores that stay inside a stage written through or written back: the
    same bytes either way, at sizes on both sides of the size rule, for both
    chain kernels; the plan reports what it will use."""
    plan = B.bcast_plan_create(P, M, C, B.BCAST_ALGO_CHAIN)
    B.bcast_plan_set_stage_store(plan, store)
    info = run_and_check(P, 1, M, C, B.BCAST_ALGO_CHAIN, noise, stages=stages, waves=waves, plan=plan)
    assert info["stage_store"] == store
    B.bcast_plan_set_stage_store(plan, B.BCAST_STORE_AUTO)
    assert B.bcast_plan_info(plan, M)["stage_store"] == (B.BCAST_STORE_BACK if M <= 2 * MiB else B.BCAST_STORE_THROUGH)
    with pytest.raises(B.BcastError):
        B.bcast_plan_set_stage_store(plan, 3)
    plan.destroy()


@pytest.mark.parametrize("P,radix", [(2, 2), (5, 3), (9, 3), (10, 3), (16, 4), (17, 4), (64, 4), (64, 8), (64, 64), (33, 2), (7, 9)])
@pytest.mark.parametrize("M", [9, 4096, MiB + 3])
def test_knomial_radices(noise, P, radix, M):
    info = run_and_check(P, P // 2, M, 0, B.BCAST_ALGO_KNOMIAL, noise, radix=radix)
    assert info["stages"] == min(radix, max(2, P))


@pytest.mark.parametrize("P,radix", [(2, 2), (3, 2), (5, 3), (9, 3), (10, 3), (17, 4), (64, 2), (64, 4), (64, 8), (64, 64), (33, 5), (7, 9)])
@pytest.mark.parametrize("M,C,lanes", [(9, 16, 0), (4096, 1024, 0), (70001, 8192, 3), (MiB + 3, 64 * KiB, 0), (2 * MiB + 77, 0, 0)])
def test_pipelined_knomial_tree(noise, P, radix, M, C, lanes):
    """One launch: every position pulls each chunk from its tree parent as soon
    as the parent has published it.  Several chunks, ragged tails, odd lane
    counts, trees of depth 1 to 6."""
    info = run_and_check(P, P // 3, M, C, B.BCAST_ALGO_KNOMIAL_PIPELINED, noise, radix=radix, lanes=lanes)
    assert info["launches"] == 1 and info["stages"] == min(radix, P)
    assert info["nchunks"] == -(-M // info["chunk_bytes"])
    assert info["grid_blocks"] * 4 >= (P - 1) * info["lanes"]


def test_defaults_without_a_table(noise):
    """No tuning table: two stages, one trip per lane and chunk, 3 KiB trips for
    8 ranks and more and large messages, 4 KiB otherwise."""
    B.bcast_tune_clear()
    info = run_and_check(32, 3, 9 * MiB + 40, 0, B.BCAST_ALGO_CHAIN, noise)
    assert (info["stages"], info["trip_bytes"], info["lanes"], info["chunk_bytes"]) == (2, 3072, 1024, 3 * MiB)
    info = run_and_check(8, 3, 9 * MiB + 40, 0, B.BCAST_ALGO_CHAIN, noise)
    assert (info["stages"], info["trip_bytes"], info["lanes"], info["chunk_bytes"]) == (2, 3072, 1024, 3 * MiB)
    info = run_and_check(4, 3, 9 * MiB + 40, 0, B.BCAST_ALGO_CHAIN, noise)
    assert (info["stages"], info["trip_bytes"], info["lanes"], info["chunk_bytes"]) == (2, 4096, 1024, 4 * MiB)
    info = run_and_check(32, 3, 1 * MiB, 0, B.BCAST_ALGO_CHAIN, noise)
    assert info["trip_bytes"] == 4096
    info = run_and_check(32, 3, 9 * MiB, 2 * MiB, B.BCAST_ALGO_CHAIN, noise)
    assert (info["trip_bytes"], info["chunk_bytes"]) == (4096, 2 * MiB)


def test_degenerate_cases(noise):
    # one rank, empty message, message shorter than the plan's size
    for algo in ALGOS:
        run_and_check(1, 0, 4096, 4096, algo, noise)
        run_and_check(4, 2, 0, 4096, algo, noise, cap=4096)
        run_and_check(4, 2, 1000, 4096, algo, noise, cap=1 * MiB)


def test_argument_errors_launch_nothing(noise):
    P, M = 4, 4096
    rb = RankBuffers(P, M)
    rb.reset(0, noise[:M])
    before = rb.to_host()
    plan = B.bcast_plan_create(P, M, 1024, B.BCAST_ALGO_CHAIN)
    ptrs = rb.ptrs()
    assert B.bcast_run_status(plan, ptrs, P, M) == B.BCAST_ERR_ARG        # root out of range
    assert B.bcast_run_status(plan, ptrs, -1, M) == B.BCAST_ERR_ARG
    assert B.bcast_run_status(plan, ptrs, 0, M + 1) == B.BCAST_ERR_ARG    # longer than the plan
    assert B.bcast_run_status(plan, [ptrs[0], ptrs[1], ptrs[1], ptrs[3]], 0, M) == B.BCAST_ERR_ARG  # duplicate
    assert B.bcast_run_status(plan, [ptrs[0], 0, ptrs[2], ptrs[3]], 0, M) == B.BCAST_ERR_ARG        # NULL
    assert B.bcast_run_status(plan, [ptrs[0], ptrs[0] + 100, ptrs[2], ptrs[3]], 0, M) == B.BCAST_ERR_ARG  # overlap
    assert B.bcast_run_status(plan, None, 0, M) == B.BCAST_ERR_ARG
    assert_same(rb.to_host(), before, "after rejected calls")
    # AUTO without a table entry
    B.bcast_tune_clear()
    auto = B.bcast_plan_create(P, M, 0, B.BCAST_ALGO_AUTO)
    assert B.bcast_run_status(auto, ptrs, 0, M) == B.BCAST_ERR_UNTUNED
    assert_same(rb.to_host(), before, "after untuned AUTO")
    auto.destroy()
    plan.destroy()


def test_burst_of_small_broadcasts_reuses_flags(noise):
    """1000 back-to-back 4 KiB broadcasts at P=64, root 17, a different message
    each time and no flag reset in between: a stale flag from an earlier run
    would let a wave forward the previous message."""
    P, root, M, N = 64, 17, 4 * KiB, 1000
    msgs = inputs.random_bytes(4, N * M).reshape(N, M)
    d_msgs = torch.from_numpy(msgs).cuda()
    rb = RankBuffers(P, M)
    rb.reset(root, msgs[0])
    last = (root + P - 1) % P
    mid = (root + 31) % P
    out_last = torch.empty((N, M), dtype=torch.uint8, device="cuda")
    out_mid = torch.empty((N, M), dtype=torch.uint8, device="cuda")
    plan = B.bcast_plan_create(P, M, 8 * KiB, B.BCAST_ALGO_CHAIN)
    ptrs = rb.ptrs()
    s0 = rb.start(root)
    stream = torch.cuda.current_stream()
    for i in range(N):
        rb.raw[root][s0: s0 + M].copy_(d_msgs[i])
        B.bcast_run(plan, ptrs, root, M, stream)
        out_last[i].copy_(rb.raw[last][rb.start(last): rb.start(last) + M])
        out_mid[i].copy_(rb.raw[mid][rb.start(mid): rb.start(mid) + M])
    torch.cuda.synchronize()
    assert B.bcast_plan_status(plan)[0] == B.BCAST_OK
    assert np.array_equal(out_last.cpu().numpy(), msgs)
    assert np.array_equal(out_mid.cpu().numpy(), msgs)
    got = rb.to_host()
    for r in range(P):
        assert np.array_equal(got[r][rb.start(r): rb.start(r) + M], msgs[N - 1]), r
    plan.destroy()


def test_epoch_count_wraps_without_stale_flags(noise):
    """The flag words hold a 32-bit run count.  A plan pushed to the end of that
    range must clear its flags and start over: 12 runs across the wrap, each
    with its own message, two lanes' worth of chunks, all checked."""
    P, root, M = 9, 4, 40 * KiB + 8
    plan = B.bcast_plan_create(P, M, 8 * KiB, B.BCAST_ALGO_CHAIN)
    B.bcast_plan_set_stages(plan, 4)
    run_and_check(P, root, M, 8 * KiB, B.BCAST_ALGO_CHAIN, noise, plan=plan)
    B.bcast_plan_debug_set_epoch(plan, (1 << 32) - 8)
    with pytest.raises(B.BcastError):
        B.bcast_plan_debug_set_epoch(plan, 5)        # never backwards
    with pytest.raises(B.BcastError):
        B.bcast_plan_debug_set_epoch(plan, 1 << 32)  # beyond the range
    for i in range(12):
        run_and_check(P, (root + i) % P, M - 16 * i, 8 * KiB, B.BCAST_ALGO_CHAIN, noise[1000 * i:], plan=plan)
    # and the wait limit still works after the wrap
    assert B.bcast_plan_status(plan)[0] == B.BCAST_OK
    plan.destroy()


def test_two_plans_alternating_and_moving_root(noise):
    P, M = 8, 512 * KiB + 48
    rb = RankBuffers(P, M)
    plan_a = B.bcast_plan_create(P, M, 32 * KiB, B.BCAST_ALGO_CHAIN)
    plan_b = B.bcast_plan_create(P, M, 128 * KiB, B.BCAST_ALGO_CHAIN)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        for it in range(12):
            root = (3 * it + 1) % P
            msg = noise[it * 1000: it * 1000 + M]
            rb.reset(root, msg)
            B.bcast_run(plan_a if it % 2 == 0 else plan_b, rb.ptrs(), root, M, stream)
            stream.synchronize()
            got = rb.to_host()
            for r in range(P):
                assert np.array_equal(got[r][rb.start(r): rb.start(r) + M], msg), (it, r)
                assert (got[r][: rb.start(r)] == FILL).all() and (got[r][rb.start(r) + M:] == FILL).all()
    assert B.bcast_plan_status(plan_a)[0] == B.BCAST_OK and B.bcast_plan_status(plan_b)[0] == B.BCAST_OK
    plan_a.destroy()
    plan_b.destroy()


def test_wait_limit_reports_timeout_and_plan_recovers(noise):
    """Position 2 never publishes (debug knob) and the wait limit is tiny, so
    position 3's waves give up: the kernel must still run to completion and the
    plan must report the timeout, then work again once the knob is off."""
    P, M = 6, 256 * KiB
    rb = RankBuffers(P, M)
    rb.reset(0, noise[:M])
    plan = B.bcast_plan_create(P, M, 16 * KiB, B.BCAST_ALGO_CHAIN)
    B.bcast_plan_set_stages(plan, P - 1)     # every position has waves of its own
    B.bcast_plan_set_debug(plan, 200000, 2)  # 2 ms of the 100 MHz clock
    B.bcast_run(plan, rb.ptrs(), 0, M)
    torch.cuda.synchronize()
    st, detail = B.bcast_plan_status(plan)
    assert st == B.BCAST_ERR_TIMEOUT
    assert detail >> 32 in (3, 4, 5) and (detail & 0xFFFFFFFF) == 0, hex(detail)
    got = rb.to_host()
    # positions 1 and 2 were fed normally
    for r in (1, 2):
        assert np.array_equal(got[r][rb.start(r): rb.start(r) + M], noise[:M])
    B.bcast_plan_clear_status(plan)
    B.bcast_plan_set_debug(plan, 0, 0)
    rb.reset(0, noise[7: 7 + M])
    B.bcast_run(plan, rb.ptrs(), 0, M)
    got = rb.to_host()
    assert B.bcast_plan_status(plan)[0] == B.BCAST_OK
    for r in range(P):
        assert np.array_equal(got[r][rb.start(r): rb.start(r) + M], noise[7: 7 + M]), r
    plan.destroy()


def test_wait_limit_in_the_pipelined_tree(noise):
    """Radix-3 tree over 9 positions; position 1 never publishes, so its
    children 4 and 7 give up after the (tiny) wait limit while every other
    position is served.  All waves exit; the plan reports it and recovers."""
    P, M = 9, 200 * KiB
    rb = RankBuffers(P, M)
    rb.reset(0, noise[:M])
    plan = B.bcast_plan_create(P, M, 16 * KiB, B.BCAST_ALGO_KNOMIAL_PIPELINED)
    B.bcast_plan_set_radix(plan, 3)
    B.bcast_plan_set_debug(plan, 200000, 1)  # 2 ms of the 100 MHz clock
    B.bcast_run(plan, rb.ptrs(), 0, M)
    torch.cuda.synchronize()
    st, detail = B.bcast_plan_status(plan)
    assert st == B.BCAST_ERR_TIMEOUT
    assert detail >> 32 in (4, 7) and (detail & 0xFFFFFFFF) == 0, hex(detail)
    got = rb.to_host()
    for r in (1, 2, 3, 5, 6, 8):
        assert np.array_equal(got[r][rb.start(r): rb.start(r) + M], noise[:M]), r
    for r in (4, 7):
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


def test_tune_then_auto(noise, tmp_path):
    P = 4
    B.bcast_tune_clear()
    path = tmp_path / "tuned.txt"
    B.bcast_tune(P, 1 * KiB, 2 * MiB, 0, None, str(path))
    assert B.bcast_tune_count() == 12
    for M in (1 * KiB, 100 * KiB, 2 * MiB, 3 * MiB + 5, 17):
        algo, chunk, usec = B.bcast_tune_lookup(P, M)
        assert algo in (B.BCAST_ALGO_CHAIN, B.BCAST_ALGO_DIRECT, B.BCAST_ALGO_BINOMIAL) and usec > 0
        info = run_and_check(P, 1, M, 0, B.BCAST_ALGO_AUTO, noise)
        assert info["algo"] == algo
    B.bcast_tune_clear()
    B.bcast_tune_load(str(path))
    assert B.bcast_tune_count() == 12
    B.bcast_tune_clear()


def test_handoff_counts_and_xcd_placement(noise):
    """Every wave of positions 2..P-1 receives each chunk through one flag
    hand-off; the diagnostic counters must account for all of them."""
    P, M, C, lanes = 8, 2 * MiB, 256 * KiB, 32
    rb = RankBuffers(P, M)
    rb.reset(0, noise[:M])
    plan = B.bcast_plan_create(P, M, C, B.BCAST_ALGO_CHAIN)
    B.bcast_plan_set_lanes(plan, lanes)
    B.bcast_plan_set_stages(plan, P - 1)
    B.bcast_plan_set_mode(plan, B.BCAST_MODE_COUNT)
    B.bcast_run(plan, rb.ptrs(), 0, M)
    near, far = B.bcast_plan_handoff_counts(plan)
    assert near + far == (P - 2) * lanes * (M // C)
    B.bcast_plan_set_stages(plan, 3)  # hops 1-3 | 4-6 | 7: two flag hand-offs per lane and chunk
    B.bcast_run(plan, rb.ptrs(), 0, M)
    near2, far2 = B.bcast_plan_handoff_counts(plan)
    assert (near2 + far2) - (near + far) == 2 * lanes * (M // C)
    got = rb.to_host()
    for r in range(P):
        assert np.array_equal(got[r][rb.start(r): rb.start(r) + M], noise[:M])
    plan.destroy()


@pytest.mark.parametrize("stages", [7, 2])
def test_chunks_overlap_across_stages_on_the_device(noise, stages):
    """The point of the pipelined chain (Sec. IV-B): chunk c+1 is received while
    chunk c is forwarded.  Device timestamps of lane 0's waves must show (a)
    causality -- a stage begins chunk c only after the stage before it finished
    storing it -- and (b) overlap -- every stage begins its first chunk before
    the stage before it has finished its last."""
    P, M, C = 8, 8 * MiB, 256 * KiB
    nchunks = M // C
    rb = RankBuffers(P, M)
    rb.reset(0, noise[:M])
    plan = B.bcast_plan_create(P, M, C, B.BCAST_ALGO_CHAIN)
    B.bcast_plan_set_stages(plan, stages)
    B.bcast_plan_enable_trace(plan, stages * nchunks)
    B.bcast_run(plan, rb.ptrs(), 0, M)
    t = B.bcast_plan_read_trace(plan, stages * nchunks)
    got = rb.to_host()
    plan.destroy()
    for r in range(P):
        assert np.array_equal(got[r][rb.start(r): rb.start(r) + M], noise[:M])
    begin = [[t[g * nchunks + c][0] for c in range(nchunks)] for g in range(stages)]
    end = [[t[g * nchunks + c][1] for c in range(nchunks)] for g in range(stages)]
    for g in range(stages):
        for c in range(nchunks):
            assert 0 < begin[g][c] <= end[g][c]
            if c:
                assert end[g][c - 1] <= begin[g][c]
            if g:
                assert end[g - 1][c] <= begin[g][c], "stage %d began chunk %d before it was published" % (g, c)
        if g:
            assert begin[g][0] < end[g - 1][nchunks - 1], "stage %d did not overlap with stage %d" % (g, g - 1)
    # Eq. 5's picture: the last stage finishes its first chunk long before the first stage finishes its last
    assert end[stages - 1][0] < end[0][nchunks - 1]


@pytest.mark.parametrize("P,stages,lanes,M,C,trip", [
    (64, 63, 4, 8 * MiB + 48, 16 * KiB, 4096),      # 513 chunks through 63 flag hand-offs
    (64, 8, 32, 24 * MiB, 96 * KiB, 3072),          # 256 chunks, one 3 KiB trip per lane
    (64, 5, 0, 32 * MiB + 3, 1 * MiB, 4096),        # unequal stages (13, 13, 13, 12, 12 hops), fixed
    (7, 4, 0, 48 * MiB, 64 * KiB, 4096),            # 768 chunks, rotating spans (2, 2, 1, 1)
    (33, 32, 64, 16 * MiB, 256 * KiB, 4096),        # every position its own stage, full grid
    (16, 2, 0, 100 * MiB + 5, 3 * MiB, 3072),       # the tuned shape for large messages
])
def test_chain_many_chunks(noise, P, stages, lanes, M, C, trip):
    """Long pipelines: hundreds of chunks through many flag hand-offs with the
    device full of waiting and copying waves; every rank checked in full."""
    big = inputs.random_bytes(12, M)
    info = run_and_check(P, P - 2, M, C, B.BCAST_ALGO_CHAIN, big, stages=stages, lanes=lanes, trip=trip)
    assert info["nchunks"] == -(-M // C)


@pytest.mark.parametrize("seed", [20240607, 7, 8])
def test_random_configurations(noise, seed):
    """Seeded sweep over the whole parameter space at small sizes: ranks, root,
    message and chunk size, stage and lane counts, pointer offsets, algorithm."""
    rng = np.random.default_rng(seed)
    algos = ALGOS
    for case in range(150):
        P = int(rng.integers(1, 65)) if case % 3 else int(rng.integers(1, 9))
        root = int(rng.integers(0, P))
        M = int(rng.choice([0, 1, 7, 16, 100, 4095, 4096, 65537, 300000, int(rng.integers(1, 3 * MiB))]))
        C = int(rng.choice([0, 16, 112, 4096, 65536, 1 << 20])) if rng.random() < 0.8 else 16 * int(rng.integers(1, 70000))
        algo = int(algos[int(rng.integers(0, len(algos)))])
        stages = int(rng.integers(0, 70)) if algo == B.BCAST_ALGO_CHAIN else 0
        lanes = int(rng.choice([0, 0, 1, 3, 32, 100]))
        kind = int(rng.integers(0, 4))
        offsets = [[0] * P, [int(rng.integers(0, 16))] * P, [int(x) for x in rng.integers(0, 4, P) * 4],
                   [int(x) for x in rng.integers(0, 33, P)]][kind]
        radix = int(rng.integers(2, 10)) if algo in (B.BCAST_ALGO_KNOMIAL, B.BCAST_ALGO_KNOMIAL_PIPELINED) else 0
        trip = int(rng.choice([0, 3072, 4096])) if algo == B.BCAST_ALGO_CHAIN else 0
        block = int(rng.choice([0, 64, 128, 256])) if algo == B.BCAST_ALGO_CHAIN else 0
        try:
            run_and_check(P, root, M, C, algo, noise, offsets=offsets, lanes=lanes, stages=stages, radix=radix, trip=trip, block=block)
        except Exception as e:
            raise AssertionError("case %d: P=%d root=%d M=%d C=%d algo=%d stages=%d lanes=%d offsets=%s radix=%d trip=%d: %s"
                                 % (case, P, root, M, C, algo, stages, lanes, kind, radix, trip, e))


def test_two_plans_on_two_streams_at_once(noise):
    """Different plans (own flags) with different buffers may run concurrently:
    two persistent kernels share the device without starving each other."""
    P, M = 16, 6 * MiB + 40
    rb1, rb2 = RankBuffers(P, M), RankBuffers(P, M)
    m1, m2 = noise[:M], noise[1234: 1234 + M]
    rb1.reset(3, m1)
    rb2.reset(9, m2)
    torch.cuda.synchronize()
    p1 = B.bcast_plan_create(P, M, 512 * KiB, B.BCAST_ALGO_CHAIN)
    p2 = B.bcast_plan_create(P, M, 256 * KiB, B.BCAST_ALGO_CHAIN)
    B.bcast_plan_set_stages(p1, 15)
    B.bcast_plan_set_stages(p2, 3)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    for _ in range(20):
        B.bcast_run(p1, rb1.ptrs(), 3, M, s1)
        B.bcast_run(p2, rb2.ptrs(), 9, M, s2)
    s1.synchronize()
    s2.synchronize()
    assert B.bcast_plan_status(p1)[0] == B.BCAST_OK and B.bcast_plan_status(p2)[0] == B.BCAST_OK
    g1, g2 = rb1.to_host(), rb2.to_host()
    for r in range(P):
        assert np.array_equal(g1[r][rb1.start(r): rb1.start(r) + M], m1), r
        assert np.array_equal(g2[r][rb2.start(r): rb2.start(r) + M], m2), r
    p1.destroy()
    p2.destroy()


def test_tune_with_every_candidate(noise, tmp_path):
    """The tuner with the optional candidates switched on (single-stage chain,
    fan-out, scatter + allgather, k-nomial) still yields runnable entries."""
    P = 8
    B.bcast_tune_clear()
    mask = sum(1 << a for a in ALGOS) | B.BCAST_TUNE_FOLDED
    log = tmp_path / "log.txt"
    B.bcast_tune_set_log(str(log))
    B.bcast_tune(P, 64 * KiB, 1 * MiB, mask, None, None)
    B.bcast_tune_set_log(None)
    assert B.bcast_tune_count() == 5
    seen_algos = set()
    for line in log.read_text().splitlines():
        if not line.startswith("#"):
            seen_algos.add(int(line.split()[2]))
    assert seen_algos == set(ALGOS)
    for M in (64 * KiB, 300 * KiB, 1 * MiB):
        e = B.bcast_tune_get(P, M)
        assert e["usec"] > 0 and e["chain_usec"] > 0 and e["chain_chunk_bytes"] > 0
        run_and_check(P, 5, M, 0, B.BCAST_ALGO_AUTO, noise)
        run_and_check(P, 5, M, 0, B.BCAST_ALGO_CHAIN, noise)
    B.bcast_tune_clear()
