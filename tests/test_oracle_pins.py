"""Pins for the CPU oracle: everything here checks the oracle against facts
that do not come from the oracle itself -- numpy row replication for the end
state (the definition of a broadcast), the paper's closed-form step counts
(Sec. III-A Eq. 1-4, Sec. IV-B Eq. 5), hand-worked fixtures under
tests/golden/, and schedule invariants derived from the text of Sec. IV-B.

The last test plants mistakes in copies of the oracle's source and checks that
this battery of pins rejects each of them.
"""
import math
import os
import subprocess

import numpy as np
import pytest

import oracle
from paper_1707_09414_amd import inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
FILL = inputs.FILL_BYTE


def make_bufs(P, root, M, cap, seed=0):
    """Root row holds a random message, every other byte anywhere is FILL."""
    rng = np.random.default_rng(seed + 1000 * P + 7 * root + 13 * M)
    bufs = np.full((P, cap), FILL, dtype=np.uint8)
    # avoid FILL in the message so an un-copied byte can never look copied
    bufs[root, :M] = rng.integers(0, 255, size=M, dtype=np.uint8)
    return bufs


def expected_end_state(before, root, M):
    """The definition: every row's first M bytes equal the root's; rest untouched."""
    exp = before.copy()
    exp[:, :M] = before[root, :M][None, :]
    return exp


def closed_form_chain_steps(P, M, C):
    """Eq. 5's step count (chunks + n - 2); zero work for P < 2 or M == 0."""
    if P < 2 or M == 0:
        return 0
    return -(-M // C) + P - 2


# ----------------------------------------------------------------------------
# individual pins, each written as a function returning None or raising
# AssertionError, so the mutant test below can run the same battery.
# ----------------------------------------------------------------------------

def pin_chain_brute_force(maxP=9, maxM=40):
    for P in range(1, maxP + 1):
        for root in range(P):
            for M in range(0, maxM + 1):
                before = make_bufs(P, root, M, 2 * maxM + 8)
                exp = expected_end_state(before, root, M)
                for C in range(1, M + 3):
                    bufs = before.copy()
                    res = oracle.chain_bcast(bufs, P, root, M, C)
                    assert np.array_equal(bufs, exp), (P, root, M, C)
                    assert res.steps == closed_form_chain_steps(P, M, C), (P, root, M, C, res.steps)
                    assert res.bytes_copied == (P - 1) * M, (P, root, M, C)


def pin_chain_schedule_invariants():
    for P in range(2, 8):
        for root in (0, P // 2, P - 1):
            for M in (1, 9, 24, 25):
                for C in (1, 4, 5, 24, 30):
                    nchunks = -(-M // C)
                    bufs = make_bufs(P, root, M, M + 40)
                    res = oracle.chain_bcast(bufs, P, root, M, C, trace=True)
                    S = res.steps
                    assert res.have.shape == (S, P)
                    # chunks held by position k after step s (0-based): the chunk front
                    # moves one hop per step starting from the root
                    for s in range(S):
                        for k in range(1, P):
                            assert res.have[s, k] == min(nchunks, max(0, s - k + 2)), (P, M, C, s, k)
                        assert res.have[s, 0] == nchunks
                    # every (position, chunk) is delivered exactly once, by the left
                    # neighbour, in step chunk + position - 1, over the chunk's byte range
                    seen = set()
                    per_step_links = {}
                    for t in res.transfers:
                        k = (t.dst_rank - root) % P
                        assert 1 <= k <= P - 1
                        assert t.src_rank == (root + k - 1) % P, "must come from the left neighbour"
                        assert t.dst_rank != root, "root only sends"
                        assert t.step == t.chunk + k - 1
                        assert t.lo == t.chunk * C and t.hi == min(M, (t.chunk + 1) * C)
                        assert (k, t.chunk) not in seen
                        seen.add((k, t.chunk))
                        assert (t.step, k) not in per_step_links, "one chunk per link per step"
                        per_step_links[(t.step, k)] = 1
                    assert len(seen) == nchunks * (P - 1)
                    # the last position never sends (no wrap-around)
                    last_rank = (root + P - 1) % P
                    assert all(t.src_rank != last_rank for t in res.transfers)


def pin_chain_forwarding_is_from_neighbour_payload():
    """If the schedule copied from the root instead of from the left neighbour, or
    forwarded a chunk before it was stored, the bytes would still match; the
    transfer log above catches the first.  This catches the second: a transfer
    may only read a chunk that an earlier step wrote (or that the root owns)."""
    P, root, M, C = 6, 2, 50, 7
    res = oracle.chain_bcast(make_bufs(P, root, M, M), P, root, M, C, trace=True)
    arrived = {}
    for t in res.transfers:
        arrived[(t.dst_rank, t.chunk)] = t.step
    for t in res.transfers:
        if t.src_rank != root:
            assert arrived[(t.src_rank, t.chunk)] < t.step


def pin_golden_counts():
    with open(os.path.join(GOLDEN, "schedule_counts.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    assert len(rows) >= 24
    for kind, n, M, C, want in rows:
        n, M, C, want = int(n), int(M), int(C), int(want)
        if kind == "chain":
            got = oracle.chain_bcast(None, n, 0, M, C).steps
        elif kind == "binomial":
            got = oracle.binomial_bcast(None, n, 0, M).steps
        elif kind == "direct":
            got = oracle.direct_bcast(None, n, 0, M).steps
        elif kind == "scatter_allgather":
            got = oracle.scatter_allgather_bcast(None, n, 0, M).steps
        elif kind.startswith("knomialpipe"):
            got = oracle.knomial_pipeline_bcast(None, n, 0, M, C, int(kind[len("knomialpipe"):])).steps
        elif kind.startswith("knomial"):
            got = oracle.knomial_bcast(None, n, 0, M, int(kind[len("knomial"):])).steps
        else:
            raise AssertionError(kind)
        assert got == want, (kind, n, M, C, got, want)


def pin_variants_end_state_and_counts(maxP=9):
    for P in range(1, maxP + 1):
        for root in range(P):
            for M in (0, 1, 5, 16, 23):
                before = make_bufs(P, root, M, M + 5)
                exp = expected_end_state(before, root, M)

                b = before.copy()
                r = oracle.direct_bcast(b, P, root, M, trace=True)
                assert np.array_equal(b, exp)
                assert r.steps == P - 1 and r.bytes_copied == (P - 1) * M
                assert all(t.src_rank == root for t in r.transfers)
                assert sorted(t.dst_rank for t in r.transfers) == [x for x in range(P) if x != root]

                b = before.copy()
                r = oracle.binomial_bcast(b, P, root, M, trace=True)
                assert np.array_equal(b, exp)
                assert r.steps == (math.ceil(math.log2(P)) if P > 1 else 0)
                assert r.bytes_copied == (P - 1) * M
                got_from = {}
                for t in r.transfers:
                    k = (t.dst_rank - root) % P
                    assert k not in got_from and k != 0
                    got_from[k] = ((t.src_rank - root) % P, t.step)
                for k in range(1, P):
                    j = k.bit_length() - 1  # floor(log2 k): the round in which k is reached
                    assert got_from[k] == (k - (1 << j), j), (P, k, got_from[k])

                for k in (2, 3, 4, 8):
                    b = before.copy()
                    r = oracle.knomial_bcast(b, P, root, M, k, trace=True)
                    assert np.array_equal(b, exp), (P, root, M, k)
                    rounds, reach = 0, 1
                    while reach < P:
                        reach *= k
                        rounds += 1
                    assert r.steps == rounds and r.bytes_copied == (P - 1) * M
                    got_from = {}
                    for t in r.transfers:
                        q = (t.dst_rank - root) % P
                        assert q not in got_from and q != 0
                        got_from[q] = ((t.src_rank - root) % P, t.step)
                    for q in range(1, P):
                        j, top = 0, 1  # top = k^j with k^j <= q < k^(j+1)
                        while top * k <= q:
                            top *= k
                            j += 1
                        # the parent is q without its leading base-k digit; reached in round j
                        assert got_from[q] == (q % top, j), (P, k, q, got_from[q])

                for k, C in ((2, 1), (3, 4), (4, 5), (3, M + 3)):
                    b = before.copy()
                    r = oracle.knomial_pipeline_bcast(b, P, root, M, C, k, trace=True)
                    assert np.array_equal(b, exp), (P, root, M, k, C)
                    levels, reach = 0, 1
                    while reach < P:
                        reach *= k
                        levels += 1
                    nchunks = -(-M // C)
                    assert r.steps == (nchunks * levels if P > 1 else 0), (P, M, C, k, r.steps)
                    assert r.bytes_copied == (P - 1) * M
                    seen = {}
                    for t in r.transfers:
                        q = (t.dst_rank - root) % P
                        assert (q, t.chunk) not in seen and q != 0
                        assert (t.lo, t.hi) == (t.chunk * C, min(M, (t.chunk + 1) * C))
                        seen[(q, t.chunk)] = ((t.src_rank - root) % P, t.step)
                    for q in range(1, P):
                        j, top = 0, 1
                        while top * k <= q:
                            top *= k
                            j += 1
                        for c in range(nchunks):
                            # parent as in the k-nomial tree; level j starts after j whole messages
                            assert seen[(q, c)] == (q % top, j * nchunks + c), (P, k, q, c, seen[(q, c)])
                    if C >= M and P > 1 and M > 0:
                        plain = oracle.knomial_bcast(before.copy(), P, root, M, k, trace=True)
                        assert [(t.src_rank, t.dst_rank) for t in plain.transfers] == [(t.src_rank, t.dst_rank) for t in r.transfers]

                b = before.copy()
                r = oracle.scatter_allgather_bcast(b, P, root, M, trace=True)
                assert np.array_equal(b, exp), (P, root, M)
                if P > 1:
                    assert r.scatter_rounds == math.ceil(math.log2(P))
                    assert r.ring_steps == P - 1
                    assert r.steps == r.scatter_rounds + r.ring_steps
                    piece = -(-M // P)
                    plen = [max(0, min(M, (q + 1) * piece) - min(M, q * piece)) for q in range(P)]
                    assert sum(plen) == M
                    # the root hands out every piece but its own exactly once during the scatter
                    sent_by_root = sum(t.hi - t.lo for t in r.transfers if t.step < r.scatter_rounds and t.src_rank == root)
                    assert sent_by_root == M - plen[0]
                    # in the ring every non-root position receives every piece but its own
                    for k in range(1, P):
                        rk = (root + k) % P
                        got = sum(t.hi - t.lo for t in r.transfers if t.step >= r.scatter_rounds and t.dst_rank == rk)
                        assert got == M - plen[k], (P, root, M, k)
                    assert all(t.dst_rank != root for t in r.transfers)

                b = before.copy()
                oracle.naive_bcast(b, root, M)
                assert np.array_equal(b, exp)


def pin_reduce_golden():
    with open(os.path.join(GOLDEN, "reduce_order.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    assert len(rows) == 9
    for row in rows:
        P, root = int(row[0]), int(row[1])
        vals = np.array([[float(v)] for v in row[2:2 + P]], dtype=np.float32)
        want = np.float32(float(row[2 + P]))
        got, _ = oracle.chain_reduce_f32(vals, P, root, 1, 1)
        assert got[0] == want, (row, got)
        # the same values in every element of a longer, chunked message
        wide = np.repeat(vals, 11, axis=1).copy()
        got, _ = oracle.chain_reduce_f32(wide, P, root, 11, 4)
        assert (got == want).all(), (row, got)


def pin_reduce_exact_integers_and_schedule(maxP=7, maxN=13):
    """Small integers sum exactly in fp32 whatever the order, so the result is
    fixed by integer arithmetic; the schedule is the chain's, run backwards."""
    rng = np.random.default_rng(5)
    for P in range(1, maxP + 1):
        for root in range(P):
            for count in range(0, maxN + 1):
                ints = rng.integers(-1000, 1001, size=(P, count))
                send = ints.astype(np.float32)
                for C in sorted({1, 2, 5, max(1, count), count + 2}):
                    keep = send.copy()
                    got, res = oracle.chain_reduce_f32(send, P, root, count, C, trace=True)
                    assert np.array_equal(send, keep), "contributions are inputs only"
                    assert np.array_equal(got.astype(np.int64), ints.sum(axis=0)), (P, root, count, C)
                    nchunks = -(-count // C)
                    if P < 2 or count == 0:
                        assert res.steps == 0 and not res.transfers
                        continue
                    assert res.steps == nchunks + P - 2
                    assert res.bytes_copied == (P - 1) * count * 4
                    seen = {}
                    for t in res.transfers:
                        k = (t.dst_rank - root) % P
                        assert (t.src_rank - root) % P == k + 1, "a partial comes from the right neighbour"
                        assert (k, t.chunk) not in seen
                        assert (t.lo, t.hi) == (4 * t.chunk * C, 4 * min(count, (t.chunk + 1) * C))
                        seen[(k, t.chunk)] = t.step
                    for k in range(P - 1):
                        for c in range(nchunks):
                            assert seen[(k, c)] == (P - 2 - k) + c, (P, k, c, seen[(k, c)])
    with pytest.raises(ValueError):
        oracle.chain_reduce_f32(np.zeros((2, 4), np.float32), 2, 2, 4, 2)
    with pytest.raises(ValueError):
        oracle.chain_reduce_f32(np.zeros((2, 4), np.float32), 2, 0, 4, 0)
    assert oracle.chain_reduce_f32(None, 64, 17, 1 << 28, 1 << 20)[1].steps == 256 + 62


def pin_reduce_rounding_bound():
    """Against the exact sum (float64 is exact enough here): the error of P - 1
    fp32 additions is at most (P - 1) u sum|x| with u = 2^-24, and it is not zero
    -- a sum carried in higher precision and rounded once would be closer."""
    rng = np.random.default_rng(6)
    for P in (2, 3, 8, 16, 64):
        send = rng.normal(0.0, 0.01, size=(P, 5000)).astype(np.float32)
        got, _ = oracle.chain_reduce_f32(send, P, P // 2, 5000, 777)
        exact = send.astype(np.float64).sum(axis=0)
        bound = (P - 1) * 2.0 ** -24 * np.abs(send.astype(np.float64)).sum(axis=0)
        err = np.abs(got.astype(np.float64) - exact)
        assert (err <= bound).all()
        if P >= 8:
            once = exact.astype(np.float32)
            assert (got != once).mean() > 0.05, "P - 1 roundings must show"


def pin_cost_models():
    with open(os.path.join(GOLDEN, "cost_models.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    assert len(rows) == 7
    for kind, n, k, M, C, ts, B, want in rows:
        n, k = int(n), int(k)
        M, C, ts, B, want = float(M), float(C), float(ts), float(B), float(want)
        got = {
            "direct": lambda: oracle.model_direct(n, M, ts, B),
            "chain": lambda: oracle.model_chain(n, M, ts, B),
            "knomial": lambda: oracle.model_knomial(n, k, M, ts, B),
            "scatter_allgather": lambda: oracle.model_scatter_allgather(n, M, ts, B),
            "chain_pipeline": lambda: oracle.model_chain_pipeline(n, M, C, ts, B),
            "knomial_pipeline": lambda: oracle.model_knomial_pipeline(n, k, M, C, ts, B),
        }[kind]()
        assert got == pytest.approx(want, rel=1e-12), (kind, got, want)
    # identities between the printed formulas
    for n in (2, 3, 8, 64):
        M, ts, B = 3.0e6, 2.5e-6, 4.0e9
        unit = ts + M / B
        assert oracle.model_chain_pipeline(n, M, M, ts, B) == pytest.approx(oracle.model_chain(n, M, ts, B), rel=1e-14)
        assert oracle.model_direct(n, M, ts, B) - oracle.model_chain(n, M, ts, B) == pytest.approx(unit, rel=1e-12)
        assert oracle.model_knomial(n, n, M, ts, B) == pytest.approx(unit, rel=1e-14)
        for k in (2, 4):
            # one chunk: the unpipelined tree; chunking only adds start-ups
            assert oracle.model_knomial_pipeline(n, k, M, M, ts, B) == pytest.approx(oracle.model_knomial(n, k, M, ts, B), rel=1e-14)
            extra = oracle.model_knomial_pipeline(n, k, M, M / 8, ts, B) - oracle.model_knomial(n, k, M, ts, B)
            assert extra == pytest.approx(7 * ts * oracle.model_knomial(n, k, M, ts, B) / unit, rel=1e-9)
    assert oracle.model_scatter_allgather(2, 1e6, 1e-6, 1e9) == pytest.approx(2e-6 + 1e-3, rel=1e-14)


BATTERY = [
    pin_chain_brute_force,
    pin_chain_schedule_invariants,
    pin_chain_forwarding_is_from_neighbour_payload,
    pin_golden_counts,
    pin_variants_end_state_and_counts,
    pin_cost_models,
    pin_reduce_golden,
    pin_reduce_exact_integers_and_schedule,
    pin_reduce_rounding_bound,
]


@pytest.mark.parametrize("pin", BATTERY, ids=lambda f: f.__name__)
def test_pin(pin):
    pin()


def test_bad_arguments_are_rejected():
    b = np.zeros((3, 8), np.uint8)
    with pytest.raises(ValueError):
        oracle.chain_bcast(b, 3, 3, 8, 4)
    with pytest.raises(ValueError):
        oracle.chain_bcast(b, 3, -1, 8, 4)
    with pytest.raises(ValueError):
        oracle.chain_bcast(b, 3, 0, 8, 0)
    with pytest.raises(ValueError):
        oracle.chain_bcast(b, 3, 0, 9, 4)  # message longer than the rows


def test_schedule_only_matches_payload_mode_and_scales():
    """bufs=None must walk the identical schedule (used where P*M exceeds host RAM)."""
    for P, M, C in [(4, 100, 7), (7, 64, 64), (9, 1, 1)]:
        a = oracle.chain_bcast(make_bufs(P, 0, M, M), P, 0, M, C, trace=True)
        b = oracle.chain_bcast(None, P, 0, M, C, trace=True)
        assert a.steps == b.steps and a.transfers == b.transfers and a.bytes_copied == b.bytes_copied
    # full-scale schedule of the 64-rank, 1 GiB case: no payload touched
    res = oracle.chain_bcast(None, 64, 17, 1 << 30, 1 << 20)
    assert res.steps == 1024 + 62 and res.bytes_copied == 63 * (1 << 30)


def test_vgg16_input_recipe():
    sizes = inputs.vgg16_tensor_bytes()
    assert len(sizes) == 32
    assert sum(sizes) == 553430176 and sum(sizes) // 4 == 138357544
    assert min(sizes) == 256 and max(sizes) == 411041792
    assert all(s % 16 == 0 for s in sizes)


# ----------------------------------------------------------------------------
# Planted mistakes: each edit below is a plausible slip in the oracle's source.
# The battery above must reject every one of them.
# ----------------------------------------------------------------------------
MUTANTS = [
    ("no_snapshot", "seen[k - 1] > c", "have[k - 1] > c"),
    ("copy_from_root", "transfer(bufs, tr, steps, rank_at(root, k - 1, P), rank_at(root, k, P), c, lo, hi);",
     "transfer(bufs, tr, steps, root, rank_at(root, k, P), c, lo, hi);"),
    ("tail_overrun", "size_t hi = lo + C < M ? lo + C : M;", "size_t hi = lo + C;"),
    ("dropped_tail_chunk", "(long)(M / C) + (M % C ? 1 : 0)", "(long)(M / C)"),
    ("wrong_chain_direction", "static int rank_at(int root, int k, int P) { return (root + k) % P; }",
     "static int rank_at(int root, int k, int P) { return ((root - k) % P + P) % P; }"),
    ("wrong_chunk_offset", "size_t lo = (size_t)c * C;", "size_t lo = (size_t)(c + 1) * C;"),
    ("binomial_wrong_child", "long child = q + reach;", "long child = q + reach + 1;"),
    ("binomial_linear_rounds", "for (long reach = 1; reach < P; reach *= 2) {", "for (long reach = 1; reach < P; reach += 1) {"),
    ("knomial_skips_last_child", "for (long i = 1; i < k; i++) {", "for (long i = 1; i < k - 1; i++) {"),
    ("knomial_wrong_stride", "long child = q + i * reach;", "long child = q + i * (reach + 1);"),
    ("knomial_reach_doubles", "for (long reach = 1; reach < P; reach *= k) {", "for (long reach = 1; reach < P; reach *= 2) {"),
    ("pipe_wrong_target", "long target = holder + d * span;", "long target = holder + d * span + 1;"),
    ("pipe_levels_double", "for (long span = 1; span < P; span *= k) {", "for (long span = 1; span < P; span *= 2) {"),
    ("pipe_drops_tail_chunk", "if (M % C) pieces++;", "if (M % C > 1) pieces++;"),
    ("pipe_chunk_overrun", "size_t to = from + C < M ? from + C : M;", "size_t to = from + C;"),
    ("pipe_step_per_level", "            steps++;\n        }\n    }\n    return steps;", "        }\n        steps++;\n    }\n    return steps;"),
    ("model_pipe_levels", "return (M / C * ceil_log(n, k)) * (ts + C / B);", "return (M / C + ceil_log(n, k)) * (ts + C / B);"),
    ("reduce_drops_own_term", "out[i] = mine[i] + in[i];", "out[i] = in[i];"),
    ("reduce_from_the_roots_end", "const float *mine = send[rank_at(root, k, P)];", "const float *mine = send[rank_at(root, P - 2 - k, P)];"),
    ("reduce_seed_from_root", "send[rank_at(root, P - 1, P)], count * sizeof(float));", "send[rank_at(root, 0, P)], count * sizeof(float));"),
    ("reduce_chunk_gap", "size_t e0 = (size_t)c * chunk_elems;\n                size_t e1 = e0 + chunk_elems < count ? e0 + chunk_elems : count;\n                if (payload) {",
     "size_t e0 = (size_t)c * chunk_elems;\n                size_t e1 = e0 + chunk_elems < count ? e0 + chunk_elems - (c == 1) : count;\n                if (payload) {"),
    ("reduce_two_hops_a_step", "if (c < nchunks && before[k + 1] > c) {", "if (c < nchunks && got[k + 1] > c) {"),
    ("direct_skips_last", "for (int k = 1; k < P; k++) {\n        transfer(bufs, tr, sends, root,",
     "for (int k = 1; k < P - 1; k++) {\n        transfer(bufs, tr, sends, root,"),
    ("ring_wrong_piece", "long pc = ((q - t) % P + P) % P;", "long pc = ((q + t) % P + P) % P;"),
    ("scatter_wrong_half", "q + stride, PIECE_LO(q + stride), PIECE_LO(last));", "q + stride, PIECE_LO(q), PIECE_LO(q + stride));"),
    ("model_pipeline_fill", "return (M / C + (n - 2)) * (ts + C / B);", "return (M / C + (n - 1)) * (ts + C / B);"),
    ("model_chain_n", "return (n - 1) * (ts + M / B); }", "return n * (ts + M / B); }"),
]


def _battery_passes():
    try:
        pin_chain_brute_force(maxP=5, maxM=12)
        pin_chain_schedule_invariants()
        pin_chain_forwarding_is_from_neighbour_payload()
        pin_golden_counts()
        pin_variants_end_state_and_counts(maxP=6)
        pin_cost_models()
        pin_reduce_golden()
        pin_reduce_exact_integers_and_schedule(maxP=5, maxN=7)
    except (AssertionError, ValueError, KeyError, IndexError):
        return False
    return True


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_reject_planted_mistake(tmp_path, name, old, new):
    src_dir = os.path.dirname(oracle.__file__)
    src = open(os.path.join(src_dir, "bcast_oracle.c")).read()
    assert src.count(old) == 1, "mutation site for %s not found exactly once" % name
    (tmp_path / "bcast_oracle.c").write_text(src.replace(old, new))
    (tmp_path / "bcast_oracle.h").write_text(open(os.path.join(src_dir, "bcast_oracle.h")).read())
    so = tmp_path / ("mutant_%s.so" % name)
    subprocess.check_call(["gcc", "-std=c99", "-O1", "-fPIC", "-shared", str(tmp_path / "bcast_oracle.c"), "-o", str(so)])
    try:
        oracle.use_library(so)
        assert not _battery_passes(), "planted mistake %r went unnoticed" % name
    finally:
        oracle.use_library(None)
    assert _battery_passes()
