"""CPU-only checks of the native library's host side: it loads, exports every
symbol the header declares, rejects bad arguments before touching the GPU, and
its chain geometry and tuning table behave as documented.  No kernel runs."""
import ctypes
import os
import re

import pytest

from paper_1707_09414_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    headers = sorted(f for f in os.listdir(os.path.join(ROOT, "include")) if f.endswith(".h"))
    assert "bcast.h" in headers and "bcast_debug.h" in headers
    header = "".join(open(os.path.join(ROOT, "include", f)).read() for f in headers)
    # strip comments, then collect identifiers followed by '(' at declaration level
    code = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(bcast_[a-z_0-9]+)\s*\(", code))
    assert declared, "no declarations found"
    lib = ctypes.CDLL(str(B.LIB_PATH))
    for name in sorted(declared):
        assert hasattr(lib, name), "library does not export %s" % name
    assert declared == set(B.EXPORTS), declared ^ set(B.EXPORTS)


def test_strerror_and_version():
    assert B.bcast_strerror(B.BCAST_OK) == "ok"
    for code in (B.BCAST_ERR_ARG, B.BCAST_ERR_NOMEM, B.BCAST_ERR_HIP, B.BCAST_ERR_TIMEOUT, B.BCAST_ERR_UNTUNED):
        assert B.bcast_strerror(code) not in ("ok", "unknown status")
    assert "gfx950" in B.bcast_version()


def test_plan_create_rejects_bad_arguments_without_gpu():
    for nranks, bytes_, chunk, algo in [(0, 1024, 64, 1), (65, 1024, 64, 1), (4, 1024, 24, 1), (4, 1024, 64, 9), (4, 1024, 64, -1)]:
        with pytest.raises(B.BcastError) as e:
            B.bcast_plan_create(nranks, bytes_, chunk, algo)
        assert e.value.status == B.BCAST_ERR_ARG


def test_chain_geometry_matches_eq5_chunking():
    # 1 MiB in 64 KiB chunks over 4 ranks: 16 chunks (Sec. IV-B)
    g = B.bcast_chain_geometry(4, 1 << 20, 64 << 10, 4096)
    assert g["nchunks"] == 16 and g["chunk_bytes"] == 64 << 10
    assert g["lanes"] * 3 <= 4096 and g["grid_blocks"] * 4 >= g["lanes"] * 3
    assert g["algorithmic_bytes"] == 2 * 3 * (1 << 20)
    # ragged tail counts as a chunk
    assert B.bcast_chain_geometry(3, 1001, 112, 64)["nchunks"] == 9
    # C >= M is the unpipelined chain: one chunk
    g = B.bcast_chain_geometry(8, 4096, 1 << 20, 4096)
    assert g["nchunks"] == 1 and g["chunk_bytes"] == 4096
    # tiny message
    g = B.bcast_chain_geometry(64, 4, 8192, 4096)
    assert g["nchunks"] == 1 and g["lanes"] == 1 and g["grid_blocks"] == 16
    # lanes never exceed what fits at once, whatever is requested
    g = B.bcast_chain_geometry(64, 1 << 30, 4 << 20, 2048, lanes_request=1000)
    assert g["lanes"] == 2048 // 63 and g["stages"] == 63 and g["hops_per_stage"] == 1
    # stages: consecutive hops grouped as evenly as possible
    g = B.bcast_chain_geometry(64, 1 << 30, 4 << 20, 8192, stages_request=8)
    assert (g["stages"], g["hops_per_stage"], g["lanes"]) == (8, 8, 1024)  # 4 MiB = 1024 trips of 4 KiB
    g = B.bcast_chain_geometry(64, 1 << 30, 4 << 20, 8192, stages_request=5)
    assert (g["stages"], g["hops_per_stage"]) == (5, 13)
    # exactly the stages asked for (up to one per hop), also where they cannot be equal
    g = B.bcast_chain_geometry(10, 1 << 20, 64 << 10, 8192, stages_request=4)
    assert (g["stages"], g["hops_per_stage"]) == (4, 3)  # 9 hops as 3+2+2+2, rotating
    g = B.bcast_chain_geometry(8, 1 << 26, 8 << 20, 8192, stages_request=100)
    assert (g["stages"], g["hops_per_stage"], g["lanes"]) == (7, 1, 1024)
    g = B.bcast_chain_geometry(8, 1 << 26, 8 << 20, 8192, stages_request=1)
    assert (g["stages"], g["hops_per_stage"], g["grid_blocks"]) == (1, 7, 512)
    # trip size: 4 KiB unless 3 KiB is asked for; a lane owns whole trips
    assert g["trip_bytes"] == 4096 and g["slice_bytes"] == 4096
    g = B.bcast_chain_geometry(64, 1 << 30, 3 << 20, 8192, stages_request=2, trip_request=3072)
    assert (g["trip_bytes"], g["lanes"], g["slice_bytes"], g["nchunks"]) == (3072, 1024, 3072, 342)
    g = B.bcast_chain_geometry(64, 1 << 30, 3 << 20, 8192, stages_request=2, trip_request=4096)
    assert (g["lanes"], g["slice_bytes"]) == (512, 8192)  # 768 trips: the next power of two below
    for bad_trip in (1024, 5120, 3000, 8192):  # built for 2, 3, 4 and 6 KiB
        with pytest.raises(B.BcastError):
            B.bcast_chain_geometry(8, 1 << 20, 4096, 64, trip_request=bad_trip)
    assert B.bcast_chain_geometry(8, 1 << 20, 64 << 10, 64, trip_request=2048)["trip_bytes"] == 2048
    # workgroups of 1, 2 or 4 wavefronts: same waves, more blocks
    for block, blocks in ((64, 2048), (128, 1024), (256, 512), (0, 512)):
        g = B.bcast_chain_geometry(64, 1 << 30, 3 << 20, 8192, stages_request=2, trip_request=3072, block_request=block)
        assert (g["lanes"], g["grid_blocks"], g["block_threads"]) == (1024, blocks, block or 256)
    g = B.bcast_chain_geometry(4, 100, 16, 64, lanes_request=1, block_request=128)
    assert g["grid_blocks"] == 2  # 3 stages x 1 lane in 2-wave workgroups
    with pytest.raises(B.BcastError):
        B.bcast_chain_geometry(8, 1 << 20, 4096, 64, block_request=32)
    # no-ops
    assert B.bcast_chain_geometry(1, 1 << 20, 4096, 64)["nchunks"] == 0
    assert B.bcast_chain_geometry(4, 0, 4096, 64)["nchunks"] == 0
    for bad in [(4, 100, 0, 64), (4, 100, 8, 64), (65, 100, 16, 64), (4, 100, 16, 2)]:
        with pytest.raises(B.BcastError):
            B.bcast_chain_geometry(*bad)


def test_stage_spans_cover_the_chain_and_rotate_evenly():
    """For every chunk the stages' spans tile hops 1..P-1 in order, each span has
    floor or ceil((P-1)/stages) hops, the stage with an extra hop is the one the
    rule names, and over `stages` consecutive chunks all stages play equally."""
    for P in list(range(2, 20)) + [31, 32, 33, 63, 64]:
        H = P - 1
        for S in range(1, H + 1):
            q, r = divmod(H, S)
            played = [0] * S
            for c in list(range(2 * S + 1)) + [10 ** 9 + 7]:
                nxt = 1
                for g in range(S):
                    first, last = B.bcast_chain_stage_span(P, S, g, c)
                    assert first == nxt, (P, S, c, g)
                    n = last - first + 1
                    assert n == q + (1 if (g + c) % S < r else 0), (P, S, c, g, n)
                    nxt = last + 1
                    if c < S:
                        played[g] += n
                assert nxt == H + 1
            assert played == [H] * S, (P, S, played)
    assert B.bcast_chain_stage_span(8, 2, 0, 0) == (1, 4) and B.bcast_chain_stage_span(8, 2, 1, 0) == (5, 7)
    assert B.bcast_chain_stage_span(8, 2, 0, 1) == (1, 3) and B.bcast_chain_stage_span(8, 2, 1, 1) == (4, 7)
    for bad in [(1, 1, 0, 0), (8, 8, 0, 0), (8, 0, 0, 0), (8, 2, 2, 0), (8, 2, -1, 0), (65, 2, 0, 0)]:
        with pytest.raises(B.BcastError):
            B.bcast_chain_stage_span(*bad)


def test_tuning_table_lookup_rules(tmp_path):
    B.bcast_tune_clear()
    assert B.bcast_tune_count() == 0
    with pytest.raises(B.BcastError) as e:
        B.bcast_tune_lookup(8, 4096)
    assert e.value.status == B.BCAST_ERR_UNTUNED
    B.bcast_tune_set(8, 1 << 12, B.BCAST_ALGO_BINOMIAL, 0, 11.0)
    B.bcast_tune_set(8, 1 << 20, B.BCAST_ALGO_CHAIN, 64 << 10, 50.0)
    B.bcast_tune_set(16, 1 << 20, B.BCAST_ALGO_DIRECT, 0, 70.0)
    # same bucket, anywhere inside it
    assert B.bcast_tune_lookup(8, (1 << 12) + 5)[0] == B.BCAST_ALGO_BINOMIAL
    # between entries: nearest at or below
    assert B.bcast_tune_lookup(8, 1 << 19)[0] == B.BCAST_ALGO_BINOMIAL
    assert B.bcast_tune_lookup(8, 1 << 26) == (B.BCAST_ALGO_CHAIN, 64 << 10, 50.0)
    # below the smallest entry: nearest above
    assert B.bcast_tune_lookup(8, 16)[0] == B.BCAST_ALGO_BINOMIAL
    # rank counts have their own entries ...
    assert B.bcast_tune_lookup(16, 4)[0] == B.BCAST_ALGO_DIRECT
    # ... and a rank count without any borrows those of the closest one in ratio
    assert B.bcast_tune_lookup(4, 4096)[0] == B.BCAST_ALGO_BINOMIAL    # 8 (x2) is closer than 16 (x4)
    assert B.bcast_tune_lookup(12, 4096)[0] == B.BCAST_ALGO_DIRECT     # 16 (x1.33) is closer than 8 (x1.5)
    assert B.bcast_tune_lookup(11, 4096)[0] == B.BCAST_ALGO_BINOMIAL   # 8 (x1.375) is closer than 16 (x1.45)
    assert B.bcast_tune_lookup(64, 1 << 20)[0] == B.BCAST_ALGO_DIRECT
    B.bcast_tune_set(32, 1 << 12, B.BCAST_ALGO_CHAIN, 4096, 9.0)
    assert B.bcast_tune_lookup(23, 4096)[0] == B.BCAST_ALGO_CHAIN     # 16 and 32 are equally close: the larger
    # chain entries need a valid chunk
    with pytest.raises(B.BcastError):
        B.bcast_tune_set(8, 1 << 20, B.BCAST_ALGO_CHAIN, 0)
    with pytest.raises(B.BcastError):
        B.bcast_tune_set(8, 1 << 20, 7, 0)

    # the chain's own best setting is kept beside the winner
    e = B.bcast_tune_get(8, 1 << 20)
    assert (e["chain_chunk_bytes"], e["chain_usec"], e["algo"]) == (64 << 10, 50.0, B.BCAST_ALGO_CHAIN)
    assert B.bcast_tune_get(16, 1 << 20)["chain_chunk_bytes"] == 0  # direct won and no chain setting is recorded
    B.bcast_tune_put(16, 1 << 20, algo=B.BCAST_ALGO_DIRECT, usec=70.0, chain_chunk_bytes=128 << 10, chain_stages=4, chain_usec=90.0)
    e = B.bcast_tune_get(16, 1 << 21)
    assert (e["algo"], e["chain_chunk_bytes"], e["chain_stages"], e["chain_usec"]) == (B.BCAST_ALGO_DIRECT, 128 << 10, 4, 90.0)
    with pytest.raises(B.BcastError):
        B.bcast_tune_put(16, 1 << 20, algo=B.BCAST_ALGO_CHAIN, chunk_bytes=24)  # not a multiple of 16
    with pytest.raises(B.BcastError):
        B.bcast_tune_put(16, 1 << 20, algo=B.BCAST_ALGO_DIRECT, chain_stages=65)
    with pytest.raises(B.BcastError):
        B.bcast_tune_put(16, 1 << 20, algo=B.BCAST_ALGO_CHAIN, chunk_bytes=4096, trip_bytes=5120)
    B.bcast_tune_put(16, 1 << 24, algo=B.BCAST_ALGO_CHAIN, chunk_bytes=3 << 20, stages=2, trip_bytes=3072, usec=80.0,
                     stage_store=B.BCAST_STORE_BACK)
    # how the chain stores inside a stage is part of a chain entry, and of nothing else
    with pytest.raises(B.BcastError):
        B.bcast_tune_put(16, 1 << 20, algo=B.BCAST_ALGO_CHAIN, chunk_bytes=4096, stage_store=3)
    with pytest.raises(B.BcastError):
        B.bcast_tune_put(16, 1 << 20, algo=B.BCAST_ALGO_DIRECT, stage_store=B.BCAST_STORE_BACK)
    # ... and so are an explicit lane count (either chain kernel) and the handling of unequal stages (the chain
    # with a wavefront per stage)
    B.bcast_tune_put(16, 1 << 25, algo=B.BCAST_ALGO_CHAIN, chunk_bytes=6 << 20, stages=2, trip_bytes=3072, usec=90.0,
                     lanes=512, spans=B.BCAST_SPANS_ROTATE)
    B.bcast_tune_put(16, 1 << 21, algo=B.BCAST_ALGO_CHAIN, chunk_bytes=1 << 20, stages=2, trip_bytes=4096, usec=9.0, lanes=64, rank_waves=1)
    assert (B.bcast_tune_get(16, 1 << 21)["lanes"], B.bcast_tune_get(16, 1 << 21)["rank_waves"]) == (64, 1)
    for bad in (dict(lanes=-1), dict(lanes=8193), dict(spans=3), dict(spans=B.BCAST_SPANS_FIXED, rank_waves=1)):
        with pytest.raises(B.BcastError):
            B.bcast_tune_put(16, 1 << 20, algo=B.BCAST_ALGO_CHAIN, chunk_bytes=4096, **bad)
    with pytest.raises(B.BcastError):
        B.bcast_tune_put(16, 1 << 20, algo=B.BCAST_ALGO_BINOMIAL, lanes=64)

    path = tmp_path / "table.txt"
    B.bcast_tune_save(str(path))
    B.bcast_tune_clear()
    B.bcast_tune_load(str(path))
    assert B.bcast_tune_count() == 7
    e = B.bcast_tune_get(16, 1 << 25)
    assert (e["lanes"], e["chain_lanes"], e["spans"], e["chain_spans"]) == (512, 512, B.BCAST_SPANS_ROTATE, B.BCAST_SPANS_ROTATE)
    e = B.bcast_tune_get(16, 1 << 24)
    assert (e["trip_bytes"], e["chain_trip_bytes"], e["chain_chunk_bytes"], e["stages"]) == (3072, 3072, 3 << 20, 2)
    assert (e["stage_store"], e["chain_stage_store"]) == (B.BCAST_STORE_BACK, B.BCAST_STORE_BACK)
    assert B.bcast_tune_get(8, 1 << 20)["stage_store"] == B.BCAST_STORE_AUTO
    assert B.bcast_tune_lookup(8, 1 << 20) == (B.BCAST_ALGO_CHAIN, 64 << 10, 50.0)
    e = B.bcast_tune_get(16, 1 << 20)
    assert (e["chain_chunk_bytes"], e["chain_stages"], e["chain_usec"]) == (128 << 10, 4, 90.0)
    # files with only the first five, seven or nine columns still load
    old = tmp_path / "old.txt"
    old.write_text("4 20 1 65536 12.5\n4 10 3 0 5.0\n4 12 2 0 5.0 8192 7.5\n4 24 1 1048576 9.0 1048576 9.0 2 2\n")
    B.bcast_tune_load(str(old))
    e = B.bcast_tune_get(4, 1 << 20)
    assert (e["chain_chunk_bytes"], e["chain_usec"], e["stages"]) == (65536, 12.5, 0)
    assert B.bcast_tune_get(4, 1 << 12)["chain_chunk_bytes"] == 8192
    e = B.bcast_tune_get(4, 1 << 24)
    assert (e["stages"], e["chain_stages"], e["trip_bytes"], e["chain_trip_bytes"]) == (2, 2, 0, 0)

    bad = tmp_path / "bad.txt"
    bad.write_text("8 20 1 65536 1.0\n8 21 1 7 1.0\n")
    B.bcast_tune_clear()
    with pytest.raises(B.BcastError):
        B.bcast_tune_load(str(bad))
    assert B.bcast_tune_count() == 0, "a malformed file must install nothing"
    with pytest.raises(B.BcastError):
        B.bcast_tune_load(str(tmp_path / "missing.txt"))
    B.bcast_tune_clear()
