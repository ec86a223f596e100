"""The two measurement kernels behind bench.py's `ceilings` rows: they must touch
exactly the bytes they are charged for, or the ceilings would be wrong."""
import numpy as np
import pytest
import torch

from paper_1707_09414_amd import binding as B

pytestmark = pytest.mark.gpu
GUARD = 256


@pytest.mark.parametrize("nbufs,tiles", [(1, 1), (3, 5), (7, 4099), (63, 64)])
def test_store_pattern_writes_every_tile_of_every_buffer_and_nothing_else(nbufs, tiles):
    n = tiles * 4096
    raws = [torch.full((GUARD + n + GUARD,), 0xFF, dtype=torch.uint8, device="cuda") for _ in range(nbufs)]
    bufs = [t[GUARD: GUARD + n] for t in raws]
    B.bcast_debug_store_pattern(bufs, n, torch.cuda.current_stream())
    torch.cuda.synchronize()
    for t in raws:
        h = t.cpu().numpy()
        assert (h[:GUARD] == 0xFF).all() and (h[GUARD + n:] == 0xFF).all()
        words = h[GUARD: GUARD + n].view(np.uint32).reshape(-1, 4)
        # every 16-byte vector ends in the two marker words; lane numbers run 0..63 along a 1 KiB row
        assert (words[:, 2] == 0x5A5A5A5A).all() and (words[:, 3] == 0xA5A5A5A5).all()
        assert np.array_equal(words[:, 1].reshape(-1, 64), np.broadcast_to(np.arange(64, dtype=np.uint32), (n // 1024, 64)))


@pytest.mark.parametrize("nbufs,tiles", [(1, 1), (2, 3), (5, 1025), (8, 300), (33, 16)])
def test_load_pattern_reads_every_buffer_once(nbufs, tiles):
    n = tiles * 4096
    rng = np.random.default_rng(nbufs * 1000 + tiles)
    host = rng.integers(0, 256, size=(nbufs, n), dtype=np.uint8)
    bufs = [torch.from_numpy(host[i]).cuda() for i in range(nbufs)]
    raw = torch.full((GUARD + n + GUARD,), 0xEE, dtype=torch.uint8, device="cuda")
    out = raw[GUARD: GUARD + n]
    B.bcast_debug_load_pattern(bufs, n, out, False, torch.cuda.current_stream())
    torch.cuda.synchronize()
    assert bool((raw == 0xEE).all()), "without write_result nothing is written"
    B.bcast_debug_load_pattern(bufs, n, out, True, torch.cuda.current_stream())
    torch.cuda.synchronize()
    h = raw.cpu().numpy()
    assert np.array_equal(h[GUARD: GUARD + n], np.bitwise_xor.reduce(host, axis=0))
    assert (h[:GUARD] == 0xEE).all() and (h[GUARD + n:] == 0xEE).all()
    for i in range(nbufs):
        assert np.array_equal(bufs[i].cpu().numpy(), host[i])


def test_pattern_argument_errors():
    a = torch.zeros(8192 + 64, dtype=torch.uint8, device="cuda")
    with pytest.raises(B.BcastError):
        B.bcast_debug_store_pattern([a], 1000)            # not a multiple of 4096
    with pytest.raises(B.BcastError):
        B.bcast_debug_store_pattern([a[4:]], 4096)         # misaligned
    with pytest.raises(B.BcastError):
        B.bcast_debug_store_pattern([a] * 65, 4096)        # too many buffers
    with pytest.raises(B.BcastError):
        B.bcast_debug_load_pattern([a], 4096, a[8:], True)  # misaligned result
    torch.cuda.synchronize()
    assert bool((a == 0).all())
