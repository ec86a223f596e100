"""Seeded synthetic messages shaped like the paper's broadcast workloads.

This module only draws random bytes / floats and lists tensor shapes.  It holds
none of the broadcast method's arithmetic and is the one module that both the
GPU tests and the CPU oracle's tests may use, so both sides see the same inputs.

The paper measured with a message-size sweep micro-benchmark and with VGG
training (Sec. V-B, V-D); neither its benchmark program, dataset nor weights are
used here.  These generators reproduce the message *sizes and mix* only.
"""
from __future__ import annotations

from typing import List, Tuple

import numpy as np

KiB = 1 << 10
MiB = 1 << 20
GiB = 1 << 30

FILL_BYTE = 0xFF  # non-root buffers start as all-ones bytes (a NaN pattern for fp32)


def random_bytes(seed: int, nbytes: int) -> np.ndarray:
    """`nbytes` uniformly random bytes from numpy's default_rng(seed)."""
    rng = np.random.default_rng(seed)
    return rng.integers(0, 256, size=nbytes, dtype=np.uint8)


def uniform_fp32_message(seed: int, numel: int) -> np.ndarray:
    """fp32 values uniform in [-1, 1), returned as their bytes."""
    rng = np.random.default_rng(seed)
    vals = (rng.random(numel, dtype=np.float32) * np.float32(2.0) - np.float32(1.0)).astype(np.float32)
    return vals.view(np.uint8)


def vgg16_tensor_shapes() -> List[Tuple[str, Tuple[int, ...]]]:
    """The 32 parameter tensors of VGG-16 (13 conv 3x3 + 3 FC, each with a bias)."""
    conv = [(3, 64), (64, 64), (64, 128), (128, 128), (128, 256), (256, 256), (256, 256),
            (256, 512), (512, 512), (512, 512), (512, 512), (512, 512), (512, 512)]
    fc = [(25088, 4096), (4096, 4096), (4096, 1000)]
    out: List[Tuple[str, Tuple[int, ...]]] = []
    for i, (cin, cout) in enumerate(conv):
        out.append(("conv%d.weight" % (i + 1), (cout, cin, 3, 3)))
        out.append(("conv%d.bias" % (i + 1), (cout,)))
    for i, (fin, fout) in enumerate(fc):
        out.append(("fc%d.weight" % (i + 1), (fout, fin)))
        out.append(("fc%d.bias" % (i + 1), (fout,)))
    return out


def vgg16_tensor_bytes() -> List[int]:
    """Byte size of each VGG-16 parameter tensor in fp32, in layer order."""
    return [4 * int(np.prod(shape)) for _, shape in vgg16_tensor_shapes()]


def vgg16_packed_message(seed: int, std: float = 0.01) -> Tuple[np.ndarray, List[Tuple[int, int]]]:
    """All VGG-16 parameters, N(0, std) fp32, packed back to back.

    Returns (bytes, [(offset, nbytes) per tensor]).  One normal draw covers the
    whole packed buffer so the per-tensor views and the packed buffer agree.
    """
    sizes = vgg16_tensor_bytes()
    total = sum(sizes)
    rng = np.random.default_rng(seed)
    vals = rng.standard_normal(total // 4, dtype=np.float32) * np.float32(std)
    spans = []
    off = 0
    for s in sizes:
        spans.append((off, s))
        off += s
    return vals.view(np.uint8), spans


def sweep_message_sizes(lo_bytes: int = 4, hi_bytes: int = 64 * MiB) -> List[int]:
    """Powers of two from lo to hi inclusive (the latency-sweep message sizes)."""
    out = []
    m = lo_bytes
    while m <= hi_bytes:
        out.append(m)
        m *= 2
    return out


def sweep_chunk_sizes(lo_bytes: int = 8 * KiB, hi_bytes: int = 4 * MiB) -> List[int]:
    """Powers of two from lo to hi inclusive (candidate chunk sizes)."""
    return sweep_message_sizes(lo_bytes, hi_bytes)
