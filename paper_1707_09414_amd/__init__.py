"""Pipelined chain broadcast for one MI355X (gfx950): P virtual ranks are P
device buffers, chunks are handed from buffer to buffer by a persistent HIP
kernel.  ``paper_1707_09414_amd.binding`` is the API (it loads the native
library and raises if it is not built); ``paper_1707_09414_amd.inputs`` holds
the seeded synthetic messages.  Importing the package itself loads nothing."""

__all__ = ["binding", "inputs", "build"]
