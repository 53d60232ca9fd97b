"""PackKV decode hot path for MI355X (gfx950): bit-packed KV cache, append-side
compressor and fused decompress + matrix-vector kernels behind a C-ABI library.

Importing the package does not load the HIP library; that happens on first use
of :mod:`paper_2512_24449_amd.binding` and fails loudly if it is missing.
"""
__all__ = ["binding", "synth", "build"]
