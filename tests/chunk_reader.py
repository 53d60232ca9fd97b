"""An independent reader of the packed chunk format, written from the format
description alone (not from the oracle's packer, not from the HIP kernels).

Chunk for packs of k tokens (k = 16 by default, or 8) = (64/k)*128 header bytes,
byte [g*128 + d] = (width << 4) | min for the pack of token group g (k tokens)
and channel d; then the pack payloads in the same order, k*width/8 bytes each,
little-endian, token i at bits [i*width, (i+1)*width); zero padding up to a
multiple of 16 bytes.
"""
import numpy as np

D, N, K = 128, 64, 16
PACKS = (N // K) * D


def read_chunk(buf, k=K):
    """buf: uint8 array holding exactly one chunk -> (codes [64,128], widths [packs], mins [packs])."""
    buf = np.asarray(buf, dtype=np.uint8)
    packs = (N // k) * D
    widths = (buf[:packs] >> 4).astype(np.int64)
    mins = (buf[:packs] & 15).astype(np.int64)
    codes = np.zeros((N, D), np.int64)
    pos = packs
    for p in range(packs):
        g, d = divmod(p, D)
        w = int(widths[p])
        nbytes = k * w // 8
        value = int.from_bytes(bytes(buf[pos:pos + nbytes]), "little")
        pos += nbytes
        for i in range(k):
            codes[g * k + i, d] = ((value >> (i * w)) & ((1 << w) - 1)) + int(mins[p])
    padded = (pos + 15) // 16 * 16
    assert padded == len(buf), (padded, len(buf))
    assert not buf[pos:].any(), "padding must be zero"
    return codes, widths, mins


def read_chunk_wide(buf):
    """Wide chunk (codes up to 255, packs of 8 tokens): 1024 width bytes, 1024 minimum bytes, both
    indexed [g*128 + d], then the packs, `width` bytes each, little-endian, token i at bits
    [i*width, (i+1)*width); zero padding to 16 bytes.  -> (codes [64,128], widths, mins)."""
    buf = np.asarray(buf, dtype=np.uint8)
    packs = (N // 8) * D
    widths = buf[:packs].astype(np.int64)
    mins = buf[packs:2 * packs].astype(np.int64)
    codes = np.zeros((N, D), np.int64)
    pos = 2 * packs
    for p in range(packs):
        g, d = divmod(p, D)
        w = int(widths[p])
        value = int.from_bytes(bytes(buf[pos:pos + w]), "little")
        pos += w
        for i in range(8):
            codes[g * 8 + i, d] = ((value >> (i * w)) & ((1 << w) - 1)) + int(mins[p])
    assert (pos + 15) // 16 * 16 == len(buf), (pos, len(buf))
    assert not buf[pos:].any(), "padding must be zero"
    return codes, widths, mins


def read_arena(arena, offsets16, B, T, H, k=K, wide=False):
    """Decode every chunk of an arena -> codes int64 [B, T, H, 128]."""
    out = np.zeros((B, T, H, D), np.int64)
    c = 0
    for blk in range(T // N):
        for b in range(B):
            for h in range(H):
                lo, hi = int(offsets16[c]) * 16, int(offsets16[c + 1]) * 16
                codes, _, _ = read_chunk_wide(arena[lo:hi]) if wide else read_chunk(arena[lo:hi], k)
                out[b, blk * N:(blk + 1) * N, h, :] = codes
                c += 1
    return out
