"""An independent reader of the packed chunk formats, written from the format
descriptions alone (not from the oracle's packer, not from the HIP kernels).

Contiguous-pack layout (packs of 8 tokens): (64/k)*128 header bytes, byte
[g*128 + d] = (width << 4) | min for the pack of token group g (k tokens) and
channel d; then the pack payloads in the same order, k*width/8 bytes each,
little-endian, token i at bits [i*width, (i+1)*width); zero padding up to a
multiple of 16 bytes.

Plane layout (packs of 16 tokens): 512 header bytes in pack-list order
(group-major: pack p = g*128 + d; channel-major: p = d*4 + g); region E: one
32-bit word per pack of width >= 2 (the low two bits of its codes) directly
followed, for width 4, by a second word (the high two bits), packs in list
order; region O: one 16-bit word per pack of odd width (the top bit of its
codes), packs in list order; zero padding to a multiple of 16 bytes.  Bit
positions: words of region E hold token i at bits 4i (i < 8) or 4(i-8)+2
(i >= 8); words of region O hold token i at bit 4*(i%4) + i//4.
"""
import numpy as np

D, N, K = 128, 64, 16
PACKS = (N // K) * D


def read_chunk_planes(buf, order="group"):
    """Plane layout, packs of 16 -> (codes [64,128], widths [512], mins [512]), the last two
    indexed [g*128 + d]."""
    buf = np.asarray(buf, dtype=np.uint8)
    assert order in ("group", "channel")
    where = [divmod(p, D) if order == "group" else (p % 4, p // 4) for p in range(PACKS)]
    widths = np.zeros(PACKS, np.int64)
    mins = np.zeros(PACKS, np.int64)
    codes = np.zeros((N, D), np.int64)
    e_words = sum((int(buf[p]) >> 4) // 2 for p in range(PACKS))
    e_pos, o_pos = PACKS, PACKS + 4 * e_words
    for p, (g, d) in enumerate(where):
        w, m = int(buf[p]) >> 4, int(buf[p]) & 15
        assert w <= 4
        widths[g * D + d], mins[g * D + d] = w, m
        low = high = top = 0
        if w >= 2:
            low = int.from_bytes(bytes(buf[e_pos:e_pos + 4]), "little")
            e_pos += 4
        if w == 4:
            high = int.from_bytes(bytes(buf[e_pos:e_pos + 4]), "little")
            e_pos += 4
        if w % 2:
            top = int.from_bytes(bytes(buf[o_pos:o_pos + 2]), "little")
            o_pos += 2
        for i in range(16):
            at = 4 * i if i < 8 else 4 * (i - 8) + 2
            c = ((low >> at) & 3) + 4 * ((high >> at) & 3)
            if w % 2:
                c += ((top >> (4 * (i % 4) + i // 4)) & 1) << (w - 1)
            codes[g * 16 + i, d] = c + m
    assert e_pos == PACKS + 4 * e_words
    assert (o_pos + 15) // 16 * 16 == len(buf), (o_pos, len(buf))
    assert not buf[o_pos:].any(), "padding must be zero"
    return codes, widths, mins


def read_chunk(buf, k=K, order="group", contiguous=False):
    """buf: uint8 array holding exactly one chunk -> (codes [64,128], widths [packs], mins [packs]).
    Packs of 16 are read in the plane layout unless contiguous is set."""
    if k == 16 and not contiguous:
        return read_chunk_planes(buf, order)
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


def read_arena(arena, offsets16, B, T, H, k=K, wide=False, order="group"):
    """Decode every chunk of an arena -> codes int64 [B, T, H, 128]."""
    out = np.zeros((B, T, H, D), np.int64)
    c = 0
    for blk in range(T // N):
        for b in range(B):
            for h in range(H):
                lo, hi = int(offsets16[c]) * 16, int(offsets16[c + 1]) * 16
                codes, _, _ = read_chunk_wide(arena[lo:hi]) if wide else read_chunk(arena[lo:hi], k, order)
                out[b, blk * N:(blk + 1) * N, h, :] = codes
                c += 1
    return out
