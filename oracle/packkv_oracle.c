/*
 * PackKV CPU oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, scalar implementation of what the PackKV decode hot path
 * computes, written from the paper (arXiv 2512.24449).  It exists only so
 * that tests, the smoke check and the benchmark's cpu_baseline leg have
 * something independent to compare the HIP library against.  It shares no
 * code, header, table or helper with the HIP path and is never linked into
 * the product library.
 *
 * Codec steps follow the paper in its own order:
 *   Sec. III-B.2 / Sec. IV-A  token-wise quantization with a relative scale
 *                             (scale = rel * (max - min), error <= scale/2)
 *   Sec. III-B.3              bit-packing: a pack of k integers along
 *                             ctx_len (k = 16 by default, k = 8 as the second
 *                             point of the pack-size study, Sec. IV-B) shares
 *                             one minimum and one width ceil(log2(range+1))
 *   Sec. III-B.4              every 2-D block becomes one contiguous chunk,
 *                             appended at the end of the buffer, plus an index
 * The matvecs are the plain definitions (Sec. III-B.3 boxed statement):
 *   scores = sm_scale * K_hat q      out = p^T V_hat
 * evaluated in fp64 on the decoded values x_hat = scale*code + min.
 *
 * Readings taken where the paper is silent:
 *   - one (scale, min) pair per token over ALL kv-heads' values of that token,
 *     per tensor, stored as fp16; quantization uses the stored fp16 values;
 *   - fp32 subtract and divide, round-half-to-even, clamp to [0, qmax],
 *     qmax = round(1/rel); scale == 0 gives code 0;
 *   - pack metadata is one byte, (width << 4) | min, as long as the codes stay
 *     below 16 (rel >= 1/15); for finer scales (codes up to 255, "wide" chunks,
 *     packs of 8 tokens only) it is two bytes: all widths (0..8) first, one
 *     byte per pack, then all minimums (0..255), one byte per pack;
 *   - chunk bytes, packs of 8: 1024 header bytes indexed [token_group*128 +
 *     channel], then the packs in the same order, each `width` bytes
 *     little-endian with the code of token i at bits [i*width, (i+1)*width),
 *     zero padded to 16 bytes;
 *   - chunk bytes, packs of 16 (orc_pack_chunk_planes): 512 header bytes, then
 *     every pack's 16*width bits as two-bit planes and a one-bit plane (a fixed
 *     order of exactly 16*width bits per pack, Sec. III-B.3), zero padded to 16
 *     bytes; the packs of a chunk are listed group-major or channel-major;
 *   - repacking (V-median and greedy orders): see the comments of
 *     orc_v_median_order and orc_greedy_order; the median and tie conventions
 *     are "parity unpinned" readings (any order is a valid cache).
 *
 * Parity pins live in tests/test_oracle_pins.py; the exact byte order inside a
 * chunk is "parity unpinned" (the paper's format figures are not available):
 * it is a choice of this build, checked only by an independent bit reader.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_D 128      /* head_dim                                  */
#define ORC_N 64       /* tokens per block (truncated block size)   */
#define ORC_K 16       /* default pack size                         */
#define ORC_GROUPS (ORC_N / ORC_K)
#define ORC_PACKS (ORC_GROUPS * ORC_D)
#define ORC_HEADER ORC_PACKS
#define ORC_CHUNK_MAX (ORC_HEADER + ORC_PACKS * 8)
/* any layout: at most 2 * 1024 header bytes + 64*128 payload bytes (wide chunks) */
#define ORC_CHUNK_MAX_ANY (4 * ORC_PACKS + ORC_N * ORC_D)

/* ---------------------------------------------------------------- fp16 -- */

/* IEEE binary16 -> binary32, exact. */
float orc_h2f(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) & 1u;
    uint32_t exp = (uint32_t)(h >> 10) & 0x1Fu;
    uint32_t man = (uint32_t)h & 0x3FFu;
    double v;
    if (exp == 0)
        v = ldexp((double)man, -24);                 /* zero / subnormal */
    else if (exp == 31)
        v = man ? (double)NAN : (double)INFINITY;
    else
        v = ldexp((double)(man + 1024u), (int)exp - 25);
    return (float)(sign ? -v : v);
}

/* binary32 -> binary16, round to nearest even, overflow to infinity. */
uint16_t orc_f2h(float f)
{
    uint16_t sign = (uint16_t)(signbit(f) ? 0x8000u : 0u);
    double a = fabs((double)f);
    if (isnan(f)) return (uint16_t)(sign | 0x7E00u);
    if (a == 0.0) return sign;
    if (isinf(f)) return (uint16_t)(sign | 0x7C00u);
    int e;
    (void)frexp(a, &e);                              /* a = m * 2^e, m in [0.5,1) */
    int ue = e - 1;                                  /* a in [2^ue, 2^(ue+1))     */
    if (ue < -14) ue = -14;                          /* subnormal spacing 2^-24   */
    /* spacing of representable values near a is 2^(ue-10) */
    double scaled = ldexp(a, 10 - ue);               /* exact power-of-two scale  */
    double r = nearbyint(scaled);                    /* default mode: ties-even   */
    double v = ldexp(r, ue - 10);
    if (v >= 65520.0) return (uint16_t)(sign | 0x7C00u);
    /* re-normalise after rounding may have crossed a power of two */
    int e2;
    (void)frexp(v, &e2);
    int ve = e2 - 1;
    uint32_t bits;
    if (v < ldexp(1.0, -14)) {
        bits = (uint32_t)ldexp(v, 24);               /* subnormal mantissa        */
    } else {
        uint32_t man = (uint32_t)(ldexp(v, 10 - ve) - 1024.0);
        bits = ((uint32_t)(ve + 15) << 10) | man;
    }
    return (uint16_t)(sign | bits);
}

/* ------------------------------------------------- quantization (lossy) -- */

/* Levels of the quantizer for a relative scale: 0 .. round(1/rel).
 * (Sec. IV-A: actual scale = rel * (max - min).) */
int orc_qmax(float rel)
{
    return (int)lround(1.0 / (double)rel);
}

/*
 * Token-wise quantization parameters (Sec. III-B.2, Sec. IV-A).
 * x is fp16 [B][T][H][D] with explicit token and batch strides in elements.
 * For every (b, t) the minimum and maximum run over the H*D values of that
 * token.  scale16 = fp16(rel32 * (max - min)) with the product and the
 * difference rounded once each in fp32; min16 is the minimum itself
 * (a zero minimum is stored as +0).
 */
void orc_token_params(const uint16_t *x, int B, int T, int H, int D,
                      int64_t batch_stride, int64_t token_stride, float rel,
                      uint16_t *scale16, uint16_t *min16)
{
    for (int b = 0; b < B; ++b)
        for (int t = 0; t < T; ++t) {
            const uint16_t *row = x + b * batch_stride + t * token_stride;
            float mn = orc_h2f(row[0]), mx = mn;
            uint16_t mn_bits = row[0];
            for (int i = 1; i < H * D; ++i) {
                float v = orc_h2f(row[i]);
                if (v < mn) { mn = v; mn_bits = row[i]; }
                if (v > mx) mx = v;
            }
            if (mn == 0.0f) mn_bits = 0;             /* canonical +0 */
            float range32 = mx - mn;
            float s32 = rel * range32;
            scale16[(int64_t)b * T + t] = orc_f2h(s32);
            min16[(int64_t)b * T + t] = mn_bits;
        }
}

/* One value -> its code (Sec. IV-A; non-negative integers, Sec. III-B.3). */
static int quantize_one(uint16_t x16, uint16_t scale16, uint16_t min16, int qmax)
{
    float s = orc_h2f(scale16);
    if (s == 0.0f) return 0;
    float num = orc_h2f(x16) - orc_h2f(min16);       /* fp32 subtract */
    float ratio = num / s;                           /* fp32 divide   */
    float r = nearbyintf(ratio);                     /* ties to even  */
    int q = (int)r;
    if (q < 0) q = 0;
    if (q > qmax) q = qmax;
    return q;
}

/* Codes for a whole tensor, q is uint8 [B][T][H][D] contiguous. */
void orc_quantize(const uint16_t *x, int B, int T, int H, int D,
                  int64_t batch_stride, int64_t token_stride, float rel,
                  const uint16_t *scale16, const uint16_t *min16, uint8_t *q)
{
    int qmax = orc_qmax(rel);
    for (int b = 0; b < B; ++b)
        for (int t = 0; t < T; ++t) {
            const uint16_t *row = x + b * batch_stride + t * token_stride;
            uint8_t *qrow = q + ((int64_t)b * T + t) * H * D;
            uint16_t s = scale16[(int64_t)b * T + t], m = min16[(int64_t)b * T + t];
            for (int i = 0; i < H * D; ++i)
                qrow[i] = (uint8_t)quantize_one(row[i], s, m, qmax);
        }
}

/* Decoded value the consumer sees: x_hat = scale * code + min, in fp64. */
double orc_xhat(uint8_t code, uint16_t scale16, uint16_t min16)
{
    return (double)orc_h2f(scale16) * (double)code + (double)orc_h2f(min16);
}

void orc_dequant(const uint8_t *q, int B, int T, int H, int D,
                 const uint16_t *scale16, const uint16_t *min16, double *xhat)
{
    for (int64_t bt = 0; bt < (int64_t)B * T; ++bt)
        for (int i = 0; i < H * D; ++i)
            xhat[bt * H * D + i] = orc_xhat(q[bt * H * D + i], scale16[bt], min16[bt]);
}

/* ------------------------------------------------- bit-packing (lossless) -- */

/* Width of a pack whose values span `range` = max - min: ceil(log2(range+1))
 * (Sec. III-B.3). */
int orc_width(int range)
{
    int w = 0;
    while ((1 << w) < range + 1) ++w;
    return w;
}

/*
 * Pack one chunk in the contiguous-pack layout: the 64 x 128 codes of one (batch,
 * kv-head, block), packs of k tokens (k = 8 is the layout of packs of 8 tokens; k = 16
 * in this layout is kept as a second, plainer statement of the same packs that the
 * tests compare the plane layout's sizes and metadata with).  q points at code (token 0, channel 0); consecutive
 * tokens are `token_stride` apart.  Writes the chunk bytes (header, payload,
 * zero padding to 16 bytes) and, when not NULL, the logical per-pack widths and
 * minimums [(64/k)*128].  Returns the chunk size in bytes (a multiple of 16).
 */
int orc_pack_chunk_k(const uint8_t *q, int64_t token_stride, uint8_t *bytes,
                     uint8_t *widths, uint8_t *mins, int k)
{
    int groups = ORC_N / k;
    int pos = groups * ORC_D;
    for (int g = 0; g < groups; ++g)
        for (int d = 0; d < ORC_D; ++d) {
            int p = g * ORC_D + d;
            int lo = 255, hi = 0;
            for (int i = 0; i < k; ++i) {
                int v = q[(int64_t)(g * k + i) * token_stride + d];
                if (v < lo) lo = v;
                if (v > hi) hi = v;
            }
            int w = orc_width(hi - lo);
            bytes[p] = (uint8_t)((w << 4) | lo);
            if (widths) widths[p] = (uint8_t)w;
            if (mins) mins[p] = (uint8_t)lo;
            uint64_t bits = 0;
            for (int i = 0; i < k; ++i) {
                uint64_t c = (uint64_t)(q[(int64_t)(g * k + i) * token_stride + d] - lo);
                bits |= c << (i * w);
            }
            for (int j = 0; j < k * w / 8; ++j)
                bytes[pos++] = (uint8_t)(bits >> (8 * j));
        }
    while (pos % 16) bytes[pos++] = 0;
    return pos;
}

/*
 * Pack one chunk whose codes may exceed 15 (quantization scales finer than
 * 1/15, codes up to 255): packs of 8 tokens, widths up to 8 bits.  Layout:
 * 1024 width bytes indexed [token_group*128 + channel], 1024 minimum bytes in
 * the same order, then the packs, `width` bytes each, code of token i at bits
 * [i*width, (i+1)*width), zero padding to 16 bytes.
 */
int orc_pack_chunk_wide(const uint8_t *q, int64_t token_stride, uint8_t *bytes,
                        uint8_t *widths, uint8_t *mins)
{
    const int k = 8, groups = ORC_N / 8, packs = groups * ORC_D;
    int pos = 2 * packs;
    for (int g = 0; g < groups; ++g)
        for (int d = 0; d < ORC_D; ++d) {
            int p = g * ORC_D + d;
            int lo = 255, hi = 0;
            for (int i = 0; i < k; ++i) {
                int v = q[(int64_t)(g * k + i) * token_stride + d];
                if (v < lo) lo = v;
                if (v > hi) hi = v;
            }
            int w = orc_width(hi - lo);
            bytes[p] = (uint8_t)w;
            bytes[packs + p] = (uint8_t)lo;
            if (widths) widths[p] = (uint8_t)w;
            if (mins) mins[p] = (uint8_t)lo;
            uint64_t bits = 0;
            for (int i = 0; i < k; ++i) {
                uint64_t c = (uint64_t)(q[(int64_t)(g * k + i) * token_stride + d] - lo);
                bits |= c << (i * w);
            }
            for (int j = 0; j < w; ++j)
                bytes[pos++] = (uint8_t)(bits >> (8 * j));
        }
    while (pos % 16) bytes[pos++] = 0;
    return pos;
}


/*
 * Pack one chunk with packs of 16 tokens (the default pack size, Sec. IV-A) in the
 * plane layout.  The paper fixes what a pack stores -- one minimum, one width w =
 * ceil(log2(range+1)) and 16 codes of w bits (Sec. III-B.3) -- and that lengths and
 * minimums come first in the block (Sec. III-C); the order of the 16*w bits is a
 * choice of this build:
 *   pack list     order 0 (group-major):   pack p = g*128 + d
 *                 order 1 (channel-major): pack p = d*4 + g
 *                 (g = token group of 16 tokens, d = channel)
 *   bytes [0,512) header, byte p = (w << 4) | min of pack p
 *   region E      for p = 0..511 in turn: if w >= 2 one little-endian 32-bit word
 *                 with the low two bits (c & 3) of the 16 codes, and if w == 4 a
 *                 second word with the high two bits (c >> 2); in both words token i
 *                 of the pack sits at bits [4i, 4i+2) for i < 8 and at
 *                 [4(i-8)+2, 4(i-8)+4) for i >= 8
 *   region O      for p = 0..511 in turn: if w is odd one little-endian 16-bit word
 *                 with the top bit (c >> (w-1)) of the 16 codes, token i at bit
 *                 4*(i & 3) + (i >> 2)
 *   zero padding to a multiple of 16 bytes
 * so a pack takes 0, 16, 32, 48 or 64 bits for w = 0..4.  widths / mins (optional)
 * receive the logical per-pack values indexed [g*128 + d] whatever the order.
 * Returns the chunk size in bytes.
 */
int orc_pack_chunk_planes(const uint8_t *q, int64_t token_stride, uint8_t *bytes,
                          uint8_t *widths, uint8_t *mins, int order)
{
    int w_of[ORC_PACKS], lo_of[ORC_PACKS], g_of[ORC_PACKS], d_of[ORC_PACKS];
    for (int p = 0; p < ORC_PACKS; ++p) {
        int g = order ? p % ORC_GROUPS : p / ORC_D;
        int d = order ? p / ORC_GROUPS : p % ORC_D;
        int lo = 255, hi = 0;
        for (int i = 0; i < ORC_K; ++i) {
            int v = q[(int64_t)(g * ORC_K + i) * token_stride + d];
            if (v < lo) lo = v;
            if (v > hi) hi = v;
        }
        int w = orc_width(hi - lo);
        g_of[p] = g, d_of[p] = d, w_of[p] = w, lo_of[p] = lo;
        bytes[p] = (uint8_t)((w << 4) | lo);
        if (widths) widths[g * ORC_D + d] = (uint8_t)w;
        if (mins) mins[g * ORC_D + d] = (uint8_t)lo;
    }
    int pos = ORC_HEADER;
    for (int p = 0; p < ORC_PACKS; ++p) {                 /* region E */
        int w = w_of[p];
        if (w < 2) continue;
        uint32_t low = 0, high = 0;
        for (int i = 0; i < ORC_K; ++i) {
            uint32_t c = (uint32_t)(q[(int64_t)(g_of[p] * ORC_K + i) * token_stride + d_of[p]] - lo_of[p]);
            int at = i < 8 ? 4 * i : 4 * (i - 8) + 2;
            low |= (c & 3u) << at;
            high |= (c >> 2) << at;
        }
        for (int j = 0; j < 4; ++j) bytes[pos++] = (uint8_t)(low >> (8 * j));
        if (w == 4)
            for (int j = 0; j < 4; ++j) bytes[pos++] = (uint8_t)(high >> (8 * j));
    }
    for (int p = 0; p < ORC_PACKS; ++p) {                 /* region O */
        int w = w_of[p];
        if (!(w & 1)) continue;
        uint32_t top = 0;
        for (int i = 0; i < ORC_K; ++i) {
            uint32_t c = (uint32_t)(q[(int64_t)(g_of[p] * ORC_K + i) * token_stride + d_of[p]] - lo_of[p]);
            top |= ((c >> (w - 1)) & 1u) << (4 * (i & 3) + (i >> 2));
        }
        bytes[pos++] = (uint8_t)top;
        bytes[pos++] = (uint8_t)(top >> 8);
    }
    while (pos % 16) bytes[pos++] = 0;
    return pos;
}

/* Packs of 16 tokens, group-major pack list. */
int orc_pack_chunk(const uint8_t *q, int64_t token_stride, uint8_t *bytes,
                   uint8_t *widths, uint8_t *mins)
{
    return orc_pack_chunk_planes(q, token_stride, bytes, widths, mins, 0);
}

/*
 * Compress a whole tensor of T = 64*nblk tokens (Sec. III-B.1 .. III-B.4).
 * Chunks are appended block by block; inside a block in (batch, kv-head)
 * order, so chunk index c = (block*B + b)*H + h.  offsets16[c] is the start of
 * chunk c in 16-byte units, offsets16[nchunks] the end of the arena.
 * meta[b*T + t] = scale16 | min16 << 16.  q_out (optional) receives the codes,
 * widths_out / mins_out (optional) the per-pack values [nchunks][(64/k)*128],
 * indexed [token_group*128 + channel].  order: pack list of the chunks with packs
 * of 16 (0 group-major, 1 channel-major; see orc_pack_chunk_planes).
 * Returns the arena size in bytes, or -1 if it would exceed arena_cap.
 */
int64_t orc_compress_k(const uint16_t *x, int B, int T, int H, int D,
                       int64_t batch_stride, int64_t token_stride, float rel,
                       uint8_t *arena, int64_t arena_cap, uint32_t *offsets16,
                       uint32_t *meta, uint8_t *q_out, uint8_t *widths_out,
                       uint8_t *mins_out, int k, int order)
{
    if (D != ORC_D || T % ORC_N || (k != 8 && k != 16)) return -2;
    if (order != 0 && (order != 1 || k != 16)) return -2;  /* the pack list order exists for packs of 16 */
    int wide = orc_qmax(rel) > 15;  /* codes do not fit the 4-bit minimum of the one-byte metadata */
    if (wide && (k != 8 || orc_qmax(rel) > 255)) return -2;
    int packs = ORC_N / k * ORC_D;
    int64_t n = (int64_t)B * T;
    uint16_t *scale16 = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)n);
    uint16_t *min16 = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)n);
    uint8_t *q = q_out ? q_out : (uint8_t *)malloc((size_t)n * H * D);
    orc_token_params(x, B, T, H, D, batch_stride, token_stride, rel, scale16, min16);
    orc_quantize(x, B, T, H, D, batch_stride, token_stride, rel, scale16, min16, q);
    for (int64_t i = 0; i < n; ++i)
        meta[i] = (uint32_t)scale16[i] | ((uint32_t)min16[i] << 16);

    int nblk = T / ORC_N;
    int64_t pos = 0, c = 0;
    uint8_t tmp[ORC_CHUNK_MAX_ANY + 16];
    int64_t rc = 0;
    for (int blk = 0; blk < nblk && rc == 0; ++blk)
        for (int b = 0; b < B && rc == 0; ++b)
            for (int h = 0; h < H; ++h, ++c) {
                const uint8_t *q0 = q + (((int64_t)b * T + (int64_t)blk * ORC_N) * H + h) * D;
                uint8_t *wo = widths_out ? widths_out + c * packs : NULL;
                uint8_t *mo = mins_out ? mins_out + c * packs : NULL;
                int sz = wide ? orc_pack_chunk_wide(q0, (int64_t)H * D, tmp, wo, mo)
                         : k == 16 ? orc_pack_chunk_planes(q0, (int64_t)H * D, tmp, wo, mo, order)
                                   : orc_pack_chunk_k(q0, (int64_t)H * D, tmp, wo, mo, k);
                if (pos + sz > arena_cap) { rc = -1; break; }
                memcpy(arena + pos, tmp, (size_t)sz);
                offsets16[c] = (uint32_t)(pos / 16);
                pos += sz;
            }
    if (rc == 0) offsets16[c] = (uint32_t)(pos / 16);
    free(scale16);
    free(min16);
    if (!q_out) free(q);
    return rc ? rc : pos;
}

int64_t orc_compress(const uint16_t *x, int B, int T, int H, int D,
                     int64_t batch_stride, int64_t token_stride, float rel,
                     uint8_t *arena, int64_t arena_cap, uint32_t *offsets16,
                     uint32_t *meta, uint8_t *q_out, uint8_t *widths_out,
                     uint8_t *mins_out)
{
    return orc_compress_k(x, B, T, H, D, batch_stride, token_stride, rel, arena, arena_cap,
                          offsets16, meta, q_out, widths_out, mins_out, ORC_K, 0);
}

/*
 * V-median repacking order (Sec. III-B.3, "Faster Repacking with V Median"):
 * inside every block of 64 tokens the token vectors (all kv-heads of a token,
 * quantized V part) are sorted by their median.  Reading of the silent points:
 * the median of the H*D codes of a token is the lower median (the element of
 * rank floor((n-1)/2), n = H*D), equal medians keep their arrival order (stable
 * sort), ascending.  q: quantized V codes [B][T][H][D]; order[b*T + blk*64 + s]
 * = in-block index (0..63) of the token stored at slot s of block blk.  K and V
 * are then packed with their tokens in that order (the permutation statement
 * of Sec. III-B.3 makes any joint order valid).
 */
void orc_v_median_order(const uint8_t *q, int B, int T, int H, int D, uint8_t *order)
{
    int64_t n = (int64_t)H * D;
    int64_t rank = (n - 1) / 2;
    for (int b = 0; b < B; ++b)
        for (int blk = 0; blk < T / ORC_N; ++blk) {
            int key[ORC_N];
            for (int i = 0; i < ORC_N; ++i) {
                const uint8_t *row = q + ((int64_t)b * T + (int64_t)blk * ORC_N + i) * n;
                int64_t hist[256];
                memset(hist, 0, sizeof(hist));
                for (int64_t e = 0; e < n; ++e) hist[row[e]]++;
                int64_t seen = 0;
                int v = 0;
                for (; v < 256; ++v) {
                    seen += hist[v];
                    if (seen > rank) break;
                }
                key[i] = v;
            }
            /* stable insertion of tokens by key */
            uint8_t *o = order + (int64_t)b * T + (int64_t)blk * ORC_N;
            int filled = 0;
            for (int v = 0; v < 256; ++v)
                for (int i = 0; i < ORC_N; ++i)
                    if (key[i] == v) o[filled++] = (uint8_t)i;
        }
}

/*
 * Greedy repacking order (Sec. III-B.3, Algorithm "Greedy Repacking for
 * Bit-Packing"), oracle only.  Inside every block of 64 tokens the token
 * vectors x_i are the quantized K codes followed by the quantized V codes of
 * all kv-heads (one joint order for both tensors).  Packs of 16 are built one
 * after the other: the seed is the remaining vector closest (Euclidean) to the
 * centroid of the remaining vectors; then the vector with the least marginal
 * cost joins until the pack is full.  Reading of the cost: the payload bits of
 * the pack, 16 * sum_d width(max_d - min_d) over all dimensions d (the per-pack
 * metadata is the same for every candidate, so it does not change the choice,
 * and with |P| equal for all candidates the marginal cost is ordered like
 * sum_d width_d(P + j)).  Ties go to the lowest token index.  Output layout as
 * orc_v_median_order.
 */
void orc_greedy_order(const uint8_t *kq, const uint8_t *vq, int B, int T, int H, int D, uint8_t *order)
{
    int64_t n = (int64_t)H * D, dim = 2 * n;
    uint8_t *lo = (uint8_t *)malloc((size_t)dim), *hi = (uint8_t *)malloc((size_t)dim);
    double *cen = (double *)malloc(sizeof(double) * (size_t)dim);
    for (int b = 0; b < B; ++b)
        for (int blk = 0; blk < T / ORC_N; ++blk) {
            const uint8_t *k0 = kq + ((int64_t)b * T + (int64_t)blk * ORC_N) * n;
            const uint8_t *v0 = vq + ((int64_t)b * T + (int64_t)blk * ORC_N) * n;
            uint8_t *o = order + (int64_t)b * T + (int64_t)blk * ORC_N;
            int left[ORC_N], n_left = ORC_N, filled = 0;
            for (int i = 0; i < ORC_N; ++i) left[i] = i;
            while (n_left > 0) {
                /* seed: closest to the centroid of the remaining vectors */
                for (int64_t d = 0; d < dim; ++d) cen[d] = 0.0;
                for (int r = 0; r < n_left; ++r) {
                    const uint8_t *xk = k0 + left[r] * n, *xv = v0 + left[r] * n;
                    for (int64_t d = 0; d < n; ++d) { cen[d] += xk[d]; cen[n + d] += xv[d]; }
                }
                for (int64_t d = 0; d < dim; ++d) cen[d] /= n_left;
                int best = 0;
                double best_d2 = -1.0;
                for (int r = 0; r < n_left; ++r) {
                    const uint8_t *xk = k0 + left[r] * n, *xv = v0 + left[r] * n;
                    double d2 = 0.0;
                    for (int64_t d = 0; d < n; ++d) {
                        double a = xk[d] - cen[d], c = xv[d] - cen[n + d];
                        d2 += a * a + c * c;
                    }
                    if (best_d2 < 0.0 || d2 < best_d2) { best_d2 = d2; best = r; }
                }
                int seed = left[best];
                for (int r = best; r + 1 < n_left; ++r) left[r] = left[r + 1];
                --n_left;
                for (int64_t d = 0; d < n; ++d) {
                    lo[d] = hi[d] = k0[seed * n + d];
                    lo[n + d] = hi[n + d] = v0[seed * n + d];
                }
                o[filled++] = (uint8_t)seed;
                /* fill the pack: least total width after joining */
                for (int size = 1; size < ORC_K && n_left > 0; ++size) {
                    int64_t best_w = -1;
                    best = 0;
                    for (int r = 0; r < n_left; ++r) {
                        const uint8_t *xk = k0 + left[r] * n, *xv = v0 + left[r] * n;
                        int64_t w = 0;
                        for (int64_t d = 0; d < dim; ++d) {
                            int x = d < n ? xk[d] : xv[d - n];
                            int l = x < lo[d] ? x : lo[d], h = x > hi[d] ? x : hi[d];
                            w += orc_width(h - l);
                        }
                        if (best_w < 0 || w < best_w) { best_w = w; best = r; }
                    }
                    int j = left[best];
                    for (int r = best; r + 1 < n_left; ++r) left[r] = left[r + 1];
                    --n_left;
                    for (int64_t d = 0; d < dim; ++d) {
                        int x = d < n ? k0[j * n + d] : v0[j * n + d - n];
                        if (x < lo[d]) lo[d] = (uint8_t)x;
                        if (x > hi[d]) hi[d] = (uint8_t)x;
                    }
                    o[filled++] = (uint8_t)j;
                }
            }
        }
    free(lo);
    free(hi);
    free(cen);
}

/* ------------------------------------------------------------- matvecs -- */

/*
 * scores[b][hq][t] = sm_scale * sum_d q[b][hq][d] * Khat[b][t][hq/G][d]
 * (attention definition, Sec. III-B.3).  Tokens t < n_packed use the decoded
 * codes, tokens n_packed <= t < T are the raw fp16 tail (Sec. III-B.1) and
 * use x itself.  codes/x are [B][T][H][D] contiguous, meta as orc_compress.
 */
void orc_k_scores(const uint8_t *codes, const uint16_t *x, const uint32_t *meta,
                  int B, int T, int n_packed, int H, int Hq, int D,
                  const uint16_t *qvec, double sm_scale, double *scores)
{
    int G = Hq / H;
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < B; ++b)
        for (int hq = 0; hq < Hq; ++hq) {
            int h = hq / G;
            const uint16_t *qv = qvec + ((int64_t)b * Hq + hq) * D;
            for (int t = 0; t < T; ++t) {
                int64_t base = (((int64_t)b * T + t) * H + h) * D;
                uint32_t mt = meta[(int64_t)b * T + t];
                double acc = 0.0;
                for (int d = 0; d < D; ++d) {
                    double kv = t < n_packed
                        ? orc_xhat(codes[base + d], (uint16_t)(mt & 0xFFFFu), (uint16_t)(mt >> 16))
                        : (double)orc_h2f(x[base + d]);
                    acc += (double)orc_h2f(qv[d]) * kv;
                }
                scores[((int64_t)b * Hq + hq) * T + t] = sm_scale * acc;
            }
        }
}

/*
 * out[b][hq][d] = sum_t p[b][hq][t] * Vhat[b][t][hq/G][d], p is fp32 with
 * leading dimension ldp (Sec. III-B.3 definition; same tail rule as above).
 */
void orc_v_out(const uint8_t *codes, const uint16_t *x, const uint32_t *meta,
               int B, int T, int n_packed, int H, int Hq, int D,
               const float *p, int64_t ldp, double *out)
{
    int G = Hq / H;
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < B; ++b)
        for (int hq = 0; hq < Hq; ++hq) {
            int h = hq / G;
            double *o = out + ((int64_t)b * Hq + hq) * D;
            for (int d = 0; d < D; ++d) o[d] = 0.0;
            for (int t = 0; t < T; ++t) {
                int64_t base = (((int64_t)b * T + t) * H + h) * D;
                uint32_t mt = meta[(int64_t)b * T + t];
                double pt = (double)p[((int64_t)b * Hq + hq) * ldp + t];
                for (int d = 0; d < D; ++d) {
                    double vv = t < n_packed
                        ? orc_xhat(codes[base + d], (uint16_t)(mt & 0xFFFFu), (uint16_t)(mt >> 16))
                        : (double)orc_h2f(x[base + d]);
                    o[d] += pt * vv;
                }
            }
        }
}

/* Softmax over the last axis in fp64 (for the end-to-end decode check). */
void orc_softmax(const double *s, int rows, int T, double *p)
{
    for (int r = 0; r < rows; ++r) {
        const double *sr = s + (int64_t)r * T;
        double *pr = p + (int64_t)r * T;
        double mx = sr[0], sum = 0.0;
        for (int t = 1; t < T; ++t) if (sr[t] > mx) mx = sr[t];
        for (int t = 0; t < T; ++t) { pr[t] = exp(sr[t] - mx); sum += pr[t]; }
        for (int t = 0; t < T; ++t) pr[t] /= sum;
    }
}

/*
 * Whole decode attention of one new query (Att(q, K, V) in the permutation
 * statement of Sec. III-B.3), written out from its definition in fp64:
 *   s_t = sm_scale * sum_d q_d Khat[t][d];  p = softmax(s);  out_d = sum_t p_t Vhat[t][d]
 * per batch element and query head, with the decoded caches for t < n_packed
 * and the raw fp16 tail after that.  kcodes/kx/kmeta describe K, vcodes/vx/vmeta V
 * (layouts as orc_k_scores / orc_v_out).  out is [B][Hq][D].
 */
void orc_attention(const uint8_t *kcodes, const uint16_t *kx, const uint32_t *kmeta,
                   const uint8_t *vcodes, const uint16_t *vx, const uint32_t *vmeta,
                   int B, int T, int n_packed, int H, int Hq, int D,
                   const uint16_t *qvec, double sm_scale, double *out)
{
    int G = Hq / H;
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < B; ++b)
        for (int hq = 0; hq < Hq; ++hq) {
            int h = hq / G;
            const uint16_t *qv = qvec + ((int64_t)b * Hq + hq) * D;
            double *s = (double *)malloc(sizeof(double) * (size_t)T);
            double *o = out + ((int64_t)b * Hq + hq) * D;
            double mx = 0.0, sum = 0.0;
            for (int t = 0; t < T; ++t) {
                int64_t base = (((int64_t)b * T + t) * H + h) * D;
                uint32_t mt = kmeta[(int64_t)b * T + t];
                double acc = 0.0;
                for (int d = 0; d < D; ++d) {
                    double kv = t < n_packed
                        ? orc_xhat(kcodes[base + d], (uint16_t)(mt & 0xFFFFu), (uint16_t)(mt >> 16))
                        : (double)orc_h2f(kx[base + d]);
                    acc += (double)orc_h2f(qv[d]) * kv;
                }
                s[t] = sm_scale * acc;
                if (t == 0 || s[t] > mx) mx = s[t];
            }
            for (int t = 0; t < T; ++t) { s[t] = exp(s[t] - mx); sum += s[t]; }
            for (int d = 0; d < D; ++d) o[d] = 0.0;
            for (int t = 0; t < T; ++t) {
                int64_t base = (((int64_t)b * T + t) * H + h) * D;
                uint32_t mt = vmeta[(int64_t)b * T + t];
                double pt = s[t] / sum;
                for (int d = 0; d < D; ++d) {
                    double vv = t < n_packed
                        ? orc_xhat(vcodes[base + d], (uint16_t)(mt & 0xFFFFu), (uint16_t)(mt >> 16))
                        : (double)orc_h2f(vx[base + d]);
                    o[d] += pt * vv;
                }
            }
            free(s);
        }
}

/* Number of OpenMP threads the matvec loops will use (1 without OpenMP). */
#ifdef _OPENMP
#include <omp.h>
int orc_threads(void) { return omp_get_max_threads(); }
void orc_set_threads(int n) { if (n > 0) omp_set_num_threads(n); }
#else
int orc_threads(void) { return 1; }
void orc_set_threads(int n) { (void)n; }
#endif
