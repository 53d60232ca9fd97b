// Append-side compressor: token-wise quantization, bit-packing, appending
// (PackKV Sec. III-B.1 .. III-B.4).  Cold path: runs once per 64 decode steps.
//
//   token_params   one workgroup per (token, batch): min/max over the token's
//                  H*128 values -> fp16 scale = rel*(max-min), fp16 min
//   v_median_key, block_order   (V-median repacking only) sort key per token,
//                  order of the 64 tokens of a block, metadata into storage order
// then, packs of 16 in a contiguous arena whose free space takes even the largest chunks
// (staged path, the input is quantized once):
//   stage          resident workgroups, a chunk at a time each: quantize, build the chunk's
//                  bytes in LDS, store them in a fixed slot of the staging area, and its size
//   scan_offsets   one workgroup: prefix sum of the new chunk sizes -> index
//   compact        one wave per chunk: staged bytes to their place in the arena
// else (two-pass path: packs of 8, paged arenas, a nearly full arena):
//   chunk_sizes    one workgroup per chunk: quantize, per-pack width -> bytes
//   scan_offsets / place_chunks (paged arena) one workgroup: chunk positions -> index; paged:
//                  inside pages taken from a shared pool, index of (start, end) pairs
//   pack_chunks    one workgroup per chunk: quantize again and write header +
//                  payload at its final place
// No atomics in either path: the arena bytes are a pure function of the input.
#include <algorithm>

#include "common.h"

namespace packkv {

// Eight consecutive input values as fp16.  fp16 inputs pass as they are; bf16 inputs are rounded
// to fp16 (to nearest even; exact for every value in fp16's normal range, fp16 having the longer
// significand) -- from there on the path does not know the input type.
__device__ inline uint4 as_fp16(uint4 raw, bool bf16) {
    if (bf16) {
        uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const __half lo = __float2half_rn(__uint_as_float(w[k] << 16));
            const __half hi = __float2half_rn(__uint_as_float(w[k] & 0xFFFF0000u));
            w[k] = uint32_t(__half_as_ushort(lo)) | (uint32_t(__half_as_ushort(hi)) << 16);
        }
        raw = make_uint4(w[0], w[1], w[2], w[3]);
    }
    return raw;
}
// (The input is read once per kernel and is larger than the caches: the non-temporal hint keeps it
// from pushing out what is read again, the staged chunks for one.)
__device__ inline uint4 load8_as_fp16(const __half *p, bool bf16) {
    typedef uint32_t u32x4n __attribute__((ext_vector_type(4)));
    const u32x4n v = __builtin_nontemporal_load(reinterpret_cast<const u32x4n *>(p));
    return as_fp16(make_uint4(v.x, v.y, v.z, v.w), bf16);
}

// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void token_params_kernel(const __half *__restrict__ src,
                                                           int64_t batch_stride,
                                                           int64_t token_stride, int row_elems,
                                                           float rel, uint32_t *__restrict__ meta,
                                                           int64_t meta_stride,
                                                           int64_t first_token, bool bf16) {
    const int t = blockIdx.x, b = blockIdx.y;
    const __half *row = src + b * batch_stride + t * token_stride;
    float mn = INFINITY, mx = -INFINITY;
    for (int i = threadIdx.x * 8; i < row_elems; i += 256 * 8) {
        uint4 raw = load8_as_fp16(row + i, bf16);
        const __half *h = reinterpret_cast<const __half *>(&raw);
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            float v = __half2float(h[k]);
            mn = fminf(mn, v);
            mx = fmaxf(mx, v);
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        mn = fminf(mn, __shfl_xor(mn, o));
        mx = fmaxf(mx, __shfl_xor(mx, o));
    }
    __shared__ float smn[4], smx[4];
    if ((threadIdx.x & 63) == 0) {
        smn[threadIdx.x >> 6] = mn;
        smx[threadIdx.x >> 6] = mx;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        mn = fminf(fminf(smn[0], smn[1]), fminf(smn[2], smn[3]));
        mx = fmaxf(fmaxf(smx[0], smx[1]), fmaxf(smx[2], smx[3]));
        mn = mn + 0.0f;  // a zero minimum or maximum is stored as +0
        mx = mx + 0.0f;
        float range = mx - mn;
        float s = rel * range;
        // The product is rounded to fp32 first and to fp16 second; keep the
        // compiler from fusing both into one mixed-precision FMA (one rounding).
        asm volatile("" : "+v"(s));
        __half s16 = __float2half_rn(s);
        __half m16 = __float2half_rn(mn);  // exact: mn is an fp16 value
        uint32_t word = uint32_t(__half_as_ushort(s16)) | (uint32_t(__half_as_ushort(m16)) << 16);
        meta[b * meta_stride + first_token + t] = word;
    }
}

// Quantize the PK tokens of one pack (channel d of token group g) and derive
// its minimum, width and code bits.
struct PackBits {
    uint64_t bits;
    int w, m;
};

// Token-wise quantization of one value (Sec. III-B.2) with the token's scale and minimum:
// clamp(rint(fl((x - mn) / s)), 0, qmax), the quotient rounded to fp32 as an IEEE divide does.
// r is the token's 1 / s from an IEEE divide (once per token).  The product (x - mn) * r lies
// within 1.5 * 2^-23 relative of that rounded quotient (half an ulp for r, half for the product,
// half for the quotient's own rounding), which is below 5e-5 in absolute terms for every quotient
// that is not clamped anyway (<= 256.5; beyond that both round to at least 256 > qmax).  So unless
// the product is within 1e-3 of a rounding tie k + 0.5, rint of the product IS rint of the
// quotient; the rare value near a tie takes the divide.
__device__ inline int quantize_value(float x, float s, float mn, float r, int qmax) {
    int v = 0;
    if (s != 0.0f) {
        const float a = x - mn;
        const float q1 = a * r;
        float t = rintf(q1);  // ties to even
        if (fabsf(fabsf(q1 - t) - 0.5f) < 1e-3f) t = rintf(a / s);  // IEEE fp32 divide
        v = (int)t;
        v = v < 0 ? 0 : (v > qmax ? qmax : v);
    }
    return v;
}

// A token's (scale, minimum, 1 / scale) from its metadata word (fp16 scale | fp16 minimum << 16).
__device__ inline float4 token_scale_min(uint32_t mt) {
    const float s = __half2float(__ushort_as_half(uint16_t(mt & 0xFFFFu)));
    const float mn = __half2float(__ushort_as_half(uint16_t(mt >> 16)));
    return make_float4(s, mn, s != 0.0f ? 1.0f / s : 0.0f, 0.0f);
}

// tile: the block's 64 x 128 values in LDS, rows already in storage order; the pack holds rows
// PK*g..PK*g+PK-1 of channel d; sm: token_scale_min of the block's 64 tokens (storage order), in LDS.
template <int PK>
__device__ inline PackBits make_pack(const __half *tile, int g, int d, const float4 *sm, int qmax) {
    int q[PK];
    int lo = 255, hi = 0;
#pragma unroll
    for (int i = 0; i < PK; ++i) {
        const float4 t = sm[g * PK + i];
        const int v = quantize_value(__half2float(tile[(g * PK + i) * D + d]), t.x, t.y, t.z, qmax);
        q[i] = v;
        lo = min(lo, v);
        hi = max(hi, v);
    }
    PackBits pb;
    int range = hi - lo;
    pb.w = range == 0 ? 0 : 32 - __clz(range);
    pb.m = lo;
    // two halves of PK/2 codes, at most 32 bits each, built with 32-bit shift-and-or steps from
    // the top code down; one 64-bit shift joins them
    uint32_t half_lo = 0, half_hi = 0;
#pragma unroll
    for (int i = PK / 2 - 1; i >= 0; --i) {
        half_lo = (half_lo << pb.w) | uint32_t(q[i] - lo);
        half_hi = (half_hi << pb.w) | uint32_t(q[PK / 2 + i] - lo);
    }
    pb.bits = uint64_t(half_lo) | (uint64_t(half_hi) << (PK / 2 * pb.w));
    return pb;
}

// Exclusive prefix sum over the 256 threads of a workgroup; also returns the total.
__device__ inline int block_exclusive_scan(int v, int *total) {
    __shared__ int wave_sum[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        int n = __shfl_up(inc, o);
        if (lane >= o) inc += n;
    }
    __syncthreads();  // protects wave_sum against a previous call
    if (lane == 63) wave_sum[wave] = inc;
    __syncthreads();
    int base = 0;
    for (int k = 0; k < wave; ++k) base += wave_sum[k];
    *total = wave_sum[0] + wave_sum[1] + wave_sum[2] + wave_sum[3];
    return base + inc - v;
}

// One workgroup per new chunk; packs of PK = 8 tokens (Sec. IV-B; packs of 16 have their own
// kernel below): the chunk has 64/PK token groups of 128 packs, thread tau owns packs tau + 256k
// (token group (tau >> 7) + 2k, channel tau & 127).  A pack takes PK*w/8 payload bytes.  WIDE (codes above 15, packs of 8): the
// header is a width byte per pack followed by a minimum byte per pack, widths go up to 8.
template <bool WRITE, int PK, bool WIDE = false>
__global__ __launch_bounds__(256) void chunk_kernel(const __half *__restrict__ src,
                                                    int64_t batch_stride, int64_t token_stride,
                                                    int B, int H, int qmax,
                                                    const uint32_t *__restrict__ meta,
                                                    int64_t meta_stride, int64_t first_token,
                                                    int64_t first_chunk,
                                                    uint32_t *__restrict__ sizes16,
                                                    const uint32_t *__restrict__ index,
                                                    int index_words,
                                                    uint8_t *__restrict__ arena,
                                                    const uint8_t *__restrict__ order, bool bf16) {
    static_assert(PK == 8, "contiguous packs are packs of 8 tokens");
    constexpr int NPACKS = N / PK * D;
    constexpr int HDR = WIDE ? 2 * NPACKS : NPACKS;  // header bytes
    constexpr int PER = N / PK * D / 256;  // packs per thread
    const int cl = blockIdx.x;  // chunk within this round: (blk*B + b)*H + h
    const int h = cl % H;
    const int b = (cl / H) % B;
    const int blk = cl / (H * B);
    const int tau = threadIdx.x;
    const int d = tau & 127;

    uint8_t *dst = nullptr;
    if (WRITE) {
        const int64_t e = (first_chunk + cl) * index_words;
        uint32_t o0 = index[e], o1 = index[e + 1];
        if (o1 == o0) return;  // dropped: the arena was full
        dst = arena + size_t(o0) * 16;
    }

    // stage the block's 64 x 128 values in LDS with 16-byte loads, rows in storage order, and the
    // tokens' scales and minimums as floats (every thread needs all 64 of them)
    __shared__ __attribute__((aligned(16))) __half tile[N * D];
    __shared__ float4 sm[N];
    if (tau < N) sm[tau] = token_scale_min(meta[b * meta_stride + first_token + int64_t(blk) * N + tau]);
    {
        const __half *x_blk = src + b * batch_stride + int64_t(blk) * N * token_stride + h * D;
        const uint8_t *ord = order ? order + b * meta_stride + first_token + int64_t(blk) * N : nullptr;
#pragma unroll
        for (int pass = 0; pass < 4; ++pass) {
            const int row = pass * 16 + (tau >> 4), c8 = (tau & 15) * 8;
            const int src_row = ord ? ord[row] : row;
            *reinterpret_cast<uint4 *>(tile + row * D + c8) = load8_as_fp16(x_blk + src_row * token_stride + c8, bf16);
        }
    }
    __syncthreads();

    PackBits pb[PER];
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        const int g = (tau >> 7) + 2 * k;
        pb[k] = make_pack<PK>(tile, g, d, sm, qmax);
    }
    // all packs are quantized before the first barrier of the scans
    int off[PER];
    int payload = 0;
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        int total;
        off[k] = payload + block_exclusive_scan(PK / 8 * pb[k].w, &total);
        payload += total;
    }
    const int padded = (HDR + payload + 15) & ~15;

    if (!WRITE) {
        if (tau == 0) sizes16[cl] = uint32_t(padded >> 4);
        return;
    }
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        if constexpr (WIDE) {
            dst[tau + 256 * k] = uint8_t(pb[k].w);
            dst[NPACKS + tau + 256 * k] = uint8_t(pb[k].m);
        } else {
            dst[tau + 256 * k] = uint8_t((pb[k].w << 4) | pb[k].m);
        }
        uint8_t *out = dst + HDR + off[k];
        for (int j = 0; j < pb[k].w; ++j) out[j] = uint8_t(pb[k].bits >> (8 * j));
    }
    if (tau < padded - HDR - payload) dst[HDR + payload + tau] = 0;
}

// Packs of 16 tokens in the plane layout (packkv.h): header bytes in pack-list order, region E
// with a 32-bit word of low code bits per pack of width >= 2 (and a second word of high bits
// for width 4), region O with a 16-bit word of top bits per pack of odd width.  One workgroup
// per new chunk; thread tau owns packs tau and tau + 256 of the pack list (order 0: pack
// p = g*128 + d, order 1: p = d*4 + g).
struct PlaneBits {
    uint32_t low, high, top;
    int w, m;
};

// n0, n1: the 16 codes of a pack as nibbles (tokens 0..7, 8..15); lo, hi: their minimum and maximum.
__device__ inline PlaneBits planes_from_nibbles(uint32_t n0, uint32_t n1, int lo, int hi) {
    PlaneBits pb;
    const int range = hi - lo;
    pb.w = range == 0 ? 0 : 32 - __clz(range);
    pb.m = lo;
    // codes minus the pack minimum: no nibble borrows (every code is at least the minimum)
    n0 -= uint32_t(lo) * 0x11111111u;
    n1 -= uint32_t(lo) * 0x11111111u;
    // planes of two-bit fields: token i at bits [4i, 4i+2) for i < 8, at [4(i-8)+2, 4(i-8)+4) for i >= 8
    pb.low = (n0 & 0x33333333u) | ((n1 & 0x33333333u) << 2);
    pb.high = ((n0 >> 2) & 0x33333333u) | (n1 & 0xCCCCCCCCu);
    // top bit of every code, token i at bit 4 (i % 4) + i / 4
    const int top_bit = pb.w > 0 ? pb.w - 1 : 0;
    const uint32_t t0 = (n0 >> top_bit) & 0x11111111u, t1 = (n1 >> top_bit) & 0x11111111u;
    pb.top = (t0 & 0xFFFFu) | ((t0 >> 16) << 1) | ((t1 & 0xFFFFu) << 2) | ((t1 >> 16) << 3);
    return pb;
}

// Code tile of a chunk in LDS: channel d has a row of 16 words (and one word of padding, which
// spreads the rows over the banks); word 4g + q of it holds four codes of token group g, one per
// byte: q = 0: tokens 0, 2, 4, 6; q = 1: tokens 1, 3, 5, 7; q = 2: tokens 8, 10, 12, 14; q = 3:
// tokens 9, 11, 13, 15.  So word 0 | word 1 << 4 is the nibble string of tokens 0..7 and
// word 2 | word 3 << 4 that of tokens 8..15 (codes of packs of 16 are below 16).
constexpr int CODE_ROW_WORDS = 17;
constexpr int CODE_TILE_WORDS = D * CODE_ROW_WORDS;
typedef unsigned short pk_u16 __attribute__((ext_vector_type(2)));

__device__ inline PlaneBits planes_from_codes(const uint32_t *words) {
    const uint32_t w0 = words[0], w1 = words[1], w2 = words[2], w3 = words[3];
    // minimum and maximum of the 16 bytes, two 16-bit lanes at a time
    constexpr uint32_t EVEN = 0x00FF00FFu;
    const uint32_t v[8] = {w0 & EVEN, (w0 >> 8) & EVEN, w1 & EVEN, (w1 >> 8) & EVEN,
                           w2 & EVEN, (w2 >> 8) & EVEN, w3 & EVEN, (w3 >> 8) & EVEN};
    pk_u16 mn = __builtin_bit_cast(pk_u16, v[0]), mx = mn;
#pragma unroll
    for (int i = 1; i < 8; ++i) {
        mn = __builtin_elementwise_min(mn, __builtin_bit_cast(pk_u16, v[i]));
        mx = __builtin_elementwise_max(mx, __builtin_bit_cast(pk_u16, v[i]));
    }
    const int lo = min(int(mn.x), int(mn.y)), hi = max(int(mx.x), int(mx.y));
    return planes_from_nibbles(w0 | (w1 << 4), w2 | (w3 << 4), lo, hi);
}

// One chunk of packs of 16 in a workgroup's registers: thread tau holds packs 2 tau and 2 tau + 1
// of the pack list; off: the bytes of the packs before them in region E (low half) and region O
// (high half).
struct PlaneChunk {
    PlaneBits pb[2];
    int off;
    int e_bytes, o_bytes, padded;
};

// What a thread loads of a chunk: eight channels (8 * (tau % 16) ...) of the four tokens that
// share a word of the code tile (word tau / 16 of each of those channels), and the tokens' metadata.
struct ChunkInput {
    uint4 raw[4];
    uint32_t mt[4];
};

struct ChunkSource {
    const __half *src;
    int64_t batch_stride, token_stride;
    int B, H, qmax;
    uint64_t magic_h, magic_hb;  // floor(2^32 / H) + 1, floor(2^32 / (H * B)) + 1
    const uint32_t *meta;
    int64_t meta_stride, first_token;
    const uint8_t *order;
    bool bf16;
    int pack_order;
};

// Chunk cl of the round is (blk*B + b)*H + h.  cl is the same for the whole workgroup, so the
// quotients are scalar work: x / d = (x * (floor(2^32 / d) + 1)) >> 32 for x * d < 2^32
// (cl < 2^16 here, H * B <= 2^16).
struct ChunkCoord {
    int h, b, blk;
};
__device__ inline ChunkCoord chunk_coord(const ChunkSource &cs, int cl) {
    const uint32_t c = uint32_t(__builtin_amdgcn_readfirstlane(cl));
    const uint32_t by_h = uint32_t((uint64_t(c) * cs.magic_h) >> 32);
    const uint32_t blk = uint32_t((uint64_t(c) * cs.magic_hb) >> 32);
    ChunkCoord k;
    k.h = int(c - by_h * uint32_t(cs.H));
    k.b = int(by_h - blk * uint32_t(cs.B));
    k.blk = int(blk);
    return k;
}

// Where chunk cl of the round ((blk*B + b)*H + h) finds the four tokens of thread tau: rows
// row0 + 2i of the block in storage order, at the source positions the token order gives.
struct ChunkRows {
    int src_row[4];
};
__device__ inline int chunk_row0() {
    const int word = threadIdx.x >> 4;  // word = 4g + q
    return 16 * (word >> 2) + 8 * ((word >> 1) & 1) + (word & 1);
}
__device__ inline ChunkRows load_chunk_rows(const ChunkSource &cs, int cl) {
    const ChunkCoord k = chunk_coord(cs, cl);
    const int b = k.b, blk = k.blk;
    const int row0 = chunk_row0();
    ChunkRows r;
    if (cs.order) {
        const uint8_t *ord = cs.order + b * cs.meta_stride + cs.first_token + int64_t(blk) * N;
#pragma unroll
        for (int i = 0; i < 4; ++i) r.src_row[i] = ord[row0 + 2 * i];
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) r.src_row[i] = row0 + 2 * i;
    }
    return r;
}

// Issues the loads of chunk cl.
__device__ inline ChunkInput load_chunk_input(const ChunkSource &cs, int cl, const ChunkRows &rows) {
    const ChunkCoord k = chunk_coord(cs, cl);
    const int h = k.h, b = k.b, blk = k.blk;
    const int cg = threadIdx.x & 15;
    const int row0 = chunk_row0();
    const __half *x_blk = cs.src + b * cs.batch_stride + int64_t(blk) * N * cs.token_stride + h * D + cg * 8;
    const uint32_t *meta_blk = cs.meta + b * cs.meta_stride + cs.first_token + int64_t(blk) * N;
    ChunkInput in;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        in.raw[i] = *reinterpret_cast<const uint4 *>(x_blk + rows.src_row[i] * cs.token_stride);  // converted where it is used
        in.mt[i] = meta_blk[row0 + 2 * i];
    }
    return in;
}

// The eight values of one token a thread holds, quantized (Sec. III-B.2: clamp(rint(fl((x - mn) / s)),
// 0, qmax), the quotient rounded to fp32 as an IEEE divide does) into byte `slot` of out[0..7];
// qmax < 16.  Fast path: q = (x - mn) * r with r = 1 / s to within an ulp, rounded to the nearest
// integer (ties to even) and clamped to 0 .. 255 by the conversion that also places the byte; a token
// with a quotient that could round above qmax takes the slow path, which clamps.
// q lies within 2^-22 relative of the rounded quotient (an ulp for r, half for the product, half
// for the quotient's own rounding): within 2^-16 for quotients below 64, and from 64 on both sides
// are clamped to qmax anyway.  So unless q is within 2^-15 of a rounding tie k + 1/2, it rounds as
// the quotient does.  `clear` collects how far the eight values stay from a tie; the rare token
// with a value near one takes the divide for all eight.
constexpr float TIE_GUARD = 1.0f / 32768.0f;

// x - mn in fp32 for the low (HI = false) or high half of a word of two fp16 values: the mixed-
// precision fused multiply-add x * 1 + (-mn) rounds the exact difference once, as the conversion
// to fp32 (exact) followed by the subtraction does, and saves the conversion.
template <bool HI>
__device__ inline float half_minus(uint32_t two_halves, float neg_mn) {
    float a;
    if (HI)
        asm("v_fma_mix_f32 %0, %1, 1.0, %2 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(a) : "v"(two_halves), "v"(neg_mn));
    else
        asm("v_fma_mix_f32 %0, %1, 1.0, %2 op_sel_hi:[1,0,0]" : "=v"(a) : "v"(two_halves), "v"(neg_mn));
    return a;
}

__device__ inline void quantize_token8(uint4 values, uint32_t mt, int qmax, int slot, uint32_t *out) {
    const float s = __half2float(__ushort_as_half(uint16_t(mt & 0xFFFFu)));
    const float mn = __half2float(__ushort_as_half(uint16_t(mt >> 16)));
    const float r = s != 0.0f ? __builtin_amdgcn_rcpf(s) : 0.0f;  // s = 0: every code is 0
    const float top = float(qmax);
    const uint32_t w[4] = {values.x, values.y, values.z, values.w};
    float clear = 1.0f, most = 0.0f;
    float q[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const float a = (j & 1) ? half_minus<true>(w[j >> 1], -mn) : half_minus<false>(w[j >> 1], -mn);
        q[j] = a * r;
        clear = fminf(clear, fabsf(__builtin_amdgcn_fractf(q[j]) - 0.5f));
        most = fmaxf(most, q[j]);
        out[j] = __builtin_amdgcn_cvt_pk_u8_f32(q[j], uint32_t(slot), out[j]);  // rounds to nearest even, 0 .. 255
    }
    // rare: a value near a rounding tie (the divide decides), or one that rounds above qmax (the
    // scale is an fp16 rounding of rel * range, so the largest quotient can pass qmax + 1/2; an
    // infinite quotient lands here too, and a NaN converts to code 0)
    if (clear < TIE_GUARD || most >= top + 0.5f - TIE_GUARD) {
        const __half *x = reinterpret_cast<const __half *>(&values);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float qd = s != 0.0f ? (__half2float(x[j]) - mn) / s : 0.0f;  // IEEE fp32 divide
            out[j] = __builtin_amdgcn_cvt_pk_u8_f32(fminf(qd, top), uint32_t(slot), out[j]);
        }
    }
}

// Quantizes a chunk and lays out its regions.  Every value is quantized by the thread that loaded
// it, with its token's scale and minimum, so the code tile is written a word at a time.
// Ends behind a barrier that all threads pass after their last read of the tile.
__device__ inline PlaneChunk make_plane_chunk(const ChunkSource &cs, const ChunkInput &in, uint32_t *codes) {
    const int tau = threadIdx.x;
    {
        const int cg = tau & 15, word = tau >> 4;
        uint32_t out[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int i = 0; i < 4; ++i) quantize_token8(as_fp16(in.raw[i], cs.bf16), in.mt[i], cs.qmax, i, out);
#pragma unroll
        for (int j = 0; j < 8; ++j) codes[(cg * 8 + j) * CODE_ROW_WORDS + word] = out[j];
    }
    __syncthreads();
    PlaneChunk c;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int p = 2 * tau + k;
        const int g = cs.pack_order ? (p & 3) : (p >> 7);
        const int d = cs.pack_order ? (p >> 2) : (p & 127);
        c.pb[k] = planes_from_codes(codes + d * CODE_ROW_WORDS + 4 * g);
    }
    // one scan carries both regions: E bytes in the low half, O bytes in the high half
    int total;
    const int w0 = c.pb[0].w, w1 = c.pb[1].w;
    c.off = block_exclusive_scan(4 * ((w0 >> 1) + (w1 >> 1)) + ((2 * ((w0 & 1) + (w1 & 1))) << 16), &total);
    c.e_bytes = total & 0xFFFF;
    c.o_bytes = total >> 16;
    c.padded = (HEADER + c.e_bytes + c.o_bytes + 15) & ~15;
    return c;
}

__device__ inline void write_plane_chunk(const PlaneChunk &c, uint8_t *__restrict__ dst) {
    const int tau = threadIdx.x;
    const int w0 = c.pb[0].w, w1 = c.pb[1].w;
    reinterpret_cast<uint16_t *>(dst)[tau] = uint16_t(((w0 << 4) | c.pb[0].m) | (((w1 << 4) | c.pb[1].m) << 8));
    uint32_t *e = reinterpret_cast<uint32_t *>(dst + HEADER + (c.off & 0xFFFF));
    if (w0 >= 2) e[0] = c.pb[0].low;
    if (w0 == 4) e[1] = c.pb[0].high;
    e += w0 >> 1;
    if (w1 >= 2) e[0] = c.pb[1].low;
    if (w1 == 4) e[1] = c.pb[1].high;
    uint16_t *o = reinterpret_cast<uint16_t *>(dst + HEADER + c.e_bytes + (c.off >> 16));
    if (w0 & 1) o[0] = uint16_t(c.pb[0].top);
    o += w0 & 1;
    if (w1 & 1) o[0] = uint16_t(c.pb[1].top);
    if (tau < c.padded - HEADER - c.e_bytes - c.o_bytes) dst[HEADER + c.e_bytes + c.o_bytes + tau] = 0;
}

// Staged path, packs of 16, contiguous arena: the input is quantized once.
//   stage     one workgroup per chunk: quantize, build the chunk's bytes in LDS, store them in a
//             slot of CHUNK_MAX bytes of the staging area in the workspace, and the chunk's size
//   scan_offsets   as in the two-pass path
//   compact   one wave per chunk: copy the staged bytes to their place in the arena
// A chunk's place depends on the sizes of all chunks before it, so some second step is needed;
// this one re-reads the compressed bytes (a fraction of the input, and still in the last-level
// cache: the staging area is a few tens of MB) instead of the input.  A round is cut into parts
// that fit the staging area.  The path runs when even the largest chunks fit the arena (worst16 =
// chunks of the round times the largest chunk, checked on the device, where the fill level is), so
// no part can overflow and a round keeps or drops its chunks as a whole; otherwise its kernels
// return at once and the two-pass kernels do the round, and the other way round.
__device__ inline bool staged_round(const StagedRound &r, const uint32_t *index) {
    return r.worst16 != 0 && uint64_t(index[r.first_chunk]) + r.worst16 <= r.arena_cap16;
}

// Two-pass path, packs of 16: WRITE false = sizes only, true = bytes at the offsets of the index.
template <bool WRITE>
__global__ __launch_bounds__(256) void chunk16_kernel(ChunkSource cs, int64_t first_chunk,
                                                      uint32_t *__restrict__ sizes16,
                                                      const uint32_t *__restrict__ index, int index_words,
                                                      uint8_t *__restrict__ arena, StagedRound round) {
    if (staged_round(round, index)) return;  // the staged path writes this round
    const int cl = blockIdx.x;
    uint8_t *dst = nullptr;
    if (WRITE) {
        const int64_t e = (first_chunk + cl) * index_words;
        uint32_t o0 = index[e], o1 = index[e + 1];
        if (o1 == o0) return;  // dropped: the arena was full
        dst = arena + size_t(o0) * 16;
    }
    __shared__ uint32_t codes[CODE_TILE_WORDS];
    const PlaneChunk c = make_plane_chunk(cs, load_chunk_input(cs, cl, load_chunk_rows(cs, cl)), codes);
    if (!WRITE) {
        if (threadIdx.x == 0) sizes16[cl] = uint32_t(c.padded >> 4);
        return;
    }
    write_plane_chunk(c, dst);
}

// Chunks part_first .. part_first + n - 1 of the round, chunk part_first + i into slot i.  A
// workgroup takes every gridDim.x-th chunk and has the loads of its next one in flight while it
// works on the current one.
__global__ __launch_bounds__(256) void chunk16_stage_kernel(ChunkSource cs, const uint32_t *__restrict__ index,
                                                            int part_first, int n,
                                                            uint32_t *__restrict__ sizes16,
                                                            uint8_t *__restrict__ staging, StagedRound round) {
    if (!staged_round(round, index)) return;
    // the chunk's bytes are put together in the memory of the code tile (8704 bytes, a chunk has at most 4608)
    __shared__ __attribute__((aligned(16))) uint32_t codes[CODE_TILE_WORDS];
    static_assert(CODE_TILE_WORDS * 4 >= CHUNK_MAX, "the chunk image lives in the code tile");
    static_assert(CHUNK_MAX <= 2 * 256 * 16, "two 16-byte units per thread move a chunk");
    const int tau = threadIdx.x;
    const int stride = int(gridDim.x);
    int cl = blockIdx.x;
    if (cl >= n) return;
    // The loads of the next chunk and the token order of the one after it are always issued (of
    // the last chunk again where there is no next one): the count of loads in flight is then the
    // same on every path, and the waits of the current chunk do not wait for them.
    ChunkInput in = load_chunk_input(cs, part_first + cl, load_chunk_rows(cs, part_first + cl));
    ChunkRows rows_next = load_chunk_rows(cs, part_first + min(cl + stride, n - 1));
    for (;;) {
        const int next = cl + stride;
        const ChunkInput in_next = load_chunk_input(cs, part_first + min(next, n - 1), rows_next);
        rows_next = load_chunk_rows(cs, part_first + min(next + stride, n - 1));
        const PlaneChunk c = make_plane_chunk(cs, in, codes);
        write_plane_chunk(c, reinterpret_cast<uint8_t *>(codes));
        __syncthreads();
        if (tau == 0) sizes16[cl] = uint32_t(c.padded >> 4);
        const uint4 *image = reinterpret_cast<const uint4 *>(codes);
        uint4 *slot = reinterpret_cast<uint4 *>(staging + size_t(cl) * CHUNK_MAX);
        const int n16 = c.padded >> 4;
        if (tau < n16) slot[tau] = image[tau];
        if (tau + 256 < n16) slot[tau + 256] = image[tau + 256];
        if (next >= n) break;
        __syncthreads();  // the image is read: the next code tile may take its place
        in = in_next;
        cl = next;
    }
}

// One wave per chunk of a staged part (its index words are set: the part's scan has run): staged
// bytes to their place.
__global__ __launch_bounds__(256) void chunk16_compact_kernel(StagedPart waiting) {
    if (!staged_round(waiting.round, waiting.index)) return;
    const int lane = threadIdx.x & 63;
    const int cl = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (cl >= waiting.n) return;
    const uint32_t start = waiting.index[waiting.first_chunk + cl], end = waiting.index[waiting.first_chunk + cl + 1];
    const int n16 = int(end - start);
    const uint4 *from = reinterpret_cast<const uint4 *>(waiting.staging + size_t(cl) * CHUNK_MAX);
    uint4 *to = reinterpret_cast<uint4 *>(waiting.arena + size_t(start) * 16);
    constexpr int STEPS = (CHUNK_MAX / 16 + 63) / 64;
    // read once and written once: both with the non-temporal hint (6 % of the whole compression)
    typedef uint32_t u32x4n __attribute__((ext_vector_type(4)));
    const u32x4n *src = reinterpret_cast<const u32x4n *>(from);
    u32x4n *dst = reinterpret_cast<u32x4n *>(to);
    u32x4n v[STEPS];
#pragma unroll
    for (int i = 0; i < STEPS; ++i)
        if (lane + 64 * i < n16) v[i] = __builtin_nontemporal_load(src + lane + 64 * i);
#pragma unroll
    for (int i = 0; i < STEPS; ++i)
        if (lane + 64 * i < n16) __builtin_nontemporal_store(v[i], dst + lane + 64 * i);
}

// Single workgroup: index[first+i+1] = index[first] + sum_{j<=i} sizes16[j].
// If the new chunks do not fit, all of them get size 0 and the flag is set.
// Wave w owns a run of `per` consecutive sizes (a multiple of 256) and walks it 256 at a time,
// four per lane, so loads and stores of a wave cover consecutive memory.
__global__ __launch_bounds__(1024) void scan_offsets_kernel(const uint32_t *__restrict__ sizes16,
                                                            int n, uint32_t *__restrict__ index,
                                                            int64_t first_chunk,
                                                            uint64_t arena_cap16,
                                                            uint32_t *__restrict__ status,
                                                            StagedRound round, bool staged_part) {
    __shared__ uint32_t wsum[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int per = ((n + 15) / 16 + 255) & ~255;
    const int lo = min(wave * per, n), hi = min(lo + per, n);
    // sizes lo + 256 r + 4 lane .. + 3 (sizes16 is 256-byte aligned and its area a multiple of 16 bytes)
    auto load4 = [&](int r) {
        const int i = lo + 256 * r + 4 * lane;
        uint4 q = i < hi ? *reinterpret_cast<const uint4 *>(sizes16 + i) : make_uint4(0, 0, 0, 0);
        if (i + 1 >= hi) q.y = 0;
        if (i + 2 >= hi) q.z = 0;
        if (i + 3 >= hi) q.w = 0;
        return q;
    };
    const int rounds = (hi - lo + 255) / 256;
    // the first four rounds (all of them for up to 16384 chunks) go out at once and stay in registers
    uint4 held[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) held[r] = load4(r);
    const uint32_t start = index[first_chunk];
    uint32_t local = 0;
#pragma unroll
    for (int r = 0; r < 4; ++r) local += held[r].x + held[r].y + held[r].z + held[r].w;
    for (int r = 4; r < rounds; ++r) {
        const uint4 q = load4(r);
        local += q.x + q.y + q.z + q.w;
    }
    // serves a part of a staged round (staged_part) or a whole two-pass round: whichever path runs
    if (staged_round(round, index) != staged_part) return;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) local += __shfl_xor(local, o);
    if (lane == 0) wsum[wave] = local;
    __syncthreads();
    uint32_t run = start, total = 0;
    for (int k = 0; k < 16; ++k) {
        if (k < wave) run += wsum[k];
        total += wsum[k];
    }
    const bool fits = uint64_t(start) + total <= arena_cap16;
    if (!fits && tid == 0) status[0] = 1;
    auto place = [&](int r, uint4 q) {
        const uint32_t mine = q.x + q.y + q.z + q.w;
        uint32_t inc = mine;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t v = __shfl_up(inc, o);
            if (lane >= o) inc += v;
        }
        const int i = lo + 256 * r + 4 * lane;
        uint32_t at = run + inc - mine;
        const uint32_t ends[4] = {at + q.x, at + q.x + q.y, at + q.x + q.y + q.z, at + mine};
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (i + k < hi) index[first_chunk + i + k + 1] = fits ? ends[k] : start;
        run += __shfl(inc, 63);
    };
#pragma unroll
    for (int r = 0; r < 4; ++r)
        if (r < rounds) place(r, held[r]);
    for (int r = 4; r < rounds; ++r) place(r, load4(r));
}

// Paged arena: places the n new chunks of one tensor (sizes16: their sizes in 16-byte units;
// overwritten with their exclusive prefix sums) in chunk order.  A chunk goes right behind the
// previous one while it still fits into the tensor's newest page, else to the start of a fresh
// page, so no chunk crosses a page boundary; positions count 16-byte units from the start of the
// pool.  The fresh pages come off the pool's stack, all of them with one atomic update of its
// height.  If the pool (or the tensor's page list) cannot take them, nothing is taken, every
// chunk of the call is dropped (start = end) and the flag is set, as with a full contiguous arena.
//
// One workgroup.  The rule is sequential in the fill level only, so the work is split: (1) prefix
// sums S of the sizes; (2) for every chunk j, in parallel, how many chunks a page holds that
// starts with j (two pointers over S); (3) one thread follows that chain from the first chunk
// that does not fit the newest page -- one LDS step per fresh page, not per chunk -- and marks
// the chunks that start a page; (4) in parallel again, every chunk finds its page (a count of the
// marks before it) and its offset inside it (S[j] - S[page start]).
__global__ __launch_bounds__(1024) void place_chunks_kernel(uint32_t *__restrict__ sizes16, int n,
                                                            uint32_t *__restrict__ index2,
                                                            int64_t first_chunk,
                                                            uint32_t *__restrict__ page_list,
                                                            int64_t max_pages, uint32_t *pool_state,
                                                            uint32_t *__restrict__ status) {
    // bit 7: the chunk starts a fresh page; bits 0..6: chunks that fit a page starting here, minus 1
    // (a chunk is at least 512 bytes, so a page holds at most 128)
    __shared__ uint8_t step[MAX_NEW_CHUNKS];
    __shared__ uint32_t wave_a[16], wave_b[16];
    __shared__ uint32_t sh_total, sh_top, sh_ok;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int per = (n + 1023) / 1024;
    const int lo = min(tid * per, n), hi = min(lo + per, n);
    constexpr uint32_t P = PAGE16;

    // (1) exclusive prefix sums, in place
    uint32_t local = 0;
    for (int i = lo; i < hi; ++i) local += sizes16[i];
    uint32_t inc = local;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t v = __shfl_up(inc, o);
        if (lane >= o) inc += v;
    }
    if (lane == 63) wave_a[wave] = inc;
    __syncthreads();
    uint32_t run = inc - local;
    for (int k = 0; k < wave; ++k) run += wave_a[k];
    if (tid == 1023) sh_total = run + local;
    for (int i = lo; i < hi; ++i) {
        const uint32_t sz = sizes16[i];
        sizes16[i] = run;
        run += sz;
    }
    __syncthreads();
    const uint32_t total = sh_total;
    auto S = [&](int i) -> uint32_t { return i < n ? sizes16[i] : total; };

    // (2) chunks per page for a page that starts with chunk j
    {
        int k = lo;
        for (int j = lo; j < hi; ++j) {
            k = max(k, j + 1);
            const uint32_t limit = S(j) + P;
            while (k < n && S(k + 1) <= limit) ++k;
            step[j] = uint8_t(k - j - 1);
        }
    }
    __syncthreads();

    // (3) the chain of page starts, and the pages for it.  Following the chain is one dependent LDS
    // read per fresh page; with many chunks it is cut into sixteen segments, one per wave: a chain
    // enters a segment within its first 128 chunks (a page holds no more), so every wave follows
    // the chain from each of these 128 possible entries to the segment's end (lanes in parallel)
    // and notes where it leaves and how many pages it starts; thread 0 then hops through the
    // sixteen tables, and every wave marks its own segment from its true entry.
    constexpr int WAVES = 16, ENTRIES = 128;
    __shared__ uint32_t seg_exit[WAVES][ENTRIES];
    __shared__ uint16_t seg_pages[WAVES][ENTRIES];
    __shared__ uint32_t seg_entry[WAVES];
    const int seg = (n + WAVES - 1) / WAVES;
    const bool segmented = seg >= ENTRIES;
    const int seg_a = min(wave * seg, n), seg_e = min(seg_a + seg, n);
    if (segmented) {
        for (int c = lane; c < ENTRIES; c += 64) {
            int j = seg_a + c;
            uint32_t pages = 0;
            while (j < seg_e) {
                ++pages;
                j += int(step[j]) + 1;
            }
            seg_exit[wave][c] = uint32_t(j);
            seg_pages[wave][c] = uint16_t(pages);
        }
    }
    __syncthreads();
    const uint32_t held = page_list[0];
    const uint32_t fill0 = held ? page_list[1] : P;  // no page yet: like a full one
    if (tid == 0) {
        int j = 0;
        while (j < n && fill0 + S(j + 1) <= P) ++j;  // these still go into the newest page
        uint32_t need = 0;
        for (int w = 0; w < (segmented ? WAVES : 1); ++w) {
            const int a = segmented ? min(w * seg, n) : 0, e = segmented ? min(a + seg, n) : n;
            seg_entry[w] = uint32_t(j);
            if (segmented && j < e && j - a < ENTRIES) {
                need += seg_pages[w][j - a];
                j = int(seg_exit[w][j - a]);
            } else {
                while (j < e) {  // few chunks, or an entry the tables do not cover: step by step
                    ++need;
                    j += int(step[j]) + 1;
                }
            }
        }
        uint32_t ok = held + need <= uint64_t(max_pages), top = 0;
        if (ok && need) {
            uint32_t old = __atomic_load_n(&pool_state[0], __ATOMIC_RELAXED);
            while (true) {
                if (old < need) {
                    ok = 0;
                    break;
                }
                const uint32_t seen = atomicCAS(&pool_state[0], old, old - need);
                if (seen == old) break;
                old = seen;
            }
            top = old;
        }
        sh_ok = ok;
        sh_top = top;
    }
    __syncthreads();
    if (sh_ok && lane == 0 && (segmented || wave == 0)) {  // mark the page starts of this wave's part
        int j = int(seg_entry[wave]);
        const int e = segmented ? seg_e : n;
        while (j < e) {
            const uint32_t c = step[j];
            step[j] = uint8_t(c | 0x80u);
            j += int(c) + 1;
        }
    }
    __syncthreads();
    if (!sh_ok) {
        if (tid == 0) status[0] = 1;
        for (int i = lo; i < hi; ++i) {
            index2[2 * (first_chunk + i)] = 0;
            index2[2 * (first_chunk + i) + 1] = 0;
        }
        return;
    }
    const uint32_t top = sh_top;

    // (4) marks before this thread's slice, and the last marked chunk before it (+1; 0 = none)
    uint32_t marks = 0, last = 0;
    for (int j = lo; j < hi; ++j)
        if (step[j] & 0x80u) ++marks, last = uint32_t(j) + 1;
    uint32_t marks_inc = marks, last_inc = last;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t a = __shfl_up(marks_inc, o), b = __shfl_up(last_inc, o);
        if (lane >= o) marks_inc += a, last_inc = max(last_inc, b);
    }
    if (lane == 63) wave_a[wave] = marks_inc, wave_b[wave] = last_inc;
    __syncthreads();
    uint32_t ord = marks_inc - marks;      // fresh pages started before the slice
    uint32_t start_j = __shfl_up(last_inc, 1);
    if (lane == 0) start_j = 0;
    for (int k = 0; k < wave; ++k) ord += wave_a[k], start_j = max(start_j, wave_b[k]);
    const uint32_t newest = held ? page_list[1 + held] : 0u;
    uint32_t page = 0, page_s = 0;  // the page the slice starts in, S of the chunk that starts it
    if (start_j) page = pool_state[top - (ord - 1)], page_s = S(int(start_j) - 1);
    for (int j = lo; j < hi; ++j) {
        if (step[j] & 0x80u) {
            page = pool_state[top - ord];  // stack entry top - 1 - ord sits at word top - ord
            page_list[2 + held + ord] = page;
            ++ord;
            page_s = S(j);
        }
        const uint32_t at = ord ? page * P + (S(j) - page_s) : newest * P + fill0 + S(j);
        index2[2 * (first_chunk + j)] = at;
        index2[2 * (first_chunk + j) + 1] = at + (S(j + 1) - S(j));
    }
    if (tid == 1023) {
        const uint32_t all_last = max(last_inc, start_j);  // with the waves before: the last marked chunk of all
        uint32_t l = all_last;
        for (int k = 0; k < 16; ++k) l = max(l, wave_b[k]);
        page_list[0] = held + ord;
        page_list[1] = l ? total - S(int(l) - 1) : fill0 + total;
    }
}

// Pool of n free pages: the stack holds n - 1 down to 0, so page 0 is handed out first.
__global__ void pool_init_kernel(uint32_t *state, int64_t n_pages) {
    const int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (i == 0) state[0] = uint32_t(n_pages);
    if (i < n_pages) state[1 + i] = uint32_t(n_pages - 1 - i);
}

// Pushes the pages of both tensors back onto the pool's stack (the newest page of a list first,
// so a cache that refills an otherwise idle pool gets its pages in the same order again) and
// empties the lists.  One wave.
__global__ __launch_bounds__(64) void release_pages_kernel(uint32_t *k_list, uint32_t *v_list,
                                                           uint32_t *pool_state, int64_t n_pages) {
    const int lane = threadIdx.x;
    for (int t = 0; t < 2; ++t) {
        uint32_t *list = t ? v_list : k_list;
        const uint32_t cnt = list[0];
        uint32_t base = 0;
        if (lane == 0 && cnt) base = atomicAdd(&pool_state[0], cnt);
        base = __builtin_amdgcn_readfirstlane(base);
        for (uint32_t i = lane; i < cnt; i += 64)
            if (int64_t(base) + i < n_pages) pool_state[1 + base + i] = list[2 + cnt - 1 - i];
    }
    __syncthreads();
    if (lane == 0) k_list[0] = k_list[1] = v_list[0] = v_list[1] = 0;
}

// New tokens of both tensors into their raw tails: blockIdx.z = 0 copies K, 1 copies V.
__global__ void tail_copy_kernel(const uint4 *__restrict__ ksrc, const uint4 *__restrict__ vsrc,
                                 int64_t src_batch_stride16, uint4 *__restrict__ kdst,
                                 uint4 *__restrict__ vdst, int64_t dst_batch_stride16, int64_t n16,
                                 bool bf16) {
    const int b = blockIdx.y;
    const uint4 *src = blockIdx.z ? vsrc : ksrc;
    uint4 *dst = blockIdx.z ? vdst : kdst;
    for (int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x; i < n16;
         i += int64_t(gridDim.x) * blockDim.x)
        dst[b * dst_batch_stride16 + i] =
            load8_as_fp16(reinterpret_cast<const __half *>(src + b * src_batch_stride16 + i), bf16);
}

__global__ void init_kernel(uint32_t *status, uint32_t *k_index, uint32_t *v_index, uint32_t *k_pages,
                            uint32_t *v_pages) {
    if (threadIdx.x < 64) status[threadIdx.x] = 0;
    if (threadIdx.x == 0) {
        k_index[0] = 0;
        v_index[0] = 0;
        if (k_pages) k_pages[0] = k_pages[1] = v_pages[0] = v_pages[1] = 0;
    }
}

// V-median repacking, step 1 (Sec. III-B.3): the lower median of the H*128 quantized V codes of
// one token, written as a sort key.  One workgroup per (token, batch).
__global__ __launch_bounds__(256) void v_median_key_kernel(const __half *__restrict__ src,
                                                           int64_t batch_stride, int64_t token_stride,
                                                           int row_elems, int qmax,
                                                           const uint32_t *__restrict__ meta,
                                                           int64_t meta_stride, int64_t first_token,
                                                           uint8_t *__restrict__ keys, bool bf16) {
    __shared__ int hist[256];
    const int t = blockIdx.x, b = blockIdx.y;
    hist[threadIdx.x] = 0;
    __syncthreads();
    const __half *row = src + b * batch_stride + t * token_stride;
    const float4 tsm = token_scale_min(meta[b * meta_stride + first_token + t]);
    if (qmax > 15) {
        // codes up to 255: count straight into the LDS histogram
        for (int i = threadIdx.x * 8; i < row_elems; i += 256 * 8) {
            uint4 raw = load8_as_fp16(row + i, bf16);
            const __half *hv = reinterpret_cast<const __half *>(&raw);
#pragma unroll
            for (int k = 0; k < 8; ++k) atomicAdd(&hist[quantize_value(__half2float(hv[k]), tsm.x, tsm.y, tsm.z, qmax)], 1);
        }
    } else {
        // sixteen 8-bit counters in two words; a thread sees at most 8 * ceil(row_elems / 2048) values
        uint64_t lo = 0, hi = 0;
        for (int i = threadIdx.x * 8; i < row_elems; i += 256 * 8) {
            uint4 raw = load8_as_fp16(row + i, bf16);
            const __half *hv = reinterpret_cast<const __half *>(&raw);
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int v = quantize_value(__half2float(hv[k]), tsm.x, tsm.y, tsm.z, qmax);
                const uint64_t one = 1ull << (8 * (v & 7));
                if (v < 8) lo += one; else hi += one;
            }
        }
        for (int bin = 0; bin <= qmax; ++bin) {
            int c = int(((bin < 8 ? lo : hi) >> (8 * (bin & 7))) & 0xFFu);
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) c += __shfl_xor(c, o);
            if ((threadIdx.x & 63) == 0) atomicAdd(&hist[bin], c);
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        const int rank = (row_elems - 1) / 2;
        int seen = 0, v = 0;
        for (; v < qmax; ++v) {
            seen += hist[v];
            if (seen > rank) break;
        }
        keys[b * meta_stride + first_token + t] = uint8_t(v);
    }
}

// Step 2: one wave per (block, batch) ranks the 64 keys (ascending, equal keys in arrival order),
// replaces them by the order and moves the token metadata of both tensors into storage order.
__global__ __launch_bounds__(64) void block_order_kernel(uint8_t *__restrict__ order, int qmax,
                                                         uint32_t *__restrict__ k_meta,
                                                         uint32_t *__restrict__ v_meta,
                                                         int64_t meta_stride, int64_t first_token) {
    __shared__ uint8_t ord[N];
    const int lane = threadIdx.x;
    const int64_t pos = blockIdx.y * meta_stride + first_token + int64_t(blockIdx.x) * N;
    const int key = order[pos + lane];
    const uint32_t km = k_meta[pos + lane], vm = v_meta[pos + lane];
    int rank = 0, base = 0;
    for (int v = 0; v <= qmax; ++v) {
        const uint64_t mask = __builtin_amdgcn_ballot_w64(key == v);
        if (key == v) rank = base + __popcll(mask & ((1ull << lane) - 1ull));
        base += __popcll(mask);
    }
    ord[rank] = uint8_t(lane);
    k_meta[pos + rank] = km;
    v_meta[pos + rank] = vm;
    __syncthreads();
    order[pos + lane] = ord[lane];
}

// ---------------------------------------------------------------------------
int launch_init(const kv_cache *c, hipStream_t s) {
    uint8_t *ws = static_cast<uint8_t *>(c->buf.workspace);
    hipLaunchKernelGGL(init_kernel, dim3(1), dim3(64), 0, s,
                       reinterpret_cast<uint32_t *>(ws + WS_STATUS),
                       static_cast<uint32_t *>(c->buf.k_index),
                       static_cast<uint32_t *>(c->buf.v_index),
                       c->pool ? static_cast<uint32_t *>(c->buf.k_pages) : nullptr,
                       c->pool ? static_cast<uint32_t *>(c->buf.v_pages) : nullptr);
    KV_HIP_CHECK(hipGetLastError());
    return KV_OK;
}

int launch_pool_init(const kv_page_pool *pool, hipStream_t s) {
    const int64_t blocks = (pool->n_pages + 255) / 256;
    hipLaunchKernelGGL(pool_init_kernel, dim3(uint32_t(blocks)), dim3(256), 0, s, pool->state, pool->n_pages);
    KV_HIP_CHECK(hipGetLastError());
    return KV_OK;
}

int launch_release_pages(const kv_cache *c, hipStream_t s) {
    if (!c->pool) return KV_ERR_ARG;
    hipLaunchKernelGGL(release_pages_kernel, dim3(1), dim3(64), 0, s,
                       static_cast<uint32_t *>(c->buf.k_pages), static_cast<uint32_t *>(c->buf.v_pages),
                       c->pool->state, c->pool->n_pages);
    KV_HIP_CHECK(hipGetLastError());
    return KV_OK;
}

int launch_tail_copy(const kv_cache *c, const __half *ksrc, const __half *vsrc, int64_t src_batch_stride,
                     int n, int tail_pos, bool bf16, hipStream_t s) {
    const int64_t row = int64_t(c->cfg.n_kv_heads) * D;  // elements per token
    const int64_t n16 = n * row / 8;
    if (n16 == 0) return KV_OK;
    const int threads = 256;
    const int blocks = int(std::min<int64_t>((n16 + threads - 1) / threads, 1024));
    __half *ktail = static_cast<__half *>(c->buf.k_tail), *vtail = static_cast<__half *>(c->buf.v_tail);
    hipLaunchKernelGGL(tail_copy_kernel, dim3(blocks, c->cfg.batch, 2), dim3(threads), 0, s,
                       reinterpret_cast<const uint4 *>(ksrc), reinterpret_cast<const uint4 *>(vsrc),
                       src_batch_stride / 8, reinterpret_cast<uint4 *>(ktail + int64_t(tail_pos) * row),
                       reinterpret_cast<uint4 *>(vtail + int64_t(tail_pos) * row),
                       int64_t(c->cfg.tail_capacity) * row / 8, n16, bf16);
    KV_HIP_CHECK(hipGetLastError());
    return KV_OK;
}

int launch_token_params(const kv_cache *c, const CompressJob &job, hipStream_t s) {
    const int B = c->cfg.batch, H = c->cfg.n_kv_heads;
    const int n_tokens = job.n_blocks * N;
    if (n_tokens <= 0) return KV_ERR_ARG;
    hipLaunchKernelGGL(token_params_kernel, dim3(n_tokens, B), dim3(256), 0, s, job.src,
                       job.batch_stride, job.token_stride, H * D, job.rel, job.meta,
                       c->max_tokens, job.first_token, job.bf16);
    KV_HIP_CHECK(hipGetLastError());
    return KV_OK;
}

int launch_v_median_order(const kv_cache *c, const CompressJob &vjob, uint32_t *k_meta, uint8_t *order,
                          hipStream_t s) {
    const int B = c->cfg.batch, H = c->cfg.n_kv_heads;
    const int n_tokens = vjob.n_blocks * N;
    if (n_tokens <= 0 || H * D / 2048 + 1 > 31) return KV_ERR_ARG;  // 8-bit per-thread counters
    hipLaunchKernelGGL(v_median_key_kernel, dim3(n_tokens, B), dim3(256), 0, s, vjob.src,
                       vjob.batch_stride, vjob.token_stride, H * D, vjob.qmax, vjob.meta,
                       c->max_tokens, vjob.first_token, order, vjob.bf16);
    hipLaunchKernelGGL(block_order_kernel, dim3(vjob.n_blocks, B), dim3(64), 0, s, order, vjob.qmax,
                       k_meta, vjob.meta, c->max_tokens, vjob.first_token);
    KV_HIP_CHECK(hipGetLastError());
    return KV_OK;
}

int launch_pack(const kv_cache *c, const CompressJob &job, hipStream_t s) {
    const int B = c->cfg.batch, H = c->cfg.n_kv_heads;
    const int n_chunks = job.n_blocks * B * H;
    if (n_chunks <= 0 || n_chunks > MAX_NEW_CHUNKS) return KV_ERR_ARG;
    uint8_t *ws = static_cast<uint8_t *>(c->buf.workspace);
    uint32_t *sizes16 = reinterpret_cast<uint32_t *>(ws + WS_SIZES);
    const bool planes = !job.wide && c->cfg.pack_size == 16;
    auto sizes_kernel = job.wide ? chunk_kernel<false, 8, true> : chunk_kernel<false, 8>;
    auto write_kernel = job.wide ? chunk_kernel<true, 8, true> : chunk_kernel<true, 8>;
    // packs of 16, contiguous arena: the staged path when even the largest chunks fit (decided on
    // the device, where the fill level is); the kernels of the other path return at once.  The
    // host knows an upper bound of the fill level: where that already says "fits", the two-pass
    // kernels are not launched at all.
    ChunkSource cs;
    cs.src = job.src;
    cs.batch_stride = job.batch_stride;
    cs.token_stride = job.token_stride;
    cs.B = B;
    cs.H = H;
    cs.qmax = job.qmax;
    cs.magic_h = (uint64_t(1) << 32) / uint64_t(H) + 1;
    cs.magic_hb = (uint64_t(1) << 32) / (uint64_t(H) * uint64_t(B)) + 1;
    cs.meta = job.meta;
    cs.meta_stride = c->max_tokens;
    cs.first_token = job.first_token;
    cs.order = job.order;
    cs.bf16 = job.bf16;
    cs.pack_order = job.pack_order;
    StagedRound round;
    round.first_chunk = job.first_chunk;
    round.worst16 = 0;
    round.arena_cap16 = job.arena_cap16;
    bool two_pass = true;
    // (a small round is bound by its launches, not by reading the input twice: two passes, three kernels)
    constexpr int STAGED_MIN_CHUNKS = 1024;
    if (planes && !c->pool && n_chunks >= STAGED_MIN_CHUNKS) {
        round.worst16 = uint32_t(n_chunks) * uint32_t(CHUNK_MAX / 16);
        two_pass = job.fill_bound16 + round.worst16 > job.arena_cap16;
        uint8_t *staging = ws + c->stage_offset;
        for (int part = 0; part < n_chunks; part += c->stage_chunks) {
            const int n = std::min(c->stage_chunks, n_chunks - part);
            static const int per_cu = resident_workgroups(reinterpret_cast<const void *>(chunk16_stage_kernel));
            const int groups = flat_groups_for(int64_t(n) * 4, per_cu, n);  // all resident, at most one per chunk
            hipLaunchKernelGGL(chunk16_stage_kernel, dim3(groups), dim3(256), 0, s, cs, job.index, part, n,
                               sizes16, staging, round);
            hipLaunchKernelGGL(scan_offsets_kernel, dim3(1), dim3(1024), 0, s, sizes16, n, job.index,
                               job.first_chunk + part, job.arena_cap16, job.status, round, true);
            StagedPart staged;
            staged.staging = staging;
            staged.index = job.index;
            staged.first_chunk = job.first_chunk + part;
            staged.n = n;
            staged.arena = job.arena;
            staged.round = round;
            hipLaunchKernelGGL(chunk16_compact_kernel, dim3((n + 3) / 4), dim3(256), 0, s, staged);
        }
    }
    if (two_pass) {
        if (planes)
            hipLaunchKernelGGL(chunk16_kernel<false>, dim3(n_chunks), dim3(256), 0, s, cs, job.first_chunk,
                               sizes16, job.index, c->index_words, job.arena, round);
        else
            hipLaunchKernelGGL(sizes_kernel, dim3(n_chunks), dim3(256), 0, s, job.src,
                               job.batch_stride, job.token_stride, B, H, job.qmax, job.meta, c->max_tokens,
                               job.first_token, job.first_chunk, sizes16, job.index, c->index_words, job.arena,
                               job.order, job.bf16);
        if (c->pool)
            hipLaunchKernelGGL(place_chunks_kernel, dim3(1), dim3(1024), 0, s, sizes16, n_chunks, job.index,
                               job.first_chunk, job.page_list, job.max_pages, c->pool->state, job.status);
        else
            hipLaunchKernelGGL(scan_offsets_kernel, dim3(1), dim3(1024), 0, s, sizes16, n_chunks,
                               job.index, job.first_chunk, job.arena_cap16, job.status, round, false);
        if (planes)
            hipLaunchKernelGGL(chunk16_kernel<true>, dim3(n_chunks), dim3(256), 0, s, cs, job.first_chunk,
                               sizes16, job.index, c->index_words, job.arena, round);
        else
            hipLaunchKernelGGL(write_kernel, dim3(n_chunks), dim3(256), 0, s, job.src,
                               job.batch_stride, job.token_stride, B, H, job.qmax, job.meta, c->max_tokens,
                               job.first_token, job.first_chunk, sizes16, job.index, c->index_words, job.arena,
                               job.order, job.bf16);
    }
    KV_HIP_CHECK(hipGetLastError());
    return KV_OK;
}

}  // namespace packkv
