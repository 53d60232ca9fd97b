// Append-side compressor: token-wise quantization, bit-packing, appending
// (PackKV Sec. III-B.1 .. III-B.4).  Cold path: runs once per 64 decode steps.
//
//   token_params   one workgroup per (token, batch): min/max over the token's
//                  H*128 values -> fp16 scale = rel*(max-min), fp16 min
//   v_median_key, block_order   (V-median repacking only) sort key per token,
//                  order of the 64 tokens of a block, metadata into storage order
//   chunk_sizes    one workgroup per chunk: quantize, per-pack width -> bytes
//   scan_offsets   one workgroup: prefix sum of the new chunk sizes -> index
//   place_chunks   (paged arena instead of scan_offsets) one workgroup: chunk positions inside
//                  pages taken from a shared pool -> index of (start, end) pairs
//   pack_chunks    one workgroup per chunk: quantize again and write header +
//                  payload at its final place (no staging copy, no atomics, so
//                  the arena bytes are a pure function of the input)
#include <algorithm>

#include "common.h"

namespace packkv {

// Eight consecutive input values as fp16.  fp16 inputs pass as they are; bf16 inputs are rounded
// to fp16 (to nearest even; exact for every value in fp16's normal range, fp16 having the longer
// significand) -- from there on the path does not know the input type.
__device__ inline uint4 load8_as_fp16(const __half *p, bool bf16) {
    uint4 raw = *reinterpret_cast<const uint4 *>(p);
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

__device__ inline PlaneBits make_planes(const __half *tile, int g, int d, const float4 *sm, int qmax) {
    int q[PACK];
    int lo = 255, hi = 0;
#pragma unroll
    for (int i = 0; i < PACK; ++i) {
        const float4 t = sm[g * PACK + i];
        const int v = quantize_value(__half2float(tile[(g * PACK + i) * D + d]), t.x, t.y, t.z, qmax);
        q[i] = v;
        lo = min(lo, v);
        hi = max(hi, v);
    }
    PlaneBits pb;
    const int range = hi - lo;
    pb.w = range == 0 ? 0 : 32 - __clz(range);
    pb.m = lo;
    pb.low = pb.high = pb.top = 0;
    const int top_bit = pb.w > 0 ? pb.w - 1 : 0;
#pragma unroll
    for (int i = 0; i < PACK; ++i) {
        const uint32_t c = uint32_t(q[i] - lo);
        const int at = i < 8 ? 4 * i : 4 * (i - 8) + 2;
        pb.low |= (c & 3u) << at;
        pb.high |= (c >> 2) << at;
        pb.top |= ((c >> top_bit) & 1u) << (4 * (i & 3) + (i >> 2));
    }
    return pb;
}

template <bool WRITE>
__global__ __launch_bounds__(256) void chunk16_kernel(const __half *__restrict__ src,
                                                      int64_t batch_stride, int64_t token_stride,
                                                      int B, int H, int qmax,
                                                      const uint32_t *__restrict__ meta,
                                                      int64_t meta_stride, int64_t first_token,
                                                      int64_t first_chunk,
                                                      uint32_t *__restrict__ sizes16,
                                                      const uint32_t *__restrict__ index,
                                                      int index_words,
                                                      uint8_t *__restrict__ arena,
                                                      const uint8_t *__restrict__ order, bool bf16,
                                                      int pack_order) {
    const int cl = blockIdx.x;  // chunk within this round: (blk*B + b)*H + h
    const int h = cl % H;
    const int b = (cl / H) % B;
    const int blk = cl / (H * B);
    const int tau = threadIdx.x;

    uint8_t *dst = nullptr;
    if (WRITE) {
        const int64_t e = (first_chunk + cl) * index_words;
        uint32_t o0 = index[e], o1 = index[e + 1];
        if (o1 == o0) return;  // dropped: the arena was full
        dst = arena + size_t(o0) * 16;
    }

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

    PlaneBits pb[2];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int p = tau + 256 * k;
        const int g = pack_order ? (p & 3) : (p >> 7);
        const int d = pack_order ? (p >> 2) : (p & 127);
        pb[k] = make_planes(tile, g, d, sm, qmax);
    }
    // one scan per pack-list half carries both regions: E bytes in the low half, O bytes in the high half
    int off[2];
    int run = 0;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        int total;
        off[k] = run + block_exclusive_scan(4 * (pb[k].w >> 1) + ((2 * (pb[k].w & 1)) << 16), &total);
        run += total;
    }
    const int e_bytes = run & 0xFFFF, o_bytes = run >> 16;
    const int padded = (HEADER + e_bytes + o_bytes + 15) & ~15;

    if (!WRITE) {
        if (tau == 0) sizes16[cl] = uint32_t(padded >> 4);
        return;
    }
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        dst[tau + 256 * k] = uint8_t((pb[k].w << 4) | pb[k].m);
        uint32_t *e = reinterpret_cast<uint32_t *>(dst + HEADER + (off[k] & 0xFFFF));
        if (pb[k].w >= 2) e[0] = pb[k].low;
        if (pb[k].w == 4) e[1] = pb[k].high;
        if (pb[k].w & 1)
            *reinterpret_cast<uint16_t *>(dst + HEADER + e_bytes + (off[k] >> 16)) = uint16_t(pb[k].top);
    }
    if (tau < padded - HEADER - e_bytes - o_bytes) dst[HEADER + e_bytes + o_bytes + tau] = 0;
}

// Single workgroup: index[first+i+1] = index[first] + sum_{j<=i} sizes16[j].
// If the new chunks do not fit, all of them get size 0 and the flag is set.
__global__ __launch_bounds__(1024) void scan_offsets_kernel(const uint32_t *__restrict__ sizes16,
                                                            int n, uint32_t *__restrict__ index,
                                                            int64_t first_chunk,
                                                            uint64_t arena_cap16,
                                                            uint32_t *__restrict__ status) {
    __shared__ uint32_t wsum[16];
    __shared__ uint32_t total_s;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int per = (n + 1023) / 1024;
    const int lo = min(tid * per, n), hi = min(lo + per, n);
    uint32_t local = 0;
    for (int i = lo; i < hi; ++i) local += sizes16[i];
    uint32_t inc = local;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        uint32_t v = __shfl_up(inc, o);
        if (lane >= o) inc += v;
    }
    if (lane == 63) wsum[wave] = inc;
    __syncthreads();
    uint32_t base = 0;
    for (int k = 0; k < wave; ++k) base += wsum[k];
    if (tid == 1023) total_s = base + inc;
    __syncthreads();
    const uint32_t start = index[first_chunk];
    const bool fits = uint64_t(start) + total_s <= arena_cap16;
    if (!fits && tid == 0) status[0] = 1;
    uint32_t run = start + base + inc - local;
    for (int i = lo; i < hi; ++i) {
        run += sizes16[i];
        index[first_chunk + i + 1] = fits ? run : start;
    }
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
    if (planes)
        hipLaunchKernelGGL(chunk16_kernel<false>, dim3(n_chunks), dim3(256), 0, s, job.src,
                           job.batch_stride, job.token_stride, B, H, job.qmax, job.meta, c->max_tokens,
                           job.first_token, job.first_chunk, sizes16, job.index, c->index_words, job.arena,
                           job.order, job.bf16, job.pack_order);
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
                           job.index, job.first_chunk, job.arena_cap16, job.status);
    if (planes)
        hipLaunchKernelGGL(chunk16_kernel<true>, dim3(n_chunks), dim3(256), 0, s, job.src,
                           job.batch_stride, job.token_stride, B, H, job.qmax, job.meta, c->max_tokens,
                           job.first_token, job.first_chunk, sizes16, job.index, c->index_words, job.arena,
                           job.order, job.bf16, job.pack_order);
    else
        hipLaunchKernelGGL(write_kernel, dim3(n_chunks), dim3(256), 0, s, job.src,
                           job.batch_stride, job.token_stride, B, H, job.qmax, job.meta, c->max_tokens,
                           job.first_token, job.first_chunk, sizes16, job.index, c->index_words, job.arena,
                           job.order, job.bf16);
    KV_HIP_CHECK(hipGetLastError());
    return KV_OK;
}

}  // namespace packkv
