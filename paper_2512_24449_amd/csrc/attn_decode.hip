// Fused decode attention over the packed cache: Att(q, K, V) = softmax(sm_scale * K q)^T V
// (definition in PackKV Sec. III-B.3) in one pass, with the per-chunk K and V work of
// Sec. III-C.1 / III-C.2 (k_planes.h, v_planes.h; pack8.h) and an online softmax in between, so the
// fp32 scores and probabilities never travel through HBM.
//
// A wave walks blocks of one (batch, kv-head) stream.  Per block it unpacks the K chunk
// into the 64 scores of the block (lane = token), turns them into weights
// p_t = 2^(s_t - m_ref) against a wave-uniform reference m_ref per head, and feeds the V
// chunk of the same block with them.  m_ref is only raised when some score exceeds it by
// more than 8 (in log2 units): then the exact wave maximum becomes the new reference and
// all running sums are rescaled once.  Weights therefore stay below 2^8, inside the range
// the V operand's weight split represents, and a reference below the true
// maximum cancels in the final division.  The wave holds one K and one V chunk buffer:
// the V chunk streams in while K is unpacked, the next K chunk while V is unpacked.
//
// The context axis is split over workgroups.  Each wave ends with (m_ref, l = sum p,
// o[128]) per head; the four waves of a workgroup and then the splits are merged in a
// fixed order with the usual 2^(m_i - M) factors by attn_combine_kernel, which also
// handles the raw fp16 tail.  No floating-point atomics: bitwise reproducible.
#include <algorithm>

#include "k_planes.h"
#include "pack8.h"
#include "v_chunk.h"
#include "v_planes.h"

namespace packkv {

constexpr float LOG2E = 1.4426950408889634f;
constexpr float RAISE_MARGIN = 8.0f;  // log2 units a score may exceed the reference by
constexpr int A_L = D;                // partial row: [0..127] outputs, [128] sum of weights,
constexpr int A_M = D + 1;            // [129] reference exponent (log2 units)

struct AArgs {
    const uint8_t *k_arena, *v_arena;
    const uint32_t *k_index, *v_index;
    const uint32_t *k_meta, *v_meta;  // [B][meta_stride]
    const __half *q;                  // [B][Hq][128]
    float *partial;                   // [splits][B*Hq][V_PART_STRIDE]
    int64_t meta_stride;
    int B, H;
    int index_words;        // index words per chunk: 1 back to back, 2 with a paged arena
    int dup;                // H counts every kv-head dup times (query groups above 8 are split): kv-head = h / dup
    int n_blocks;                     // packed blocks per stream
    int blocks_per_split;
    float sm_log2;                    // sm_scale * log2(e)
};

__device__ inline float wave_all_max(float v) {
    v = fmaxf(v, dpp_f32<DPP_ROW_ROR8>(v));
    v = fmaxf(v, __shfl_xor(v, 4));
    v = fmaxf(v, dpp_f32<DPP_QUAD_XOR2>(v));
    v = fmaxf(v, dpp_f32<DPP_QUAD_XOR1>(v));
    v = fmaxf(v, __shfl_xor(v, 16));
    v = fmaxf(v, __shfl_xor(v, 32));
    return v;
}

__device__ inline float wave_all_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// 2^(a - b) with the convention that an empty side (a = -inf) weighs nothing.
__device__ inline float exp2_diff(float a, float b) { return a == -INFINITY ? 0.0f : exp2f(a - b); }

// Online softmax bookkeeping: raise a head's reference only when a score of this block runs
// away from it, and rescale the running sums then.  s: this lane's scores (log2 units).
template <int G>
__device__ inline void attn_raise_reference(const float (&s)[G], float (&m_ref)[G], float (&l_lane)[G],
                                            VState<G> &st, int col) {
    bool raise = false;
#pragma unroll
    for (int g = 0; g < G; ++g) raise |= s[g] > m_ref[g] + RAISE_MARGIN;
    if (__builtin_amdgcn_ballot_w64(raise) != 0) {
        float alpha_col = 1.0f;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            // the same value in every lane: keep it in a scalar register
            const float m_new = __int_as_float(__builtin_amdgcn_readfirstlane(
                __float_as_int(fmaxf(m_ref[g], wave_all_max(s[g])))));
            const float alpha = exp2_diff(m_ref[g], m_new);
            m_ref[g] = m_new;
            l_lane[g] *= alpha;
            st.pm[g] *= alpha;
            if constexpr (!fold_min<G>()) {
#pragma unroll
                for (int j = 0; j < 8; ++j) st.macc[g][j] *= alpha;
            }
            if ((col >> 1) == g) alpha_col = alpha;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) st.acc[j] *= alpha_col;
    }
}

// The same for the running sums of the plane-layout V phase (v_planes.h): the result tiles hold
// one digit of one head per column.
template <int G>
__device__ inline void attn_raise_reference(const float (&s)[G], float (&m_ref)[G], float (&l_lane)[G],
                                            VPlaneState<G> &st, int col) {
    bool raise = false;
#pragma unroll
    for (int g = 0; g < G; ++g) raise |= s[g] > m_ref[g] + RAISE_MARGIN;
    if (__builtin_amdgcn_ballot_w64(raise) != 0) {
        float alpha_col = 1.0f;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float m_new = __int_as_float(__builtin_amdgcn_readfirstlane(
                __float_as_int(fmaxf(m_ref[g], wave_all_max(s[g])))));
            const float alpha = exp2_diff(m_ref[g], m_new);
            m_ref[g] = m_new;
            l_lane[g] *= alpha;
            st.pm[g] *= alpha;
#pragma unroll
            for (int j = 0; j < 8; ++j) st.macc[g][j] *= alpha;
            if (col / v_pieces<G>() == g) alpha_col = alpha;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) st.acc[j] *= alpha_col;
    }
}

template <int G>
__device__ inline void attn_store_state(const VState<G> &st, float (*red)[D + 4], int lane, float code_scale) {
    v_state_store<G>(st, red, lane, code_scale);
}
template <int G>
__device__ inline void attn_store_state(const VPlaneState<G> &st, float (*red)[D + 4], int lane, float) {
    v_planes_store<G>(st, red, lane);
}

// End of a fused attention workgroup: merges the four waves' running sums (each with its own
// softmax reference) and writes the split's partial row.  red aliases the chunk buffers.
template <int G, class State>
__device__ inline void attn_store_partial(const AArgs &a, const State &st, const float (&l_lane)[G],
                                          const float (&m_ref)[G], float (*red)[G][D + 4], int wave,
                                          int lane, int split, int64_t head0,
                                          float code_scale = CODE_SCALE_LIFTED) {
    __syncthreads();  // every wave is done with its chunk buffers: reuse them as red[][][]

    attn_store_state<G>(st, red[wave], lane, code_scale);
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const float l = wave_all_sum(l_lane[g]);
        if (lane == 0) {
            red[wave][g][D + 1] = l;
            red[wave][g][D + 2] = m_ref[g];
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < G * (D + 1); i += 256) {
        const int g = i / (D + 1), d = i % (D + 1);
        const float m0 = red[0][g][D + 2], m1 = red[1][g][D + 2], m2 = red[2][g][D + 2], m3 = red[3][g][D + 2];
        const float M = fmaxf(fmaxf(m0, m1), fmaxf(m2, m3));
        const float f0 = exp2_diff(m0, M), f1 = exp2_diff(m1, M), f2 = exp2_diff(m2, M), f3 = exp2_diff(m3, M);
        float *dst = a.partial + (int64_t(split) * a.B * a.H * G + head0 + g) * V_PART_STRIDE;
        if (d < D) {
            // outputs carry the per-head sum p*min term
            dst[d] = (f0 * (red[0][g][d] + red[0][g][D]) + f1 * (red[1][g][d] + red[1][g][D])) +
                     (f2 * (red[2][g][d] + red[2][g][D]) + f3 * (red[3][g][d] + red[3][g][D]));
        } else {
            dst[A_L] = (f0 * red[0][g][D + 1] + f1 * red[1][g][D + 1]) +
                       (f2 * red[2][g][D + 1] + f3 * red[3][g][D + 1]);
            dst[A_M] = M;
        }
    }
}

// HIGH: the V codes of the cache may need four bits (a plane H exists).
template <int G, bool HIGH>
__global__ __launch_bounds__(256) void attn_kernel(AArgs a) {
    // per wave: buffer 0 holds the K chunk (and then its tiles, k_planes.h), buffer 1 the V chunk of
    // the block in flight; after the main loop the same memory holds the cross-wave reduction array
    // red[4][G][D + 4]
    __shared__ __attribute__((aligned(16))) uint8_t lds_all[4 * 2 * CHUNK_LDS + LDS_TAIL_PAD];
    constexpr int VB = vb_bytes<G>();
    __shared__ __attribute__((aligned(16))) uint8_t vb_all[4 * VB];  // digit staging of the V phase
    __shared__ uint4 ktable[5];                                      // K chunks: plane layout, channel-major
    __shared__ uint4 vtable[PLANE_TABLE_ENTRIES];                    // V chunks: plane layout, group-major
    __shared__ uint32_t vhighs[PLANE_TABLE_ENTRIES];
    static_assert(sizeof(float) * 4 * G * (D + 4) <= 4 * 2 * CHUNK_LDS, "reduction array must fit");
    static_assert(K_TILES_BYTES <= CHUNK_LDS && CHUNK_LDS % 16 == 0, "the K tiles are built in the K buffer");
    float(*red)[G][D + 4] = reinterpret_cast<float(*)[G][D + 4]>(lds_all);
    for (int i = threadIdx.x; i < 4 * VB / 4; i += 256) reinterpret_cast<uint32_t *>(vb_all)[i] = 0;
    build_k_plane_table(ktable);
    build_plane_table(vtable, vhighs);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int split = blockIdx.x;
    const int bh = blockIdx.y;
    const int h = bh % a.H, b = bh / a.H;
    const int col = lane & 15;
    const int kbuf = wave * 2 * CHUNK_LDS, vbuf = kbuf + CHUNK_LDS;
    const int64_t head0 = int64_t(b) * a.H * G + h * G;

    KQueryPlanes<G> kq;
    kq.load(a.q + head0 * D, lane);
    uint8_t *vb = vb_all + wave * VB;
    VPlaneState<G> st;
    st.clear();
    float m_ref[G], l_lane[G];
#pragma unroll
    for (int g = 0; g < G; ++g) m_ref[g] = -INFINITY, l_lane[g] = 0.0f;

    const int blk_begin = split * a.blocks_per_split;
    const int blk_end = min(blk_begin + a.blocks_per_split, a.n_blocks);
    for (int first = blk_begin + wave; first < blk_end; first += 4 * 64) {
        IndexBatch ik, iv;
        ik.load(a.k_index, a.index_words, first, 4, blk_end, a.B, a.H / a.dup, b, h / a.dup, lane);
        iv.load(a.v_index, a.index_words, first, 4, blk_end, a.B, a.H / a.dup, b, h / a.dup, lane);
        const int n_it = min(64, (blk_end - first + 3) / 4);
        chunk_issue_lds<CHUNK_MAX, HEADER, true>(a.k_arena, ik.start16(0), ik.end16(0), lds_all + kbuf, lane);
        const int64_t tok0 = b * a.meta_stride + int64_t(first) * N + lane;
        uint32_t kmt_next = a.k_meta[tok0], vmt_next = a.v_meta[tok0];
        for (int it = 0; it < n_it; ++it) {
            // a block dropped by an arena overflow (in either tensor) takes no part
            const bool valid = ik.end16(it) - ik.start16(it) >= uint32_t(HEADER / 16) &&
                               iv.end16(it) - iv.start16(it) >= uint32_t(HEADER / 16);
            wait_chunk_landed();  // K chunk of this block
            uint32_t kmt = kmt_next, vmt = vmt_next;
            consume_here(kmt), consume_here(vmt);
            lds_reads_returned();  // the previous V chunk has been read completely
            chunk_issue_lds<CHUNK_MAX, HEADER, true>(a.v_arena, iv.start16(it), iv.end16(it), lds_all + vbuf, lane);
            if (it + 1 < n_it) {
                const int64_t tok = b * a.meta_stride + int64_t(first + 4 * (it + 1)) * N + lane;
                kmt_next = a.k_meta[tok];
                vmt_next = a.v_meta[tok];
            }

            float s[G];  // scores of token `lane` in log2 units
            if (valid) {
                float u[G];
                k_planes_chunk<G>(lds_all, kbuf, ktable, lds_all + kbuf, kq, u, []() {});
                const float kscale = __half2float(__ushort_as_half(uint16_t(kmt & 0xFFFFu)));
                const float kmn = __half2float(__ushort_as_half(uint16_t(kmt >> 16)));
#pragma unroll
                for (int g = 0; g < G; ++g) s[g] = a.sm_log2 * fmaf(kscale, u[g], kmn * kq.qsum[g]);

                attn_raise_reference<G>(s, m_ref, l_lane, st, col);
            }
            wait_chunk_landed();  // V chunk of this block
            lds_reads_returned();  // the K tiles have been read completely before the next chunk overwrites them
            if (it + 1 < n_it)
                chunk_issue_lds<CHUNK_MAX, HEADER, true>(a.k_arena, ik.start16(it + 1), ik.end16(it + 1), lds_all + kbuf, lane);
            if (!valid) continue;
            float pt[G];
#pragma unroll
            for (int g = 0; g < G; ++g) {
                pt[g] = exp2f(s[g] - m_ref[g]);
                l_lane[g] += pt[g];
            }
            v_planes_chunk<G, HIGH>(lds_all, vbuf, vtable, vhighs, vb, vmt, pt, st);
        }
        wait_chunk_landed();
    }
    attn_store_partial<G>(a, st, l_lane, m_ref, red, wave, lane, split, head0);
}

// The same for chunks with packs of 8 tokens (Sec. IV-B; pack8.h): the K phase runs the
// pairwise dot-product form for all G heads and leaves lane l with token
// k8_token_of_block_lane(l) of the block; the V phase stages the weights in that order.
// KW / VW: that tensor uses the wide chunk layout (codes above 15); the two tensors choose
// their layout independently, and a wide chunk needs a buffer twice as large.  With both wide,
// two buffers per wave would leave room for one workgroup per compute unit only (measured 0.76 ms
// at the headline shape, slower than the three-step path); the K and the V chunk then take turns
// in ONE buffer, transfers overlap with the unpacking of other waves only, and three workgroups
// fit.
template <int G, bool KW, bool VW>
__global__ __launch_bounds__(256) void attn8_kernel(AArgs a) {
    constexpr bool SHARED = KW && VW;
    constexpr int KLDS = KW ? CHUNKW_LDS : CHUNK8_LDS, VLDS = SHARED ? 0 : (VW ? CHUNKW_LDS : CHUNK8_LDS);
    constexpr int KMAX = KW ? CHUNKW_MAX : CHUNK8_MAX, VMAX = VW ? CHUNKW_MAX : CHUNK8_MAX;
    constexpr int KHDR = KW ? HEADERW : HEADER8, VHDR = VW ? HEADERW : HEADER8;
    __shared__ __attribute__((aligned(16))) uint8_t lds_all[4 * (KLDS + VLDS) + LDS_TAIL_PAD];
    __shared__ __attribute__((aligned(16))) uint8_t blds_all[4 * BLds<G>::BYTES];
    __shared__ uint2 table[KW ? 16 : PACK_TABLE_ENTRIES];   // K: the wide K table, or the pair table
    __shared__ uint4 vtable[VW ? 16 : PACK_TABLE_ENTRIES];  // V: the wide V table, or lifted codes
    static_assert(sizeof(float) * 4 * G * (D + 4) <= 4 * (KLDS + VLDS), "reduction array must fit");
    static_assert(WIDE_TABLE_ENTRIES <= 16, "table sizes above");
    float(*red)[G][D + 4] = reinterpret_cast<float(*)[G][D + 4]>(lds_all);
    if constexpr (!KW) build_pair_table(table);
    if constexpr (!VW) build_pack_table(vtable, CODE_LIFT, fold_min<G>());
    if constexpr (KW || VW) build_wide_tables(KW ? table : nullptr, VW ? vtable : nullptr);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int split = blockIdx.x;
    const int bh = blockIdx.y;
    const int h = bh % a.H, b = bh / a.H;
    const int col = lane & 15;
    const int kbuf = wave * (KLDS + VLDS), vbuf = SHARED ? kbuf : kbuf + KLDS;
    const int64_t head0 = int64_t(b) * a.H * G + h * G;
    const int tok_in_blk = k8_token_of_block_lane(lane);

    KQuery8<G> kq;
    kq.load(a.q + head0 * D, lane);
    VLane<G> vl;
    vl.init(blds_all + wave * BLds<G>::BYTES, lane);
    vl.bslot = v8_bslot<G>(tok_in_blk);
    VState<G> st;
    st.clear();
    float m_ref[G], l_lane[G];
#pragma unroll
    for (int g = 0; g < G; ++g) m_ref[g] = -INFINITY, l_lane[g] = 0.0f;

    const int blk_begin = split * a.blocks_per_split;
    const int blk_end = min(blk_begin + a.blocks_per_split, a.n_blocks);
    for (int first = blk_begin + wave; first < blk_end; first += 4 * 64) {
        IndexBatch ik, iv;
        ik.load(a.k_index, a.index_words, first, 4, blk_end, a.B, a.H / a.dup, b, h / a.dup, lane);
        iv.load(a.v_index, a.index_words, first, 4, blk_end, a.B, a.H / a.dup, b, h / a.dup, lane);
        const int n_it = min(64, (blk_end - first + 3) / 4);
        chunk_issue_lds<KMAX, KHDR>(a.k_arena, ik.start16(0), ik.end16(0), lds_all + kbuf, lane);
        const int64_t tok0 = b * a.meta_stride + int64_t(first) * N + tok_in_blk;
        uint32_t kmt_next = a.k_meta[tok0], vmt_next = a.v_meta[tok0];
        for (int it = 0; it < n_it; ++it) {
            // a block dropped by an arena overflow (in either tensor) takes no part
            const bool valid = ik.end16(it) - ik.start16(it) >= uint32_t(KHDR / 16) &&
                               iv.end16(it) - iv.start16(it) >= uint32_t(VHDR / 16);
            wait_chunk_landed();  // K chunk of this block
            uint32_t kmt = kmt_next, vmt = vmt_next;
            consume_here(kmt), consume_here(vmt);
            if constexpr (!SHARED) {
                lds_reads_returned();  // the previous V chunk has been read completely
                chunk_issue_lds<VMAX, VHDR>(a.v_arena, iv.start16(it), iv.end16(it), lds_all + vbuf, lane);
            }
            if (it + 1 < n_it) {
                const int64_t tok = b * a.meta_stride + int64_t(first + 4 * (it + 1)) * N + tok_in_blk;
                kmt_next = a.k_meta[tok];
                vmt_next = a.v_meta[tok];
            }

            float s[G];  // scores of this lane's token in log2 units
            if (valid) {
                float u0[G], u1[G];
                if constexpr (KW) {
                    const uint2 w0 = *reinterpret_cast<const uint2 *>(lds_all + kbuf + lane * 8);
                    const uint2 m0 = *reinterpret_cast<const uint2 *>(lds_all + kbuf + 1024 + lane * 8);
                    LanePacksW lp0;
                    lp0.init(w0, m0, kbuf + HEADERW);
                    kw_half<G>(lds_all, table, lp0, kq, lane, u0);
                    const uint2 w1 = *reinterpret_cast<const uint2 *>(lds_all + kbuf + 512 + lane * 8);
                    const uint2 m1 = *reinterpret_cast<const uint2 *>(lds_all + kbuf + 1536 + lane * 8);
                    LanePacksW lp1;
                    lp1.init(w1, m1, lp0.end_all);
                    kw_half<G>(lds_all, table, lp1, kq, lane, u1);
                } else {
                    const uint2 hdr0 = *reinterpret_cast<const uint2 *>(lds_all + kbuf + lane * 8);
                    LanePacks8 lp0;
                    lp0.init(hdr0.x, hdr0.y, kbuf + HEADER8);
                    k8_half<G>(lds_all, table, lp0, kq, lane, u0);
                    const uint2 hdr1 = *reinterpret_cast<const uint2 *>(lds_all + kbuf + 512 + lane * 8);
                    LanePacks8 lp1;
                    lp1.init(hdr1.x, hdr1.y, lp0.end_all);
                    k8_half<G>(lds_all, table, lp1, kq, lane, u1);
                }
                const float kscale = __half2float(__ushort_as_half(uint16_t(kmt & 0xFFFFu)));
                const float kmn = __half2float(__ushort_as_half(uint16_t(kmt >> 16)));
#pragma unroll
                for (int g = 0; g < G; ++g)
                    s[g] = a.sm_log2 * fmaf(kscale, (lane & 1) ? u1[g] : u0[g], kmn * kq.qsum[g]);
                attn_raise_reference<G>(s, m_ref, l_lane, st, col);
            }
            if constexpr (SHARED) {
                // one buffer: the K chunk has been read completely before the V chunk overwrites it
                lds_reads_returned();
                chunk_issue_lds<VMAX, VHDR>(a.v_arena, iv.start16(it), iv.end16(it), lds_all + vbuf, lane);
            }
            wait_chunk_landed();  // V chunk of this block
            if constexpr (!SHARED) {
                lds_reads_returned();  // the K chunk has been read completely before the next one overwrites it
                if (it + 1 < n_it)
                    chunk_issue_lds<KMAX, KHDR>(a.k_arena, ik.start16(it + 1), ik.end16(it + 1), lds_all + kbuf, lane);
            }
            if (valid) {
                float pt[G];
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    pt[g] = exp2f(s[g] - m_ref[g]);
                    l_lane[g] += pt[g];
                }
                if constexpr (VW)
                    vw_chunk<G, true>(lds_all, vbuf, vtable, vl, vmt, pt, st);
                else
                    v8_chunk<G, true>(lds_all, vbuf, vtable, vl, vmt, pt, st);
            }
            if constexpr (SHARED) {
                lds_reads_returned();
                if (it + 1 < n_it)
                    chunk_issue_lds<KMAX, KHDR>(a.k_arena, ik.start16(it + 1), ik.end16(it + 1), lds_all + kbuf, lane);
            }
        }
        wait_chunk_landed();
    }
    // wide V codes enter the matrix cores as the numbers themselves
    attn_store_partial<G>(a, st, l_lane, m_ref, red, wave, lane, split, head0, VW ? 1.0f : CODE_SCALE_LIFTED);
}

// Merges the splits of one (batch, query head) row in a fixed order and adds the raw fp16
// tail tokens (Sec. III-B.1 buffer), whose scores are plain dot products.
__global__ __launch_bounds__(256) void attn_combine_kernel(const float *__restrict__ partial,
                                                           int n_splits, int n_rows,
                                                           const __half *__restrict__ q,
                                                           const __half *__restrict__ k_tail,
                                                           const __half *__restrict__ v_tail,
                                                           int n_tail, int tail_cap, int H, int G,
                                                           float sm_log2, float *__restrict__ out) {
    __shared__ float st[N];             // tail scores (log2 units), then tail weights
    __shared__ float ms[V_SPLITS_MAX];  // split references, then split factors
    __shared__ float red[16][V_PART_STRIDE];
    static_assert(A_L == 128, "the splits' weight sums sit in the column the reduction returns separately");
    const int r = blockIdx.x;           // b*Hq + hq
    const int hq = r % (H * G), b = r / (H * G);
    const int h = hq / G;
    // every global load of the kernel is issued before the first result is needed
    SplitRows rows;
    TailRows trows;
    rows.load(partial, n_splits, n_rows, r);
    trows.load(v_tail + (int64_t(b) * tail_cap * H + h) * D, int64_t(H) * D, n_tail);
    if (int(threadIdx.x) < n_splits)
        ms[threadIdx.x] = partial[(int64_t(threadIdx.x) * n_rows + r) * V_PART_STRIDE + A_M];
    // tail scores: thread (t, seg) takes 32 channels of tail token t, four threads per token
    {
        const int t = threadIdx.x >> 2, seg = threadIdx.x & 3;
        float s = 0.0f;
        if (t < n_tail) {
            const __half *krow = k_tail + ((int64_t(b) * tail_cap + t) * H + h) * D + 32 * seg;
            const __half *qrow = q + int64_t(r) * D + 32 * seg;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint4 kr = *reinterpret_cast<const uint4 *>(krow + 8 * c);
                const uint4 qr = *reinterpret_cast<const uint4 *>(qrow + 8 * c);
                const __half *kk = reinterpret_cast<const __half *>(&kr);
                const __half *qq = reinterpret_cast<const __half *>(&qr);
#pragma unroll
                for (int e = 0; e < 8; ++e) s = fmaf(__half2float(kk[e]), __half2float(qq[e]), s);
            }
        }
        s += dpp_f32<DPP_QUAD_XOR1>(s);
        s += dpp_f32<DPP_QUAD_XOR2>(s);
        if (seg == 0 && t < n_tail) st[t] = sm_log2 * s;
    }
    __syncthreads();
    float M = -INFINITY;
    for (int s = 0; s < n_splits; ++s) M = fmaxf(M, ms[s]);
    for (int t = 0; t < n_tail; ++t) M = fmaxf(M, st[t]);
    __syncthreads();
    if (int(threadIdx.x) < n_splits) ms[threadIdx.x] = exp2_diff(ms[threadIdx.x], M);
    if (threadIdx.x >= 64 && int(threadIdx.x) - 64 < n_tail) st[threadIdx.x - 64] = exp2f(st[threadIdx.x - 64] - M);
    __syncthreads();
    // weighted sum of the split rows (column 128 = the splits' weight sums), then the tail tokens
    float l;
    float o = rows.sum(n_splits, red, &l, ms);
    if (n_tail > 0) {
        o += trows.sum(st, n_tail, red);
        for (int t = 0; t < n_tail; ++t) l += st[t];
    }
    const int d = threadIdx.x;
    if (d < D) out[int64_t(r) * D + d] = l > 0.0f ? o / l : 0.0f;  // every block dropped and no tail: defined output
}

int v_splits_for(int n_blocks, int streams);

int launch_decode_attention(const kv_cache *c, const __half *q, float sm_scale, float *out, hipStream_t s) {
    // Hs: kv-heads as the stream kernels count them (each dup times, see head_split); the combine
    // kernel works per query head and sees the real kv-head count and the whole group
    const int B = c->cfg.batch, H = c->cfg.n_kv_heads, G = c->group, Hs = H * c->head_split, Gq = G * c->head_split;
    const int n_blocks = int(c->packed_tokens / N);
    uint8_t *ws = static_cast<uint8_t *>(c->buf.workspace);
    float *partial = reinterpret_cast<float *>(ws + WS_VPART);
    const float sm_log2 = sm_scale * LOG2E;
    int n_splits = 0;
    if (n_blocks > 0) {
        n_splits = v_splits_for(n_blocks, B * Hs);
        AArgs a;
        a.k_arena = static_cast<const uint8_t *>(c->buf.k_arena);
        a.v_arena = static_cast<const uint8_t *>(c->buf.v_arena);
        a.k_index = static_cast<const uint32_t *>(c->buf.k_index);
        a.v_index = static_cast<const uint32_t *>(c->buf.v_index);
        a.k_meta = static_cast<const uint32_t *>(c->buf.k_token_meta);
        a.v_meta = static_cast<const uint32_t *>(c->buf.v_token_meta);
        a.q = q;
        a.partial = partial;
        a.meta_stride = c->max_tokens;
        a.B = B;
        a.index_words = c->index_words;
        a.H = Hs;
        a.dup = c->head_split;
        a.n_blocks = n_blocks;
        a.blocks_per_split = (n_blocks + n_splits - 1) / n_splits;
        a.sm_log2 = sm_log2;
        n_splits = (n_blocks + a.blocks_per_split - 1) / a.blocks_per_split;
        dim3 grid(n_splits, B * Hs);
        if (c->cfg.pack_size == 8) {
#define PACKKV_LAUNCH_A8NN(g) hipLaunchKernelGGL((attn8_kernel<g, false, false>), grid, dim3(256), 0, s, a)
#define PACKKV_LAUNCH_A8WN(g) hipLaunchKernelGGL((attn8_kernel<g, true, false>), grid, dim3(256), 0, s, a)
#define PACKKV_LAUNCH_A8NW(g) hipLaunchKernelGGL((attn8_kernel<g, false, true>), grid, dim3(256), 0, s, a)
#define PACKKV_LAUNCH_A8WW(g) hipLaunchKernelGGL((attn8_kernel<g, true, true>), grid, dim3(256), 0, s, a)
#define PACKKV_LAUNCH_A(g) hipLaunchKernelGGL((attn_kernel<g, false>), grid, dim3(256), 0, s, a)
#define PACKKV_LAUNCH_AH(g) hipLaunchKernelGGL((attn_kernel<g, true>), grid, dim3(256), 0, s, a)
            if (c->wide_k && c->wide_v) {
                PACKKV_DISPATCH_GROUP(G, PACKKV_LAUNCH_A8WW)
            } else if (c->wide_k) {
                PACKKV_DISPATCH_GROUP(G, PACKKV_LAUNCH_A8WN)
            } else if (c->wide_v) {
                PACKKV_DISPATCH_GROUP(G, PACKKV_LAUNCH_A8NW)
            } else {
                PACKKV_DISPATCH_GROUP(G, PACKKV_LAUNCH_A8NN)
            }
        } else if (c->qmax_v > 7) {
            PACKKV_DISPATCH_GROUP4(G, PACKKV_LAUNCH_AH)
        } else {
            PACKKV_DISPATCH_GROUP4(G, PACKKV_LAUNCH_A)
        }
#undef PACKKV_LAUNCH_A8NN
#undef PACKKV_LAUNCH_A8WN
#undef PACKKV_LAUNCH_A8NW
#undef PACKKV_LAUNCH_A8WW
#undef PACKKV_LAUNCH_A
#undef PACKKV_LAUNCH_AH
    }
    hipLaunchKernelGGL(attn_combine_kernel, dim3(B * H * Gq), dim3(256), 0, s, partial, n_splits,
                       B * H * Gq, q, static_cast<const __half *>(c->buf.k_tail),
                       static_cast<const __half *>(c->buf.v_tail), c->tail_tokens,
                       c->cfg.tail_capacity, H, Gq, sm_log2, out);
    KV_HIP_CHECK(hipGetLastError());
    return KV_OK;
}

}  // namespace packkv
