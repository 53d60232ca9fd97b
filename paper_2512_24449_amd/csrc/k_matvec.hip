// Fused K path (PackKV Sec. III-C.1): scores = sm_scale * Khat q, streaming the
// packed K cache once and unpacking in registers.
//
// The paper walks a 32-lane warp over K rows and reduces with a warp sum.
// Here a 64-lane wave owns whole chunks (64 tokens x 128 channels): lane l
// owns token group g = l/16 and channels 8*(l%16)..+7 (unpack.h).  It keeps 16
// per-token partial sums over its 8 channels, fed by mixed-precision FMAs that
// read the unpacked fp16 code halves directly; a reduce-scatter inside the
// 16-lane row then leaves token 16g+i's dot product in lane 16g+i and the 64
// scores leave as one coalesced 256-byte store.  De-quantization is folded in:
//   score_t = sm_scale * (scale_t * (sum_d q_d code[t,d] + sum_d q_d m[g,d])
//                         + min_t * sum_d q_d)
// so a pack minimum costs one FMA per pack and (scale_t, min_t) one per token.
// A workgroup of four waves walks a contiguous range of blocks of one
// (batch, kv-head) stream; every wave double-buffers whole chunks in LDS with
// direct global->LDS transfers, so the next chunk is in flight while the
// current one is unpacked; the raw fp16 tail is handled by extra workgroups of
// the same launch (one launch covers everything, Sec. III-B.4).
#include <algorithm>

#include "unpack.h"

namespace packkv {

struct KArgs {
    const uint8_t *arena;
    const uint32_t *index;
    const uint32_t *meta;   // [B][meta_stride]
    const __half *q;        // [B][Hq][128]
    float *scores;          // [B][Hq][ld]
    const __half *tail;     // [B][tail_cap][H][128]
    int64_t ld;
    int64_t meta_stride;
    int64_t packed_tokens;
    int B, H;
    int n_blocks;           // packed blocks per stream
    int blocks_per_group;   // blocks walked by one workgroup
    int groups_per_stream;
    int n_stream_groups;    // workgroups that process chunks
    int n_tail, tail_cap;
    float sm_scale;
};

// lds0: the workgroup's chunk buffers; this wave owns the two buffers at byte
// offsets buf_base and buf_base + CHUNK_LDS.
template <int G>
__device__ inline void k_stream(const KArgs &a, int bh, int blk_begin, int blk_end, int wave,
                                int lane, uint8_t *lds0, int buf_base, const uint4 *table) {
    const int h = bh % a.H, b = bh / a.H;
    const int ch0 = 8 * (lane & 15);
    // query slices of this lane's 8 channels, for the G query heads of kv-head h
    float qf[G][8], qsum[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        uint4 raw = *reinterpret_cast<const uint4 *>(a.q + (int64_t(b) * a.H * G + h * G + g) * D + ch0);
        const __half *hq = reinterpret_cast<const __half *>(&raw);
        float s = 0.0f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            qf[g][j] = __half2float(hq[j]);
            s += qf[g][j];
        }
        qsum[g] = row_all_reduce16(s);
    }

    for (int first = blk_begin + wave; first < blk_end; first += 4 * 64) {
        IndexBatch ib;
        ib.load(a.index, first, 4, blk_end, a.B, a.H, b, h, lane);
        const int n_it = min(64, (blk_end - first + 3) / 4);
        chunk_issue_lds(a.arena, ib.start16(0), ib.end16(0), lds0 + buf_base, lane);
        uint32_t mt_next = a.meta[b * a.meta_stride + int64_t(first) * N + lane];
        for (int it = 0; it < n_it; ++it) {
            const int cur = buf_base + (it & 1) * CHUNK_LDS;
            const int64_t tok = int64_t(first + 4 * it) * N + lane;  // this lane's token after the reduction
            const bool valid = ib.end16(it) - ib.start16(it) >= uint32_t(HEADER / 16);
            wait_chunk_landed();
            const uint32_t mt = mt_next;
            // the next chunk streams into the other buffer while this one is unpacked
            if (it + 1 < n_it) {
                chunk_issue_lds(a.arena, ib.start16(it + 1), ib.end16(it + 1),
                                lds0 + buf_base + ((it + 1) & 1) * CHUNK_LDS, lane);
                mt_next = a.meta[b * a.meta_stride + int64_t(first + 4 * (it + 1)) * N + lane];
            }
            if (!valid) {  // block dropped by an arena overflow: defined output
#pragma unroll
                for (int g = 0; g < G; ++g)
                    a.scores[(int64_t(b) * a.H * G + h * G + g) * a.ld + tok] = 0.0f;
                continue;
            }
            const uint2 hdr = *reinterpret_cast<const uint2 *>(lds0 + cur + lane * 8);
            LanePacks lp;
            lp.init(hdr.x, hdr.y, cur + HEADER);

            float acc[G][16], msum[G];
#pragma unroll
            for (int g = 0; g < G; ++g) {
                msum[g] = 0.0f;
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[g][i] = 0.0f;
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                uint32_t P[8];
                const PackRaw raw = fetch_pack(lds0, table, lp.pos(j), lp.header_byte(j));
                expand_pack(raw, P);
                const float m = __uint_as_float(raw.k.w);
#pragma unroll
                for (int g = 0; g < G; ++g) msum[g] = fmaf(qf[g][j], m, msum[g]);
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    // P[k] holds tokens (k, k+8) of the group
                    const float cl = half_lo(P[k]), chh = half_hi(P[k]);
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        acc[g][k] = fmaf(qf[g][j], cl, acc[g][k]);
                        acc[g][k + 8] = fmaf(qf[g][j], chh, acc[g][k + 8]);
                    }
                }
            }

            const float scale = __half2float(__ushort_as_half(uint16_t(mt & 0xFFFFu)));
            const float mn = __half2float(__ushort_as_half(uint16_t(mt >> 16)));
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const float dot = row_reduce_scatter16(acc[g], lane) * CODE_SCALE;
                const float ms = row_all_reduce16(msum[g]);
                a.scores[(int64_t(b) * a.H * G + h * G + g) * a.ld + tok] =
                    a.sm_scale * fmaf(scale, dot + ms, mn * qsum[g]);
            }
        }
        wait_chunk_landed();  // nothing may still be streaming into LDS when the buffers are reused
    }
}

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float float4_u __attribute__((ext_vector_type(4), aligned(4)));

// Matrix-core form of the K walk.  The codes of a pack sit along the token axis
// inside a lane, the dot product runs along the channel axis across lanes, so the
// wave first turns the tile with a 0/1 selection product and then contracts it
// with q:
//   C1[channel i][column n] = sum_k A1[i][k] S_x[k][n]         (16x16x32 fp16 MFMA)
//     A1: the unpacked words of pack slot j (row i = lane%16 = channel 8i+j, the
//         32 k-slots = 8 tokens of each token group lane/16), S_x: selects the
//         16 k-slots with bit 1 of the in-lane slot equal to x, times 2^10
//   C2[head][column n] += sum_k Q[head][k] cvt16(C1)[k][n]      (16x16x32 fp16 MFMA)
//     the fp32 tile C1 of lane (r, n) holds channels 4r..4r+3 of column n, which is
//     exactly the k-run a B operand lane needs; two pack slots fill its 8 k-values.
// Every value in C1 is an integer code times 2^-14, so its fp16 conversion is
// exact.  With the k-slot -> column assignment below, lane n (< 16) ends up with
// four consecutive tokens of the block, 16*(n>>2) + 4*((n>>1)&1) + 8*(n&1) + {0..3},
// in the four accumulators, for the heads 4*(lane/16)..+3 in their four registers.
template <int G>
__device__ inline void k_stream_mfma(const KArgs &a, int bh, int blk_begin, int blk_end, int wave,
                                     int lane, uint8_t *lds0, int buf_base, const uint4 *table) {
    const int h = bh % a.H, b = bh / a.H;
    const int row = lane >> 4, col = lane & 15;
    const int64_t head0 = int64_t(b) * a.H * G + h * G;

    // q of this lane's 8 channels as fp16 pairs (pack-minimum term) and its sum per head
    uint32_t qh[G][4];
    float qsum[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const uint4 raw = *reinterpret_cast<const uint4 *>(a.q + (head0 + g) * D + 8 * col);
        qh[g][0] = raw.x, qh[g][1] = raw.y, qh[g][2] = raw.z, qh[g][3] = raw.w;
        float s = 0.0f;
#pragma unroll
        for (int k = 0; k < 4; ++k) s += half_lo(qh[g][k]) + half_hi(qh[g][k]);
        qsum[g] = row_all_reduce16(s);
    }
    // Q operands of the second product, one per pair of pack slots (2jp, 2jp+1): row = head
    // lane%16, k-value e of k-run lane/16 = channel 8*(4*(lane/16) + (e&3)) + 2jp + (e>>2)
    half8 qA[4];
    {
        uint32_t rw[4][4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            uint4 raw = make_uint4(0, 0, 0, 0);
            if (col < G) raw = *reinterpret_cast<const uint4 *>(a.q + (head0 + col) * D + 8 * (4 * row + e));
            rw[e][0] = raw.x, rw[e][1] = raw.y, rw[e][2] = raw.z, rw[e][3] = raw.w;
        }
#pragma unroll
        for (int jp = 0; jp < 4; ++jp) {
            const uint32_t w0 = __builtin_amdgcn_perm(rw[1][jp], rw[0][jp], 0x05040100u);
            const uint32_t w1 = __builtin_amdgcn_perm(rw[3][jp], rw[2][jp], 0x05040100u);
            const uint32_t w2 = __builtin_amdgcn_perm(rw[1][jp], rw[0][jp], 0x07060302u);
            const uint32_t w3 = __builtin_amdgcn_perm(rw[3][jp], rw[2][jp], 0x07060302u);
            qA[jp] = __builtin_bit_cast(half8, u32x4{w0, w1, w2, w3});
        }
    }
    // selection operands: lane (k-run kg = lane/16, column n = lane%16) holds S_x[8kg+e][n];
    // slot e of run kg goes to column 4kg + 2(e>>2) + (e&1) when ((e>>1)&1) == x
    half8 sel[2];
#pragma unroll
    for (int x = 0; x < 2; ++x) {
        uint32_t wsel[4] = {0, 0, 0, 0};
        const int e = ((col >> 1) & 1) * 4 + x * 2 + (col & 1);
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if ((col >> 2) == row && (e >> 1) == k) wsel[k] = 0x6400u << (16 * (e & 1));  // fp16 1024
        sel[x] = __builtin_bit_cast(half8, u32x4{wsel[0], wsel[1], wsel[2], wsel[3]});
    }
    // this lane's four output tokens inside a block, the heads it holds, where its
    // token group's pack-minimum sums come from
    const int tok_base = 16 * (col >> 2) + 4 * ((col >> 1) & 1) + 8 * (col & 1);
    const int src_lane = 16 * (col >> 2);
    float qs[4];
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        qs[x] = x < G ? qsum[x] : 0.0f;
        if (G > 4 && row == 1) qs[x] = qsum[(4 + x) % G];
    }
    const bool writer = 4 * row < G;
    constexpr float OUT_SCALE = 16384.0f;  // codes enter as code * 2^-24, selection adds 2^10

    for (int first = blk_begin + wave; first < blk_end; first += 4 * 64) {
        IndexBatch ib;
        ib.load(a.index, first, 4, blk_end, a.B, a.H, b, h, lane);
        const int n_it = min(64, (blk_end - first + 3) / 4);
        chunk_issue_lds(a.arena, ib.start16(0), ib.end16(0), lds0 + buf_base, lane);
        const uint32_t *meta = a.meta + b * a.meta_stride + tok_base;
        uint4 mt_next = *reinterpret_cast<const uint4 *>(meta + int64_t(first) * N);
        for (int it = 0; it < n_it; ++it) {
            const int cur = buf_base + (it & 1) * CHUNK_LDS;
            const int64_t tok = int64_t(first + 4 * it) * N + tok_base;
            const bool valid = ib.end16(it) - ib.start16(it) >= uint32_t(HEADER / 16);
            wait_chunk_landed();
            const uint4 mt = mt_next;
            // the next chunk streams into the other buffer while this one is unpacked
            if (it + 1 < n_it) {
                chunk_issue_lds(a.arena, ib.start16(it + 1), ib.end16(it + 1),
                                lds0 + buf_base + ((it + 1) & 1) * CHUNK_LDS, lane);
                mt_next = *reinterpret_cast<const uint4 *>(meta + int64_t(first + 4 * (it + 1)) * N);
            }
            if (!valid) {  // block dropped by an arena overflow: defined output
                if (writer) {
#pragma unroll
                    for (int x = 0; x < 4; ++x)
                        if (4 * row + x < G)
                            *reinterpret_cast<float4_u *>(a.scores + (head0 + 4 * row + x) * a.ld + tok) =
                                float4_u{0.0f, 0.0f, 0.0f, 0.0f};
                }
                continue;
            }
            const uint2 hdr = *reinterpret_cast<const uint2 *>(lds0 + cur + lane * 8);
            LanePacks lp;
            lp.init(hdr.x, hdr.y, cur + HEADER);

            float4_t acc[4];  // [token offset 0..3] x [head register]
#pragma unroll
            for (int t = 0; t < 4; ++t) acc[t] = float4_t{0.0f, 0.0f, 0.0f, 0.0f};
            float msum[G];
#pragma unroll
            for (int g = 0; g < G; ++g) msum[g] = 0.0f;
            const float4_t zero = float4_t{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int jp = 0; jp < 4; ++jp) {
                float4_t c1[2][4];
#pragma unroll
                for (int jj = 0; jj < 2; ++jj) {
                    const int j = 2 * jp + jj;
                    uint32_t P[8];
                    const PackRaw raw = fetch_pack(lds0, table, lp.pos(j), lp.header_byte(j));
                    expand_pack(raw, P);
                    const float m = __uint_as_float(raw.k.w);
#pragma unroll
                    for (int g = 0; g < G; ++g)
                        msum[g] = fmaf(jj ? half_hi(qh[g][jp]) : half_lo(qh[g][jp]), m, msum[g]);
                    // P[t + 2i]: tokens (t + 2i, t + 2i + 8); column token offset t = parity + 2x
                    const half8 a0 = __builtin_bit_cast(half8, u32x4{P[0], P[2], P[4], P[6]});
                    const half8 a1 = __builtin_bit_cast(half8, u32x4{P[1], P[3], P[5], P[7]});
                    c1[jj][0] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0, sel[0], zero, 0, 0, 0);
                    c1[jj][1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1, sel[0], zero, 0, 0, 0);
                    c1[jj][2] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0, sel[1], zero, 0, 0, 0);
                    c1[jj][3] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1, sel[1], zero, 0, 0, 0);
                }
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const u32x4 bw = {
                        __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(c1[0][t][0], c1[0][t][1])),
                        __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(c1[0][t][2], c1[0][t][3])),
                        __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(c1[1][t][0], c1[1][t][1])),
                        __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(c1[1][t][2], c1[1][t][3]))};
                    acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(qA[jp], __builtin_bit_cast(half8, bw),
                                                                     acc[t], 0, 0, 0);
                }
            }

            // pack-minimum term of this lane's token group, per head register
            float ms[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const float v = __shfl(row_all_reduce16(msum[g]), src_lane);
                if (g < 4) {
                    if (G <= 4 || row == 0) ms[g] = v;
                } else if (row == 1) {
                    ms[g - 4] = v;
                }
            }
            if (writer) {
                const uint32_t mtw[4] = {mt.x, mt.y, mt.z, mt.w};
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    if (4 * row + x < G) {
                        float4_u o;
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            const float scale = __half2float(__ushort_as_half(uint16_t(mtw[t] & 0xFFFFu)));
                            const float mn = __half2float(__ushort_as_half(uint16_t(mtw[t] >> 16)));
                            o[t] = a.sm_scale * fmaf(scale, acc[t][x] * OUT_SCALE + ms[x], mn * qs[x]);
                        }
                        *reinterpret_cast<float4_u *>(a.scores + (head0 + 4 * row + x) * a.ld + tok) = o;
                    }
                }
            }
        }
        wait_chunk_landed();  // nothing may still be streaming into LDS when the buffers are reused
    }
}

// Raw fp16 tail (Sec. III-B.1 buffer): plain dot products, one lane per token.
template <int G>
__device__ inline void k_tail(const KArgs &a, int bh, int lane) {
    const int h = bh % a.H, b = bh / a.H;
    if (lane >= a.n_tail) return;
    const __half *row = a.tail + ((int64_t(b) * a.tail_cap + lane) * a.H + h) * D;
    float acc[G];
#pragma unroll
    for (int g = 0; g < G; ++g) acc[g] = 0.0f;
    for (int d0 = 0; d0 < D; d0 += 8) {
        uint4 raw = *reinterpret_cast<const uint4 *>(row + d0);
        const __half *kv = reinterpret_cast<const __half *>(&raw);
#pragma unroll
        for (int g = 0; g < G; ++g) {
            uint4 qraw = *reinterpret_cast<const uint4 *>(a.q + (int64_t(b) * a.H * G + h * G + g) * D + d0);
            const __half *qv = reinterpret_cast<const __half *>(&qraw);
#pragma unroll
            for (int k = 0; k < 8; ++k) acc[g] = fmaf(__half2float(qv[k]), __half2float(kv[k]), acc[g]);
        }
    }
#pragma unroll
    for (int g = 0; g < G; ++g)
        a.scores[(int64_t(b) * a.H * G + h * G + g) * a.ld + a.packed_tokens + lane] = a.sm_scale * acc[g];
}

template <int G>
__global__ __launch_bounds__(256) void k_matvec_kernel(KArgs a) {
    __shared__ __attribute__((aligned(16))) uint8_t lds_all[4 * 2 * CHUNK_LDS + LDS_TAIL_PAD];
    __shared__ uint4 table[PACK_TABLE_ENTRIES];
    build_pack_table(table);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int grp = blockIdx.x;
    if (grp < a.n_stream_groups) {
        const int bh = grp / a.groups_per_stream;
        const int part = grp % a.groups_per_stream;
        const int blk_begin = part * a.blocks_per_group;
        const int blk_end = min(blk_begin + a.blocks_per_group, a.n_blocks);
        // one query head per kv-head: plain FMAs cost the same issue slots as the two matrix
        // products and need fewer registers; with grouped queries the unpack is shared by
        // the G heads only in the matrix-core form
        if constexpr (G == 1)
            k_stream<G>(a, bh, blk_begin, blk_end, wave, lane, lds_all, wave * 2 * CHUNK_LDS, table);
        else
            k_stream_mfma<G>(a, bh, blk_begin, blk_end, wave, lane, lds_all, wave * 2 * CHUNK_LDS, table);
    } else {
        const int bh = (grp - a.n_stream_groups) * 4 + wave;
        if (bh < a.B * a.H) k_tail<G>(a, bh, lane);
    }
}

int launch_k_matvec(const kv_cache *c, const __half *q, float sm_scale, float *scores,
                    int64_t ld_scores, hipStream_t s) {
    KArgs a;
    a.arena = static_cast<const uint8_t *>(c->buf.k_arena);
    a.index = static_cast<const uint32_t *>(c->buf.k_index);
    a.meta = static_cast<const uint32_t *>(c->buf.k_token_meta);
    a.q = q;
    a.scores = scores;
    a.tail = static_cast<const __half *>(c->buf.k_tail);
    a.ld = ld_scores;
    a.meta_stride = c->max_tokens;
    a.packed_tokens = c->packed_tokens;
    a.B = c->cfg.batch;
    a.H = c->cfg.n_kv_heads;
    a.n_blocks = int(c->packed_tokens / N);
    const int streams = a.B * a.H;
    // never less than one block per wave
    const int64_t want_groups =
        std::max<int64_t>(1, target_workgroups(int64_t(a.n_blocks) * streams) / streams);
    int bpg = int((a.n_blocks + want_groups - 1) / want_groups);
    bpg = std::max(4, (bpg + 3) / 4 * 4);
    a.blocks_per_group = bpg;
    a.groups_per_stream = a.n_blocks > 0 ? (a.n_blocks + bpg - 1) / bpg : 0;
    a.n_stream_groups = a.groups_per_stream * streams;
    a.n_tail = c->tail_tokens;
    a.tail_cap = c->cfg.tail_capacity;
    a.sm_scale = sm_scale;
    const int tail_groups = a.n_tail > 0 ? (streams + 3) / 4 : 0;
    const int grid = a.n_stream_groups + tail_groups;
    if (grid == 0) return KV_OK;
    switch (c->group) {
        case 1: hipLaunchKernelGGL(k_matvec_kernel<1>, dim3(grid), dim3(256), 0, s, a); break;
        case 2: hipLaunchKernelGGL(k_matvec_kernel<2>, dim3(grid), dim3(256), 0, s, a); break;
        case 4: hipLaunchKernelGGL(k_matvec_kernel<4>, dim3(grid), dim3(256), 0, s, a); break;
        case 8: hipLaunchKernelGGL(k_matvec_kernel<8>, dim3(grid), dim3(256), 0, s, a); break;
        default: return KV_ERR_UNSUPPORTED;
    }
    KV_HIP_CHECK(hipGetLastError());
    return KV_OK;
}

}  // namespace packkv
