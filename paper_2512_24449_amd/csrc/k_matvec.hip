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
        k_stream<G>(a, bh, blk_begin, blk_end, wave, lane, lds_all, wave * 2 * CHUNK_LDS, table);
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
    // about 4096 workgroups over the chip, never less than one block per wave
    int64_t want_groups = std::max<int64_t>(1, 4096 / streams);
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
