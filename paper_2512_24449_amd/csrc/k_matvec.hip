// Fused K path (PackKV Sec. III-C.1): scores = sm_scale * Khat q, streaming the packed K cache
// once and decoding it on chip.
//
// The paper walks a 32-lane warp over K rows and reduces with a warp sum.  Here a 64-lane wave
// owns whole chunks (64 tokens x 128 channels).  Chunks with packs of 16 tokens (plane layout)
// are turned in LDS and contracted on the matrix cores for all query heads of the kv-head at
// once (k_planes.h); chunks with packs of 8 tokens and wide chunks have their own kernels here
// and their helpers in pack8.h.  De-quantization is folded in:
//   score_t = sm_scale * (scale_t * (sum_d q_d code[t,d] + sum_d q_d m[g,d])
//                         + min_t * sum_d q_d)
// so the pack minimums cost a few instructions per chunk and (scale_t, min_t) one FMA per token.
// Whole chunks travel global memory -> LDS directly, the next one while the current one is
// decoded; the raw fp16 tail is handled by extra workgroups of the same launch (one launch covers
// everything, Sec. III-B.4).
#include <algorithm>

#include "k_planes.h"
#include "pack8.h"

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
    int index_words;        // index words per chunk: 1 back to back, 2 with a paged arena
    int dup;                // H counts every kv-head dup times (query groups above 8 are split): kv-head = h / dup
    int n_blocks;           // packed blocks per stream
    int blocks_per_group;   // blocks walked by one workgroup
    int groups_per_stream;
    int n_stream_groups;    // workgroups that process chunks
    int n_tail, tail_cap;
    float sm_scale;
};

// Packs of 8 tokens (Sec. IV-B), any group size: every chunk is decoded as two halves of 32
// tokens (pack8.h).  After the two reductions lane (r, i) holds token 32 (i & 1) + 8 r + (i >> 1)
// of the block, for every head; one 256-byte store per head.
template <int G>
__device__ inline void k8_stream(const KArgs &a, int bh, int blk_begin, int blk_end, int wave, int lane,
                                 uint8_t *lds0, int buf_base, const uint2 *table) {
    const int h = bh % a.H, b = bh / a.H;
    const int64_t head0 = int64_t(b) * a.H * G + h * G;
    KQuery8<G> kq;
    kq.load(a.q + head0 * D, lane);
    const int row = lane >> 4, i = lane & 15;
    const int tok_in_blk = 32 * (i & 1) + 8 * row + k8_token_of_lane(i);

    for (int first = blk_begin + wave; first < blk_end; first += 4 * 64) {
        IndexBatch ib;
        ib.load(a.index, a.index_words, first, 4, blk_end, a.B, a.H / a.dup, b, h / a.dup, lane);
        const int n_it = min(64, (blk_end - first + 3) / 4);
        vmem_order_fence();
        chunk_issue_lds<CHUNK8_MAX, HEADER8>(a.arena, ib.start16(0), ib.end16(0), lds0 + buf_base, lane);
        vmem_order_fence();
        const uint32_t *meta = a.meta + b * a.meta_stride + tok_in_blk;
        uint32_t mt_next = meta[int64_t(first) * N];
        for (int it = 0; it < n_it; ++it) {
            const int cur = buf_base + (it & 1) * CHUNK8_LDS;
            const int64_t tok = int64_t(first + 4 * it) * N + tok_in_blk;
            const bool valid = ib.end16(it) - ib.start16(it) >= uint32_t(HEADER8 / 16);
            // issued after this chunk's transfers, and allowed to stay in flight: the metadata
            // load and, from the second iteration on, the previous iteration's G score stores
            if (it == 0)
                wait_chunk_landed_except<1>();
            else
                wait_chunk_landed_except<1 + G>();
            uint32_t mt = mt_next;
            consume_here(mt);
            if (it + 1 < n_it) {
                chunk_issue_lds<CHUNK8_MAX, HEADER8>(a.arena, ib.start16(it + 1), ib.end16(it + 1),
                                                     lds0 + buf_base + ((it + 1) & 1) * CHUNK8_LDS, lane);
                vmem_order_fence();
                mt_next = meta[int64_t(first + 4 * (it + 1)) * N];
            }
            if (!valid) {  // block dropped by an arena overflow: no softmax weight
#pragma unroll
                for (int g = 0; g < G; ++g) a.scores[(head0 + g) * a.ld + tok] = -INFINITY;
                wait_chunk_landed();  // rare path: keep the next wait's count independent of it
                continue;
            }
            float u0[G], u1[G];
            const uint2 hdr0 = *reinterpret_cast<const uint2 *>(lds0 + cur + lane * 8);
            LanePacks8 lp0;
            lp0.init(hdr0.x, hdr0.y, cur + HEADER8);
            k8_half<G>(lds0, table, lp0, kq, lane, u0);
            const uint2 hdr1 = *reinterpret_cast<const uint2 *>(lds0 + cur + 512 + lane * 8);
            LanePacks8 lp1;
            lp1.init(hdr1.x, hdr1.y, lp0.end_all);
            k8_half<G>(lds0, table, lp1, kq, lane, u1);
            const float scale = __half2float(__ushort_as_half(uint16_t(mt & 0xFFFFu)));
            const float mn = __half2float(__ushort_as_half(uint16_t(mt >> 16)));
#pragma unroll
            for (int g = 0; g < G; ++g)
                a.scores[(head0 + g) * a.ld + tok] =
                    a.sm_scale * fmaf(scale, (i & 1) ? u1[g] : u0[g], mn * kq.qsum[g]);
        }
        wait_chunk_landed();  // nothing may still be streaming into LDS when the buffers are reused
    }
}

// Wide chunks (codes above 15; pack8.h): same result layout as k8_stream.  A wide chunk is up to
// 10 KB, so each wave has one buffer: the transfer is waited for before the unpack starts, and
// the overlap comes from the other waves of the compute unit only.
template <int G>
__device__ inline void kw_stream(const KArgs &a, int bh, int blk_begin, int blk_end, int wave, int lane,
                                 uint8_t *lds0, int buf, const uint2 *ktable) {
    const int h = bh % a.H, b = bh / a.H;
    const int64_t head0 = int64_t(b) * a.H * G + h * G;
    KQuery8<G> kq;
    kq.load(a.q + head0 * D, lane);
    const int tok_in_blk = k8_token_of_block_lane(lane);
    const uint32_t *meta = a.meta + b * a.meta_stride + tok_in_blk;

    for (int first = blk_begin + wave; first < blk_end; first += 4 * 64) {
        IndexBatch ib;
        ib.load(a.index, a.index_words, first, 4, blk_end, a.B, a.H / a.dup, b, h / a.dup, lane);
        const int n_it = min(64, (blk_end - first + 3) / 4);
        for (int it = 0; it < n_it; ++it) {
            const int64_t tok = int64_t(first + 4 * it) * N + tok_in_blk;
            const bool valid = ib.end16(it) - ib.start16(it) >= uint32_t(HEADERW / 16);
            chunk_issue_lds<CHUNKW_MAX, HEADERW>(a.arena, ib.start16(it), ib.end16(it), lds0 + buf, lane);
            const uint32_t mt = meta[int64_t(first + 4 * it) * N];
            wait_chunk_landed();
            if (!valid) {  // block dropped by an arena overflow: no softmax weight
#pragma unroll
                for (int g = 0; g < G; ++g) a.scores[(head0 + g) * a.ld + tok] = -INFINITY;
                continue;
            }
            float u0[G], u1[G];
            const uint2 w0 = *reinterpret_cast<const uint2 *>(lds0 + buf + lane * 8);
            const uint2 m0 = *reinterpret_cast<const uint2 *>(lds0 + buf + 1024 + lane * 8);
            LanePacksW lp0;
            lp0.init(w0, m0, buf + HEADERW);
            kw_half<G>(lds0, ktable, lp0, kq, lane, u0);
            const uint2 w1 = *reinterpret_cast<const uint2 *>(lds0 + buf + 512 + lane * 8);
            const uint2 m1 = *reinterpret_cast<const uint2 *>(lds0 + buf + 1536 + lane * 8);
            LanePacksW lp1;
            lp1.init(w1, m1, lp0.end_all);
            kw_half<G>(lds0, ktable, lp1, kq, lane, u1);
            const float scale = __half2float(__ushort_as_half(uint16_t(mt & 0xFFFFu)));
            const float mn = __half2float(__ushort_as_half(uint16_t(mt >> 16)));
#pragma unroll
            for (int g = 0; g < G; ++g)
                a.scores[(head0 + g) * a.ld + tok] =
                    a.sm_scale * fmaf(scale, (lane & 1) ? u1[g] : u0[g], mn * kq.qsum[g]);
            lds_reads_returned();  // one buffer: read completely before the next transfer overwrites it
        }
    }
}

// Raw fp16 tail (Sec. III-B.1 buffer): plain dot products, one lane per token.
template <int G>
__device__ inline void k_tail(const KArgs &a, int bh, int lane) {
    const int h = bh % a.H, b = bh / a.H;
    if (lane >= a.n_tail) return;
    const __half *row = a.tail + ((int64_t(b) * a.tail_cap + lane) * (a.H / a.dup) + h / a.dup) * D;
    // the whole row first: sixteen independent 16-byte loads, one memory latency
    uint4 kr[D / 8];
#pragma unroll
    for (int i = 0; i < D / 8; ++i) kr[i] = *reinterpret_cast<const uint4 *>(row + 8 * i);
    float acc[G];
#pragma unroll
    for (int g = 0; g < G; ++g) acc[g] = 0.0f;
#pragma unroll
    for (int i = 0; i < D / 8; ++i) {
        const __half *kv = reinterpret_cast<const __half *>(&kr[i]);
#pragma unroll
        for (int g = 0; g < G; ++g) {
            uint4 qraw = *reinterpret_cast<const uint4 *>(a.q + (int64_t(b) * a.H * G + h * G + g) * D + 8 * i);
            const __half *qv = reinterpret_cast<const __half *>(&qraw);
#pragma unroll
            for (int k = 0; k < 8; ++k) acc[g] = fmaf(__half2float(qv[k]), __half2float(kv[k]), acc[g]);
        }
    }
#pragma unroll
    for (int g = 0; g < G; ++g)
        a.scores[(int64_t(b) * a.H * G + h * G + g) * a.ld + a.packed_tokens + lane] = a.sm_scale * acc[g];
}

// Packs of 16 tokens, plane layout (k_planes.h), G <= 4 heads per kv-head.  The chunks of all
// streams form one work list cut into equal ranges, one per workgroup (FlatPlan); the four waves
// of a workgroup take every fourth block of its range.  A wave keeps ONE chunk buffer and its
// tiles: the planes of a chunk are copied to the tiles in the first part of its decode, and the
// next chunk streams into the buffer during the rest (the products, the score exchange, the
// stores), so five workgroups fit a compute unit and their waves hide one another's waits.  The
// token metadata of a chunk travels the same way as the chunk (one dword per lane, global memory
// -> LDS, behind the chunk in its buffer).  Workgroups past the plan's take the raw fp16 tail.
template <int G>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(5))) void k_planes_kernel(KArgs a, FlatPlan plan) {
    constexpr int SIDE = CHUNK_MAX + LDS_TAIL_PAD;  // metadata row behind the chunk
    constexpr int BUF = SIDE + 256;
    static_assert(BUF % 16 == 0, "buffers are 16-byte aligned");
    __shared__ __attribute__((aligned(16))) uint8_t lds_all[4 * BUF];
    __shared__ __attribute__((aligned(16))) uint8_t tiles_all[4 * K_TILES_BYTES];
    __shared__ uint4 table[5];
    build_k_plane_table(table);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int grp = blockIdx.x;
    if (grp >= plan.n_groups) {
        const int bh = (grp - plan.n_groups) * 4 + wave;
        if (bh < a.B * a.H) k_tail<G>(a, bh, lane);
        return;
    }
    const int cur = wave * BUF;
    uint8_t *tiles = tiles_all + wave * K_TILES_BYTES;
    const int64_t range_end = plan.begin(grp + 1);

    for (int64_t f = plan.begin(grp); f < range_end;) {
        const int stream = int(f / plan.n_blocks);
        const int blk_begin = int(f - int64_t(stream) * plan.n_blocks);
        const int blk_end = int(min<int64_t>(plan.n_blocks, blk_begin + (range_end - f)));
        f += blk_end - blk_begin;
        const int h = stream % a.H, b = stream / a.H;
        const uint32_t *meta = a.meta + b * a.meta_stride;
        const int64_t head0 = int64_t(stream) * G;
        KQueryPlanes<G> kq;
        kq.fetch(a.q + head0 * D, lane);

        auto issue = [&](const IndexBatch &ib, int it, int blk) {
            uint8_t *buf = lds_all + cur;
            row_issue_lds(meta + int64_t(blk) * N, buf + SIDE, lane);
            chunk_issue_lds<CHUNK_MAX, HEADER, true>(a.arena, ib.start16(it), ib.end16(it), buf, lane);
        };
        // index words of up to 64 blocks of this wave, then the first chunk of the batch
        auto start_batch = [&](IndexBatch &ib, int first) {
            if (first >= blk_end) return;
            ib.load(a.index, a.index_words, first, 4, blk_end, a.B, a.H / a.dup, b, h / a.dup, lane);
            wait_chunk_landed();  // the index words and the query (the only loads the compiler sees)
            issue(ib, 0, first);
        };

        IndexBatch ib;
        start_batch(ib, blk_begin + wave);
        // the query operand is built while the first chunk is on its way, a quarter per wave (the tiles
        // of the workgroup are idle between two segments and carry the exchange)
        kq.build_shared(lane, wave, reinterpret_cast<uint32_t *>(tiles_all));
        for (int first = blk_begin + wave; first < blk_end; first += 4 * 64) {
            const int n_it = min(64, (blk_end - first + 3) / 4);
            for (int it = 0; it < n_it; ++it) {
                const bool valid = ib.end16(it) - ib.start16(it) >= uint32_t(HEADER / 16);
                wait_chunk_landed();  // chunk it with its metadata row (and the score stores before it)
                const int64_t tok = int64_t(first + 4 * it) * N + lane;
                const uint32_t mt = *reinterpret_cast<const uint32_t *>(lds_all + cur + SIDE + 4 * lane);
                auto refill = [&]() {
                    if (it + 1 < n_it) issue(ib, it + 1, first + 4 * (it + 1));
                };
                if (!valid) {  // block dropped by an arena overflow: no softmax weight
                    lds_reads_returned();
                    refill();
#pragma unroll
                    for (int g = 0; g < G; ++g) a.scores[(head0 + g) * a.ld + tok] = -INFINITY;
                    continue;
                }
                float u[G];
                k_planes_chunk<G>(lds_all, cur, table, tiles, kq, u, refill);
                const float scale = __half2float(__ushort_as_half(uint16_t(mt & 0xFFFFu)));
                const float mn = __half2float(__ushort_as_half(uint16_t(mt >> 16)));
#pragma unroll
                for (int g = 0; g < G; ++g)
                    a.scores[(head0 + g) * a.ld + tok] = a.sm_scale * fmaf(scale, u[g], mn * kq.qsum[g]);
            }
            wait_chunk_landed();
            start_batch(ib, first + 4 * 64);
        }
    }
}

template <int G>
__global__ __launch_bounds__(256) void k8_matvec_kernel(KArgs a) {
    __shared__ __attribute__((aligned(16))) uint8_t lds_all[4 * 2 * CHUNK8_LDS + LDS_TAIL_PAD];
    __shared__ uint2 table[PACK_TABLE_ENTRIES];
    build_pair_table(table);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int grp = blockIdx.x;
    if (grp < a.n_stream_groups) {
        const int bh = grp / a.groups_per_stream;
        const int part = grp % a.groups_per_stream;
        const int blk_begin = part * a.blocks_per_group;
        const int blk_end = min(blk_begin + a.blocks_per_group, a.n_blocks);
        k8_stream<G>(a, bh, blk_begin, blk_end, wave, lane, lds_all, wave * 2 * CHUNK8_LDS, table);
    } else {
        const int bh = (grp - a.n_stream_groups) * 4 + wave;
        if (bh < a.B * a.H) k_tail<G>(a, bh, lane);
    }
}

template <int G>
__global__ __launch_bounds__(256) void kw_matvec_kernel(KArgs a) {
    __shared__ __attribute__((aligned(16))) uint8_t lds_all[4 * CHUNKW_LDS + LDS_TAIL_PAD];
    __shared__ uint2 ktable[16];
    build_wide_tables(ktable, nullptr);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int grp = blockIdx.x;
    if (grp < a.n_stream_groups) {
        const int bh = grp / a.groups_per_stream;
        const int part = grp % a.groups_per_stream;
        const int blk_begin = part * a.blocks_per_group;
        const int blk_end = min(blk_begin + a.blocks_per_group, a.n_blocks);
        kw_stream<G>(a, bh, blk_begin, blk_end, wave, lane, lds_all, wave * CHUNKW_LDS, ktable);
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
    a.index_words = c->index_words;
    a.dup = c->head_split;
    a.H = c->cfg.n_kv_heads * c->head_split;
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
#define PACKKV_LAUNCH_KW(g) hipLaunchKernelGGL(kw_matvec_kernel<g>, dim3(grid), dim3(256), 0, s, a)
#define PACKKV_LAUNCH_K8(g) hipLaunchKernelGGL(k8_matvec_kernel<g>, dim3(grid), dim3(256), 0, s, a)
    if (c->wide_k) {
        PACKKV_DISPATCH_GROUP(c->group, PACKKV_LAUNCH_KW)
    } else if (c->cfg.pack_size == 8) {
        PACKKV_DISPATCH_GROUP(c->group, PACKKV_LAUNCH_K8)
    } else {
        FlatPlan plan;
        plan.n_blocks = a.n_blocks;
        plan.total = int64_t(a.n_blocks) * streams;
        // one round of resident workgroups, never less than one block per wave
#define PACKKV_LAUNCH_KP(g)                                                                                   \
    {                                                                                                         \
        static const int per_cu = resident_workgroups(reinterpret_cast<const void *>(k_planes_kernel<g>));    \
        plan.n_groups = plan.total > 0 ? flat_groups_for(plan.total, per_cu, int64_t(1) << 30) : 0;  \
        hipLaunchKernelGGL(k_planes_kernel<g>, dim3(plan.n_groups + tail_groups), dim3(256), 0, s, a, plan); \
    }
        PACKKV_DISPATCH_GROUP4(c->group, PACKKV_LAUNCH_KP)
#undef PACKKV_LAUNCH_KP
    }
#undef PACKKV_LAUNCH_KW
#undef PACKKV_LAUNCH_K8
    KV_HIP_CHECK(hipGetLastError());
    return KV_OK;
}

}  // namespace packkv
