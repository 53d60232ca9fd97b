// Fused V path (PackKV Sec. III-C.2): out = p^T Vhat, streaming the packed V cache once and
// decoding it on chip.
//
// The paper gives each thread one pack (a dot-product segment along ctx_len) and combines
// segments with fp32 atomic adds.  Here the contraction runs along the pack direction, so it maps
// onto the matrix cores without any transposition: the planes of a pack are FP4 operands as they
// are stored (v_planes.h; packs of 8 tokens and wide chunks: fp16 operands, pack8.h), the
// softmax weights times the token scales are the other operand, and the G query heads of a group
// share one decode.  Accumulation is fp32 inside the matrix instruction, in a fixed order: the
// context axis is split over workgroups whose partial sums are combined by a second small kernel
// -- no atomics, bitwise reproducible.  De-quantization is folded in:
//   out_d = sum_t w_t code[t,d] + sum_g m[g,d] sum_{t in g} w_t + sum_t p_t min_t
#include <algorithm>
#include <mutex>

#include "pack8.h"
#include "v_chunk.h"
#include "v_planes.h"

#ifndef PACKKV_V_NBUF
#define PACKKV_V_NBUF 2
#endif

namespace packkv {

struct VArgs {
    const uint8_t *arena;
    const uint32_t *index;
    const uint32_t *meta;   // [B][meta_stride]
    const float *p;         // [B][Hq][ld]
    float *partial;         // [splits][B*Hq][V_PART_STRIDE]
    int64_t ld;
    int64_t meta_stride;
    int B, H;
    int index_words;        // index words per chunk: 1 back to back, 2 with a paged arena
    int dup;                // H counts every kv-head dup times (query groups above 8 are split): kv-head = h / dup
    int n_blocks;           // packed blocks per stream
    int blocks_per_split;
};

// Packs of 16 tokens, plane layout (v_planes.h).  HIGH: the codes of the cache may need four bits
// (otherwise a chunk is at most 512 + 512 * 6 bytes).  The chunks of all streams form one work
// list that is cut into equal ranges, one per workgroup (FlatPlan): a launch is one round of
// long-lived workgroups whatever the numbers of streams and blocks are.  The four waves of a
// workgroup take every fourth block of its range.  A wave keeps NBUF chunk buffers: the next
// chunks stream in while one is decoded, and the token metadata and the weights of a chunk
// travel the same way (one dword per lane, global memory -> LDS, behind the chunk in its buffer):
// no vector memory instruction of the loop is visible to the compiler, so the only waits are the
// counted ones below.
template <int G, bool HIGH>
__global__ __launch_bounds__(256) void v_matvec_kernel(VArgs a, FlatPlan plan) {
    constexpr int CHUNK_BYTES = HIGH ? CHUNK_MAX : HEADER + PACKS * 6;
    constexpr int SLICES = (CHUNK_BYTES + 1023) / 1024;
    constexpr int SIDE = CHUNK_BYTES + LDS_TAIL_PAD;   // metadata row, then G weight rows
    constexpr int BUF = SIDE + (1 + G) * 256;          // bytes of one chunk buffer
    constexpr int NBUF = PACKKV_V_NBUF;                // chunks n+1 .. n+NBUF-1 in flight
    static_assert(NBUF == 2 || NBUF == 3, "wait counts below");
    // between the ranges of two streams the chunk buffers hold the cross-wave reduction array
    __shared__ __attribute__((aligned(16))) uint8_t lds_all[4 * NBUF * BUF];
    constexpr int VB = vb_bytes<G>();
    __shared__ __attribute__((aligned(16))) uint8_t vb_all[4 * VB];
    __shared__ uint4 table[PLANE_TABLE_ENTRIES];
    __shared__ uint32_t highs[PLANE_TABLE_ENTRIES];
    static_assert(sizeof(float) * 4 * G * (D + 4) <= 4 * NBUF * BUF, "reduction array must fit");
    static_assert(BUF % 16 == 0, "buffers are 16-byte aligned");
    float(*red)[G][D + 4] = reinterpret_cast<float(*)[G][D + 4]>(lds_all);
    for (int i = threadIdx.x; i < 4 * VB / 4; i += 256) reinterpret_cast<uint32_t *>(vb_all)[i] = 0;
    build_plane_table(table, highs);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int buf_base = wave * NBUF * BUF;
    uint8_t *vb = vb_all + wave * VB;
    const int grp = blockIdx.x;
    const int64_t range_end = plan.begin(grp + 1);

    for (int64_t f = plan.begin(grp); f < range_end;) {
        const int stream = int(f / plan.n_blocks);
        const int blk_begin = int(f - int64_t(stream) * plan.n_blocks);
        const int blk_end = int(min<int64_t>(plan.n_blocks, blk_begin + (range_end - f)));
        f += blk_end - blk_begin;
        const int h = stream % a.H, b = stream / a.H;
        const uint32_t *meta = a.meta + b * a.meta_stride;
        const float *prow = a.p + int64_t(stream) * G * a.ld;
        VPlaneState<G> st;
        st.clear();

        // everything chunk `blk` needs, into buffer `slot`: 1 + G row transfers, then the chunk
        // itself (with the streaming hint: the weights, which the softmax kernel has just written,
        // then stay in the caches); returns the number of transfer instructions of the chunk
        auto issue = [&](const IndexBatch &ib, int it, int blk, int slot) -> int {
            uint8_t *buf = lds_all + buf_base + slot * BUF;
            row_issue_lds(meta + int64_t(blk) * N, buf + SIDE, lane);
#pragma unroll
            for (int g = 0; g < G; ++g) row_issue_lds(prow + g * a.ld + int64_t(blk) * N, buf + SIDE + 256 * (1 + g), lane);
            return chunk_issue_lds_counted<CHUNK_BYTES, HEADER, true>(a.arena, ib.start16(it), ib.end16(it), buf, lane);
        };

        for (int first = blk_begin + wave; first < blk_end; first += 4 * 64) {
            IndexBatch ib;
            ib.load(a.index, a.index_words, first, 4, blk_end, a.B, a.H / a.dup, b, h / a.dup, lane);
            const int n_it = min(64, (blk_end - first + 3) / 4);
            wait_chunk_landed();  // the index words (the only loads the compiler sees)
            issue(ib, 0, first, 0);
            int slices_next = 0;  // transfer instructions of chunk it + 1
            if (NBUF == 3 && n_it > 1) slices_next = issue(ib, 1, first + 4, 1);
            int slot = 0;         // buffer of chunk it
            for (int it = 0; it < n_it; ++it) {
                const int cur = buf_base + slot * BUF;
                const bool valid = ib.end16(it) - ib.start16(it) >= uint32_t(HEADER / 16);
                // chunk it with its rows has landed; with three buffers the 1 + G rows and the
                // chunk of it + 1 may still be in flight
                if (NBUF == 3 && it + 1 < n_it)
                    wait_vmem_except<1 + G, SLICES>(slices_next);
                else
                    wait_chunk_landed();
                if (it + NBUF - 1 < n_it) {
                    // into the buffer chunk it - 1 was decoded from: its LDS reads have returned
                    lds_reads_returned();
                    slices_next = issue(ib, it + NBUF - 1, first + 4 * (it + NBUF - 1), slot == 0 ? NBUF - 1 : slot - 1);
                }
                slot = slot == NBUF - 1 ? 0 : slot + 1;
                if (!valid) continue;  // a block dropped by an arena overflow contributes nothing
                const uint32_t mt = *reinterpret_cast<const uint32_t *>(lds_all + cur + SIDE + 4 * lane);
                float pt[G];
#pragma unroll
                for (int g = 0; g < G; ++g)
                    pt[g] = *reinterpret_cast<const float *>(lds_all + cur + SIDE + 256 * (1 + g) + 4 * lane);
                v_planes_chunk<G, HIGH>(lds_all, cur, table, highs, vb, mt, pt, st);
            }
            wait_chunk_landed();
        }
        __syncthreads();  // every wave is done with its chunk buffers: reuse them as red[][][]

        v_planes_store<G>(st, red[wave], lane);
        __syncthreads();
        float *dst = a.partial + int64_t(grp + stream) * G * V_PART_STRIDE;
        for (int i = threadIdx.x; i < G * (D + 1); i += 256) {
            const int g = i / (D + 1), d = i % (D + 1);
            dst[g * V_PART_STRIDE + d] = (red[0][g][d] + red[1][g][d]) + (red[2][g][d] + red[3][g][d]);
        }
        __syncthreads();  // red[][][] has been read: the buffers may be filled again
    }
}

// The same for chunks with packs of 8 tokens (Sec. IV-B; pack8.h).
template <int G>
__global__ __launch_bounds__(256) void v8_matvec_kernel(VArgs a) {
    // two chunk buffers per wave; after the main loop the same memory holds the
    // cross-wave reduction array red[4][G][D + 4]
    __shared__ __attribute__((aligned(16))) uint8_t lds_all[4 * 2 * CHUNK8_LDS + LDS_TAIL_PAD];
    __shared__ __attribute__((aligned(16))) uint8_t blds_all[4 * BLds<G>::BYTES];
    __shared__ uint4 table[PACK_TABLE_ENTRIES];
    static_assert(sizeof(float) * 4 * G * (D + 4) <= 4 * 2 * CHUNK8_LDS, "reduction array must fit");
    float(*red)[G][D + 4] = reinterpret_cast<float(*)[G][D + 4]>(lds_all);
    build_pack_table(table, CODE_LIFT, fold_min<G>());

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int split = blockIdx.x;
    const int bh = blockIdx.y;
    const int h = bh % a.H, b = bh / a.H;
    const int buf_base = wave * 2 * CHUNK8_LDS;
    VLane<G> vl;
    vl.init(blds_all + wave * BLds<G>::BYTES, lane);
    vl.bslot = v8_bslot<G>(lane);  // lane l is token l of the block
    VState<G> st;
    st.clear();

    const int blk_begin = split * a.blocks_per_split;
    const int blk_end = min(blk_begin + a.blocks_per_split, a.n_blocks);
    for (int first = blk_begin + wave; first < blk_end; first += 4 * 64) {
        IndexBatch ib;
        ib.load(a.index, a.index_words, first, 4, blk_end, a.B, a.H / a.dup, b, h / a.dup, lane);
        const int n_it = min(64, (blk_end - first + 3) / 4);
        chunk_issue_lds<CHUNK8_MAX, HEADER8>(a.arena, ib.start16(0), ib.end16(0), lds_all + buf_base, lane);
        uint32_t mt_next = a.meta[b * a.meta_stride + int64_t(first) * N + lane];
        float p_next[G];
#pragma unroll
        for (int g = 0; g < G; ++g)
            p_next[g] = a.p[(int64_t(b) * a.H * G + h * G + g) * a.ld + int64_t(first) * N + lane];
        for (int it = 0; it < n_it; ++it) {
            const int cur = buf_base + (it & 1) * CHUNK8_LDS;
            const bool valid = ib.end16(it) - ib.start16(it) >= uint32_t(HEADER8 / 16);
            wait_chunk_landed();
            uint32_t mt = mt_next;
            consume_here(mt);
            float pt[G];
#pragma unroll
            for (int g = 0; g < G; ++g) {
                pt[g] = p_next[g];
                consume_here(pt[g]);
            }
            // the next chunk streams into the other buffer while this one is unpacked
            if (it + 1 < n_it) {
                chunk_issue_lds<CHUNK8_MAX, HEADER8>(a.arena, ib.start16(it + 1), ib.end16(it + 1),
                                lds_all + buf_base + ((it + 1) & 1) * CHUNK8_LDS, lane);
                const int64_t tok = int64_t(first + 4 * (it + 1)) * N + lane;
                mt_next = a.meta[b * a.meta_stride + tok];
#pragma unroll
                for (int g = 0; g < G; ++g) p_next[g] = a.p[(int64_t(b) * a.H * G + h * G + g) * a.ld + tok];
            }
            if (!valid) continue;  // a block dropped by an arena overflow contributes nothing
            v8_chunk<G>(lds_all, cur, table, vl, mt, pt, st);
        }
        wait_chunk_landed();
    }
    __syncthreads();  // every wave is done with its chunk buffers: reuse them as red[][][]

    v_state_store<G>(st, red[wave], lane);
    __syncthreads();
    for (int i = threadIdx.x; i < G * (D + 1); i += 256) {
        const int g = i / (D + 1), d = i % (D + 1);
        const float v = (red[0][g][d] + red[1][g][d]) + (red[2][g][d] + red[3][g][d]);
        a.partial[(int64_t(split) * a.B * a.H * G + (int64_t(b) * a.H * G + h * G + g)) * V_PART_STRIDE + d] = v;
    }
}

// Wide chunks (codes above 15; pack8.h): one buffer per wave (a chunk is up to 10 KB), so the
// transfer is waited for before the unpack; the other waves of the compute unit overlap with it.
template <int G>
__global__ __launch_bounds__(256) void vw_matvec_kernel(VArgs a) {
    __shared__ __attribute__((aligned(16))) uint8_t lds_all[4 * CHUNKW_LDS + LDS_TAIL_PAD];
    __shared__ __attribute__((aligned(16))) uint8_t blds_all[4 * BLds<G>::BYTES];
    __shared__ uint4 vtable[16];
    static_assert(sizeof(float) * 4 * G * (D + 4) <= 4 * CHUNKW_LDS, "reduction array must fit");
    float(*red)[G][D + 4] = reinterpret_cast<float(*)[G][D + 4]>(lds_all);
    build_wide_tables(nullptr, vtable);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int split = blockIdx.x;
    const int bh = blockIdx.y;
    const int h = bh % a.H, b = bh / a.H;
    const int buf = wave * CHUNKW_LDS;
    VLane<G> vl;
    vl.init(blds_all + wave * BLds<G>::BYTES, lane);
    vl.bslot = v8_bslot<G>(lane);  // lane l is token l of the block
    VState<G> st;
    st.clear();

    const int blk_begin = split * a.blocks_per_split;
    const int blk_end = min(blk_begin + a.blocks_per_split, a.n_blocks);
    for (int first = blk_begin + wave; first < blk_end; first += 4 * 64) {
        IndexBatch ib;
        ib.load(a.index, a.index_words, first, 4, blk_end, a.B, a.H / a.dup, b, h / a.dup, lane);
        const int n_it = min(64, (blk_end - first + 3) / 4);
        for (int it = 0; it < n_it; ++it) {
            const bool valid = ib.end16(it) - ib.start16(it) >= uint32_t(HEADERW / 16);
            lds_reads_returned();  // one buffer: the previous chunk has been read completely
            chunk_issue_lds<CHUNKW_MAX, HEADERW>(a.arena, ib.start16(it), ib.end16(it), lds_all + buf, lane);
            const int64_t tok = int64_t(first + 4 * it) * N + lane;
            const uint32_t mt = a.meta[b * a.meta_stride + tok];
            float pt[G];
#pragma unroll
            for (int g = 0; g < G; ++g) pt[g] = a.p[(int64_t(b) * a.H * G + h * G + g) * a.ld + tok];
            wait_chunk_landed();
            if (!valid) continue;  // a block dropped by an arena overflow contributes nothing
            vw_chunk<G>(lds_all, buf, vtable, vl, mt, pt, st);
        }
    }
    __syncthreads();  // every wave is done with its chunk buffer: reuse the memory as red[][][]

    v_state_store<G>(st, red[wave], lane, 1.0f);  // the wide path feeds the codes as numbers
    __syncthreads();
    for (int i = threadIdx.x; i < G * (D + 1); i += 256) {
        const int g = i / (D + 1), d = i % (D + 1);
        const float v = (red[0][g][d] + red[1][g][d]) + (red[2][g][d] + red[3][g][d]);
        a.partial[(int64_t(split) * a.B * a.H * G + (int64_t(b) * a.H * G + h * G + g)) * V_PART_STRIDE + d] = v;
    }
}

// Fixed-order combination of the split partial sums, plus the raw fp16 tail.  plan.n_groups > 0:
// the partial rows come from a kernel that walks the flat work list (kv-head group size Gk per
// stream); the row sets of stream s are those of the workgroups that hold one of its chunks.
__global__ __launch_bounds__(256) void v_reduce_kernel(const float *__restrict__ partial,
                                                       int n_splits, int n_rows, FlatPlan plan, int Gk,
                                                       const float *__restrict__ p, int64_t ld,
                                                       int64_t packed_tokens,
                                                       const __half *__restrict__ tail, int n_tail,
                                                       int tail_cap, int H, int G,
                                                       float *__restrict__ out) {
    __shared__ float lds[16][V_PART_STRIDE];
    __shared__ float wt[N];
    const int r = blockIdx.x;  // b*Hq + hq
    const int d = threadIdx.x;
    const int hq = r % (H * G), b = r / (H * G);
    const int h = hq / G;
    // every global load of the kernel is issued before the first result is needed
    SplitRows rows;
    TailRows trows;
    if (plan.n_groups > 0) {
        const int stream = r / Gk, g = r % Gk;
        const int w_lo = plan.group_of(int64_t(stream) * plan.n_blocks);
        const int w_hi = plan.group_of(int64_t(stream + 1) * plan.n_blocks - 1);
        n_splits = w_hi - w_lo + 1;
        rows.load_strided(partial + (int64_t(w_lo + stream) * Gk + g) * V_PART_STRIDE, n_splits, Gk);
    } else {
        rows.load(partial, n_splits, n_rows, r);
    }
    trows.load(tail + (int64_t(b) * tail_cap * H + h) * D, int64_t(H) * D, n_tail);
    if (d < n_tail) wt[d] = p[int64_t(r) * ld + packed_tokens + d];
    float pmin;
    float acc = rows.sum(n_splits, lds, &pmin);  // its barriers also publish wt
    acc += pmin;
    if (n_tail > 0) acc += trows.sum(wt, n_tail, lds);
    if (d < D) out[int64_t(r) * D + d] = acc;
}

int v_splits_for(int n_blocks, int streams) {
    const int64_t want = (target_workgroups(int64_t(n_blocks) * streams) + streams - 1) / streams;
    const int by_blocks = (n_blocks + 3) / 4;  // at least one block per wave
    int64_t s = want < by_blocks ? want : by_blocks;
    if (s > V_SPLITS_MAX) s = V_SPLITS_MAX;
    if (s < 1) s = 1;
    return int(s);
}

// partial: [splits][B * H_q][V_PART_STRIDE] floats for the split sums; max_split_rows: how many
// such rows it can take (the split count is lowered to fit).
// Workgroups of 256 threads of `kernel` that fit one compute unit (registers, LDS); 1 if the
// runtime cannot tell.
int resident_workgroups(const void *kernel) {
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kernel, 256, 0) != hipSuccess || n < 1) n = 1;
    return n;
}

// Workgroups for the flat work list of `total` chunks: one round of resident workgroups (per_cu
// of them fit a compute unit), never less than one block per wave, at most `most`.
int flat_groups_for(int64_t total, int per_cu, int64_t most) {
    static int n_cu = 0;
    if (n_cu == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
            n_cu = v;
        else
            n_cu = 256;
    }
    int64_t w = int64_t(n_cu) * per_cu;
    w = std::min<int64_t>(w, (total + 3) / 4);
    w = std::min<int64_t>(w, most);
    return int(std::max<int64_t>(w, 1));
}

// partial: [row sets][V_PART_STRIDE] floats for the split sums; max_split_rows: how many rows
// (one per query head and split or row set) it can take.
static int launch_v_matvec_into(const kv_cache *c, const float *p, int64_t ld_p, float *out, float *partial,
                                int64_t max_split_rows, hipStream_t s) {
    // Hs: kv-heads as the stream kernels count them (each dup times, see head_split); the combine
    // kernel works per query head and sees the real kv-head count and the whole group
    const int B = c->cfg.batch, H = c->cfg.n_kv_heads, G = c->group, Hs = H * c->head_split, Gq = G * c->head_split;
    const int n_blocks = int(c->packed_tokens / N);
    const int64_t rows = int64_t(B) * H * Gq;
    if (rows > max_split_rows) return KV_ERR_CAPACITY;
    const bool planes = !c->wide_v && c->cfg.pack_size == PACK;
    int n_splits = 0;
    FlatPlan plan = {n_blocks, 0, int64_t(B) * Hs * n_blocks};
    VArgs a;
    a.arena = static_cast<const uint8_t *>(c->buf.v_arena);
    a.index = static_cast<const uint32_t *>(c->buf.v_index);
    a.meta = static_cast<const uint32_t *>(c->buf.v_token_meta);
    a.p = p;
    a.partial = partial;
    a.ld = ld_p;
    a.meta_stride = c->max_tokens;
    a.B = B;
    a.index_words = c->index_words;
    a.H = Hs;
    a.dup = c->head_split;
    a.n_blocks = n_blocks;
    a.blocks_per_split = 0;
    if (n_blocks > 0 && planes) {
        // row sets: one per (workgroup, stream it touches), G rows each
        if (max_split_rows / G <= int64_t(B) * Hs) return KV_ERR_CAPACITY;
        // one round of resident workgroups: how many fit a compute unit depends on the instance; at
        // most 62 per stream (the combine kernel takes up to 64 row sets per stream)
        const int64_t most_groups = std::min<int64_t>(int64_t(62) * B * Hs, max_split_rows / G - int64_t(B) * Hs);
#define PACKKV_LAUNCH_VX(g, high)                                                                          \
    {                                                                                                      \
        static const int per_cu = resident_workgroups(reinterpret_cast<const void *>(v_matvec_kernel<g, high>)); \
        plan.n_groups = flat_groups_for(plan.total, per_cu, most_groups);                                 \
        hipLaunchKernelGGL((v_matvec_kernel<g, high>), dim3(plan.n_groups), dim3(256), 0, s, a, plan);      \
    }
#define PACKKV_LAUNCH_V(g) PACKKV_LAUNCH_VX(g, false)
#define PACKKV_LAUNCH_VH(g) PACKKV_LAUNCH_VX(g, true)
        if (c->qmax_v > 7) {
            PACKKV_DISPATCH_GROUP4(G, PACKKV_LAUNCH_VH)
        } else {
            PACKKV_DISPATCH_GROUP4(G, PACKKV_LAUNCH_V)
        }
#undef PACKKV_LAUNCH_VH
#undef PACKKV_LAUNCH_V
#undef PACKKV_LAUNCH_VX
    } else if (n_blocks > 0) {
        n_splits = int(std::min<int64_t>(v_splits_for(n_blocks, B * Hs), max_split_rows / rows));
        a.blocks_per_split = (n_blocks + n_splits - 1) / n_splits;
        n_splits = (n_blocks + a.blocks_per_split - 1) / a.blocks_per_split;
        dim3 grid(n_splits, B * Hs);
#define PACKKV_LAUNCH_VW(g) hipLaunchKernelGGL(vw_matvec_kernel<g>, grid, dim3(256), 0, s, a)
#define PACKKV_LAUNCH_V8(g) hipLaunchKernelGGL(v8_matvec_kernel<g>, grid, dim3(256), 0, s, a)
        if (c->wide_v) {
            PACKKV_DISPATCH_GROUP(G, PACKKV_LAUNCH_VW)
        } else {
            PACKKV_DISPATCH_GROUP(G, PACKKV_LAUNCH_V8)
        }
#undef PACKKV_LAUNCH_VW
#undef PACKKV_LAUNCH_V8
    }
    hipLaunchKernelGGL(v_reduce_kernel, dim3(B * H * Gq), dim3(256), 0, s, partial, n_splits,
                       B * H * Gq, plan, G, p, ld_p, c->packed_tokens,
                       static_cast<const __half *>(c->buf.v_tail), c->tail_tokens,
                       c->cfg.tail_capacity, H, Gq, out);
    KV_HIP_CHECK(hipGetLastError());
    return KV_OK;
}

int launch_v_matvec(const kv_cache *c, const float *p, int64_t ld_p, float *out, hipStream_t s) {
    uint8_t *ws = static_cast<uint8_t *>(c->buf.workspace);
    return launch_v_matvec_into(c, p, ld_p, out, reinterpret_cast<float *>(ws + WS_VPART),
                                int64_t(V_SPLITS_MAX) * c->cfg.batch * c->cfg.n_q_heads, s);
}

// ---- the V product for callers that cannot allocate ------------------------------------------
// The split sums go to a file-scope device array instead of the caller's workspace.  Every GPU
// the library runs on holds its own copy of the array (at its own address) until the process
// ends; the address is looked up once per device, with that device current, and kept.
static __device__ __align__(256) float scratch[size_t(KV_NOALLOC_MAX_SPLIT_ROWS) * V_PART_STRIDE];

static int scratch_of_current_device(float **out) {
    constexpr int MAX_DEVICES = 64;
    static float *ptr_of_device[MAX_DEVICES];
    static std::mutex lock;
    int dev = -1;
    KV_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return KV_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> guard(lock);
    if (!ptr_of_device[dev]) {
        float *p = nullptr;
        KV_HIP_CHECK(hipGetSymbolAddress(reinterpret_cast<void **>(&p), HIP_SYMBOL(scratch)));
        if (!p) return KV_ERR_HIP;
        ptr_of_device[dev] = p;
    }
    *out = ptr_of_device[dev];
    return KV_OK;
}

int launch_v_matvec_noalloc(const kv_cache *c, const float *p, int64_t ld_p, float *out, hipStream_t s) {
    float *partial = nullptr;
    const int rc = scratch_of_current_device(&partial);
    if (rc != KV_OK) return rc;
    // every split row that the combine kernel reads is written in full by the stream kernel of
    // the same call: nothing in the array has to start at zero
    return launch_v_matvec_into(c, p, ld_p, out, partial, KV_NOALLOC_MAX_SPLIT_ROWS, s);
}

}  // namespace packkv
