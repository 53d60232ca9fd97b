// Fused V path (PackKV Sec. III-C.2): out = p^T Vhat, streaming the packed V
// cache once and unpacking in registers.
//
// The paper gives each thread one pack (a dot-product segment along ctx_len)
// and combines segments with fp32 atomic adds.  Here the contraction runs
// along the pack direction, so it maps onto the matrix cores without any
// transposition: for pack slot jj the wave issues
//     C_jj[channel row i][column] += A[i][k] * B[k][column]      (16x16x32 fp16 MFMA)
// where row i is lane%16 (channel 8i+jj), the 32 k-slots are 8 tokens of each
// of the 4 token groups (lane/16), A holds the unpacked codes exactly as
// unpack_pairs leaves them (fp16 code * 2^-24) and B holds the weights
// w_t = p_t * scale_t split into fp16 hi and lo*2^11 parts, one column pair per
// query head (so fp32-accurate weights cost no extra MFMA and G query heads of
// a GQA group share one unpack).  Accumulation is fp32 inside the MFMA, in a
// fixed order: the context axis is split over workgroups whose partial sums
// are combined by a second small kernel -- no atomics, bitwise reproducible.
// De-quantization is folded in:
//   out_d = sum_t w_t code[t,d] + sum_g m[g,d] sum_{t in g} w_t + sum_t p_t min_t
#include <algorithm>
#include <mutex>

#include "pack8.h"
#include "v_chunk.h"

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

template <int G>
__global__ __launch_bounds__(256) void v_matvec_kernel(VArgs a) {
    // two chunk buffers per wave; after the main loop the same memory holds the
    // cross-wave reduction array red[4][G][D + 4]
    __shared__ __attribute__((aligned(16))) uint8_t lds_all[4 * 2 * CHUNK_LDS + LDS_TAIL_PAD];
    __shared__ __attribute__((aligned(16))) uint8_t blds_all[4 * BLds<G>::BYTES];
    __shared__ uint4 table[PACK_TABLE_ENTRIES];
    static_assert(sizeof(float) * 4 * G * (D + 4) <= 4 * 2 * CHUNK_LDS, "reduction array must fit");
    float(*red)[G][D + 4] = reinterpret_cast<float(*)[G][D + 4]>(lds_all);
    build_pack_table(table, CODE_LIFT, fold_min<G>());

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int split = blockIdx.x;
    const int bh = blockIdx.y;
    const int h = bh % a.H, b = bh / a.H;
    const int buf_base = wave * 2 * CHUNK_LDS;
    VLane<G> vl;
    vl.init(blds_all + wave * BLds<G>::BYTES, lane);
    VState<G> st;
    st.clear();

    const int blk_begin = split * a.blocks_per_split;
    const int blk_end = min(blk_begin + a.blocks_per_split, a.n_blocks);
    for (int first = blk_begin + wave; first < blk_end; first += 4 * 64) {
        IndexBatch ib;
        ib.load(a.index, a.index_words, first, 4, blk_end, a.B, a.H / a.dup, b, h / a.dup, lane);
        const int n_it = min(64, (blk_end - first + 3) / 4);
        chunk_issue_lds(a.arena, ib.start16(0), ib.end16(0), lds_all + buf_base, lane);
        uint32_t mt_next = a.meta[b * a.meta_stride + int64_t(first) * N + lane];
        float p_next[G];
#pragma unroll
        for (int g = 0; g < G; ++g)
            p_next[g] = a.p[(int64_t(b) * a.H * G + h * G + g) * a.ld + int64_t(first) * N + lane];
        for (int it = 0; it < n_it; ++it) {
            const int cur = buf_base + (it & 1) * CHUNK_LDS;
            const bool valid = ib.end16(it) - ib.start16(it) >= uint32_t(HEADER / 16);
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
                chunk_issue_lds(a.arena, ib.start16(it + 1), ib.end16(it + 1),
                                lds_all + buf_base + ((it + 1) & 1) * CHUNK_LDS, lane);
                const int64_t tok = int64_t(first + 4 * (it + 1)) * N + lane;
                mt_next = a.meta[b * a.meta_stride + tok];
#pragma unroll
                for (int g = 0; g < G; ++g) p_next[g] = a.p[(int64_t(b) * a.H * G + h * G + g) * a.ld + tok];
            }
            if (!valid) continue;  // a block dropped by an arena overflow contributes nothing
            v_chunk<G>(lds_all, cur, table, vl, mt, pt, st);
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

// Fixed-order combination of the split partial sums, plus the raw fp16 tail.
__global__ __launch_bounds__(256) void v_reduce_kernel(const float *__restrict__ partial,
                                                       int n_splits, int n_rows,
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
    rows.load(partial, n_splits, n_rows, r);
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
static int launch_v_matvec_into(const kv_cache *c, const float *p, int64_t ld_p, float *out, float *partial,
                                int64_t max_split_rows, hipStream_t s) {
    // Hs: kv-heads as the stream kernels count them (each dup times, see head_split); the combine
    // kernel works per query head and sees the real kv-head count and the whole group
    const int B = c->cfg.batch, H = c->cfg.n_kv_heads, G = c->group, Hs = H * c->head_split, Gq = G * c->head_split;
    const int n_blocks = int(c->packed_tokens / N);
    const int64_t rows = int64_t(B) * H * Gq;
    if (rows > max_split_rows) return KV_ERR_CAPACITY;
    int n_splits = 0;
    if (n_blocks > 0) {
        n_splits = int(std::min<int64_t>(v_splits_for(n_blocks, B * Hs), max_split_rows / rows));
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
        a.blocks_per_split = (n_blocks + n_splits - 1) / n_splits;
        n_splits = (n_blocks + a.blocks_per_split - 1) / a.blocks_per_split;
        dim3 grid(n_splits, B * Hs);
#define PACKKV_LAUNCH_VW(g) hipLaunchKernelGGL(vw_matvec_kernel<g>, grid, dim3(256), 0, s, a)
#define PACKKV_LAUNCH_V8(g) hipLaunchKernelGGL(v8_matvec_kernel<g>, grid, dim3(256), 0, s, a)
#define PACKKV_LAUNCH_V(g) hipLaunchKernelGGL(v_matvec_kernel<g>, grid, dim3(256), 0, s, a)
        if (c->wide_v) {
            PACKKV_DISPATCH_GROUP(G, PACKKV_LAUNCH_VW)
        } else if (c->cfg.pack_size == 8) {
            PACKKV_DISPATCH_GROUP(G, PACKKV_LAUNCH_V8)
        } else {
            PACKKV_DISPATCH_GROUP(G, PACKKV_LAUNCH_V)
        }
#undef PACKKV_LAUNCH_VW
#undef PACKKV_LAUNCH_V8
#undef PACKKV_LAUNCH_V
    }
    hipLaunchKernelGGL(v_reduce_kernel, dim3(B * H * Gq), dim3(256), 0, s, partial, n_splits,
                       B * H * Gq, p, ld_p, c->packed_tokens,
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
