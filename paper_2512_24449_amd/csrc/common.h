// Internal definitions shared by the HIP translation units of libpackkv.
// gfx950 only: 64-wide wavefronts, LDS staging, DPP row operations.
#pragma once

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "packkv.h"

namespace packkv {

constexpr int D = KV_HEAD_DIM;         // 128 channels
constexpr int N = KV_BLOCK_TOKENS;     // 64 tokens per block
constexpr int PACK = KV_PACK_SIZE;     // 16 tokens per pack
constexpr int GROUPS = N / PACK;       // 4 token groups per block
constexpr int PACKS = GROUPS * D;      // 512 packs per chunk
constexpr int HEADER = KV_CHUNK_HEADER;
constexpr int CHUNK_MAX = KV_CHUNK_MAX_BYTES;
// packs of 8 tokens: 8 token groups, twice the header bytes
constexpr int HEADER8 = KV_CHUNK_HEADER_PACK8;
constexpr int CHUNK8_MAX = KV_CHUNK_MAX_BYTES_PACK8;
// wide chunks (codes above 15; packs of 8 tokens): a width byte and a minimum byte per pack
constexpr int HEADERW = KV_CHUNK_HEADER_WIDE;
constexpr int CHUNKW_MAX = KV_CHUNK_MAX_BYTES_WIDE;
inline bool wide_codes(float rel) { return lround(1.0 / double(rel)) > 15; }
inline int chunk_header_bytes(int pack_size, bool wide = false) {
    return wide ? HEADERW : (pack_size == 8 ? HEADER8 : HEADER);
}
inline int chunk_max_bytes(int pack_size, bool wide = false) {
    return wide ? CHUNKW_MAX : (pack_size == 8 ? CHUNK8_MAX : CHUNK_MAX);
}

// Workspace layout (bytes).
constexpr size_t WS_STATUS = 0;                 // uint32 status[64]
constexpr size_t WS_STATUS_BYTES = 256;
constexpr int MAX_NEW_CHUNKS = 65536;           // chunks compressed per round
constexpr size_t WS_SIZES = WS_STATUS_BYTES;    // uint32 sizes16[MAX_NEW_CHUNKS]
constexpr size_t WS_SIZES_BYTES = size_t(MAX_NEW_CHUNKS) * 4;
constexpr size_t WS_VPART = WS_SIZES + WS_SIZES_BYTES;
constexpr int V_SPLITS_MAX = 64;                // split-L partial sums of the V path
constexpr int V_PART_STRIDE = 132;              // floats: 128 outputs, [128] = sum p*min
constexpr int PAGE16 = KV_PAGE_BYTES / 16;      // 16-byte units per page of a paged arena

enum { ST_OVERFLOW_K = 0, ST_OVERFLOW_V = 1 };

// Workgroups (of four waves, one chunk per wave at a time) to spread `total_blocks` chunks
// over: a workgroup's start-up (constant table, query operands, first index and chunk
// loads) costs about as much as unpacking two chunks, so a wave should see about eight
// chunks; below that 512 workgroups -- two per compute unit -- measured fastest, and
// beyond a few thousand there is nothing left to gain.
inline int64_t target_workgroups(int64_t total_blocks) {
    const int64_t w = total_blocks / 32;
    return w < 512 ? 512 : (w > 4096 ? 4096 : w);
}

// Work list of the kernels that walk chunks in the plane layout: the chunks of all streams in one
// sequence (stream-major, n_blocks per stream), cut into n_groups equal ranges, one per workgroup.
// A workgroup that crosses a stream boundary writes one partial row set per stream it touches:
// the set of workgroup w for stream s has number w + s (unique, below n_groups + streams).
struct FlatPlan {
    int n_blocks;    // packed blocks per stream
    int n_groups;    // workgroups
    int64_t total;   // streams * n_blocks
    __host__ __device__ int64_t begin(int w) const { return w * total / n_groups; }
    // workgroup that holds flattened chunk f
    __host__ __device__ int group_of(int64_t f) const { return int(((f + 1) * n_groups - 1) / total); }
};

// Workgroups of 256 threads of `kernel` that fit one compute unit; workgroups for a flat work
// list of `total` chunks, at most `most` (v_matvec.hip).
int resident_workgroups(const void *kernel);
int flat_groups_for(int64_t total, int per_cu, int64_t most);

// Staging area of the compressor (packs of 16): chunks it holds, each in a slot of the largest
// chunk's size.  64 blocks of the cache at a time, within 256 .. 16384 chunks (1.2 .. 75 MB):
// large enough to fill the chip, small enough to stay in the last-level cache until it is read back.
inline int stage_chunks_for(int batch, int n_kv_heads) {
    const int64_t want = int64_t(batch) * n_kv_heads * 64;
    return int(want < 256 ? 256 : want > 16384 ? 16384 : want);
}

inline size_t v_partial_bytes(int batch, int n_q_heads) {
    return size_t(V_SPLITS_MAX) * batch * n_q_heads * V_PART_STRIDE * sizeof(float);
}

// The two small reductions that end a split-L pass, for a workgroup of 256 threads.  Each is cut
// into a load step and a sum step so that a kernel can issue ALL its global loads first and pay
// one memory latency instead of one per phase (these kernels run for a few microseconds).
//
// Split rows: partial[(s * n_rows + r) * V_PART_STRIDE + 0..128] for s < n_splits <= 64.  Eight
// thread groups take every eighth split with 16-byte loads; the sum step adds row s weight[s]
// times (weight null: once), the eight group sums pairwise, all in a fixed order.
struct SplitRows {
    float4 v[V_SPLITS_MAX / 8];
    float last[V_SPLITS_MAX / 8];  // column 128, thread group leaders only

    __device__ inline void load(const float *__restrict__ partial, int n_splits, int n_rows, int r) {
        load_strided(partial + int64_t(r) * V_PART_STRIDE, n_splits, n_rows);
    }
    // Rows first_row, first_row + row_stride * V_PART_STRIDE, ... (n_splits of them).
    __device__ inline void load_strided(const float *__restrict__ first_row, int n_splits, int64_t row_stride) {
        const int sg = threadIdx.x >> 5, q4 = threadIdx.x & 31;
#pragma unroll
        for (int i = 0; i < V_SPLITS_MAX / 8; ++i) {
            const int s = sg + 8 * i;
            v[i] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            last[i] = 0.0f;
            if (s < n_splits) {
                const float *src = first_row + int64_t(s) * row_stride * V_PART_STRIDE;
                v[i] = *reinterpret_cast<const float4 *>(src + 4 * q4);
                if (q4 == 0) last[i] = src[128];
            }
        }
    }
    // Returns column d = threadIdx.x (threads < 128; others 0) and the sum of column 128.  All
    // 256 threads must call; lds is free again when the call returns.
    __device__ inline float sum(int n_splits, float (*lds)[V_PART_STRIDE], float *col128,
                                const float *weight = nullptr) const {
        const int sg = threadIdx.x >> 5, q4 = threadIdx.x & 31;
        float4 acc = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        float l = 0.0f;
#pragma unroll
        for (int i = 0; i < V_SPLITS_MAX / 8; ++i) {
            const int s = sg + 8 * i;
            if (s < n_splits) {
                const float w = weight ? weight[s] : 1.0f;
                acc.x = fmaf(w, v[i].x, acc.x), acc.y = fmaf(w, v[i].y, acc.y);
                acc.z = fmaf(w, v[i].z, acc.z), acc.w = fmaf(w, v[i].w, acc.w);
                l = fmaf(w, last[i], l);
            }
        }
        *reinterpret_cast<float4 *>(&lds[sg][4 * q4]) = acc;
        if (q4 == 0) lds[sg][128] = l;
        __syncthreads();
        const int d = threadIdx.x < 128 ? threadIdx.x : 128;
        const float out = ((lds[0][d] + lds[1][d]) + (lds[2][d] + lds[3][d])) +
                          ((lds[4][d] + lds[5][d]) + (lds[6][d] + lds[7][d]));
        *col128 = ((lds[0][128] + lds[1][128]) + (lds[2][128] + lds[3][128])) +
                  ((lds[4][128] + lds[5][128]) + (lds[6][128] + lds[7][128]));
        __syncthreads();
        return threadIdx.x < 128 ? out : 0.0f;
    }
};

inline __device__ float reduce_split_partials(const float *__restrict__ partial, int n_splits, int n_rows,
                                              int r, float (*lds)[V_PART_STRIDE], float *col128) {
    SplitRows rows;
    rows.load(partial, n_splits, n_rows, r);
    return rows.sum(n_splits, lds, col128);
}

// Raw tail: sum_t weight[t] * V[t][d] over the n_tail <= 64 raw fp16 tail tokens of one (batch,
// kv-head).  Thread (token lane x / 16, channel group x % 16) takes tokens lane, lane + 16, ..
// with 16-byte loads; the sixteen token lanes are added in a fixed order.  vrow: the head's 128
// values of tail token 0; token_stride in elements.
struct TailRows {
    uint4 raw[4];

    __device__ inline void load(const __half *__restrict__ vrow, int64_t token_stride, int n_tail) {
        const int cg = threadIdx.x & 15, tl = threadIdx.x >> 4;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int t = tl + 16 * i;
            raw[i] = make_uint4(0, 0, 0, 0);
            if (t < n_tail) raw[i] = *reinterpret_cast<const uint4 *>(vrow + t * token_stride + 8 * cg);
        }
    }
    // weight: n_tail floats (LDS or global).  Returns column d = threadIdx.x (threads < 128;
    // others 0).  All 256 threads must call; lds is free again when the call returns.
    __device__ inline float sum(const float *weight, int n_tail, float (*lds)[V_PART_STRIDE]) const {
        const int cg = threadIdx.x & 15, tl = threadIdx.x >> 4;
        float acc[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) acc[k] = 0.0f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int t = tl + 16 * i;
            if (t < n_tail) {
                const __half *hv = reinterpret_cast<const __half *>(&raw[i]);
                const float w = weight[t];
#pragma unroll
                for (int k = 0; k < 8; ++k) acc[k] = fmaf(w, __half2float(hv[k]), acc[k]);
            }
        }
        *reinterpret_cast<float4 *>(&lds[tl][8 * cg]) = make_float4(acc[0], acc[1], acc[2], acc[3]);
        *reinterpret_cast<float4 *>(&lds[tl][8 * cg + 4]) = make_float4(acc[4], acc[5], acc[6], acc[7]);
        __syncthreads();
        float v = 0.0f;
        if (threadIdx.x < 128) {
            const int d = threadIdx.x;
            v = (((lds[0][d] + lds[1][d]) + (lds[2][d] + lds[3][d])) + ((lds[4][d] + lds[5][d]) + (lds[6][d] + lds[7][d]))) +
                (((lds[8][d] + lds[9][d]) + (lds[10][d] + lds[11][d])) + ((lds[12][d] + lds[13][d]) + (lds[14][d] + lds[15][d])));
        }
        __syncthreads();
        return v;
    }
};

}  // namespace packkv

// A pool of fixed-size pages shared by paged caches.  Device state: uint32 state[0] = number of
// free pages, state[1 + i] for i < state[0] = the free page numbers, the top of the stack last.
struct kv_page_pool {
    uint8_t *pages;
    uint32_t *state;
    int64_t n_pages;
};

// Staged compression of packs of 16 (compress.hip).  A round whose chunks fit the arena even at
// their largest takes the staged path; the test runs on the device, where the fill level is.
struct StagedRound {
    int64_t first_chunk;   // first chunk of the whole round
    uint32_t worst16;      // chunks of the round times the largest chunk, in 16-byte units; 0: two-pass only
    uint64_t arena_cap16;
};

// A staged part: chunks in their slots, to be copied to the arena once the part's scan has set
// their index words.
struct StagedPart {
    const uint8_t *staging;   // slot i holds chunk first_chunk + i
    const uint32_t *index;
    int64_t first_chunk;      // absolute chunk number
    int n;
    uint8_t *arena;
    StagedRound round;        // of the part's tensor
};


struct kv_cache {
    kv_config_t cfg;
    kv_buffers_t buf;
    kv_sizes_t sizes;
    int64_t max_tokens;     // rounded up to a block
    int64_t max_chunks;     // per tensor
    int group;              // query heads per kv head as the kernels see them (1..8)
    int head_split;         // groups above 8 are split: every kv-head counts head_split times, with `group` heads each
    int qmax_k, qmax_v;
    bool wide_k, wide_v;    // codes above 15: wide chunk layout for that tensor
    int64_t packed_tokens;  // per batch element
    int32_t tail_tokens;
    size_t stage_offset;    // staging area of the compressor inside the workspace (packs of 16; else unused)
    int stage_chunks;       // chunks it holds
    uint64_t fill_bound16[2];  // K, V: upper bound of the arena's fill level, every chunk so far at its largest
    // paged arena: both tensors live in the pool's pages (buf.k_arena = buf.v_arena = pool->pages),
    // the index has a (start, end) pair per chunk, buf.k_pages / buf.v_pages list the pages held
    kv_page_pool *pool;     // null: chunks back to back in the cache's own arenas
    int index_words;        // 1, or 2 when paged
    int64_t max_pages_k, max_pages_v;  // what the caller's page lists can take
};

// Runs LAUNCH(g) with the group size as a compile-time constant; group sizes 1..8.
#define PACKKV_DISPATCH_GROUP(group, LAUNCH)   \
    switch (group) {                           \
        case 1: LAUNCH(1); break;              \
        case 2: LAUNCH(2); break;              \
        case 3: LAUNCH(3); break;              \
        case 4: LAUNCH(4); break;              \
        case 5: LAUNCH(5); break;              \
        case 6: LAUNCH(6); break;              \
        case 7: LAUNCH(7); break;              \
        case 8: LAUNCH(8); break;              \
        default: return KV_ERR_UNSUPPORTED;    \
    }

// The same for the kernels of the plane layout (packs of 16 tokens): group sizes 1..4.
#define PACKKV_DISPATCH_GROUP4(group, LAUNCH)  \
    switch (group) {                           \
        case 1: LAUNCH(1); break;              \
        case 2: LAUNCH(2); break;              \
        case 3: LAUNCH(3); break;              \
        case 4: LAUNCH(4); break;              \
        default: return KV_ERR_UNSUPPORTED;    \
    }

#define KV_HIP_CHECK(expr)                      \
    do {                                        \
        hipError_t e_ = (expr);                 \
        if (e_ != hipSuccess) return KV_ERR_HIP; \
    } while (0)

// ---- launchers implemented in the kernel translation units -----------------
namespace packkv {

struct CompressJob {
    const __half *src;        // first token of the first block, batch 0
    bool bf16;                // src holds bf16 values (read as their fp16 roundings); else fp16
    int64_t batch_stride;     // elements
    int64_t token_stride;     // elements (= H*128)
    int n_blocks;             // blocks of 64 tokens to compress
    int64_t first_token;      // destination token index of the first block
    int64_t first_chunk;      // destination chunk index
    float rel;
    int qmax;
    bool wide;                // wide chunk layout
    uint8_t *arena;
    uint64_t arena_cap16;     // capacity in 16-byte units
    uint32_t *index;
    uint32_t *meta;
    uint32_t *status;         // status word to set on overflow
    uint32_t *page_list;      // paged arena: [0] pages held, [1] 16-byte units used in the newest, [2..] page numbers
    int64_t max_pages;        // page numbers the list has room for
    const uint8_t *order;     // [B][max_tokens] source position of each storage slot inside its block, or null
    int pack_order;           // packs of 16 (plane layout): 0 group-major pack list (V), 1 channel-major (K)
    uint64_t fill_bound16;    // the arena holds at most this much before the round (every chunk so far at its largest)
};

int launch_token_params(const kv_cache *c, const CompressJob &job, hipStream_t s);
int launch_pack(const kv_cache *c, const CompressJob &job, hipStream_t s);
// V-median order of the job's blocks (job describes V); permutes the token metadata of both
// tensors into storage order and fills `order`.
int launch_v_median_order(const kv_cache *c, const CompressJob &vjob, uint32_t *k_meta, uint8_t *order,
                          hipStream_t s);
int launch_tail_copy(const kv_cache *c, const __half *ksrc, const __half *vsrc, int64_t src_batch_stride,
                     int n, int tail_pos, bool bf16, hipStream_t s);
int launch_init(const kv_cache *c, hipStream_t s);
int launch_pool_init(const kv_page_pool *pool, hipStream_t s);
// Gives the pages of both tensors back to the pool and empties the page lists.
int launch_release_pages(const kv_cache *c, hipStream_t s);
int launch_k_matvec(const kv_cache *c, const __half *q, float sm_scale, float *scores,
                    int64_t ld_scores, hipStream_t s);
int launch_v_matvec(const kv_cache *c, const float *p, int64_t ld_p, float *out, hipStream_t s);
int launch_v_matvec_noalloc(const kv_cache *c, const float *p, int64_t ld_p, float *out, hipStream_t s);
int launch_decode_attention(const kv_cache *c, const __half *q, float sm_scale, float *out, hipStream_t s);

}  // namespace packkv
