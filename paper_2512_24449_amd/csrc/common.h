// Internal definitions shared by the HIP translation units of libpackkv.
// gfx950 only: 64-wide wavefronts, LDS staging, DPP row operations.
#pragma once

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
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

// Workspace layout (bytes).
constexpr size_t WS_STATUS = 0;                 // uint32 status[64]
constexpr size_t WS_STATUS_BYTES = 256;
constexpr int MAX_NEW_CHUNKS = 65536;           // chunks compressed per round
constexpr size_t WS_SIZES = WS_STATUS_BYTES;    // uint32 sizes16[MAX_NEW_CHUNKS]
constexpr size_t WS_SIZES_BYTES = size_t(MAX_NEW_CHUNKS) * 4;
constexpr size_t WS_VPART = WS_SIZES + WS_SIZES_BYTES;
constexpr int V_SPLITS_MAX = 64;                // split-L partial sums of the V path
constexpr int V_PART_STRIDE = 132;              // floats: 128 outputs, [128] = sum p*min

enum { ST_OVERFLOW_K = 0, ST_OVERFLOW_V = 1 };

inline size_t v_partial_bytes(int batch, int n_q_heads) {
    return size_t(V_SPLITS_MAX) * batch * n_q_heads * V_PART_STRIDE * sizeof(float);
}

}  // namespace packkv

struct kv_cache {
    kv_config_t cfg;
    kv_buffers_t buf;
    kv_sizes_t sizes;
    int64_t max_tokens;     // rounded up to a block
    int64_t max_chunks;     // per tensor
    int group;              // query heads per kv head
    int qmax_k, qmax_v;
    int64_t packed_tokens;  // per batch element
    int32_t tail_tokens;
};

#define KV_HIP_CHECK(expr)                      \
    do {                                        \
        hipError_t e_ = (expr);                 \
        if (e_ != hipSuccess) return KV_ERR_HIP; \
    } while (0)

// ---- launchers implemented in the kernel translation units -----------------
namespace packkv {

struct CompressJob {
    const __half *src;        // first token of the first block, batch 0
    int64_t batch_stride;     // elements
    int64_t token_stride;     // elements (= H*128)
    int n_blocks;             // blocks of 64 tokens to compress
    int64_t first_token;      // destination token index of the first block
    int64_t first_chunk;      // destination chunk index
    float rel;
    int qmax;
    uint8_t *arena;
    uint64_t arena_cap16;     // capacity in 16-byte units
    uint32_t *index;
    uint32_t *meta;
    uint32_t *status;         // status word to set on overflow
};

int launch_compress(const kv_cache *c, const CompressJob &job, hipStream_t s);
int launch_tail_copy(const kv_cache *c, const __half *src, int64_t src_batch_stride, int n,
                     __half *tail, int tail_pos, hipStream_t s);
int launch_init(const kv_cache *c, hipStream_t s);
int launch_k_matvec(const kv_cache *c, const __half *q, float sm_scale, float *scores,
                    int64_t ld_scores, hipStream_t s);
int launch_v_matvec(const kv_cache *c, const float *p, int64_t ld_p, float *out, hipStream_t s);

}  // namespace packkv
