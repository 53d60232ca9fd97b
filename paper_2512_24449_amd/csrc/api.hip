// Host side of the C ABI declared in packkv.h: argument checks, host
// bookkeeping and kernel launches.  Allocates no device memory.
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <initializer_list>
#include <new>

#include "common.h"

using namespace packkv;

namespace {

bool aligned256(const void *p) { return p && (reinterpret_cast<uintptr_t>(p) & 255u) == 0; }

// The kernels take up to 4 query heads per kv-head with packs of 16 tokens (the heads of a group
// times the pieces of their operands fill the 16 rows or columns of a matrix-core tile) and up to
// 8 with packs of 8.  Larger groups run as `split` groups of g / split heads over the same
// kv-head.  Returns the smallest such split, 0 if there is none up to 16.
int head_split_for(int g, int pack_size) {
    const int most = pack_size == PACK ? 4 : 8;
    for (int split = 1; split <= 16; ++split)
        if (g % split == 0 && g / split <= most) return split;
    return 0;
}

// Capacity of an arena in the 16-byte units of the 32-bit index words: what lies beyond the last
// addressable unit of a larger buffer stays unused.
uint32_t arena_units(size_t bytes) {
    return uint32_t(std::min<size_t>(bytes / 16, 0xFFFFFFFFu));
}

int check_config(const kv_config_t *c) {
    if (!c) return KV_ERR_ARG;
    if (c->batch < 1 || c->n_kv_heads < 1 || c->n_q_heads < 1 || c->max_tokens < 1) return KV_ERR_ARG;
    if (c->head_dim != D || c->block_tokens != N || (c->pack_size != PACK && c->pack_size != 8) ||
        (c->repack != KV_REPACK_NONE && c->repack != KV_REPACK_V_MEDIAN) ||
        c->tail_capacity != N)
        return KV_ERR_UNSUPPORTED;
    if (c->n_q_heads % c->n_kv_heads) return KV_ERR_ARG;
    const int g = c->n_q_heads / c->n_kv_heads;
    if (head_split_for(g, c->pack_size) == 0) return KV_ERR_UNSUPPORTED;
    // one pack byte holds a 4-bit minimum: codes above 15 need the wide layout, which exists
    // for packs of 8 tokens only; a code is one byte at most
    for (float rel : {c->k_rel_scale, c->v_rel_scale}) {
        if (!(rel > 0.0f) || rel > 1.0f) return KV_ERR_ARG;
        const long qmax = lround(1.0 / double(rel));
        if (qmax > 255) return KV_ERR_UNSUPPORTED;
        if (qmax > 15 && c->pack_size != 8) return KV_ERR_UNSUPPORTED;
    }
    if (int64_t(c->batch) * c->n_kv_heads * head_split_for(g, c->pack_size) > 65535) return KV_ERR_UNSUPPORTED;
    const int64_t max_tokens = (c->max_tokens + N - 1) / N * N;
    const int64_t max_chunks = max_tokens / N * c->batch * c->n_kv_heads;
    if (max_chunks > 0x7FFFFFF0) return KV_ERR_UNSUPPORTED;
    return KV_OK;
}

size_t round256(size_t n) { return (n + 255) & ~size_t(255); }

// Pages one tensor of a paged cache can come to hold: every chunk at its largest.
int64_t worst_case_pages(int64_t max_chunks, int pack_size, bool wide) {
    const int64_t per_page = KV_PAGE_BYTES / chunk_max_bytes(pack_size, wide);
    return (max_chunks + per_page - 1) / per_page + 1;
}

}  // namespace

extern "C" int kv_query_sizes(const kv_config_t *cfg, double bits_per_element_budget, kv_sizes_t *out) {
    int rc = check_config(cfg);
    if (rc) return rc;
    if (!out || bits_per_element_budget < 0.0) return KV_ERR_ARG;
    const int64_t max_tokens = (cfg->max_tokens + N - 1) / N * N;
    const int64_t max_chunks = max_tokens / N * cfg->batch * cfg->n_kv_heads;
    size_t arena[2];
    int t = 0;
    for (float rel : {cfg->k_rel_scale, cfg->v_rel_scale}) {
        const bool wide = wide_codes(rel);
        const int header = chunk_header_bytes(cfg->pack_size, wide);
        const double worst_bits = double(chunk_max_bytes(cfg->pack_size, wide)) * 8.0 / (N * D);
        double bits = bits_per_element_budget == 0.0 ? worst_bits : bits_per_element_budget;
        if (bits > worst_bits) bits = worst_bits;
        // never less than the headers, plus one worst-case chunk of slack per stream for padding
        double per_chunk = bits * (N * D) / 8.0;
        if (per_chunk < header + 16) per_chunk = header + 16;
        arena[t] = size_t(std::ceil(per_chunk * double(max_chunks))) + 16;
        if (arena[t] > size_t(0xFFFFFFFFull) * 16) return KV_ERR_UNSUPPORTED;  // index is in 16-byte units
        ++t;
    }
    out->k_arena = round256(arena[0]);
    out->v_arena = round256(arena[1]);
    out->k_index = out->v_index = round256(size_t(max_chunks + 1) * 4);
    out->k_token_meta = out->v_token_meta = round256(size_t(cfg->batch) * max_tokens * 4);
    out->k_tail = out->v_tail =
        round256(size_t(cfg->batch) * cfg->tail_capacity * cfg->n_kv_heads * D * 2);
    out->workspace = round256(WS_VPART + v_partial_bytes(cfg->batch, cfg->n_q_heads));
    if (cfg->pack_size == 16)  // staging area of the compressor behind the rest
        out->workspace += round256(size_t(stage_chunks_for(cfg->batch, cfg->n_kv_heads)) * chunk_max_bytes(16));
    out->token_order = cfg->repack ? round256(size_t(cfg->batch) * max_tokens) : 0;
    out->k_pages = out->v_pages = 0;
    return KV_OK;
}

extern "C" int kv_query_sizes_paged(const kv_config_t *cfg, kv_sizes_t *out) {
    int rc = kv_query_sizes(cfg, 0.0, out);
    if (rc) return rc;
    const int64_t max_tokens = (cfg->max_tokens + N - 1) / N * N;
    const int64_t max_chunks = max_tokens / N * cfg->batch * cfg->n_kv_heads;
    out->k_arena = out->v_arena = 0;
    out->k_index = out->v_index = round256(size_t(max_chunks) * 8);
    out->k_pages = round256(size_t(2 + worst_case_pages(max_chunks, cfg->pack_size, wide_codes(cfg->k_rel_scale))) * 4);
    out->v_pages = round256(size_t(2 + worst_case_pages(max_chunks, cfg->pack_size, wide_codes(cfg->v_rel_scale))) * 4);
    return KV_OK;
}

extern "C" size_t kv_page_pool_state_bytes(int64_t n_pages) {
    return n_pages < 1 ? 0 : round256(size_t(n_pages + 1) * 4);
}

extern "C" int kv_page_pool_create(void *pages, int64_t n_pages, void *state, void *hip_stream,
                                   kv_page_pool_t **out) {
    if (!out || !aligned256(pages) || !aligned256(state)) return KV_ERR_ARG;
    if (n_pages < 1 || n_pages >= (int64_t(1) << 20)) return KV_ERR_ARG;  // positions are uint32 16-byte units
    kv_page_pool *pool = new (std::nothrow) kv_page_pool;
    if (!pool) return KV_ERR_ARG;
    pool->pages = static_cast<uint8_t *>(pages);
    pool->state = static_cast<uint32_t *>(state);
    pool->n_pages = n_pages;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    int rc = launch_pool_init(pool, s);
    if (rc == KV_OK && hipStreamSynchronize(s) != hipSuccess) rc = KV_ERR_HIP;
    if (rc) {
        delete pool;
        return rc;
    }
    *out = pool;
    return KV_OK;
}

extern "C" int kv_page_pool_destroy(kv_page_pool_t *pool) {
    if (!pool) return KV_ERR_ARG;
    delete pool;
    return KV_OK;
}

extern "C" int kv_page_pool_free_pages(kv_page_pool_t *pool, int64_t *free_pages, void *hip_stream) {
    if (!pool || !free_pages) return KV_ERR_ARG;
    KV_HIP_CHECK(hipStreamSynchronize(static_cast<hipStream_t>(hip_stream)));
    uint32_t n = 0;
    KV_HIP_CHECK(hipMemcpy(&n, pool->state, 4, hipMemcpyDeviceToHost));
    *free_pages = n;
    return KV_OK;
}

namespace {

int create_cache(const kv_config_t *cfg, kv_page_pool *pool, const kv_buffers_t *buffers,
                 const kv_sizes_t *sizes, kv_cache_t **out) {
    int rc = check_config(cfg);
    if (rc) return rc;
    if (!buffers || !sizes || !out) return KV_ERR_ARG;
    kv_sizes_t need;
    rc = pool ? kv_query_sizes_paged(cfg, &need) : kv_query_sizes(cfg, 0.0, &need);
    if (rc) return rc;
    const void *ptrs[] = {buffers->k_index, buffers->v_index, buffers->k_token_meta,
                          buffers->v_token_meta, buffers->k_tail, buffers->v_tail, buffers->workspace,
                          pool ? buffers->k_pages : buffers->k_arena,
                          pool ? buffers->v_pages : buffers->v_arena};
    for (const void *p : ptrs)
        if (!aligned256(p)) return KV_ERR_ARG;
    // arenas may be any size >= one chunk; everything else must be complete
    if (pool) {
        if (sizes->k_pages < need.k_pages || sizes->v_pages < need.v_pages) return KV_ERR_ARG;
    } else if (sizes->k_arena < size_t(chunk_max_bytes(cfg->pack_size, wide_codes(cfg->k_rel_scale))) ||
               sizes->v_arena < size_t(chunk_max_bytes(cfg->pack_size, wide_codes(cfg->v_rel_scale)))) {
        return KV_ERR_ARG;
    }
    if (sizes->k_index < need.k_index ||
        sizes->v_index < need.v_index || sizes->k_token_meta < need.k_token_meta ||
        sizes->v_token_meta < need.v_token_meta || sizes->k_tail < need.k_tail ||
        sizes->v_tail < need.v_tail || sizes->workspace < need.workspace)
        return KV_ERR_ARG;
    if (cfg->repack && (!aligned256(buffers->token_order) || sizes->token_order < need.token_order))
        return KV_ERR_ARG;
    kv_cache *c = new (std::nothrow) kv_cache;
    if (!c) return KV_ERR_ARG;
    c->cfg = *cfg;
    c->buf = *buffers;
    c->sizes = *sizes;
    c->max_tokens = (cfg->max_tokens + N - 1) / N * N;
    c->max_chunks = c->max_tokens / N * cfg->batch * cfg->n_kv_heads;
    c->head_split = head_split_for(cfg->n_q_heads / cfg->n_kv_heads, cfg->pack_size);
    c->group = cfg->n_q_heads / cfg->n_kv_heads / c->head_split;
    c->qmax_k = int(lround(1.0 / double(cfg->k_rel_scale)));
    c->qmax_v = int(lround(1.0 / double(cfg->v_rel_scale)));
    c->wide_k = c->qmax_k > 15;
    c->wide_v = c->qmax_v > 15;
    c->packed_tokens = 0;
    c->tail_tokens = 0;
    c->fill_bound16[0] = c->fill_bound16[1] = 0;
    c->stage_offset = round256(WS_VPART + v_partial_bytes(cfg->batch, cfg->n_q_heads));
    c->stage_chunks = stage_chunks_for(cfg->batch, cfg->n_kv_heads);
    c->pool = pool;
    c->index_words = pool ? 2 : 1;
    c->max_pages_k = c->max_pages_v = 0;
    if (pool) {
        c->buf.k_arena = c->buf.v_arena = pool->pages;
        c->sizes.k_arena = c->sizes.v_arena = size_t(pool->n_pages) * KV_PAGE_BYTES;
        c->max_pages_k = int64_t(sizes->k_pages / 4) - 2;
        c->max_pages_v = int64_t(sizes->v_pages / 4) - 2;
    }
    rc = launch_init(c, nullptr);
    if (rc == KV_OK && hipStreamSynchronize(nullptr) != hipSuccess) rc = KV_ERR_HIP;
    if (rc) {
        delete c;
        return rc;
    }
    *out = c;
    return KV_OK;
}

}  // namespace

extern "C" int kv_cache_create(const kv_config_t *cfg, const kv_buffers_t *buffers,
                               const kv_sizes_t *sizes, kv_cache_t **out) {
    return create_cache(cfg, nullptr, buffers, sizes, out);
}

extern "C" int kv_cache_create_paged(const kv_config_t *cfg, kv_page_pool_t *pool,
                                     const kv_buffers_t *buffers, const kv_sizes_t *sizes,
                                     kv_cache_t **out) {
    if (!pool) return KV_ERR_ARG;
    return create_cache(cfg, pool, buffers, sizes, out);
}

extern "C" int kv_cache_release(kv_cache_t *c, void *hip_stream) {
    if (!c) return KV_ERR_ARG;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    int rc;
    if (c->pool && (rc = launch_release_pages(c, s))) return rc;
    if ((rc = launch_init(c, s))) return rc;  // status words, index[0]; the page lists are empty already
    c->packed_tokens = 0;
    c->tail_tokens = 0;
    c->fill_bound16[0] = c->fill_bound16[1] = 0;
    return KV_OK;
}

extern "C" int kv_cache_destroy(kv_cache_t *cache) {
    if (!cache) return KV_ERR_ARG;
    int rc = KV_OK;
    if (cache->pool && cache->packed_tokens > 0) {
        rc = kv_cache_release(cache, nullptr);
        if (rc == KV_OK && hipStreamSynchronize(nullptr) != hipSuccess) rc = KV_ERR_HIP;
    }
    delete cache;
    return rc;
}

namespace {

// Compress `n_blocks` full blocks whose tokens start at `src` (batch 0).
int compress_blocks(kv_cache *c, const __half *ksrc, const __half *vsrc, int64_t batch_stride,
                    int n_blocks, bool bf16, hipStream_t s) {
    const int B = c->cfg.batch, H = c->cfg.n_kv_heads;
    const int per_round = std::max(1, MAX_NEW_CHUNKS / (B * H));
    uint8_t *ws = static_cast<uint8_t *>(c->buf.workspace);
    uint32_t *status = reinterpret_cast<uint32_t *>(ws + WS_STATUS);
    int done = 0;
    while (done < n_blocks) {
        const int nb = std::min(per_round, n_blocks - done);
        CompressJob job;
        job.batch_stride = batch_stride;
        job.token_stride = int64_t(H) * D;
        job.n_blocks = nb;
        job.first_token = c->packed_tokens;
        job.first_chunk = c->packed_tokens / N * B * H;
        job.order = nullptr;
        job.pack_order = 0;
        job.bf16 = bf16;
        CompressJob kjob = job, vjob = job;
        kjob.src = ksrc + int64_t(done) * N * job.token_stride;
        kjob.rel = c->cfg.k_rel_scale;
        kjob.qmax = c->qmax_k;
        kjob.wide = c->wide_k;
        kjob.pack_order = 1;  // K chunks list their packs channel-major (what the K kernel's lanes own)
        kjob.arena = static_cast<uint8_t *>(c->buf.k_arena);
        kjob.arena_cap16 = arena_units(c->sizes.k_arena);
        kjob.index = static_cast<uint32_t *>(c->buf.k_index);
        kjob.meta = static_cast<uint32_t *>(c->buf.k_token_meta);
        kjob.status = status + ST_OVERFLOW_K;
        kjob.page_list = static_cast<uint32_t *>(c->buf.k_pages);
        kjob.max_pages = c->max_pages_k;
        vjob.src = vsrc + int64_t(done) * N * job.token_stride;
        vjob.rel = c->cfg.v_rel_scale;
        vjob.qmax = c->qmax_v;
        vjob.wide = c->wide_v;
        vjob.arena = static_cast<uint8_t *>(c->buf.v_arena);
        vjob.arena_cap16 = arena_units(c->sizes.v_arena);
        vjob.index = static_cast<uint32_t *>(c->buf.v_index);
        vjob.meta = static_cast<uint32_t *>(c->buf.v_token_meta);
        vjob.status = status + ST_OVERFLOW_V;
        vjob.page_list = static_cast<uint32_t *>(c->buf.v_pages);
        vjob.max_pages = c->max_pages_v;
        int rc;
        if ((rc = launch_token_params(c, kjob, s))) return rc;
        if ((rc = launch_token_params(c, vjob, s))) return rc;
        if (c->cfg.repack == KV_REPACK_V_MEDIAN) {
            uint8_t *order = static_cast<uint8_t *>(c->buf.token_order);
            if ((rc = launch_v_median_order(c, vjob, kjob.meta, order, s))) return rc;
            kjob.order = vjob.order = order;
        }
        kjob.fill_bound16 = c->fill_bound16[0];
        vjob.fill_bound16 = c->fill_bound16[1];
        if ((rc = launch_pack(c, kjob, s))) return rc;
        if ((rc = launch_pack(c, vjob, s))) return rc;
        c->fill_bound16[0] += uint64_t(nb) * B * H * (chunk_max_bytes(c->cfg.pack_size, c->wide_k) / 16);
        c->fill_bound16[1] += uint64_t(nb) * B * H * (chunk_max_bytes(c->cfg.pack_size, c->wide_v) / 16);
        c->packed_tokens += int64_t(nb) * N;
        done += nb;
    }
    return KV_OK;
}

}  // namespace

namespace {

// bf16: the new tokens are bf16 values; they enter as their fp16 roundings (the tail stores fp16).
int append_tokens(kv_cache_t *c, const void *k_new, const void *v_new, int32_t n_new, bool bf16,
                  void *hip_stream) {
    if (!c || n_new < 0) return KV_ERR_ARG;
    if (n_new == 0) return KV_OK;
    if (!k_new || !v_new) return KV_ERR_ARG;
    if ((reinterpret_cast<uintptr_t>(k_new) | reinterpret_cast<uintptr_t>(v_new)) & 15u) return KV_ERR_ARG;
    if (c->packed_tokens + c->tail_tokens + n_new > c->max_tokens) return KV_ERR_CAPACITY;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const int B = c->cfg.batch, H = c->cfg.n_kv_heads;
    (void)B;
    const int64_t row = int64_t(H) * D;
    const int64_t src_batch_stride = int64_t(n_new) * row;
    const __half *ksrc = static_cast<const __half *>(k_new);
    const __half *vsrc = static_cast<const __half *>(v_new);
    __half *ktail = static_cast<__half *>(c->buf.k_tail);
    __half *vtail = static_cast<__half *>(c->buf.v_tail);
    int64_t pos = 0, remaining = n_new;
    int rc;

    if (c->tail_tokens > 0 || remaining < N) {
        const int take = int(std::min<int64_t>(remaining, N - c->tail_tokens));
        if ((rc = launch_tail_copy(c, ksrc, vsrc, src_batch_stride, take, c->tail_tokens, bf16, s))) return rc;
        c->tail_tokens += take;
        pos += take;
        remaining -= take;
        if (c->tail_tokens == N) {
            if ((rc = compress_blocks(c, ktail, vtail, int64_t(c->cfg.tail_capacity) * row, 1, false, s))) return rc;
            c->tail_tokens = 0;
        }
    }
    const int full = int(remaining / N);
    if (full > 0) {
        if ((rc = compress_blocks(c, ksrc + pos * row, vsrc + pos * row, src_batch_stride, full, bf16, s))) return rc;
        pos += int64_t(full) * N;
        remaining -= int64_t(full) * N;
    }
    if (remaining > 0) {
        if ((rc = launch_tail_copy(c, ksrc + pos * row, vsrc + pos * row, src_batch_stride, int(remaining), 0, bf16, s)))
            return rc;
        c->tail_tokens = int(remaining);
    }
    return KV_OK;
}

}  // namespace

extern "C" int kv_compress_append(kv_cache_t *c, const void *k_new, const void *v_new, int32_t n_new,
                                  void *hip_stream) {
    return append_tokens(c, k_new, v_new, n_new, false, hip_stream);
}

extern "C" int kv_compress_append_bf16(kv_cache_t *c, const void *k_new, const void *v_new, int32_t n_new,
                                       void *hip_stream) {
    return append_tokens(c, k_new, v_new, n_new, true, hip_stream);
}

extern "C" int kv_k_matvec(kv_cache_t *c, const void *q, float sm_scale, float *scores,
                           int64_t ld_scores, void *hip_stream) {
    if (!c || !q || !scores) return KV_ERR_ARG;
    if (reinterpret_cast<uintptr_t>(q) & 15u) return KV_ERR_ARG;
    if (ld_scores < c->packed_tokens + c->tail_tokens) return KV_ERR_ARG;
    return launch_k_matvec(c, static_cast<const __half *>(q), sm_scale, scores, ld_scores,
                           static_cast<hipStream_t>(hip_stream));
}

extern "C" int kv_v_matvec(kv_cache_t *c, const float *p, int64_t ld_p, float *out, void *hip_stream) {
    if (!c || !p || !out) return KV_ERR_ARG;
    if (ld_p < c->packed_tokens + c->tail_tokens) return KV_ERR_ARG;
    return launch_v_matvec(c, p, ld_p, out, static_cast<hipStream_t>(hip_stream));
}

extern "C" int kv_v_matvec_noalloc(kv_cache_t *c, const float *p, int64_t ld_p, float *out, void *hip_stream) {
    if (!c || !p || !out) return KV_ERR_ARG;
    if (ld_p < c->packed_tokens + c->tail_tokens) return KV_ERR_ARG;
    return launch_v_matvec_noalloc(c, p, ld_p, out, static_cast<hipStream_t>(hip_stream));
}

extern "C" int kv_decode_attention(kv_cache_t *c, const void *q, float sm_scale, float *out,
                                   void *hip_stream) {
    if (!c || !q || !out || !(sm_scale == sm_scale)) return KV_ERR_ARG;
    if (reinterpret_cast<uintptr_t>(q) & 15u) return KV_ERR_ARG;
    if (c->packed_tokens + c->tail_tokens < 1) return KV_ERR_ARG;  // softmax over nothing
    return launch_decode_attention(c, static_cast<const __half *>(q), sm_scale, out,
                                   static_cast<hipStream_t>(hip_stream));
}

namespace packkv {
// Sums, over the chunks of one tensor, the chunk bytes and the payload bytes their headers
// announce: one wave per chunk, widths read from the header (high nibble of a pack byte, or a
// width byte per pack in wide chunks).  sums[0] += chunks present, [1] += chunk bytes,
// [2] += payload bytes.
__global__ __launch_bounds__(256) void chunk_bytes_kernel(const uint8_t *__restrict__ arena,
                                                          const uint32_t *__restrict__ index, int index_words,
                                                          int64_t n_chunks, int width_bytes, bool nibble,
                                                          int bytes_per_width, unsigned long long *sums) {
    const int lane = threadIdx.x & 63;
    const int64_t wave0 = (int64_t(blockIdx.x) * blockDim.x + threadIdx.x) >> 6;
    const int64_t n_waves = (int64_t(gridDim.x) * blockDim.x) >> 6;
    unsigned long long present = 0, bytes = 0, payload = 0;
    for (int64_t c = wave0; c < n_chunks; c += n_waves) {
        const uint32_t o0 = index[c * index_words], o1 = index[c * index_words + 1];
        if (o1 == o0) continue;  // dropped
        const uint8_t *hdr = arena + size_t(o0) * 16;
        int wsum = 0;
        for (int i = lane * 4; i < width_bytes; i += 256) {
            const uint32_t w4 = *reinterpret_cast<const uint32_t *>(hdr + i);
            const uint32_t w = nibble ? (w4 >> 4) & 0x0F0F0F0Fu : w4;
            wsum += int((w & 0xFF) + ((w >> 8) & 0xFF) + ((w >> 16) & 0xFF) + (w >> 24));
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) wsum += __shfl_xor(wsum, o);
        present += 1;
        bytes += (unsigned long long)(o1 - o0) * 16;
        payload += (unsigned long long)wsum * bytes_per_width;
    }
    if (lane == 0 && present) {
        atomicAdd(&sums[0], present);
        atomicAdd(&sums[1], bytes);
        atomicAdd(&sums[2], payload);
    }
}
}  // namespace packkv

extern "C" int kv_cache_stats(kv_cache_t *c, kv_stats_t *out, void *hip_stream) {
    if (!c || !out) return KV_ERR_ARG;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    KV_HIP_CHECK(hipStreamSynchronize(s));
    const int64_t n_chunks = c->packed_tokens / N * c->cfg.batch * c->cfg.n_kv_heads;
    uint32_t kend = 0, vend = 0, status[2] = {0, 0};
    // contiguous: the arena end in 16-byte units; paged: the number of pages held
    const void *kword = c->pool ? c->buf.k_pages : static_cast<uint32_t *>(c->buf.k_index) + n_chunks;
    const void *vword = c->pool ? c->buf.v_pages : static_cast<uint32_t *>(c->buf.v_index) + n_chunks;
    KV_HIP_CHECK(hipMemcpy(&kend, kword, 4, hipMemcpyDeviceToHost));
    KV_HIP_CHECK(hipMemcpy(&vend, vword, 4, hipMemcpyDeviceToHost));
    KV_HIP_CHECK(hipMemcpy(status, static_cast<uint8_t *>(c->buf.workspace) + WS_STATUS, 8, hipMemcpyDeviceToHost));
    std::memset(out, 0, sizeof(*out));
    out->tokens = c->packed_tokens + c->tail_tokens;
    out->packed_tokens = c->packed_tokens;
    out->tail_tokens = c->tail_tokens;
    out->n_chunks = n_chunks;
    const int64_t unit = c->pool ? KV_PAGE_BYTES : 16;
    out->k_bytes = int64_t(kend) * unit;
    out->v_bytes = int64_t(vend) * unit;
    out->index_bytes = c->pool ? n_chunks * 8 : (n_chunks + 1) * 4;
    out->token_meta_bytes = int64_t(c->cfg.batch) * c->packed_tokens * 4;
    out->overflow = (status[ST_OVERFLOW_K] || status[ST_OVERFLOW_V]) ? 1 : 0;
    if (n_chunks > 0) {
        // byte split of the chunks: six 64-bit sums in the status area (words 16..27)
        unsigned long long *sums = reinterpret_cast<unsigned long long *>(
            static_cast<uint8_t *>(c->buf.workspace) + WS_STATUS + 64);
        unsigned long long host[6];
        KV_HIP_CHECK(hipMemsetAsync(sums, 0, sizeof(host), s));
        const int grid = int(std::min<int64_t>((n_chunks + 3) / 4, 4096));
        for (int t = 0; t < 2; ++t) {
            const bool wide = t ? c->wide_v : c->wide_k;
            const int packs = N / c->cfg.pack_size * D;
            hipLaunchKernelGGL(chunk_bytes_kernel, dim3(grid), dim3(256), 0, s,
                               static_cast<const uint8_t *>(t ? c->buf.v_arena : c->buf.k_arena),
                               static_cast<const uint32_t *>(t ? c->buf.v_index : c->buf.k_index), c->index_words,
                               n_chunks, packs, !wide, c->cfg.pack_size / 8, sums + 3 * t);
        }
        KV_HIP_CHECK(hipGetLastError());
        KV_HIP_CHECK(hipMemcpyAsync(host, sums, sizeof(host), hipMemcpyDeviceToHost, s));
        KV_HIP_CHECK(hipStreamSynchronize(s));
        for (int t = 0; t < 2; ++t) {
            const bool wide = t ? c->wide_v : c->wide_k;
            const int64_t header = int64_t(host[3 * t]) * chunk_header_bytes(c->cfg.pack_size, wide);
            const int64_t payload = int64_t(host[3 * t + 2]);
            const int64_t padding = int64_t(host[3 * t + 1]) - header - payload;
            (t ? out->v_header_bytes : out->k_header_bytes) = header;
            (t ? out->v_payload_bytes : out->k_payload_bytes) = payload;
            (t ? out->v_padding_bytes : out->k_padding_bytes) = padding;
        }
    }
    return KV_OK;
}

extern "C" int kv_cache_restore(kv_cache_t *c, int64_t tokens) {
    if (!c || tokens < 0 || tokens > c->max_tokens) return KV_ERR_ARG;
    c->packed_tokens = tokens / N * N;
    c->tail_tokens = int(tokens - c->packed_tokens);
    return KV_OK;
}

extern "C" int64_t kv_cache_tokens(const kv_cache_t *c) {
    return c ? c->packed_tokens + c->tail_tokens : KV_ERR_ARG;
}

extern "C" const char *kv_strerror(int code) {
    switch (code) {
        case KV_OK: return "ok";
        case KV_ERR_ARG: return "invalid argument";
        case KV_ERR_UNSUPPORTED: return "unsupported configuration";
        case KV_ERR_CAPACITY: return "cache capacity exceeded";
        case KV_ERR_HIP: return "HIP runtime error";
        default: return "unknown error";
    }
}
