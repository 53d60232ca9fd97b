/*
 * packkv.h -- C ABI of the PackKV decode hot path for AMD MI355X (gfx950).
 *
 * A KV cache that is token-wise quantized and bit-packed in independent
 * 64-token blocks (PackKV, arXiv 2512.24449, Sec. III), an append-side
 * compressor, and fused kernels that stream the packed cache from HBM,
 * decode it on chip and compute q.K^T and p.V without ever writing
 * decompressed data back (Sec. III-C).
 *
 * Conventions for every entry point
 *   - "device" pointers are HIP device memory of the current device, owned by
 *     the caller; the library allocates no device memory and keeps only host
 *     bookkeeping inside kv_cache_t.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = default stream).
 *     Work is enqueued on it and the call returns without synchronizing
 *     unless stated otherwise.
 *   - Return value: KV_OK (0) or a negative KV_ERR_* code.  No exceptions, no
 *     aborts.  kv_strerror() gives a short text.
 *   - A kv_cache_t is not thread-safe; distinct handles are independent.
 *   - Inputs must be finite fp16 values; NaN/Inf never cause out-of-bounds
 *     accesses but produce unspecified codes.
 *
 * Cache layout (Sec. II-A): tokens arrive as fp16 [batch][n][n_kv_heads][128].
 * Packed format (Sec. III-B.3, III-B.4, III-C): one chunk per
 * (block of 64 tokens, batch, kv-head), chunk index c = (block*B + b)*H + h,
 * chunks stored back to back in c order in one arena per tensor.  A pack is the
 * 16 codes of one channel d in one token group g (tokens 16g..16g+15) with their
 * minimum subtracted: `width` = ceil(log2(range + 1)) bits per code, 0..4.  The
 * default layout (packs of 16 tokens) stores exactly 16*width bits per pack as
 * bit planes, which the decode kernels feed to the matrix cores as they are:
 *     pack list       V chunks: pack p = g*128 + d (group-major)
 *                     K chunks: pack p = d*4 + g   (channel-major)
 *     bytes [0,512)   header, byte p = (width << 4) | min of pack p
 *     region E        for p = 0..511 in turn: if width >= 2 a 32-bit word L with
 *                     the low two bits of the 16 codes, and if width == 4 a
 *                     second word H with their high two bits; in both, token i
 *                     of the group sits at bits [4i, 4i+2) for i < 8 and at
 *                     [4(i-8)+2, 4(i-8)+4) for i >= 8
 *     region O        for p = 0..511 in turn: if width is odd a 16-bit word T
 *                     with the top bit (bit width-1) of the 16 codes, token i
 *                     at bit 4*(i%4) + i/4
 *     then            zero padding to a multiple of 16 bytes
 * (all words little-endian; see kv_config_t for packs of 8 tokens and for the
 * wide layout that fine quantization scales use, which keep contiguous packs).
 * index[c] (uint32) is the chunk start in 16-byte units, index[n_chunks] the
 * arena end.  token_meta[b*max_tokens + t] (uint32) = scale_fp16 | min_fp16<<16
 * (Sec. III-B.2: one scale and minimum per token over all kv-heads).
 */
#ifndef PACKKV_H
#define PACKKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define KV_OK 0
#define KV_ERR_ARG (-1)          /* null pointer, bad size, misaligned buffer        */
#define KV_ERR_UNSUPPORTED (-2)  /* head_dim != 128, block != 64, pack size, rel...  */
#define KV_ERR_CAPACITY (-3)     /* append beyond max_tokens / arena too small       */
#define KV_ERR_HIP (-4)          /* a HIP runtime call failed                        */

#define KV_HEAD_DIM 128
#define KV_BLOCK_TOKENS 64
#define KV_PACK_SIZE 16                      /* default pack size                      */
#define KV_CHUNK_HEADER 512                  /* header bytes of a chunk, packs of 16   */
#define KV_CHUNK_MAX_BYTES (512 + 512 * 8)   /* largest chunk, packs of 16             */
#define KV_CHUNK_HEADER_PACK8 1024           /* the same with packs of 8 tokens        */
#define KV_CHUNK_MAX_BYTES_PACK8 (1024 + 1024 * 4)
#define KV_CHUNK_HEADER_WIDE 2048            /* wide chunks: codes above 15            */
#define KV_CHUNK_MAX_BYTES_WIDE (2048 + 1024 * 8)
#define KV_PAGE_BYTES 65536                  /* page of a paged arena (kv_page_pool_t) */

typedef struct kv_cache kv_cache_t; /* opaque, host memory owned by the library */
typedef struct kv_page_pool kv_page_pool_t; /* the same: pages shared by paged caches */

#define KV_REPACK_NONE 0
#define KV_REPACK_V_MEDIAN 1

/* Parameters of Sec. IV-A: relative quantization scales (K 0.1, V 0.2 are the
 * paper's defaults), pack size 16, repacking none, block 64.  Pack size 8 (the
 * other good point of the pack-size study, Sec. IV-B): a chunk then has 1024
 * header bytes, indexed [token_group * 128 + channel] with token groups of 8,
 * and packs of `width` bytes.  A relative scale below 1/15 gives codes above 15
 * ("wide" chunks for that tensor: packs of 8 tokens with widths up to 8 bits,
 * 1024 width bytes followed by 1024 minimum bytes, then the packs); it needs
 * pack_size 8, and its lower bound is 1/255.
 * KV_REPACK_V_MEDIAN
 * (Sec. III-B.3, "Faster Repacking with V Median"): inside every block of 64
 * tokens, K and V are packed with their tokens sorted by the lower median of the
 * token's quantized V vector over all kv-heads (ascending, ties in arrival
 * order); scores then come out in that storage order (see token_order). */
typedef struct {
    int32_t batch;         /* B >= 1                                              */
    int32_t n_kv_heads;    /* H_kv >= 1                                           */
    int32_t n_q_heads;     /* H_q, a multiple of H_kv; H_q / H_kv from 1 to 4 (packs of 16;
                              1 to 8 with packs of 8), or a product s * g with s <= 16 and g
                              in that range (8, 12, 16, 64 ...): such a group runs as s groups
                              of g heads over the same kv-head; B * H_kv * s at most 65535 */
    int32_t head_dim;      /* must be 128                                         */
    int32_t block_tokens;  /* must be 64                                          */
    int32_t pack_size;     /* 16 or 8                                             */
    int32_t repack;        /* KV_REPACK_NONE or KV_REPACK_V_MEDIAN                */
    int32_t tail_capacity; /* raw fp16 tail buffer in tokens, must be 64          */
    float k_rel_scale;     /* in [1/15, 1]; down to 1/255 with pack_size 8        */
    float v_rel_scale;     /* the same                                            */
    int64_t max_tokens;    /* per batch element, rounded up to a block internally */
} kv_config_t;

/* Bytes of each caller-provided device buffer. */
typedef struct {
    size_t k_arena, v_arena;           /* packed chunks                           */
    size_t k_index, v_index;           /* uint32 [max_chunks + 1]                 */
    size_t k_token_meta, v_token_meta; /* uint32 [B][max_tokens]                  */
    size_t k_tail, v_tail;             /* fp16 [B][tail_capacity][H_kv][128]      */
    size_t workspace;                  /* status words, chunk sizes, V partials, and (packs of
                                          16) the compressor's staging area: at most 75 MB */
    size_t token_order;                /* uint8 [B][max_tokens]; 0 without repacking */
    size_t k_pages, v_pages;           /* paged caches only: uint32 page lists; else 0 */
} kv_sizes_t;

/* Device buffers, each at least as large as kv_query_sizes said and 256-byte
 * aligned.  They must stay valid until kv_cache_destroy. */
typedef struct {
    void *k_arena, *v_arena;
    void *k_index, *v_index;
    void *k_token_meta, *v_token_meta;
    void *k_tail, *v_tail;
    void *workspace;
    /* With repacking: token_order[b][blk*64 + s] = position inside block blk (0..63,
     * arrival order) of the token stored at slot s; scores[b][hq][blk*64 + s] belongs
     * to token blk*64 + token_order[b][blk*64 + s].  Unused (may be null) without. */
    void *token_order;
    /* Paged caches only (kv_cache_create_paged; k_arena and v_arena are then unused and may be
     * null): [0] = pages held by the tensor, [1] = 16-byte units used in the newest of them,
     * [2 + i] = number of the i-th page taken.  Written by the library. */
    void *k_pages, *v_pages;
} kv_buffers_t;

/* Filled by kv_cache_stats. */
typedef struct {
    int64_t tokens;        /* cached tokens per batch element (packed + tail)     */
    int64_t packed_tokens; /* tokens living in chunks                             */
    int64_t tail_tokens;   /* tokens in the raw fp16 tail                         */
    int64_t n_chunks;      /* chunks per tensor                                   */
    int64_t k_bytes;       /* K arena bytes in use (header + payload + padding)   */
    int64_t v_bytes;
    int64_t index_bytes;   /* per tensor                                          */
    int64_t token_meta_bytes; /* per tensor                                       */
    int32_t overflow;      /* sticky: an append did not fit into an arena         */
    /* what the chunk bytes of each tensor consist of (chunks dropped by an overflow
     * count nothing): pack metadata (the header bytes), payload (exactly
     * pack_size * width bits per pack) and the zero padding up to 16 bytes       */
    int64_t k_header_bytes, k_payload_bytes, k_padding_bytes;
    int64_t v_header_bytes, v_payload_bytes, v_padding_bytes;
} kv_stats_t;

/*
 * Buffer sizes for a configuration.  `bits_per_element_budget` sizes the two
 * arenas: 0 means worst case (every pack at its largest width: 4.5 bits per
 * element with headers for packs of 16, 5 for packs of 8, 10 for wide chunks);
 * a positive value reserves that many bits per cached element
 * (it is clamped to the worst case).  Host only.
 */
int kv_query_sizes(const kv_config_t *cfg, double bits_per_element_budget, kv_sizes_t *out);

/*
 * Create an empty cache over caller-owned device buffers.  Enqueues a small
 * kernel on the default stream that clears the status words and index[0] and
 * synchronizes with it.  `sizes` are the real sizes of the buffers (arenas may
 * be larger or smaller than kv_query_sizes proposed; smaller arenas can
 * overflow, see kv_cache_stats).
 */
int kv_cache_create(const kv_config_t *cfg, const kv_buffers_t *buffers, const kv_sizes_t *sizes,
                    kv_cache_t **out);
int kv_cache_destroy(kv_cache_t *cache);

/*
 * Buffering, quantization, bit-packing and appending (Sec. III-B.1-4).
 * k_new, v_new: device fp16 [B][n_new][H_kv][128].  Tokens go to the raw
 * tail; whenever the tail holds 64 tokens they are quantized token-wise
 * (scale = rel*(max-min) over the token's H_kv*128 values, fp16 scale and
 * minimum), bit-packed in packs of 16 (or 8) tokens per channel, and appended to the
 * arenas as one chunk per (batch, kv-head); the tail then empties.  Several
 * full blocks in one call are compressed straight from k_new/v_new.
 * Errors: KV_ERR_CAPACITY if tokens + n_new > max_tokens (nothing is done).
 * An arena that is too small is detected on the device: the block is dropped
 * from that tensor and a sticky overflow flag is set.  Rule for dropped blocks:
 * kv_k_matvec scores the tokens of a block missing from K as -infinity, so
 * kv_softmax gives them weight 0 (a row of nothing else comes out as zeros);
 * kv_v_matvec adds nothing for a block missing from V; kv_decode_attention
 * leaves a block out when either tensor dropped it.  The three-step path and
 * the fused path therefore agree whenever no block is missing from V alone.
 * An arena larger than 2^32 * 16 bytes is used up to that size only.
 */
int kv_compress_append(kv_cache_t *cache, const void *k_new, const void *v_new, int32_t n_new,
                       void *hip_stream);
/*
 * The same for bf16 inputs (device bf16 [B][n_new][H_kv][128]): every value enters as
 * its fp16 rounding (to nearest even) -- exact for values in fp16's normal range,
 * since fp16 has the longer significand; smaller magnitudes round in fp16's
 * subnormal grid, magnitudes above 65504 become infinities (see "Inputs must be
 * finite").  From there on the path is the fp16 one: the tail stores fp16, and the
 * packed bytes are those kv_compress_append gives for the rounded values.
 */
int kv_compress_append_bf16(kv_cache_t *cache, const void *k_new, const void *v_new, int32_t n_new,
                            void *hip_stream);

/*
 * Fused K path (Sec. III-C.1): scores[b][hq][t] = sm_scale * sum_d
 * q[b][hq][d] * Khat[b][t][hq / G][d] for every cached token t, where Khat is
 * scale_t*code + min_t for packed tokens and the raw fp16 value for tail
 * tokens.  q: device fp16 [B][H_q][128]; scores: device fp32 [B][H_q][ld_scores],
 * ld_scores >= tokens (q 16-byte aligned).  fp32 accumulation.  One launch covers
 * all chunks.  With packs of 16 the products run on the matrix cores: the codes
 * enter exactly, q as three 4-bit pieces per value (a head's values below 2^-12
 * of its largest magnitude lose their low bits), sums in fp32.
 */
int kv_k_matvec(kv_cache_t *cache, const void *q, float sm_scale, float *scores, int64_t ld_scores,
                void *hip_stream);

/*
 * Fused V path (Sec. III-C.2): out[b][hq][d] = sum_t p[b][hq][t] *
 * Vhat[b][t][hq / G][d].  p: device fp32 [B][H_q][ld_p], ld_p >= tokens;
 * out: device fp32 [B][H_q][128].  fp32 accumulation in a fixed order (no
 * floating-point atomics): the result is bitwise reproducible.  Uses the
 * workspace for per-split partial sums; calls on one cache must not overlap.
 * With packs of 16 the products run on the matrix cores: the codes enter
 * exactly, the weights p_t * scale_t of a block rounded to 20 bits (16 with four
 * query heads per kv-head) below the block's largest weight of that head, and
 * the same rounded weights multiply the codes, the pack minimums and the token
 * minimums.  p must be non-negative.
 */
int kv_v_matvec(kv_cache_t *cache, const float *p, int64_t ld_p, float *out, void *hip_stream);

/*
 * kv_v_matvec for callers that cannot allocate device memory or hand over a
 * workspace for the call: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same kernels, same result
 * (bitwise, as long as the split count is not lowered, see below); the per-split
 * partial sums go to a fixed array inside the library (KV_NOALLOC_MAX_SPLIT_ROWS
 * rows of 132 floats, about 4.3 MB, held by every GPU the library runs on until
 * the process ends) instead of the cache's workspace.  The call allocates and
 * frees nothing.  The context axis is split over at most
 * KV_NOALLOC_MAX_SPLIT_ROWS / (batch * n_q_heads) workgroups per stream;
 * KV_ERR_CAPACITY if batch * n_q_heads exceeds KV_NOALLOC_MAX_SPLIT_ROWS.
 * All calls on one GPU share the array: calls that overlap on one GPU (other
 * streams, other caches, other threads) race and give wrong results; calls on
 * one stream are ordered and safe.
 */
#define KV_NOALLOC_MAX_SPLIT_ROWS 8192
int kv_v_matvec_noalloc(kv_cache_t *cache, const float *p, int64_t ld_p, float *out, void *hip_stream);

/*
 * Row softmax between the two matvecs (smx in the attention definition of
 * Sec. III-B.3), in place: scores[b][hq][0..tokens) <- softmax over the cached
 * tokens, for every (b, hq); entries [tokens, ld_scores) are left alone.
 * scores: device fp32 [B][H_q][ld_scores] as written by kv_k_matvec.  fp32,
 * reductions in a fixed order (bitwise reproducible).  Long rows are cut into
 * segments whose statistics pass through the workspace; calls on one cache
 * must not overlap.  KV_ERR_ARG on an empty cache or ld_scores < tokens.
 */
int kv_softmax(kv_cache_t *cache, float *scores, int64_t ld_scores, void *hip_stream);

/*
 * Fused decode attention (the attention of one new query as defined in
 * Sec. III-B.3, Att(q, K, V) = softmax(sm_scale * K q)^T V, computed with the
 * fused decompression of Sec. III-C):
 *   out[b][hq][:] = sum_t softmax_t(sm_scale * q[b][hq] . Khat[b][t][hq / G]) * Vhat[b][t][hq / G][:]
 * over all cached tokens (packed blocks and raw tail) in one pass: scores and
 * probabilities stay on chip.  q: device fp16 [B][H_q][128]; out: device fp32
 * [B][H_q][128].  Equivalent to kv_k_matvec -> softmax -> kv_v_matvec up to
 * fp32 rounding.  Fixed-order fp32 accumulation, bitwise reproducible.  Uses the
 * workspace for per-split partial results; calls on one cache must not overlap.
 * KV_ERR_ARG on an empty cache or if q is not 16-byte aligned.  Blocks dropped by
 * an arena overflow (in either tensor) are left out of the softmax.
 */
int kv_decode_attention(kv_cache_t *cache, const void *q, float sm_scale, float *out, void *hip_stream);

/*
 * ---- paged arena ------------------------------------------------------------
 * The packed format stores chunks wherever the index says (Sec. III-B.4 needs an
 * appendable layout, not a contiguous one).  A paged cache keeps no arena of its
 * own: its chunks live in fixed pages of KV_PAGE_BYTES that it takes, as it grows,
 * from a pool shared with other caches, and gives back with kv_cache_release -- so
 * the memory a cache holds follows its compressed size, not its worst case.
 *   - a chunk never crosses a page boundary: a chunk that does not fit behind the
 *     previous one of its tensor starts a fresh page (K and V fill their own pages);
 *   - the index of a paged cache has two words per chunk, index[2c] = start and
 *     index[2c + 1] = end, in 16-byte units from the start of the pool's pages
 *     (a pool is therefore limited to 64 GiB); a dropped chunk has start = end;
 *   - pages are taken and returned on the device, inside the stream of the call
 *     (no host synchronization).  If the pool cannot cover an append, all chunks of
 *     that tensor in that call are dropped and the sticky overflow flag is set,
 *     exactly as with a full contiguous arena.
 *   - calls that take or return pages of one pool (kv_compress_append,
 *     kv_cache_release, kv_cache_destroy of its caches) must be ordered by the
 *     caller: one stream, or events between streams.  Reads never touch the pool state.
 * Everything else (token metadata, tails, token order, every read entry point)
 * works as with a contiguous cache and gives bitwise the same results.
 */
/* Device bytes of the pool's bookkeeping (`state`) for n_pages pages. */
size_t kv_page_pool_state_bytes(int64_t n_pages);
/*
 * pages: device, n_pages * KV_PAGE_BYTES bytes, 256-byte aligned; state: device,
 * kv_page_pool_state_bytes(n_pages), 256-byte aligned; both caller-owned and valid
 * until kv_page_pool_destroy.  1 <= n_pages < 2^20.  Marks every page free (a
 * small kernel on `hip_stream`, synchronized before returning); page 0 is handed
 * out first.
 */
int kv_page_pool_create(void *pages, int64_t n_pages, void *state, void *hip_stream, kv_page_pool_t **out);
/* Host bookkeeping only; destroy the caches that use the pool first. */
int kv_page_pool_destroy(kv_page_pool_t *pool);
/* Number of free pages.  Reads device state: synchronizes `hip_stream`. */
int kv_page_pool_free_pages(kv_page_pool_t *pool, int64_t *free_pages, void *hip_stream);
/*
 * Buffer sizes of a paged cache: arenas 0, indices of 2 * max_chunks words, page
 * lists sized for the worst case, the rest as kv_query_sizes.  Host only.
 */
int kv_query_sizes_paged(const kv_config_t *cfg, kv_sizes_t *out);
/*
 * As kv_cache_create, over the pages of `pool` (buffers->k_arena / v_arena are ignored).
 */
int kv_cache_create_paged(const kv_config_t *cfg, kv_page_pool_t *pool, const kv_buffers_t *buffers,
                          const kv_sizes_t *sizes, kv_cache_t **out);
/*
 * Empties the cache: 0 tokens, overflow flag cleared; a paged cache gives all its
 * pages back to its pool (a kernel on `hip_stream`, no synchronization).  The
 * cache can be filled again.  kv_cache_destroy of a paged cache that still holds
 * tokens does the same on the default stream and synchronizes.
 */
int kv_cache_release(kv_cache_t *cache, void *hip_stream);

/* Counters and byte accounting.  Reads device state: synchronizes `hip_stream`.
 * For a paged cache k_bytes / v_bytes are the bytes of the pages held and
 * index_bytes counts two words per chunk. */
int kv_cache_stats(kv_cache_t *cache, kv_stats_t *out, void *hip_stream);

/*
 * Adopt externally written buffer contents (a cache restored from a copy of
 * its arenas, indices, token metadata, tails and, with repacking, token
 * order): afterwards the cache holds
 * `tokens` tokens per batch element, floor(tokens/64)*64 of them packed.
 * Host bookkeeping only; the caller is responsible for the buffer contents.
 */
int kv_cache_restore(kv_cache_t *cache, int64_t tokens);

/* Cached tokens per batch element (host bookkeeping, no synchronization). */
int64_t kv_cache_tokens(const kv_cache_t *cache);

const char *kv_strerror(int code);

/* ---- measurement companions (same shapes, uncompressed fp16 cache) ---------
 * The comparison kernels of Sec. IV-E, hand-written for the same shapes:
 * plain fp16 matrix-vector products over an uncompressed cache stored as
 * fp16 [B][H_kv][tokens][128] (head-major, each (b, h) matrix contiguous).
 * n_q_heads / n_kv_heads from 1 to 8 (KV_ERR_UNSUPPORTED otherwise).
 */
int kv_fp16_k_matvec(const void *k_cache, const void *q, float sm_scale, float *scores,
                     int64_t ld_scores, int32_t batch, int32_t n_kv_heads, int32_t n_q_heads,
                     int64_t tokens, void *hip_stream);
/* workspace: device, at least kv_fp16_v_workspace_bytes(...) bytes. */
int kv_fp16_v_matvec(const void *v_cache, const float *p, int64_t ld_p, float *out, int32_t batch,
                     int32_t n_kv_heads, int32_t n_q_heads, int64_t tokens, void *workspace,
                     void *hip_stream);
size_t kv_fp16_v_workspace_bytes(int32_t batch, int32_t n_q_heads);
/* Streaming-read ceiling: reads `bytes` (multiple of 16) of device memory with
 * sixteen independent 16-byte loads per thread and xors every word into
 * checksum[0] (device uint32; accumulated, the caller clears it): one kernel
 * launch and nothing else.  Used to measure achievable HBM read bandwidth next
 * to the 8 TB/s peak. */
int kv_stream_read(const void *src, size_t bytes, uint32_t *checksum, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* PACKKV_H */
