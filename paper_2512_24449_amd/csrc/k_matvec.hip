// Fused K path (PackKV Sec. III-C.1): scores = sm_scale * Khat q, streaming the
// packed K cache once and unpacking in registers.
//
// The paper walks a 32-lane warp over K rows and reduces with a warp sum.
// Here one 64-lane wave owns one chunk (64 tokens x 128 channels): lane l
// reads header bytes 8l..8l+7, so it owns token group g = l/16 and channels
// 8*(l%16)..+7, whose payload bytes are contiguous.  It keeps 16 per-token
// partial sums over its 8 channels; a reduce-scatter inside the 16-lane row
// then leaves token 16g+i's dot product in lane 16g+i, and the 64 scores are
// stored with one coalesced 256-byte write.  De-quantization is folded in:
//   score_t = sm_scale * (scale_t * (sum_d q_d code[t,d] + sum_d q_d m[g,d])
//                         + min_t * sum_d q_d)
// so the pack minimum costs one FMA per pack and (scale_t, min_t) one per token.
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
    int n_chunks;
    int n_chunk_groups;     // workgroups that process chunks
    int n_tail, tail_cap;
    float sm_scale;
};

template <int G>
__device__ inline void k_chunk(const KArgs &a, int c, int lane, uint8_t *lds) {
    const int h = c % a.H;
    const int b = (c / a.H) % a.B;
    const int blk = c / (a.H * a.B);
    const uint32_t o0 = a.index[c], o1 = a.index[c + 1];
    const int64_t tok = int64_t(blk) * N + lane;  // this lane's token after the reduction

    float result[G];
    if (o1 - o0 < uint32_t(HEADER / 16)) {  // dropped block: defined output
#pragma unroll
        for (int g = 0; g < G; ++g)
            a.scores[(int64_t(b) * a.H * G + h * G + g) * a.ld + tok] = 0.0f;
        return;
    }
    const uint8_t *chunk = a.arena + size_t(o0) * 16;
    const int payload_bytes = int(o1 - o0) * 16 - HEADER;

    // issue all global loads of the chunk before anything depends on them
    LaneHeader hd;
    {
        uint2 raw = *reinterpret_cast<const uint2 *>(chunk + lane * 8);
        hd.lo = raw.x;
        hd.hi = raw.y;
    }
    stage_payload(chunk + HEADER, payload_bytes, lds, lane);
    const uint32_t mt = a.meta[b * a.meta_stride + tok];

    // query slices of this lane's 8 channels, for the G query heads of kv-head h
    const int ch0 = 8 * (lane & 15);
    float qf[G][8], qsum[G], msum[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        uint4 raw = *reinterpret_cast<const uint4 *>(a.q + (int64_t(b) * a.H * G + h * G + g) * D + ch0);
        const __half *hq = reinterpret_cast<const __half *>(&raw);
        qsum[g] = 0.0f;
        msum[g] = 0.0f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            qf[g][j] = __half2float(hq[j]);
            qsum[g] += qf[g][j];
        }
    }

    const int my_bytes = hd.bytes();
    int pos = wave_inclusive_scan(my_bytes, lane) - my_bytes;

    float acc[G][16];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[g][i] = 0.0f;

    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int w = hd.width(j);
        const float m = float(hd.min(j));
        uint32_t lo, hi, L, Hh;
        read_pack(lds, pos, lo, hi);
        split_pack(lo, hi, w, L, Hh);
        pos += 2 * w;
#pragma unroll
        for (int g = 0; g < G; ++g) msum[g] = fmaf(qf[g][j], m, msum[g]);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float cl = float(__builtin_amdgcn_ubfe(L, i * w, w));
            const float chh = float(__builtin_amdgcn_ubfe(Hh, i * w, w));
#pragma unroll
            for (int g = 0; g < G; ++g) {
                acc[g][i] = fmaf(qf[g][j], cl, acc[g][i]);
                acc[g][i + 8] = fmaf(qf[g][j], chh, acc[g][i + 8]);
            }
        }
    }
    // the next chunk of this wave must not overwrite LDS before all lanes read it
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();

    const float scale = __half2float(__ushort_as_half(uint16_t(mt & 0xFFFFu)));
    const float mn = __half2float(__ushort_as_half(uint16_t(mt >> 16)));
#pragma unroll
    for (int g = 0; g < G; ++g) {
        float dot = row_reduce_scatter16(acc[g], lane);
        float ms = row_all_reduce16(msum[g]);
        float qs = row_all_reduce16(qsum[g]);
        result[g] = a.sm_scale * fmaf(scale, dot + ms, mn * qs);
        a.scores[(int64_t(b) * a.H * G + h * G + g) * a.ld + tok] = result[g];
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
    __shared__ __attribute__((aligned(16))) uint8_t lds_all[4 * PAYLOAD_LDS];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int unit = blockIdx.x * 4 + wave;
    if (blockIdx.x < a.n_chunk_groups) {
        if (unit < a.n_chunks) k_chunk<G>(a, unit, lane, lds_all + wave * PAYLOAD_LDS);
    } else {
        const int bh = (blockIdx.x - a.n_chunk_groups) * 4 + wave;
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
    a.n_chunks = int(c->packed_tokens / N) * a.B * a.H;
    a.n_chunk_groups = (a.n_chunks + 3) / 4;
    a.n_tail = c->tail_tokens;
    a.tail_cap = c->cfg.tail_capacity;
    a.sm_scale = sm_scale;
    const int tail_groups = a.n_tail > 0 ? (a.B * a.H + 3) / 4 : 0;
    const int grid = a.n_chunk_groups + tail_groups;
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
