// Measurement companions: plain fp16 matrix-vector products over an
// UNCOMPRESSED cache (the comparison of PackKV Sec. IV-E, where the paper uses
// a vendor GEMV), hand-written for the same shapes, and a streaming-read kernel
// that measures the achievable HBM read rate.  Cache layout here is head-major
// fp16 [B][H_kv][L][128] so that every (b, h) matrix is one contiguous stream.
#include <algorithm>

#include "unpack.h"

namespace packkv {

// 16 bytes that are read once: with the non-temporal hint, as the packed kernels read their chunks.
__device__ inline uint4 load16_stream(const void *p) {
    typedef uint32_t u32x4n __attribute__((ext_vector_type(4)));
    const u32x4n v = __builtin_nontemporal_load(static_cast<const u32x4n *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}


typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

// K: one wave per 64 consecutive tokens of one (b, h).  Per step the wave reads
// four 256-byte rows (lane l: row l/16, channels 8*(l%16)..+7) with 16-byte
// loads; 16 steps leave 16 partial dot products per lane, reduce-scattered
// inside the 16-lane row so that every lane ends with one token's score.
template <int G>
__global__ __launch_bounds__(256) void fp16_k_kernel(const __half *__restrict__ kc,
                                                     const __half *__restrict__ q, float sm_scale,
                                                     float *__restrict__ scores, int64_t ld,
                                                     int H, int64_t L, int64_t tiles_per_stream,
                                                     int64_t n_units) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t unit = int64_t(blockIdx.x) * 4 + wave;
    if (unit >= n_units) return;
    const int64_t bh = unit / tiles_per_stream;
    const int64_t t0 = (unit % tiles_per_stream) * 64;
    const int h = int(bh % H);
    const int64_t b = bh / H;
    const int row = lane >> 4, ch0 = 8 * (lane & 15);

    half2_t qv[G][4];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        uint4 raw = *reinterpret_cast<const uint4 *>(q + ((b * H + h) * G + g) * D + ch0);
        const half2_t *hp = reinterpret_cast<const half2_t *>(&raw);
#pragma unroll
        for (int k = 0; k < 4; ++k) qv[g][k] = hp[k];
    }
    const __half *base = kc + (bh * L + t0) * D;
    uint4 raw[16];
#pragma unroll
    for (int it = 0; it < 16; ++it) {
        const int64_t t = t0 + 4 * it + row;
        raw[it] = t < L ? load16_stream(base + (4 * it + row) * D + ch0)
                        : make_uint4(0, 0, 0, 0);
    }
    float acc[G][16];
#pragma unroll
    for (int it = 0; it < 16; ++it) {
        const half2_t *kp = reinterpret_cast<const half2_t *>(&raw[it]);
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float s = 0.0f;
#pragma unroll
            for (int k = 0; k < 4; ++k) s = __builtin_amdgcn_fdot2(kp[k], qv[g][k], s, false);
            acc[g][it] = s;
        }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const float dot = row_reduce_scatter16(acc[g], lane);
        const int64_t t = t0 + 4 * (lane & 15) + row;  // lane i of row r holds step i, row r
        if (t < L) scores[((b * H + h) * G + g) * ld + t] = sm_scale * dot;
    }
}

// V: the context axis is split over workgroups; a wave walks its tokens four
// rows per step, each lane accumulating its 8 channels in fp32.
template <int G>
__global__ __launch_bounds__(256) void fp16_v_kernel(const __half *__restrict__ vc,
                                                     const float *__restrict__ p, int64_t ld,
                                                     float *__restrict__ partial, int H, int64_t L,
                                                     int64_t tokens_per_split) {
    __shared__ float red[4][G][D];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int split = blockIdx.x;
    const int64_t bh = blockIdx.y;
    const int h = int(bh % H);
    const int64_t b = bh / H;
    const int row = lane >> 4, ch0 = 8 * (lane & 15);
    const int64_t t_begin = split * tokens_per_split;
    const int64_t t_end = min(t_begin + tokens_per_split, L);

    float acc[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[g][j] = 0.0f;

    // each wave takes tiles of 64 tokens: tile k of the split goes to wave k % 4
    for (int64_t t0 = t_begin + 64 * wave; t0 < t_end; t0 += 256) {
        float pw[G];
#pragma unroll
        for (int g = 0; g < G; ++g)
            pw[g] = t0 + lane < t_end ? p[((b * H + h) * G + g) * ld + t0 + lane] : 0.0f;
        uint4 raw[16];
#pragma unroll
        for (int it = 0; it < 16; ++it) {
            const int64_t t = t0 + 4 * it + row;
            raw[it] = t < t_end ? load16_stream(vc + (bh * L + t) * D + ch0)
                                : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int it = 0; it < 16; ++it) {
            const __half *vp = reinterpret_cast<const __half *>(&raw[it]);
            float vf[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) vf[j] = __half2float(vp[j]);
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const float w = __shfl(pw[g], 4 * it + row);
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[g][j] = fmaf(w, vf[j], acc[g][j]);
            }
        }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            float v = acc[g][j];
            v += __shfl_xor(v, 16);
            v += __shfl_xor(v, 32);
            if (lane < 16) red[wave][g][8 * lane + j] = v;
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < G * D; i += 256) {
        const int g = i / D, d = i % D;
        const float v = (red[0][g][d] + red[1][g][d]) + (red[2][g][d] + red[3][g][d]);
        partial[(int64_t(split) * gridDim.y * G + (bh * G + g)) * V_PART_STRIDE + d] = v;
    }
}

__global__ __launch_bounds__(256) void fp16_v_reduce_kernel(const float *__restrict__ partial,
                                                            int n_splits, int n_rows,
                                                            float *__restrict__ out) {
    __shared__ float lds[8][V_PART_STRIDE];
    float unused;
    const float acc = reduce_split_partials(partial, n_splits, n_rows, blockIdx.x, lds, &unused);
    if (threadIdx.x < D) out[int64_t(blockIdx.x) * D + threadIdx.x] = acc;
}

// Streaming read: every thread keeps sixteen independent 16-byte loads in flight (a workgroup
// reads 64 KiB per round, 4 KiB per load instruction), xor-folded so the loads cannot be dropped.
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4 *__restrict__ src, size_t n16,
                                                          uint32_t *__restrict__ checksum) {
    constexpr int DEPTH = 16;
    uint32_t acc = 0;
    const size_t tile = size_t(DEPTH) * 256;
    const size_t n_tiles = n16 / tile;
    for (size_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
        const uint4 *p = src + t * tile + threadIdx.x;
        uint4 v[DEPTH];
#pragma unroll
        for (int k = 0; k < DEPTH; ++k) v[k] = load16_stream(p + k * 256);
#pragma unroll
        for (int k = 0; k < DEPTH; ++k) acc ^= v[k].x ^ v[k].y ^ v[k].z ^ v[k].w;
    }
    for (size_t i = n_tiles * tile + size_t(blockIdx.x) * 256 + threadIdx.x; i < n16; i += size_t(gridDim.x) * 256) {
        const uint4 a = src[i];
        acc ^= a.x ^ a.y ^ a.z ^ a.w;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc ^= __shfl_xor(acc, o);
    if ((threadIdx.x & 63) == 0 && acc != 0) atomicXor(checksum, acc);
}

}  // namespace packkv

using namespace packkv;

extern "C" int kv_fp16_k_matvec(const void *k_cache, const void *q, float sm_scale, float *scores,
                                int64_t ld_scores, int32_t batch, int32_t n_kv_heads,
                                int32_t n_q_heads, int64_t tokens, void *hip_stream) {
    if (!k_cache || !q || !scores || batch < 1 || n_kv_heads < 1 || tokens < 1 ||
        n_q_heads % n_kv_heads || ld_scores < tokens)
        return KV_ERR_ARG;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const int G = n_q_heads / n_kv_heads;
    const int64_t tiles = (tokens + 63) / 64;
    const int64_t units = tiles * batch * n_kv_heads;
    const int64_t grid = (units + 3) / 4;
    if (grid > 0x7FFFFFFF) return KV_ERR_ARG;
    const __half *kc = static_cast<const __half *>(k_cache);
    const __half *qq = static_cast<const __half *>(q);
#define LAUNCH(GG)                                                                               \
    hipLaunchKernelGGL(fp16_k_kernel<GG>, dim3((unsigned)grid), dim3(256), 0, s, kc, qq, sm_scale, \
                       scores, ld_scores, n_kv_heads, tokens, tiles, units)
    PACKKV_DISPATCH_GROUP(G, LAUNCH)
#undef LAUNCH
    KV_HIP_CHECK(hipGetLastError());
    return KV_OK;
}

extern "C" size_t kv_fp16_v_workspace_bytes(int32_t batch, int32_t n_q_heads) {
    return v_partial_bytes(batch, n_q_heads);
}

extern "C" int kv_fp16_v_matvec(const void *v_cache, const float *p, int64_t ld_p, float *out,
                                int32_t batch, int32_t n_kv_heads, int32_t n_q_heads,
                                int64_t tokens, void *workspace, void *hip_stream) {
    if (!v_cache || !p || !out || !workspace || batch < 1 || n_kv_heads < 1 || tokens < 1 ||
        n_q_heads % n_kv_heads || ld_p < tokens || batch * n_kv_heads > 65535)
        return KV_ERR_ARG;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const int G = n_q_heads / n_kv_heads;
    const int streams = batch * n_kv_heads;
    const int64_t tiles = (tokens + 63) / 64;
    // same split rule as the packed V path
    int n_splits = int(std::min<int64_t>(
        std::min<int64_t>((target_workgroups(tiles * streams) + streams - 1) / streams, (tiles + 3) / 4),
        V_SPLITS_MAX));
    if (n_splits < 1) n_splits = 1;
    int64_t tiles_per_split = (tiles + n_splits - 1) / n_splits;
    n_splits = int((tiles + tiles_per_split - 1) / tiles_per_split);
    float *partial = static_cast<float *>(workspace);
    const __half *vc = static_cast<const __half *>(v_cache);
    dim3 grid(n_splits, streams);
#define LAUNCH(GG)                                                                            \
    hipLaunchKernelGGL(fp16_v_kernel<GG>, grid, dim3(256), 0, s, vc, p, ld_p, partial, n_kv_heads, \
                       tokens, tiles_per_split * 64)
    PACKKV_DISPATCH_GROUP(G, LAUNCH)
#undef LAUNCH
    hipLaunchKernelGGL(fp16_v_reduce_kernel, dim3(batch * n_q_heads), dim3(256), 0, s, partial,
                       n_splits, batch * n_q_heads, out);
    KV_HIP_CHECK(hipGetLastError());
    return KV_OK;
}

extern "C" int kv_stream_read(const void *src, size_t bytes, uint32_t *checksum, void *hip_stream) {
    if (!src || !checksum || bytes % 16) return KV_ERR_ARG;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const size_t n16 = bytes / 16;
    // one launch, nothing else: persistent workgroups, eight per compute unit
    size_t blocks = (n16 + 256 * 16 - 1) / (256 * 16);
    if (blocks > 256 * 8) blocks = 256 * 8;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)blocks), dim3(256), 0, s,
                       static_cast<const uint4 *>(src), n16, checksum);
    KV_HIP_CHECK(hipGetLastError());
    return KV_OK;
}
