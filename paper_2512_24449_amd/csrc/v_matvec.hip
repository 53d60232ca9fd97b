// Fused V path (PackKV Sec. III-C.2): out = p^T Vhat, streaming the packed V
// cache once and unpacking in registers.
//
// The paper gives each thread one pack (a dot-product segment along ctx_len)
// and combines segments with fp32 atomic adds.  Here a wave owns whole chunks
// with the same lane-to-pack mapping as the K path (lane l: token group l/16,
// channels 8*(l%16)..+7), keeps its 8 channel sums in registers across all the
// chunks it visits, and the context axis is split over workgroups whose partial
// sums are combined in a fixed order by a second small kernel: no atomics, so
// the result is bitwise reproducible.  De-quantization is folded in:
//   out_d = sum_t (p_t scale_t) code[t,d] + sum_g m[g,d] sum_{t in g} p_t scale_t
//           + sum_t p_t min_t
// The weights p_t*scale_t of a chunk's 64 tokens are staged in LDS.
#include "unpack.h"

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
    int n_blocks;           // packed blocks per stream
    int blocks_per_split;
};

template <int G>
__global__ __launch_bounds__(256) void v_matvec_kernel(VArgs a) {
    __shared__ __attribute__((aligned(16))) uint8_t lds_all[4 * PAYLOAD_LDS];
    __shared__ __attribute__((aligned(16))) float wlds_all[4][G][N];
    __shared__ float red[4][G][D + 1];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int split = blockIdx.x;
    const int bh = blockIdx.y;
    const int h = bh % a.H, b = bh / a.H;
    uint8_t *lds = lds_all + wave * PAYLOAD_LDS;
    const int row = lane >> 4;

    float acc[G][8];
    float pm[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        pm[g] = 0.0f;
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[g][j] = 0.0f;
    }

    const int blk_begin = split * a.blocks_per_split;
    const int blk_end = min(blk_begin + a.blocks_per_split, a.n_blocks);
    for (int blk = blk_begin + wave; blk < blk_end; blk += 4) {
        const int c = (blk * a.B + b) * a.H + h;
        const uint32_t o0 = a.index[c], o1 = a.index[c + 1];
        if (o1 - o0 < uint32_t(HEADER / 16)) continue;  // dropped block contributes nothing
        const uint8_t *chunk = a.arena + size_t(o0) * 16;
        const int payload_bytes = int(o1 - o0) * 16 - HEADER;
        const int64_t tok = int64_t(blk) * N + lane;

        LaneHeader hd;
        {
            uint2 raw = *reinterpret_cast<const uint2 *>(chunk + lane * 8);
            hd.lo = raw.x;
            hd.hi = raw.y;
        }
        stage_payload(chunk + HEADER, payload_bytes, lds, lane);
        const uint32_t mt = a.meta[b * a.meta_stride + tok];
        const float scale = __half2float(__ushort_as_half(uint16_t(mt & 0xFFFFu)));
        const float mn = __half2float(__ushort_as_half(uint16_t(mt >> 16)));
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float pt = a.p[(int64_t(b) * a.H * G + h * G + g) * a.ld + tok];
            wlds_all[wave][g][lane] = pt * scale;
            pm[g] = fmaf(pt, mn, pm[g]);
        }
        const int my_bytes = hd.bytes();
        int pos = wave_inclusive_scan(my_bytes, lane) - my_bytes;

        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // the 16 weights of this lane's token group, and their sum
        float wv[G][16], wsum[G];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float4 *src = reinterpret_cast<const float4 *>(&wlds_all[wave][g][row * 16]);
            wsum[g] = 0.0f;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                float4 v = src[k];
                wv[g][4 * k + 0] = v.x;
                wv[g][4 * k + 1] = v.y;
                wv[g][4 * k + 2] = v.z;
                wv[g][4 * k + 3] = v.w;
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) wsum[g] += wv[g][i];
        }

#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int w = hd.width(j);
            const float m = float(hd.min(j));
            uint32_t lo, hi, L, Hh;
            read_pack(lds, pos, lo, hi);
            split_pack(lo, hi, w, L, Hh);
            pos += 2 * w;
            float part[G];
#pragma unroll
            for (int g = 0; g < G; ++g) part[g] = m * wsum[g];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float cl = float(__builtin_amdgcn_ubfe(L, i * w, w));
                const float chh = float(__builtin_amdgcn_ubfe(Hh, i * w, w));
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    part[g] = fmaf(wv[g][i], cl, part[g]);
                    part[g] = fmaf(wv[g][i + 8], chh, part[g]);
                }
            }
#pragma unroll
            for (int g = 0; g < G; ++g) acc[g][j] += part[g];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }

    // combine the four token-group rows of the wave, then the four waves
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            float v = acc[g][j];
            v += __shfl_xor(v, 16);
            v += __shfl_xor(v, 32);
            acc[g][j] = v;
        }
        float s = pm[g];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
        pm[g] = s;
        if (lane < 16) {
#pragma unroll
            for (int j = 0; j < 8; ++j) red[wave][g][8 * lane + j] = acc[g][j];
        }
        if (lane == 0) red[wave][g][D] = pm[g];
    }
    __syncthreads();
    for (int i = threadIdx.x; i < G * (D + 1); i += 256) {
        const int g = i / (D + 1), d = i % (D + 1);
        const float v = (red[0][g][d] + red[1][g][d]) + (red[2][g][d] + red[3][g][d]);
        a.partial[(int64_t(split) * a.B * a.H * G + (int64_t(b) * a.H * G + h * G + g)) * V_PART_STRIDE + d] = v;
    }
}

// Fixed-order combination of the split partial sums, plus the raw fp16 tail.
__global__ __launch_bounds__(128) void v_reduce_kernel(const float *__restrict__ partial,
                                                       int n_splits, int n_rows,
                                                       const float *__restrict__ p, int64_t ld,
                                                       int64_t packed_tokens,
                                                       const __half *__restrict__ tail, int n_tail,
                                                       int tail_cap, int H, int G,
                                                       float *__restrict__ out) {
    const int r = blockIdx.x;  // b*Hq + hq
    const int d = threadIdx.x;
    float acc = 0.0f, pmin = 0.0f;
    for (int s = 0; s < n_splits; ++s) {
        const float *src = partial + (int64_t(s) * n_rows + r) * V_PART_STRIDE;
        acc += src[d];
        pmin += src[D];
    }
    acc += pmin;
    if (n_tail > 0) {
        const int hq = r % (H * G), b = r / (H * G);
        const int h = hq / G;
        for (int t = 0; t < n_tail; ++t) {
            const float pt = p[int64_t(r) * ld + packed_tokens + t];
            const float v = __half2float(tail[((int64_t(b) * tail_cap + t) * H + h) * D + d]);
            acc = fmaf(pt, v, acc);
        }
    }
    out[int64_t(r) * D + d] = acc;
}

int v_splits_for(int n_blocks, int streams) {
    // enough workgroups to fill 256 CUs a few times over, at least one block per wave
    int want = (2048 + streams - 1) / streams;
    int by_blocks = (n_blocks + 3) / 4;
    int s = want < by_blocks ? want : by_blocks;
    if (s > V_SPLITS_MAX) s = V_SPLITS_MAX;
    if (s < 1) s = 1;
    return s;
}

int launch_v_matvec(const kv_cache *c, const float *p, int64_t ld_p, float *out, hipStream_t s) {
    const int B = c->cfg.batch, H = c->cfg.n_kv_heads, G = c->group;
    const int n_blocks = int(c->packed_tokens / N);
    uint8_t *ws = static_cast<uint8_t *>(c->buf.workspace);
    float *partial = reinterpret_cast<float *>(ws + WS_VPART);
    int n_splits = 0;
    if (n_blocks > 0) {
        n_splits = v_splits_for(n_blocks, B * H);
        VArgs a;
        a.arena = static_cast<const uint8_t *>(c->buf.v_arena);
        a.index = static_cast<const uint32_t *>(c->buf.v_index);
        a.meta = static_cast<const uint32_t *>(c->buf.v_token_meta);
        a.p = p;
        a.partial = partial;
        a.ld = ld_p;
        a.meta_stride = c->max_tokens;
        a.B = B;
        a.H = H;
        a.n_blocks = n_blocks;
        a.blocks_per_split = (n_blocks + n_splits - 1) / n_splits;
        n_splits = (n_blocks + a.blocks_per_split - 1) / a.blocks_per_split;
        dim3 grid(n_splits, B * H);
        switch (G) {
            case 1: hipLaunchKernelGGL(v_matvec_kernel<1>, grid, dim3(256), 0, s, a); break;
            case 2: hipLaunchKernelGGL(v_matvec_kernel<2>, grid, dim3(256), 0, s, a); break;
            case 4: hipLaunchKernelGGL(v_matvec_kernel<4>, grid, dim3(256), 0, s, a); break;
            case 8: hipLaunchKernelGGL(v_matvec_kernel<8>, grid, dim3(256), 0, s, a); break;
            default: return KV_ERR_UNSUPPORTED;
        }
    }
    hipLaunchKernelGGL(v_reduce_kernel, dim3(B * H * G), dim3(128), 0, s, partial, n_splits,
                       B * H * G, p, ld_p, c->packed_tokens,
                       static_cast<const __half *>(c->buf.v_tail), c->tail_tokens,
                       c->cfg.tail_capacity, H, G, out);
    KV_HIP_CHECK(hipGetLastError());
    return KV_OK;
}

}  // namespace packkv
