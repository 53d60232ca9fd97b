// Row softmax between the two fused matvecs (the smx of the attention definition,
// PackKV Sec. III-B.3): p[r][t] = exp(s[r][t] - max_t s[r]) / sum_t exp(s[r][t] - max_t s[r])
// over the first `tokens` entries of every row, in place, fp32.
//
// One workgroup of 1024 threads per row.  Rows of up to 64 Ki tokens are held in
// registers between the passes, so the scores are read once and written once; longer
// rows are re-read (from the last-level cache at these sizes).  Reductions run in a fixed
// order: bitwise reproducible.
#include <algorithm>

#include "common.h"

namespace packkv {

constexpr int SMX_THREADS = 1024;

__device__ inline float block_reduce(float v, bool is_max, float *lds) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float u = __shfl_xor(v, o);
        v = is_max ? fmaxf(v, u) : v + u;
    }
    __syncthreads();  // protects lds against the previous reduction
    if (lane == 0) lds[wave] = v;
    __syncthreads();
    float r = lds[0];
#pragma unroll
    for (int k = 1; k < SMX_THREADS / 64; ++k) r = is_max ? fmaxf(r, lds[k]) : r + lds[k];
    return r;
}

// NREG > 0: thread t holds elements t, t + 1024, ... (NREG of them) in registers.
// Scores of -inf (blocks dropped by an arena overflow) get weight 0; a row that holds nothing else
// comes out as zeros.
__device__ inline float finite_max(float mx) { return mx == -INFINITY ? 0.0f : mx; }
__device__ inline float safe_inverse(float sum) { return sum > 0.0f ? 1.0f / sum : 0.0f; }

// NREG == 0: rows of any length, three passes over memory.
template <int NREG>
__global__ __launch_bounds__(SMX_THREADS) void softmax_kernel(float *__restrict__ s, int64_t ld,
                                                              int64_t tokens) {
    __shared__ float lds[SMX_THREADS / 64];
    float *row = s + int64_t(blockIdx.x) * ld;
    constexpr float LOG2E = 1.4426950408889634f;
    if constexpr (NREG > 0) {
        float x[NREG];
        float mx = -INFINITY;
#pragma unroll
        for (int k = 0; k < NREG; ++k) {
            const int64_t i = int64_t(k) * SMX_THREADS + threadIdx.x;
            x[k] = i < tokens ? row[i] : -INFINITY;
            mx = fmaxf(mx, x[k]);
        }
        mx = finite_max(block_reduce(mx, true, lds));
        float sum = 0.0f;
#pragma unroll
        for (int k = 0; k < NREG; ++k) {
            x[k] = exp2f((x[k] - mx) * LOG2E);  // 0 for the padding entries
            sum += x[k];
        }
        sum = block_reduce(sum, false, lds);
        const float inv = safe_inverse(sum);
#pragma unroll
        for (int k = 0; k < NREG; ++k) {
            const int64_t i = int64_t(k) * SMX_THREADS + threadIdx.x;
            if (i < tokens) row[i] = x[k] * inv;
        }
    } else {
        float mx = -INFINITY;
        for (int64_t i = threadIdx.x; i < tokens; i += SMX_THREADS) mx = fmaxf(mx, row[i]);
        mx = finite_max(block_reduce(mx, true, lds));
        float sum = 0.0f;
        for (int64_t i = threadIdx.x; i < tokens; i += SMX_THREADS) sum += exp2f((row[i] - mx) * LOG2E);
        sum = block_reduce(sum, false, lds);
        const float inv = safe_inverse(sum);
        for (int64_t i = threadIdx.x; i < tokens; i += SMX_THREADS)
            row[i] = exp2f((row[i] - mx) * LOG2E) * inv;
    }
}

// Long rows and few of them: every row is cut into segments so that the chip is filled.
// First kernel: (max, sum of exp relative to that max) per segment; second kernel: merge the
// segment statistics of the row in a fixed order and write the normalized segment.
__global__ __launch_bounds__(SMX_THREADS) void softmax_stats_kernel(const float *__restrict__ s,
                                                                    int64_t ld, int64_t tokens,
                                                                    int64_t seg, float2 *__restrict__ stats) {
    __shared__ float lds[SMX_THREADS / 64];
    constexpr float LOG2E = 1.4426950408889634f;
    const float *row = s + int64_t(blockIdx.y) * ld;
    const int64_t lo = int64_t(blockIdx.x) * seg, hi = lo + seg < tokens ? lo + seg : tokens;
    float mx = -INFINITY;
    for (int64_t i = lo + threadIdx.x; i < hi; i += SMX_THREADS) mx = fmaxf(mx, row[i]);
    mx = block_reduce(mx, true, lds);
    const float ref = finite_max(mx);
    float sum = 0.0f;
    for (int64_t i = lo + threadIdx.x; i < hi; i += SMX_THREADS) sum += exp2f((row[i] - ref) * LOG2E);
    sum = block_reduce(sum, false, lds);
    if (threadIdx.x == 0) stats[int64_t(blockIdx.y) * gridDim.x + blockIdx.x] = make_float2(mx, sum);
}

__global__ __launch_bounds__(SMX_THREADS) void softmax_apply_kernel(float *__restrict__ s, int64_t ld,
                                                                    int64_t tokens, int64_t seg,
                                                                    const float2 *__restrict__ stats) {
    constexpr float LOG2E = 1.4426950408889634f;
    float *row = s + int64_t(blockIdx.y) * ld;
    const float2 *st = stats + int64_t(blockIdx.y) * gridDim.x;
    float mx = -INFINITY;
    for (unsigned k = 0; k < gridDim.x; ++k) mx = fmaxf(mx, st[k].x);
    mx = finite_max(mx);
    float sum = 0.0f;
    for (unsigned k = 0; k < gridDim.x; ++k) sum += st[k].y * exp2f((st[k].x - mx) * LOG2E);
    const float inv = safe_inverse(sum);
    const int64_t lo = int64_t(blockIdx.x) * seg, hi = lo + seg < tokens ? lo + seg : tokens;
    for (int64_t i = lo + threadIdx.x; i < hi; i += SMX_THREADS) row[i] = exp2f((row[i] - mx) * LOG2E) * inv;
}

int launch_softmax(const kv_cache *c, float *scores, int64_t ld, hipStream_t s) {
    const int64_t rows = int64_t(c->cfg.batch) * c->cfg.n_q_heads;
    const int64_t tokens = c->packed_tokens + c->tail_tokens;
    // one workgroup per row when the rows alone fill the 256 compute units (one pass over memory);
    // otherwise segments of at least 4096 tokens, enough for about 512 workgroups, at most 64
    int64_t splits = rows >= 256 ? 1
                                 : std::min<int64_t>(std::min<int64_t>((512 + rows - 1) / rows, tokens / 4096),
                                                     V_SPLITS_MAX);
    if (splits <= 1) {
        const dim3 grid(static_cast<unsigned>(rows)), block(SMX_THREADS);
        if (tokens <= 8 * SMX_THREADS)
            hipLaunchKernelGGL(softmax_kernel<8>, grid, block, 0, s, scores, ld, tokens);
        else if (tokens <= 32 * SMX_THREADS)
            hipLaunchKernelGGL(softmax_kernel<32>, grid, block, 0, s, scores, ld, tokens);
        else if (tokens <= 64 * SMX_THREADS)
            hipLaunchKernelGGL(softmax_kernel<64>, grid, block, 0, s, scores, ld, tokens);
        else
            hipLaunchKernelGGL(softmax_kernel<0>, grid, block, 0, s, scores, ld, tokens);
    } else {
        const int64_t seg = ((tokens + splits - 1) / splits + 63) / 64 * 64;
        splits = (tokens + seg - 1) / seg;
        // segment statistics live where the V splits put their partial sums later in the step
        float2 *stats = reinterpret_cast<float2 *>(static_cast<uint8_t *>(c->buf.workspace) + WS_VPART);
        const dim3 grid(static_cast<unsigned>(splits), static_cast<unsigned>(rows)), block(SMX_THREADS);
        hipLaunchKernelGGL(softmax_stats_kernel, grid, block, 0, s, scores, ld, tokens, seg, stats);
        hipLaunchKernelGGL(softmax_apply_kernel, grid, block, 0, s, scores, ld, tokens, seg, stats);
    }
    KV_HIP_CHECK(hipGetLastError());
    return KV_OK;
}

}  // namespace packkv

using namespace packkv;

extern "C" int kv_softmax(kv_cache_t *c, float *scores, int64_t ld_scores, void *hip_stream) {
    if (!c || !scores) return KV_ERR_ARG;
    const int64_t tokens = c->packed_tokens + c->tail_tokens;
    if (tokens < 1 || ld_scores < tokens) return KV_ERR_ARG;
    if (int64_t(c->cfg.batch) * c->cfg.n_q_heads > 65535) return KV_ERR_UNSUPPORTED;
    return launch_softmax(c, scores, ld_scores, static_cast<hipStream_t>(hip_stream));
}
