// Per-chunk V work shared by the V kernel and the fused decode-attention kernel
// (PackKV Sec. III-C.2): out += w^T code for the 64 tokens of one chunk that sits in
// an LDS buffer, w_t = p_t * scale_t.
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
#pragma once

#include "unpack.h"

namespace packkv {

typedef _Float16 vhalf8 __attribute__((ext_vector_type(8)));
typedef float vfloat4 __attribute__((ext_vector_type(4)));

// B operand staging per wave: [token group][half][column < 2G][8 fp16], then 16 zero
// bytes that the lanes of the unused columns (>= 2G) read instead.
template <int G>
struct BLds {
    static constexpr int COLS = 2 * G;
    static constexpr int ZERO = 4 * 2 * COLS * 16;
    static constexpr int BYTES = ZERO + 16;
};

// Per-lane constants of the B operand staging; `blds` is this wave's BLds<G>::BYTES array.
template <int G>
struct VLane {
    uint8_t *blds;
    int bslot;           // where this lane's own token (16*row + col) sits in the B operand (column 0)
    int bread0, bread1;  // where this lane reads its B operand halves from

    __device__ inline void init(uint8_t *wave_blds, int lane) {
        constexpr int COLS = BLds<G>::COLS;
        const int row = lane >> 4, col = lane & 15;
        blds = wave_blds;
        if (lane < 4) reinterpret_cast<uint32_t *>(blds + BLds<G>::ZERO)[lane] = 0;
        const int tm = col & 7;
        bslot = (((row * 2 + (tm >> 2)) * COLS) * 8 + 2 * (tm & 3) + (col >> 3)) * 2;
        bread0 = col < COLS ? ((row * 2 + 0) * COLS + col) * 16 : BLds<G>::ZERO;
        bread1 = col < COLS ? ((row * 2 + 1) * COLS + col) * 16 : BLds<G>::ZERO;
    }
};

// Running sums of one wave: MFMA tiles (lane = column col, rows 4*row+r of pack slot j), the
// pack-minimum term (lane = token group row, channels 8*col+j) and sum p*min per head.
template <int G>
struct VState {
    vfloat4 acc[8];
    float macc[fold_min<G>() ? 1 : G][8];  // unused when the minimum is folded into the codes
    float pm[G];

    __device__ inline void clear() {
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = vfloat4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int g = 0; g < G; ++g) pm[g] = 0.0f;
#pragma unroll
        for (int g = 0; g < (fold_min<G>() ? 1 : G); ++g)
#pragma unroll
            for (int j = 0; j < 8; ++j) macc[g][j] = 0.0f;
    }
};

// Adds the chunk in the LDS buffer at byte offset `cur` of lds_all: lane l is token l of the
// block with weight pt[g] for head g and token metadata mt (scale | min << 16).  `table` must
// have been built with lift CODE_LIFT and fold = fold_min<G>().
template <int G>
__device__ inline void v_chunk(const uint8_t *lds_all, int cur, const uint4 *table, const VLane<G> &vl,
                               uint32_t mt, const float (&pt)[G], VState<G> &st) {
    const float scale = __half2float(__ushort_as_half(uint16_t(mt & 0xFFFFu)));
    const float mn = __half2float(__ushort_as_half(uint16_t(mt >> 16)));
    float wsum[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const float w = pt[g] * scale;
        st.pm[g] = fmaf(pt[g], mn, st.pm[g]);
        // w = hi + lo with both parts fp16 (lo scaled by 2^11); hi is truncated, so lo >= 0
        const _Float16 hi = __builtin_bit_cast(
            _Float16, uint16_t(__builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(w, 0.0f)) & 0xFFFFu));
        const float lo = (w - float(hi)) * 2048.0f;
        const _Float16 lo16 = _Float16(lo);  // to nearest: the residual's rounding error has no sign bias
        *reinterpret_cast<_Float16 *>(vl.blds + vl.bslot + (2 * g) * 16) = hi;
        *reinterpret_cast<_Float16 *>(vl.blds + vl.bslot + (2 * g + 1) * 16) = lo16;
        if (!fold_min<G>()) wsum[g] = row_all_reduce16(w);
    }
    const uint2 hdr = *reinterpret_cast<const uint2 *>(lds_all + cur + (threadIdx.x & 63) * 8);
    LanePacks lp;
    lp.init(hdr.x, hdr.y, cur + HEADER);
    wave_lds_fence();

    const vhalf8 b0 = *reinterpret_cast<const vhalf8 *>(vl.blds + vl.bread0);
    const vhalf8 b1 = *reinterpret_cast<const vhalf8 *>(vl.blds + vl.bread1);
    PackRaw raw_next = fetch_pack(lds_all, table, lp.pos(0), lp.header_byte(0));
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        uint32_t P[8];
        const PackRaw raw = raw_next;
        // LDS reads run exactly one pack ahead of their use (the scheduling barrier keeps
        // the compiler from hoisting all eight fetches and blowing up register use)
        if (j < 7) raw_next = fetch_pack(lds_all, table, lp.pos(j + 1), lp.header_byte(j + 1));
        __builtin_amdgcn_sched_barrier(0);
        expand_pack<CODE_LIFT, fold_min<G>()>(raw, P);
        if constexpr (!fold_min<G>()) {
            const float m = __uint_as_float(raw.k.w);
#pragma unroll
            for (int g = 0; g < G; ++g) st.macc[g][j] = fmaf(m, wsum[g], st.macc[g][j]);
        }
        typedef uint32_t u32x4v __attribute__((ext_vector_type(4)));
        const vhalf8 a0 = __builtin_bit_cast(vhalf8, u32x4v{P[0], P[1], P[2], P[3]});
        const vhalf8 a1 = __builtin_bit_cast(vhalf8, u32x4v{P[4], P[5], P[6], P[7]});
        st.acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0, b0, st.acc[j], 0, 0, 0);
        st.acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1, b1, st.acc[j], 0, 0, 0);
    }
    wave_lds_fence();  // the B operand is rewritten by the next chunk
}

// Writes this wave's sums as red[g][0..127] (outputs) and red[g][128] (sum p*min).
// code_scale: what one unit of the A operand stands for (codes enter as code * 2^-24 * 2^lift).
template <int G>
__device__ inline void v_state_store(const VState<G> &st, float (*red)[D + 4], int lane,
                                     float code_scale = CODE_SCALE_LIFTED) {
    const int row = lane >> 4, col = lane & 15;
    const int head = col >> 1;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            float v = st.acc[j][r] * ((col & 1) ? code_scale / 2048.0f : code_scale);
            v += dpp_f32<DPP_QUAD_XOR1>(v);  // hi column + lo column
            if (!(col & 1) && head < G) red[head][8 * (4 * row + r) + j] = v;
        }
    }
    wave_lds_fence();
#pragma unroll
    for (int g = 0; g < G; ++g) {
        if constexpr (!fold_min<G>()) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                float v = st.macc[g][j];
                v += __shfl_xor(v, 16);
                v += __shfl_xor(v, 32);
                if (lane < 16) red[g][8 * lane + j] += v;
            }
        }
        float s = st.pm[g];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
        if (lane == 0) red[g][D] = s;
    }
}

}  // namespace packkv
