// Weight staging and running sums of the V paths for chunks with packs of 8 tokens and for wide
// chunks (pack8.h; PackKV Sec. III-C.2): out += w^T code for the 64 tokens of one chunk that sits
// in an LDS buffer, w_t = p_t * scale_t.
//
// The contraction runs along the pack direction, so it maps onto the matrix cores without any
// transposition: for pack slot jj the wave issues
//     C_jj[channel row i][column] += A[i][k] * B[k][column]      (16x16x32 fp16 MFMA)
// where row i is lane%16 (channel 8i+jj), A holds the unpacked codes (fp16 code * 2^-24, lifted)
// and B holds the weights w_t = p_t * scale_t split into fp16 hi and lo*2^11 parts, one column
// pair per query head (fp32-accurate weights cost no extra MFMA and the G query heads of a group
// share one unpack).  Accumulation is fp32 inside the MFMA, in a fixed order; de-quantization is
// folded in:
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
