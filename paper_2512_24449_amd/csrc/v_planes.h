// Per-chunk V work for chunks in the plane layout (packs of 16 tokens), shared by the V kernel
// and the fused decode-attention kernel (PackKV Sec. III-C.2): out += w^T code for the 64 tokens
// of one chunk that sits in an LDS buffer, w_t = p_t * scale_t.
//
// The contraction runs along the pack direction, so the planes of a pack go to the matrix cores
// as they are stored, widened to FP4 nibbles (planes.h): for pack slot j the wave issues
//     C_j[channel row][column] += A[row][k] * B[k][column]       (16x16x128, A FP4, B FP8)
// where row = lane % 16 is channel 8 * row + j, lane / 16 is the token group, and a lane's 32
// k-values are the 16 tokens of its pack in plane L followed by the same 16 tokens in plane T
// (for caches whose codes need four bits, plane H takes a second instruction).  B holds the weights of the chunk's 64 tokens in the same token order, the same
// bytes for both planes: a weight is an integer of 4 * PIECES bits relative to the largest weight
// of the chunk (round to nearest), one four-bit digit per column -- an FP8 byte below 16 is the
// number byte * 2^-9 -- and the chunk's power-of-two unit is the instruction's block scale on B.
// Place values inside a pack: plane H counts 4 (the block scale of its instruction), plane T
// counts 1 or 4 (bit position 0 or 2 inside the nibble: FP4 0.5 or 2.0).  Accumulation is fp32
// inside the instruction; the columns of a head are added up, with their powers of 16, once at
// the end.  De-quantization is folded in, with the SAME rounded weights w' in every term so that
// the rounding acts as a perturbation of p and is not amplified by the cancellation between the
// terms:
//   out_d = sum_t w'_t code[t,d] + sum_g m[g,d] sum_{t in g} w'_t + sum_t (w'_t / scale_t) min_t
#pragma once

#include "planes.h"

namespace packkv {

// Four-bit digits per weight: as many as fit the 16 columns, at most five (the rounding uses the
// fp32 "add 2^23" trick, exact below 2^23).
template <int G>
constexpr int v_pieces() { return G <= 3 ? 5 : 4; }

// Per-width constants (LDS, entry w = 0..4): x = mask of plane L (two-bit fields, or 0 without
// the plane), y = mask of plane T once widened (one bit per nibble at the bit's place value: bit 0
// for width 1, bit 2 for width 3, or 0 without the plane), z, w = right rotations that bring the
// doubled word of plane T under that mask for tokens 0..7 and 8..15.  highs[w] = mask of plane H.
constexpr int PLANE_TABLE_ENTRIES = 5;
__device__ inline void build_plane_table(uint4 *table, uint32_t *highs) {
    const uint32_t w = threadIdx.x;
    if (w < PLANE_TABLE_ENTRIES) {
        table[w] = make_uint4(w >= 2 ? FIELD2_MASK : 0u, w == 1 ? 0x11111111u : w == 3 ? 0x44444444u : 0u,
                              w == 3 ? 30u : 0u, w == 3 ? 0u : 2u);
        if (highs) highs[w] = w == 4 ? FIELD2_MASK : 0u;
    }
    __syncthreads();
}

// B operand staging per wave: digit bytes [column][token 0..63] for the columns in use, then a row
// of zeros that the lanes of the unused columns read.
template <int G>
constexpr int vb_bytes() { return (v_pieces<G>() * G + 1) * 64; }

template <int G>
struct VPlaneState {
    pk_v4f acc[8];     // lane (column n, row group rg): channels 8 * (4 rg + r) + j, column n
    float macc[G][8];  // pack-minimum term: lane (token group, channel 8 * (lane % 16) + j)
    float pm[G];       // sum of w' / scale * min over this lane's tokens

    __device__ inline void clear() {
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = pk_v4f{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int g = 0; g < G; ++g) {
            pm[g] = 0.0f;
#pragma unroll
            for (int j = 0; j < 8; ++j) macc[g][j] = 0.0f;
        }
    }
};

struct PlaneRaw {
    uint32_t L, H, T;  // words as stored (H, T arbitrary when the pack has no such plane)
    uint4 k;           // plane table entry
    uint32_t kh;       // mask of plane H
};

// wsel: the lane's eight header bytes with the minimum nibble cleared (16 * width per byte), split
// in two words like the header itself.
template <bool HIGH>
__device__ inline PlaneRaw fetch_planes(const uint8_t *lds0, const uint4 *table, const uint32_t *highs,
                                        const LanePlanes &lp, uint32_t wsel_lo, uint32_t wsel_hi, int j) {
    PlaneRaw r;
    const uint32_t *e = reinterpret_cast<const uint32_t *>(lds0 + lp.e_pos(j));
    r.L = e[0];
    r.H = HIGH ? e[1] : 0u;
    r.T = *reinterpret_cast<const uint16_t *>(lds0 + lp.o_pos(j));
    const uint32_t w16 = ((j < 4 ? wsel_lo : wsel_hi) >> (8 * (j & 3))) & 0xFFu;   // 16 * width: the entry's byte offset
    r.k = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint8_t *>(table) + w16);
    r.kh = HIGH ? *reinterpret_cast<const uint32_t *>(reinterpret_cast<const uint8_t *>(highs) + (w16 >> 2)) : 0u;
    return r;
}

// Plane T widened to nibbles in token order: two words, tokens 0..7 and 8..15.  The bit of token
// t = 4r + s sits at 4s + r of the stored word T; in y = T | T << 15 the bits of tokens 0..7 sit
// at 4n and those of tokens 8..15 at 4n + 2 (n = token % 8), and a rotation moves them to the bit
// of the nibble that carries the plane's place value.
__device__ inline void widen_top_plane(const PlaneRaw &r, uint32_t &t0, uint32_t &t1) {
    const uint32_t y = r.T | (r.T << 15);
    t0 = __builtin_amdgcn_alignbit(y, y, r.k.z) & r.k.y;
    t1 = __builtin_amdgcn_alignbit(y, y, r.k.w) & r.k.y;
}

// Adds the chunk in the LDS buffer at byte offset `cur` of lds_all: lane l is token l of the
// block with weight pt[g] for head g and token metadata mt (scale | min << 16).  vb: this wave's
// vb_bytes<G>() staging array (its last row zeroed once).  HIGH: the cache's codes may need four
// bits (a plane H exists).
template <int G, bool HIGH>
__device__ inline void v_planes_chunk(const uint8_t *lds_all, int cur, const uint4 *table, const uint32_t *highs,
                                      uint8_t *vb, uint32_t mt, const float (&pt)[G], VPlaneState<G> &st) {
    constexpr int NP = v_pieces<G>(), BITS = 4 * NP;
    constexpr float MAGIC = 8388608.0f;  // 2^23
    const int lane = threadIdx.x & 63;
    const float scale = __half2float(__ushort_as_half(uint16_t(mt & 0xFFFFu)));
    const float mn = __half2float(__ushort_as_half(uint16_t(mt >> 16)));
    const float ratio = scale != 0.0f ? mn * __builtin_amdgcn_rcpf(scale) : 0.0f;
    float wsum[G];
    int sb[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const float w = pt[g] * scale;
        // the chunk's unit: with E the biased exponent of the largest weight, weights are counted
        // in steps of 2^(E - 126 - BITS), so every count stays below 2^BITS
        const int E = int(wave_max_bits(w) >> 23);
        const int mul_field = min(254, 253 + BITS - E);     // 2^(BITS + 126 - E), capped
        const int unit_field = max(0, E + 1 - BITS);        // 2^(E - 126 - BITS), or 0 below the float range
        const float y = fmaf(w, __int_as_float(mul_field << 23), MAGIC);  // round to nearest even
        const uint32_t X = min(uint32_t(__float_as_int(y)) & 0x7FFFFFu, (1u << BITS) - 1u);
        const float wq = float(X) * __int_as_float(unit_field << 23);      // the rounded weight w'
        st.pm[g] = fmaf(scale != 0.0f ? wq : pt[g], scale != 0.0f ? ratio : mn, st.pm[g]);
        wsum[g] = row_all_reduce16(wq);
#pragma unroll
        for (int k = 0; k < NP; ++k) vb[(NP * g + k) * 64 + lane] = uint8_t((X >> (4 * k)) & 15u);
        sb[g] = min(252, unit_field) + 1;  // E8M0 byte of the unit, one above (see v_planes_scale)
    }
    const uint2 hdr = *reinterpret_cast<const uint2 *>(lds_all + cur + lane * 8);
    LanePlanes lp;
    lp.init(hdr.x, hdr.y, cur + HEADER);
    wave_lds_fence();

    // B operand of this lane: column n = lane % 16, k-groups lane / 16 and 4 + lane / 16, i.e. the
    // tokens of token groups (lane / 32) and 2 + (lane / 32)
    const int col = lane & 15, kgb = lane >> 4;
    const int brow = (col < NP * G ? col : NP * G) * 64 + (kgb >> 1) * 16;
    const uint4 b_lo = *reinterpret_cast<const uint4 *>(vb + brow);
    const uint4 b_hi = *reinterpret_cast<const uint4 *>(vb + brow + 32);
    const pk_v8i B = {int(b_lo.x), int(b_lo.y), int(b_lo.z), int(b_lo.w), int(b_hi.x), int(b_hi.y), int(b_hi.z), int(b_hi.w)};
    int sbv = sb[0];
#pragma unroll
    for (int g = 1; g < G; ++g) sbv = (col >= NP * g) ? sb[g] : sbv;

    const uint32_t wsel_lo = hdr.x & 0xF0F0F0F0u, wsel_hi = hdr.y & 0xF0F0F0F0u;
    const uint32_t min_lo = hdr.x & 0x0F0F0F0Fu, min_hi = hdr.y & 0x0F0F0F0Fu;
    PlaneRaw raw_next = fetch_planes<HIGH>(lds_all, table, highs, lp, wsel_lo, wsel_hi, 0);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const PlaneRaw raw = raw_next;
        // LDS reads run one pack ahead of their use
        if (j < 7) raw_next = fetch_planes<HIGH>(lds_all, table, highs, lp, wsel_lo, wsel_hi, j + 1);
        __builtin_amdgcn_sched_barrier(0);
        uint32_t t0, t1;
        widen_top_plane(raw, t0, t1);
        const uint32_t l0 = raw.L & raw.k.x, l1 = (raw.L >> 2) & raw.k.x;
        const pk_v8i a = {int(l0), int(l1), int(t0), int(t1), 0, 0, 0, 0};
        st.acc[j] = mfma_fp4_fp8(a, B, st.acc[j], E8M0_ONE, sbv);
        if constexpr (HIGH) {
            // a block scale covers the 32 k-values of a lane, so plane H, which counts 4, takes an
            // instruction of its own
            const uint32_t h0 = raw.H & raw.kh, h1 = (raw.H >> 2) & raw.kh;
            const pk_v8i a_high = {int(h0), int(h1), 0, 0, 0, 0, 0, 0};
            st.acc[j] = mfma_fp4_fp8(a_high, B, st.acc[j], E8M0_ONE + 2, sbv);
        }
        const float m = float(((j < 4 ? min_lo : min_hi) >> (8 * (j & 3))) & 0xFFu);
#pragma unroll
        for (int g = 0; g < G; ++g) st.macc[g][j] = fmaf(m, wsum[g], st.macc[g][j]);
    }
    wave_lds_fence();  // the staging array is rewritten by the next chunk
}

// What one unit of a result tile stands for: FP4 nibbles are field / 2, FP8 digits byte * 2^-9,
// and the block scale was taken one above the unit.
constexpr float V_PLANES_OUT_SCALE = 512.0f;  // 2 * 2^9 / 2

template <int N_SHIFT>
__device__ inline float row_shl0(float v) {   // lane i <- lane i + N_SHIFT of its row of 16, 0 past the row's end
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x100 + N_SHIFT, 0xF, 0xF, true));
}

// Writes this wave's sums as red[g][0..127] (outputs) and red[g][128] (the token-minimum term).
// The digits of a head sit in neighbouring columns (lanes of a row): the first of them collects
// the others in a fixed order.
template <int G>
__device__ inline void v_planes_store(const VPlaneState<G> &st, float (*red)[D + 4], int lane) {
    constexpr int NP = v_pieces<G>();
    const int rg = lane >> 4, col = lane & 15;
    const int head = col / NP, piece = col % NP;
    const float place = head < G ? V_PLANES_OUT_SCALE * float(1u << (4 * piece)) : 0.0f;
    // pack-minimum term first: lanes 0..15 cover every channel of every head
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            float v = st.macc[g][j];
            v += __shfl_xor(v, 16);
            v += __shfl_xor(v, 32);
            if (lane < 16) red[g][8 * lane + j] = v;
        }
        float s = st.pm[g];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
        if (lane == 0) red[g][D] = s;
    }
    wave_lds_fence();
    const bool first = piece == 0 && head < G;
    float *row = red[first ? head : 0] + 32 * rg;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        // four sums at a time keep the register count of the main loop
        float sum[4], cur[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float v = st.acc[j][r] * place;
            float t = v + row_shl0<1>(v);
            t += row_shl0<2>(v);
            t += row_shl0<3>(v);
            if constexpr (NP == 5) t += row_shl0<4>(v);
            sum[r] = t;
        }
        if (first) {
#pragma unroll
            for (int r = 0; r < 4; ++r) cur[r] = row[8 * r + j];
#pragma unroll
            for (int r = 0; r < 4; ++r) row[8 * r + j] = cur[r] + sum[r];
        }
    }
}

}  // namespace packkv
