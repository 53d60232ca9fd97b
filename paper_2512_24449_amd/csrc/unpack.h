// Device helpers shared by the fused K and V kernels: wave-level prefix sum,
// staging of a chunk's payload in LDS, reading one pack out of LDS, and the
// 16-lane reduce-scatter used by the K path.  gfx950, wave64.
#pragma once

#include "common.h"

namespace packkv {

// LDS bytes reserved per wave for a chunk payload: 512 packs * 8 bytes plus
// slack for the 12 bytes a pack read may touch past the payload end.
constexpr int PAYLOAD_LDS = PACKS * 8 + 16;

// DPP controls (wave64, rows of 16 lanes).
constexpr int DPP_QUAD_XOR1 = 0xB1;  // quad_perm [1,0,3,2]
constexpr int DPP_QUAD_XOR2 = 0x4E;  // quad_perm [2,3,0,1]
constexpr int DPP_ROW_ROR8 = 0x128;  // lane i <- lane i^8 of its row

template <int CTRL>
__device__ inline float dpp_f32(float v) {
    return __int_as_float(
        __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}

// Inclusive prefix sum over the 64 lanes of a wave.
__device__ inline int wave_inclusive_scan(int v, int lane) {
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        int n = __shfl_up(v, o);
        if (lane >= o) v += n;
    }
    return v;
}

// Sum of the four bytes of x.
__device__ inline uint32_t byte_sum(uint32_t x) { return (x * 0x01010101u) >> 24; }

// Per-lane view of a chunk header: lane l owns packs 8l .. 8l+7, i.e. token
// group g = l / 16 and channels 8*(l % 16) .. +7.
struct LaneHeader {
    uint32_t lo, hi;  // eight header bytes, pack j in byte j
    __device__ inline int width(int j) const { return ((j < 4 ? lo : hi) >> (8 * (j & 3) + 4)) & 15; }
    __device__ inline int min(int j) const { return ((j < 4 ? lo : hi) >> (8 * (j & 3))) & 15; }
    // payload bytes of this lane's eight packs
    __device__ inline int bytes() const {
        return 2 * int(byte_sum((lo >> 4) & 0x0F0F0F0Fu) + byte_sum((hi >> 4) & 0x0F0F0F0Fu));
    }
};

// Copy `payload_bytes` (multiple of 16 after padding) of a chunk payload from
// global memory into this wave's LDS region with 16-byte lane accesses.
__device__ inline void stage_payload(const uint8_t *__restrict__ payload, int payload_bytes,
                                     uint8_t *lds, int lane) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        int off = (lane + 64 * k) * 16;
        if (off < payload_bytes)
            *reinterpret_cast<uint4 *>(lds + off) = *reinterpret_cast<const uint4 *>(payload + off);
    }
}

// The 64-bit window of LDS starting at byte `pos` (2-byte aligned).
__device__ inline void read_pack(const uint8_t *lds, int pos, uint32_t &lo, uint32_t &hi) {
    const uint32_t *p = reinterpret_cast<const uint32_t *>(lds + (pos & ~3));
    uint32_t d0 = p[0], d1 = p[1], d2 = p[2];
    uint32_t sh = (pos & 2) * 8;
    lo = __builtin_amdgcn_alignbit(d1, d0, sh);
    hi = __builtin_amdgcn_alignbit(d2, d1, sh);
}

// Split a pack into the words holding tokens 0..7 (L) and 8..15 (Hh): token m
// of either half sits at bit m*w of its word.
__device__ inline void split_pack(uint32_t lo, uint32_t hi, int w, uint32_t &L, uint32_t &Hh) {
    L = lo;
    uint32_t shifted = __builtin_amdgcn_alignbit(hi, lo, 8 * w);  // w < 4: bits [8w, 8w+32)
    Hh = w == 4 ? hi : shifted;
}

// Reduce-scatter inside each row of 16 lanes: on entry every lane holds 16
// partial sums v[0..15]; on return lane i of the row holds sum over the row's
// lanes of v[i].
__device__ inline float row_reduce_scatter16(float (&v)[16], int lane) {
    float a[8], b[4], c[2];
    const bool b3 = lane & 8, b2 = lane & 4, b1 = lane & 2, b0 = lane & 1;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        float keep = b3 ? v[k + 8] : v[k];
        float send = b3 ? v[k] : v[k + 8];
        a[k] = keep + dpp_f32<DPP_ROW_ROR8>(send);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        float keep = b2 ? a[k + 4] : a[k];
        float send = b2 ? a[k] : a[k + 4];
        b[k] = keep + __shfl_xor(send, 4);
    }
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        float keep = b1 ? b[k + 2] : b[k];
        float send = b1 ? b[k] : b[k + 2];
        c[k] = keep + dpp_f32<DPP_QUAD_XOR2>(send);
    }
    float keep = b0 ? c[1] : c[0];
    float send = b0 ? c[0] : c[1];
    return keep + dpp_f32<DPP_QUAD_XOR1>(send);
}

// Sum over the 16 lanes of a row, result in every lane of the row.
__device__ inline float row_all_reduce16(float v) {
    v += dpp_f32<DPP_ROW_ROR8>(v);
    v += __shfl_xor(v, 4);
    v += dpp_f32<DPP_QUAD_XOR2>(v);
    v += dpp_f32<DPP_QUAD_XOR1>(v);
    return v;
}

}  // namespace packkv
