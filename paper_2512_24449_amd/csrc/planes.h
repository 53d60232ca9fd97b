// Device helpers for chunks in the plane layout (packs of 16 tokens, packkv.h): where the
// planes of a lane's eight packs sit in an LDS chunk buffer, and the matrix-core instruction
// both fused kernels feed them to.
//
// A pack of width w stores its 16 codes as two-bit planes -- a word L with the low two bits of
// every code when w >= 2, a word H with the high two bits when w == 4, both in region E -- and
// a one-bit plane, a 16-bit word T with the top bit of every code when w is odd, in region O.
// The planes feed v_mfma_scale_f32_16x16x128_f8f6f4 as FP4 (E2M1) operands: a nibble holding a
// two-bit field f is the FP4 number f/2 and a nibble holding one bit at position 0 or 1 is 0.5
// or 1.0, so widening a plane to nibbles is all the unpacking there is:
//     L & 0x33333333, (L >> 2) & 0x33333333      tokens 0..7, tokens 8..15 of the pack
// and the place value of a plane (1 for L, 4 for H, 1 or 4 for T) is a power of two that the
// instruction's per-lane block scales apply for free.  The other operand (softmax weights for V,
// the query for K) is split into FP8 (E4M3) pieces.
//
// Operand layout of the instruction (measured on gfx950): k runs in eight groups of 16; a lane
// holds row or column lane % 16; an FP4 operand lane (4 registers) holds k-groups 2*(lane/16)
// and 2*(lane/16) + 1, nibble i of the 32 <-> k = 32*(lane/16) + i; an FP8 operand lane
// (8 registers) holds k-group lane/16 in bytes 0..15 and k-group 4 + lane/16 in bytes 16..31.
// The result tile is the usual one: register r of lane (n = lane % 16, rg = lane / 16) is
// row 4*rg + r, column n.  A block scale is an E8M0 byte (127 = 1.0) per lane.
#pragma once

#include "unpack.h"

namespace packkv {

typedef int pk_v8i __attribute__((ext_vector_type(8)));
typedef float pk_v4f __attribute__((ext_vector_type(4)));

constexpr uint32_t FIELD2_MASK = 0x33333333u;   // the low two bits of every nibble
constexpr int E8M0_ONE = 127;

// D = A (FP8 E4M3, 16 x 128) * B (FP4 E2M1, 128 x 16) + C with per-lane block scales.
__device__ inline pk_v4f mfma_fp8_fp4(const pk_v8i &a, const pk_v8i &b, pk_v4f c, int scale_a, int scale_b) {
    return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c, 0, 4, 0, scale_a, 0, scale_b);
}
// D = A (FP4, 16 x 128) * B (FP8, 128 x 16) + C.
__device__ inline pk_v4f mfma_fp4_fp8(const pk_v8i &a, const pk_v8i &b, pk_v4f c, int scale_a, int scale_b) {
    return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c, 4, 0, 0, scale_a, 0, scale_b);
}

// Per-lane view of a chunk header in the plane layout: lane l owns packs 8l..8l+7 of the pack
// list (header bytes 8l..8l+7); their planes sit in list order in regions E and O.
struct LanePlanes {
    uint32_t hlo, hhi;    // eight header bytes, pack j in byte j
    uint32_t elo, ehi;    // byte j: region-E bytes of packs 0..j (elo) resp. 4..j (ehi) of this lane
    uint32_t olo, ohi;    // the same for region O
    int e0, e4, o0, o4;   // LDS byte addresses of the region-E / region-O data of packs 0 and 4

    // lds_payload: LDS byte address of region E of this chunk (right behind the header)
    __device__ inline void init(uint32_t lo, uint32_t hi, int lds_payload) {
        hlo = lo;
        hhi = hi;
        const uint32_t tl = lo >> 3, th = hi >> 3;          // width nibble moved to bits 1..3 of each byte
        elo = byte_prefix_sums(tl & 0x0C0C0C0Cu);           // 4 bytes per two-bit plane: 4 * (w >> 1)
        ehi = byte_prefix_sums(th & 0x0C0C0C0Cu);
        olo = byte_prefix_sums(tl & 0x02020202u);           // 2 bytes for an odd width
        ohi = byte_prefix_sums(th & 0x02020202u);
        const int e_mid = int(elo >> 24), o_mid = int(olo >> 24);
        const int e_lane = e_mid + int(ehi >> 24), o_lane = o_mid + int(ohi >> 24);
        // one scan carries both regions: E bytes in the low half, O bytes in the high half
        const int both = e_lane | (o_lane << 16);
        const int inc = wave_inclusive_scan(both);
        const int total = __builtin_amdgcn_readlane(inc, 63);
        const int excl = inc - both;
        e0 = lds_payload + (excl & 0xFFFF);
        o0 = lds_payload + (total & 0xFFFF) + (excl >> 16);
        e4 = e0 + e_mid;
        o4 = o0 + o_mid;
    }
    __device__ inline uint32_t header_byte(int j) const { return ((j < 4 ? hlo : hhi) >> (8 * (j & 3))) & 0xFFu; }
    // LDS byte address of the region-E data (word L, then H) of pack j
    __device__ inline int e_pos(int j) const {
        if (j == 0) return e0;
        if (j == 4) return e4;
        const int k = j - 1;
        return (j < 4 ? e0 : e4) + int(((j < 4 ? elo : ehi) >> (8 * (k & 3))) & 0xFFu);
    }
    // LDS byte address of the region-O word of pack j
    __device__ inline int o_pos(int j) const {
        if (j == 0) return o0;
        if (j == 4) return o4;
        const int k = j - 1;
        return (j < 4 ? o0 : o4) + int(((j < 4 ? olo : ohi) >> (8 * (k & 3))) & 0xFFu);
    }
};

// Largest float bit pattern of the non-negative values v over the wave, the same in every lane
// (non-negative floats order like their bit patterns).
__device__ inline uint32_t wave_max_bits(float v) {
    int x = __float_as_int(v);
    x = max(x, __builtin_amdgcn_update_dpp(0, x, DPP_ROW_ROR8, 0xF, 0xF, false));
    x = max(x, __builtin_amdgcn_update_dpp(0, x, DPP_ROW_ROR4, 0xF, 0xF, false));
    x = max(x, __builtin_amdgcn_update_dpp(0, x, DPP_QUAD_XOR2, 0xF, 0xF, false));
    x = max(x, __builtin_amdgcn_update_dpp(0, x, DPP_QUAD_XOR1, 0xF, 0xF, false));
    const int r0 = __builtin_amdgcn_readlane(x, 0), r1 = __builtin_amdgcn_readlane(x, 16);
    const int r2 = __builtin_amdgcn_readlane(x, 32), r3 = __builtin_amdgcn_readlane(x, 48);
    return uint32_t(max(max(r0, r1), max(r2, r3)));
}

}  // namespace packkv
