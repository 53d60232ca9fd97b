// Device helpers shared by the fused K and V kernels (gfx950, wave64):
// DPP wave scan and row reductions, chunk prologue (header -> per-pack LDS
// positions, payload staging) and the register unpack of one pack into
// fp16 pairs.
//
// Lane-to-pack mapping used by both kernels: lane l of the wave that owns a
// chunk reads header bytes 8l..8l+7, i.e. it owns token group g = l/16
// (tokens 16g..16g+15) and channels 8*(l%16)..+7; its eight packs are
// contiguous in the payload.
//
// Unpack: the codes of a pack never become fp32 one by one.  Aligned LDS reads
// and funnel shifts fetch tokens 0..7 and 8..15; byte permutes build two words
// whose low/high 16-bit halves hold tokens (m, m+8) at equal bit offsets, and
// a rotate + mask per token pair leaves each code in the low bits of a 16-bit
// half.  Read as fp16 that bit pattern is the subnormal code * 2^-24 -- exact,
// no conversion instruction -- ready for v_fma_mix_f32 or an fp16 MFMA; the
// factor 2^24 is applied once per output.
#pragma once

#include "common.h"

namespace packkv {

// LDS bytes reserved per wave for a chunk payload: 512 packs * 8 bytes plus
// slack for the bytes a pack read may touch past the payload end.
constexpr int PAYLOAD_LDS = PACKS * 8 + 16;
constexpr float CODE_SCALE = 16777216.0f;  // 2^24: fp16 subnormal unit^-1

// DPP controls (wave64, rows of 16 lanes).
constexpr int DPP_QUAD_XOR1 = 0xB1;  // quad_perm [1,0,3,2]
constexpr int DPP_QUAD_XOR2 = 0x4E;  // quad_perm [2,3,0,1]
constexpr int DPP_ROW_ROR8 = 0x128;  // lane i <- lane i^8 of its row
constexpr int DPP_ROW_SHR1 = 0x111, DPP_ROW_SHR2 = 0x112, DPP_ROW_SHR4 = 0x114, DPP_ROW_SHR8 = 0x118;
constexpr int DPP_ROW_BCAST15 = 0x142, DPP_ROW_BCAST31 = 0x143;

template <int CTRL>
__device__ inline float dpp_f32(float v) {
    return __int_as_float(
        __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}

// Lanes without a valid source read 0 (bound_ctrl), masked-out rows keep 0.
template <int CTRL, int ROW_MASK>
__device__ inline int dpp_shift0(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, ROW_MASK, 0xF, true);
}

// Inclusive prefix sum over the 64 lanes of a wave (six DPP adds).
__device__ inline int wave_inclusive_scan(int v) {
    v += dpp_shift0<DPP_ROW_SHR1, 0xF>(v);
    v += dpp_shift0<DPP_ROW_SHR2, 0xF>(v);
    v += dpp_shift0<DPP_ROW_SHR4, 0xF>(v);
    v += dpp_shift0<DPP_ROW_SHR8, 0xF>(v);
    v += dpp_shift0<DPP_ROW_BCAST15, 0xA>(v);
    v += dpp_shift0<DPP_ROW_BCAST31, 0xC>(v);
    return v;
}

// Per-lane view of a chunk header and of where its eight packs sit in LDS.
struct LanePacks {
    uint32_t hlo, hhi;  // eight header bytes, pack j in byte j
    uint32_t plo, phi;  // byte j = w_0 + .. + w_j (inclusive prefix of the widths)
    int start;          // payload byte offset of pack 0

    __device__ inline void init(uint32_t lo, uint32_t hi) {
        hlo = lo;
        hhi = hi;
        uint32_t wl = (lo >> 4) & 0x0F0F0F0Fu, wh = (hi >> 4) & 0x0F0F0F0Fu;
        wl += wl << 8;
        wl += wl << 16;
        wh += wh << 8;
        wh += wh << 16;
        wh += (wl >> 24) * 0x01010101u;
        plo = wl;
        phi = wh;
        const int bytes = 2 * int(wh >> 24);
        start = wave_inclusive_scan(bytes) - bytes;
    }
    __device__ inline int width(int j) const { return ((j < 4 ? hlo : hhi) >> (8 * (j & 3) + 4)) & 15; }
    __device__ inline int min(int j) const { return ((j < 4 ? hlo : hhi) >> (8 * (j & 3))) & 15; }
    // payload byte offset of pack j
    __device__ inline int pos(int j) const {
        if (j == 0) return start;
        const int k = j - 1;
        return start + 2 * int(((k < 4 ? plo : phi) >> (8 * (k & 3))) & 0xFF);
    }
};

// Copy a chunk payload (payload_bytes, padded to 16) from global memory into
// this wave's LDS region with 16-byte lane accesses.
__device__ inline void stage_payload(const uint8_t *__restrict__ payload, int payload_bytes,
                                     uint8_t *lds, int lane) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        int off = (lane + 64 * k) * 16;
        if (off < payload_bytes)
            *reinterpret_cast<uint4 *>(lds + off) = *reinterpret_cast<const uint4 *>(payload + off);
    }
}

// LDS writes of this wave become visible to its own later LDS reads in program
// order; the fences only stop the compiler from moving accesses across.
__device__ inline void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Unpack the pack of width w at LDS byte `pos` into eight fp16-pair words:
// P[m] (m = 0..3) = tokens (m, m+8), P[4+m] = tokens (4+m, 12+m); each half is
// the bit pattern of fp16(code * 2^-24).
__device__ inline void unpack_pairs(const uint8_t *lds, int pos, int w, uint32_t (&P)[8]) {
    // aligned dword reads + funnel shifts: packs start on 2-byte boundaries and
    // misaligned LDS reads, although legal on gfx950, were measured several times slower
    const uint32_t *pp = reinterpret_cast<const uint32_t *>(lds + (pos & ~3));
    const uint32_t d0 = pp[0], d1 = pp[1], d2 = pp[2];
    const uint32_t sh = (pos & 2) * 8;
    const uint32_t A = __builtin_amdgcn_alignbit(d1, d0, sh);    // pack bits [0, 32): tokens 0..7
    const uint32_t hi_ = __builtin_amdgcn_alignbit(d2, d1, sh);  // pack bits [32, 64)
    const uint32_t R = w == 4 ? hi_ : __builtin_amdgcn_alignbit(hi_, A, 8 * w);  // bits [8w, 8w+32): tokens 8..15
    uint32_t M = __builtin_amdgcn_ubfe(0xFFFFFFFFu, 0, w);                       // (1 << w) - 1
    M |= M << 16;
    const uint32_t s = 4 * w;
    uint32_t Z0 = __builtin_amdgcn_perm(R, A, 0x05040100u);            // [A.lo16 | R.lo16]
    uint32_t Z1 = __builtin_amdgcn_perm(R >> s, A >> s, 0x05040100u);  // tokens 4..7 | 12..15
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        P[m] = Z0 & M;
        P[4 + m] = Z1 & M;
        if (m < 3) {
            Z0 = __builtin_amdgcn_alignbit(Z0, Z0, w);
            Z1 = __builtin_amdgcn_alignbit(Z1, Z1, w);
        }
    }
}

__device__ inline float half_lo(uint32_t p) { return float(__builtin_bit_cast(_Float16, uint16_t(p & 0xFFFFu))); }
__device__ inline float half_hi(uint32_t p) { return float(__builtin_bit_cast(_Float16, uint16_t(p >> 16))); }

// Reduce-scatter inside each row of 16 lanes: on entry every lane holds 16
// partial sums v[0..15]; on return lane i of the row holds the row's sum of v[i].
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
