// Decode-side pieces for chunks whose packs hold 8 tokens (the second pack size of the
// pack-size study, PackKV Sec. IV-B).
//
// Such a chunk has 1024 header bytes, indexed [token group of 8][channel], and packs of
// `width` bytes in the same order.  It is decoded as two halves of 32 tokens: half s covers
// token groups 4s..4s+3, its header bytes are the contiguous range [512s, 512s + 512) and its
// packs the contiguous payload range that follows the packs of half 0 -- so each half has
// exactly the shape the wave mapping of the 16-token packs is built for (512 packs, lane l
// owns token group l/16 of the half and channels 8(l%16)..+7, eight contiguous packs), and
// only the pack decode itself differs: 8 codes in at most 32 bits, two 16-bit fields.
#pragma once

#include "k_dot.h"
#include "unpack.h"
#include "v_chunk.h"

namespace packkv {

constexpr int CHUNK8_LDS = CHUNK8_MAX;
constexpr float V8_WEIGHT_MAX = 32752.0f;  // largest weight p_t * scale_t the fp16 hi/lo split of the V paths here carries
constexpr int DPP_ROW_HALF_MIRROR = 0x141;  // lane i <- lane 7 - i of its half row

// Per-lane view of the header of one half and of where its eight packs sit in LDS.
struct LanePacks8 {
    uint32_t hlo, hhi;  // eight header bytes, pack j in byte j
    uint32_t plo, phi;  // byte j = w_0 + .. + w_j: payload bytes up to and including pack j
    int start;          // LDS byte address of pack 0
    int end_all;        // LDS byte address behind the last pack of the half (wave-uniform)

    // lds_base: LDS byte address of the half's payload
    __device__ inline void init(uint32_t lo, uint32_t hi, int lds_base) {
        hlo = lo;
        hhi = hi;
        uint32_t wl = (lo >> 4) & 0x0F0F0F0Fu, wh = (hi >> 4) & 0x0F0F0F0Fu;  // width = bytes per pack
        wl = byte_prefix_sums(wl);
        wh = byte_prefix_sums(wh);
        const uint32_t tl = wl >> 24;
        wh += tl | (tl << 8) | (tl << 16) | (tl << 24);
        plo = wl;
        phi = wh;
        const int bytes = int(wh >> 24);
        const int inc = wave_inclusive_scan(bytes);
        start = inc - bytes + lds_base;
        end_all = __builtin_amdgcn_readlane(inc, 63) + lds_base;
    }
    __device__ inline uint32_t header_byte(int j) const { return ((j < 4 ? hlo : hhi) >> (8 * (j & 3))) & 0xFFu; }
    __device__ inline int pos(int j) const {
        if (j == 0) return start;
        const int k = j - 1;
        return start + int(((k < 4 ? plo : phi) >> (8 * (k & 3))) & 0xFFu);
    }
};

// The 32-bit window of a pack of 8 (its 8w <= 32 bits, from bit 0 up): two aligned dwords and
// a byte funnel shift; pos is byte aligned.
__device__ inline uint32_t fetch_window8(const uint8_t *lds0, int pos) {
    const uint32_t *pp = reinterpret_cast<const uint32_t *>(lds0 + (pos & ~3));
    return __builtin_amdgcn_alignbyte(pp[1], pp[0], uint32_t(pos));
}

// ---- K -------------------------------------------------------------------------------
template <int G>
struct KQuery8 {
    uint32_t qp[G][4];  // q of this lane's 8 channels as fp16 pairs, per head
    uint32_t qe[G][4];  // the same in the pairing pack_min_dot reads the header in
    float qsum[G];      // sum of all 128 q values per head

    // q_group: the G query heads of the kv-head, [G][128] fp16
    __device__ inline void load(const __half *q_group, int lane) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const uint4 raw = *reinterpret_cast<const uint4 *>(q_group + g * D + 8 * (lane & 15));
            qp[g][0] = raw.x, qp[g][1] = raw.y, qp[g][2] = raw.z, qp[g][3] = raw.w;
            qe[g][0] = __builtin_amdgcn_perm(qp[g][1], qp[g][0], 0x05040100u);
            qe[g][1] = __builtin_amdgcn_perm(qp[g][1], qp[g][0], 0x07060302u);
            qe[g][2] = __builtin_amdgcn_perm(qp[g][3], qp[g][2], 0x05040100u);
            qe[g][3] = __builtin_amdgcn_perm(qp[g][3], qp[g][2], 0x07060302u);
            float s = 0.0f;
#pragma unroll
            for (int k = 0; k < 4; ++k) s += half_lo(qp[g][k]) + half_hi(qp[g][k]);
            qsum[g] = row_all_reduce16(s);
        }
    }
};

// Token (0..7 of its group) whose sum lane i of a row holds after row_reduce_scatter8.
__device__ inline int k8_token_of_lane(int i) { return i >> 1; }

// Reduce-scatter inside each row of 16 lanes for eight sums per lane (v[t] belongs to token
// t): on return lanes 2t and 2t+1 of the row both hold the row's sum for token t.  The first
// two rounds use DPP adds whose write is restricted to half of the row (see
// row_reduce_scatter16, also for the wait states the leading s_nop stands for).
__device__ inline float row_reduce_scatter8(float (&v)[8], int lane) {
    float a[4], b[2];
    asm("s_nop 3\n\t"
        "v_add_f32_dpp %0, %4, %4 row_ror:8 row_mask:0xf bank_mask:0x3\n\t"
        "v_add_f32_dpp %1, %5, %5 row_ror:8 row_mask:0xf bank_mask:0x3\n\t"
        "v_add_f32_dpp %2, %6, %6 row_ror:8 row_mask:0xf bank_mask:0x3\n\t"
        "v_add_f32_dpp %3, %7, %7 row_ror:8 row_mask:0xf bank_mask:0x3\n\t"
        "v_add_f32_dpp %0, %8, %8 row_ror:8 row_mask:0xf bank_mask:0xc\n\t"
        "v_add_f32_dpp %1, %9, %9 row_ror:8 row_mask:0xf bank_mask:0xc\n\t"
        "v_add_f32_dpp %2, %10, %10 row_ror:8 row_mask:0xf bank_mask:0xc\n\t"
        "v_add_f32_dpp %3, %11, %11 row_ror:8 row_mask:0xf bank_mask:0xc"
        : "=&v"(a[0]), "=&v"(a[1]), "=&v"(a[2]), "=&v"(a[3])
        : "v"(v[0]), "v"(v[1]), "v"(v[2]), "v"(v[3]), "v"(v[4]), "v"(v[5]), "v"(v[6]), "v"(v[7]));
    asm("s_nop 1\n\t"
        "v_add_f32_dpp %0, %2, %2 row_ror:12 row_mask:0xf bank_mask:0x5\n\t"
        "v_add_f32_dpp %1, %3, %3 row_ror:12 row_mask:0xf bank_mask:0x5\n\t"
        "v_add_f32_dpp %0, %4, %4 row_ror:4 row_mask:0xf bank_mask:0xa\n\t"
        "v_add_f32_dpp %1, %5, %5 row_ror:4 row_mask:0xf bank_mask:0xa"
        : "=&v"(b[0]), "=&v"(b[1])
        : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]));
    const bool b1 = lane & 2;
    const float keep = b1 ? b[1] : b[0];
    const float send = b1 ? b[0] : b[1];
    float c = keep + dpp_f32<DPP_QUAD_XOR2>(send);
    c += dpp_f32<DPP_QUAD_XOR1>(c);
    return c;
}

// One half (32 tokens) of a chunk: u[g] = sum_d q[g][d] (code[t, d] + m[group, d]) for token
// t = 8 * (lane / 16) + k8_token_of_lane(lane % 16) of the half, head g.  `table`: the pair
// table (build_pair_table).  Two packs (channels 2jp, 2jp+1) are unpacked side by side and
// contracted with two-element fp16 dot products, as in the single-head path of the 16-token
// packs; with G heads the unpacked words are reused G times.
template <int G>
__device__ inline void k8_half(const uint8_t *lds0, const uint2 *table, const LanePacks8 &lp,
                               const KQuery8<G> &kq, int lane, float (&u)[G]) {
    // every accumulator starts from the lane's pack-minimum term (see k_chunk_fma)
    float acc[G][8], ms[G];
#pragma unroll
    for (int g = 0; g < G; ++g) ms[g] = pack_min_dot(lp.hlo, lp.hhi, kq.qe[g]);
#pragma unroll
    for (int jp = 0; jp < 4; ++jp) {
        const uint32_t Aa = fetch_window8(lds0, lp.pos(2 * jp));
        const uint32_t Ab = fetch_window8(lds0, lp.pos(2 * jp + 1));
        const uint2 ka = table[lp.header_byte(2 * jp)], kb = table[lp.header_byte(2 * jp + 1)];
        // fields of four codes: tokens 0..3 from bit 0, tokens 4..7 from bit 4w (clean)
        const uint32_t Fa[2] = {Aa, __builtin_amdgcn_ubfe(Aa, ka.x, ka.x)};
        const uint32_t Fb[2] = {Ab, __builtin_amdgcn_ubfe(Ab, kb.x, kb.x)};
        const u16x2 widths = __builtin_bit_cast(u16x2, __builtin_amdgcn_perm(kb.x, ka.x, 0x0c050c01u));
        const uint32_t masks = __builtin_amdgcn_perm(kb.x, ka.x, 0x07060302u);
#pragma unroll
        for (int f = 0; f < 2; ++f) {
            u16x2 Z = __builtin_bit_cast(u16x2, __builtin_amdgcn_perm(Fb[f], Fa[f], 0x05040100u));
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                const uint32_t P = __builtin_bit_cast(uint32_t, Z) & (f == 1 && m == 3 ? ~0u : masks);
#pragma unroll
                for (int g = 0; g < G; ++g)
                    acc[g][4 * f + m] = dot2_f16(P, kq.qp[g][jp], jp == 0 ? ms[g] : acc[g][4 * f + m]);
                if (m < 3) Z = Z >> widths;
            }
        }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) u[g] = row_reduce_scatter8(acc[g], lane) * CODE_SCALE;
}

// ---- V -------------------------------------------------------------------------------
// Where token t (0..63) of a block sits in the B operand staging (column 0): half s = t / 32
// takes the place of the `half` index of the 16-token layout, k-run t / 8 % 4, and inside the
// run the order in which v8_half leaves the codes: words of tokens (m, m + 4).
template <int G>
__device__ inline int v8_bslot(int t) {
    const int s = t >> 5, kg = (t >> 3) & 3, uu = t & 7;
    const int e = uu < 4 ? 2 * uu : 2 * (uu - 4) + 1;
    return (((kg * 2 + s) * BLds<G>::COLS) * 8 + e) * 2;
}

// Sum over the aligned groups of eight lanes, result in every lane of the group.
__device__ inline float lanes8_all_reduce(float v) {
    v += dpp_f32<DPP_QUAD_XOR1>(v);
    v += dpp_f32<DPP_QUAD_XOR2>(v);
    v += dpp_f32<DPP_ROW_HALF_MIRROR>(v);
    return v;
}

// Token of the block that lane `lane` holds after the two K halves (k8_half, second half in the
// odd lanes): 32 (i & 1) + 8 (lane / 16) + (i >> 1), i = lane % 16.
__device__ inline int k8_token_of_block_lane(int lane) {
    const int i = lane & 15;
    return 32 * (i & 1) + 8 * (lane >> 4) + k8_token_of_lane(i);
}

// Adds one chunk (both halves) from the LDS buffer at byte offset `cur`.  The lane is token
// `lane` of the block (K8_ORDER false: the three-step path), or token
// k8_token_of_block_lane(lane) (K8_ORDER true: the fused attention, where the K phase leaves
// the scores in that order); pt[g]: its weight for head g, mt: its token metadata.  `table`:
// build_pack_table with lift CODE_LIFT and fold = fold_min<G>().  vl.bslot must be
// v8_bslot of the lane's token.
template <int G, bool K8_ORDER = false>
__device__ inline void v8_chunk(const uint8_t *lds_all, int cur, const uint4 *table, const VLane<G> &vl,
                                uint32_t mt, const float (&pt)[G], VState<G> &st) {
    const int lane = threadIdx.x & 63;
    const float scale = __half2float(__ushort_as_half(uint16_t(mt & 0xFFFFu)));
    const float mn = __half2float(__ushort_as_half(uint16_t(mt >> 16)));
    float wsum[2][G];  // per half: sum of the weights of this lane's token group (8 tokens)
#pragma unroll
    for (int g = 0; g < G; ++g) {
        // the fp16 split holds weights below 2^15 (hi rounds toward zero, the residual times 2^11 stays
        // finite); a larger product -- a token range in the thousands times a weight near 2^8 -- is
        // clamped there instead of turning into infinities
        const float w = fminf(pt[g] * scale, V8_WEIGHT_MAX);
        st.pm[g] = fmaf(pt[g], mn, st.pm[g]);
        const _Float16 hi = __builtin_bit_cast(
            _Float16, uint16_t(__builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(w, 0.0f)) & 0xFFFFu));
        const float lo = (w - float(hi)) * 2048.0f;
        const _Float16 lo16 = _Float16(lo);  // to nearest: the residual's rounding error has no sign bias
        *reinterpret_cast<_Float16 *>(vl.blds + vl.bslot + (2 * g) * 16) = hi;
        *reinterpret_cast<_Float16 *>(vl.blds + vl.bslot + (2 * g + 1) * 16) = lo16;
        if (!fold_min<G>()) {
            if constexpr (K8_ORDER) {
                // the eight tokens of group (half s, row) sit in the lanes of this row with i & 1 = s
                float v = w + dpp_f32<DPP_ROW_ROR8>(w);
                v += dpp_f32<DPP_ROW_ROR4>(v);
                v += dpp_f32<DPP_QUAD_XOR2>(v);
                const float other = dpp_f32<DPP_QUAD_XOR1>(v);
                wsum[0][g] = (lane & 1) ? other : v;
                wsum[1][g] = (lane & 1) ? v : other;
            } else {
                const float w8 = lanes8_all_reduce(w);  // tokens 8k..8k+7 live in lanes 8k..8k+7
                wsum[0][g] = __shfl(w8, 8 * (lane >> 4));
                wsum[1][g] = __shfl(w8, 32 + 8 * (lane >> 4));
            }
        }
    }
    wave_lds_fence();
    const vhalf8 b0 = *reinterpret_cast<const vhalf8 *>(vl.blds + vl.bread0);
    const vhalf8 b1 = *reinterpret_cast<const vhalf8 *>(vl.blds + vl.bread1);

    int payload = cur + HEADER8;
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const uint2 hdr = *reinterpret_cast<const uint2 *>(lds_all + cur + 512 * s + lane * 8);
        LanePacks8 lp;
        lp.init(hdr.x, hdr.y, payload);
        payload = lp.end_all;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t A = fetch_window8(lds_all, lp.pos(j));
            const uint4 k = table[lp.header_byte(j)];
            const uint32_t w = k.y, M = k.x;
            // tokens 0..3 in the low half, tokens 4..7 in the high half, lifted together
            uint32_t Z = __builtin_amdgcn_perm(shr_by_byte1(A, k.y), A, 0x05040100u);  // byte 1 of the field: 4w
            Z = __builtin_amdgcn_alignbit(Z, Z, 32 - CODE_LIFT);
            uint32_t P[4];
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                P[m] = (Z & M) + (fold_min<G>() ? k.w : 0u);
                if (m < 3) Z = __builtin_amdgcn_alignbit(Z, Z, w);
            }
            if constexpr (!fold_min<G>()) {
                const float m = __uint_as_float(k.w);
#pragma unroll
                for (int g = 0; g < G; ++g) st.macc[g][j] = fmaf(m, wsum[s][g], st.macc[g][j]);
            }
            typedef uint32_t u32x4v __attribute__((ext_vector_type(4)));
            const vhalf8 a = __builtin_bit_cast(vhalf8, u32x4v{P[0], P[1], P[2], P[3]});
            st.acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, s ? b1 : b0, st.acc[j], 0, 0, 0);
        }
    }
    wave_lds_fence();  // the B operand is rewritten by the next chunk
}

// ---- wide chunks -----------------------------------------------------------------------
// Codes above 15 (relative scales below 1/15): packs of 8 tokens with widths up to 8 bits; the
// header is 1024 width bytes followed by 1024 minimum bytes, both indexed [token group][channel].
// Decoded as two halves of 32 tokens like the narrow 8-token packs; a pack is at most 64 bits
// (three aligned dwords), a 16-bit field holds two codes.  Codes up to 255 are still fp16
// subnormals (code * 2^-24), so the K dot products stay exact.  The V path cannot lift them far
// enough inside the subnormal range for the matrix cores (255 << 2 is the limit, and with two
// bits the measured output error at 32 Ki tokens and 255 levels was 6e-3): it turns every
// pair into the normal numbers `code` instead, exactly: OR in the bit pattern of 1024.0, then
// subtract 1024.0 in packed fp16 -- two instructions per word.
constexpr int CHUNKW_LDS = CHUNKW_MAX;
constexpr int WIDE_TABLE_ENTRIES = 9;   // widths 0..8
typedef _Float16 vhalf2 __attribute__((ext_vector_type(2)));

// K form: x = 2w in bits 0..4 (bit-field offset/width), w in byte 1, the w-bit mask in the high
// half; y = 4w (64-bit shift amount).  V form: x = mask in both halves, y = w, z = 4w, w = 2w.
__device__ inline void build_wide_tables(uint2 *ktable, uint4 *vtable) {
    const uint32_t w = threadIdx.x;
    if (w < WIDE_TABLE_ENTRIES) {
        const uint32_t m1 = (1u << w) - 1u;
        if (ktable) ktable[w] = make_uint2((2 * w) | (w << 8) | (m1 << 16), 4 * w);
        if (vtable) vtable[w] = make_uint4(m1 * 0x10001u, w, 4 * w, 2 * w);
    }
    __syncthreads();
}

// Per-lane view of one half: eight width bytes, eight minimum bytes, pack positions.
struct LanePacksW {
    uint32_t wlo, whi;  // widths, pack j in byte j
    uint32_t mlo, mhi;  // minimums
    uint32_t plo, phi;  // byte j = w_0 + .. + w_j
    int start, end_all;

    __device__ inline void init(uint2 widths, uint2 mins, int lds_base) {
        wlo = widths.x, whi = widths.y, mlo = mins.x, mhi = mins.y;
        uint32_t wl = byte_prefix_sums(wlo), wh = byte_prefix_sums(whi);
        const uint32_t tl = wl >> 24;
        wh += tl | (tl << 8) | (tl << 16) | (tl << 24);
        plo = wl;
        phi = wh;
        const int bytes = int(wh >> 24);
        const int inc = wave_inclusive_scan(bytes);
        start = inc - bytes + lds_base;
        end_all = __builtin_amdgcn_readlane(inc, 63) + lds_base;
    }
    __device__ inline uint32_t width(int j) const { return ((j < 4 ? wlo : whi) >> (8 * (j & 3))) & 0xFFu; }
    __device__ inline uint32_t minimum(int j) const { return ((j < 4 ? mlo : mhi) >> (8 * (j & 3))) & 0xFFu; }
    __device__ inline int pos(int j) const {
        if (j == 0) return start;
        const int k = j - 1;
        return start + int(((k < 4 ? plo : phi) >> (8 * (k & 3))) & 0xFFu);
    }
};

// The 64-bit window of a wide pack: low dword and the dword that starts 4w bits in.
__device__ inline void fetch_window_wide(const uint8_t *lds0, int pos, uint32_t shift4w, uint32_t &A, uint32_t &R) {
    const uint32_t *pp = reinterpret_cast<const uint32_t *>(lds0 + (pos & ~3));
    const uint32_t d0 = pp[0], d1 = pp[1], d2 = pp[2];
    A = __builtin_amdgcn_alignbyte(d1, d0, uint32_t(pos));
    const uint32_t hi = __builtin_amdgcn_alignbyte(d2, d1, uint32_t(pos));
    R = uint32_t(((uint64_t(hi) << 32) | A) >> (shift4w & 63u));
}

// Pack-minimum term from eight minimum bytes (see pack_min_dot): bytes, not nibbles.
__device__ inline float pack_min_dot_bytes(uint32_t mlo, uint32_t mhi, const uint32_t (&qe)[4]) {
    float ms = dot2_f16(mlo & 0x00FF00FFu, qe[0], 0.0f);
    ms = dot2_f16((mlo >> 8) & 0x00FF00FFu, qe[1], ms);
    ms = dot2_f16(mhi & 0x00FF00FFu, qe[2], ms);
    ms = dot2_f16((mhi >> 8) & 0x00FF00FFu, qe[3], ms);
    return ms;
}

// K, one half of a wide chunk; same result layout as k8_half.  ktable: build_wide_tables.
template <int G>
__device__ inline void kw_half(const uint8_t *lds0, const uint2 *ktable, const LanePacksW &lp,
                               const KQuery8<G> &kq, int lane, float (&u)[G]) {
    float acc[G][8], ms[G];
#pragma unroll
    for (int g = 0; g < G; ++g) ms[g] = pack_min_dot_bytes(lp.mlo, lp.mhi, kq.qe[g]);
#pragma unroll
    for (int jp = 0; jp < 4; ++jp) {
        const uint2 ka = ktable[lp.width(2 * jp)], kb = ktable[lp.width(2 * jp + 1)];
        uint32_t Aa, Ra, Ab, Rb;
        fetch_window_wide(lds0, lp.pos(2 * jp), ka.y, Aa, Ra);
        fetch_window_wide(lds0, lp.pos(2 * jp + 1), kb.y, Ab, Rb);
        // fields of two codes: tokens (0,1) (2,3) (4,5) (6,7); the odd fields are clean
        const uint32_t Fa[4] = {Aa, __builtin_amdgcn_ubfe(Aa, ka.x, ka.x), Ra, __builtin_amdgcn_ubfe(Ra, ka.x, ka.x)};
        const uint32_t Fb[4] = {Ab, __builtin_amdgcn_ubfe(Ab, kb.x, kb.x), Rb, __builtin_amdgcn_ubfe(Rb, kb.x, kb.x)};
        const u16x2 widths = __builtin_bit_cast(u16x2, __builtin_amdgcn_perm(kb.x, ka.x, 0x0c050c01u));
        const uint32_t masks = __builtin_amdgcn_perm(kb.x, ka.x, 0x07060302u);
#pragma unroll
        for (int f = 0; f < 4; ++f) {
            u16x2 Z = __builtin_bit_cast(u16x2, __builtin_amdgcn_perm(Fb[f], Fa[f], 0x05040100u));
#pragma unroll
            for (int m = 0; m < 2; ++m) {
                const uint32_t P = __builtin_bit_cast(uint32_t, Z) & ((f & 1) && m == 1 ? ~0u : masks);
#pragma unroll
                for (int g = 0; g < G; ++g)
                    acc[g][2 * f + m] = dot2_f16(P, kq.qp[g][jp], jp == 0 ? ms[g] : acc[g][2 * f + m]);
                if (m < 1) Z = Z >> widths;
            }
        }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) u[g] = row_reduce_scatter8(acc[g], lane) * CODE_SCALE;
}

// V, one wide chunk (both halves); the lane's token as in v8_chunk (K8_ORDER).  vtable:
// build_wide_tables.  The A operand holds the codes as numbers: accumulators in units of 1.
template <int G, bool K8_ORDER = false>
__device__ inline void vw_chunk(const uint8_t *lds_all, int cur, const uint4 *vtable, const VLane<G> &vl,
                                uint32_t mt, const float (&pt)[G], VState<G> &st) {
    const int lane = threadIdx.x & 63;
    const float scale = __half2float(__ushort_as_half(uint16_t(mt & 0xFFFFu)));
    const float mn = __half2float(__ushort_as_half(uint16_t(mt >> 16)));
    float wsum[2][G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        // the fp16 split holds weights below 2^15 (hi rounds toward zero, the residual times 2^11 stays
        // finite); a larger product -- a token range in the thousands times a weight near 2^8 -- is
        // clamped there instead of turning into infinities
        const float w = fminf(pt[g] * scale, V8_WEIGHT_MAX);
        st.pm[g] = fmaf(pt[g], mn, st.pm[g]);
        const _Float16 hi = __builtin_bit_cast(
            _Float16, uint16_t(__builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(w, 0.0f)) & 0xFFFFu));
        const float lo = (w - float(hi)) * 2048.0f;
        const _Float16 lo16 = _Float16(lo);  // to nearest: the residual's rounding error has no sign bias
        *reinterpret_cast<_Float16 *>(vl.blds + vl.bslot + (2 * g) * 16) = hi;
        *reinterpret_cast<_Float16 *>(vl.blds + vl.bslot + (2 * g + 1) * 16) = lo16;
        if (!fold_min<G>()) {
            if constexpr (K8_ORDER) {
                // the eight tokens of group (half s, row) sit in the lanes of this row with i & 1 = s
                float v = w + dpp_f32<DPP_ROW_ROR8>(w);
                v += dpp_f32<DPP_ROW_ROR4>(v);
                v += dpp_f32<DPP_QUAD_XOR2>(v);
                const float other = dpp_f32<DPP_QUAD_XOR1>(v);
                wsum[0][g] = (lane & 1) ? other : v;
                wsum[1][g] = (lane & 1) ? v : other;
            } else {
                const float w8 = lanes8_all_reduce(w);
                wsum[0][g] = __shfl(w8, 8 * (lane >> 4));
                wsum[1][g] = __shfl(w8, 32 + 8 * (lane >> 4));
            }
        }
    }
    wave_lds_fence();
    const vhalf8 b0 = *reinterpret_cast<const vhalf8 *>(vl.blds + vl.bread0);
    const vhalf8 b1 = *reinterpret_cast<const vhalf8 *>(vl.blds + vl.bread1);

    int payload = cur + HEADERW;
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const uint2 wb = *reinterpret_cast<const uint2 *>(lds_all + cur + 512 * s + lane * 8);
        const uint2 mb = *reinterpret_cast<const uint2 *>(lds_all + cur + 1024 + 512 * s + lane * 8);
        LanePacksW lp;
        lp.init(wb, mb, payload);
        payload = lp.end_all;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint4 k = vtable[lp.width(j)];
            uint32_t A, R;
            fetch_window_wide(lds_all, lp.pos(j), k.z, A, R);
            const uint32_t w = k.y, M = k.x, s2 = k.w;
            const uint32_t mj = lp.minimum(j);
            const uint32_t fold = fold_min<G>() ? mj * 0x10001u : 0u;   // code + minimum < 256
            // tokens (0,1 | 4,5) and (2,3 | 6,7): low half | high half
            const uint32_t Z0 = __builtin_amdgcn_perm(R, A, 0x05040100u);
            const uint32_t Z1 = __builtin_amdgcn_perm(R >> s2, A >> s2, 0x05040100u);
            const uint32_t raw[4] = {Z0, __builtin_amdgcn_alignbit(Z0, Z0, w), Z1, __builtin_amdgcn_alignbit(Z1, Z1, w)};
            uint32_t P[4];   // tokens (0,4) (1,5) (2,6) (3,7) as fp16 numbers
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                const uint32_t biased = ((raw[m] & M) | 0x64006400u) + fold;   // 1024 + code (+ minimum), exact
                P[m] = __builtin_bit_cast(uint32_t, __builtin_bit_cast(vhalf2, biased) - vhalf2{1024.0f16, 1024.0f16});
            }
            if constexpr (!fold_min<G>()) {
                const float m = float(mj);
#pragma unroll
                for (int g = 0; g < G; ++g) st.macc[g][j] = fmaf(m, wsum[s][g], st.macc[g][j]);
            }
            typedef uint32_t u32x4v __attribute__((ext_vector_type(4)));
            const vhalf8 a = __builtin_bit_cast(vhalf8, u32x4v{P[0], P[1], P[2], P[3]});
            st.acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, s ? b1 : b0, st.acc[j], 0, 0, 0);
        }
    }
    wave_lds_fence();
}

}  // namespace packkv
