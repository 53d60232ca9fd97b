// Per-chunk K work shared by the K kernel and the fused decode-attention kernel
// (PackKV Sec. III-C.1): q . code sums of the 64 tokens of one chunk that sits in
// an LDS buffer, for the G query heads of its kv-head.  De-quantization is folded
// by the callers:
//   score_t = sm_scale * (scale_t * (sum_d q_d code[t,d] + sum_d q_d m[g,d]) + min_t * sum_d q_d)
//
// Two forms.  With one query head per kv-head, two-element fp16 dot products read
// unpacked channel pairs directly and a reduce-scatter inside the 16-lane row
// leaves token 16g+i in lane 16g+i.  With grouped queries the tile is turned on
// the matrix cores so that one unpack serves all G heads:
//   C1[channel i][column n] = sum_k A1[i][k] S_x[k][n]         (16x16x32 fp16 MFMA)
//     A1: the unpacked words of pack slot j (row i = lane%16 = channel 8i+j, the
//         32 k-slots = 8 tokens of each token group lane/16), S_x: selects the
//         16 k-slots with bit 1 of the in-lane slot equal to x, times 2^10
//   C2[head][column n] += sum_k Q[head][k] cvt16(C1)[k][n]      (16x16x32 fp16 MFMA)
//     the fp32 tile C1 of lane (r, n) holds channels 4r..4r+3 of column n, which is
//     exactly the k-run a B operand lane needs; two pack slots fill its 8 k-values.
// Every value in C1 is an integer code times 2^-14, so its fp16 conversion is
// exact.  With the k-slot -> column assignment below, lane n (< 16) ends up with
// four consecutive tokens of the block, 16*(n>>2) + 4*((n>>1)&1) + 8*(n&1) + {0..3},
// in the four accumulators, for the heads 4*(lane/16)..+3 in their four registers.
#pragma once

#include "unpack.h"

namespace packkv {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float float4_u __attribute__((ext_vector_type(4), aligned(4)));

// ---- one query head per kv-head ------------------------------------------------
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

struct KQueryFma {
    uint32_t qp[4];  // q of this lane's 8 channels as fp16 pairs (channels 2k, 2k+1 in word k)
    uint32_t qe[4];  // the same paired as (0,2) (1,3) (4,6) (5,7): the order pack_min_dot reads the header in
    float qsum;      // sum of all 128 q values

    // q_head: the 128 fp16 values of the query head
    __device__ inline void load(const __half *q_head, int lane) {
        const uint4 raw = *reinterpret_cast<const uint4 *>(q_head + 8 * (lane & 15));
        qp[0] = raw.x, qp[1] = raw.y, qp[2] = raw.z, qp[3] = raw.w;
        qe[0] = __builtin_amdgcn_perm(qp[1], qp[0], 0x05040100u);
        qe[1] = __builtin_amdgcn_perm(qp[1], qp[0], 0x07060302u);
        qe[2] = __builtin_amdgcn_perm(qp[3], qp[2], 0x05040100u);
        qe[3] = __builtin_amdgcn_perm(qp[3], qp[2], 0x07060302u);
        float s = 0.0f;
#pragma unroll
        for (int k = 0; k < 4; ++k) s += half_lo(qp[k]) + half_hi(qp[k]);
        qsum = row_all_reduce16(s);
    }
};

// d = a.lo * b.lo + a.hi * b.hi + c with a, b pairs of fp16 and fp32 accumulation: the
// three-address dot-product instruction, from inline assembly.  The compiler's own choice is the
// two-address form, which costs a register copy for every accumulator that starts from a live
// value.  Dot-product results need three wait states before an instruction of another kind reads
// or overwrites them, which the compiler does not track into inline assembly: every dot product
// of the K paths goes through this one function, so that their results are only ever consumed as
// the addend of the same instruction (no wait states needed) or by the reduce-scatter, whose
// assembly starts with the wait states.
__device__ inline float dot2_f16(uint32_t a, uint32_t b, float c) {
    float d;
    asm("v_dot2_f32_f16 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
    return d;
}

// Pack-minimum term of a lane: sum_j q_j m_j * 2^-24 over its eight packs, straight from the
// eight header bytes (minimum = low nibble): two nibbles at a time are, as they stand, a pair
// of fp16 subnormals m * 2^-24, the scale the unpacked codes have too.  qe: KQueryFma::qe order.
__device__ inline float pack_min_dot(uint32_t hlo, uint32_t hhi, const uint32_t (&qe)[4]) {
    float ms = dot2_f16(hlo & 0x000F000Fu, qe[0], 0.0f);
    ms = dot2_f16((hlo >> 8) & 0x000F000Fu, qe[1], ms);
    ms = dot2_f16(hhi & 0x000F000Fu, qe[2], ms);
    ms = dot2_f16((hhi >> 8) & 0x000F000Fu, qe[3], ms);
    return ms;
}

// The four 16-bit fields of a pack, each in the low half of a word (the high half is
// don't-care): F[f] holds the codes of tokens 4f..4f+3, w bits each, from bit 0 up.  The odd
// fields come out of a bit-field extract with nothing above their 4w bits.
__device__ inline void pack_fields(const PackRawPair &r, uint32_t (&F)[4]) {
    const uint32_t A = __builtin_amdgcn_alignbyte(r.d1, r.d0, r.sh);   // pack bits [0, 32)
    const uint32_t hi_ = __builtin_amdgcn_alignbyte(r.d2, r.d1, r.sh); // pack bits [32, 64)
    const uint32_t R = uint32_t(((uint64_t(hi_) << 32) | A) >> (r.k.y & 63u));  // bits [8w, 8w+32)
    const uint32_t s = r.k.x;  // low five bits, all the extract reads: 4w
    F[0] = A, F[1] = __builtin_amdgcn_ubfe(A, s, s), F[2] = R, F[3] = __builtin_amdgcn_ubfe(R, s, s);
}

// Returns, in lane l, sum_d q_d (code[l, d] + m[l / 16, d]) for token l of the chunk whose
// header has been parsed into `lp`; `table`: the pair table.
//
// Two packs (channels 2jp, 2jp+1 of the lane) are unpacked side by side, one in each
// 16-bit half of a word: a packed 16-bit shift moves each half by its own pack's width, so
// every unpacked word is the pair (channel 2jp, channel 2jp+1) of one token, which a
// two-element fp16 dot product with fp32 accumulation contracts against the matching q pair
// in one instruction.  The codes stay fp16 subnormal bit patterns (code * 2^-24); the
// products are exact.
__device__ inline float k_chunk_fma(const uint8_t *lds0, const uint2 *table, const LanePacks &lp,
                                    const KQueryFma &kq, int lane) {
    // every accumulator starts from the lane's pack-minimum term (the row reduction then adds the
    // sixteen lanes' terms up): no accumulator to clear, no separate reduction for that term
    const float ms = pack_min_dot(lp.hlo, lp.hhi, kq.qe);
    float acc[16];
#pragma unroll
    for (int jp = 0; jp < 4; ++jp) {
        const PackRawPair ra = fetch_pack_pair(lds0, table, lp.pos(2 * jp), lp.header_byte(2 * jp));
        const PackRawPair rb = fetch_pack_pair(lds0, table, lp.pos(2 * jp + 1), lp.header_byte(2 * jp + 1));
        uint32_t Fa[4], Fb[4];
        pack_fields(ra, Fa);
        pack_fields(rb, Fb);
        const u16x2 widths = __builtin_bit_cast(u16x2, __builtin_amdgcn_perm(rb.k.x, ra.k.x, 0x0c050c01u));
        const uint32_t masks = __builtin_amdgcn_perm(rb.k.x, ra.k.x, 0x07060302u);
#pragma unroll
        for (int f = 0; f < 4; ++f) {
            u16x2 Z = __builtin_bit_cast(u16x2, __builtin_amdgcn_perm(Fb[f], Fa[f], 0x05040100u));
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                // token 4f+m, both channels; the last code of a clean field needs no mask
                const uint32_t P = __builtin_bit_cast(uint32_t, Z) & ((f & 1) && m == 3 ? ~0u : masks);
                acc[4 * f + m] = dot2_f16(P, kq.qp[jp], jp == 0 ? ms : acc[4 * f + m]);
                if (m < 3) Z = Z >> widths;
            }
        }
    }
    return row_reduce_scatter16(acc, lane) * CODE_SCALE;
}

// ---- grouped queries -------------------------------------------------------------
constexpr float K_MFMA_OUT_SCALE = 16384.0f;  // codes enter as code * 2^-24, the selection adds 2^10

// Token offset inside a block of the first of the four consecutive tokens that lane%16 = n
// holds after k_chunk_mfma.
__device__ inline int k_mfma_token_base(int n) { return 16 * (n >> 2) + 4 * ((n >> 1) & 1) + 8 * (n & 1); }

template <int G, bool FOLD = fold_min<G>()>
struct KQueryMfma {
    uint32_t qh[FOLD ? 1 : G][4];  // q of this lane's 8 channels as fp16 pairs (pack-minimum term)
    float qsum[G];      // sum of all 128 q values per head
    half8 qA[4];        // Q operand per pair of pack slots
    half8 sel[2];       // selection operands S_0, S_1

    // q_group: the G query heads of the kv-head, [G][128] fp16
    __device__ inline void load(const __half *q_group, int lane) {
        const int row = lane >> 4, col = lane & 15;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const uint4 raw = *reinterpret_cast<const uint4 *>(q_group + g * D + 8 * col);
            const uint32_t rq[4] = {raw.x, raw.y, raw.z, raw.w};
            float s = 0.0f;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                if (!FOLD) qh[g][k] = rq[k];
                s += half_lo(rq[k]) + half_hi(rq[k]);
            }
            qsum[g] = row_all_reduce16(s);
        }
        // row = head lane%16, k-value e of k-run lane/16 = channel 8*(4*(lane/16) + (e&3)) + 2jp + (e>>2)
        uint32_t rw[4][4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            uint4 raw = make_uint4(0, 0, 0, 0);
            if (col < G) raw = *reinterpret_cast<const uint4 *>(q_group + col * D + 8 * (4 * row + e));
            rw[e][0] = raw.x, rw[e][1] = raw.y, rw[e][2] = raw.z, rw[e][3] = raw.w;
        }
#pragma unroll
        for (int jp = 0; jp < 4; ++jp) {
            const uint32_t w0 = __builtin_amdgcn_perm(rw[1][jp], rw[0][jp], 0x05040100u);
            const uint32_t w1 = __builtin_amdgcn_perm(rw[3][jp], rw[2][jp], 0x05040100u);
            const uint32_t w2 = __builtin_amdgcn_perm(rw[1][jp], rw[0][jp], 0x07060302u);
            const uint32_t w3 = __builtin_amdgcn_perm(rw[3][jp], rw[2][jp], 0x07060302u);
            qA[jp] = __builtin_bit_cast(half8, u32x4{w0, w1, w2, w3});
        }
        // lane (k-run kg = lane/16, column n = lane%16) holds S_x[8kg+e][n]; slot e of run kg
        // goes to column 4kg + 2(e>>2) + (e&1) when ((e>>1)&1) == x
#pragma unroll
        for (int x = 0; x < 2; ++x) {
            uint32_t wsel[4] = {0, 0, 0, 0};
            const int e = ((col >> 1) & 1) * 4 + x * 2 + (col & 1);
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if ((col >> 2) == row && (e >> 1) == k) wsel[k] = 0x6400u << (16 * (e & 1));  // fp16 1024
            sel[x] = __builtin_bit_cast(half8, u32x4{wsel[0], wsel[1], wsel[2], wsel[3]});
        }
    }
};

// acc[t][x] (lane (r, n)): sum_d q[head 4r+x][d] code[token, d] / K_MFMA_OUT_SCALE for token
// k_mfma_token_base(n) + t; ms_row[g] (every lane of row r): sum_d q[g][d] m[group r, d], or 0
// when the minimum is folded into the codes (FOLD, table built with fold).
template <int G, bool FOLD = fold_min<G>()>
__device__ inline void k_chunk_mfma(const uint8_t *lds0, const uint4 *table, const LanePacks &lp,
                                    const KQueryMfma<G, FOLD> &kq, float4_t (&acc)[4], float (&ms_row)[G]) {
    const float4_t zero = float4_t{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[t] = zero;
    float msum[G];
#pragma unroll
    for (int g = 0; g < G; ++g) msum[g] = 0.0f;
#pragma unroll
    for (int jp = 0; jp < 4; ++jp) {
        uint32_t P[2][8];
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            const int j = 2 * jp + jj;
            const PackRaw raw = fetch_pack(lds0, table, lp.pos(j), lp.header_byte(j));
            expand_pack<0, FOLD>(raw, P[jj]);
            if constexpr (!FOLD) {
                const float m = __uint_as_float(raw.k.w);
#pragma unroll
                for (int g = 0; g < G; ++g)
                    msum[g] = fmaf(jj ? half_hi(kq.qh[g][jp]) : half_lo(kq.qh[g][jp]), m, msum[g]);
            }
        }
        // P[jj][t + 2i]: tokens (t + 2i, t + 2i + 8) of pack slot 2jp+jj; column token offset
        // t = parity + 2x
        const half8 a00 = __builtin_bit_cast(half8, u32x4{P[0][0], P[0][2], P[0][4], P[0][6]});
        const half8 a01 = __builtin_bit_cast(half8, u32x4{P[0][1], P[0][3], P[0][5], P[0][7]});
        const half8 a10 = __builtin_bit_cast(half8, u32x4{P[1][0], P[1][2], P[1][4], P[1][6]});
        const half8 a11 = __builtin_bit_cast(half8, u32x4{P[1][1], P[1][3], P[1][5], P[1][7]});
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const float4_t ca = __builtin_amdgcn_mfma_f32_16x16x32_f16((t & 1) ? a01 : a00, kq.sel[t >> 1], zero, 0, 0, 0);
            const float4_t cb = __builtin_amdgcn_mfma_f32_16x16x32_f16((t & 1) ? a11 : a10, kq.sel[t >> 1], zero, 0, 0, 0);
            const u32x4 bw = {__builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(ca[0], ca[1])),
                              __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(ca[2], ca[3])),
                              __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(cb[0], cb[1])),
                              __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(cb[2], cb[3]))};
            acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(kq.qA[jp], __builtin_bit_cast(half8, bw),
                                                             acc[t], 0, 0, 0);
        }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) ms_row[g] = FOLD ? 0.0f : row_all_reduce16(msum[g]);
}

}  // namespace packkv
