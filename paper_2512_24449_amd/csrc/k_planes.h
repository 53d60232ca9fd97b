// Per-chunk K work for chunks in the plane layout (packs of 16 tokens, channel-major pack list),
// shared by the K kernel and the fused decode-attention kernel (PackKV Sec. III-C.1): the sums
//   u[head][t] = sum_d q[head][d] * (code[t, d] + m[group(t), d])
// of the 64 tokens of one chunk that sits in an LDS buffer, for the G <= 4 query heads of its
// kv-head.  De-quantization is folded by the callers:
//   score_t = sm_scale * (scale_t * u[head][t] + min_t * sum_d q[head][d])
//
// The contraction runs over channels, while a plane word holds 16 tokens of ONE channel, so the
// planes are turned once per chunk: every lane copies the words of its eight packs (two channels
// x four token groups) to fixed places of two LDS tiles [channel][group] -- tile L with the low
// two bits of every code, tile H with the high two bits; the one-bit plane T of an odd width is
// widened to two-bit fields on the way and lands in L (width 1) or H (width 3), absent planes
// become zeros -- and ds_read_b64_tr_b4 reads them back transposed: a lane then holds, for one
// token pair, the two-bit fields of 16 channels, one per nibble, which IS an FP4 operand
// (field f = the number f/2) of v_mfma_scale_f32_16x16x128_f8f6f4 with k = channel, n = token.
// The other operand is the query, split into three FP8 (E4M3) pieces per head (rows 4*head +
// piece; block scales 2^(e - 4*piece) with e the exponent of the head's largest |q|), so every
// product is exact and the sum carries fp16's eleven bits of q.  The place value of tile H (4)
// is the block scale of that instruction's FP4 operand.  The pack minimums go the same way: a
// third tile holds them as two two-bit fields per (channel, group), one more instruction gives
// sum_d q_d m[g, d] for the four groups.  One unpack serves all heads.
#pragma once

#include "planes.h"

namespace packkv {

typedef int pk_v2i __attribute__((ext_vector_type(2)));

// Per wave: one plane tile of 128 channels x 4 groups of words, which holds tile L and then, once
// the transposed reads of L have been issued (LDS operations of a wave execute in order), tile H;
// and [128 channels] x 8 bytes with the pack minimums (nibble 2g = m & 3, nibble 2g + 1 = m >> 2),
// which later carries u[head][token] on its way to lane = token.
// Plane tile: the 16 bytes of an even channel c sit at 16 (c / 2) as groups 0 1 2 3, those of an
// odd channel at 1024 + 16 (c / 2) as groups 2 3 0 1: every lane writes two runs that are
// contiguous across the wave, and the 16 rows of a transposed read fall into different banks.
constexpr int K_TILE_P = 0;
constexpr int K_TILE_M = 2048;
constexpr int K_TILES_BYTES = 2048 + 1024;
__device__ inline int k_tile_row(int c, int gp) { return (c & 1) * 1024 + (c >> 1) * 16 + 8 * (gp ^ (c & 1)); }
// Channel of k-slot r (0..15) of the x-th transposed read of row group kb: the two reads of a lane
// take the two halves of its 32 channels in an order that alternates with kb, so that neighbouring
// row groups read different banks; the query operand is laid out to match.
__device__ inline int k_read_channel(int kb, int x, int r) { return 32 * kb + 16 * (x ^ (kb & 1)) + r; }
static_assert(4 * N * 4 <= 1024, "the score tile reuses the minimum tile");

// Per-width constants (LDS, entry w = 0..4): x = mask of plane L (whole word or 0), y = mask of
// plane H, z / w = mask that sends the widened plane T to tile L (width 1) / tile H (width 3).
__device__ inline void build_k_plane_table(uint4 *table) {
    const uint32_t w = threadIdx.x;
    if (w < 5)
        table[w] = make_uint4(w >= 2 ? ~0u : 0u, w == 4 ? ~0u : 0u, w == 1 ? 0x55555555u : 0u,
                              w == 3 ? 0x55555555u : 0u);
    __syncthreads();
}

// The query side of the product for one (batch, kv-head) stream: lane (m = lane % 16, kb =
// lane / 16) holds row m = 4 * head + piece of the FP8 operand for the channels of its k-groups
// (k 16 kb .. 16 kb + 15 and 64 + 16 kb .. 64 + 16 kb + 15; k_read_channel says which channels those are).
template <int G>
struct KQueryPlanes {
    pk_v8i a;       // FP8 operand
    int scale_a;    // E8M0 block scale of this lane's row
    float qsum[G];  // sum_d q[head][d], the same in every lane

    uint4 raw[4];   // fetch() -> build(): this lane's 32 query values as loaded

    // Issues the loads of this lane's part of q_group (the G query heads of the kv-head, [G][128]
    // fp16); build() turns them into the operand.  Kept apart so that a caller can start a chunk
    // transfer between the two and pay one memory latency for both.
    __device__ inline void fetch(const __half *q_group, int lane) {
        const int m = lane & 15, kb = lane >> 4;
        const int head = m >> 2;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            raw[2 * half] = raw[2 * half + 1] = make_uint4(0, 0, 0, 0);
            if (head < G) {
                // bytes 16 half .. 16 half + 15 are k-group kg = 4 half + kb: the (kg & 1)-th read of row group kg / 2
                const int kg = 4 * half + kb;
                const __half *src = q_group + head * D + k_read_channel(kg >> 1, kg & 1, 0);
                raw[2 * half] = *reinterpret_cast<const uint4 *>(src);
                raw[2 * half + 1] = *reinterpret_cast<const uint4 *>(src + 8);
            }
        }
    }

    __device__ inline void load(const __half *q_group, int lane) {
        fetch(q_group, lane);
        build(lane);
    }

    // The pieces of the value pairs first .. first + count - 1 (of this lane's 16 pairs), as FP8
    // byte pairs in out[pair / 2] (even pair: low half).  down: 2^-(e - 127).
    __device__ inline void pieces(int first, int count, int piece, float down, uint32_t (&out)[8]) const {
        const uint32_t w[16] = {raw[0].x, raw[0].y, raw[0].z, raw[0].w, raw[1].x, raw[1].y, raw[1].z, raw[1].w,
                                raw[2].x, raw[2].y, raw[2].z, raw[2].w, raw[3].x, raw[3].y, raw[3].z, raw[3].w};
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            if (k < first || k >= first + count) continue;
            // two values at a time: piece p is the FP8 rounding of what the pieces before it left, times 16^p
            float r0 = half_lo(w[k]) * down, r1 = half_hi(w[k]) * down;
            uint32_t pk = 0;
#pragma unroll
            for (int p = 0; p < 3; ++p) {
                const uint32_t c = uint32_t(__builtin_amdgcn_cvt_pk_fp8_f32(r0, r1, 0, false)) & 0xFFFFu;
                if (p == piece) pk = c;
                r0 = (r0 - __builtin_amdgcn_cvt_f32_fp8(int(c), 0)) * 16.0f;
                r1 = (r1 - __builtin_amdgcn_cvt_f32_fp8(int(c), 1)) * 16.0f;
            }
            if (k & 1)
                out[k >> 1] |= pk << 16;
            else
                out[k >> 1] = pk;
        }
    }

    // Exponent of the head's largest |q| and the sums: what every wave needs of all 32 values.
    // Returns e, the biased exponent of the largest |q| of the head (fp16 inputs: 103 .. 142; 127 for a zero head).
    __device__ inline int scan_values() {
        typedef _Float16 h2 __attribute__((ext_vector_type(2)));
        const uint32_t w[16] = {raw[0].x, raw[0].y, raw[0].z, raw[0].w, raw[1].x, raw[1].y, raw[1].z, raw[1].w,
                                raw[2].x, raw[2].y, raw[2].z, raw[2].w, raw[3].x, raw[3].y, raw[3].z, raw[3].w};
        h2 big2 = {_Float16(0.0f), _Float16(0.0f)};
        const h2 ones = {_Float16(1.0f), _Float16(1.0f)};
        float s = 0.0f;
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            big2 = __builtin_elementwise_max(big2, __builtin_bit_cast(h2, w[k] & 0x7FFF7FFFu));
            s = __builtin_amdgcn_fdot2(__builtin_bit_cast(h2, w[k]), ones, s, false);  // exact products, fp32 sum
        }
        float big = fmaxf(float(big2[0]), float(big2[1]));
        // the four lanes of a row (kb = 0..3) cover the 128 channels of its head
        s += __shfl_xor(s, 16);
        s += __shfl_xor(s, 32);
        big = fmaxf(big, __shfl_xor(big, 16));
        big = fmaxf(big, __shfl_xor(big, 32));
        // the sum of head g sits in the lanes of its rows
#pragma unroll
        for (int g = 0; g < G; ++g)
            qsum[g] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(s), 4 * g));
        const int e = int(__float_as_uint(big) >> 23);
        return e == 0 ? 127 : e;
    }

    __device__ inline void build(int lane) {
        const int m = lane & 15;
        const int head = m >> 2, piece = m & 3;
        const bool used = head < G && piece < 3;
        const int e = scan_values();
        uint32_t bytes[8];
        pieces(0, 16, piece, __uint_as_float(uint32_t(254 - e) << 23), bytes);
#pragma unroll
        for (int k = 0; k < 8; ++k) a[k] = used ? int(bytes[k]) : 0;
        scale_a = used ? e - 4 * piece : E8M0_ONE;
    }

    // The same with the piece arithmetic shared by the four waves of a workgroup that all need the
    // operand of one stream: wave w converts the value pairs 4w .. 4w + 3 of every lane and the
    // waves exchange the bytes through `share` (workgroup-shared LDS, 64 x 8 dwords, free for the
    // duration of the call).  Contains workgroup barriers: every wave of the workgroup must call it.
    __device__ inline void build_shared(int lane, int wave, uint32_t *share) {
        const int m = lane & 15;
        const int head = m >> 2, piece = m & 3;
        const bool used = head < G && piece < 3;
        const int e = scan_values();
        const float down = __uint_as_float(uint32_t(254 - e) << 23);
        uint32_t bytes[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        if (wave == 0) pieces(0, 4, piece, down, bytes);
        if (wave == 1) pieces(4, 4, piece, down, bytes);
        if (wave == 2) pieces(8, 4, piece, down, bytes);
        if (wave == 3) pieces(12, 4, piece, down, bytes);
        __syncthreads();  // `share` is free: every wave has left what used it before
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (wave == q) *reinterpret_cast<uint2 *>(share + lane * 8 + 2 * q) = make_uint2(bytes[2 * q], bytes[2 * q + 1]);
        __syncthreads();
        const uint4 lo = *reinterpret_cast<const uint4 *>(share + lane * 8);
        const uint4 hi = *reinterpret_cast<const uint4 *>(share + lane * 8 + 4);
        const uint32_t all[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
#pragma unroll
        for (int k = 0; k < 8; ++k) a[k] = used ? int(all[k]) : 0;
        scale_a = used ? e - 4 * piece : E8M0_ONE;
        __syncthreads();  // read by every wave: `share` may be reused
    }
};

// Where the columns of the result tiles are: column i of tile t holds token k_planes_token(i, t)
// of the block.
__device__ inline int k_planes_token(int i, int t) { return 32 * (t >> 1) + 8 * (t & 1) + (i & 7) + 16 * (i >> 3); }

// u[g] (lane = token `lane` of the block, every head g < G) for the chunk in the LDS buffer at
// byte offset `cur` of lds_all.  tiles: this wave's K_TILES_BYTES (16-byte aligned; it may be the
// chunk's own buffer).  chunk_read() is called once every lane's reads of the chunk have been
// issued and have returned: the buffer may be refilled from then on.
template <int G, class F>
__device__ inline void k_planes_chunk(const uint8_t *lds_all, int cur, const uint4 *table, uint8_t *tiles,
                                      const KQueryPlanes<G> &kq, float (&u)[G], F chunk_read) {
    float *sc = reinterpret_cast<float *>(tiles + K_TILE_M);
    const int lane = threadIdx.x & 63;
    const int i = lane & 15, kb = lane >> 4;
    const uint2 hdr = *reinterpret_cast<const uint2 *>(lds_all + cur + lane * 8);
    LanePlanes lp;
    lp.init(hdr.x, hdr.y, cur + HEADER);
    const uint32_t wsel_lo = hdr.x & 0xF0F0F0F0u, wsel_hi = hdr.y & 0xF0F0F0F0u;

    // ---- planes to their fixed places: lane l owns channels 2l, 2l + 1, pack j = (channel 2l + j / 4, group j % 4)
    uint32_t lo[8], hi[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uint32_t *e = reinterpret_cast<const uint32_t *>(lds_all + lp.e_pos(j));
        const uint32_t T = *reinterpret_cast<const uint16_t *>(lds_all + lp.o_pos(j));
        const uint32_t L = e[0], H = e[1];
        const uint32_t w16 = ((j < 4 ? wsel_lo : wsel_hi) >> (8 * (j & 3))) & 0xFFu;
        const uint4 k = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint8_t *>(table) + w16);
        // the bit of token t = 4r + s sits at 4s + r of T; in y the tokens 0..7 sit at bit 4n and the
        // tokens 8..15 at bit 4n + 2 (n = token % 8): bit 0 of the two-bit fields of a plane word
        const uint32_t y = T | (T << 15);
        lo[j] = (L & k.x) | (y & k.z);
        hi[j] = (H & k.y) | (y & k.w);
    }
    lds_reads_returned();  // every lane has read what it needs of the chunk
    wave_lds_fence();
    chunk_read();
    uint4 *tp = reinterpret_cast<uint4 *>(tiles + K_TILE_P + lane * 16);
    tp[0] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
    tp[64] = make_uint4(lo[6], lo[7], lo[4], lo[5]);
    // minimums: byte g of a header word = (w << 4) | m  ->  byte g = (m & 3) | (m >> 2) << 4
    const uint32_t m0 = (hdr.x & 0x03030303u) | ((hdr.x & 0x0C0C0C0Cu) << 2);
    const uint32_t m1 = (hdr.y & 0x03030303u) | ((hdr.y & 0x0C0C0C0Cu) << 2);
    *reinterpret_cast<uint4 *>(tiles + K_TILE_M + lane * 16) = make_uint4(m0, 0u, m1, 0u);
    wave_lds_fence();

    // ---- transposed reads and the products: rows = channels 32 kb + 16 half + i
    typedef __attribute__((address_space(3))) pk_v2i *lds_v2i;
    pk_v4f acc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[t] = pk_v4f{0.0f, 0.0f, 0.0f, 0.0f};
    const int c0 = k_read_channel(kb, 0, i), c1 = k_read_channel(kb, 1, i);
#pragma unroll
    for (int plane = 0; plane < 2; ++plane) {
        const uint8_t *tile = tiles + K_TILE_P;
        const int scale_b = E8M0_ONE + 1 + 2 * plane;  // a field f reads f / 2; tile H counts 4
        if (plane == 1) {
            // behind the reads of tile L in the wave's LDS queue
            wave_lds_fence();
            tp[0] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
            tp[64] = make_uint4(hi[6], hi[7], hi[4], hi[5]);
            wave_lds_fence();
        }
#pragma unroll
        for (int gp = 0; gp < 2; ++gp) {
            const pk_v2i r0 = __builtin_amdgcn_ds_read_tr4_b64_v2i32((lds_v2i)(tile + k_tile_row(c0, gp)));
            const pk_v2i r1 = __builtin_amdgcn_ds_read_tr4_b64_v2i32((lds_v2i)(tile + k_tile_row(c1, gp)));
            const int M = int(FIELD2_MASK);
            const pk_v8i b_lo = {r0[0] & M, r0[1] & M, r1[0] & M, r1[1] & M, 0, 0, 0, 0};
            const pk_v8i b_hi = {int(uint32_t(r0[0]) >> 2) & M, int(uint32_t(r0[1]) >> 2) & M,
                                 int(uint32_t(r1[0]) >> 2) & M, int(uint32_t(r1[1]) >> 2) & M, 0, 0, 0, 0};
            acc[2 * gp] = mfma_fp8_fp4(kq.a, b_lo, acc[2 * gp], kq.scale_a, scale_b);
            acc[2 * gp + 1] = mfma_fp8_fp4(kq.a, b_hi, acc[2 * gp + 1], kq.scale_a, scale_b);
        }
    }
    // pack minimums: column i = 2 g + part (i < 8), the high part counts 4
    float ms;
    {
        const uint8_t *tile = tiles + K_TILE_M;
        const pk_v2i r0 = __builtin_amdgcn_ds_read_tr4_b64_v2i32((lds_v2i)(tile + c0 * 8));
        const pk_v2i r1 = __builtin_amdgcn_ds_read_tr4_b64_v2i32((lds_v2i)(tile + c1 * 8));
        const pk_v8i b = {r0[0], r0[1], r1[0], r1[1], 0, 0, 0, 0};
        const pk_v4f zero = {0.0f, 0.0f, 0.0f, 0.0f};
        const pk_v4f mm = mfma_fp8_fp4(kq.a, b, zero, kq.scale_a, E8M0_ONE + 1 + 2 * (i & 1));
        ms = (mm[0] + mm[1]) + mm[2];
        ms += dpp_f32<DPP_QUAD_XOR1>(ms);  // both parts: lanes 2g and 2g + 1 of the row hold group g
    }
    const int rg = kb;
    const float ms_a = __shfl(ms, (lane & 48) | ((i >> 3) << 1));        // groups 0, 1: tiles 0, 1
    const float ms_b = __shfl(ms, (lane & 48) | ((i >> 3) << 1) | 4);    // groups 2, 3: tiles 2, 3
    // The matrix instructions take operands from all 64 lanes whatever the execution mask is, but the
    // compiler treats them as per-lane arithmetic and would move them, with the operand set-up, into
    // the lane-dependent branch below, where the other rows' lanes no longer compute their operands:
    // the results are pinned here, in uniform control flow.
#pragma unroll
    for (int t = 0; t < 4; ++t) asm volatile("" : "+v"(acc[t]));
    // ---- to lane = token through LDS: lane (i, rg) holds head rg for the tokens k_planes_token(i, t)
    if (rg < G) {
#pragma unroll
        for (int t = 0; t < 4; ++t)
            sc[rg * N + k_planes_token(i, t)] = ((acc[t][0] + acc[t][1]) + acc[t][2]) + (t < 2 ? ms_a : ms_b);
    }
    wave_lds_fence();
#pragma unroll
    for (int g = 0; g < G; ++g) u[g] = sc[g * N + lane];
    wave_lds_fence();  // the tiles and sc are rewritten by the next chunk
}

}  // namespace packkv
