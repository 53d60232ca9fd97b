// Device helpers shared by the fused K, V and attention kernels (gfx950, wave64): DPP wave scan
// and row reductions, the index batch of a wave, direct global -> LDS transfers of whole chunks
// and of metadata rows with their counted waits, and the pack tables of the kernels for packs of
// 8 tokens and wide chunks (pack8.h).  The decode of chunks with packs of 16 tokens (plane
// layout) is in planes.h, k_planes.h and v_planes.h.
//
// In the paths of pack8.h the codes of a pack never become fp32 one by one: the unpack leaves each
// code in the low bits of a 16-bit half, which read as fp16 is the subnormal code * 2^-24 --
// exact, no conversion instruction -- ready for an fp16 dot-product instruction or an fp16 MFMA;
// the factor 2^24 is applied once per output.
#pragma once

#include "common.h"

namespace packkv {

// A pack read may touch a few bytes past the end of a chunk buffer (at most 12).
constexpr int LDS_TAIL_PAD = 16;
constexpr float CODE_SCALE = 16777216.0f;  // 2^24: fp16 subnormal unit^-1
// The matrix cores align the products of one instruction to the largest nominal exponent
// and keep about 24 bits below it.  A code in the lowest bits of a subnormal leaves up to
// ten leading zeros in its significand, so products of tokens whose weights differ by 2^8
// or more were measured to lose bits from 2^-17 on.  The V path therefore places each code
// six bits higher (still subnormal for codes up to 15): value code * 2^-18.
constexpr int CODE_LIFT = 6;
constexpr float CODE_SCALE_LIFTED = 262144.0f;  // 2^18

// DPP controls (wave64, rows of 16 lanes).
constexpr int DPP_QUAD_XOR1 = 0xB1;  // quad_perm [1,0,3,2]
constexpr int DPP_QUAD_XOR2 = 0x4E;  // quad_perm [2,3,0,1]
constexpr int DPP_ROW_ROR8 = 0x128;  // lane i <- lane i^8 of its row
constexpr int DPP_ROW_ROR4 = 0x124;  // lane i <- lane (i-4) mod 16 of its row
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

// Per-header-byte constants, kept in LDS so that a pack's width-dependent
// values cost one LDS read instead of several vector instructions:
//   x = pair mask ((1 << w) - 1) * 0x10001, y = w (bits 0..4, a rotate amount as it stands)
//   with 4w in byte 1, z = 8 * w, w = float(min)
// Valid header bytes are below 0x50 (width <= 4); a corrupt byte would index past
// the table, which on this hardware reads other LDS contents or zero, never faults.
constexpr int PACK_TABLE_ENTRIES = 80;

// With many query heads per kv-head the per-head pack-minimum terms cost more registers and
// instructions than adding the minimum to the codes themselves (eight integer adds per pack,
// code + m <= 15 still fits the subnormal): from this group size on the kernels fold it in.
template <int G>
constexpr bool fold_min() { return G >= 4; }

// Built once per workgroup, followed by a workgroup barrier.  lift: bit position of a code
// inside its 16-bit half after the unpack (0 or CODE_LIFT).  fold: the last field is
// the pack minimum as a bit pattern for both halves (to be added to the unpacked words)
// instead of float(min).
__device__ inline void build_pack_table(uint4 *table, int lift = 0, bool fold = false) {
    const uint32_t hb = threadIdx.x;
    if (hb < PACK_TABLE_ENTRIES) {
        const uint32_t w = hb >> 4, m = hb & 15u;
        const uint32_t m1 = ((1u << w) - 1u) << lift;
        table[hb] = make_uint4(m1 | (m1 << 16), w | (4 * w << 8), 8 * w,
                               fold ? (m << lift) * 0x10001u : __float_as_uint(float(m)));
    }
    __syncthreads();
}

// Pack table of the K paths that unpack two packs side by side (pack8.h): eight bytes
// per entry (half the LDS traffic and bank conflicts of the 16-byte form), every field placed
// where its consumer reads it without a shift:
//   x: 4w in bits 0..4 (a bit-field offset/width as it stands), w in byte 1, the w-bit code
//      mask in the high half
//   y: 8w in bits 0..5 (a 64-bit shift amount as it stands), fp16(pack minimum) in the high half
__device__ inline void build_pair_table(uint2 *table) {
    const uint32_t hb = threadIdx.x;
    if (hb < PACK_TABLE_ENTRIES) {
        const uint32_t w = hb >> 4, m = hb & 15u;
        const uint32_t m16 = __half_as_ushort(__float2half(float(m)));
        table[hb] = make_uint2((4 * w) | (w << 8) | (((1u << w) - 1u) << 16), (8 * w) | (m16 << 16));
    }
    __syncthreads();
}

// Inclusive prefix sums of the four bytes of x (no byte overflows for the callers' values):
// two shift-and-add instructions.  Written out as such because the compiler turns the plain C
// form into a multiplication by 0x01010101, i.e. quarter-rate 32-bit multiplies, one of them a
// 64-bit multiply-add whose undefined upper addend register made it wait for whatever load
// happened to be in flight into that register -- which serialized transfer and unpack again.
__device__ inline uint32_t byte_prefix_sums(uint32_t x) {
    uint32_t y;
    asm("v_lshl_add_u32 %0, %1, 8, %1" : "=v"(y) : "v"(x));
    asm("v_lshl_add_u32 %0, %1, 16, %1" : "=v"(x) : "v"(y));
    return x;
}

// Chunk offsets of up to 64 blocks of one wave, one block per lane: lane i holds
// the index words of block first + stride*i of stream (b, h).  Read once per 64
// blocks; iterations pick their words with v_readlane, so no chunk waits on an
// index load.  words = 1: chunks lie back to back, chunk c spans index[c]..index[c+1];
// words = 2 (paged arena): index[2c] and index[2c+1] are the chunk's own start and end.
struct IndexBatch {
    uint32_t o0, o1;
    __device__ inline void load(const uint32_t *__restrict__ index, int words, int first, int stride,
                                int end, int B, int H, int b, int h, int lane) {
        const int blk = first + stride * lane;
        const int64_t c = blk < end ? (int64_t(blk) * B + b) * H + h : 0;
        o0 = index[c * words];
        o1 = index[c * words + 1];
    }
    __device__ inline uint32_t start16(int it) const { return __builtin_amdgcn_readlane(o0, it); }
    __device__ inline uint32_t end16(int it) const { return __builtin_amdgcn_readlane(o1, it); }
};

// One LDS buffer holds one whole chunk (header + payload).
constexpr int CHUNK_LDS = CHUNK_MAX;

// Start the transfer of a chunk straight from global memory into an LDS buffer
// (global_load_lds_dwordx4: lane i's 16 bytes land at buf + 1024k + 16i, no
// vector registers involved), so that it is in flight while the previous chunk
// is unpacked.  o0/o1: the chunk's index words; buf: wave-uniform.  A dropped
// block (size 0) transfers nothing.  Lanes past the chunk end re-read its last
// 16 bytes into buffer bytes nobody decodes; the last slice only uses the lanes
// that stay inside the buffer (0..31 of the fifth slice for the 4608-byte buffer).
//
// The instruction is issued from inline assembly on purpose.  Issued through the
// compiler's builtin, every later LDS read of the wave -- also of the OTHER buffer --
// is preceded by a compiler-inserted wait for all outstanding transfers (it cannot tell the
// buffers apart), which serializes transfer and unpack inside a wave.  Here the waits
// are explicit (wait_chunk_landed*), counted by the callers.  M0 carries the LDS base;
// the s_nop is the wait state between writing M0 and the transfer that reads it.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"  // M0 is a reserved register; naming it as clobbered is the point
// MAXB: buffer bytes = largest chunk; HDR: header bytes, the smallest valid chunk.  STREAM: the
// transfers carry the non-temporal hint -- a chunk is read once, and without the hint it pushes
// out of the caches what the kernel reads again, what the kernel before it has just written (the
// weights of the V product) and what the kernel after it reads first (the scores of the K product).
#define PACKKV_CHUNK_TRANSFERS(POLICY)                                                                                  \
    for (int k = 0; k < (MAXB + 1023) / 1024; ++k) {                                                                    \
        if (k * 1024 < size && ((k + 1) * 1024 <= MAXB || k * 1024 + lane * 16 < MAXB)) {                               \
            const int off = lane * 16;                                                                                  \
            const int lim = last - k * 1024;                                                                            \
            const int voff = off < lim ? off : lim;                                                                     \
            if (k == 0) asm volatile("global_load_lds_dwordx4 %0, %1" POLICY : : "v"(voff), "s"(chunk) : "memory", "m0"); \
            if (k == 1) asm volatile("global_load_lds_dwordx4 %0, %1 offset:1024" POLICY : : "v"(voff), "s"(chunk) : "memory", "m0"); \
            if (k == 2) asm volatile("global_load_lds_dwordx4 %0, %1 offset:2048" POLICY : : "v"(voff), "s"(chunk) : "memory", "m0"); \
            if (k == 3) asm volatile("global_load_lds_dwordx4 %0, %1 offset:3072" POLICY : : "v"(voff), "s"(chunk) : "memory", "m0"); \
            if (k >= 4)                                                                                                 \
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" POLICY                       \
                             :                                                                                          \
                             : "s"(lds + k * 1024), "v"(voff), "s"(chunk + k * 1024)                                    \
                             : "memory", "m0");                                                                         \
        }                                                                                                               \
    }
template <int MAXB = CHUNK_MAX, int HDR = HEADER, bool STREAM = false>
__device__ inline void chunk_issue_lds(const uint8_t *__restrict__ arena, uint32_t o0, uint32_t o1,
                                       uint8_t *buf, int lane) {
    const int size = int(o1 - o0) * 16;
    if (size < HDR) return;
    const uint8_t *chunk = arena + size_t(o0) * 16;
    const int last = size - 16;
    const uint32_t lds = uint32_t(uintptr_t((__attribute__((address_space(3))) void *)buf));
    // One M0 write per chunk for the first four slices: the instruction offset moves the global
    // and the LDS address alike.  Nothing between these statements touches M0 (no LDS-DMA
    // builtin, no indexed register access, no message).
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0" : : "s"(lds) : "memory", "m0");
    if constexpr (STREAM) {
#pragma unroll
        PACKKV_CHUNK_TRANSFERS(" nt")
    } else {
#pragma unroll
        PACKKV_CHUNK_TRANSFERS("")
    }
}
#undef PACKKV_CHUNK_TRANSFERS
#pragma clang diagnostic pop

// All outstanding global->LDS transfers (and other vector memory operations) of
// this wave have landed.
__device__ inline void wait_chunk_landed() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// The same while the LATER newest vector memory operations of this wave (issued after the
// chunk's transfers: a metadata load, a result store) may stay in flight; the counter retires
// in issue order.  Callers keep the issue order fixed with vmem_order_fence().
template <int LATER>
__device__ inline void wait_chunk_landed_except() {
    static_assert(LATER >= 0 && LATER < 64, "the counter has six bits");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LATER) : "memory");
}
// Compiler-only fence: memory operations are not moved across it.
__device__ inline void vmem_order_fence() { asm volatile("" ::: "memory"); }
// Three chunk buffers per wave (chunks n+1 and n+2 in flight while chunk n is decoded): the same
// transfer, with the number of transfer instructions it issued as the result (wave-uniform; 0 for
// a dropped block), which the caller needs to count the vector memory operations that may stay in
// flight at its next wait.
template <int MAXB = CHUNK_MAX, int HDR = HEADER, bool STREAM = false>
__device__ inline int chunk_issue_lds_counted(const uint8_t *__restrict__ arena, uint32_t o0, uint32_t o1,
                                              uint8_t *buf, int lane) {
    const int size = int(o1 - o0) * 16;
    if (size < HDR) return 0;
    chunk_issue_lds<MAXB, HDR, STREAM>(arena, o0, o1, buf, lane);
    const int slices = (size + 1023) >> 10;
    constexpr int MOST = (MAXB + 1023) / 1024;
    return slices < MOST ? slices : MOST;
}

// One dword per lane straight from global memory into LDS: lane i's word row[i] lands at
// buf + 4 i (one transfer instruction; same rules as chunk_issue_lds).  row, buf: wave-uniform.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ inline void row_issue_lds(const void *__restrict__ row, uint8_t *buf, int lane) {
    const uint32_t lds = uint32_t(uintptr_t((__attribute__((address_space(3))) void *)buf));
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
                 :
                 : "s"(lds), "v"(lane * 4), "s"(row)
                 : "memory", "m0");
}
#pragma clang diagnostic pop

// Waits until at most `later` (wave-uniform, 0..MOST) + FIXED of this wave's newest vector memory
// operations are still in flight (the counter retires in issue order).
template <int FIXED, int MOST>
__device__ inline void wait_vmem_except(int later) {
    static_assert(FIXED + MOST < 64, "the counter has six bits");
    switch (later) {
        case 0: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(FIXED) : "memory"); break;
        case 1: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(FIXED + (MOST >= 1 ? 1 : 0)) : "memory"); break;
        case 2: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(FIXED + (MOST >= 2 ? 2 : 0)) : "memory"); break;
        case 3: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(FIXED + (MOST >= 3 ? 3 : 0)) : "memory"); break;
        case 4: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(FIXED + (MOST >= 4 ? 4 : 0)) : "memory"); break;
        default: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(FIXED + (MOST >= 5 ? 5 : 0)) : "memory"); break;
    }
}

// Makes a value that was loaded ahead count as used here, so that the compiler's own wait
// for that load sits at this point (right after an explicit wait, where it costs nothing) and
// not later, behind the next chunk's transfers, which it would then wait for as well.
__device__ inline void consume_here(uint32_t &x) { asm volatile("" : "+v"(x)); }
__device__ inline void consume_here(float &x) { asm volatile("" : "+v"(x)); }

// Every LDS read this wave has issued has returned its data (needed before a transfer may
// overwrite a buffer the wave has just decoded: the transfer does not queue behind LDS reads).
__device__ inline void lds_reads_returned() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// LDS writes of this wave become visible to its own later LDS reads in program
// order; the fences only stop the compiler from moving accesses across.
__device__ inline void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// x >> (byte 1 of amount): the sub-dword operand select reads the byte in place, which saves
// the instruction that would extract it (the compiler does not form this by itself).
__device__ inline uint32_t shr_by_byte1(uint32_t x, uint32_t amount) {
    uint32_t y;
    asm("v_lshrrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_1 src1_sel:DWORD"
        : "=v"(y)
        : "v"(amount), "v"(x));
    return y;
}

__device__ inline float half_lo(uint32_t p) { return float(__builtin_bit_cast(_Float16, uint16_t(p & 0xFFFFu))); }
__device__ inline float half_hi(uint32_t p) { return float(__builtin_bit_cast(_Float16, uint16_t(p >> 16))); }

// Reduce-scatter inside each row of 16 lanes.  On entry every lane holds 16 partial sums
// (v[i] belongs to index i); on return lane i of the row holds the row's sum for index i.  The first
// round adds the partner lane's value (eight lanes away) with the write restricted to one
// half of the row per instruction: lanes 0..7 take index k, lanes 8..15 index k+8 -- two adds
// per output and no selects; the second round does the same with the lane four away.  The
// leading s_nop covers the wait states between the instruction that produced an input and
// its DPP read, which the compiler does not track into inline assembly: two after an ordinary
// vector instruction, three after a dot-product instruction (the callers' accumulators) --
// four are inserted.
__device__ inline float row_reduce_scatter16(float (&v)[16], int lane) {
    float a[8], b[4], c[2];
    const bool b1 = lane & 2, b0 = lane & 1;
    asm("s_nop 3\n\t"
        "v_add_f32_dpp %0, %8, %8 row_ror:8 row_mask:0xf bank_mask:0x3\n\t"
        "v_add_f32_dpp %1, %9, %9 row_ror:8 row_mask:0xf bank_mask:0x3\n\t"
        "v_add_f32_dpp %2, %10, %10 row_ror:8 row_mask:0xf bank_mask:0x3\n\t"
        "v_add_f32_dpp %3, %11, %11 row_ror:8 row_mask:0xf bank_mask:0x3\n\t"
        "v_add_f32_dpp %4, %12, %12 row_ror:8 row_mask:0xf bank_mask:0x3\n\t"
        "v_add_f32_dpp %5, %13, %13 row_ror:8 row_mask:0xf bank_mask:0x3\n\t"
        "v_add_f32_dpp %6, %14, %14 row_ror:8 row_mask:0xf bank_mask:0x3\n\t"
        "v_add_f32_dpp %7, %15, %15 row_ror:8 row_mask:0xf bank_mask:0x3\n\t"
        "v_add_f32_dpp %0, %16, %16 row_ror:8 row_mask:0xf bank_mask:0xc\n\t"
        "v_add_f32_dpp %1, %17, %17 row_ror:8 row_mask:0xf bank_mask:0xc\n\t"
        "v_add_f32_dpp %2, %18, %18 row_ror:8 row_mask:0xf bank_mask:0xc\n\t"
        "v_add_f32_dpp %3, %19, %19 row_ror:8 row_mask:0xf bank_mask:0xc\n\t"
        "v_add_f32_dpp %4, %20, %20 row_ror:8 row_mask:0xf bank_mask:0xc\n\t"
        "v_add_f32_dpp %5, %21, %21 row_ror:8 row_mask:0xf bank_mask:0xc\n\t"
        "v_add_f32_dpp %6, %22, %22 row_ror:8 row_mask:0xf bank_mask:0xc\n\t"
        "v_add_f32_dpp %7, %23, %23 row_ror:8 row_mask:0xf bank_mask:0xc"
        : "=&v"(a[0]), "=&v"(a[1]), "=&v"(a[2]), "=&v"(a[3]), "=&v"(a[4]), "=&v"(a[5]), "=&v"(a[6]), "=&v"(a[7])
        : "v"(v[0]), "v"(v[1]), "v"(v[2]), "v"(v[3]), "v"(v[4]), "v"(v[5]), "v"(v[6]), "v"(v[7]),
          "v"(v[8]), "v"(v[9]), "v"(v[10]), "v"(v[11]), "v"(v[12]), "v"(v[13]), "v"(v[14]), "v"(v[15]));
    // second round, partner four lanes away: lanes 0..3 and 8..11 of the row (banks 0, 2) take
    // index k from the lane four above (rotate right by 12), the others index k+4 from four below
    asm("s_nop 1\n\t"
        "v_add_f32_dpp %0, %4, %4 row_ror:12 row_mask:0xf bank_mask:0x5\n\t"
        "v_add_f32_dpp %1, %5, %5 row_ror:12 row_mask:0xf bank_mask:0x5\n\t"
        "v_add_f32_dpp %2, %6, %6 row_ror:12 row_mask:0xf bank_mask:0x5\n\t"
        "v_add_f32_dpp %3, %7, %7 row_ror:12 row_mask:0xf bank_mask:0x5\n\t"
        "v_add_f32_dpp %0, %8, %8 row_ror:4 row_mask:0xf bank_mask:0xa\n\t"
        "v_add_f32_dpp %1, %9, %9 row_ror:4 row_mask:0xf bank_mask:0xa\n\t"
        "v_add_f32_dpp %2, %10, %10 row_ror:4 row_mask:0xf bank_mask:0xa\n\t"
        "v_add_f32_dpp %3, %11, %11 row_ror:4 row_mask:0xf bank_mask:0xa"
        : "=&v"(b[0]), "=&v"(b[1]), "=&v"(b[2]), "=&v"(b[3])
        : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]), "v"(a[4]), "v"(a[5]), "v"(a[6]), "v"(a[7]));
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
    v += dpp_f32<DPP_ROW_ROR4>(v);  // lanes i, i+4, i+8, i+12: the set is closed under the rotation
    v += dpp_f32<DPP_QUAD_XOR2>(v);
    v += dpp_f32<DPP_QUAD_XOR1>(v);
    return v;
}

}  // namespace packkv
