// Two-element fp16 dot products for the K paths of chunks with packs of 8 tokens and of wide
// chunks (pack8.h; PackKV Sec. III-C.1): unpacked channel pairs are contracted against the
// matching query pair in one instruction, and the pack minimums come straight from the header.
#pragma once

#include "unpack.h"

namespace packkv {

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

// d = a.lo * b.lo + a.hi * b.hi + c with a, b pairs of fp16 and fp32 accumulation: the
// three-address dot-product instruction, from inline assembly.  The compiler's own choice is the
// two-address form, which costs a register copy for every accumulator that starts from a live
// value.  Dot-product results need three wait states before an instruction of another kind reads
// or overwrites them, which the compiler does not track into inline assembly: every dot product
// of these paths goes through this one function, so that their results are only ever consumed as
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

}  // namespace packkv
