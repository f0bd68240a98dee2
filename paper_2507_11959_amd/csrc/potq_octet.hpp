// Decode of one "octet" (eight consecutive weights of a row) of the canonical packed layout into
// eight fp16 weights, shared by the stand-alone de-quantisation and the canonical-layout GEMV.
#pragma once

#include "potq_device.hpp"

namespace potq {

// 32 (bits=4), 24 (bits=3) or 16 (bits=2) code bits of octet `o`, from aligned 32-bit words.
template <int BITS>
__device__ __forceinline__ uint32_t load_octet_bits(const uint32_t *__restrict__ words, int64_t o)
{
    if (BITS == 3) {
        const int64_t byte = 3 * o;
        const uint32_t a = words[byte >> 2];
        const uint32_t b = words[(byte + 2) >> 2];        // word holding the octet's last byte
        return __builtin_amdgcn_alignbyte(b, a, (uint32_t)(byte & 3)) & 0xFFFFFFu;
    } else if (BITS == 4) {
        return words[o];
    } else {
        const uint32_t a = words[o >> 1];
        return (a >> (16 * (uint32_t)(o & 1))) & 0xFFFFu;
    }
}

// Sec. 4.2 for two codes at once, one per 16-bit half of a register: the field
// (sign, 000, E) << 10 of each code is added, as a 16-bit integer, to the bit
// pattern of the scale (v_pk_add_u16: the halves wrap independently, which is
// the documented behaviour for scales outside the exact domain).
typedef uint16_t u16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t add_u16x2(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_bit_cast(u16x2, a) + __builtin_bit_cast(u16x2, b));
}

// Two adjacent codes (2*BITS bits at bit `pos` of f) -> code A in bits [0,BITS), code B in [16,16+BITS).
template <int BITS>
__device__ __forceinline__ uint32_t spread_pair(uint32_t f, int pos)
{
    const uint32_t y = __builtin_amdgcn_ubfe(f, pos, 2 * BITS);
    return __umul24(y, (1u << (16 - BITS)) | 1u) & (((1u << BITS) - 1u) * 0x00010001u);
}

template <int BITS>
__device__ __forceinline__ u32x4 pot_octet(uint32_t f, uint32_t scale_bits)
{
    const uint32_t s2 = scale_bits | (scale_bits << 16);
    u32x4 out;
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        const uint32_t pair = spread_pair<BITS>(f, 2 * BITS * m);
        // c * (2^10 + 2^(16-BITS)) puts E on bits 10.. and the sign on bit 15; stray copies are masked off
        // (with four bits the two copies would overlap, so the sign is moved separately)
        const uint32_t t = (BITS == 3)   ? (__umul24(pair, 0x2400u) & 0x8C008C00u)
                           : (BITS == 2) ? (__umul24(pair, 0x4400u) & 0x84008400u)
                                         : (((pair & 0x00070007u) << 10) | ((pair & 0x00080008u) << 12));
        out[m] = add_u16x2(s2, t);
    }
    return out;
}

// Uniform baseline, Sec. 4.1 Eq. (9): q -> fp16 by or-ing it into the mantissa
// of 1024.0 (0x6400), then (1024 + q) + (Z - 1024) = q + Z exactly and one
// rounded multiply by S.
template <int BITS>
__device__ __forceinline__ u32x4 int_octet(uint32_t f, half2_t zm1024, half2_t s2)
{
    u32x4 out;
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        const uint32_t pair = spread_pair<BITS>(f, 2 * BITS * m) | 0x64006400u;
        const half2_t w = (as_half2(pair) + zm1024) * s2;
        out[m] = as_u32(w);
    }
    return out;
}

}  // namespace potq
