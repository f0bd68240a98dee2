// Device-side helpers shared by the gfx950 kernels of the potq library.
//
// Everything here is integer bit manipulation on packed code words and fp16 bit
// patterns (Sec. 4.1-4.2 of PoT-PTQ): no floating-point instruction takes part
// in turning a PoT code into an fp16 weight.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace potq {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;

// v_perm_b32: each selector byte picks one byte of the 64-bit value {hi, lo}
// (0-3: bytes of lo, 4-7: bytes of hi).
__device__ __forceinline__ uint32_t byte_perm(uint32_t hi, uint32_t lo, uint32_t sel)
{
    return __builtin_amdgcn_perm(hi, lo, sel);
}

// Add two words as four independent bytes (each byte wraps modulo 256).
__device__ __forceinline__ uint32_t add_bytes(uint32_t a, uint32_t b)
{
    return ((a & 0x7F7F7F7Fu) + (b & 0x7F7F7F7Fu)) ^ ((a ^ b) & 0x80808080u);
}

__device__ __forceinline__ half2_t as_half2(uint32_t v)
{
    return __builtin_bit_cast(half2_t, v);
}

__device__ __forceinline__ uint32_t as_u32(half2_t v)
{
    return __builtin_bit_cast(uint32_t, v);
}

// A 16-byte store of output that the pass does not read again: marked streaming (nt) and written
// through at system scope (sc0 sc1) instead of resting in the L2 until it is evicted.  On the
// 70B-sized de-quantisation pass the three bits together measured 2 % faster than nt alone (what
// __builtin_nontemporal_store emits) and 7 % faster than a plain store.  The compiler does not
// count the store in its s_waitcnt bookkeeping, which can only make a later wait longer (the
// counter is in order); the hardware waits for outstanding stores when the wavefront ends.
// Nor does it know the hazard of a store of more than 8 bytes whose data registers the next
// vector instruction overwrites before they have been read: the s_nop covers the two wait
// states that needs.  No "memory" clobber: the pointee is output that the kernel never reads,
// and the clobber would keep the loads of later steps from being issued ahead of the store.
__device__ __forceinline__ void store_streaming(u32x4 *p, u32x4 v)
{
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1 nt\n\ts_nop 1" : : "v"(p), "v"(v));
}

// ---------------------------------------------------------------------------
// Private bit map of POTQ_LAYOUT_TILE16.
//
// A tile holds 16 rows x 128 columns (one scale group per row).  It is stored
// as `bits` slabs of 16 x 16 bytes: slab j, row r is the uint4 L_j[r].  Column
// block t (t = 0..3, columns 32t..32t+31 of the tile) of row r lives in word t
// of every slab: (L_0[r].w[t], L_1[r].w[t] [, L_2[r].w[t]]).
//
// Inside a block the 32 codes are arranged as 8 "selectors" of 4 codes, one
// code per byte lane, so that (word >> shift) & mask is directly a v_perm_b32
// selector:
//   bits = 3, words (w0, w1, w2):
//     selector m = 0..5 : byte j holds code = (w[m/2] >> (8j + 3(m%2))) & 7
//     selector 6        : exponent = (w0 >> (8j+6)) & 3, sign = (w2 >> (8j+6)) & 1
//     selector 7        : exponent = (w1 >> (8j+6)) & 3, sign = (w2 >> (8j+7)) & 1
//   bits = 2, words (w0, w1):
//     selector m = 0..7 : byte j holds code = (w[m/4] >> (8j + 2(m%4))) & 3
//   bits = 4, words (w0, w1, w2, w3):
//     selector m = 0..7 : byte j holds code = (w[m/2] >> (8j + 4(m%2))) & 15
// Selector m, byte j is column 4m + p(j) of the block, p = (0, 2, 1, 3): bytes
// 0 and 2 are an adjacent column pair, bytes 1 and 3 the next pair.
// ---------------------------------------------------------------------------
constexpr int kTileRows = 16;
constexpr int kTileCols = 128;

__host__ __device__ constexpr int tile_bytes(int bits) { return bits * 16 * 16; }

// The eight selectors of a 3-bit block.
__device__ __forceinline__ void selectors3(uint32_t w0, uint32_t w1, uint32_t w2, uint32_t sel[8])
{
    const uint32_t m7 = 0x07070707u;
    sel[0] = w0 & m7;
    sel[1] = (w0 >> 3) & m7;
    sel[2] = w1 & m7;
    sel[3] = (w1 >> 3) & m7;
    sel[4] = w2 & m7;
    sel[5] = (w2 >> 3) & m7;
    sel[6] = ((w0 >> 6) & 0x03030303u) | ((w2 >> 4) & 0x04040404u);
    sel[7] = ((w1 >> 6) & 0x03030303u) | ((w2 >> 5) & 0x04040404u);
}

// The eight selectors of a 2-bit block.
__device__ __forceinline__ void selectors2(uint32_t w0, uint32_t w1, uint32_t sel[8])
{
    const uint32_t m3 = 0x03030303u;
    sel[0] = w0 & m3;
    sel[1] = (w0 >> 2) & m3;
    sel[2] = (w0 >> 4) & m3;
    sel[3] = (w0 >> 6) & m3;
    sel[4] = w1 & m3;
    sel[5] = (w1 >> 2) & m3;
    sel[6] = (w1 >> 4) & m3;
    sel[7] = (w1 >> 6) & m3;
}

// ---------------------------------------------------------------------------
// PoT group table (Sec. 4.2 hoisted to once per group).  The integer add of
// (sign, 000, E) << 10 into the scale only changes the scale's high byte:
// high' = high + ((sign << 7) | (E << 2)) (mod 256), low byte untouched.  So
// the 2^bits possible high bytes of a group are computed once, by that integer
// add, and every weight of the group is then a byte look-up.
// ---------------------------------------------------------------------------
struct PotTable {
    uint32_t lo;    // high bytes for codes 0..3
    uint32_t hi;    // high bytes for codes 4..7 (3-bit only)
    uint32_t low2;  // the scale's low byte in bytes 0 and 2
};

template <int BITS>
__device__ __forceinline__ PotTable pot_table(uint32_t scale_bits)
{
    PotTable t;
    const uint32_t sh = (scale_bits >> 8) & 0xFFu;
    const uint32_t rep = sh * 0x01010101u;
    if (BITS == 3) {
        t.lo = add_bytes(rep, 0x0C080400u);   // +E<<2, sign 0
        t.hi = add_bytes(rep, 0x8C888480u);   // +E<<2, sign 1
    } else {
        t.lo = add_bytes(rep, 0x84800400u);   // codes 00, 01, 10, 11 = +1, +2, -1, -2
        t.hi = t.lo;
    }
    const uint32_t sl = scale_bits & 0xFFu;
    t.low2 = sl | (sl << 16);
    return t;
}

// Four codes (one selector) -> two packed fp16 pairs:
//   even = (column 4m, 4m+1), odd = (column 4m+2, 4m+3).
__device__ __forceinline__ void pot_lookup(const PotTable &t, uint32_t sel, uint32_t &even, uint32_t &odd)
{
    const uint32_t r = byte_perm(t.hi, t.lo, sel);          // four high bytes
    even = byte_perm(r, t.low2, 0x06000400u);               // [low, r.b0, low, r.b2]
    odd = (r & 0xFF00FF00u) | t.low2;                       // [low, r.b1, low, r.b3]
}

// ---------------------------------------------------------------------------
// Uniform baseline group table (Sec. 4.1 Eq. (9)): the 2^bits values
// fp16((q + Z) * S) of a group, one rounding each, split into a table of high
// bytes and a table of low bytes.
// ---------------------------------------------------------------------------
struct IntTable {
    uint32_t hlo, hhi;  // high bytes for codes 0..3 / 4..7
    uint32_t llo, lhi;  // low bytes
};

template <int BITS>
__device__ __forceinline__ IntTable int_table(uint32_t scale_bits, uint32_t zero_bits)
{
    const _Float16 S = __builtin_bit_cast(_Float16, (uint16_t)scale_bits);
    const _Float16 Z = __builtin_bit_cast(_Float16, (uint16_t)zero_bits);
    uint32_t v[8];
#pragma unroll
    for (int q = 0; q < (1 << BITS); ++q) {
        const _Float16 w = ((_Float16)(float)q + Z) * S;   // q + Z exact, one rounding in the product
        v[q] = (uint32_t)__builtin_bit_cast(uint16_t, w);
    }
    IntTable t;
    t.hlo = (v[0] >> 8) | (v[1] & 0xFF00u) | ((v[2] & 0xFF00u) << 8) | ((v[3] & 0xFF00u) << 16);
    t.llo = (v[0] & 0xFFu) | ((v[1] & 0xFFu) << 8) | ((v[2] & 0xFFu) << 16) | ((v[3] & 0xFFu) << 24);
    if (BITS == 3) {
        t.hhi = (v[4] >> 8) | (v[5] & 0xFF00u) | ((v[6] & 0xFF00u) << 8) | ((v[7] & 0xFF00u) << 16);
        t.lhi = (v[4] & 0xFFu) | ((v[5] & 0xFFu) << 8) | ((v[6] & 0xFFu) << 16) | ((v[7] & 0xFFu) << 24);
    } else {
        t.hhi = t.hlo;
        t.lhi = t.llo;
    }
    return t;
}

__device__ __forceinline__ void int_lookup(const IntTable &t, uint32_t sel, uint32_t &even, uint32_t &odd)
{
    const uint32_t rh = byte_perm(t.hhi, t.hlo, sel);
    const uint32_t rl = byte_perm(t.lhi, t.llo, sel);
    even = byte_perm(rh, rl, 0x06020400u);   // [rl.b0, rh.b0, rl.b2, rh.b2]
    odd = byte_perm(rh, rl, 0x07030501u);    // [rl.b1, rh.b1, rl.b3, rh.b3]
}

// The eight selectors of a 4-bit block, as whole nibbles (uniform baseline) ...
__device__ __forceinline__ void selectors4(const uint32_t (&w)[4], uint32_t sel[8])
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        sel[2 * i] = w[i] & 0x0F0F0F0Fu;
        sel[2 * i + 1] = (w[i] >> 4) & 0x0F0F0F0Fu;
    }
}

// ... and split into exponent selectors and sign masks (PoT): the exponent indexes the
// eight-entry byte table, the sign lands on bit 7 of each byte, where it is XOR-ed into
// the looked-up high byte (adding 0x8000 to a 16-bit word is flipping its top bit).
__device__ __forceinline__ void selectors4_pot(const uint32_t (&w)[4], uint32_t sel[8], uint32_t sgn[8])
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        sel[2 * i] = w[i] & 0x07070707u;
        sel[2 * i + 1] = (w[i] >> 4) & 0x07070707u;
        sgn[2 * i] = (w[i] << 4) & 0x80808080u;
        sgn[2 * i + 1] = w[i] & 0x80808080u;
    }
}

// ---------------------------------------------------------------------------
// Decoder: everything a fused kernel needs to turn the codes of one row of one
// 32-column block into fp16 pairs, for every (bits, PoT / uniform) combination.
//   set_group(scale, zero)  once per scale group: builds the group's table
//   set_block(w)            once per 32-column block: builds the eight selectors
//   get(m, even, odd)       selector m -> pairs (column 4m, 4m+1) and (4m+2, 4m+3)
// ---------------------------------------------------------------------------
template <int BITS, bool IS_INT>
struct Decoder;

template <int BITS>
struct Decoder<BITS, false> {
    static_assert(BITS == 2 || BITS == 3, "4-bit PoT has its own specialisation");
    PotTable t;
    uint32_t sel[8];
    __device__ __forceinline__ void set_group(uint32_t s, uint32_t) { t = pot_table<BITS>(s); }
    __device__ __forceinline__ void set_block(const uint32_t (&w)[BITS])
    {
        if (BITS == 3)
            selectors3(w[0], w[1], w[BITS - 1], sel);
        else
            selectors2(w[0], w[1], sel);
    }
    __device__ __forceinline__ void get(int m, uint32_t &even, uint32_t &odd) const { pot_lookup(t, sel[m], even, odd); }
};

template <>
struct Decoder<4, false> {
    PotTable t;          // high bytes for E = 0..3 / 4..7 of the positive sign
    uint32_t sel[8], sgn[8];
    __device__ __forceinline__ void set_group(uint32_t s, uint32_t)
    {
        const uint32_t rep = ((s >> 8) & 0xFFu) * 0x01010101u;
        t.lo = add_bytes(rep, 0x0C080400u);
        t.hi = add_bytes(rep, 0x1C181410u);
        const uint32_t sl = s & 0xFFu;
        t.low2 = sl | (sl << 16);
    }
    __device__ __forceinline__ void set_block(const uint32_t (&w)[4]) { selectors4_pot(w, sel, sgn); }
    __device__ __forceinline__ void get(int m, uint32_t &even, uint32_t &odd) const
    {
        const uint32_t r = byte_perm(t.hi, t.lo, sel[m]) ^ sgn[m];
        even = byte_perm(r, t.low2, 0x06000400u);
        odd = (r & 0xFF00FF00u) | t.low2;
    }
};

template <int BITS>
struct Decoder<BITS, true> {
    static_assert(BITS == 2 || BITS == 3, "4-bit uniform has its own specialisation");
    IntTable t;
    uint32_t sel[8];
    __device__ __forceinline__ void set_group(uint32_t s, uint32_t z) { t = int_table<BITS>(s, z); }
    __device__ __forceinline__ void set_block(const uint32_t (&w)[BITS])
    {
        if (BITS == 3)
            selectors3(w[0], w[1], w[BITS - 1], sel);
        else
            selectors2(w[0], w[1], sel);
    }
    __device__ __forceinline__ void get(int m, uint32_t &even, uint32_t &odd) const { int_lookup(t, sel[m], even, odd); }
};

// Sixteen levels do not fit the byte-permute tables: the 4-bit uniform path computes
// (q + Z) * S with packed fp16 arithmetic instead -- q is OR-ed into the mantissa of 1024.0,
// (1024 + q) + (Z - 1024) is exact, the product is rounded once (Sec. 4.1 Eq. (9)).
template <>
struct Decoder<4, true> {
    half2_t zm1024, s2;
    uint32_t sel[8];
    __device__ __forceinline__ void set_group(uint32_t s, uint32_t z)
    {
        const _Float16 S = __builtin_bit_cast(_Float16, (uint16_t)s);
        const _Float16 Z = __builtin_bit_cast(_Float16, (uint16_t)z) - (_Float16)1024.0f;
        s2 = half2_t{S, S};
        zm1024 = half2_t{Z, Z};
    }
    __device__ __forceinline__ void set_block(const uint32_t (&w)[4]) { selectors4(w, sel); }
    __device__ __forceinline__ void get(int m, uint32_t &even, uint32_t &odd) const
    {
        const uint32_t qe = (sel[m] & 0x00FF00FFu) | 0x64006400u;          // bytes 0 and 2
        const uint32_t qo = ((sel[m] >> 8) & 0x00FF00FFu) | 0x64006400u;   // bytes 1 and 3
        even = as_u32((as_half2(qe) + zm1024) * s2);
        odd = as_u32((as_half2(qo) + zm1024) * s2);
    }
};

}  // namespace potq
