// Fused de-quantise + GEMV in the exponent form of the PoT product, gfx950.
//
// A power-of-two weight only shifts the exponent of the activation it meets
// (Sec. 4.2, the additivity of exponents), so the group's scale can stay out
// of the inner loop and be applied once per group to the partial sum:
//     y[n] = sum_g s[n,g] * sum_{k in g} (+-2^E[n,k]) x[k].
// The inner sums are integer work.  +-2^E is a signed byte, one v_perm_b32
// look-up per four codes in a table that is the same for every group (no
// per-group table, no merge with the scale's low byte: the vector ALU, the
// scarce unit of the fp16 GEMV, does about 40 % less).  The activations are
// turned, once per workgroup, into 32-bit fixed point -- every scale group
// against the largest exponent among its own 128 activations -- and cut into
// four signed 8-bit digits, x = 2^-k sum_p 256^p d_p;
// digit sums run on the matrix pipe (v_mfma_i32_16x16x64_i8, exact).  The
// digits of the four groups a wavefront works on sit block-diagonally in the A
// operand -- row 4q + p holds digit p of the group of lane group q in k-slice q
// and zeros elsewhere -- so lane (r, q) receives the four digit sums of row r
// of its own group, recombines them and multiplies by its own scale.
//
// Exactness: every fp16 activation within 2^19 of the largest one of its group
// is represented exactly (smaller ones are rounded to 2^-30 of that largest
// one); the digit sums are exact; one fp32 rounding per group in the recombination and
// one in the accumulation, as many as the fp16 form has per four MFMA steps.
// The scale must lie in the domain on which the integer add of Sec. 4.2 is the
// multiplication by 2^E (every scale pot_quantize produces does).
#include <type_traits>

#include "potq_device.hpp"
#include "potq_launch.hpp"

namespace potq {

constexpr int kExpSplit = 8;          // wavefronts that share one 16-row tile and split its scale groups
constexpr int kPieceRun = 9;          // uint4 per (group, digit) in LDS: 128 bytes + 16 of padding
constexpr int kExpOctetsPerThread = 4;   // x octets a thread stages: K <= 4 * 8 * (threads of the workgroup)

typedef int int4_t __attribute__((ext_vector_type(4)));
typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));

template <int BITS>
struct ExpDecoder {
    static_assert(BITS == 2 || BITS == 3, "+-2^E must fit a signed byte");
    // the signed bytes +-2^E by code (sign in the code's top bit)
    static constexpr uint32_t lo = BITS == 2 ? 0xFEFF0201u : 0x08040201u;
    static constexpr uint32_t hi = BITS == 2 ? 0xFEFF0201u : 0xF8FCFEFFu;
    uint32_t sel[8];
    __device__ __forceinline__ void set_block(const uint32_t (&w)[BITS])
    {
        if constexpr (BITS == 3)
            selectors3(w[0], w[1], w[2], sel);
        else
            selectors2(w[0], w[1], sel);
    }
    // selector m -> the four weights of columns 4m + (0, 2, 1, 3) of the block
    __device__ __forceinline__ uint32_t get(int m) const { return byte_perm(hi, lo, sel[m]); }
};

// Eight 16-byte LDS reads by the lanes of `lanes` only, which leave the registers of the other
// lanes untouched: the off-diagonal lanes of the A operand hold zeros, written once, and never
// read LDS.  The compiler does not count these reads, so lds_wait() stands between them and
// their first use.  They overwrite registers that the MFMAs of the previous round read, and the
// compiler sees neither that nor the hazards of the instructions inside the block: an MFMA that
// has been issued may not have read its operands yet (re-reading the registers right after
// issuing the MFMAs gave wrong results).  `after` is a value computed from the results of those
// MFMAs (the running row sum): as an input of the block it keeps every instruction that produces
// it -- the MFMAs, which by then have long read their operands, and the recombination of their
// results -- ahead of the reads.  The block also changes SCC (s_and_b64).
typedef __attribute__((address_space(3))) u32x4 lds_u32x4;
__device__ __forceinline__ void lds_read_keep(u32x4 (&xa)[8], uint32_t lds_byte_address, uint64_t lanes, float after)
{
    uint64_t saved;
    asm volatile("s_mov_b64 %[saved], exec\n\t"
                 "s_and_b64 exec, exec, %[lanes]\n\t"
                 "ds_read_b128 %[x0], %[at]\n\t"
                 "ds_read_b128 %[x1], %[at] offset:16\n\t"
                 "ds_read_b128 %[x2], %[at] offset:32\n\t"
                 "ds_read_b128 %[x3], %[at] offset:48\n\t"
                 "ds_read_b128 %[x4], %[at] offset:64\n\t"
                 "ds_read_b128 %[x5], %[at] offset:80\n\t"
                 "ds_read_b128 %[x6], %[at] offset:96\n\t"
                 "ds_read_b128 %[x7], %[at] offset:112\n\t"
                 "s_mov_b64 exec, %[saved]"
                 : [x0] "+v"(xa[0]), [x1] "+v"(xa[1]), [x2] "+v"(xa[2]), [x3] "+v"(xa[3]), [x4] "+v"(xa[4]),
                   [x5] "+v"(xa[5]), [x6] "+v"(xa[6]), [x7] "+v"(xa[7]), [saved] "=&s"(saved)
                 : [at] "v"(lds_byte_address), [lanes] "s"(lanes), [after] "v"(after)
                 : "scc");
}
__device__ __forceinline__ void lds_wait(u32x4 (&xa)[8])
{
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(xa[0]), "+v"(xa[1]), "+v"(xa[2]), "+v"(xa[3]), "+v"(xa[4]), "+v"(xa[5]), "+v"(xa[6]), "+v"(xa[7]));
}

// Blocks b0 .. b1-1 (32 columns each) of one group of one row against the lane's A operand
// (xa[2b + h]: digit bytes of columns 32b + 16h .. + 15, in selector order).
template <int BITS>
__device__ __forceinline__ void exp_blocks(const u32x4 (&L)[BITS], const u32x4 (&xa)[8], int b0, int b1, int4_t &d)
{
    ExpDecoder<BITS> dec;
#pragma unroll
    for (int b = b0; b < b1; ++b) {
        uint32_t w[BITS];
#pragma unroll
        for (int j = 0; j < BITS; ++j) w[j] = L[j][b];
        dec.set_block(w);
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const u32x4 wt{dec.get(4 * h), dec.get(4 * h + 1), dec.get(4 * h + 2), dec.get(4 * h + 3)};
            d = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(int4_t, xa[2 * b + h]),
                                                      __builtin_bit_cast(int4_t, wt), d, 0, 0, 0);
        }
    }
}

// The four digit sums of a group -> the group's sum in units of 2^-k, as fp32.
__device__ __forceinline__ float exp_recombine(const int4_t d)
{
    const int hi = d[3] * 256 + d[2];               // |d_p| <= 128 * 8 * 128
    const int lo = d[1] * 256 + d[0];
    return __builtin_fmaf((float)hi, 65536.f, (float)lo);
}

// Activations with an infinity or a NaN among them have no fixed-point form.  Their products are
// taken one by one in binary32 instead: (+-2^E) * x[k] is exact, an infinity keeps the sign the
// weight gives it, a NaN stays one, so a row whose infinite terms agree in sign comes out as that
// infinity and any other as NaN, which is what the definition of the product gives; the finite
// activations add finite amounts that do not matter next to them.  Blocks b0 .. b1-1 of one
// group of one row against xg[0 .. 127], the fp16 activations of that group.  Speed is no concern.
template <int BITS>
__device__ __forceinline__ float exp_blocks_plain(const u32x4 (&L)[BITS], const uint16_t *__restrict__ xg, int b0, int b1)
{
    ExpDecoder<BITS> dec;
    float sum = 0.f;
#pragma unroll 1
    for (int b = b0; b < b1; ++b) {
        uint32_t w[BITS];
#pragma unroll
        for (int j = 0; j < BITS; ++j) w[j] = b == 0 ? L[j][0] : b == 1 ? L[j][1] : b == 2 ? L[j][2] : L[j][3];
        dec.set_block(w);
#pragma unroll
        for (int m = 0; m < 8; ++m) {
            const uint32_t wt = dec.get(m);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int column = 32 * b + 4 * m + ((j & 1) << 1) + (j >> 1);     // byte j of a selector: column (0, 2, 1, 3)[j]
                const float wv = (float)(int)(int8_t)(wt >> (8 * j));
                sum = __builtin_fmaf(wv, (float)__builtin_bit_cast(_Float16, xg[column]), sum);
            }
        }
    }
    return sum;
}

// The largest of a value over the 16 lanes of a row (lanes 16j .. 16j+15), in every lane of the
// row: four data-parallel-primitive steps on the vector ALU (lane pairs, quads, the two quads
// of a half row, the two half rows), no trip through the LDS crossbar.
__device__ __forceinline__ uint32_t row_max_u32(uint32_t v)
{
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, true));    // quad_perm [1,0,3,2]
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, true));    // quad_perm [2,3,0,1]
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xF, 0xF, true));   // row_half_mirror
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xF, 0xF, true));   // row_mirror
    return v;
}

// Eight fp16 activations (columns 8i .. 8i+7) -> fixed point m = rne(x * 2^k), each m cut into
// four signed digits (m + 0x00808080 makes the three low bytes excess-128), the digits stored
// per digit plane in the order the selectors deliver the weights: (c0, c2, c1, c3, c4, c6, c5, c7).
__device__ __forceinline__ void stage_digits(const u32x4 xv, u32x4 *__restrict__ pieces, int i, float two_k)
{
    const int g = i >> 4, at = i & 15;              // group, octet inside the group
    uint32_t u[8];
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const half2_t h = as_half2(xv[w]);
        u[2 * w] = (uint32_t)(int)__builtin_rintf((float)h[0] * two_k) + 0x00808080u;
        u[2 * w + 1] = (uint32_t)(int)__builtin_rintf((float)h[1] * two_k) + 0x00808080u;
    }
    uint32_t plane[4][2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const uint32_t a = u[4 * q], b = u[4 * q + 1], c = u[4 * q + 2], d = u[4 * q + 3];
        const uint32_t ac_lo = byte_perm(c, a, 0x05010400u);     // a.0 c.0 a.1 c.1
        const uint32_t ac_hi = byte_perm(c, a, 0x07030602u);     // a.2 c.2 a.3 c.3
        const uint32_t bd_lo = byte_perm(d, b, 0x05010400u);
        const uint32_t bd_hi = byte_perm(d, b, 0x07030602u);
        plane[0][q] = byte_perm(bd_lo, ac_lo, 0x05040100u) ^ 0x80808080u;   // a.0 c.0 b.0 d.0
        plane[1][q] = byte_perm(bd_lo, ac_lo, 0x07060302u) ^ 0x80808080u;
        plane[2][q] = byte_perm(bd_hi, ac_hi, 0x05040100u) ^ 0x80808080u;
        plane[3][q] = byte_perm(bd_hi, ac_hi, 0x07060302u);                 // top digit: two's complement as is
    }
#pragma unroll
    for (int p = 0; p < 4; ++p) ((u32x2 *)(pieces + (g * 4 + p) * kPieceRun))[at] = u32x2{plane[p][0], plane[p][1]};
}

// A workgroup of WAVES wavefronts stages the digits of x once and serves, WAVES / 8 at a time,
// the row tiles (first + i * stride) * (WAVES / 8) + slot below rowtiles.  The eight wavefronts
// of a slot split the scale groups of its tile (wavefront p, lane group t: groups 4p + t,
// 4p + t + 32, ...).  The codes of the next step -- the next round of the tile or the first round
// of the next tile -- are requested before the current ones are expanded (requests two or three
// steps ahead measured slower); the very first request goes out right after the request for x,
// before x is converted.
template <int BITS, bool G64, int WAVES>
__device__ __forceinline__ void gemv_exp_body(const u32x4 *__restrict__ codes, const uint16_t *__restrict__ scales,
                                              const u32x4 *__restrict__ x, uint16_t *__restrict__ y, int K,
                                              int64_t rowtiles, int64_t first, int64_t stride)
{
    constexpr int gs = G64 ? 1 : 0;
    constexpr int kStep = 4 * kExpSplit;                // groups per round of a slot
    constexpr int SLOTS = WAVES / kExpSplit;
    static_assert(WAVES % kExpSplit == 0, "whole slots");
    extern __shared__ u32x4 smem[];
    const int G = K / kTileCols;
    u32x4 *pieces = smem;                               // [group][digit] runs of kPieceRun uint4
    u32x4 *zero_block = smem + G * 4 * kPieceRun;       // 8 uint4 of zeros
    float *red = (float *)(zero_block + 8);             // 2 x WAVES x 16 partial sums
    uint32_t *nonfinite_part = (uint32_t *)(red + 2 * WAVES * kTileRows);   // per wavefront: saw an infinity or NaN
    float *group_unit = (float *)(nonfinite_part + WAVES);                  // per scale group: 2^-k of its fixed point

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform, kept in a scalar
    const int part = wave % kExpSplit;
    const int slot = wave / kExpSplit;
    const int r = lane & 15;
    const int t = lane >> 4;
    const int scale_owner = (4 * r + t) * 4;            // ds_bpermute byte address
    // rounds in which this wavefront has a group (G >= 32: at least one)
    const int my_rounds = (G - part * 4 + kStep - 1) / kStep;
    // tile of this slot in tile set q; a slot past the last tile works on the last one and stores nothing
    auto tile_of = [&](int64_t q) { return min(q * SLOTS + slot, rowtiles - 1); };

    // Codes of (tile, round) for lane (r, t); scales in memory order (lane l: row l/4, group
    // first + l%4; handed to their owners by a permute) or, for group size 64, the lane's own pair.
    // Indices past the end of the row are clamped into it: valid memory, multiplied by zeros.
    // Every step requests the codes of the next one; the wavefront's last step, which has none
    // to request, is taken out of the loop (see `step` below).
    auto fetch = [&](int64_t tile, int round, u32x4 (&Lx)[BITS], uint32_t &sx) {
        const int g0 = round * kStep + part * 4;                        // uniform
        const int gc = min(g0 + t, G - 1);
        const u32x4 *tile_codes = codes + tile * G * (BITS * 16);       // uniform
        const uint32_t at = (uint32_t)(gc * (BITS * 16) + r);
#pragma unroll
        for (int j = 0; j < BITS; ++j) Lx[j] = __builtin_nontemporal_load(tile_codes + at + 16 * j);
        if (gs) {
            const uint32_t *tile_scales = (const uint32_t *)(scales + tile * kTileRows * (int64_t)(2 * G));
            sx = tile_scales[(uint32_t)(r * G + gc)];
        } else {
            const uint16_t *tile_scales = scales + tile * kTileRows * (int64_t)G;
            sx = tile_scales[(uint32_t)((lane >> 2) * G + min(g0 + (lane & 3), G - 1))];
        }
    };

    // The steps of a wavefront are its (tile set, round) pairs in order.  `fq`/`fround` is the
    // step of the next request and `more` tells whether there is one.
    int64_t fq = first;
    int fround = 0;
    auto advance = [&]() -> bool {
        if (fround + 1 < my_rounds) {
            ++fround;
            return true;
        }
        if ((fq + stride) * SLOTS < rowtiles) {
            fq += stride;
            fround = 0;
            return true;
        }
        return false;
    };
    // x is requested before the codes of the first step: loads return in order, x comes from the
    // L2 and its conversion can run while the codes are on their way from HBM.
    const int octets = K / 8;
    u32x4 xin[kExpOctetsPerThread];
#pragma unroll
    for (int n = 0; n < kExpOctetsPerThread; ++n) {
        const int i = tid + n * (WAVES * kWave);
        xin[n] = i < octets ? x[i] : u32x4{0u, 0u, 0u, 0u};
    }
    u32x4 L[BITS];
    uint32_t s;
    fetch(tile_of(fq), fround, L, s);
    advance();

    // --- activations: fixed point digits into LDS, every scale group against its own largest exponent ---
    // The sixteen octets of a group sit in sixteen consecutive lanes, so the group's largest
    // exponent is four cross-lane steps away and nothing waits for the rest of the vector: one
    // barrier between the loads of x and the first MFMA (a common exponent for the whole vector
    // needs a second one, behind a reduction over the workgroup, which cost 5-12 % of the launch
    // on the 13B to 70B shapes).  |x| < 2^(e-14) with e = max(exponent field, 1): k = 44 - e puts
    // every |m| below 2^30; the group's sums are in units of 2^-k, kept per group in LDS.
    bool saw_nonfinite = false;
#pragma unroll
    for (int n = 0; n < kExpOctetsPerThread; ++n) {
        if (n * (WAVES * kWave) >= octets) break;       // uniform: no thread has an octet in this pass
        const int i = tid + n * (WAVES * kWave);
        const u32x4 xv = xin[n];
        uint32_t am = 0u;
#pragma unroll
        for (int w = 0; w < 4; ++w)
            am = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(ushort2_t, am),
                                                                        __builtin_bit_cast(ushort2_t, xv[w] & 0x7FFF7FFFu)));
        am = max(am & 0xFFFFu, am >> 16);
        am = row_max_u32(am);
        const int e = max((int)(am >> 10), 1);
        saw_nonfinite = saw_nonfinite || e == 31;
        const int k = 44 - e;
        if (i < octets) {
            stage_digits(xv, pieces, i, __builtin_bit_cast(float, (uint32_t)(k + 127) << 23));
            if ((i & 15) == 0) group_unit[i >> 4] = __builtin_bit_cast(float, (uint32_t)(127 - k) << 23);
        }
    }
    const bool wave_saw_nonfinite = __builtin_amdgcn_ballot_w64(saw_nonfinite) != 0;
    if (lane == 0) nonfinite_part[wave] = wave_saw_nonfinite ? 1u : 0u;
    if (tid < 8) zero_block[tid] = u32x4{0u, 0u, 0u, 0u};
    __syncthreads();
    uint32_t nonfinite = 0u;
#pragma unroll
    for (int p = 0; p < WAVES; ++p) nonfinite |= nonfinite_part[p];

    // lane (r, t) holds the groups of lane group t of row r: add the lane groups, then the
    // wavefronts of the slot, in a fixed order.  The buffer alternates between tile sets, so one
    // barrier per set separates the writes of set i + 2 from the reads of set i.
    auto finish_tiles = [&](int64_t q, int it, float row_sum) {
        float *red_it = red + (it & 1) * (WAVES * kTileRows);
        row_sum += __shfl_xor(row_sum, 16, kWave);
        row_sum += __shfl_xor(row_sum, 32, kWave);
        if (t == 0) red_it[wave * kTileRows + r] = row_sum;
        __syncthreads();
        if (tid < SLOTS * kTileRows) {
            const int of_slot = tid / kTileRows, row = tid % kTileRows;
            const int64_t tile = q * SLOTS + of_slot;
            float sum = 0.f;
#pragma unroll
            for (int p = 0; p < kExpSplit; ++p) sum += red_it[(of_slot * kExpSplit + p) * kTileRows + row];
            const _Float16 h = (_Float16)sum;
            if (tile < rowtiles) y[tile * kTileRows + row] = __builtin_bit_cast(uint16_t, h);
        }
    };

    // An infinity or NaN among the activations (the same for every workgroup of the launch):
    // plain binary32 products, same tiles, same reduction.
    if (nonfinite) {
        int it = 0;
        for (int64_t q = first; q * SLOTS < rowtiles; q += stride, ++it) {
            float row_sum = 0.f;
            for (int round = 0; round < my_rounds; ++round) {
                u32x4 Lp[BITS];
                uint32_t sp;
                fetch(tile_of(q), round, Lp, sp);
                const int g = round * kStep + part * 4 + t;
                const uint16_t *xg = (const uint16_t *)x + (size_t)min(g, G - 1) * kTileCols;
                if (gs) {
                    const float v0 = exp_blocks_plain<BITS>(Lp, xg, 0, 2), v1 = exp_blocks_plain<BITS>(Lp, xg, 2, 4);
                    if (g < G) {      // a lane past the end of the row adds nothing (not even 0 * inf)
                        row_sum = __builtin_fmaf((float)__builtin_bit_cast(_Float16, (uint16_t)(sp & 0xFFFFu)), v0, row_sum);
                        row_sum = __builtin_fmaf((float)__builtin_bit_cast(_Float16, (uint16_t)(sp >> 16)), v1, row_sum);
                    }
                } else {
                    const uint32_t so = (uint32_t)__builtin_amdgcn_ds_bpermute(scale_owner, (int)sp);
                    const float v = exp_blocks_plain<BITS>(Lp, xg, 0, 4);
                    if (g < G) row_sum = __builtin_fmaf((float)__builtin_bit_cast(_Float16, (uint16_t)so), v, row_sum);
                }
            }
            finish_tiles(q, it, row_sum);
        }
        return;
    }

    // The A operand: lanes on the block diagonal carry digit (lane % 4) of their own group; the
    // others hold zeros from here on (lds_read_keep never writes them).
    const uint64_t diagonal_lanes = __builtin_amdgcn_ballot_w64((r >> 2) == t);
    u32x4 xa[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) xa[j] = u32x4{0u, 0u, 0u, 0u};
    const uint32_t pieces_at = (uint32_t)(uintptr_t)(lds_u32x4 *)pieces;
    const uint32_t zeros_at = (uint32_t)(uintptr_t)(lds_u32x4 *)zero_block;

    int it = 0;
    float consumed = 0.f;       // the latest value computed from MFMA results: orders lds_read_keep behind them
    // One step: the codes in L against the digits of the step's groups; `request` says whether the
    // codes of the next step are asked for first.  It is a compile-time choice: the loop below
    // takes the wavefront's very last step out of the steady state, which then neither tests for
    // it nor fetches anything twice.  (Fetching the last step's 3 KB once more instead cost 8 %
    // more HBM reads on 28672 x 8192; a test inside the loop, or a request redirected to a dummy
    // address, was scheduled worse by the compiler than the reads cost on tall matrices.  Peeled:
    // 13824 x 5120 8.8 -> 8.3 us, 8192 x 8192 7.6 -> 7.2, 28672 x 8192 16.7 -> 16.4, at 2 bits 14.7 -> 13.8.)
    auto step = [&](int round, auto request, float &row_sum) {
        u32x4 Ln[BITS];
        uint32_t sn = 0u;
        if constexpr (decltype(request)::value) {
            fetch(tile_of(fq), fround, Ln, sn);
            advance();
        }
        const int g = round * kStep + part * 4 + t;
        const float unit = group_unit[min(g, G - 1)];
        // a lane past the end of the row multiplies the (valid) last group by zeros
        lds_read_keep(xa, g < G ? pieces_at + (uint32_t)((g * 4 + (lane & 3)) * (kPieceRun * 16)) : zeros_at,
                      diagonal_lanes, consumed);
        if (gs) {
            lds_wait(xa);
            int4_t d0{0, 0, 0, 0}, d1{0, 0, 0, 0};
            exp_blocks<BITS>(L, xa, 0, 2, d0);
            exp_blocks<BITS>(L, xa, 2, 4, d1);
            // scale * 2^-k is exact (a power of two times an fp16, far inside binary32's range)
            row_sum = __builtin_fmaf((float)__builtin_bit_cast(_Float16, (uint16_t)(s & 0xFFFFu)) * unit,
                                     exp_recombine(d0), row_sum);
            row_sum = __builtin_fmaf((float)__builtin_bit_cast(_Float16, (uint16_t)(s >> 16)) * unit,
                                     exp_recombine(d1), row_sum);
        } else {
            const uint32_t so = (uint32_t)__builtin_amdgcn_ds_bpermute(scale_owner, (int)s);
            lds_wait(xa);
            int4_t d{0, 0, 0, 0};
            exp_blocks<BITS>(L, xa, 0, 4, d);
            row_sum = __builtin_fmaf((float)__builtin_bit_cast(_Float16, (uint16_t)so) * unit, exp_recombine(d), row_sum);
        }
        consumed = row_sum;
        if constexpr (decltype(request)::value) {
#pragma unroll
            for (int j = 0; j < BITS; ++j) L[j] = Ln[j];
            s = sn;
        }
    };
    for (int64_t q = first; q * SLOTS < rowtiles; q += stride, ++it) {
        float row_sum = 0.f;
        const bool last_set = (q + stride) * SLOTS >= rowtiles;
        const int requesting = last_set ? my_rounds - 1 : my_rounds;
        for (int round = 0; round < requesting; ++round) step(round, std::true_type{}, row_sum);
        if (last_set) step(my_rounds - 1, std::false_type{}, row_sum);
        finish_tiles(q, it, row_sum);
    }
}

template <int BITS, bool G64, int WAVES>
__global__ __launch_bounds__(WAVES * kWave) void gemv_exp_kernel(
    const u32x4 *__restrict__ codes, const uint16_t *__restrict__ scales, const u32x4 *__restrict__ x,
    uint16_t *__restrict__ y, int K, int64_t rowtiles)
{
    gemv_exp_body<BITS, G64, WAVES>(codes, scales, x, y, K, rowtiles, blockIdx.x, gridDim.x);
}

// ---------------------------------------------------------------------------
// Two to four activation vectors at once (a GEMM with two to four tokens), group size 128:
// the matrix is decoded once per step and every vector costs one more MFMA per step and its
// own digit planes in LDS (its own fixed-point exponent per scale group).  Here all lanes read
// LDS -- the off-diagonal ones a block of zeros -- so the A operands need no registers of their
// own between steps.  Vectors past `tokens` count as zero.  Results y[m * ystride + n].
// ---------------------------------------------------------------------------
template <int BITS, int WAVES, int MT>
__global__ __launch_bounds__(WAVES * kWave) void gemv_exp_multi_kernel(
    const u32x4 *__restrict__ codes, const uint16_t *__restrict__ scales, const u32x4 *__restrict__ x,
    uint16_t *__restrict__ y, int K, int64_t rowtiles, int tokens, int64_t ystride)
{
    constexpr int kStep = 4 * kExpSplit;
    constexpr int SLOTS = WAVES / kExpSplit;
    constexpr int THREADS = WAVES * kWave;
    extern __shared__ u32x4 smem[];
    const int G = K / kTileCols;
    u32x4 *pieces = smem;                               // [vector][group][digit] runs of kPieceRun uint4
    u32x4 *zero_block = smem + MT * G * 4 * kPieceRun;  // 8 uint4 of zeros
    float *red = (float *)(zero_block + 8);             // 2 x WAVES x MT x 16 partial sums
    uint32_t *nonfinite_part = (uint32_t *)(red + 2 * WAVES * MT * kTileRows);   // per wavefront: saw an infinity or NaN
    float *group_unit = (float *)(nonfinite_part + WAVES);                        // [vector][group]: 2^-k of its fixed point

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int part = wave % kExpSplit;
    const int slot = wave / kExpSplit;
    const int r = lane & 15;
    const int t = lane >> 4;
    const int scale_owner = (4 * r + t) * 4;
    const int my_rounds = (G - part * 4 + kStep - 1) / kStep;
    const int64_t first = blockIdx.x, stride = gridDim.x;
    auto tile_of = [&](int64_t q) { return min(q * SLOTS + slot, rowtiles - 1); };

    auto fetch = [&](int64_t tile, int round, u32x4 (&Lx)[BITS], uint32_t &sx) {   // as in gemv_exp_body
        const int g0 = round * kStep + part * 4;
        const int gc = min(g0 + t, G - 1);
        const u32x4 *tile_codes = codes + tile * G * (BITS * 16);
        const uint32_t at = (uint32_t)(gc * (BITS * 16) + r);
#pragma unroll
        for (int j = 0; j < BITS; ++j) Lx[j] = __builtin_nontemporal_load(tile_codes + at + 16 * j);
        const uint16_t *tile_scales = scales + tile * kTileRows * (int64_t)G;
        sx = tile_scales[(uint32_t)((lane >> 2) * G + min(g0 + (lane & 3), G - 1))];
    };
    int64_t fq = first;
    int fround = 0;
    auto advance = [&]() -> bool {
        if (fround + 1 < my_rounds) {
            ++fround;
            return true;
        }
        if ((fq + stride) * SLOTS < rowtiles) {
            fq += stride;
            fround = 0;
            return true;
        }
        return false;
    };
    // x before the codes of the first step, as in gemv_exp_body
    const int per = K / 8;                              // octets per vector
    const int octets = MT * per;
    u32x4 xin[kExpOctetsPerThread];
#pragma unroll
    for (int n = 0; n < kExpOctetsPerThread; ++n) {
        const int i = tid + n * THREADS;
        xin[n] = (i < octets && i / per < tokens) ? x[i] : u32x4{0u, 0u, 0u, 0u};
    }
    u32x4 L[BITS];
    uint32_t s;
    fetch(tile_of(fq), fround, L, s);
    advance();

    // --- activations: fixed point digits into LDS, every scale group of every vector against its
    // own largest exponent (see gemv_exp_body: the sixteen lanes of a row hold one group) ---
    bool saw_nonfinite = false;
#pragma unroll
    for (int n = 0; n < kExpOctetsPerThread; ++n) {
        if (n * THREADS >= octets) break;               // uniform: no thread has an octet in this pass
        const int i = tid + n * THREADS;
        const int vec = i / per, o = i - vec * per;     // vector, octet inside the vector
        const u32x4 xv = xin[n];
        uint32_t a = 0u;
#pragma unroll
        for (int w = 0; w < 4; ++w)
            a = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(ushort2_t, a),
                                                                       __builtin_bit_cast(ushort2_t, xv[w] & 0x7FFF7FFFu)));
        a = row_max_u32(max(a & 0xFFFFu, a >> 16));
        const int e = max((int)(a >> 10), 1);
        saw_nonfinite = saw_nonfinite || e == 31;
        const int k = 44 - e;
        if (i < octets) {
            stage_digits(xv, pieces + vec * G * 4 * kPieceRun, o, __builtin_bit_cast(float, (uint32_t)(k + 127) << 23));
            if ((o & 15) == 0) group_unit[vec * G + (o >> 4)] = __builtin_bit_cast(float, (uint32_t)(127 - k) << 23);
        }
    }
    const bool wave_saw_nonfinite = __builtin_amdgcn_ballot_w64(saw_nonfinite) != 0;
    if (lane == 0) nonfinite_part[wave] = wave_saw_nonfinite ? 1u : 0u;
    if (tid < 8) zero_block[tid] = u32x4{0u, 0u, 0u, 0u};
    __syncthreads();
    uint32_t non_finite = 0u;
#pragma unroll
    for (int p = 0; p < WAVES; ++p) non_finite |= nonfinite_part[p];

    auto finish_tiles = [&](int64_t q, int it, const float (&row_sum)[MT]) {
        float *red_it = red + (it & 1) * (WAVES * MT * kTileRows);
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            float v = row_sum[m];
            v += __shfl_xor(v, 16, kWave);
            v += __shfl_xor(v, 32, kWave);
            if (t == 0) red_it[(wave * MT + m) * kTileRows + r] = v;
        }
        __syncthreads();
        if (tid < SLOTS * MT * kTileRows) {
            const int of_slot = tid / (MT * kTileRows), m = (tid / kTileRows) % MT, row = tid % kTileRows;
            const int64_t tile = q * SLOTS + of_slot;
            float sum = 0.f;
#pragma unroll
            for (int p = 0; p < kExpSplit; ++p) sum += red_it[((of_slot * kExpSplit + p) * MT + m) * kTileRows + row];
            const _Float16 h = (_Float16)sum;
            if (tile < rowtiles && m < tokens) y[m * ystride + tile * kTileRows + row] = __builtin_bit_cast(uint16_t, h);
        }
    };

    // An infinity or NaN in any of the vectors (the same for every workgroup of the launch): all
    // vectors take plain binary32 products (see exp_blocks_plain), same tiles, same reduction.
    if (non_finite) {
        int it = 0;
        for (int64_t q = first; q * SLOTS < rowtiles; q += stride, ++it) {
            float row_sum[MT];
#pragma unroll
            for (int m = 0; m < MT; ++m) row_sum[m] = 0.f;
            for (int round = 0; round < my_rounds; ++round) {
                u32x4 Lp[BITS];
                uint32_t sp;
                fetch(tile_of(q), round, Lp, sp);
                const int g = round * kStep + part * 4 + t;
                const float sf = (float)__builtin_bit_cast(_Float16, (uint16_t)__builtin_amdgcn_ds_bpermute(scale_owner, (int)sp));
#pragma unroll 1
                for (int m = 0; m < MT; ++m) {
                    if (m >= tokens) break;
                    const uint16_t *xg = (const uint16_t *)x + (size_t)m * K + (size_t)min(g, G - 1) * kTileCols;
                    const float v = exp_blocks_plain<BITS>(Lp, xg, 0, 4);
                    float add = __builtin_fmaf(sf, v, 0.f);
#pragma unroll
                    for (int mm = 0; mm < MT; ++mm)
                        if (mm == m && g < G) row_sum[mm] += add;
                }
            }
            finish_tiles(q, it, row_sum);
        }
        return;
    }

    const bool diagonal = (r >> 2) == t;
    int it = 0;
    for (int64_t q = first; q * SLOTS < rowtiles; q += stride, ++it) {
        float row_sum[MT];
#pragma unroll
        for (int m = 0; m < MT; ++m) row_sum[m] = 0.f;
        // as in gemv_exp_body: the wavefront's last step, which has no successor to request, is
        // taken out of the steady-state loop
        auto step = [&](int round, auto request) {
            u32x4 Ln[BITS];
            uint32_t sn = 0u;
            if constexpr (decltype(request)::value) {
                fetch(tile_of(fq), fround, Ln, sn);
                advance();
            }
            const int g = round * kStep + part * 4 + t;
            const bool mine = diagonal && g < G;
            const u32x4 *xq[MT];
#pragma unroll
            for (int m = 0; m < MT; ++m)
                xq[m] = mine ? pieces + ((m * G + g) * 4 + (lane & 3)) * kPieceRun : zero_block;
            const uint32_t so = (uint32_t)__builtin_amdgcn_ds_bpermute(scale_owner, (int)s);
            int4_t d[MT];
#pragma unroll
            for (int m = 0; m < MT; ++m) d[m] = int4_t{0, 0, 0, 0};
            ExpDecoder<BITS> dec;
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                uint32_t w[BITS];
#pragma unroll
                for (int j = 0; j < BITS; ++j) w[j] = L[j][b];
                dec.set_block(w);
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const u32x4 wt{dec.get(4 * h), dec.get(4 * h + 1), dec.get(4 * h + 2), dec.get(4 * h + 3)};
#pragma unroll
                    for (int m = 0; m < MT; ++m)
                        d[m] = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(int4_t, xq[m][2 * b + h]),
                                                                     __builtin_bit_cast(int4_t, wt), d[m], 0, 0, 0);
                }
            }
            const float sf = (float)__builtin_bit_cast(_Float16, (uint16_t)so);
#pragma unroll
            for (int m = 0; m < MT; ++m)     // scale * 2^-k is exact
                row_sum[m] = __builtin_fmaf(sf * group_unit[m * G + min(g, G - 1)], exp_recombine(d[m]), row_sum[m]);
            if constexpr (decltype(request)::value) {
#pragma unroll
                for (int j = 0; j < BITS; ++j) L[j] = Ln[j];
                s = sn;
            }
        };
        const bool last_set = (q + stride) * SLOTS >= rowtiles;
        const int requesting = last_set ? my_rounds - 1 : my_rounds;
        for (int round = 0; round < requesting; ++round) step(round, std::true_type{});
        if (last_set) step(my_rounds - 1, std::false_type{});
        finish_tiles(q, it, row_sum);
    }
}

// Several matrices that consume the same activation vector in one launch: a workgroup belongs
// to one matrix and walks that matrix's tiles as in the single launch.
constexpr int kMaxExpBatch = 16;
struct ExpBatch {
    const u32x4 *codes[kMaxExpBatch];
    const uint16_t *scales[kMaxExpBatch];
    uint16_t *y[kMaxExpBatch];
    int64_t rowtiles[kMaxExpBatch];
    uint32_t first_block[kMaxExpBatch + 1];   // workgroups first_block[i] .. first_block[i+1]-1 serve matrix i
    int count;
};

template <int BITS, bool G64, int WAVES>
__global__ __launch_bounds__(WAVES * kWave) void gemv_exp_batch_kernel(const ExpBatch batch,
                                                                       const u32x4 *__restrict__ x, int K)
{
    int i = 0;
    while (i + 1 < batch.count && blockIdx.x >= batch.first_block[i + 1]) ++i;   // uniform: scalar code
    gemv_exp_body<BITS, G64, WAVES>(batch.codes[i], batch.scales[i], x, batch.y[i], K, batch.rowtiles[i],
                                    blockIdx.x - batch.first_block[i],
                                    batch.first_block[i + 1] - batch.first_block[i]);
}

static size_t exp_lds_bytes(int64_t K, int waves)
{
    return (size_t)(K / kTileCols) * 4 * kPieceRun * 16 + 8 * 16 + 2 * (size_t)waves * kTileRows * sizeof(float) +
           (size_t)waves * sizeof(uint32_t) + (size_t)(K / kTileCols) * sizeof(float);
}

// Workgroups per launch: what the chip holds at once (two per compute unit at this register
// and LDS footprint), each with an equal share of the row tiles, so that x is staged as few
// times as possible and nobody waits for a second wave of workgroups.
constexpr int kExpGroups = 512;
constexpr int64_t kExpMinWeights = 60ll << 20;
constexpr size_t kExpLdsSmall = kLdsDefaultLimit, kExpLdsLarge = kLdsPerWorkgroup;

// Wavefronts per workgroup.  A single matrix always takes sixteen (two tiles at a time, one
// workgroup per compute unit): x is converted once per compute unit instead of twice, which
// measured 3-8 % faster than two workgroups of eight on every eligible shape (28672 x 8192:
// 17.4 against 17.9 us, 5120 x 13824: 10.2 against 11.1 us).  Matrices sharing x keep eight
// while two workgroups' digits of x fit the LDS of a compute unit together (no consistent
// difference there, and small members of a batch get a finer share of the workgroups).
static int exp_waves(int64_t K, bool batch) { return batch && exp_lds_bytes(K, 8) <= kExpLdsSmall ? 8 : 16; }

// Whether the exponent form can serve a PoT GEMV at all: signed-byte weights (2 or 3 bits), rows
// long enough for eight wavefronts per tile, the digits of x within LDS and within the staging
// registers of a thread.
static bool exp_form_fits(int64_t K, int bits)
{
    const int64_t G = K / kTileCols;
    if (bits != 2 && bits != 3) return false;
    if (G < 32) return false;
    // (the eight-wavefront variant is only used where its footprint is smaller still)
    if (K > (int64_t)kExpOctetsPerThread * 16 * kWave * 8) return false;
    return exp_lds_bytes(K, 16) <= kExpLdsLarge;
}

// Whether it pays for a single matrix: the conversion of x has to be won back by the cheaper
// decode.  From about 60 M weights up it always is (28672 x 8192: 22 us in the fp16 form against
// 15.7 us).  Below, down to 24 M, it is where there are rows for 160 workgroups (kernel times:
// 6144 x 4096 4.95 against 5.44 us, 8192 x 4096 5.17 against 5.86, 11008 x 4096 6.13 against
// 6.51, 5120 x 5120 5.1 against 6.0); matrices with few rows (4096 x 11008: 7.12 against
// 6.74 us, 4096 x 8192: 6.02 against 5.76, 1024 x 8192: 5.78 against 4.97) and the smaller ones
// (4096 x 4096: 4.72 against 4.43 us) stay on the fp16 form.
constexpr int64_t kExpMinWeightsManyRows = 24ll << 20, kExpManyRows = 5120;
bool gemv_exp_ok(int64_t N, int64_t K, int bits)
{
    if (!exp_form_fits(K, bits)) return false;
    return N * K >= kExpMinWeights || (N * K >= kExpMinWeightsManyRows && N >= kExpManyRows);
}

// Matrices that share x (N = the sum of their rows): x is converted once for all of them and the
// eight-wavefront workgroups of the batch kernel split small matrices finely, so the exponent
// form won on every batch tried, down to two matrices of 512 rows (kernel times, fp16 form
// against exponent form: 3 x 4096 x 4096 7.22 / 6.88 us, 2 x 2048 x 4096 4.74 / 4.37,
// 2 x 1024 x 8192 5.73 / 5.29, 3 x 1024 x 4096 4.30 / 3.91, 2 x 512 x 4096 4.23 / 3.94).
bool gemv_exp_batch_ok(int count, int64_t rows_total, int64_t K, int bits)
{
    (void)rows_total;
    return count <= kMaxExpBatch && exp_form_fits(K, bits);
}

template <int BITS, bool G64, int WAVES, bool BATCH>
static hipError_t exp_allow_lds(size_t lds)
{
    static std::atomic<uint64_t> raised{0};           // one flag word per kernel instantiation
    if constexpr (BATCH)
        return allow_large_lds((const void *)gemv_exp_batch_kernel<BITS, G64, WAVES>, lds, raised);
    else
        return allow_large_lds((const void *)gemv_exp_kernel<BITS, G64, WAVES>, lds, raised);
}

// Workgroups for a matrix of `sets` tile sets when it may use `cap` of them: equal shares of sets.
static int64_t exp_groups(int64_t sets, int64_t cap)
{
    if (cap < 1) cap = 1;
    const int64_t per_group = (sets + cap - 1) / cap;
    return (sets + per_group - 1) / per_group;
}

template <int BITS, bool G64, int WAVES>
static hipError_t launch_exp(const void *codes, const void *scales, const void *x, void *y, int64_t N, int64_t K,
                             hipStream_t stream)
{
    const size_t lds = exp_lds_bytes(K, WAVES);
    const hipError_t e = exp_allow_lds<BITS, G64, WAVES, false>(lds);
    if (e != hipSuccess) return e;
    constexpr int SLOTS = WAVES / kExpSplit;
    const int64_t rowtiles = N / kTileRows;
    const dim3 grid((unsigned)exp_groups((rowtiles + SLOTS - 1) / SLOTS, kExpGroups / SLOTS)), block(WAVES * kWave);
    hipLaunchKernelGGL((gemv_exp_kernel<BITS, G64, WAVES>), grid, block, lds, stream, (const u32x4 *)codes,
                       (const uint16_t *)scales, (const u32x4 *)x, (uint16_t *)y, (int)K, rowtiles);
    return hipGetLastError();
}

hipError_t run_gemv_exp(const void *codes, const void *scales, const void *x, void *y, int64_t N, int64_t K, int bits,
                        int group, hipStream_t stream)
{
    constexpr int WAVES = 16;
    if (group == 64)
        return bits == 3 ? launch_exp<3, true, WAVES>(codes, scales, x, y, N, K, stream)
                         : launch_exp<2, true, WAVES>(codes, scales, x, y, N, K, stream);
    return bits == 3 ? launch_exp<3, false, WAVES>(codes, scales, x, y, N, K, stream)
                     : launch_exp<2, false, WAVES>(codes, scales, x, y, N, K, stream);
}


template <int BITS, bool G64, int WAVES>
static hipError_t launch_exp_batch(int count, const void *const *codes, const void *const *scales, void *const *y,
                                   const int64_t *N, const void *x, int64_t K, hipStream_t stream)
{
    const size_t lds = exp_lds_bytes(K, WAVES);
    constexpr int SLOTS = WAVES / kExpSplit;
    int64_t sets_total = 0;
    for (int i = 0; i < count; ++i) sets_total += (N[i] / kTileRows + SLOTS - 1) / SLOTS;
    ExpBatch b;
    uint64_t blocks = 0;
    for (int i = 0; i < kMaxExpBatch; ++i) {
        const bool live = i < count;
        b.codes[i] = live ? (const u32x4 *)codes[i] : nullptr;
        b.scales[i] = live ? (const uint16_t *)scales[i] : nullptr;
        b.y[i] = live ? (uint16_t *)y[i] : nullptr;
        b.rowtiles[i] = live ? N[i] / kTileRows : 0;
        b.first_block[i] = (uint32_t)blocks;
        if (live) {
            // each matrix gets the share of the resident workgroups that its share of the tiles asks for
            const int64_t sets = (b.rowtiles[i] + SLOTS - 1) / SLOTS;
            const int64_t cap = (kExpGroups / SLOTS) * sets / sets_total;
            blocks += (uint64_t)exp_groups(sets, cap);
        }
    }
    b.first_block[kMaxExpBatch] = (uint32_t)blocks;
    b.count = count;
    const dim3 grid((unsigned)blocks), block(WAVES * kWave);
    const hipError_t e = exp_allow_lds<BITS, G64, WAVES, true>(lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((gemv_exp_batch_kernel<BITS, G64, WAVES>), grid, block, lds, stream, b, (const u32x4 *)x, (int)K);
    return hipGetLastError();
}

// `count` non-empty matrices (count <= kMaxExpBatch) that share x, K, bits and group.
hipError_t run_gemv_exp_batch(int count, const void *const *codes, const void *const *scales, void *const *y,
                              const int64_t *N, const void *x, int64_t K, int bits, int group, hipStream_t stream)
{
    const bool g64 = group == 64;
#define POTQ_LAUNCH_EXPB(BITS, WAVES)                                                             \
    (g64 ? launch_exp_batch<BITS, true, WAVES>(count, codes, scales, y, N, x, K, stream)          \
         : launch_exp_batch<BITS, false, WAVES>(count, codes, scales, y, N, x, K, stream))
    if (exp_waves(K, true) == 8) return bits == 3 ? POTQ_LAUNCH_EXPB(3, 8) : POTQ_LAUNCH_EXPB(2, 8);
    return bits == 3 ? POTQ_LAUNCH_EXPB(3, 16) : POTQ_LAUNCH_EXPB(2, 16);
#undef POTQ_LAUNCH_EXPB
}

// ---- two to four tokens ----
static size_t exp_multi_lds_bytes(int64_t K, int waves, int mt)
{
    return (size_t)mt * (K / kTileCols) * 4 * kPieceRun * 16 + 8 * 16 +
           2 * (size_t)waves * mt * kTileRows * sizeof(float) + (size_t)waves * sizeof(uint32_t) +
           (size_t)mt * (K / kTileCols) * sizeof(float);
}

// eight wavefronts while two workgroups fit the LDS of a compute unit together, else sixteen
static int exp_multi_waves(int64_t K, int mt) { return 2 * exp_multi_lds_bytes(K, 8, mt) <= kExpLdsLarge ? 8 : 16; }

// Whether a PoT GEMM with M = 2..4 tokens is served in the exponent form: the conditions of the
// GEMV plus group size 128, room in LDS for the digits of all vectors, and a matrix tall enough
// for a workgroup to reuse them on several row tiles.  Measured at 3 bits against the kernels
// that serve the other shapes: two tokens, 28672 x 8192: 20.3 against 26.6 us, 17920 x 6656: 15.3
// against 17.2 us, 13824 x 5120: 11.3 against 11.9 us, but 8192 x 8192 (one tile per workgroup):
// 11.0 against 8.8 us; three and four tokens (LDS reads of four vectors' digits weigh more):
// 17920 x 6656: 21.5 against 26.5 us, 28672 x 8192: 27.7 against 27.9 us, but 13824 x 5120: 15.2
// against 11.9 us.
bool gemv_exp_multi_ok(int64_t M, int64_t N, int64_t K, int bits, int group)
{
    if (M < 2 || M > 4 || group != 128 || !gemv_exp_ok(N, K, bits)) return false;
    if (N / kTileRows < (M == 2 ? kExpGroups + 1 : 2 * kExpGroups)) return false;
    const int mt = M <= 2 ? 2 : 4;
    const int waves = exp_multi_waves(K, mt);
    if ((int64_t)mt * K > (int64_t)kExpOctetsPerThread * waves * kWave * 8) return false;
    return exp_multi_lds_bytes(K, waves, mt) <= kExpLdsLarge;
}

template <int BITS, int WAVES, int MT>
static hipError_t launch_exp_multi(const void *codes, const void *scales, const void *X, void *Y, int64_t M, int64_t N,
                                   int64_t K, hipStream_t stream)
{
    static std::atomic<uint64_t> raised{0};
    const size_t lds = exp_multi_lds_bytes(K, WAVES, MT);
    const hipError_t e = allow_large_lds((const void *)gemv_exp_multi_kernel<BITS, WAVES, MT>, lds, raised);
    if (e != hipSuccess) return e;
    constexpr int SLOTS = WAVES / kExpSplit;
    const int64_t rowtiles = N / kTileRows;
    const dim3 grid((unsigned)exp_groups((rowtiles + SLOTS - 1) / SLOTS, kExpGroups / SLOTS)), block(WAVES * kWave);
    hipLaunchKernelGGL((gemv_exp_multi_kernel<BITS, WAVES, MT>), grid, block, lds, stream, (const u32x4 *)codes,
                       (const uint16_t *)scales, (const u32x4 *)X, (uint16_t *)Y, (int)K, rowtiles, (int)M, N);
    return hipGetLastError();
}

hipError_t run_gemv_exp_multi(const void *codes, const void *scales, const void *X, void *Y, int64_t M, int64_t N,
                              int64_t K, int bits, hipStream_t stream)
{
    const int mt = M <= 2 ? 2 : 4;
    const int waves = exp_multi_waves(K, mt);
#define POTQ_LAUNCH_EXPM(BITS)                                                                              \
    (waves == 8 ? (mt == 2 ? launch_exp_multi<BITS, 8, 2>(codes, scales, X, Y, M, N, K, stream)             \
                           : launch_exp_multi<BITS, 8, 4>(codes, scales, X, Y, M, N, K, stream))            \
                : (mt == 2 ? launch_exp_multi<BITS, 16, 2>(codes, scales, X, Y, M, N, K, stream)            \
                           : launch_exp_multi<BITS, 16, 4>(codes, scales, X, Y, M, N, K, stream)))
    return bits == 3 ? POTQ_LAUNCH_EXPM(3) : POTQ_LAUNCH_EXPM(2);
#undef POTQ_LAUNCH_EXPM
}

}  // namespace potq
