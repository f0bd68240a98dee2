// Fused de-quantise + GEMV (batch-1 decode) on the tiled layout, gfx950.
//
// y[n] = sum_k W~[n,k] x[k].  One workgroup owns a 16-row tile of W and walks
// its K/128 scale groups.  Lane (r = lane % 16, t = lane / 16) of a wavefront
// owns row r of one group: it fetches the group's 128 codes with `bits`
// 16-byte loads, builds the group's table of fp16 high bytes by integer
// addition into the scale's exponent field (Sec. 4.2, once per group) and turns
// four codes at a time into fp16 pairs with byte permutes.  The multiply-adds
// run on the otherwise idle matrix pipe (the vector ALU is the scarce resource
// of this kernel): x, held in LDS, is the B operand replicated in all columns.
// Partial sums are combined in a fixed order, so results are reproducible.
#include "potq_device.hpp"

namespace potq {

// One group (128 columns) of one row: codes in L, table from (s, z), x in LDS.
// Eight weights at a time become the A operand (row = lane % 16, k-slice =
// lane / 16) of v_mfma_f32_16x16x32_f16; the B operand is the matching eight x
// values, the same in all 16 columns, so every column of the 16x16 result holds
// the partial products of the 16 rows.  Products are exact, sums fp32.
template <int BITS, bool IS_INT>
__device__ __forceinline__ void gemv_group(const u32x4 (&L)[BITS], uint32_t s, uint32_t z,
                                           const u32x4 *__restrict__ xg, float4_t (&acc)[4])
{
    PotTable pt;
    IntTable it;
    if (IS_INT)
        it = int_table<BITS>(s, z);
    else
        pt = pot_table<BITS>(s);
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        uint32_t sel[8];
        if (BITS == 3)
            selectors3(L[0][b], L[1][b], L[BITS - 1][b], sel);
        else
            selectors2(L[0][b], L[1][b], sel);
#pragma unroll
        for (int m = 0; m < 8; m += 2) {
#if defined(POTQ_GEMV_DEBUG) && (POTQ_GEMV_DEBUG == 3 || POTQ_GEMV_DEBUG == 5)
            const u32x4 xv = u32x4{s, s + 1, z, s ^ 5u};
#else
            const u32x4 xv = xg[b * 4 + m / 2];     // columns 32b + 4m .. + 7
#endif
            uint32_t e0, o0, e1, o1;
            if (IS_INT) {
                int_lookup(it, sel[m], e0, o0);
                int_lookup(it, sel[m + 1], e1, o1);
            } else {
                pot_lookup(pt, sel[m], e0, o0);
                pot_lookup(pt, sel[m + 1], e1, o1);
            }
            const half8_t av = __builtin_bit_cast(half8_t, (u32x4{e0, o0, e1, o1}));
#if defined(POTQ_GEMV_DEBUG) && (POTQ_GEMV_DEBUG == 4 || POTQ_GEMV_DEBUG == 5)
            acc[m / 2] += __builtin_bit_cast(float4_t, (u32x4{e0, o0, e1, o1} ^ xv) & 0x3fffffffu);
#else
            acc[m / 2] = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, __builtin_bit_cast(half8_t, xv), acc[m / 2], 0, 0, 0);
#endif
        }
    }
}

constexpr int kXRun = 17;   // uint4 per scale group of x in LDS (16 + 1 of padding)

// WAVES wavefronts per workgroup share one 16-row tile: wavefront w, lane group
// t takes scale groups 4w + t, 4w + t + 4*WAVES, ...  The codes of the next
// group are requested before the current one is expanded, and the first request
// goes out before x is staged, so HBM latency overlaps the staging and the math.
template <int BITS, bool IS_INT, int WAVES>
__global__ __launch_bounds__(WAVES * kWave) void gemv_tile16_kernel(
    const u32x4 *__restrict__ codes, const uint16_t *__restrict__ scales, const uint16_t *__restrict__ zeros,
    const u32x4 *__restrict__ x, uint16_t *__restrict__ y, int K)
{
    extern __shared__ u32x4 smem[];
    // x as fp16 pairs, one 256-byte run per scale group, runs padded to 272 bytes so
    // that the four lane groups of a wavefront (four consecutive groups) read
    // from different LDS banks
    u32x4 *xs = smem;

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid >> 6;
    const int r = lane & 15;
    const int t = lane >> 4;
    const int G = K / kTileCols;
    constexpr int kStep = 4 * WAVES;
    const int64_t rowtile = blockIdx.x;
    const int64_t row = rowtile * kTileRows + r;
    const u32x4 *tile0 = codes + rowtile * G * (BITS * 16) + r;
    const uint16_t *srow = scales + row * G;
    const uint16_t *zrow = IS_INT ? zeros + row * G : nullptr;

    // MFMA ignores the execution mask, so the group loop must be uniform: every
    // lane runs ceil(G / kStep) rounds.  A lane whose group index runs past G
    // re-reads the last group (valid memory), takes the scale 1.0 (finite
    // weights) and multiplies by a block of zeros instead of x.
    const int rounds = (G + kStep - 1) / kStep;
    u32x4 *zero_block = smem + (K / kTileCols) * kXRun; // 16 uint4 of zeros
    float *red = (float *)(zero_block + 16);            // WAVES * 16 partial sums

    int g = wave * 4 + t;
    u32x4 L[BITS];
    uint32_t s, z = 0;
    {
        const int gc = g < G ? g : G - 1;
#pragma unroll
        for (int j = 0; j < BITS; ++j) L[j] = __builtin_nontemporal_load(tile0 + (int64_t)gc * (BITS * 16) + 16 * j);
        s = g < G ? (uint32_t)srow[gc] : 0x3C00u;
        if (IS_INT) z = g < G ? (uint32_t)zrow[gc] : 0u;
    }

    for (int i = tid; i < K / 8; i += WAVES * kWave) xs[(i >> 4) * kXRun + (i & 15)] = x[i];
    if (tid < 16) zero_block[tid] = u32x4{0u, 0u, 0u, 0u};
    __syncthreads();

    float4_t acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = float4_t{0.f, 0.f, 0.f, 0.f};
    for (int round = 0; round < rounds; ++round) {
        const int gn = g + kStep;
        u32x4 Ln[BITS];
        uint32_t sn = 0x3C00u, zn = 0;
        if (round + 1 < rounds) {
            const int gc = gn < G ? gn : G - 1;
#pragma unroll
            for (int j = 0; j < BITS; ++j)
#if defined(POTQ_GEMV_DEBUG) && POTQ_GEMV_DEBUG >= 2
                Ln[j] = L[j] + (uint32_t)gc;
#else
                Ln[j] = __builtin_nontemporal_load(tile0 + (int64_t)gc * (BITS * 16) + 16 * j);
#endif
            if (gn < G) {
                sn = srow[gc];
                if (IS_INT) zn = zrow[gc];
            }
        }
#if defined(POTQ_GEMV_DEBUG) && POTQ_GEMV_DEBUG == 1
        for (int j = 0; j < BITS; ++j) acc[0] += __builtin_bit_cast(float4_t, L[j] & 0x3fffffffu);
        acc[1][0] += (float)s;
#else
        gemv_group<BITS, IS_INT>(L, s, z, g < G ? xs + g * kXRun : zero_block, acc);
#endif
        g = gn;
#pragma unroll
        for (int j = 0; j < BITS; ++j) L[j] = Ln[j];
        s = sn;
        z = zn;
    }

    // The MFMA already summed the four lane groups.  Lane (c, q) holds rows 4q..4q+3
    // (identical in every column c); combine the wavefronts in a fixed order.
    const float4_t part = (acc[0] + acc[1]) + (acc[2] + acc[3]);
    if (r == 0) *(float4_t *)(red + wave * kTileRows + 4 * t) = part;
    __syncthreads();
    if (tid < kTileRows) {
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) sum += red[w * kTileRows + tid];
        const _Float16 h = (_Float16)sum;
        y[rowtile * kTileRows + tid] = __builtin_bit_cast(uint16_t, h);
    }
}

constexpr int kGemvMaxWaves = 16;

size_t gemv_lds_bytes(int64_t K)
{
    return (size_t)(K / kTileCols) * kXRun * 16 + 256 + kGemvMaxWaves * kTileRows * sizeof(float);
}

template <int BITS, bool IS_INT>
static void launch_gemv(const void *codes, const void *scales, const void *zeros, const void *x, void *y,
                        int64_t N, int64_t K, hipStream_t stream)
{
    const dim3 grid((unsigned)(N / kTileRows));
    const size_t lds = gemv_lds_bytes(K);
    const int64_t G = K / kTileCols;
    // 8 wavefronts (32 scale groups in flight per tile) measured best; few-row matrices get 16
#define POTQ_LAUNCH_GEMV(W)                                                                                  \
    hipLaunchKernelGGL((gemv_tile16_kernel<BITS, IS_INT, W>), grid, dim3(W * kWave), lds, stream,            \
                       (const u32x4 *)codes, (const uint16_t *)scales, (const uint16_t *)zeros,              \
                       (const u32x4 *)x, (uint16_t *)y, (int)K)
#ifdef POTQ_GEMV_WAVES
    POTQ_LAUNCH_GEMV(POTQ_GEMV_WAVES);
#else
    if (G <= 16) POTQ_LAUNCH_GEMV(4);
    else if (N >= 2048 || G <= 32) POTQ_LAUNCH_GEMV(8);
    else POTQ_LAUNCH_GEMV(16);
#endif
#undef POTQ_LAUNCH_GEMV
}

hipError_t run_gemv_tile16(bool is_int, const void *codes, const void *scales, const void *zeros, const void *x,
                           void *y, int64_t N, int64_t K, int bits, hipStream_t stream)
{
    if (is_int) {
        if (bits == 3) launch_gemv<3, true>(codes, scales, zeros, x, y, N, K, stream);
        else launch_gemv<2, true>(codes, scales, zeros, x, y, N, K, stream);
    } else {
        if (bits == 3) launch_gemv<3, false>(codes, scales, zeros, x, y, N, K, stream);
        else launch_gemv<2, false>(codes, scales, zeros, x, y, N, K, stream);
    }
    return hipGetLastError();
}

}  // namespace potq
