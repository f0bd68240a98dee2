// Fused de-quantise + GEMM on the matrix cores (tiled layout), gfx950.
//
// Y[m,n] = sum_k X[m,k] W~[n,k].  A wavefront owns one 16-row tile of W and a
// strip of tokens.  Per scale group (128 columns) lane (r = lane % 16,
// q = lane / 16) fetches the 32 codes of row r, column block q, builds the
// group's byte table by integer addition into the scale's exponent field
// (Sec. 4.2) and expands the codes, eight at a time, straight into the A
// operand of v_mfma_f32_16x16x32_f16: A row = weight row r, A k-slot (q, i) =
// column 32q + 8*step + i of the group.  The B operand is X with the same
// k-slot assignment, so each lane reads 16 contiguous bytes of a token's row.
// Accumulation is fp32 in the MFMA accumulators; one rounding to fp16 at the end.
#include "potq_device.hpp"

namespace potq {

constexpr int kGemmBlock = 256;
constexpr int kGemmWaves = kGemmBlock / kWave;
constexpr int kTokTiles = 4;                       // 16-token MFMA tiles per wavefront
constexpr int kTokPerBlock = 16 * kTokTiles;

template <int BITS, bool IS_INT>
__global__ __launch_bounds__(kGemmBlock) void gemm_tile16_kernel(
    const uint32_t *__restrict__ codes, const uint16_t *__restrict__ scales, const uint16_t *__restrict__ zeros,
    const uint16_t *__restrict__ X, uint16_t *__restrict__ Y, int M, int64_t N, int K)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int r = lane & 15;
    const int q = lane >> 4;
    const int G = K / kTileCols;
    const int64_t rowtile = (int64_t)blockIdx.x * kGemmWaves + wave;
    if (rowtile * kTileRows >= N) return;
    const int m0 = blockIdx.y * kTokPerBlock;
    const int64_t row = rowtile * kTileRows + r;

    float4_t acc[kTokTiles];
#pragma unroll
    for (int c = 0; c < kTokTiles; ++c) acc[c] = float4_t{0.f, 0.f, 0.f, 0.f};

    // token row of this lane in each token tile (B operand column = lane % 16)
    const uint16_t *xrow[kTokTiles];
    bool xok[kTokTiles];
#pragma unroll
    for (int c = 0; c < kTokTiles; ++c) {
        const int m = m0 + 16 * c + r;
        xok[c] = m < M;
        xrow[c] = X + (int64_t)(xok[c] ? m : 0) * K + 32 * q;
    }

    for (int g = 0; g < G; ++g) {
        const uint32_t *tp = codes + (rowtile * G + g) * (BITS * 64) + r * 4 + q;
        uint32_t w[BITS];
#pragma unroll
        for (int j = 0; j < BITS; ++j) w[j] = tp[64 * j];
        const uint32_t s = scales[row * G + g];
        PotTable pt;
        IntTable it;
        if (IS_INT)
            it = int_table<BITS>(s, zeros[row * G + g]);
        else
            pt = pot_table<BITS>(s);
        uint32_t sel[8];
        if (BITS == 3)
            selectors3(w[0], w[1], w[BITS - 1], sel);
        else
            selectors2(w[0], w[1], sel);
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            uint32_t a0, a1, a2, a3;
            if (IS_INT) {
                int_lookup(it, sel[2 * st], a0, a1);
                int_lookup(it, sel[2 * st + 1], a2, a3);
            } else {
                pot_lookup(pt, sel[2 * st], a0, a1);
                pot_lookup(pt, sel[2 * st + 1], a2, a3);
            }
            const half8_t av = __builtin_bit_cast(half8_t, (u32x4{a0, a1, a2, a3}));
#pragma unroll
            for (int c = 0; c < kTokTiles; ++c) {
                u32x4 b = u32x4{0u, 0u, 0u, 0u};
                if (xok[c]) b = *(const u32x4 *)(xrow[c] + g * kTileCols + 8 * st);
                acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, __builtin_bit_cast(half8_t, b), acc[c], 0, 0, 0);
            }
        }
    }

    // D: lane holds token m0 + 16c + (lane % 16), weight rows 4*(lane / 16) + i
#pragma unroll
    for (int c = 0; c < kTokTiles; ++c) {
        const int m = m0 + 16 * c + r;
        if (m < M) {
            typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
            half4_t h;
#pragma unroll
            for (int i = 0; i < 4; ++i) h[i] = (_Float16)acc[c][i];
            *(half4_t *)(Y + (int64_t)m * N + rowtile * kTileRows + 4 * q) = h;
        }
    }
}

hipError_t run_gemm_tile16(bool is_int, const void *codes, const void *scales, const void *zeros, const void *X,
                           void *Y, int64_t M, int64_t N, int64_t K, int bits, hipStream_t stream)
{
    const int64_t rowtiles = N / kTileRows;
    const dim3 grid((unsigned)((rowtiles + kGemmWaves - 1) / kGemmWaves),
                    (unsigned)((M + kTokPerBlock - 1) / kTokPerBlock));
    const dim3 block(kGemmBlock);
#define POTQ_LAUNCH_GEMM(B, I)                                                                             \
    hipLaunchKernelGGL((gemm_tile16_kernel<B, I>), grid, block, 0, stream, (const uint32_t *)codes,        \
                       (const uint16_t *)scales, (const uint16_t *)zeros, (const uint16_t *)X, (uint16_t *)Y, \
                       (int)M, N, (int)K)
    if (is_int) {
        if (bits == 3) POTQ_LAUNCH_GEMM(3, true); else POTQ_LAUNCH_GEMM(2, true);
    } else {
        if (bits == 3) POTQ_LAUNCH_GEMM(3, false); else POTQ_LAUNCH_GEMM(2, false);
    }
#undef POTQ_LAUNCH_GEMM
    return hipGetLastError();
}

}  // namespace potq
