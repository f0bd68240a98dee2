// Fused de-quantise + GEMV (batch-1 decode) on the tiled layout, gfx950.
//
// y[n] = sum_k W~[n,k] x[k].  One workgroup owns a 16-row tile of W and walks
// its K/128 scale groups.  Lane (r = lane % 16, t = lane / 16) of a wavefront
// owns row r of one group: it fetches the group's 128 codes with `bits`
// 16-byte loads, builds the group's table of fp16 high bytes by integer
// addition into the scale's exponent field (Sec. 4.2, once per group), turns
// four codes at a time into fp16 pairs with byte permutes and feeds them to
// v_dot2_f32_f16 (exact products, fp32 accumulation) against x held in LDS.
// Partial sums are combined in a fixed order, so results are reproducible.
#include "potq_device.hpp"

namespace potq {

constexpr int kGemvBlock = 256;
constexpr int kGemvWaves = kGemvBlock / kWave;

template <int BITS, bool IS_INT>
__global__ __launch_bounds__(kGemvBlock) void gemv_tile16_kernel(
    const u32x4 *__restrict__ codes, const uint16_t *__restrict__ scales, const uint16_t *__restrict__ zeros,
    const u32x4 *__restrict__ x, uint16_t *__restrict__ y, int K)
{
    extern __shared__ u32x4 smem[];
    u32x4 *xs = smem;                                   // K/8 uint4 = x as fp16 pairs
    float *red = (float *)(smem + K / 8);               // kGemvBlock partial sums

    const int tid = threadIdx.x;
    for (int i = tid; i < K / 8; i += kGemvBlock) xs[i] = x[i];
    __syncthreads();

    const int lane = tid & (kWave - 1);
    const int wave = tid >> 6;
    const int r = lane & 15;
    const int t = lane >> 4;
    const int G = K / kTileCols;
    const int64_t rowtile = blockIdx.x;
    const int64_t row = rowtile * kTileRows + r;

    float acc0 = 0.f, acc1 = 0.f;
    for (int g = wave * 4 + t; g < G; g += 4 * kGemvWaves) {
        const u32x4 *tp = codes + (rowtile * G + g) * (BITS * 16) + r;
        u32x4 L[BITS];
#pragma unroll
        for (int j = 0; j < BITS; ++j) L[j] = tp[16 * j];
        const uint32_t s = scales[row * G + g];
        PotTable pt;
        IntTable it;
        if (IS_INT)
            it = int_table<BITS>(s, zeros[row * G + g]);
        else
            pt = pot_table<BITS>(s);
        const u32x4 *xg = xs + g * 16;                  // 128 fp16 = 16 uint4
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            uint32_t sel[8];
            if (BITS == 3)
                selectors3(L[0][b], L[1][b], L[BITS - 1][b], sel);
            else
                selectors2(L[0][b], L[1][b], sel);
#pragma unroll
            for (int m = 0; m < 8; m += 2) {
                const u32x4 xv = xg[b * 4 + m / 2];     // columns 32b + 4m .. + 7
                uint32_t e0, o0, e1, o1;
                if (IS_INT) {
                    int_lookup(it, sel[m], e0, o0);
                    int_lookup(it, sel[m + 1], e1, o1);
                } else {
                    pot_lookup(pt, sel[m], e0, o0);
                    pot_lookup(pt, sel[m + 1], e1, o1);
                }
                acc0 = __builtin_amdgcn_fdot2(as_half2(e0), as_half2(xv[0]), acc0, false);
                acc1 = __builtin_amdgcn_fdot2(as_half2(o0), as_half2(xv[1]), acc1, false);
                acc0 = __builtin_amdgcn_fdot2(as_half2(e1), as_half2(xv[2]), acc0, false);
                acc1 = __builtin_amdgcn_fdot2(as_half2(o1), as_half2(xv[3]), acc1, false);
            }
        }
    }

    red[tid] = acc0 + acc1;
    __syncthreads();
    if (tid < kTileRows) {
        float sum = 0.f;
#pragma unroll
        for (int i = 0; i < kGemvBlock / kTileRows; ++i) sum += red[i * kTileRows + tid];
        const _Float16 h = (_Float16)sum;
        y[rowtile * kTileRows + tid] = __builtin_bit_cast(uint16_t, h);
    }
}

size_t gemv_lds_bytes(int64_t K) { return (size_t)K * 2 + kGemvBlock * sizeof(float); }

hipError_t run_gemv_tile16(bool is_int, const void *codes, const void *scales, const void *zeros, const void *x,
                           void *y, int64_t N, int64_t K, int bits, hipStream_t stream)
{
    const dim3 grid((unsigned)(N / kTileRows)), block(kGemvBlock);
    const size_t lds = gemv_lds_bytes(K);
#define POTQ_LAUNCH_GEMV(B, I)                                                                              \
    hipLaunchKernelGGL((gemv_tile16_kernel<B, I>), grid, block, lds, stream, (const u32x4 *)codes,          \
                       (const uint16_t *)scales, (const uint16_t *)zeros, (const u32x4 *)x, (uint16_t *)y, (int)K)
    if (is_int) {
        if (bits == 3) POTQ_LAUNCH_GEMV(3, true); else POTQ_LAUNCH_GEMV(2, true);
    } else {
        if (bits == 3) POTQ_LAUNCH_GEMV(3, false); else POTQ_LAUNCH_GEMV(2, false);
    }
#undef POTQ_LAUNCH_GEMV
    return hipGetLastError();
}

}  // namespace potq
