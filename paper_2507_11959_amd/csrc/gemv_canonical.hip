// Fused de-quantise + GEMV on the canonical packed layout (the format at the boundary), gfx950.
//
// The tiled layout exists because turning a dense K-major bit stream into matrix-core operands
// costs vector-ALU work per weight; this kernel pays that cost so that weights can be consumed
// exactly as pot_quantize (or any other producer of the boundary format) wrote them, without
// the one-off potq_repack.  It decodes as the stand-alone pass does -- eight weights ("octet")
// per lane and step, the integer add of Sec. 4.2 into the scale's exponent field, two weights
// per register -- and multiplies the fp16 pairs into an fp32 sum with v_dot2_f32_f16.  About two
// vector-ALU instructions per weight against the 1.1 of the exponent form on the tiled layout:
// meant for convenience and for matrices where HBM time still dominates, not as the fast path.
//
// A wavefront owns a row at a time: lane l takes the 32-weight pieces ("quads" of four octets:
// 4 * bits bytes, one load) l, l + 64, ... of the row, so 64 lanes read 256 * bits consecutive
// bytes per step; x sits in LDS as one 16-byte piece per octet, the pieces of octet j of all
// quads together, so that a step's four reads are conflict-free; the lanes' sums are added by
// butterfly shuffles in a fixed order.  Workgroups are resident and walk the rows with a stride,
// so x is staged once per workgroup of sixteen wavefronts.
#include "potq_device.hpp"
#include "potq_launch.hpp"
#include "potq_octet.hpp"

namespace potq {

constexpr int kCanonWaves = 16;           // wavefronts per workgroup
constexpr int64_t kCanonGroups = 512;     // workgroups at most: two per compute unit

// The code bits of the four octets of a quad from its `BITS` 32-bit words.
template <int BITS>
__device__ __forceinline__ void quad_octets(const uint32_t *__restrict__ p, uint32_t (&f)[4])
{
    if constexpr (BITS == 2) {
        const u32x2 w = *(const u32x2 *)p;
        f[0] = w[0] & 0xFFFFu;
        f[1] = w[0] >> 16;
        f[2] = w[1] & 0xFFFFu;
        f[3] = w[1] >> 16;
    } else if constexpr (BITS == 3) {
        const uint32_t w0 = p[0], w1 = p[1], w2 = p[2];
        f[0] = w0 & 0xFFFFFFu;
        f[1] = __builtin_amdgcn_alignbyte(w1, w0, 3) & 0xFFFFFFu;
        f[2] = __builtin_amdgcn_alignbyte(w2, w1, 2) & 0xFFFFFFu;
        f[3] = w2 >> 8;
    } else {
        const u32x4 w = *(const u32x4 *)p;
        f[0] = w[0];
        f[1] = w[1];
        f[2] = w[2];
        f[3] = w[3];
    }
}

// Sum of a value over the 64 lanes of a wavefront, valid in lane 63: six data-parallel-primitive
// adds on the vector ALU (lane pairs, quads, half rows, rows of 16, then lane 15 of rows 0 and 2
// into rows 1 and 3, then lane 31 into rows 2 and 3) instead of six trips through the LDS
// crossbar, each of which a row's single wavefront would wait out.
template <int CTRL, int ROWS>
__device__ __forceinline__ float dpp_or_zero(float x)      // x of the lane CTRL names; 0 in rows outside ROWS and for lanes without a source
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, ROWS, 0xF, ROWS == 0xF));
}
__device__ __forceinline__ float wave_sum_in_lane_63(float v)
{
    v += dpp_or_zero<0xB1, 0xF>(v);      // quad_perm [1,0,3,2]
    v += dpp_or_zero<0x4E, 0xF>(v);      // quad_perm [2,3,0,1]
    v += dpp_or_zero<0x141, 0xF>(v);     // row_half_mirror
    v += dpp_or_zero<0x140, 0xF>(v);     // row_mirror: every lane holds its row's sum
    v += dpp_or_zero<0x142, 0xA>(v);     // row_bcast15 into rows 1 and 3
    v += dpp_or_zero<0x143, 0xC>(v);     // row_bcast31 into rows 2 and 3
    return v;
}

template <int BITS, bool IS_INT>
__global__ __launch_bounds__(kCanonWaves * kWave) void gemv_canonical_kernel(
    const uint32_t *__restrict__ codes, const uint16_t *__restrict__ scales, const uint16_t *__restrict__ zeros,
    const u32x4 *__restrict__ x, uint16_t *__restrict__ y, int64_t N, int K, int group_shift)
{
    extern __shared__ u32x4 xs[];             // x: piece of octet o at (o % 4) * quads + o / 4
    const int octets = K / 8;
    const int quads = K / 32;
    for (int o = threadIdx.x; o < octets; o += kCanonWaves * kWave) xs[(o & 3) * quads + (o >> 2)] = x[o];
    __syncthreads();

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int64_t stride = (int64_t)gridDim.x * kCanonWaves;
    const int quad_shift = group_shift - 5;   // quads per group = group / 32
    const int groups = K >> group_shift;
    for (int64_t n = (int64_t)blockIdx.x * kCanonWaves + wave; n < N; n += stride) {
        const uint32_t *crow = codes + n * ((int64_t)quads * BITS);    // the row's 32-bit words
        const uint16_t *srow = scales + n * groups;
        const uint16_t *zrow = IS_INT ? zeros + n * groups : nullptr;
        float sum = 0.f;
#pragma unroll 4
        for (int q = lane; q < quads; q += kWave) {
            uint32_t f[4];
            quad_octets<BITS>(crow + (int64_t)q * BITS, f);
            const int g = q >> quad_shift;
            const uint32_t s = srow[g];
            half2_t zm, sm;
            if (IS_INT) {
                const _Float16 S = __builtin_bit_cast(_Float16, (uint16_t)s);
                const _Float16 Z = __builtin_bit_cast(_Float16, zrow[g]) - (_Float16)1024.0f;
                zm = half2_t{Z, Z};
                sm = half2_t{S, S};
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const u32x4 w = IS_INT ? int_octet<BITS>(f[j], zm, sm) : pot_octet<BITS>(f[j], s);
                const u32x4 xv = xs[j * quads + q];
#pragma unroll
                for (int m = 0; m < 4; ++m) sum = __builtin_amdgcn_fdot2(as_half2(w[m]), as_half2(xv[m]), sum, false);
            }
        }
        sum = wave_sum_in_lane_63(sum);
        if (lane == kWave - 1) y[n] = __builtin_bit_cast(uint16_t, (_Float16)sum);
    }
}

size_t gemv_canonical_lds_bytes(int64_t K) { return (size_t)K * 2; }

template <int BITS, bool IS_INT>
static hipError_t launch_gemv_canonical(const void *codes, const void *scales, const void *zeros, const void *x,
                                        void *y, int64_t N, int64_t K, int group, hipStream_t stream)
{
    const size_t lds = gemv_canonical_lds_bytes(K);
    const hipError_t e = allow_large_lds<gemv_canonical_kernel<BITS, IS_INT>>(lds);
    if (e != hipSuccess) return e;
    int64_t blocks = (N + kCanonWaves - 1) / kCanonWaves;
    if (blocks > kCanonGroups) blocks = kCanonGroups;
    hipLaunchKernelGGL((gemv_canonical_kernel<BITS, IS_INT>), dim3((unsigned)blocks), dim3(kCanonWaves * kWave), lds,
                       stream, (const uint32_t *)codes, (const uint16_t *)scales, (const uint16_t *)zeros,
                       (const u32x4 *)x, (uint16_t *)y, N, (int)K, group == 128 ? 7 : 6);
    return hipGetLastError();
}

hipError_t run_gemv_canonical(bool is_int, const void *codes, const void *scales, const void *zeros, const void *x,
                              void *y, int64_t N, int64_t K, int bits, int group, hipStream_t stream)
{
    if (is_int)
        return bits == 4   ? launch_gemv_canonical<4, true>(codes, scales, zeros, x, y, N, K, group, stream)
               : bits == 3 ? launch_gemv_canonical<3, true>(codes, scales, zeros, x, y, N, K, group, stream)
                           : launch_gemv_canonical<2, true>(codes, scales, zeros, x, y, N, K, group, stream);
    return bits == 4   ? launch_gemv_canonical<4, false>(codes, scales, zeros, x, y, N, K, group, stream)
           : bits == 3 ? launch_gemv_canonical<3, false>(codes, scales, zeros, x, y, N, K, group, stream)
                       : launch_gemv_canonical<2, false>(codes, scales, zeros, x, y, N, K, group, stream);
}

}  // namespace potq
