// Step 1 of PoT-PTQ on the GPU: data-agnostic scale search (Sec. 3.2, Algorithm 1).
//
// For every group of G weights: s0 = max|w| / (2^qmax - 1); for the 200 multipliers
// b = 0.01 i the group is quantised with s = fp16(s0 b) (E = clamp(round(log2(|w|/s)), 0, qmax),
// w~ = sign(w) s 2^E) and the squared error summed; the first multiplier with the
// smallest error wins; its scale (fp16) and codes are written out in the canonical
// packed layout, ready for pot_dequant / potq_repack.
//
// The paper does not fix the arithmetic.  This kernel uses IEEE binary32, one rounding
// per operation and no contraction, in exactly the order documented with
// `pot_quantize` in potq.h, so that its integer decisions can be reproduced elsewhere:
// one thread owns one multiplier and walks the group's weights in ascending order.
// The search is plain vector-ALU work (about ten operations per weight and
// multiplier), embarrassingly parallel over groups.
#include "potq_device.hpp"

#pragma clang fp contract(off)

namespace potq {

constexpr int kCandidates = 200;
constexpr int kGroupsPerBlock = 2;
constexpr int kQuantThreads = 448;       // 7 wavefronts: 400 (group, multiplier) pairs + the tail

// (float)2^(e - 1/2), e = 1..7: the decision thresholds of round(log2(.)), relative to the scale
__device__ __constant__ const float kRoundThreshold[8] = {
    0.0f, 1.41421356237309504880f, 2.82842712474619009760f, 5.65685424949238019521f,
    11.3137084989847603904f, 22.6274169979695207808f, 45.2548339959390415616f, 90.5096679918780831232f};

// Candidate i of a group as it would be stored and used at inference (Sec. 4.2 keeps the scale
// as FP16): s0 * (0.01 i) rounded once to binary16 and clamped into the domain on which the
// de-quantisation recipe is exact; returned as its bit pattern.
template <int BITS>
__device__ __forceinline__ uint32_t quantize_candidate(float s0, int i)
{
    constexpr int qmax = (1 << (BITS - 1)) - 1;
    float s = s0 * ((float)i * 0.01f);
    // The product is rounded to binary32 first and to binary16 second, as documented.  Left to
    // itself the compiler fuses multiply and conversion into one mixed-precision instruction
    // with a single rounding, which differs when the binary32 product lands on a binary16
    // midpoint; the empty asm makes the binary32 value the conversion's operand.
    asm volatile("" : "+v"(s));
    const uint32_t sb = __builtin_bit_cast(uint16_t, (_Float16)s);
    const uint32_t lo = 0x0400u, hi = ((30u - qmax) << 10) | 0x3FFu;
    return sb < lo ? lo : (sb > hi ? hi : sb);
}

__device__ __forceinline__ float half_bits_to_float(uint32_t bits)
{
    return (float)__builtin_bit_cast(_Float16, (uint16_t)bits);
}

template <int BITS>
__global__ __launch_bounds__(kQuantThreads) void quantize_kernel(
    const uint16_t *__restrict__ W, uint32_t *__restrict__ codes, uint16_t *__restrict__ scales,
    int64_t total_groups, int groups_per_row, int group)
{
    constexpr int qmax = (1 << (BITS - 1)) - 1;
    __shared__ float w[kGroupsPerBlock][128];
    __shared__ float qs[kGroupsPerBlock][kCandidates];
    __shared__ float wmax_s[kGroupsPerBlock];
    __shared__ int best_s[kGroupsPerBlock];
    __shared__ uint32_t packed[kGroupsPerBlock][4 * BITS];

    const int tid = threadIdx.x;
    const int64_t g0 = (int64_t)blockIdx.x * kGroupsPerBlock;
    (void)groups_per_row;

    // stage the weights (binary16 -> binary32 is exact) and find max |w| per group
    if (tid < kGroupsPerBlock * 128) {
        const int gi = tid >> 7, k = tid & 127;
        float v = 0.f;
        if (g0 + gi < total_groups && k < group)
            v = (float)__builtin_bit_cast(_Float16, W[(g0 + gi) * group + k]);
        w[gi][k] = v;
    }
    if (tid < kGroupsPerBlock * 4 * BITS) packed[tid / (4 * BITS)][tid % (4 * BITS)] = 0u;
    __syncthreads();
    if (tid < kGroupsPerBlock * 64) {                   // one wavefront per group
        const int gi = tid >> 6, lane = tid & 63;
        float m = fmaxf(fabsf(w[gi][lane]), fabsf(w[gi][lane + 64]));
        for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
        if (lane == 0) wmax_s[gi] = m;
    }
    __syncthreads();

    // one thread per (group, multiplier): sequential error sum in ascending k
    if (tid < kGroupsPerBlock * kCandidates) {
        const int gi = tid / kCandidates, i = tid % kCandidates + 1;
        const float s0 = __fdiv_rn(wmax_s[gi], (float)((1 << qmax) - 1));
        const float s = half_bits_to_float(quantize_candidate<BITS>(s0, i));
        float thr[qmax + 1], mag_of[qmax + 1];
#pragma unroll
        for (int e = 0; e <= qmax; ++e) {
            thr[e] = s * kRoundThreshold[e];            // thr[0] is not used
            mag_of[e] = s * (float)(1 << e);            // exact
        }
        float q = 0.f;
        for (int k = 0; k < group; ++k) {
            const float a = fabsf(w[gi][k]);
            float mag = mag_of[0];
#pragma unroll
            for (int e = 1; e <= qmax; ++e) mag = a >= thr[e] ? mag_of[e] : mag;
            // (w - sign(w) mag)^2 = (|w| - mag)^2 exactly: the two differences are negatives of each other
            const float d = a - mag;
            q = __builtin_fmaf(d, d, q);
        }
        qs[gi][i - 1] = q;
    }
    __syncthreads();

    // first multiplier with the smallest error (strict '<' in ascending order)
    if (tid < kGroupsPerBlock * 64) {
        const int gi = tid >> 6, lane = tid & 63;
        float qb = INFINITY;
        int ib = kCandidates + 1;
        for (int i = lane; i < kCandidates; i += 64) {
            const float q = qs[gi][i];
            if (q < qb) {
                qb = q;
                ib = i + 1;
            }
        }
        for (int off = 32; off > 0; off >>= 1) {
            const float qo = __shfl_xor(qb, off, 64);
            const int io = __shfl_xor(ib, off, 64);
            if (qo < qb || (qo == qb && io < ib)) {
                qb = qo;
                ib = io;
            }
        }
        if (lane == 0) best_s[gi] = ib > kCandidates ? 1 : ib;
    }
    __syncthreads();

    // codes under the winning scale, packed little-endian along K; the scale rounded once to fp16
    if (tid < kGroupsPerBlock * 128) {
        const int gi = tid >> 7, k = tid & 127;
        if (g0 + gi < total_groups && k < group) {
            const float s0 = __fdiv_rn(wmax_s[gi], (float)((1 << qmax) - 1));
            const uint32_t sb = quantize_candidate<BITS>(s0, best_s[gi]);
            const float s = half_bits_to_float(sb);
            const float x = w[gi][k];
            int E = 0;
#pragma unroll
            for (int e = 1; e <= qmax; ++e) E = fabsf(x) >= s * kRoundThreshold[e] ? e : E;
            const uint32_t code = (uint32_t)E | (x < 0.f ? (1u << (BITS - 1)) : 0u);
            const int pos = BITS * k, idx = pos >> 5, sh = pos & 31;
            atomicOr(&packed[gi][idx], code << sh);
            if (sh + BITS > 32) atomicOr(&packed[gi][idx + 1], code >> (32 - sh));
            if (k == 0) scales[g0 + gi] = (uint16_t)sb;
        }
    }
    __syncthreads();
    const int words = group * BITS / 32;                // 32-bit words of one packed group
    if (tid < kGroupsPerBlock * words) {
        const int gi = tid / words, j = tid % words;
        if (g0 + gi < total_groups) codes[(g0 + gi) * words + j] = packed[gi][j];
    }
}

hipError_t run_quantize(const void *W, void *codes, void *scales, int64_t N, int64_t K, int bits, int group,
                        hipStream_t stream)
{
    const int64_t total_groups = N * (K / group);
    const unsigned blocks = (unsigned)((total_groups + kGroupsPerBlock - 1) / kGroupsPerBlock);
    if (bits == 4)
        hipLaunchKernelGGL((quantize_kernel<4>), dim3(blocks), dim3(kQuantThreads), 0, stream, (const uint16_t *)W,
                           (uint32_t *)codes, (uint16_t *)scales, total_groups, (int)(K / group), group);
    else if (bits == 3)
        hipLaunchKernelGGL((quantize_kernel<3>), dim3(blocks), dim3(kQuantThreads), 0, stream, (const uint16_t *)W,
                           (uint32_t *)codes, (uint16_t *)scales, total_groups, (int)(K / group), group);
    else
        hipLaunchKernelGGL((quantize_kernel<2>), dim3(blocks), dim3(kQuantThreads), 0, stream, (const uint16_t *)W,
                           (uint32_t *)codes, (uint16_t *)scales, total_groups, (int)(K / group), group);
    return hipGetLastError();
}

}  // namespace potq
