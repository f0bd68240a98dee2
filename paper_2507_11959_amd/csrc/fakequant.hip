// Step 2 of the method (Sec. 3.3, Algorithm 2): the weight path of one
// fine-tuning iteration.  Forward rebuilds the power-of-two weights under the
// refined scale S^ = S (1 + Gamma); backward turns the gradient with respect to
// those weights into the gradient with respect to Gamma (one value per group)
// under the straight-through estimator.
//
// Both passes are plain streaming kernels bound by HBM: forward reads and
// writes 2 bytes per weight, backward reads 4.  A lane handles an octet (eight
// consecutive weights, one 16-byte load); the lanes that share a group combine
// their partial sums with wavefront shuffles in a fixed order.
//
// The exponent decisions are taken in IEEE binary32 through the thresholds of
// round(log2(.)), exactly as documented for the entry points in potq.h, so the
// results are reproducible bit for bit.
#include "potq_device.hpp"

#pragma clang fp contract(off)

namespace potq {

constexpr int kFqBlock = 256;

// (float)2^(e - 1/2), e = 0..8
__device__ __constant__ const float kHalfStep[9] = {
    0.70710678118654752440f, 1.41421356237309504880f, 2.82842712474619009760f, 5.65685424949238019521f,
    11.3137084989847603904f, 22.6274169979695207808f, 45.2548339959390415616f, 90.5096679918780831232f,
    181.019335983756166246f};

template <int BITS>
struct FqGroup {
    static constexpr int qmax = (1 << (BITS - 1)) - 1;
    float thr[qmax + 1];     // thr[e] = S^ * 2^(e-1/2), e = 0..qmax   (thr[0]: lower edge of the clamp's range)
    float top;               // S^ * 2^(qmax+1/2): upper edge
    float mag[qmax + 1];     // S^ * 2^e, exact

    __device__ __forceinline__ FqGroup(float s, float gamma)
    {
        const float shat = s * (1.0f + gamma);
#pragma unroll
        for (int e = 0; e <= qmax; ++e) {
            thr[e] = shat * kHalfStep[e];
            mag[e] = shat * (float)(1 << e);
        }
        top = shat * kHalfStep[qmax + 1];
    }
    // reconstruction magnitude, and 2^E when the clamp is active (else 0)
    __device__ __forceinline__ void decide(float a, float &m, float &p_if_clamped) const
    {
        m = mag[0];
        float p = 1.0f;
#pragma unroll
        for (int e = 1; e <= qmax; ++e) {
            const bool ge = a >= thr[e];
            m = ge ? mag[e] : m;
            p = ge ? (float)(1 << e) : p;
        }
        p_if_clamped = (a < thr[0] || a >= top) ? p : 0.0f;
    }
};

__device__ __forceinline__ float half_at(const u32x4 &v, int i)
{
    const uint32_t word = v[i >> 1];
    return (float)__builtin_bit_cast(_Float16, (uint16_t)((i & 1) ? (word >> 16) : (word & 0xFFFFu)));
}

template <int BITS>
__global__ __launch_bounds__(kFqBlock) void fakequant_forward_kernel(
    const u32x4 *__restrict__ W, const uint16_t *__restrict__ S, const float *__restrict__ Gamma,
    u32x4 *__restrict__ Wq, int64_t n_octets, int octet_shift)
{
    const int64_t o = (int64_t)blockIdx.x * kFqBlock + threadIdx.x;
    if (o >= n_octets) return;
    const int64_t g = o >> octet_shift;
    const FqGroup<BITS> grp((float)__builtin_bit_cast(_Float16, S[g]), Gamma[g]);
    const u32x4 w = __builtin_nontemporal_load(&W[o]);
    u32x4 out;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        uint32_t packed = 0;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const float x = half_at(w, 2 * i + h);
            float m, p;
            grp.decide(fabsf(x), m, p);
            const _Float16 r = (_Float16)(x < 0.0f ? -m : m);      // one rounding, to nearest even
            packed |= (uint32_t)__builtin_bit_cast(uint16_t, r) << (16 * h);
        }
        out[i] = packed;
    }
    __builtin_nontemporal_store(out, &Wq[o]);
}

template <int BITS>
__global__ __launch_bounds__(kFqBlock) void fakequant_backward_kernel(
    const u32x4 *__restrict__ W, const uint16_t *__restrict__ S, const float *__restrict__ Gamma,
    const u32x4 *__restrict__ dWq, float *__restrict__ dGamma, int64_t n_octets, int octet_shift)
{
    const int64_t o = (int64_t)blockIdx.x * kFqBlock + threadIdx.x;
    const bool live = o < n_octets;
    const int64_t oc = live ? o : n_octets - 1;                      // whole wavefronts take part in the shuffles
    const int64_t g = oc >> octet_shift;
    const float s = (float)__builtin_bit_cast(_Float16, S[g]);
    const FqGroup<BITS> grp(s, Gamma[g]);
    const u32x4 w = __builtin_nontemporal_load(&W[oc]);
    const u32x4 d = __builtin_nontemporal_load(&dWq[oc]);
    float sum = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const float x = half_at(w, i);
        float m, p;
        grp.decide(fabsf(x), m, p);
        const float term = half_at(d, i) * (x < 0.0f ? -p : p);      // exact: a power of two times an fp16
        sum += term;
    }
    // the 2^octet_shift lanes of a group are consecutive and aligned in the wavefront (n_octets is a multiple)
    const int lanes = 1 << octet_shift;
    for (int off = lanes >> 1; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
    if (live && (threadIdx.x & (lanes - 1)) == 0) dGamma[g] = s * sum;
}

hipError_t run_fakequant_forward(const void *W, const void *S, const void *Gamma, void *Wq, int64_t N, int64_t K,
                                 int bits, int group, hipStream_t stream)
{
    const int64_t n_octets = N * K / 8;
    const unsigned blocks = (unsigned)((n_octets + kFqBlock - 1) / kFqBlock);
    const int octet_shift = (group == 128) ? 4 : 3;
#define POTQ_FQ_FWD(B)                                                                                            \
    hipLaunchKernelGGL((fakequant_forward_kernel<B>), dim3(blocks), dim3(kFqBlock), 0, stream, (const u32x4 *)W,  \
                       (const uint16_t *)S, (const float *)Gamma, (u32x4 *)Wq, n_octets, octet_shift)
    if (bits == 4) POTQ_FQ_FWD(4);
    else if (bits == 3) POTQ_FQ_FWD(3);
    else POTQ_FQ_FWD(2);
#undef POTQ_FQ_FWD
    return hipGetLastError();
}

hipError_t run_fakequant_backward(const void *W, const void *S, const void *Gamma, const void *dWq, void *dGamma,
                                  int64_t N, int64_t K, int bits, int group, hipStream_t stream)
{
    const int64_t n_octets = N * K / 8;
    const unsigned blocks = (unsigned)((n_octets + kFqBlock - 1) / kFqBlock);
    const int octet_shift = (group == 128) ? 4 : 3;
#define POTQ_FQ_BWD(B)                                                                                            \
    hipLaunchKernelGGL((fakequant_backward_kernel<B>), dim3(blocks), dim3(kFqBlock), 0, stream, (const u32x4 *)W, \
                       (const uint16_t *)S, (const float *)Gamma, (const u32x4 *)dWq, (float *)dGamma, n_octets,  \
                       octet_shift)
    if (bits == 4) POTQ_FQ_BWD(4);
    else if (bits == 3) POTQ_FQ_BWD(3);
    else POTQ_FQ_BWD(2);
#undef POTQ_FQ_BWD
    return hipGetLastError();
}

}  // namespace potq
