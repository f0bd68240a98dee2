// Stand-alone de-quantisation kernels (canonical layout), gfx950.
//
// The whole matrix is one linear stream: because K is a multiple of 128, the
// packed codes, the scales and the fp16 output are all contiguous and "octet"
// o (eight consecutive weights) sits at code byte `bits*o`, output byte 16*o
// and scale index (8*o)/group, whatever the row.  The pass is bound by HBM
// writes (2 bytes out per weight against bits/8 + 2/group in), so the mapping
// is chosen for the store side: every lane writes one 16-byte octet per store
// instruction and 16 neighbouring lanes cover one 256-byte run, four such runs
// per wavefront instruction, all full cache lines.
#include "potq_device.hpp"
#include "potq_octet.hpp"

namespace potq {

// Shape of the launch by code width: octets (16-byte stores) per lane, threads per workgroup,
// and the order in which the workgroups take the 48 KB pieces of the output.  Chosen by
// measurement on a 70B-sized layer with code buffers that are not resident in the last-level
// cache: three octets per lane and 1024 threads are 4-10 % faster than any other pair tried
// (one to seven octets, 256 to 1024 threads, runs of 8 to 64 lanes) at 2 and 3 bits, two and
// 512 are at 4 bits.  Workgroups are dealt to the eight XCDs in turn (workgroup b runs on XCD
// b % 8); at 3 bits it pays (76.9 -> 80.2 % of the HBM peak) to renumber them so that each XCD
// takes runs of sixteen consecutive pieces, at 2 bits it costs 1 %.
template <int BITS> struct DequantShape {
    static constexpr int octets = (BITS == 4) ? 2 : 3;
    static constexpr int block = (BITS == 4) ? 512 : 1024;
    static constexpr int xcd_run = (BITS == 3) ? 16 : 0;     // 0: workgroups take the pieces in launch order
    // how the output is stored: streaming and written through at system scope, all stores of a lane after
    // all its loads (store_streaming), or streaming only, scheduled by the compiler (its non-temporal
    // store).  Same-process A/B on the 70B layer: at 3 bits the first is 0.8-1.2 % faster (80.1 against
    // 79.0 % of the HBM peak), at 2 bits 2.5 % slower.
    static constexpr bool write_through = BITS == 3;
};

constexpr int kXcds = 8;

// Piece of the output that workgroup `bid` of `nblocks` works on: a bijection of [0, nblocks).
// Whole rounds of 8 * RUN workgroups are renumbered so that the workgroups of one XCD (equal
// bid % 8) take RUN consecutive pieces; the incomplete last round keeps the launch order.
template <int RUN>
__device__ __forceinline__ int64_t xcd_piece(int64_t bid, int64_t nblocks)
{
    if constexpr (RUN == 0) {
        return bid;
    } else {
        constexpr int64_t round = (int64_t)kXcds * RUN;
        if (bid >= nblocks / round * round) return bid;
        const int64_t in = bid % round;
        return bid - in + (in % kXcds) * RUN + in / kXcds;
    }
}

// The work of one workgroup: `block` indexes the workgroup-sized pieces of the matrix's octet stream.
template <int BITS, bool IS_INT>
__device__ __forceinline__ void dequant_block(const uint32_t *__restrict__ codes, const uint16_t *__restrict__ scales,
                                              const uint16_t *__restrict__ zeros, u32x4 *__restrict__ out,
                                              int64_t n_octets, int group_shift, int64_t block)
{
    const int lane = threadIdx.x & (kWave - 1);
    constexpr int kOctetsPerLane = DequantShape<BITS>::octets;
    constexpr int kDequantBlock = DequantShape<BITS>::block;
    constexpr int kOctetsPerWave = kWave * kOctetsPerLane;
    const int64_t wave = block * (kDequantBlock / kWave) + (threadIdx.x >> 6);
    const int64_t base = wave * kOctetsPerWave;
    if (base >= n_octets) return;
    // lane = (quarter, l): quarter q owns a run of 16*U octets, visited 16 lanes (256 output bytes) at a time
    const int64_t o0 = base + (lane >> 4) * (16 * kOctetsPerLane) + (lane & 15);
    const int octet_shift = group_shift - 3;   // octets per group = group / 8

    if constexpr (!DequantShape<BITS>::write_through) {
        // the compiler hoists the loads of all steps ahead of the first store and paces the stores
        // between the decodes; written any other way this shape loses up to 10 points at 2 bits
#pragma unroll
        for (int j = 0; j < kOctetsPerLane; ++j) {
            const int64_t o = o0 + 16 * j;
            if (o < n_octets) {
                const uint32_t f = load_octet_bits<BITS>(codes, o);
                const int64_t g = o >> octet_shift;
                const uint32_t s = scales[g];
                u32x4 w;
                if (IS_INT) {
                    const _Float16 S = __builtin_bit_cast(_Float16, (uint16_t)s);
                    const _Float16 Z = __builtin_bit_cast(_Float16, zeros[g]) - (_Float16)1024.0f;
                    w = int_octet<BITS>(f, half2_t{Z, Z}, half2_t{S, S});
                } else {
                    w = pot_octet<BITS>(f, s);
                }
                __builtin_nontemporal_store(w, &out[o]);   // the output is not read again by this pass
            }
        }
    } else {
        // All loads first, then decode, then the stores (inline asm: the compiler does not move
        // loads across them).  A wavefront that lies wholly inside the matrix -- all but the last
        // one -- runs without any per-lane condition; in the last one an octet past the end
        // re-reads the last octet (valid memory) and stores nothing.
        const bool whole = base + kOctetsPerWave <= n_octets;     // wavefront-uniform
        uint32_t f[kOctetsPerLane], s[kOctetsPerLane], z[kOctetsPerLane];
#pragma unroll
        for (int j = 0; j < kOctetsPerLane; ++j) {
            const int64_t o = whole ? o0 + 16 * j : min(o0 + 16 * j, n_octets - 1);
            f[j] = load_octet_bits<BITS>(codes, o);
            const int64_t g = o >> octet_shift;
            s[j] = scales[g];
            z[j] = IS_INT ? (uint32_t)zeros[g] : 0u;
        }
        u32x4 w[kOctetsPerLane];
#pragma unroll
        for (int j = 0; j < kOctetsPerLane; ++j) {
            if (IS_INT) {
                const _Float16 S = __builtin_bit_cast(_Float16, (uint16_t)s[j]);
                const _Float16 Z = __builtin_bit_cast(_Float16, (uint16_t)z[j]) - (_Float16)1024.0f;
                w[j] = int_octet<BITS>(f[j], half2_t{Z, Z}, half2_t{S, S});
            } else {
                w[j] = pot_octet<BITS>(f[j], s[j]);
            }
        }
        if (whole) {
#pragma unroll
            for (int j = 0; j < kOctetsPerLane; ++j) store_streaming(&out[o0 + 16 * j], w[j]);
        } else {
#pragma unroll
            for (int j = 0; j < kOctetsPerLane; ++j)
                if (o0 + 16 * j < n_octets) store_streaming(&out[o0 + 16 * j], w[j]);
        }
    }
}

template <int BITS, bool IS_INT>
__global__ __launch_bounds__(DequantShape<BITS>::block) void dequant_kernel(
    const uint32_t *__restrict__ codes, const uint16_t *__restrict__ scales,
    const uint16_t *__restrict__ zeros, u32x4 *__restrict__ out, int64_t n_octets, int group_shift)
{
    dequant_block<BITS, IS_INT>(codes, scales, zeros, out, n_octets, group_shift,
                                xcd_piece<DequantShape<BITS>::xcd_run>(blockIdx.x, gridDim.x));
}

// Several matrices in one launch: every launch costs a fixed ramp-up and drain
// (about 1.5 us here) during which HBM idles, so the matrices of a decoder
// layer are best done together.  The descriptor table travels as a kernel argument.
constexpr int kMaxBatch = 16;
// The time between the start of a workgroup and its first load shows in the throughput of this
// pass (512 idle cycles there cost 11 %), so the table is laid out for two rounds of scalar
// loads: the starts of all matrices in one block at the head (slots from `count` on hold the
// total, so they never count), then one 64-byte descriptor per matrix, fetched whole.
struct DequantEntry {
    const uint32_t *codes;
    const uint16_t *scales;
    const uint16_t *zeros;
    u32x4 *out;
    int64_t n_octets;
    uint32_t first_block;     // workgroups of the launch that come before this matrix
    uint32_t pad[5];
};
static_assert(sizeof(DequantEntry) == 64, "one descriptor = one 64-byte scalar load");
struct DequantBatch {
    uint32_t below[kMaxBatch];       // below[k] = first_block of matrix k minus one; the total minus one from `count` on
    DequantEntry entry[kMaxBatch];
    int count;
};

template <int BITS, bool IS_INT>
__global__ __launch_bounds__(DequantShape<BITS>::block) void dequant_batch_kernel(const DequantBatch batch, int group_shift)
{
    // the pieces of all matrices form one sequence, renumbered as a whole
    const uint32_t piece = (uint32_t)xcd_piece<DequantShape<BITS>::xcd_run>(blockIdx.x, gridDim.x);
    // Matrices that start at or before this piece, less one.  Workgroup counts stay below 2^31,
    // so the top bit of below[k] - piece says piece >= first_block[k]; written as arithmetic so
    // that it stays on the scalar unit.
    uint32_t i = 0;
#pragma unroll
    for (int k = 1; k < 8; ++k) i += (batch.below[k] - piece) >> 31;
    if (batch.count > 8) {
#pragma unroll
        for (int k = 8; k < kMaxBatch; ++k) i += (batch.below[k] - piece) >> 31;
    }
    const DequantEntry e = batch.entry[i];
    // all fields in one round: left alone, the compiler fetches the pointers only after the
    // bounds test on n_octets, a third dependent round
    asm volatile("" : : "s"(e.codes), "s"(e.scales), "s"(e.zeros), "s"(e.out), "s"(e.n_octets), "s"(e.first_block), "s"(group_shift));
    dequant_block<BITS, IS_INT>(e.codes, e.scales, e.zeros, e.out, e.n_octets, group_shift, piece - e.first_block);
}

static int dequant_block_threads(int bits) { return bits == 4 ? DequantShape<4>::block : DequantShape<2>::block; }

static int64_t dequant_blocks(int64_t n_octets, int bits)
{
    static_assert(DequantShape<2>::octets == DequantShape<3>::octets && DequantShape<2>::block == DequantShape<3>::block,
                  "2- and 3-bit launches share one shape");
    const int64_t per_wave = kWave * (bits == 4 ? DequantShape<4>::octets : DequantShape<2>::octets);
    const int64_t waves_per_block = dequant_block_threads(bits) / kWave;
    const int64_t waves = (n_octets + per_wave - 1) / per_wave;
    return (waves + waves_per_block - 1) / waves_per_block;
}

template <int BITS, bool IS_INT>
static hipError_t launch_dequant(const void *codes, const void *scales, const void *zeros, void *out,
                                 int64_t N, int64_t K, int group, hipStream_t stream)
{
    const int64_t n_octets = N * K / 8;
    const int group_shift = (group == 128) ? 7 : 6;
    hipLaunchKernelGGL((dequant_kernel<BITS, IS_INT>), dim3((unsigned)dequant_blocks(n_octets, BITS)), dim3(DequantShape<BITS>::block),
                       0, stream, (const uint32_t *)codes, (const uint16_t *)scales, (const uint16_t *)zeros,
                       (u32x4 *)out, n_octets, group_shift);
    return hipGetLastError();
}

hipError_t run_dequant(bool is_int, const void *codes, const void *scales, const void *zeros, void *out,
                       int64_t N, int64_t K, int bits, int group, hipStream_t stream)
{
    if (is_int)
        return bits == 4   ? launch_dequant<4, true>(codes, scales, zeros, out, N, K, group, stream)
               : bits == 3 ? launch_dequant<3, true>(codes, scales, zeros, out, N, K, group, stream)
                           : launch_dequant<2, true>(codes, scales, zeros, out, N, K, group, stream);
    return bits == 4   ? launch_dequant<4, false>(codes, scales, zeros, out, N, K, group, stream)
           : bits == 3 ? launch_dequant<3, false>(codes, scales, zeros, out, N, K, group, stream)
                       : launch_dequant<2, false>(codes, scales, zeros, out, N, K, group, stream);
}

int dequant_max_batch() { return kMaxBatch; }

// items: `count` non-empty matrices (count <= kMaxBatch), already validated by the caller.
hipError_t run_dequant_batch(bool is_int, int count, const void *const *codes, const void *const *scales,
                             const void *const *zeros, void *const *out, const int64_t *N, const int64_t *K,
                             int bits, int group, hipStream_t stream)
{
    // largest matrix first: the workgroups of the small ones then fill the tail of the launch
    int order[kMaxBatch];
    for (int i = 0; i < count; ++i) order[i] = i;
    for (int i = 1; i < count; ++i)
        for (int j = i; j > 0 && N[order[j]] * K[order[j]] > N[order[j - 1]] * K[order[j - 1]]; --j) {
            const int t = order[j];
            order[j] = order[j - 1];
            order[j - 1] = t;
        }
    DequantBatch b;
    b.count = count;
    uint64_t blocks = 0;
    for (int i = 0; i < kMaxBatch; ++i) {
        const bool live = i < count;
        const int k = live ? order[i] : 0;
        DequantEntry &e = b.entry[i];
        e.codes = live ? (const uint32_t *)codes[k] : nullptr;
        e.scales = live ? (const uint16_t *)scales[k] : nullptr;
        e.zeros = (live && is_int) ? (const uint16_t *)zeros[k] : nullptr;
        e.out = live ? (u32x4 *)out[k] : nullptr;
        e.n_octets = live ? N[k] * K[k] / 8 : 0;
        e.first_block = (uint32_t)blocks;
        for (uint32_t &p : e.pad) p = 0;
        b.below[i] = (uint32_t)blocks - 1u;
        if (live) blocks += (uint64_t)dequant_blocks(e.n_octets, bits);
    }
    if (blocks == 0) return hipSuccess;
    if (blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const int group_shift = (group == 128) ? 7 : 6;
    const dim3 grid((unsigned)blocks), block((unsigned)dequant_block_threads(bits));
    if (is_int) {
        if (bits == 4) hipLaunchKernelGGL((dequant_batch_kernel<4, true>), grid, block, 0, stream, b, group_shift);
        else if (bits == 3) hipLaunchKernelGGL((dequant_batch_kernel<3, true>), grid, block, 0, stream, b, group_shift);
        else hipLaunchKernelGGL((dequant_batch_kernel<2, true>), grid, block, 0, stream, b, group_shift);
    } else {
        if (bits == 4) hipLaunchKernelGGL((dequant_batch_kernel<4, false>), grid, block, 0, stream, b, group_shift);
        else if (bits == 3) hipLaunchKernelGGL((dequant_batch_kernel<3, false>), grid, block, 0, stream, b, group_shift);
        else hipLaunchKernelGGL((dequant_batch_kernel<2, false>), grid, block, 0, stream, b, group_shift);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Scale-domain check: positive, normal, exponent field <= 30 - q_max.
// ---------------------------------------------------------------------------
__global__ void zero_count_kernel(unsigned long long *count) { *count = 0ull; }

__global__ __launch_bounds__(256) void check_scales_kernel(const uint16_t *__restrict__ scales, int64_t count,
                                                           int max_exp, unsigned long long *bad)
{
    unsigned long long local = 0;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count;
         i += (int64_t)gridDim.x * blockDim.x) {
        const uint32_t s = scales[i];
        const uint32_t e = (s >> 10) & 31u;
        local += ((s >> 15) != 0u) || e < 1u || e > (uint32_t)max_exp;
    }
    // wave-level sum, then one integer atomic per wave (integer adds commute: deterministic)
    for (int off = 32; off > 0; off >>= 1) local += __shfl_down(local, off, 64);
    if ((threadIdx.x & 63) == 0 && local) atomicAdd(bad, local);
}

hipError_t run_check_scales(const void *scales, int64_t count, int bits, void *bad_count_dev, hipStream_t stream)
{
    const int qmax = (1 << (bits - 1)) - 1;
    hipLaunchKernelGGL(zero_count_kernel, dim3(1), dim3(1), 0, stream, (unsigned long long *)bad_count_dev);
    if (count > 0) {
        int64_t blocks = (count + 255) / 256;
        if (blocks > 2048) blocks = 2048;
        hipLaunchKernelGGL(check_scales_kernel, dim3((unsigned)blocks), dim3(256), 0, stream,
                           (const uint16_t *)scales, count, 30 - qmax, (unsigned long long *)bad_count_dev);
    }
    return hipGetLastError();
}

// Zero-fill of `count` 16-bit words (results of products over an empty K).
__global__ __launch_bounds__(256) void fill_zero_kernel(uint16_t *p, int64_t count)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count;
         i += (int64_t)gridDim.x * blockDim.x)
        p[i] = 0;
}

hipError_t run_fill_zero(void *p, int64_t count, hipStream_t stream)
{
    int64_t blocks = (count + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, (uint16_t *)p, count);
    return hipGetLastError();
}

}  // namespace potq
