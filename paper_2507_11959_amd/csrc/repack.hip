// Layout conversion canonical <-> tile16 (a one-off pass when weights are loaded).
//
// One thread handles one (row, 32-column block): it reads the block's `bits`
// 32-bit words in one layout, moves every code to its place in the other and
// writes `bits` words.  The bit map of the tiled layout is documented in
// potq_device.hpp; the canonical layout is the dense little-endian bit stream
// along K.
#include "potq_device.hpp"

namespace potq {

// Column inside a block for selector m, byte lane j.
__device__ __forceinline__ int block_col(int m, int j)
{
    const int p = (j == 0) ? 0 : (j == 1) ? 2 : (j == 2) ? 1 : 3;
    return 4 * m + p;
}

template <int BITS>
__device__ __forceinline__ uint32_t stream_get(const uint32_t w[BITS], int i)
{
    const int pos = BITS * i;
    const int idx = pos >> 5, sh = pos & 31;
    uint32_t v = w[idx] >> sh;
    if (sh + BITS > 32) v |= w[idx + 1] << (32 - sh);
    return v & ((1u << BITS) - 1u);
}

template <int BITS>
__device__ __forceinline__ void stream_put(uint32_t w[BITS], int i, uint32_t c)
{
    const int pos = BITS * i;
    const int idx = pos >> 5, sh = pos & 31;
    w[idx] |= c << sh;
    if (sh + BITS > 32) w[idx + 1] |= c >> (32 - sh);
}

template <int BITS>
__device__ __forceinline__ uint32_t tile_get(const uint32_t w[BITS], int m, int j)
{
    if (BITS == 3) {
        if (m < 6) return (w[m >> 1] >> (8 * j + 3 * (m & 1))) & 7u;
        const uint32_t e = (w[m - 6] >> (8 * j + 6)) & 3u;
        const uint32_t s = (w[2] >> (8 * j + m)) & 1u;      // m = 6 -> bit 6, m = 7 -> bit 7
        return e | (s << 2);
    }
    if (BITS == 4) return (w[m >> 1] >> (8 * j + 4 * (m & 1))) & 15u;
    return (w[m >> 2] >> (8 * j + 2 * (m & 3))) & 3u;
}

template <int BITS>
__device__ __forceinline__ void tile_put(uint32_t w[BITS], int m, int j, uint32_t c)
{
    if (BITS == 3) {
        if (m < 6) {
            w[m >> 1] |= c << (8 * j + 3 * (m & 1));
        } else {
            w[m - 6] |= (c & 3u) << (8 * j + 6);
            w[2] |= (c >> 2) << (8 * j + m);
        }
    } else if (BITS == 4) {
        w[m >> 1] |= c << (8 * j + 4 * (m & 1));
    } else {
        w[m >> 2] |= c << (8 * j + 2 * (m & 3));
    }
}

template <int BITS, bool TO_TILED>
__global__ __launch_bounds__(256) void repack_kernel(const uint32_t *__restrict__ src, uint32_t *__restrict__ dst,
                                                     int64_t N, int64_t K)
{
    const int64_t blocks_per_row = K / 32;
    const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= N * blocks_per_row) return;
    // consecutive threads walk the tiled side contiguously: (tile, row, block)
    const int64_t tiles_per_rowtile = K / kTileCols;
    const int t = (int)(id & 3);
    const int r = (int)((id >> 2) & 15);
    const int64_t tile = id >> 6;
    const int64_t n = (tile / tiles_per_rowtile) * kTileRows + r;
    const int64_t blk = (tile % tiles_per_rowtile) * 4 + t;

    const int64_t canon = (n * blocks_per_row + blk) * BITS;           // word index of the block
    const int64_t tiled = tile * (BITS * 64) + r * 4 + t;              // word t of row r in slab 0

    uint32_t in[BITS], out[BITS];
#pragma unroll
    for (int i = 0; i < BITS; ++i) {
        in[i] = TO_TILED ? src[canon + i] : src[tiled + 64 * i];
        out[i] = 0;
    }
#pragma unroll
    for (int m = 0; m < 8; ++m)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (TO_TILED)
                tile_put<BITS>(out, m, j, stream_get<BITS>(in, block_col(m, j)));
            else
                stream_put<BITS>(out, block_col(m, j), tile_get<BITS>(in, m, j));
        }
#pragma unroll
    for (int i = 0; i < BITS; ++i) {
        if (TO_TILED)
            dst[tiled + 64 * i] = out[i];
        else
            dst[canon + i] = out[i];
    }
}

hipError_t run_repack(const void *src, void *dst, int64_t N, int64_t K, int bits, bool to_tiled, hipStream_t stream)
{
    const int64_t threads = N * (K / 32);
    const unsigned blocks = (unsigned)((threads + 255) / 256);
    const uint32_t *s = (const uint32_t *)src;
    uint32_t *d = (uint32_t *)dst;
    if (bits == 4) {
        if (to_tiled)
            hipLaunchKernelGGL((repack_kernel<4, true>), dim3(blocks), dim3(256), 0, stream, s, d, N, K);
        else
            hipLaunchKernelGGL((repack_kernel<4, false>), dim3(blocks), dim3(256), 0, stream, s, d, N, K);
    } else if (bits == 3) {
        if (to_tiled)
            hipLaunchKernelGGL((repack_kernel<3, true>), dim3(blocks), dim3(256), 0, stream, s, d, N, K);
        else
            hipLaunchKernelGGL((repack_kernel<3, false>), dim3(blocks), dim3(256), 0, stream, s, d, N, K);
    } else {
        if (to_tiled)
            hipLaunchKernelGGL((repack_kernel<2, true>), dim3(blocks), dim3(256), 0, stream, s, d, N, K);
        else
            hipLaunchKernelGGL((repack_kernel<2, false>), dim3(blocks), dim3(256), 0, stream, s, d, N, K);
    }
    return hipGetLastError();
}

}  // namespace potq
