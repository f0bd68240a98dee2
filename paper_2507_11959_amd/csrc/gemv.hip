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
//
// The same file holds the fused GEMM for up to 16 tokens (gemm_fewtok_kernel),
// which keeps this lane-owns-a-group scheme and makes the tokens the B operand.
#include <type_traits>

#include "potq_device.hpp"
#include "potq_launch.hpp"

namespace potq {

// One group (128 columns) of one row: codes in L, table from (s, z), x in LDS.
// Eight weights at a time become the A operand (row = lane % 16, k-slice =
// lane / 16) of v_mfma_f32_16x16x32_f16; the B operand is the matching eight x
// values, the same in all 16 columns, so every column of the 16x16 result holds
// the partial products of the 16 rows.  Products are exact, sums fp32.
// `s`/`z` serve columns 0..63, `s_hi`/`z_hi` columns 64..127 (the same values for group size 128).
// `bfrag(j)` returns the B operand of step j (j = 0..15: columns 8j .. 8j+7 of the group).
template <int BITS, bool IS_INT, int NCOL, typename BFrag>
__device__ __forceinline__ void gemv_group(const u32x4 (&L)[BITS], uint32_t s, uint32_t z, uint32_t s_hi,
                                           uint32_t z_hi, bool two_scales, BFrag bfrag, float4_t (&acc)[4])
{
    Decoder<BITS, IS_INT> dec;
    // The B operand of a block's four steps.  With NCOL > 0 only the first NCOL columns of the
    // result are used (the GEMV: column 0), so only the lanes of those columns fetch it -- an LDS
    // read returns 16 bytes per active lane, and the other lanes' share is wasted bandwidth.  The fetch of the
    // next block is issued before the current block is expanded.
    const bool fetches = NCOL == 0 || (int)(threadIdx.x & 15) < NCOL;
    u32x4 xq[4], xn[4];
    if (fetches) {
#pragma unroll
        for (int i = 0; i < 4; ++i) xq[i] = bfrag(i);
    }
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        if (b == 0 || (b == 2 && two_scales))       // wave-uniform: the second table exists only for group size 64
            dec.set_group(b ? s_hi : s, b ? z_hi : z);
        if (b < 3 && fetches) {
#pragma unroll
            for (int i = 0; i < 4; ++i) xn[i] = bfrag((b + 1) * 4 + i);
        }
        uint32_t w[BITS];
#pragma unroll
        for (int j = 0; j < BITS; ++j) w[j] = L[j][b];
        dec.set_block(w);
#pragma unroll
        for (int m = 0; m < 8; m += 2) {
            const u32x4 xv = xq[m / 2];             // columns 32b + 4m .. + 7
            uint32_t e0, o0, e1, o1;
            dec.get(m, e0, o0);
            dec.get(m + 1, e1, o1);
            const half8_t av = __builtin_bit_cast(half8_t, (u32x4{e0, o0, e1, o1}));
            acc[m / 2] = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, __builtin_bit_cast(half8_t, xv), acc[m / 2], 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) xq[i] = xn[i];
    }
}

constexpr int kXRun = 17;   // uint4 per scale group of x in LDS (16 + 1 of padding)
constexpr int kGemvWaves = 8;

// A workgroup of 8 wavefronts stages x in LDS once and serves 8/S row tiles of 16
// rows.  S wavefronts share a tile and split its scale groups: wavefront part p,
// lane group t takes groups 4p + t, 4p + t + 4S, ...  Long rows want S = 8 (all
// of K in flight at once), tall matrices want S = 1 or 2 (long-lived wavefronts,
// no cross-wavefront sums).  The codes of the next round are requested before
// the current one is expanded; the first request goes out right after the request for x and
// before x is written to LDS.
// MT > 1: the same kernel for MT activation vectors at once (a GEMM with two to four tokens: rows
// m < tokens of x, K apart; results y[m * ystride + n]).  Vector m is the B operand of column m, so the
// matrix is decoded once and every vector costs only LDS space: column m of the MFMA result is its y.
template <int BITS, bool IS_INT, int S, bool G64, bool COL0, int MT = 1>
__device__ __forceinline__ void gemv_tile16_body(
    const u32x4 *__restrict__ codes, const uint16_t *__restrict__ scales, const uint16_t *__restrict__ zeros,
    const u32x4 *__restrict__ x, uint16_t *__restrict__ y, int64_t rowtiles, int K, int64_t block, int tokens = 1,
    int64_t ystride = 0)
{
    constexpr int gs = G64 ? 1 : 0;
    // gs = 0: one scale per 128 columns; gs = 1: one per 64 (two per tile row)
    constexpr int R = kGemvWaves / S;                   // row tiles per workgroup
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
    constexpr int kStep = 4 * S;
    const int part = wave % S;
    int64_t rowtile = block * R + wave / S;
    const bool live = rowtile < rowtiles;
    if (!live) rowtile = rowtiles - 1;                  // surplus wavefronts redo the last tile, store nothing
    const int64_t row = rowtile * kTileRows + r;
    const u32x4 *tile0 = codes + rowtile * G * (BITS * 16) + r;
    // Scales are fetched in memory order -- lane l takes row l/4, group (first group of the
    // round) + l%4, so four consecutive lanes share one 64-byte line, which is the unit the
    // L1 processes per cycle -- and a cross-lane permute hands lane (r, t) its own scale.
    const uint16_t *srow = scales + (rowtile * kTileRows + (lane >> 2)) * G;
    const uint16_t *zrow = IS_INT ? zeros + (rowtile * kTileRows + (lane >> 2)) * G : nullptr;
    const int scale_owner = (4 * r + t) * 4;            // ds_bpermute byte address
    // group size 64: lane (r, t) reads its own two scales as one 32-bit word (less well coalesced)
    const uint32_t *srow2 = (const uint32_t *)(scales + row * (int64_t)(2 * G));
    const uint32_t *zrow2 = IS_INT ? (const uint32_t *)(zeros + row * (int64_t)(2 * G)) : nullptr;

    // MFMA ignores the execution mask, so the group loop must be uniform: every
    // lane runs ceil(G / kStep) rounds.  A lane whose group index runs past G
    // re-reads the last group (valid memory), takes the scale 1.0 (finite
    // weights) and multiplies by a block of zeros instead of x.
    const int rounds = (G + kStep - 1) / kStep;
    u32x4 *zero_block = smem + MT * (K / kTileCols) * kXRun;   // 16 uint4 of zeros
    float *red = (float *)(zero_block + 16);            // 8 wavefronts x MT x 16 partial sums

    // Activations first: loads return in order, and x (from the L2) has to be in LDS before the
    // barrier, while the codes (from HBM) are not needed until after it.  The first pieces of
    // every thread (all of x up to K = 8192) are requested here and written once the codes of
    // the first round have been requested too; longer rows take the rest afterwards.
    // Vector m occupies runs m*G .. m*G + G-1; vectors past `tokens` count as zero.
    constexpr int kXFirst = 2;
    constexpr int kThreads = kGemvWaves * kWave;
    const int per = K / 8, pieces = MT * per;
    auto x_piece = [&](int i) {
        const int m = MT == 1 ? 0 : i / per;
        return (i < pieces && m < tokens) ? x[i] : u32x4{0u, 0u, 0u, 0u};
    };
    auto x_slot = [&](int i) {
        const int m = MT == 1 ? 0 : i / per, o = i - m * per;
        return (m * G + (o >> 4)) * kXRun + (o & 15);
    };
    u32x4 xfirst[kXFirst];
#pragma unroll
    for (int u = 0; u < kXFirst; ++u) xfirst[u] = x_piece(tid + u * kThreads);

    int g = part * 4 + t;
    u32x4 L[BITS];
    uint32_t s, z = 0;       // raw loads (memory order); permuted to their owners when consumed
    {
        const int gc = g < G ? g : G - 1;
#pragma unroll
        for (int j = 0; j < BITS; ++j) L[j] = __builtin_nontemporal_load(tile0 + (int64_t)gc * (BITS * 16) + 16 * j);
        if (gs) {
            s = srow2[gc];
            if (IS_INT) z = zrow2[gc];
        } else {
            const int gq = min(part * 4 + (lane & 3), G - 1);
            s = srow[gq];
            if (IS_INT) z = zrow[gq];
        }
    }

#pragma unroll
    for (int u = 0; u < kXFirst; ++u)
        if (tid + u * kThreads < pieces) xs[x_slot(tid + u * kThreads)] = xfirst[u];
    for (int i = tid + kXFirst * kThreads; i < pieces; i += kThreads) xs[x_slot(i)] = x_piece(i);
    if (tid < 16) zero_block[tid] = u32x4{0u, 0u, 0u, 0u};
    __syncthreads();

    float4_t acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = float4_t{0.f, 0.f, 0.f, 0.f};
    // One round; `request` says whether the codes of the next round are asked for first.  The
    // wavefront's last round has no successor: it is taken out of the loop, so that a launch
    // whose wavefronts have a single round (K = 4096) issues no second request at all -- a
    // request nobody consumes still keeps the wavefront alive until it returns.
    auto step = [&](int round, auto request) {
        const int gn = g + kStep;
        u32x4 Ln[BITS];
        uint32_t sn = 0, zn = 0;
        if constexpr (decltype(request)::value) {
            const int gc = gn < G ? gn : G - 1;         // a lane past the end of the row: the last group, times zeros
#pragma unroll
            for (int j = 0; j < BITS; ++j)
                Ln[j] = __builtin_nontemporal_load(tile0 + (int64_t)gc * (BITS * 16) + 16 * j);
            if (gs) {
                sn = srow2[gc];
                if (IS_INT) zn = zrow2[gc];
            } else {
                const int gq = min(part * 4 + (round + 1) * kStep + (lane & 3), G - 1);
                sn = srow[gq];
                if (IS_INT) zn = zrow[gq];
            }
        }
        uint32_t so, zo = 0u, so_hi, zo_hi = 0u;
        if (gs) {
            so = s & 0xFFFFu;
            so_hi = s >> 16;
            if (IS_INT) {
                zo = z & 0xFFFFu;
                zo_hi = z >> 16;
            }
        } else {
            so = (uint32_t)__builtin_amdgcn_ds_bpermute(scale_owner, (int)s);
            if (IS_INT) zo = (uint32_t)__builtin_amdgcn_ds_bpermute(scale_owner, (int)z);
            so_hi = so;
            zo_hi = zo;
        }
        if (g >= G) {
            so = so_hi = 0x3C00u;
            zo = zo_hi = 0u;
        }
        // column c of the B operand: vector c (vector 0 in the columns that are not used)
        const int vec = (MT > 1 && r < MT) ? r : 0;
        const u32x4 *xg = g < G ? xs + (vec * G + g) * kXRun : zero_block;
        gemv_group<BITS, IS_INT, (MT > 1 ? MT : (COL0 ? 1 : 0))>(L, so, zo, so_hi, zo_hi, gs != 0,
                                                               [&](int j) { return xg[j]; }, acc);
        g = gn;
        if constexpr (decltype(request)::value) {
#pragma unroll
            for (int j = 0; j < BITS; ++j) L[j] = Ln[j];
            s = sn;
            z = zn;
        }
    };
    // rounds in which this wavefront has a group (wave-uniform; K = 5120 has 40 groups for 64 slots
    // of two rounds: the wavefronts of parts 2..7 have one round)
    const int my_rounds = min(rounds, (G - part * 4 + kStep - 1) / kStep);
    for (int round = 0; round + 1 < my_rounds; ++round) step(round, std::true_type{});
    if (my_rounds > 0) step(my_rounds - 1, std::false_type{});

    // The MFMA already summed the four lane groups.  Lane (c, q) holds rows 4q..4q+3
    // (identical in every column c); combine the S wavefronts of a tile in a fixed order.
    const float4_t part_sum = (acc[0] + acc[1]) + (acc[2] + acc[3]);
    if (S == 1) {
        if (live && r == 0) {
            typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
            half4_t h;
#pragma unroll
            for (int i = 0; i < 4; ++i) h[i] = (_Float16)part_sum[i];
            *(half4_t *)(y + rowtile * kTileRows + 4 * t) = h;
        }
        return;
    }
    if (r < MT) *(float4_t *)(red + (wave * MT + r) * kTileRows + 4 * t) = part_sum;
    __syncthreads();
    if (tid < R * MT * kTileRows) {
        const int tile = tid / (MT * kTileRows), m = (tid / kTileRows) % MT, rr = tid % kTileRows;
        const int64_t rt = block * R + tile;
        float sum = 0.f;
#pragma unroll
        for (int p = 0; p < S; ++p) sum += red[((tile * S + p) * MT + m) * kTileRows + rr];
        const _Float16 h = (_Float16)sum;
        if (rt < rowtiles && m < tokens) y[m * ystride + rt * kTileRows + rr] = __builtin_bit_cast(uint16_t, h);
    }
}

template <int BITS, bool IS_INT, int S, bool G64, bool COL0>
__global__ __launch_bounds__(kGemvWaves * kWave) void gemv_tile16_kernel(
    const u32x4 *__restrict__ codes, const uint16_t *__restrict__ scales, const uint16_t *__restrict__ zeros,
    const u32x4 *__restrict__ x, uint16_t *__restrict__ y, int64_t rowtiles, int K)
{
    gemv_tile16_body<BITS, IS_INT, S, G64, COL0>(codes, scales, zeros, x, y, rowtiles, K, blockIdx.x);
}

// The GEMV for large matrices: the same arithmetic, in the same order, as gemv_tile16_kernel with
// eight wavefronts per tile, but a workgroup stages x once and walks the row tiles first,
// first + stride, ...; the codes of the next step -- the next round of the tile or the first
// round of the next tile -- are requested before the current ones are expanded, so the memory
// traffic of a wavefront never pauses at a tile boundary, and the grid is no larger than what
// the chip holds at once.  (The exponent-form kernel of gemv_exp.hip is built the same way;
// this one serves what that one cannot: the uniform baseline and 4-bit codes.)
template <int BITS, bool IS_INT, bool G64, bool COL0>
__global__ __launch_bounds__(kGemvWaves * kWave) void gemv_tile16_walk_kernel(
    const u32x4 *__restrict__ codes, const uint16_t *__restrict__ scales, const uint16_t *__restrict__ zeros,
    const u32x4 *__restrict__ x, uint16_t *__restrict__ y, int64_t rowtiles, int K)
{
    static_assert(kGemvWaves == 8, "eight wavefronts share a tile");
    constexpr int gs = G64 ? 1 : 0;
    constexpr int kStep = 4 * kGemvWaves;
    extern __shared__ u32x4 smem[];
    u32x4 *xs = smem;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int part = __builtin_amdgcn_readfirstlane(tid >> 6);   // wavefront index: uniform, kept in a scalar
    const int r = lane & 15;
    const int t = lane >> 4;
    const int G = K / kTileCols;
    const int scale_owner = (4 * r + t) * 4;
    const int my_rounds = (G - part * 4 + kStep - 1) / kStep;   // G >= 32: at least one
    u32x4 *zero_block = smem + G * kXRun;               // 16 uint4 of zeros
    float *red = (float *)(zero_block + 16);            // 2 x 8 wavefronts x 16 partial sums
    const int64_t first = blockIdx.x, stride = gridDim.x;

    auto fetch = [&](int64_t tile, int round, u32x4 (&Lx)[BITS], uint32_t &sx, uint32_t &zx) {
        const int g0 = round * kStep + part * 4;                        // uniform
        const int gc = min(g0 + t, G - 1);
        const u32x4 *tile_codes = codes + tile * G * (BITS * 16);       // uniform
        const uint32_t at = (uint32_t)(gc * (BITS * 16) + r);
#pragma unroll
        for (int j = 0; j < BITS; ++j) Lx[j] = __builtin_nontemporal_load(tile_codes + at + 16 * j);
        zx = 0u;
        if (gs) {
            const uint32_t i = (uint32_t)(r * G + gc);
            sx = ((const uint32_t *)(scales + tile * kTileRows * (int64_t)(2 * G)))[i];
            if (IS_INT) zx = ((const uint32_t *)(zeros + tile * kTileRows * (int64_t)(2 * G)))[i];
        } else {
            const uint32_t i = (uint32_t)((lane >> 2) * G + min(g0 + (lane & 3), G - 1));
            sx = (scales + tile * kTileRows * (int64_t)G)[i];
            if (IS_INT) zx = (zeros + tile * kTileRows * (int64_t)G)[i];
        }
    };
    int64_t ftile = first;
    int fround = 0;
    auto advance = [&]() {
        if (fround + 1 < my_rounds) {
            ++fround;
        } else if (ftile + stride < rowtiles) {
            ftile += stride;
            fround = 0;
        }
    };
    u32x4 L[BITS];
    uint32_t s, z;
    fetch(ftile, fround, L, s, z);
    advance();

    for (int i = tid; i < K / 8; i += kGemvWaves * kWave) xs[(i >> 4) * kXRun + (i & 15)] = x[i];
    if (tid < 16) zero_block[tid] = u32x4{0u, 0u, 0u, 0u};
    __syncthreads();

    int it = 0;
    for (int64_t tile = first; tile < rowtiles; tile += stride, ++it) {
        float4_t acc[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] = float4_t{0.f, 0.f, 0.f, 0.f};
        for (int round = 0; round < my_rounds; ++round) {
            u32x4 Ln[BITS];
            uint32_t sn, zn;
            fetch(ftile, fround, Ln, sn, zn);
            advance();
            const int g = round * kStep + part * 4 + t;
            uint32_t so, zo = 0u, so_hi, zo_hi = 0u;
            if (gs) {
                so = s & 0xFFFFu;
                so_hi = s >> 16;
                if (IS_INT) {
                    zo = z & 0xFFFFu;
                    zo_hi = z >> 16;
                }
            } else {
                so = (uint32_t)__builtin_amdgcn_ds_bpermute(scale_owner, (int)s);
                if (IS_INT) zo = (uint32_t)__builtin_amdgcn_ds_bpermute(scale_owner, (int)z);
                so_hi = so;
                zo_hi = zo;
            }
            if (g >= G) {                               // past the end of the row: finite weights times zeros
                so = so_hi = 0x3C00u;
                zo = zo_hi = 0u;
            }
            const u32x4 *xg = g < G ? xs + g * kXRun : zero_block;
            gemv_group<BITS, IS_INT, (COL0 ? 1 : 0)>(L, so, zo, so_hi, zo_hi, gs != 0, [&](int j) { return xg[j]; }, acc);
#pragma unroll
            for (int j = 0; j < BITS; ++j) L[j] = Ln[j];
            s = sn;
            z = zn;
        }
        // as in gemv_tile16_kernel: lane (c, q) holds rows 4q..4q+3; the eight wavefronts' sums are
        // added in a fixed order.  The buffer alternates between tiles, so one barrier per tile
        // separates the writes of tile i + 2 from the reads of tile i.
        const float4_t part_sum = (acc[0] + acc[1]) + (acc[2] + acc[3]);
        float *red_it = red + (it & 1) * (kGemvWaves * kTileRows);
        if (r == 0) *(float4_t *)(red_it + part * kTileRows + 4 * t) = part_sum;
        __syncthreads();
        if (tid < kTileRows) {
            float sum = 0.f;
#pragma unroll
            for (int p = 0; p < kGemvWaves; ++p) sum += red_it[p * kTileRows + tid];
            const _Float16 h = (_Float16)sum;
            y[tile * kTileRows + tid] = __builtin_bit_cast(uint16_t, h);
        }
    }
}

// Several matrices that consume the same activation vector (q/k/v, gate/up) in one launch:
// a batch-1 GEMV on a 4096x4096 matrix is a 4 us kernel of which most is launch and memory
// latency, so sharing one launch pays more than anything inside the kernel.
constexpr int kMaxGemvBatch = 16;
struct GemvBatch {
    const u32x4 *codes[kMaxGemvBatch];
    const uint16_t *scales[kMaxGemvBatch];
    const uint16_t *zeros[kMaxGemvBatch];
    uint16_t *y[kMaxGemvBatch];
    int64_t rowtiles[kMaxGemvBatch];
    uint32_t first_block[kMaxGemvBatch + 1];
    int count;
};

template <int BITS, bool IS_INT, int S, bool G64, bool COL0>
__global__ __launch_bounds__(kGemvWaves * kWave) void gemv_tile16_batch_kernel(
    const GemvBatch batch, const u32x4 *__restrict__ x, int K)
{
    int i = 0;
    while (i + 1 < batch.count && blockIdx.x >= batch.first_block[i + 1]) ++i;   // uniform: scalar code
    gemv_tile16_body<BITS, IS_INT, S, G64, COL0>(batch.codes[i], batch.scales[i], batch.zeros[i], x, batch.y[i],
                                           batch.rowtiles[i], K, blockIdx.x - batch.first_block[i]);
}

// ---------------------------------------------------------------------------
// Fused GEMM for at most 16 tokens (batched decoding), built like the GEMV:
// lane (r, t) owns row r of one scale group (16-byte code loads, one table per
// 128 weights, no cross-lane traffic for the codes), and the B operand of the
// MFMA holds the 16 tokens instead of 16 copies of x, so all 256 results of
// v_mfma_f32_16x16x32_f16 are used: D[row][token].
//
// A workgroup of 8 (16) wavefronts serves 2 (4) row tiles; the 4 wavefronts of a
// tile take 4 consecutive groups each, so a round of the workgroup covers 16
// groups (2048 columns).  The X chunk of a round (16 tokens x 2048 columns, 64 KB) sits
// in LDS as [group][step][token] 16-byte runs, the token index rotated by
// 4 * (step % 4) so that the staging writes (a quad of lanes holds four
// consecutive runs of one token) spread over the banks.  The chunk of the next
// round travels through registers while the current one is consumed.
// ---------------------------------------------------------------------------
constexpr int kFewSplit = 4;                          // wavefronts per row tile
constexpr int kFewChunk = 4 * kFewSplit;              // scale groups per round
constexpr int kFewDepth = 1;                          // rounds of codes requested ahead (two or three measured no better)

template <int BITS, bool IS_INT, bool G64, int kFewWaves>
__global__ __launch_bounds__(kFewWaves * kWave)
__attribute__((amdgpu_waves_per_eu(kFewWaves == 16 ? 4 : 1, kFewWaves == 16 ? 4 : 8))) void gemm_fewtok_kernel(
    const u32x4 *__restrict__ codes, const uint16_t *__restrict__ scales, const uint16_t *__restrict__ zeros,
    const uint16_t *__restrict__ X, uint16_t *__restrict__ Y, int M, int64_t N, int K)
{
    constexpr int gs = G64 ? 1 : 0;
    constexpr int R = kFewWaves / kFewSplit;
    constexpr int kFewPieces = kFewChunk * 256 / (kFewWaves * kWave);   // 16-byte X pieces per thread and round
    extern __shared__ u32x4 smem[];                     // [16 groups][16 steps][16 tokens]

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid >> 6;
    const int r = lane & 15;
    const int t = lane >> 4;
    const int G = K / kTileCols;
    const int64_t rowtiles = N / kTileRows;
    const int part = wave % kFewSplit;
    int64_t rowtile = (int64_t)blockIdx.x * R + wave / kFewSplit;
    const bool live = rowtile < rowtiles;
    if (!live) rowtile = rowtiles - 1;                  // surplus wavefronts redo the last tile, store nothing
    const int64_t row = rowtile * kTileRows + r;
    const u32x4 *tile0 = codes + rowtile * G * (BITS * 16) + r;
    const uint16_t *srow = scales + (rowtile * kTileRows + (lane >> 2)) * G;
    const uint16_t *zrow = IS_INT ? zeros + (rowtile * kTileRows + (lane >> 2)) * G : nullptr;
    const int scale_owner = (4 * r + t) * 4;
    const uint32_t *srow2 = (const uint32_t *)(scales + row * (int64_t)(2 * G));
    const uint32_t *zrow2 = IS_INT ? (const uint32_t *)(zeros + row * (int64_t)(2 * G)) : nullptr;
    const int rounds = (G + kFewChunk - 1) / kFewChunk;

    struct Fetched {
        u32x4 L[BITS];
        uint32_t s, z;
    };
    auto fetch = [&](int rnd, Fetched &f) {             // indices clamped into the matrix, as in the GEMV
        const int gc = min(rnd * kFewChunk + part * 4 + t, G - 1);
#pragma unroll
        for (int j = 0; j < BITS; ++j)
            f.L[j] = __builtin_nontemporal_load(tile0 + (int64_t)gc * (BITS * 16) + 16 * j);
        f.z = 0;
        if (gs) {
            f.s = srow2[gc];
            if (IS_INT) f.z = zrow2[gc];
        } else {
            const int gq = min(rnd * kFewChunk + part * 4 + (lane & 3), G - 1);
            f.s = srow[gq];
            if (IS_INT) f.z = zrow[gq];
        }
    };

    // X pieces of this thread: piece p = tid + (threads) i is run (p % 4) + 4 (p/64 % 4) of group p/256
    // for token (p/4) % 16 -- four consecutive lanes read 64 contiguous bytes of one token.  The
    // thread count is a multiple of 256, so token and run are the same for all pieces of a thread
    // and piece i lies kFewWaves/4 groups after piece i - 1: one address, one slot, constant steps.
    constexpr int kPieceGroups = kFewWaves / 4;         // groups between consecutive pieces of a thread
    const int xrun = (wave & 3) * 4 + (tid & 3);        // run of 8 columns inside the group
    const int xc = (tid >> 2) & 15;                     // token
    const int xgrp0 = wave >> 2;                        // group of piece 0 inside the chunk
    const bool xtok = xc < M;
    const uint16_t *xsrc = X + (int64_t)(xtok ? xc : 0) * K + 8 * xrun;
    const int xslot0 = (xgrp0 * 16 + xrun) * 16 + ((xc + 4 * (tid & 3)) & 15);
    u32x4 xr[kFewPieces];
    auto fetch_x = [&](int rnd) {
#pragma unroll
        for (int i = 0; i < kFewPieces; ++i) {
            const int g = rnd * kFewChunk + xgrp0 + kPieceGroups * i;
            // tokens past M and groups past K count as zero, and are not requested
            u32x4 v = u32x4{0u, 0u, 0u, 0u};
            if (xtok && g < G) v = *(const u32x4 *)(xsrc + (int64_t)g * kTileCols);
            xr[i] = v;
        }
    };
    // B operand of step j for lane (token r, k-slice t): group 4*part + t of the chunk
    const u32x4 *xq[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) xq[k] = smem + (part * 4 + t) * 256 + ((r + 4 * k) & 15);

    Fetched q[kFewDepth];                               // rounds of codes in flight ahead of the arithmetic
    fetch_x(0);
#pragma unroll
    for (int d = 0; d < kFewDepth; ++d) fetch(d, q[d]);

    float4_t acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = float4_t{0.f, 0.f, 0.f, 0.f};
    for (int round = 0; round < rounds; ++round) {
        if (round) __syncthreads();                     // the previous chunk has been consumed
#pragma unroll
        for (int i = 0; i < kFewPieces; ++i) smem[xslot0 + kPieceGroups * 256 * i] = xr[i];
        __syncthreads();
        // X first: loads return in order, and the chunk (from L2) is wanted at the top of the next round,
        // before the codes (from HBM) are
        fetch_x(round + 1);                             // past the end: nothing is requested
        Fetched nx;
        fetch(round + kFewDepth, nx);
        const Fetched &cur = q[0];

        const int g = round * kFewChunk + part * 4 + t;
        uint32_t so, zo = 0u, so_hi, zo_hi = 0u;
        if (gs) {
            so = cur.s & 0xFFFFu;
            so_hi = cur.s >> 16;
            if (IS_INT) {
                zo = cur.z & 0xFFFFu;
                zo_hi = cur.z >> 16;
            }
        } else {
            so = (uint32_t)__builtin_amdgcn_ds_bpermute(scale_owner, (int)cur.s);
            if (IS_INT) zo = (uint32_t)__builtin_amdgcn_ds_bpermute(scale_owner, (int)cur.z);
            so_hi = so;
            zo_hi = zo;
        }
        if (g >= G) {                                   // finite weights against a zero B operand
            so = so_hi = 0x3C00u;
            zo = zo_hi = 0u;
        }
        gemv_group<BITS, IS_INT, 0>(cur.L, so, zo, so_hi, zo_hi, gs != 0, [&](int j) { return xq[j & 3][j * 16]; }, acc);
#pragma unroll
        for (int d = 0; d + 1 < kFewDepth; ++d) q[d] = q[d + 1];
        q[kFewDepth - 1] = nx;
    }

    // D: lane (c, q) holds token c, rows 4q .. 4q+3.  Add the four wavefronts of a tile in a fixed order.
    float4_t *red = (float4_t *)smem;
    const float4_t part_sum = (acc[0] + acc[1]) + (acc[2] + acc[3]);
    __syncthreads();                                    // every wavefront is done with the X chunk
    red[wave * kWave + lane] = part_sum;
    __syncthreads();
    if (part != 0 || !live || r >= M) return;
    float4_t sum = red[wave * kWave + lane];
#pragma unroll
    for (int p = 1; p < kFewSplit; ++p) sum += red[(wave + p) * kWave + lane];
    typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
    half4_t h;
#pragma unroll
    for (int i = 0; i < 4; ++i) h[i] = (_Float16)sum[i];
    *(half4_t *)(Y + (int64_t)r * N + rowtile * kTileRows + 4 * t) = h;
}

template <int BITS, bool IS_INT, bool G64, int WAVES>
static void launch_gemm_fewtok_cfg(const void *codes, const void *scales, const void *zeros, const void *X, void *Y,
                                   int64_t M, int64_t N, int64_t K, hipStream_t stream)
{
    const int64_t rowtiles = N / kTileRows;
    constexpr int R = WAVES / kFewSplit;
    const dim3 grid((unsigned)((rowtiles + R - 1) / R)), block(WAVES * kWave);
    const size_t lds = (size_t)kFewChunk * 256 * sizeof(u32x4);
    hipLaunchKernelGGL((gemm_fewtok_kernel<BITS, IS_INT, G64, WAVES>), grid, block, lds, stream, (const u32x4 *)codes,
                       (const uint16_t *)scales, (const uint16_t *)zeros, (const uint16_t *)X, (uint16_t *)Y, (int)M, N,
                       (int)K);
}

// Workgroups of 16 wavefronts (four row tiles share every X chunk, one workgroup per compute unit)
// or of 8 (two row tiles, two workgroups per compute unit): either way the chip takes 1024 row
// tiles at a time.  Sixteen are faster while the last such round is more than half full (11008 x
// 4096: 8.8 against 11.0 us, 13824 x 5120: 11.9 / 14.5, 28672 x 8192: 31.0 / 35.0); when it is not,
// they leave half of the compute units idle in it and eight win (8192 x 8192: 11.6 against 13.9 us,
// 5120 x 5120: 8.1 / 10.8, 17920 x 6656: 25.0 / 27.0, 24576 x 4096: 15.8 / 17.4).
static bool fewtok_sixteen_wavefronts(int64_t N)
{
    const int64_t in_last_round = (N / kTileRows) % 1024;
    return in_last_round == 0 || in_last_round > 512;
}

template <int BITS, bool IS_INT>
static void launch_gemm_fewtok(const void *codes, const void *scales, const void *zeros, const void *X, void *Y,
                               int64_t M, int64_t N, int64_t K, int group, hipStream_t stream)
{
    const bool tall = fewtok_sixteen_wavefronts(N);
    if (group == 64) {
        if (tall) launch_gemm_fewtok_cfg<BITS, IS_INT, true, 16>(codes, scales, zeros, X, Y, M, N, K, stream);
        else launch_gemm_fewtok_cfg<BITS, IS_INT, true, 8>(codes, scales, zeros, X, Y, M, N, K, stream);
    } else {
        if (tall) launch_gemm_fewtok_cfg<BITS, IS_INT, false, 16>(codes, scales, zeros, X, Y, M, N, K, stream);
        else launch_gemm_fewtok_cfg<BITS, IS_INT, false, 8>(codes, scales, zeros, X, Y, M, N, K, stream);
    }
}

// M <= 16 tokens, tiled layout.
hipError_t run_gemm_fewtok(bool is_int, const void *codes, const void *scales, const void *zeros, const void *X,
                           void *Y, int64_t M, int64_t N, int64_t K, int bits, int group, hipStream_t stream)
{
    if (is_int) {
        if (bits == 4) launch_gemm_fewtok<4, true>(codes, scales, zeros, X, Y, M, N, K, group, stream);
        else if (bits == 3) launch_gemm_fewtok<3, true>(codes, scales, zeros, X, Y, M, N, K, group, stream);
        else launch_gemm_fewtok<2, true>(codes, scales, zeros, X, Y, M, N, K, group, stream);
    } else {
        if (bits == 4) launch_gemm_fewtok<4, false>(codes, scales, zeros, X, Y, M, N, K, group, stream);
        else if (bits == 3) launch_gemm_fewtok<3, false>(codes, scales, zeros, X, Y, M, N, K, group, stream);
        else launch_gemm_fewtok<2, false>(codes, scales, zeros, X, Y, M, N, K, group, stream);
    }
    return hipGetLastError();
}

// Two to four tokens through the GEMV kernel (eight wavefronts per tile, group size 128).
template <int BITS, bool IS_INT, int MT>
__global__ __launch_bounds__(kGemvWaves * kWave) void gemv_tile16_multi_kernel(
    const u32x4 *__restrict__ codes, const uint16_t *__restrict__ scales, const uint16_t *__restrict__ zeros,
    const u32x4 *__restrict__ X, uint16_t *__restrict__ Y, int64_t rowtiles, int K, int tokens, int64_t N)
{
    gemv_tile16_body<BITS, IS_INT, 8, false, false, MT>(codes, scales, zeros, X, Y, rowtiles, K, blockIdx.x, tokens, N);
}

static size_t gemv_multi_lds_bytes(int64_t K, int mt)
{
    return (size_t)mt * (K / kTileCols) * kXRun * 16 + 256 + (size_t)kGemvWaves * mt * kTileRows * sizeof(float);
}

// Whether run_gemv_multi serves this shape: 2..4 tokens, group 128, rows long enough for eight
// wavefronts per tile, the padded vectors within 64 KB of LDS, and not three or four vectors
// where the few-token kernel runs its sixteen-wavefront workgroups (13824 x 5120 at four tokens:
// 13.1 us against 11.4 us for the few-token kernel, 11008 x 4096: 9.8 against 8.8; elsewhere
// the GEMV kernel measured 1.1-1.8x faster than the few-token kernel at two to four tokens).
bool gemv_multi_ok(int64_t M, int64_t N, int64_t K, int group)
{
    const int64_t G = K / kTileCols;
    if (M < 2 || M > 4 || group != 128 || kGemvWaves != 8 || G < 32) return false;
    if (M > 2 && fewtok_sixteen_wavefronts(N)) return false;
    return gemv_multi_lds_bytes(K, M <= 2 ? 2 : 4) <= 64 * 1024;
}

template <int BITS, bool IS_INT>
static void launch_gemv_multi(const void *codes, const void *scales, const void *zeros, const void *X, void *Y,
                              int64_t M, int64_t N, int64_t K, hipStream_t stream)
{
    const int64_t rowtiles = N / kTileRows;
    const dim3 grid((unsigned)rowtiles), block(kGemvWaves * kWave);
    if (M <= 2)
        hipLaunchKernelGGL((gemv_tile16_multi_kernel<BITS, IS_INT, 2>), grid, block, gemv_multi_lds_bytes(K, 2), stream,
                           (const u32x4 *)codes, (const uint16_t *)scales, (const uint16_t *)zeros, (const u32x4 *)X,
                           (uint16_t *)Y, rowtiles, (int)K, (int)M, N);
    else
        hipLaunchKernelGGL((gemv_tile16_multi_kernel<BITS, IS_INT, 4>), grid, block, gemv_multi_lds_bytes(K, 4), stream,
                           (const u32x4 *)codes, (const uint16_t *)scales, (const uint16_t *)zeros, (const u32x4 *)X,
                           (uint16_t *)Y, rowtiles, (int)K, (int)M, N);
}

hipError_t run_gemv_multi(bool is_int, const void *codes, const void *scales, const void *zeros, const void *X,
                          void *Y, int64_t M, int64_t N, int64_t K, int bits, hipStream_t stream)
{
    if (is_int) {
        if (bits == 4) launch_gemv_multi<4, true>(codes, scales, zeros, X, Y, M, N, K, stream);
        else if (bits == 3) launch_gemv_multi<3, true>(codes, scales, zeros, X, Y, M, N, K, stream);
        else launch_gemv_multi<2, true>(codes, scales, zeros, X, Y, M, N, K, stream);
    } else {
        if (bits == 4) launch_gemv_multi<4, false>(codes, scales, zeros, X, Y, M, N, K, stream);
        else if (bits == 3) launch_gemv_multi<3, false>(codes, scales, zeros, X, Y, M, N, K, stream);
        else launch_gemv_multi<2, false>(codes, scales, zeros, X, Y, M, N, K, stream);
    }
    return hipGetLastError();
}

size_t gemv_lds_bytes(int64_t K)
{
    return (size_t)(K / kTileCols) * kXRun * 16 + 256 + kGemvWaves * kTileRows * sizeof(float);
}

// Long rows (several rounds per wavefront) let only the lanes of result column 0 read x from
// LDS (4096 x 11008: 7.7 -> 7.0 us, 8192 x 28672: 23.4 -> 20.4 us); with one or two rounds per
// wavefront the masked reads measured slower (11008 x 4096: 6.8 -> 8.0 us) and all lanes read.
static bool gemv_col0_fetch(int64_t K) { return K > 8192; }

// Eight wavefronts per tile measured best or equal on every decoder shape (all of a row's
// groups in flight at once); short rows take fewer so that no wavefront idles.
static int gemv_split(int64_t G)
{
    int split = kGemvWaves < 8 ? kGemvWaves : 8;
    while (split > 1 && G < 4 * split) split /= 2;
    return split;
}

constexpr int64_t kWalkGroups = 512;                  // two resident workgroups per compute unit
constexpr int64_t kWalkMinWeights = 256ll << 20;

static size_t gemv_walk_lds_bytes(int64_t K)
{
    return (size_t)(K / kTileCols) * kXRun * 16 + 256 + 2 * kGemvWaves * kTileRows * sizeof(float);
}

// Whether the tile-walking kernel serves this GEMV: rows long enough for eight wavefronts per
// tile and a very large matrix.  Unlike the exponent form, this kernel is bound by its decode
// work, not by the structure of its launch: at 128256 x 4096 it measured 10 % faster than one
// workgroup per tile (INT3 54 -> 49 us, 4-bit PoT 54 -> 47 us), from 28672 x 8192 down the same
// or slower (17920 x 6656, INT3: 15.3 -> 16.5 us), so it only takes the vocabulary-sized ones.
static bool gemv_walk_ok(int64_t N, int64_t K)
{
    return kGemvWaves == 8 && K / kTileCols >= 32 && N * K >= kWalkMinWeights &&
           gemv_walk_lds_bytes(K) <= kLdsPerWorkgroup;
}

template <int BITS, bool IS_INT>
static hipError_t launch_gemv_walk(const void *codes, const void *scales, const void *zeros, const void *x, void *y,
                                   int64_t N, int64_t K, int group, hipStream_t stream)
{
    const int64_t rowtiles = N / kTileRows;
    const size_t lds = gemv_walk_lds_bytes(K);
    const int64_t cap = kWalkGroups;
    const int64_t per_group = (rowtiles + cap - 1) / cap;
    const dim3 grid((unsigned)((rowtiles + per_group - 1) / per_group)), block(kGemvWaves * kWave);
#define POTQ_LAUNCH_WALK(G64, COL0)                                                                               \
    do {                                                                                                          \
        if (const hipError_t e_ = allow_large_lds<gemv_tile16_walk_kernel<BITS, IS_INT, G64, COL0>>(lds)) return e_; \
        hipLaunchKernelGGL((gemv_tile16_walk_kernel<BITS, IS_INT, G64, COL0>), grid, block, lds, stream,          \
                           (const u32x4 *)codes, (const uint16_t *)scales, (const uint16_t *)zeros,               \
                           (const u32x4 *)x, (uint16_t *)y, rowtiles, (int)K);                                    \
    } while (0)
    // 2- and 3-bit PoT matrices only come here with rows too long for the exponent form
    // (K > 32768), which always take the column-0 fetch: the other instances are not built
    constexpr bool kShortRowsPossible = IS_INT || BITS == 4;
    const bool col0 = !kShortRowsPossible || gemv_col0_fetch(K);
    if (group == 64) {
        if (col0) POTQ_LAUNCH_WALK(true, true);
        else if constexpr (kShortRowsPossible) POTQ_LAUNCH_WALK(true, false);
    } else {
        if (col0) POTQ_LAUNCH_WALK(false, true);
        else if constexpr (kShortRowsPossible) POTQ_LAUNCH_WALK(false, false);
    }
#undef POTQ_LAUNCH_WALK
    return hipGetLastError();
}

template <int BITS, bool IS_INT>
static hipError_t launch_gemv(const void *codes, const void *scales, const void *zeros, const void *x, void *y,
                        int64_t N, int64_t K, int group, hipStream_t stream)
{
    if (gemv_walk_ok(N, K)) return launch_gemv_walk<BITS, IS_INT>(codes, scales, zeros, x, y, N, K, group, stream);
    const int64_t rowtiles = N / kTileRows;
    const size_t lds = gemv_lds_bytes(K);
    const int64_t G = K / kTileCols;
#define POTQ_LAUNCH_GEMV(SPLIT, COL0)                                                                              \
    do {                                                                                                           \
        const dim3 grid((unsigned)((rowtiles + (kGemvWaves / SPLIT) - 1) / (kGemvWaves / SPLIT)));                 \
        if (group == 64) {                                                                                         \
            if (const hipError_t e_ = allow_large_lds<gemv_tile16_kernel<BITS, IS_INT, SPLIT, true, COL0>>(lds))   \
                return e_;                                                                                         \
            hipLaunchKernelGGL((gemv_tile16_kernel<BITS, IS_INT, SPLIT, true, COL0>), grid,                        \
                               dim3(kGemvWaves * kWave), lds, stream, (const u32x4 *)codes,                        \
                               (const uint16_t *)scales, (const uint16_t *)zeros, (const u32x4 *)x, (uint16_t *)y, \
                               rowtiles, (int)K);                                                                  \
        } else {                                                                                                   \
            if (const hipError_t e_ = allow_large_lds<gemv_tile16_kernel<BITS, IS_INT, SPLIT, false, COL0>>(lds))  \
                return e_;                                                                                         \
            hipLaunchKernelGGL((gemv_tile16_kernel<BITS, IS_INT, SPLIT, false, COL0>), grid,                       \
                               dim3(kGemvWaves * kWave), lds, stream, (const u32x4 *)codes,                        \
                               (const uint16_t *)scales, (const uint16_t *)zeros, (const u32x4 *)x, (uint16_t *)y, \
                               rowtiles, (int)K);                                                                  \
        }                                                                                                          \
    } while (0)
    // Eight wavefronts per tile measured best or equal on every decoder shape (all of a
    // row's groups in flight at once); short rows take fewer so that no wavefront idles.
    const int split = gemv_split(G);
    if (split == 8 && kGemvWaves >= 8) {
        if (gemv_col0_fetch(K)) POTQ_LAUNCH_GEMV((kGemvWaves >= 8 ? 8 : 1), true);
        else POTQ_LAUNCH_GEMV((kGemvWaves >= 8 ? 8 : 1), false);
    } else if (split == 4) POTQ_LAUNCH_GEMV(4, false);
    else if (split == 2) POTQ_LAUNCH_GEMV(2, false);
    else POTQ_LAUNCH_GEMV(1, false);
#undef POTQ_LAUNCH_GEMV
    return hipGetLastError();
}

int gemv_max_batch() { return kMaxGemvBatch; }

template <int BITS, bool IS_INT>
static hipError_t launch_gemv_batch(const GemvBatch &b, unsigned blocks, const void *x, int64_t K, int group, int split,
                              hipStream_t stream)
{
    const size_t lds = gemv_lds_bytes(K);
#define POTQ_LAUNCH_GEMVB(SPLIT, COL0)                                                                             \
    do {                                                                                                           \
        if (group == 64) {                                                                                         \
            if (const hipError_t e_ = allow_large_lds<gemv_tile16_batch_kernel<BITS, IS_INT, SPLIT, true, COL0>>(lds)) \
                return e_;                                                                                         \
            hipLaunchKernelGGL((gemv_tile16_batch_kernel<BITS, IS_INT, SPLIT, true, COL0>), dim3(blocks),          \
                               dim3(kGemvWaves * kWave), lds, stream, b, (const u32x4 *)x, (int)K);                \
        } else {                                                                                                   \
            if (const hipError_t e_ = allow_large_lds<gemv_tile16_batch_kernel<BITS, IS_INT, SPLIT, false, COL0>>(lds)) \
                return e_;                                                                                         \
            hipLaunchKernelGGL((gemv_tile16_batch_kernel<BITS, IS_INT, SPLIT, false, COL0>), dim3(blocks),         \
                               dim3(kGemvWaves * kWave), lds, stream, b, (const u32x4 *)x, (int)K);                \
        }                                                                                                          \
    } while (0)
    // batches of 2- and 3-bit PoT matrices with rows of 32 groups or more run in the exponent form
    // up to the row length it can stage (K = 32768): only longer rows reach this kernel
    constexpr bool kLongRowsOnly = !IS_INT && BITS < 4;
    if (split == 8 && kGemvWaves >= 8) {
        if (gemv_col0_fetch(K)) POTQ_LAUNCH_GEMVB((kGemvWaves >= 8 ? 8 : 1), true);
        else if constexpr (!kLongRowsOnly) POTQ_LAUNCH_GEMVB((kGemvWaves >= 8 ? 8 : 1), false);
        else return hipErrorInvalidValue;
    } else if (split == 4) POTQ_LAUNCH_GEMVB(4, false);
    else if (split == 2) POTQ_LAUNCH_GEMVB(2, false);
    else POTQ_LAUNCH_GEMVB(1, false);
#undef POTQ_LAUNCH_GEMVB
    return hipGetLastError();
}

// The exponent form of the PoT GEMV (gemv_exp.hip).
bool gemv_exp_ok(int64_t N, int64_t K, int bits);
bool gemv_exp_batch_ok(int count, int64_t rows_total, int64_t K, int bits);
hipError_t run_gemv_exp(const void *codes, const void *scales, const void *x, void *y, int64_t N, int64_t K, int bits,
                        int group, hipStream_t stream);
hipError_t run_gemv_exp_batch(int count, const void *const *codes, const void *const *scales, void *const *y,
                              const int64_t *N, const void *x, int64_t K, int bits, int group, hipStream_t stream);

// `count` non-empty matrices (count <= kMaxGemvBatch), validated by the caller; all share x, K, bits, group.
hipError_t run_gemv_tile16_batch(bool is_int, int count, const void *const *codes, const void *const *scales,
                                 const void *const *zeros, void *const *y, const int64_t *N, const void *x,
                                 int64_t K, int bits, int group, hipStream_t stream)
{
    if (!is_int) {
        int64_t rows = 0;
        for (int i = 0; i < count; ++i) rows += N[i];
        if (gemv_exp_batch_ok(count, rows, K, bits))
            return run_gemv_exp_batch(count, codes, scales, y, N, x, K, bits, group, stream);
    }
    const int split = gemv_split(K / kTileCols);
    const int R = kGemvWaves / split;
    GemvBatch b;
    uint64_t blocks = 0;
    for (int i = 0; i < kMaxGemvBatch; ++i) {
        const bool live = i < count;
        b.codes[i] = live ? (const u32x4 *)codes[i] : nullptr;
        b.scales[i] = live ? (const uint16_t *)scales[i] : nullptr;
        b.zeros[i] = (live && is_int) ? (const uint16_t *)zeros[i] : nullptr;
        b.y[i] = live ? (uint16_t *)y[i] : nullptr;
        b.rowtiles[i] = live ? N[i] / kTileRows : 0;
        b.first_block[i] = (uint32_t)blocks;
        if (live) blocks += (uint64_t)((b.rowtiles[i] + R - 1) / R);
    }
    b.first_block[kMaxGemvBatch] = (uint32_t)blocks;
    b.count = count;
    if (blocks == 0) return hipSuccess;
    if (blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    if (is_int) {
        if (bits == 4) return launch_gemv_batch<4, true>(b, (unsigned)blocks, x, K, group, split, stream);
        else if (bits == 3) return launch_gemv_batch<3, true>(b, (unsigned)blocks, x, K, group, split, stream);
        else return launch_gemv_batch<2, true>(b, (unsigned)blocks, x, K, group, split, stream);
    } else {
        if (bits == 4) return launch_gemv_batch<4, false>(b, (unsigned)blocks, x, K, group, split, stream);
        else if (bits == 3) return launch_gemv_batch<3, false>(b, (unsigned)blocks, x, K, group, split, stream);
        else return launch_gemv_batch<2, false>(b, (unsigned)blocks, x, K, group, split, stream);
    }
}


hipError_t run_gemv_tile16(bool is_int, const void *codes, const void *scales, const void *zeros, const void *x,
                           void *y, int64_t N, int64_t K, int bits, int group, hipStream_t stream)
{
    // large PoT matrices at 2 and 3 bits: the exponent form (scale applied per group, integer inner sums)
    if (!is_int && gemv_exp_ok(N, K, bits)) return run_gemv_exp(codes, scales, x, y, N, K, bits, group, stream);
    if (is_int) {
        if (bits == 4) return launch_gemv<4, true>(codes, scales, zeros, x, y, N, K, group, stream);
        else if (bits == 3) return launch_gemv<3, true>(codes, scales, zeros, x, y, N, K, group, stream);
        else return launch_gemv<2, true>(codes, scales, zeros, x, y, N, K, group, stream);
    } else {
        if (bits == 4) return launch_gemv<4, false>(codes, scales, zeros, x, y, N, K, group, stream);
        else if (bits == 3) return launch_gemv<3, false>(codes, scales, zeros, x, y, N, K, group, stream);
        else return launch_gemv<2, false>(codes, scales, zeros, x, y, N, K, group, stream);
    }
}

}  // namespace potq
