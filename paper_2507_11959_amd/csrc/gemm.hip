// Fused de-quantise + GEMM on the matrix cores (tiled layout), gfx950.
//
// Y[m,n] = sum_k X[m,k] W~[n,k], for more than 16 tokens (up to 16 tokens take
// the kernel in gemv.hip that is built like the GEMV).  A workgroup of WAVES
// wavefronts owns (WAVES/KS)*RM 16-row tiles of W and a strip of 16*CN tokens,
// and walks K in chunks of GC*KS scale groups (128 columns each), one workgroup
// barrier per chunk; the KS wavefronts that share row tiles take GC groups of
// every chunk each and add their tiles through LDS at the end.
//
//  - Weights never touch LDS.  Lane (r = lane % 16, q = lane / 16) fetches the
//    32 codes of row r, column block q of the group (`bits` dwords), builds the
//    group's byte table by integer addition into the scale's exponent field
//    (Sec. 4.2) and expands the codes, eight at a time, straight into the A
//    operand of v_mfma_f32_16x16x32_f16: A row = weight row r, A k-slot (q, i)
//    = column 32q + 8*step + i of the group.
//  - X goes through LDS, double buffered, already in B-operand order: for
//    k-slot group (step, q) the 16*CN tokens' 8-value runs are contiguous, so a
//    B fragment is one conflict-free ds_read_b128 per lane and is reused by all
//    RM row tiles of the wavefront.
//  - Accumulation is fp32 in the MFMA accumulators; one rounding to fp16 at the end.
//  - Shapes without enough output tiles to occupy 256 CUs split K: inside the
//    workgroup (KS > 1), and/or over blockIdx.z, where every split writes its
//    fp32 sums to the caller's workspace and a small second kernel adds them in
//    a fixed order.
#include "potq_device.hpp"
#include "potq_launch.hpp"

namespace potq {

// wavefronts per SIMD the register allocator is asked to make room for in the tiles of 16 or more fragments
constexpr int kGemmWavesPerSimd = 2;

template <int BITS, bool IS_INT, int WAVES, int RM, int CN, int GC, int KS>
__global__ __launch_bounds__(WAVES * kWave) __attribute__((amdgpu_waves_per_eu((RM * CN >= 16) ? kGemmWavesPerSimd : 1, 8)))
void gemm_tile16_kernel(
    const uint32_t *__restrict__ codes, const uint16_t *__restrict__ scales, const uint16_t *__restrict__ zeros,
    const uint16_t *__restrict__ X, uint16_t *__restrict__ Y, float *__restrict__ partial, int M, int64_t N, int K,
    int groups_per_split, int gs)
{
    // gs = 0: one scale per 128 columns; gs = 1: one per 64 (lane (r, q) then uses scale column 2g + q/2)
    // KS wavefronts share a set of row tiles and split every chunk of K between them: a chunk is
    // CW = GC * KS scale groups wide, wavefront part `kpart` takes groups kpart*GC .. kpart*GC+GC-1 of
    // it, and the KS partial tiles are added through LDS at the end, in a fixed order.
    constexpr int MT = 16 * CN;                       // tokens per workgroup
    constexpr int THREADS = WAVES * kWave;
    constexpr int CW = GC * KS;                       // scale groups per chunk
    constexpr int RS = WAVES / KS;                    // row-tile slots per workgroup
    constexpr int PPT = (CW * MT * 16) / THREADS;     // 16-byte pieces of an X chunk per thread
    static_assert(WAVES % KS == 0, "wavefronts must divide evenly over the K parts");
    static_assert((CW * MT * 16) % THREADS == 0, "X chunk must divide evenly over the workgroup");
    extern __shared__ u32x4 smem[];                   // [2 buffers][CW groups][16 k-slot groups][MT tokens]

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid >> 6;
    const int r = lane & 15;
    const int q = lane >> 4;
    const int G = K / kTileCols;
    const int64_t rowtiles = N / kTileRows;
    const int kpart = wave % KS;
    const int64_t rt0 = ((int64_t)blockIdx.x * RS + wave / KS) * RM;
    const int m0 = blockIdx.y * MT;
    // split-K: blockIdx.z owns scale groups [g_begin, g_end); its fp32 sums go to partial[z] when gridDim.z > 1
    const int g_begin = blockIdx.z * groups_per_split;
    const int g_end = min(G, g_begin + groups_per_split);

    // Weight side.  The L1 processes a load instruction one 64-byte line per group
    // of four consecutive lanes, so loads are issued in memory order -- lane l takes
    // word l of a slab, and the scale of row l/4, group (g & ~3) + l%4 -- and a
    // cross-lane permute (ds_bpermute) then hands lane (r, q) the word 4r + q and the
    // scale of row r it needs as MFMA operand owner.
    const uint32_t *cptr[RM];
    const uint16_t *sptr[RM];
    const uint16_t *zptr[RM];
#pragma unroll
    for (int rm = 0; rm < RM; ++rm) {
        int64_t rt = rt0 + rm;
        if (rt >= rowtiles) rt = rowtiles - 1;        // surplus wavefronts redo the last tile and store nothing
        cptr[rm] = codes + rt * G * (BITS * 64) + lane;
        sptr[rm] = scales + (rt * kTileRows + (lane >> 2)) * ((int64_t)G << gs);
        zptr[rm] = IS_INT ? zeros + (rt * kTileRows + (lane >> 2)) * ((int64_t)G << gs) : nullptr;
    }
    const int word_owner = (4 * r + q) * 4;           // ds_bpermute byte address of the lane holding word 4r + q

    // X side: this thread's pieces of a chunk (16 tokens x 4 consecutive 8-value runs per wavefront).
    // A thread takes the same PG pieces of every scale group of the chunk, so addresses and LDS
    // slots are kept for one group only; piece i belongs to group i / PG of the chunk.
    constexpr int PG = (MT * 16) / THREADS;           // pieces per thread and scale group
    static_assert((MT * 16) % THREADS == 0 && PPT == PG * CW, "a group's pieces must divide evenly over the workgroup");
    const uint16_t *xsrc[PG];
    int xslot[PG];
    bool xok[PG];
#pragma unroll
    for (int i = 0; i < PG; ++i) {
        const int p = tid + THREADS * i;              // piece index inside the group
        const int st = p & 3;                         // run inside a 32-column block = MFMA step
        const int blk = p >> 6;
        const int m = ((p >> 2) & 15) + 16 * (blk % CN);   // four consecutive lanes read 64 contiguous bytes
        const int qq = blk / CN;                      // 32-column block = A/B k-slice
        xok[i] = (m0 + m) < M;
        xsrc[i] = X + (int64_t)(xok[i] ? m0 + m : 0) * K + 32 * qq + 8 * st;
        // rotate the token index inside its 16-token tile by 4*st: the four lanes of a quad (same
        // token, st = 0..3) then write to four different LDS bank groups
        xslot[i] = (st * 4 + qq) * MT + (m & ~15) + ((m + 4 * st) & 15);
    }

    // with few output tiles per wavefront the MFMAs of one tile form a dependent chain:
    // two accumulator sets, alternated by MFMA step, halve it
    constexpr int ACCS = (RM * CN <= 2) ? 2 : 1;
    float4_t acc[ACCS][RM][CN];
#pragma unroll
    for (int a = 0; a < ACCS; ++a)
#pragma unroll
        for (int rm = 0; rm < RM; ++rm)
#pragma unroll
            for (int c = 0; c < CN; ++c) acc[a][rm][c] = float4_t{0.f, 0.f, 0.f, 0.f};

    // Software pipeline, two chunks of GC scale groups deep; one barrier per chunk.
    // Every load is unconditional (indices are clamped, tokens past M are masked to
    // zero afterwards) and every iteration issues the same loads in the same order.
    constexpr bool kAlignedChunks = (GC % 4 == 0);     // chunks start on multiples of four groups (see launch)
    // register stages of X (the LDS buffer is one more stage); the big tiles keep one to stay at two wavefronts per SIMD
    constexpr int kXStages = PPT <= 4 ? 2 : 1;
    uint32_t wr[2][GC][RM][BITS], sr[2][GC][RM], zr[2][GC][RM];
    u32x4 xreg[kXStages][PPT];
    uint32_t xmask[PG];
#pragma unroll
    for (int i = 0; i < PG; ++i) xmask[i] = xok[i] ? 0xFFFFFFFFu : 0u;

    auto fetch_x = [&](int stage, int g0) {
#pragma unroll
        for (int i = 0; i < PPT; ++i) {
            const int gc = min(g0 + i / PG, g_end - 1);             // past the end: re-read the last group
            xreg[stage][i] = *(const u32x4 *)(xsrc[i % PG] + gc * kTileCols);
        }
    };
    auto fetch_w = [&](int stage, int g0) {
#pragma unroll
        for (int gi = 0; gi < GC; ++gi) {
            const int gc = min(g0 + kpart * GC + gi, g_end - 1);
#pragma unroll
            for (int rm = 0; rm < RM; ++rm) {
#pragma unroll
                for (int j = 0; j < BITS; ++j)
                    wr[stage][gi][rm][j] = cptr[rm][(int64_t)gc * (BITS * 64) + 64 * j];
                // one scale load serves the four groups of an aligned quadruple
                if (gi % 4 == 0 || !kAlignedChunks || gs) {
                    const int gq = min(((gc << gs) & ~3) + (lane & 3), (G << gs) - 1);
                    sr[stage][gi][rm] = sptr[rm][gq];
                    zr[stage][gi][rm] = IS_INT ? (uint32_t)zptr[rm][gq] : 0u;
                } else {
                    sr[stage][gi][rm] = sr[stage][gi & ~3][rm];
                    zr[stage][gi][rm] = zr[stage][gi & ~3][rm];
                }
            }
        }
    };

    // Hands lane (r, q) the words and scales of chunk g0 that `stage` holds in memory order.
    auto permute_w = [&](int stage, int g0, uint32_t (&w)[GC][RM][BITS], uint32_t (&s)[GC][RM], uint32_t (&z)[GC][RM]) {
#pragma unroll
        for (int gi = 0; gi < GC; ++gi) {
            const int gc = min(g0 + kpart * GC + gi, g_end - 1);
            const int scale_owner = (4 * r + (((gc << gs) + ((q >> 1) & -gs)) & 3)) * 4;
#pragma unroll
            for (int rm = 0; rm < RM; ++rm) {
#pragma unroll
                for (int j = 0; j < BITS; ++j)
                    w[gi][rm][j] = (uint32_t)__builtin_amdgcn_ds_bpermute(word_owner, (int)wr[stage][gi][rm][j]);
                s[gi][rm] = (uint32_t)__builtin_amdgcn_ds_bpermute(scale_owner, (int)sr[stage][gi][rm]);
                z[gi][rm] = IS_INT ? (uint32_t)__builtin_amdgcn_ds_bpermute(scale_owner, (int)zr[stage][gi][rm]) : 0u;
            }
        }
    };

    // The big tiles run two wavefronts per SIMD, and the barrier puts both at the start of a chunk
    // at the same time: whatever a wavefront must wait for there, the matrix pipe waits for too.
    // So the cross-lane hand-over of a chunk's words happens during the MFMAs of the chunk before
    // (`wn`, `sn`, `zn` carry the result across the barrier), and inside a chunk the token
    // fragments of a step are requested from LDS before the MFMAs of the step before are issued.
    // Both cost registers (15 and 32); they are on where the kernel still fits two wavefronts per
    // SIMD without spilling: the 2- and 3-bit PoT wide tile (the uniform decoder's two tables and
    // the 4-bit decoder's sign masks leave no room).
    constexpr bool kAhead = CN == 8 && RM == 2 && GC == 1 && !IS_INT && BITS < 4;   // the hand-over
    constexpr bool kFragAhead = kAhead;                                             // the token fragments
    uint32_t wn[GC][RM][BITS], sn[GC][RM], zn[GC][RM];

    auto process = [&](int stage, int g0) {
        u32x4 *buf = smem + stage * (CW * 16 * MT);
#pragma unroll
        for (int i = 0; i < PPT; ++i)
            buf[(i / PG) * 16 * MT + xslot[i % PG]] = xreg[kXStages == 2 ? stage : 0][i] & xmask[i % PG];
        __syncthreads();    // this buffer was last read two chunks ago, before the previous barrier
        fetch_x(kXStages == 2 ? stage : 0, g0 + kXStages * CW);

        uint32_t w[GC][RM][BITS], s[GC][RM], z[GC][RM];
        if constexpr (kAhead) {
#pragma unroll
            for (int gi = 0; gi < GC; ++gi)
#pragma unroll
                for (int rm = 0; rm < RM; ++rm) {
#pragma unroll
                    for (int j = 0; j < BITS; ++j) w[gi][rm][j] = wn[gi][rm][j];
                    s[gi][rm] = sn[gi][rm];
                    z[gi][rm] = zn[gi][rm];
                }
        } else {
            permute_w(stage, g0, w, s, z);
            fetch_w(stage, g0 + 2 * CW);
        }

#pragma unroll
        for (int gi = 0; gi < GC; ++gi) {
            if (g0 + kpart * GC + gi >= g_end) break; // wavefront-uniform: only the last chunk of a split can be short
            const u32x4 *xb = buf + (kpart * GC + gi) * 16 * MT;
            Decoder<BITS, IS_INT> dec[RM];
#pragma unroll
            for (int rm = 0; rm < RM; ++rm) {
                dec[rm].set_group(s[gi][rm], z[gi][rm]);
                dec[rm].set_block(w[gi][rm]);
            }
            half8_t b[kFragAhead ? 2 : 1][CN];
            auto read_b = [&](int st, half8_t (&dst)[CN]) {
#pragma unroll
                for (int c = 0; c < CN; ++c)
                    dst[c] = __builtin_bit_cast(half8_t, xb[(st * 4 + q) * MT + 16 * c + ((r + 4 * st) & 15)]);
            };
            if constexpr (kFragAhead) read_b(0, b[0]);
#pragma unroll
            for (int st = 0; st < 4; ++st) {
                half8_t(&bc)[CN] = b[kFragAhead ? (st & 1) : 0];
                if constexpr (kFragAhead) {
                    if (st < 3) read_b(st + 1, b[(st + 1) & 1]);
                } else {
                    read_b(st, bc);
                }
#pragma unroll
                for (int rm = 0; rm < RM; ++rm) {
                    uint32_t a0, a1, a2, a3;
                    dec[rm].get(2 * st, a0, a1);
                    dec[rm].get(2 * st + 1, a2, a3);
                    const half8_t av = __builtin_bit_cast(half8_t, (u32x4{a0, a1, a2, a3}));
#pragma unroll
                    for (int c = 0; c < CN; ++c)
                        acc[(st & (ACCS - 1))][rm][c] =
                            __builtin_amdgcn_mfma_f32_16x16x32_f16(av, bc[c], acc[(st & (ACCS - 1))][rm][c], 0, 0, 0);
                }
            }
        }
        if constexpr (kAhead) {
            // the other register stage holds the next chunk's words (requested a chunk ago): hand them
            // over now, then reuse the stage for the chunk after the one already in flight
            permute_w(stage ^ 1, g0 + CW, wn, sn, zn);
            fetch_w(stage ^ 1, g0 + 3 * CW);
        }
    };

    fetch_x(0, g_begin);
    if (kXStages == 2) fetch_x(1, g_begin + CW);
    fetch_w(0, g_begin);
    fetch_w(1, g_begin + CW);
    if constexpr (kAhead) {
        permute_w(0, g_begin, wn, sn, zn);
        fetch_w(0, g_begin + 2 * CW);
    }
    int g = g_begin;
    for (; g + CW < g_end; g += 2 * CW) {
        process(0, g);
        process(1, g + CW);
    }
    if (g < g_end) process(0, g);

    // K parts of a row-tile slot: every wavefront leaves its tiles in LDS, part 0 adds them in
    // ascending part order (reproducible) and goes on to the store
    if constexpr (KS > 1) {
        float4_t *red = (float4_t *)smem;             // [wave][rm][c][lane]
        __syncthreads();                              // every wavefront is done reading X from LDS
#pragma unroll
        for (int rm = 0; rm < RM; ++rm)
#pragma unroll
            for (int c = 0; c < CN; ++c) {
                const float4_t mine = ACCS == 2 ? acc[0][rm][c] + acc[ACCS - 1][rm][c] : acc[0][rm][c];
                red[((wave * RM + rm) * CN + c) * kWave + lane] = mine;
            }
        __syncthreads();
        if (kpart != 0) return;
#pragma unroll
        for (int rm = 0; rm < RM; ++rm)
#pragma unroll
            for (int c = 0; c < CN; ++c) {
                float4_t sum = red[((wave * RM + rm) * CN + c) * kWave + lane];
#pragma unroll
                for (int p = 1; p < KS; ++p) sum += red[(((wave + p) * RM + rm) * CN + c) * kWave + lane];
                acc[0][rm][c] = sum;
                if (ACCS == 2) acc[ACCS - 1][rm][c] = float4_t{0.f, 0.f, 0.f, 0.f};
            }
    }

    // D: lane holds token m0 + 16c + (lane % 16), weight rows 4*(lane / 16) + i of each row tile
    typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int rm = 0; rm < RM; ++rm) {
        const int64_t rt = rt0 + rm;
        if (rt >= rowtiles) continue;
#pragma unroll
        for (int c = 0; c < CN; ++c) {
            const int m = m0 + 16 * c + r;
            if (m < M) {
                const int64_t at = (int64_t)m * N + rt * kTileRows + 4 * q;
                const float4_t total = ACCS == 2 ? acc[0][rm][c] + acc[ACCS - 1][rm][c] : acc[0][rm][c];
                if (gridDim.z > 1) {
                    *(float4_t *)(partial + (int64_t)blockIdx.z * M * N + at) = total;
                } else {
                    half4_t h;
#pragma unroll
                    for (int i = 0; i < 4; ++i) h[i] = (_Float16)total[i];
                    *(half4_t *)(Y + at) = h;
                }
            }
        }
    }
}

// Y = fp16(sum over splits of partial[s]), summed in ascending s: reproducible.
__global__ __launch_bounds__(256) void gemm_reduce_kernel(const float4_t *__restrict__ partial,
                                                          uint16_t *__restrict__ Y, int64_t quads, int splits)
{
    typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= quads) return;
    float4_t sum = partial[i];
    for (int s = 1; s < splits; ++s) sum += partial[(int64_t)s * quads + i];
    half4_t h;
#pragma unroll
    for (int k = 0; k < 4; ++k) h[k] = (_Float16)sum[k];
    *(half4_t *)(Y + 4 * i) = h;
}

constexpr int64_t kSplitTargetWorkgroups = 768;   // four-wavefront workgroups' worth of wavefronts a split aims at
constexpr int64_t kSplitMinGroups = 4;            // scale groups a K split keeps at least

// Number of K splits with at most 64 tokens: enough workgroups to occupy the chip about
// three times over, at least four scale groups per split, and only as many as the workspace holds.
static int choose_splits(int64_t workgroups, int waves, int ks, int64_t G, int64_t M, int64_t N,
                         size_t workspace_bytes)
{
    const int64_t units = workgroups * waves / 4;
    int64_t want = (kSplitTargetWorkgroups + units - 1) / units;
    if (want > G / (kSplitMinGroups * ks)) want = G / (kSplitMinGroups * ks);
    if (want > 16) want = 16;
    const int64_t fit = (int64_t)(workspace_bytes / ((size_t)M * (size_t)N * sizeof(float)));
    if (want > fit) want = fit;
    return want < 2 ? 1 : (int)want;
}

template <int BITS, bool IS_INT, int WAVES, int RM, int CN, int GC, int KS = 1>
static hipError_t launch_gemm_cfg(const void *codes, const void *scales, const void *zeros, const void *X, void *Y,
                            int64_t M, int64_t N, int64_t K, int group, void *workspace, size_t workspace_bytes,
                            hipStream_t stream, int planned_splits = 0)
{
    const int64_t rowtiles = N / kTileRows;
    const int64_t G = K / kTileCols;
    constexpr int RS = WAVES / KS;                    // row-tile slots per workgroup
    constexpr int CW = GC * KS;                       // scale groups per chunk
    const unsigned gx = (unsigned)((rowtiles + RS * RM - 1) / (RS * RM));
    const unsigned gy = (unsigned)((M + 16 * CN - 1) / (16 * CN));
    // more than 64 tokens: the caller's plan; otherwise chosen here from the number of workgroups
    int splits = planned_splits > 0 ? planned_splits
                 : workspace    ? choose_splits((int64_t)gx * gy, WAVES, KS, G, M, N, workspace_bytes)
                                : 1;
    int per = (int)((G + splits - 1) / splits);
    per = (per + CW - 1) / CW * CW;                   // whole chunks
    splits = (int)((G + per - 1) / per);              // no empty split
    size_t lds = (size_t)2 * CW * 16 * (16 * CN) * sizeof(u32x4);
    const size_t red = KS > 1 ? (size_t)WAVES * RM * CN * kWave * sizeof(float4_t) : 0;
    if (red > lds) lds = red;
    static std::atomic<uint64_t> lds_raised{0};       // per instantiation of this launcher, i.e. per kernel
    const hipError_t lds_status =
        allow_large_lds((const void *)gemm_tile16_kernel<BITS, IS_INT, WAVES, RM, CN, GC, KS>, lds, lds_raised);
    if (lds_status != hipSuccess) return lds_status;
    hipLaunchKernelGGL((gemm_tile16_kernel<BITS, IS_INT, WAVES, RM, CN, GC, KS>), dim3(gx, gy, (unsigned)splits),
                       dim3(WAVES * kWave), lds, stream, (const uint32_t *)codes, (const uint16_t *)scales,
                       (const uint16_t *)zeros, (const uint16_t *)X, (uint16_t *)Y, (float *)workspace, (int)M, N,
                       (int)K, per, group == 64 ? 1 : 0);
    if (splits > 1) {
        const int64_t quads = M * N / 4;
        hipLaunchKernelGGL(gemm_reduce_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, stream,
                           (const float4_t *)workspace, (uint16_t *)Y, quads, splits);
    }
    return hipGetLastError();
}


// More than 64 tokens: eight wavefronts per workgroup and one of three tiles -- "wide" (two row
// tiles per wavefront, 128 tokens: the decode of a weight serves eight token tiles), "narrow"
// (two row tiles, 64 tokens: twice the workgroups) or "tall" (three row tiles, 128 tokens: a token
// fragment read from LDS serves three MFMAs; the most efficient per output, the coarsest to
// place) -- with K split over 1 to 8 workgroups.  Which of the 24 combinations is fastest
// depends on how evenly its workgroups cover the 256 CUs and on what the split costs in
// workspace traffic, and no rule of thumb tracked that: the choice is made by a small cost model,
//     time = ceil(workgroups / 256) * groups_per_split * t_tile * (1 + 0.22 * occupied share of the CUs)
//            [+ 5.6 us + 0.18 us per MB of partial sums written and read back, if split]
// fitted to 400 timings of the six 13B / 70B projection shapes at 128 to 4096 tokens (3-bit PoT;
// rms error 6 %; the model's choice is on average 0.3 % and at worst 5 % slower than the best
// measured combination; 2- and 4-bit kernels differ by -4 % / +7 %, which does not move the
// choice).  Against a rule by tile count alone (wide unless 65..119 wide tiles; split only below 120
// workgroups) it is 10-40 % faster at 128 tokens and up to 36 % at 512.
struct BigTile {
    int rows, tokens;
    double us_per_group;      // one workgroup, one scale group of K, on an otherwise idle chip
};
constexpr BigTile kBigTiles[3] = {{256, 128, 1.66}, {256, 64, 1.04}, {384, 128, 2.15}};
enum { kTileWide = 0, kTileNarrow = 1, kTileTall = 2 };
constexpr double kLoadedSlowdown = 0.22, kReduceFixedUs = 5.6, kReduceUsPerMB = 0.18;
constexpr int kBigMaxSplits = 8;

struct BigPlan {
    int tile, splits;
};

static BigPlan plan_big(int64_t M, int64_t N, int64_t K, int64_t splits_that_fit, bool tall_allowed)
{
    const int64_t G = K / kTileCols;
    BigPlan best{kTileWide, 1};
    if (G <= 0) return best;
    double best_us = 0.0;
    for (int t = 0; t < (tall_allowed ? 3 : 2); ++t) {
        const BigTile &tile = kBigTiles[t];
        const int64_t tiles = ((N + tile.rows - 1) / tile.rows) * ((M + tile.tokens - 1) / tile.tokens);
        for (int want = 1; want <= kBigMaxSplits; ++want) {
            if (want > 1 && (want > splits_that_fit || G / want < kSplitMinGroups)) break;
            const int64_t per = (G + want - 1) / want;
            const int64_t splits = (G + per - 1) / per;           // no empty split
            if (splits != want) continue;                         // the same launch as a smaller `want`
            const int64_t workgroups = tiles * splits;
            const double rounds = (double)((workgroups + 255) / 256);
            const double load = (double)(workgroups < 256 ? workgroups : 256) / 256.0;
            double us = rounds * (double)per * tile.us_per_group * (1.0 + kLoadedSlowdown * load);
            if (splits > 1) us += kReduceFixedUs + kReduceUsPerMB * (double)splits * (double)M * (double)N * 8e-6;
            if (best_us == 0.0 || us < best_us) {
                best_us = us;
                best = BigPlan{t, (int)splits};
            }
        }
    }
    return best;
}

// Workspace that lets every supported shape use its preferred number of splits.
size_t gemm_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    if (M <= 16) return 0;                            // the few-token kernel splits K inside the workgroup
    if (M <= 64) return (size_t)16 * M * N * sizeof(float);
    // enough for the plan with the tall tile (PoT) and for the one without it (uniform baseline)
    const int with_tall = plan_big(M, N, K, kBigMaxSplits, true).splits;
    const int without = plan_big(M, N, K, kBigMaxSplits, false).splits;
    const int splits = with_tall > without ? with_tall : without;
    return splits > 1 ? (size_t)splits * M * N * sizeof(float) : 0;
}

template <int BITS, bool IS_INT>
static hipError_t launch_gemm(const void *codes, const void *scales, const void *zeros, const void *X, void *Y,
                              int64_t M, int64_t N, int64_t K, int group, void *ws, size_t ws_bytes,
                              hipStream_t stream)
{
    // 17 to 64 tokens: not enough output tiles for the chip; eight wavefronts per workgroup.
    // Small, short matrices (K <= 8192, N <= 8192) let pairs of wavefronts split K inside the
    // workgroup and add their tiles through LDS (no second kernel, no workspace traffic: 16.3 us
    // against 19.3 us on 5120 x 5120 at 64 tokens); the others give every wavefront one row tile
    // and split K over workgroups through the caller's workspace (25.8 against 29.8 us on 13824 x 5120).
    const bool in_group_split = K <= 8192 && N <= 8192;
    // Large matrices with few row tiles (N <= 8192: the 70B / 30B q, o and down projections) give
    // every wavefront four row tiles, so that a token fragment read from LDS serves four MFMAs
    // instead of one or two: with K <= 8192 four wavefronts split K inside the workgroup
    // (8192 x 8192: 16.6 against 20.5 us at 32 tokens, 24.2 against 30.4 us at 64), longer rows
    // split K over workgroups (8192 x 28672: 39 against 48 us, 49 against 69 us).  Smaller or
    // taller matrices measured equal or slower with four row tiles.
    const bool short_and_big = N <= 8192 && N * K >= (40ll << 20);
    if (M <= 64 && short_and_big && (K <= 8192 || N * K >= (100ll << 20))) {
        if (M <= 32) {
            if (K <= 8192)
                return launch_gemm_cfg<BITS, IS_INT, 8, 4, 2, 1, 4>(codes, scales, zeros, X, Y, M, N, K, group, ws, ws_bytes, stream);
            else
                return launch_gemm_cfg<BITS, IS_INT, 8, 4, 2, 1, 1>(codes, scales, zeros, X, Y, M, N, K, group, ws, ws_bytes, stream);
        } else {
            if (K <= 8192)
                return launch_gemm_cfg<BITS, IS_INT, 8, 4, 4, 1, 4>(codes, scales, zeros, X, Y, M, N, K, group, ws, ws_bytes, stream);
            else
                return launch_gemm_cfg<BITS, IS_INT, 8, 4, 4, 1, 1>(codes, scales, zeros, X, Y, M, N, K, group, ws, ws_bytes, stream);
        }
    }
    if (M <= 32) {
        if (in_group_split)
            return launch_gemm_cfg<BITS, IS_INT, 8, 2, 2, 1, 2>(codes, scales, zeros, X, Y, M, N, K, group, ws, ws_bytes, stream);
        else
            return launch_gemm_cfg<BITS, IS_INT, 8, 1, 2, 1, 1>(codes, scales, zeros, X, Y, M, N, K, group, ws, ws_bytes, stream);
    } else if (M <= 64) {
        if (in_group_split)
            return launch_gemm_cfg<BITS, IS_INT, 8, 2, 4, 1, 2>(codes, scales, zeros, X, Y, M, N, K, group, ws, ws_bytes, stream);
        else
            return launch_gemm_cfg<BITS, IS_INT, 8, 1, 4, 1, 1>(codes, scales, zeros, X, Y, M, N, K, group, ws, ws_bytes, stream);
    } else {
        const int64_t fit = ws ? (int64_t)(ws_bytes / ((size_t)M * (size_t)N * sizeof(float))) : 1;
        // the uniform decoder (two look-up tables per group) does not fit the tall tile's registers
        // (it spills and runs at half speed), so its plans are made without that tile
        const BigPlan plan = plan_big(M, N, K, fit, !IS_INT);
        if constexpr (!IS_INT) {
            if (plan.tile == kTileTall)
                return launch_gemm_cfg<BITS, IS_INT, 8, 3, 8, 1>(codes, scales, zeros, X, Y, M, N, K, group, ws, ws_bytes, stream, plan.splits);
        }
        if (plan.tile == kTileNarrow)
            return launch_gemm_cfg<BITS, IS_INT, 8, 2, 4, 1>(codes, scales, zeros, X, Y, M, N, K, group, ws, ws_bytes, stream, plan.splits);
        return launch_gemm_cfg<BITS, IS_INT, 8, 2, 8, 1>(codes, scales, zeros, X, Y, M, N, K, group, ws, ws_bytes, stream, plan.splits);
    }
}

// ---------------------------------------------------------------------------
// Split-K partial sums for callers that may not allocate: one array in the code object itself.
// Every GPU the library runs on holds its own copy at its own address until the process ends;
// in host code the array's name is only a handle for hipGetSymbolAddress, never an address.
// ---------------------------------------------------------------------------
constexpr size_t kScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

size_t gemm_static_scratch_bytes() { return kScratchBytes; }

// Device address of `scratch` on the current device, asked for once per device and process.
hipError_t gemm_static_scratch(void **ptr)
{
    constexpr int kKnownDevices = 64;
    static std::atomic<void *> address[kKnownDevices];   // zero-initialised: not asked yet
    int device = 0;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess) return e;
    void *p = (device >= 0 && device < kKnownDevices) ? address[device].load(std::memory_order_acquire) : nullptr;
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        if (device >= 0 && device < kKnownDevices) address[device].store(p, std::memory_order_release);
    }
    *ptr = p;
    return hipSuccess;
}

hipError_t run_gemm_fewtok(bool is_int, const void *codes, const void *scales, const void *zeros, const void *X,
                           void *Y, int64_t M, int64_t N, int64_t K, int bits, int group, hipStream_t stream);

bool gemv_multi_ok(int64_t M, int64_t N, int64_t K, int group);
bool gemv_exp_multi_ok(int64_t M, int64_t N, int64_t K, int bits, int group);
hipError_t run_gemv_exp_multi(const void *codes, const void *scales, const void *X, void *Y, int64_t M, int64_t N,
                              int64_t K, int bits, hipStream_t stream);
size_t gemv_lds_bytes(int64_t K);
hipError_t run_gemv_tile16(bool is_int, const void *codes, const void *scales, const void *zeros, const void *x,
                           void *y, int64_t N, int64_t K, int bits, int group, hipStream_t stream);
hipError_t run_gemv_multi(bool is_int, const void *codes, const void *scales, const void *zeros, const void *X,
                          void *Y, int64_t M, int64_t N, int64_t K, int bits, hipStream_t stream);

hipError_t run_gemm_tile16(bool is_int, const void *codes, const void *scales, const void *zeros, const void *X,
                           void *Y, int64_t M, int64_t N, int64_t K, int bits, int group, void *ws, size_t ws_bytes,
                           hipStream_t stream)
{
    // up to 16 tokens: the kernel built like the GEMV (one table per 128 weights, no cross-lane code traffic)
    // one token is a GEMV
    if (M == 1 && gemv_lds_bytes(K) <= kLdsPerWorkgroup)
        return run_gemv_tile16(is_int, codes, scales, zeros, X, Y, N, K, bits, group, stream);
    // two to four tokens on a large PoT matrix: the exponent form of the GEMV with one MFMA per vector and step
    if (!is_int && gemv_exp_multi_ok(M, N, K, bits, group))
        return run_gemv_exp_multi(codes, scales, X, Y, M, N, K, bits, stream);
    // two to four tokens: the GEMV kernel with one activation vector per result column
    if (gemv_multi_ok(M, N, K, group)) return run_gemv_multi(is_int, codes, scales, zeros, X, Y, M, N, K, bits, stream);
    if (M <= 16)
        return run_gemm_fewtok(is_int, codes, scales, zeros, X, Y, M, N, K, bits, group, stream);
    if (is_int) {
        if (bits == 4) return launch_gemm<4, true>(codes, scales, zeros, X, Y, M, N, K, group, ws, ws_bytes, stream);
        else if (bits == 3) return launch_gemm<3, true>(codes, scales, zeros, X, Y, M, N, K, group, ws, ws_bytes, stream);
        else return launch_gemm<2, true>(codes, scales, zeros, X, Y, M, N, K, group, ws, ws_bytes, stream);
    } else {
        if (bits == 4) return launch_gemm<4, false>(codes, scales, zeros, X, Y, M, N, K, group, ws, ws_bytes, stream);
        else if (bits == 3) return launch_gemm<3, false>(codes, scales, zeros, X, Y, M, N, K, group, ws, ws_bytes, stream);
        else return launch_gemm<2, false>(codes, scales, zeros, X, Y, M, N, K, group, ws, ws_bytes, stream);
    }
}

}  // namespace potq
