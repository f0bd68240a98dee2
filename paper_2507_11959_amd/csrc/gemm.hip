// Fused de-quantise + GEMM on the matrix cores (tiled layout), gfx950.
//
// Y[m,n] = sum_k X[m,k] W~[n,k].  A workgroup of WAVES wavefronts owns
// WAVES*RM 16-row tiles of W and a strip of 16*CN tokens, and walks K one scale
// group (128 columns) at a time.
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
//  - Few-token shapes do not have enough output tiles to occupy 256 CUs, so K is
//    split over blockIdx.z: every split writes its fp32 sums to the caller's
//    workspace and a small second kernel adds them in a fixed order.
#include "potq_device.hpp"

namespace potq {

#ifndef POTQ_GEMM_DEPTH_BIG
#define POTQ_GEMM_DEPTH_BIG 2
#endif
#ifndef POTQ_GEMM_DEPTH_SMALL
#define POTQ_GEMM_DEPTH_SMALL 2
#endif
#ifndef POTQ_GEMM_NT
#define POTQ_GEMM_NT 0
#endif

template <int BITS, bool IS_INT, int WAVES, int RM, int CN>
__global__ __launch_bounds__(WAVES * kWave) void gemm_tile16_kernel(
    const uint32_t *__restrict__ codes, const uint16_t *__restrict__ scales, const uint16_t *__restrict__ zeros,
    const uint16_t *__restrict__ X, uint16_t *__restrict__ Y, float *__restrict__ partial, int M, int64_t N, int K,
    int groups_per_split)
{
    constexpr int MT = 16 * CN;                       // tokens per workgroup
    constexpr int THREADS = WAVES * kWave;
    constexpr int PPT = (MT * 16) / THREADS;          // 16-byte pieces of an X chunk per thread
    static_assert((MT * 16) % THREADS == 0, "X chunk must divide evenly over the workgroup");
    extern __shared__ u32x4 smem[];                   // [2 buffers][16 k-slot groups][MT tokens]

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid >> 6;
    const int r = lane & 15;
    const int q = lane >> 4;
    const int G = K / kTileCols;
    const int64_t rowtiles = N / kTileRows;
    const int64_t rt0 = ((int64_t)blockIdx.x * WAVES + wave) * RM;
    const int m0 = blockIdx.y * MT;
    // split-K: blockIdx.z owns scale groups [g_begin, g_end); its fp32 sums go to partial[z] when gridDim.z > 1
    const int g_begin = blockIdx.z * groups_per_split;
    const int g_end = min(G, g_begin + groups_per_split);

    // weight side: per row tile, pointer to this lane's word of slab 0 of group 0, and its scale row
    const uint32_t *cptr[RM];
    const uint16_t *sptr[RM];
    const uint16_t *zptr[RM];
#pragma unroll
    for (int rm = 0; rm < RM; ++rm) {
        int64_t rt = rt0 + rm;
        if (rt >= rowtiles) rt = rowtiles - 1;        // surplus wavefronts redo the last tile and store nothing
        cptr[rm] = codes + rt * G * (BITS * 64) + r * 4 + q;
        sptr[rm] = scales + (rt * kTileRows + r) * G;
        zptr[rm] = IS_INT ? zeros + (rt * kTileRows + r) * G : nullptr;
    }

    // X side: this thread's pieces of a chunk (16 tokens x 4 consecutive 8-value runs per wavefront)
    const uint16_t *xsrc[PPT];
    int xslot[PPT];
    bool xok[PPT];
#pragma unroll
    for (int i = 0; i < PPT; ++i) {
        const int p = tid + THREADS * i;
        const int st = (p >> 4) & 3;                  // run inside a 32-column block = MFMA step
        const int blk = p >> 6;
        const int m = (p & 15) + 16 * (blk % CN);
        const int qq = blk / CN;                      // 32-column block = A/B k-slice
        xok[i] = (m0 + m) < M;
        xsrc[i] = X + (int64_t)(xok[i] ? m0 + m : 0) * K + 32 * qq + 8 * st;
        xslot[i] = (st * 4 + qq) * MT + m;
    }

    float4_t acc[RM][CN];
#pragma unroll
    for (int rm = 0; rm < RM; ++rm)
#pragma unroll
        for (int c = 0; c < CN; ++c) acc[rm][c] = float4_t{0.f, 0.f, 0.f, 0.f};

    // Software pipeline.  Packed codes stream from HBM: they are requested kDepth
    // groups ahead into a small register ring.  X comes from L2: it is requested
    // kXStages groups ahead into registers and moves through two LDS buffers.
    constexpr int kDepth = (CN >= 8) ? POTQ_GEMM_DEPTH_BIG : POTQ_GEMM_DEPTH_SMALL;
    constexpr int kXStages = (PPT <= 4) ? 2 : 1;
    static_assert(kDepth % 2 == 0, "LDS buffer and X stage are selected by the parity of the unrolled index");
    uint32_t wr[kDepth][RM][BITS], sr[kDepth][RM], zr[kDepth][RM];
    u32x4 xreg[kXStages][PPT];

    auto fetch_codes = [&](int slot, int g) {
        const int gc = g < g_end ? g : g_end - 1;     // past the end: re-read the last group, never used
#pragma unroll
        for (int rm = 0; rm < RM; ++rm) {
#pragma unroll
            for (int j = 0; j < BITS; ++j)
#if POTQ_GEMM_NT
                wr[slot][rm][j] = __builtin_nontemporal_load(cptr[rm] + (int64_t)gc * (BITS * 64) + 64 * j);
#else
                wr[slot][rm][j] = cptr[rm][(int64_t)gc * (BITS * 64) + 64 * j];
#endif
            sr[slot][rm] = sptr[rm][gc];
            zr[slot][rm] = IS_INT ? (uint32_t)zptr[rm][gc] : 0u;
        }
    };
    auto fetch_x = [&](int stage, int g) {
        const int gc = g < g_end ? g : g_end - 1;
#pragma unroll
        for (int i = 0; i < PPT; ++i)
            xreg[stage][i] = xok[i] ? *(const u32x4 *)(xsrc[i] + gc * kTileCols) : u32x4{0u, 0u, 0u, 0u};
    };

#pragma unroll
    for (int d = 0; d < kDepth; ++d) fetch_codes(d, g_begin + d);
#pragma unroll
    for (int x = 0; x < kXStages; ++x) fetch_x(x, g_begin + x);

    for (int gb = g_begin; gb < g_end; gb += kDepth) {
#pragma unroll
        for (int d = 0; d < kDepth; ++d) {
            const int g = gb + d;
            if (g >= g_end) break;                    // uniform over the workgroup
            u32x4 *buf = smem + (d & 1) * (16 * MT);  // (g - g_begin) & 1 == d & 1
#pragma unroll
            for (int i = 0; i < PPT; ++i) buf[xslot[i]] = xreg[d % kXStages][i];
            __syncthreads();    // this buffer was last read two groups ago, before the previous barrier
            fetch_x(d % kXStages, g + kXStages);

            uint32_t w[RM][BITS], s[RM], z[RM];
#pragma unroll
            for (int rm = 0; rm < RM; ++rm) {
#pragma unroll
                for (int j = 0; j < BITS; ++j) w[rm][j] = wr[d][rm][j];
                s[rm] = sr[d][rm];
                z[rm] = zr[d][rm];
            }
            fetch_codes(d, g + kDepth);

            PotTable pt[RM];
            IntTable it[RM];
            uint32_t sel[RM][8];
#pragma unroll
            for (int rm = 0; rm < RM; ++rm) {
                if (IS_INT)
                    it[rm] = int_table<BITS>(s[rm], z[rm]);
                else
                    pt[rm] = pot_table<BITS>(s[rm]);
                if (BITS == 3)
                    selectors3(w[rm][0], w[rm][1], w[rm][BITS - 1], sel[rm]);
                else
                    selectors2(w[rm][0], w[rm][1], sel[rm]);
            }
#pragma unroll
            for (int st = 0; st < 4; ++st) {
                half8_t b[CN];
#pragma unroll
                for (int c = 0; c < CN; ++c)
                    b[c] = __builtin_bit_cast(half8_t, buf[(st * 4 + q) * MT + 16 * c + r]);
#pragma unroll
                for (int rm = 0; rm < RM; ++rm) {
                    uint32_t a0, a1, a2, a3;
                    if (IS_INT) {
                        int_lookup(it[rm], sel[rm][2 * st], a0, a1);
                        int_lookup(it[rm], sel[rm][2 * st + 1], a2, a3);
                    } else {
                        pot_lookup(pt[rm], sel[rm][2 * st], a0, a1);
                        pot_lookup(pt[rm], sel[rm][2 * st + 1], a2, a3);
                    }
                    const half8_t av = __builtin_bit_cast(half8_t, (u32x4{a0, a1, a2, a3}));
#pragma unroll
                    for (int c = 0; c < CN; ++c)
                        acc[rm][c] = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, b[c], acc[rm][c], 0, 0, 0);
                }
            }
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
                if (gridDim.z > 1) {
                    *(float4_t *)(partial + (int64_t)blockIdx.z * M * N + at) = acc[rm][c];
                } else {
                    half4_t h;
#pragma unroll
                    for (int i = 0; i < 4; ++i) h[i] = (_Float16)acc[rm][c][i];
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

// Number of K splits: enough workgroups to occupy the chip about three times over,
// at least four scale groups per split, and only as many as the workspace holds.
static int choose_splits(int64_t workgroups, int64_t G, int64_t M, int64_t N, size_t workspace_bytes)
{
    int64_t want = (768 + workgroups - 1) / workgroups;
    if (want > G / 4) want = G / 4;
    if (want > 16) want = 16;
    const int64_t fit = (int64_t)(workspace_bytes / ((size_t)M * (size_t)N * sizeof(float)));
    if (want > fit) want = fit;
    return want < 2 ? 1 : (int)want;
}

template <int BITS, bool IS_INT, int WAVES, int RM, int CN>
static void launch_gemm_cfg(const void *codes, const void *scales, const void *zeros, const void *X, void *Y,
                            int64_t M, int64_t N, int64_t K, void *workspace, size_t workspace_bytes,
                            hipStream_t stream)
{
    const int64_t rowtiles = N / kTileRows;
    const int64_t G = K / kTileCols;
    const unsigned gx = (unsigned)((rowtiles + WAVES * RM - 1) / (WAVES * RM));
    const unsigned gy = (unsigned)((M + 16 * CN - 1) / (16 * CN));
    int splits = workspace ? choose_splits((int64_t)gx * gy, G, M, N, workspace_bytes) : 1;
    int per = (int)((G + splits - 1) / splits);
    splits = (int)((G + per - 1) / per);              // no empty split
    const size_t lds = (size_t)2 * 16 * (16 * CN) * sizeof(u32x4);
    hipLaunchKernelGGL((gemm_tile16_kernel<BITS, IS_INT, WAVES, RM, CN>), dim3(gx, gy, (unsigned)splits),
                       dim3(WAVES * kWave), lds, stream, (const uint32_t *)codes, (const uint16_t *)scales,
                       (const uint16_t *)zeros, (const uint16_t *)X, (uint16_t *)Y, (float *)workspace, (int)M, N,
                       (int)K, per);
    if (splits > 1) {
        const int64_t quads = M * N / 4;
        hipLaunchKernelGGL(gemm_reduce_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, stream,
                           (const float4_t *)workspace, (uint16_t *)Y, quads, splits);
    }
}

// Workspace that lets every supported shape use its preferred number of splits.
size_t gemm_workspace_bytes(int64_t M, int64_t N) { return M <= 64 ? (size_t)16 * M * N * sizeof(float) : 0; }

#ifndef POTQ_GEMM_BIG_RM
#define POTQ_GEMM_BIG_RM 2
#endif
#ifndef POTQ_GEMM_BIG_CN
#define POTQ_GEMM_BIG_CN 8
#endif

template <int BITS, bool IS_INT>
static void launch_gemm(const void *codes, const void *scales, const void *zeros, const void *X, void *Y,
                        int64_t M, int64_t N, int64_t K, void *ws, size_t ws_bytes, hipStream_t stream)
{
    if (M <= 16)
        launch_gemm_cfg<BITS, IS_INT, 4, 1, 1>(codes, scales, zeros, X, Y, M, N, K, ws, ws_bytes, stream);
    else if (M <= 32)
        launch_gemm_cfg<BITS, IS_INT, 4, 1, 2>(codes, scales, zeros, X, Y, M, N, K, ws, ws_bytes, stream);
    else if (M <= 64)
        launch_gemm_cfg<BITS, IS_INT, 4, 1, 4>(codes, scales, zeros, X, Y, M, N, K, ws, ws_bytes, stream);
    else
        launch_gemm_cfg<BITS, IS_INT, 4, POTQ_GEMM_BIG_RM, POTQ_GEMM_BIG_CN>(codes, scales, zeros, X, Y, M, N, K,
                                                                              nullptr, 0, stream);
}

hipError_t run_gemm_tile16(bool is_int, const void *codes, const void *scales, const void *zeros, const void *X,
                           void *Y, int64_t M, int64_t N, int64_t K, int bits, void *ws, size_t ws_bytes,
                           hipStream_t stream)
{
    if (is_int) {
        if (bits == 3) launch_gemm<3, true>(codes, scales, zeros, X, Y, M, N, K, ws, ws_bytes, stream);
        else launch_gemm<2, true>(codes, scales, zeros, X, Y, M, N, K, ws, ws_bytes, stream);
    } else {
        if (bits == 3) launch_gemm<3, false>(codes, scales, zeros, X, Y, M, N, K, ws, ws_bytes, stream);
        else launch_gemm<2, false>(codes, scales, zeros, X, Y, M, N, K, ws, ws_bytes, stream);
    }
    return hipGetLastError();
}

}  // namespace potq
