// Host side of the C ABI declared in include/potq.h: argument validation and
// dispatch.  Nothing here allocates device memory or synchronises.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "potq.h"

namespace potq {
hipError_t run_dequant(bool is_int, const void *codes, const void *scales, const void *zeros, void *out,
                       int64_t N, int64_t K, int bits, int group, hipStream_t stream);
int dequant_max_batch();
hipError_t run_dequant_batch(bool is_int, int count, const void *const *codes, const void *const *scales,
                             const void *const *zeros, void *const *out, const int64_t *N, const int64_t *K,
                             int bits, int group, hipStream_t stream);
hipError_t run_check_scales(const void *scales, int64_t count, int bits, void *bad_count_dev, hipStream_t stream);
hipError_t run_repack(const void *src, void *dst, int64_t N, int64_t K, int bits, bool to_tiled, hipStream_t stream);
hipError_t run_fill_zero(void *p, int64_t count, hipStream_t stream);
size_t gemv_lds_bytes(int64_t K);
hipError_t run_gemv_tile16(bool is_int, const void *codes, const void *scales, const void *zeros, const void *x,
                           void *y, int64_t N, int64_t K, int bits, int group, hipStream_t stream);
size_t gemv_canonical_lds_bytes(int64_t K);
hipError_t run_gemv_canonical(bool is_int, const void *codes, const void *scales, const void *zeros, const void *x,
                              void *y, int64_t N, int64_t K, int bits, int group, hipStream_t stream);
int gemv_max_batch();
bool gemv_exp_ok(int64_t N, int64_t K, int bits);
bool gemv_exp_batch_ok(int count, int64_t rows_total, int64_t K, int bits);
hipError_t run_gemv_tile16_batch(bool is_int, int count, const void *const *codes, const void *const *scales,
                                 const void *const *zeros, void *const *y, const int64_t *N, const void *x,
                                 int64_t K, int bits, int group, hipStream_t stream);
hipError_t run_gemm_tile16(bool is_int, const void *codes, const void *scales, const void *zeros, const void *X,
                           void *Y, int64_t M, int64_t N, int64_t K, int bits, int group, void *ws, size_t ws_bytes,
                           hipStream_t stream);
size_t gemm_workspace_bytes(int64_t M, int64_t N, int64_t K);
size_t gemm_static_scratch_bytes();
hipError_t gemm_static_scratch(void **ptr);
hipError_t run_fakequant_forward(const void *W, const void *S, const void *Gamma, void *Wq, int64_t N, int64_t K,
                                 int bits, int group, hipStream_t stream);
hipError_t run_fakequant_backward(const void *W, const void *S, const void *Gamma, const void *dWq, void *dGamma,
                                  int64_t N, int64_t K, int bits, int group, hipStream_t stream);
hipError_t run_quantize(const void *W, void *codes, void *scales, int64_t N, int64_t K, int bits, int group,
                        hipStream_t stream);
}  // namespace potq

namespace {

constexpr int64_t kMaxDim = (int64_t)1 << 30;
constexpr size_t kMaxLdsBytes = 160 * 1024;        // LDS a gfx950 workgroup can be given

bool misaligned(const void *p, uintptr_t a = 16) { return ((uintptr_t)p & (a - 1)) != 0; }

// Shared checks; returns POTQ_OK when the call should proceed.
int check_common(int64_t N, int64_t K, int bits, int group, bool fused)
{
    if (bits < 2 || bits > 4) return POTQ_ERR_BITS;
    (void)fused;
    if (group != 64 && group != 128) return POTQ_ERR_GROUP;
    if (N < 0 || K < 0 || N > kMaxDim || K > kMaxDim || (K % 128) != 0) return POTQ_ERR_SHAPE;
    return POTQ_OK;
}

int finish(hipError_t e) { return e == hipSuccess ? POTQ_OK : POTQ_ERR_LAUNCH; }

int dequant_entry(bool is_int, const void *codes, const void *scales, const void *zeros, void *out,
                  int64_t N, int64_t K, int bits, int group, void *stream)
{
    const int st = check_common(N, K, bits, group, false);
    if (st != POTQ_OK) return st;
    if (N == 0 || K == 0) return POTQ_OK;
    if (!codes || !scales || !out || (is_int && !zeros)) return POTQ_ERR_NULL;
    if (misaligned(codes) || misaligned(scales) || misaligned(out) || (is_int && misaligned(zeros)))
        return POTQ_ERR_ALIGN;
    return finish(potq::run_dequant(is_int, codes, scales, zeros, out, N, K, bits, group, (hipStream_t)stream));
}

int dequant_batch_entry(bool is_int, const potq_dequant_item *items, int count, int bits, int group, void *stream)
{
    if (bits < 2 || bits > 4) return POTQ_ERR_BITS;
    if (group != 64 && group != 128) return POTQ_ERR_GROUP;
    if (count < 0 || count > potq::dequant_max_batch()) return POTQ_ERR_SHAPE;
    if (count == 0) return POTQ_OK;
    if (!items) return POTQ_ERR_NULL;
    const void *codes[POTQ_MAX_BATCH], *scales[POTQ_MAX_BATCH], *zeros[POTQ_MAX_BATCH];
    void *out[POTQ_MAX_BATCH];
    int64_t N[POTQ_MAX_BATCH], K[POTQ_MAX_BATCH];
    int live = 0;
    for (int i = 0; i < count; ++i) {
        const potq_dequant_item &it = items[i];
        const int st = check_common(it.N, it.K, bits, group, false);
        if (st != POTQ_OK) return st;
        if (it.N == 0 || it.K == 0) continue;
        if (!it.codes || !it.scales || !it.out_f16 || (is_int && !it.zeros)) return POTQ_ERR_NULL;
        if (misaligned(it.codes) || misaligned(it.scales) || misaligned(it.out_f16) ||
            (is_int && misaligned(it.zeros)))
            return POTQ_ERR_ALIGN;
        codes[live] = it.codes;
        scales[live] = it.scales;
        zeros[live] = it.zeros;
        out[live] = it.out_f16;
        N[live] = it.N;
        K[live] = it.K;
        ++live;
    }
    return finish(potq::run_dequant_batch(is_int, live, codes, scales, zeros, out, N, K, bits, group,
                                          (hipStream_t)stream));
}

int gemv_entry(bool is_int, const void *codes, const void *scales, const void *zeros, const void *x, void *y,
               int64_t N, int64_t K, int bits, int group, int layout, void *stream)
{
    const int st = check_common(N, K, bits, group, true);
    if (st != POTQ_OK) return st;
    if (layout != POTQ_LAYOUT_TILE16 && layout != POTQ_LAYOUT_CANONICAL) return POTQ_ERR_LAYOUT;
    const bool tiled = layout == POTQ_LAYOUT_TILE16;
    if (tiled && N % 16 != 0) return POTQ_ERR_SHAPE;
    if (N == 0) return POTQ_OK;
    if (!y) return POTQ_ERR_NULL;
    if (misaligned(y, tiled ? 16 : 2)) return POTQ_ERR_ALIGN;
    if (K == 0) return finish(potq::run_fill_zero(y, N, (hipStream_t)stream));
    if (!codes || !scales || !x || (is_int && !zeros)) return POTQ_ERR_NULL;
    if (misaligned(codes) || misaligned(scales, tiled ? 16 : 2) || misaligned(x) ||
        (is_int && misaligned(zeros, tiled ? 16 : 2)))
        return POTQ_ERR_ALIGN;
    if (!tiled) {
        if (potq::gemv_canonical_lds_bytes(K) > kMaxLdsBytes) return POTQ_ERR_SHAPE;
        return finish(potq::run_gemv_canonical(is_int, codes, scales, zeros, x, y, N, K, bits, group,
                                               (hipStream_t)stream));
    }
    if (potq::gemv_lds_bytes(K) > kMaxLdsBytes) return POTQ_ERR_SHAPE;
    return finish(potq::run_gemv_tile16(is_int, codes, scales, zeros, x, y, N, K, bits, group, (hipStream_t)stream));
}

int gemv_batch_entry(bool is_int, const potq_gemv_item *items, int count, const void *x, int64_t K, int bits,
                     int group, int layout, void *stream)
{
    if (bits < 2 || bits > 4) return POTQ_ERR_BITS;
    if (group != 64 && group != 128) return POTQ_ERR_GROUP;
    if (K < 0 || K > kMaxDim || (K % 128) != 0) return POTQ_ERR_SHAPE;
    if (count < 0 || count > potq::gemv_max_batch()) return POTQ_ERR_SHAPE;
    if (layout != POTQ_LAYOUT_TILE16) return POTQ_ERR_LAYOUT;
    if (count == 0) return POTQ_OK;
    if (!items) return POTQ_ERR_NULL;
    const void *codes[POTQ_MAX_BATCH], *scales[POTQ_MAX_BATCH], *zeros[POTQ_MAX_BATCH];
    void *y[POTQ_MAX_BATCH];
    int64_t N[POTQ_MAX_BATCH];
    int live = 0;
    for (int i = 0; i < count; ++i) {
        const potq_gemv_item &it = items[i];
        if (it.N < 0 || it.N > kMaxDim || (it.N % 16) != 0) return POTQ_ERR_SHAPE;
        if (it.N == 0) continue;
        if (!it.y_f16) return POTQ_ERR_NULL;
        if (misaligned(it.y_f16)) return POTQ_ERR_ALIGN;
        if (K == 0) {
            const int st = finish(potq::run_fill_zero(it.y_f16, it.N, (hipStream_t)stream));
            if (st != POTQ_OK) return st;
            continue;
        }
        if (!it.codes || !it.scales || (is_int && !it.zeros)) return POTQ_ERR_NULL;
        if (misaligned(it.codes) || misaligned(it.scales) || (is_int && misaligned(it.zeros))) return POTQ_ERR_ALIGN;
        codes[live] = it.codes;
        scales[live] = it.scales;
        zeros[live] = it.zeros;
        y[live] = it.y_f16;
        N[live] = it.N;
        ++live;
    }
    if (live == 0) return POTQ_OK;
    if (!x) return POTQ_ERR_NULL;
    if (misaligned(x)) return POTQ_ERR_ALIGN;
    if (potq::gemv_lds_bytes(K) > kMaxLdsBytes) return POTQ_ERR_SHAPE;
    return finish(potq::run_gemv_tile16_batch(is_int, live, codes, scales, zeros, y, N, x, K, bits, group,
                                              (hipStream_t)stream));
}

int gemm_entry(bool is_int, const void *codes, const void *scales, const void *zeros, const void *X, void *Y,
               int64_t M, int64_t N, int64_t K, int bits, int group, int layout, void *workspace,
               size_t workspace_bytes, void *stream, bool static_scratch = false)
{
    const int st = check_common(N, K, bits, group, true);
    if (st != POTQ_OK) return st;
    if (M < 0 || M > kMaxDim) return POTQ_ERR_SHAPE;
    if (layout != POTQ_LAYOUT_TILE16) return POTQ_ERR_LAYOUT;
    if (N % 16 != 0) return POTQ_ERR_SHAPE;
    if (N == 0 || M == 0) return POTQ_OK;
    if (!Y) return POTQ_ERR_NULL;
    if (misaligned(Y)) return POTQ_ERR_ALIGN;
    if (K == 0) return finish(potq::run_fill_zero(Y, M * N, (hipStream_t)stream));
    if (!codes || !scales || !X || (is_int && !zeros)) return POTQ_ERR_NULL;
    if (misaligned(codes) || misaligned(scales) || misaligned(X) || (is_int && misaligned(zeros)))
        return POTQ_ERR_ALIGN;
    if (static_scratch) {
        // the library's built-in buffer takes the place of the caller's workspace.  Shapes whose
        // preferred split does not fit it are refused, so that the result is always the one the
        // call gives with the workspace potq_gemm_workspace_bytes() asks for.
        if (potq::gemm_workspace_bytes(M, N, K) > potq::gemm_static_scratch_bytes()) return POTQ_ERR_WORKSPACE;
        if (potq::gemm_static_scratch(&workspace) != hipSuccess) return POTQ_ERR_LAUNCH;
        workspace_bytes = potq::gemm_static_scratch_bytes();
    }
    if (workspace && misaligned(workspace)) return POTQ_ERR_ALIGN;
    if (!workspace) workspace_bytes = 0;
    return finish(potq::run_gemm_tile16(is_int, codes, scales, zeros, X, Y, M, N, K, bits, group, workspace, workspace_bytes,
                                        (hipStream_t)stream));
}

}  // namespace

extern "C" {

int potq_version(void) { return 100; }

const char *potq_strerror(int status)
{
    switch (status) {
    case POTQ_OK: return "ok";
    case POTQ_ERR_NULL: return "a required pointer is NULL";
    case POTQ_ERR_BITS: return "bits must be 2, 3 or 4";
    case POTQ_ERR_GROUP: return "group size not supported (64 or 128)";
    case POTQ_ERR_SHAPE: return "bad shape (negative, K not a multiple of 128, N not a multiple of 16, or K too large)";
    case POTQ_ERR_ALIGN: return "a pointer is not 16-byte aligned";
    case POTQ_ERR_LAYOUT: return "layout not supported by this entry point";
    case POTQ_ERR_LAUNCH: return "the HIP runtime refused the launch";
    case POTQ_ERR_WORKSPACE: return "the shape needs more scratch memory than the library's built-in buffer holds";
    default: return "unknown status";
    }
}

size_t potq_packed_row_bytes(int64_t K, int bits)
{
    if (K < 0 || bits <= 0 || (K % 8) != 0) return 0;
    return (size_t)(K / 8) * (size_t)bits;
}

size_t potq_packed_bytes(int64_t N, int64_t K, int bits)
{
    if (N < 0) return 0;
    return (size_t)N * potq_packed_row_bytes(K, bits);
}

int pot_dequant(const void *codes, const void *scales, void *out_f16, int64_t N, int64_t K, int bits, int group,
                void *hip_stream)
{
    return dequant_entry(false, codes, scales, nullptr, out_f16, N, K, bits, group, hip_stream);
}

int int_dequant(const void *codes, const void *scales, const void *zeros, void *out_f16, int64_t N, int64_t K,
                int bits, int group, void *hip_stream)
{
    return dequant_entry(true, codes, scales, zeros, out_f16, N, K, bits, group, hip_stream);
}

int pot_dequant_batch(const potq_dequant_item *items_host, int count, int bits, int group, void *hip_stream)
{
    return dequant_batch_entry(false, items_host, count, bits, group, hip_stream);
}

int int_dequant_batch(const potq_dequant_item *items_host, int count, int bits, int group, void *hip_stream)
{
    return dequant_batch_entry(true, items_host, count, bits, group, hip_stream);
}

int potq_repack(const void *src, void *dst, int64_t N, int64_t K, int bits, int to_layout, void *hip_stream)
{
    const int st = check_common(N, K, bits, 128, false);
    if (st != POTQ_OK) return st;
    if (to_layout != POTQ_LAYOUT_TILE16 && to_layout != POTQ_LAYOUT_CANONICAL) return POTQ_ERR_LAYOUT;
    if (N % 16 != 0) return POTQ_ERR_SHAPE;
    if (N == 0 || K == 0) return POTQ_OK;
    if (!src || !dst) return POTQ_ERR_NULL;
    if (misaligned(src) || misaligned(dst)) return POTQ_ERR_ALIGN;
    return finish(potq::run_repack(src, dst, N, K, bits, to_layout == POTQ_LAYOUT_TILE16, (hipStream_t)hip_stream));
}

int pot_gemv(const void *codes, const void *scales, const void *x_f16, void *y_f16, int64_t N, int64_t K, int bits,
             int group, int layout, void *hip_stream)
{
    return gemv_entry(false, codes, scales, nullptr, x_f16, y_f16, N, K, bits, group, layout, hip_stream);
}

int int_gemv(const void *codes, const void *scales, const void *zeros, const void *x_f16, void *y_f16, int64_t N,
             int64_t K, int bits, int group, int layout, void *hip_stream)
{
    return gemv_entry(true, codes, scales, zeros, x_f16, y_f16, N, K, bits, group, layout, hip_stream);
}

int potq_gemv_exponent_form(int64_t N, int64_t K, int bits)
{
    if (N <= 0 || K <= 0 || (K % 128) != 0 || (N % 16) != 0) return 0;
    return potq::gemv_exp_ok(N, K, bits) ? 1 : 0;
}

int potq_gemv_batch_exponent_form(int count, int64_t K, int bits)
{
    if (count <= 0 || count > potq::gemv_max_batch() || K <= 0 || (K % 128) != 0) return 0;
    return potq::gemv_exp_batch_ok(count, 0, K, bits) ? 1 : 0;
}

int pot_gemv_batch(const potq_gemv_item *items_host, int count, const void *x_f16, int64_t K, int bits, int group,
                   int layout, void *hip_stream)
{
    return gemv_batch_entry(false, items_host, count, x_f16, K, bits, group, layout, hip_stream);
}

int int_gemv_batch(const potq_gemv_item *items_host, int count, const void *x_f16, int64_t K, int bits, int group,
                   int layout, void *hip_stream)
{
    return gemv_batch_entry(true, items_host, count, x_f16, K, bits, group, layout, hip_stream);
}

size_t potq_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K, int bits)
{
    if (M <= 0 || N <= 0 || M > kMaxDim) return 0;
    if (check_common(N, K, bits, 128, true) != POTQ_OK || N % 16 != 0) return 0;     // a shape pot_gemm refuses
    return potq::gemm_workspace_bytes(M, N, K);
}

int pot_gemm(const void *codes, const void *scales, const void *X_f16, void *Y_f16, int64_t M, int64_t N, int64_t K,
             int bits, int group, int layout, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return gemm_entry(false, codes, scales, nullptr, X_f16, Y_f16, M, N, K, bits, group, layout, workspace,
                      workspace_bytes, hip_stream);
}

int int_gemm(const void *codes, const void *scales, const void *zeros, const void *X_f16, void *Y_f16, int64_t M,
             int64_t N, int64_t K, int bits, int group, int layout, void *workspace, size_t workspace_bytes,
             void *hip_stream)
{
    return gemm_entry(true, codes, scales, zeros, X_f16, Y_f16, M, N, K, bits, group, layout, workspace,
                      workspace_bytes, hip_stream);
}

int pot_gemm_noalloc(const void *codes, const void *scales, const void *X_f16, void *Y_f16, int64_t M, int64_t N,
                     int64_t K, int bits, int group, int layout, void *hip_stream)
{
    return gemm_entry(false, codes, scales, nullptr, X_f16, Y_f16, M, N, K, bits, group, layout, nullptr, 0,
                      hip_stream, true);
}

int pot_quantize(const void *W_f16, void *codes_out, void *scales_out, int64_t N, int64_t K, int bits, int group,
                 void *hip_stream)
{
    const int st = check_common(N, K, bits, group, false);
    if (st != POTQ_OK) return st;
    if (N == 0 || K == 0) return POTQ_OK;
    if (!W_f16 || !codes_out || !scales_out) return POTQ_ERR_NULL;
    if (misaligned(W_f16) || misaligned(codes_out) || misaligned(scales_out, 2)) return POTQ_ERR_ALIGN;
    return finish(potq::run_quantize(W_f16, codes_out, scales_out, N, K, bits, group, (hipStream_t)hip_stream));
}

int pot_fakequant_forward(const void *W_f16, const void *S_f16, const void *Gamma_f32, void *Wq_f16, int64_t N,
                          int64_t K, int bits, int group, void *hip_stream)
{
    const int st = check_common(N, K, bits, group, false);
    if (st != POTQ_OK) return st;
    if (N == 0 || K == 0) return POTQ_OK;
    if (!W_f16 || !S_f16 || !Gamma_f32 || !Wq_f16) return POTQ_ERR_NULL;
    if (misaligned(W_f16) || misaligned(Wq_f16) || misaligned(S_f16, 2) || misaligned(Gamma_f32, 4))
        return POTQ_ERR_ALIGN;
    return finish(potq::run_fakequant_forward(W_f16, S_f16, Gamma_f32, Wq_f16, N, K, bits, group,
                                              (hipStream_t)hip_stream));
}

int pot_fakequant_backward(const void *W_f16, const void *S_f16, const void *Gamma_f32, const void *dWq_f16,
                           void *dGamma_f32, int64_t N, int64_t K, int bits, int group, void *hip_stream)
{
    const int st = check_common(N, K, bits, group, false);
    if (st != POTQ_OK) return st;
    if (N == 0 || K == 0) return POTQ_OK;
    if (!W_f16 || !S_f16 || !Gamma_f32 || !dWq_f16 || !dGamma_f32) return POTQ_ERR_NULL;
    if (misaligned(W_f16) || misaligned(dWq_f16) || misaligned(S_f16, 2) || misaligned(Gamma_f32, 4) ||
        misaligned(dGamma_f32, 4))
        return POTQ_ERR_ALIGN;
    return finish(potq::run_fakequant_backward(W_f16, S_f16, Gamma_f32, dWq_f16, dGamma_f32, N, K, bits, group,
                                               (hipStream_t)hip_stream));
}

int pot_check_scales(const void *scales, int64_t count, int bits, void *bad_count_dev, void *hip_stream)
{
    if (bits < 2 || bits > 4) return POTQ_ERR_BITS;
    if (count < 0) return POTQ_ERR_SHAPE;
    if (!bad_count_dev || (count > 0 && !scales)) return POTQ_ERR_NULL;
    if (misaligned(bad_count_dev, 8) || misaligned(scales, 2)) return POTQ_ERR_ALIGN;
    return finish(potq::run_check_scales(scales, count, bits, bad_count_dev, (hipStream_t)hip_stream));
}

}  // extern "C"
