/*
 * potq.h -- C ABI of the MI355X (gfx950) power-of-two weight de-quantisation library.
 *
 * The library implements the inference hot path of PoT-PTQ (arXiv 2507.11959):
 * low-bit power-of-two weight codes (one sign bit + exponent bits, one fp16
 * scale per group of input features) are turned into fp16 weights by integer
 * addition into the scale's exponent field, either as a stand-alone pass or
 * fused into the GEMV / GEMM that consumes the weights.  A uniform-integer
 * (scale + zero-point) path built to the same standard serves as baseline.
 *
 * Conventions for every entry point
 * ---------------------------------
 *  - All data pointers are DEVICE pointers (HIP global memory) unless a
 *    parameter name ends in `_host`.  The caller owns every buffer; the library
 *    never allocates, frees or keeps device memory.  Its only state that
 *    outlives a call is a set of process-wide flags and addresses that are set
 *    once per device and never change afterwards (the raised on-chip memory
 *    limit of the kernels that need it, the address of pot_gemm_noalloc's
 *    built-in buffer); they are atomics, so calls are re-entrant and may come
 *    from several host threads.
 *  - `hip_stream` is a `hipStream_t` passed as `void*` (NULL = the null stream).
 *    Every call only enqueues work on that stream and returns; nothing
 *    synchronises.
 *  - Matrices: W is N x K (N output features, K input features, nn.Linear
 *    order).  `scales` (and `zeros`) are N x (K/group) fp16, row-major.  fp16
 *    values are IEEE binary16 stored as 16-bit words.
 *  - Requirements: bits in {2,3,4} (the paper evaluates 2 and 3); group in {64,128};
 *    K a multiple of 128; every pointer 16-byte aligned; the tiled layout also
 *    needs N to be a multiple of 16.  Sizes of zero are valid and do nothing.
 *  - Return value: POTQ_OK or an error code; arguments are validated on the
 *    host before anything is launched, and no entry point aborts or throws.
 *
 * Packed code layouts
 * -------------------
 *  POTQ_LAYOUT_CANONICAL  The format at the boundary.  Each row is a dense
 *      little-endian bit stream along K: code k occupies stream bits
 *      [bits*k, bits*k + bits); stream bit i is bit (i mod 8) of byte (i div 8);
 *      inside a code the exponent is in the low bits-1 bits and the sign is the
 *      top bit (Sec. 4.2, step 1(a): a 3-bit code reads S0 E1 E2).  Row stride
 *      is K*bits/8 bytes, rows are contiguous.  Exactly `bits` bits per weight
 *      (Table 2, "Avg Bits" = bits + 16/group).
 *  POTQ_LAYOUT_TILE16     A kernel-native permutation of the same bits (still
 *      exactly `bits` bits per weight, same total size) produced by
 *      potq_repack(): 16-row x 128-column tiles stored contiguously, tile index
 *      (n/16)*(K/128) + k/128, laid out so that one wavefront fetches a tile
 *      with 16-byte loads per lane and so that four codes can be turned into
 *      byte-permute selectors with one shift and one mask.  The exact bit map
 *      is private to the library; potq_repack() converts in both directions.
 */
#ifndef POTQ_H
#define POTQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    POTQ_OK = 0,
    POTQ_ERR_NULL = 1,       /* a required pointer is NULL */
    POTQ_ERR_BITS = 2,       /* bits not in {2,3,4} */
    POTQ_ERR_GROUP = 3,      /* group size not 64 or 128 */
    POTQ_ERR_SHAPE = 4,      /* negative size, K not a multiple of 128, N not a multiple of 16 (tiled) */
    POTQ_ERR_ALIGN = 5,      /* a pointer is not 16-byte aligned */
    POTQ_ERR_LAYOUT = 6,     /* layout id unknown or not supported by this entry point */
    POTQ_ERR_LAUNCH = 7,     /* the HIP runtime refused the launch */
    POTQ_ERR_WORKSPACE = 8   /* pot_gemm_noalloc: the shape needs more scratch than the built-in buffer holds */
} potq_status;

typedef enum {
    POTQ_LAYOUT_CANONICAL = 0,
    POTQ_LAYOUT_TILE16 = 1
} potq_layout;

/* Library version, major*100 + minor. */
int potq_version(void);

/* Static, human-readable text for a status code. */
const char *potq_strerror(int status);

/* Bytes of one canonical row: K*bits/8 (K must be a multiple of 8). */
size_t potq_packed_row_bytes(int64_t K, int bits);

/* Bytes of a whole packed N x K code matrix; identical for both layouts. */
size_t potq_packed_bytes(int64_t N, int64_t K, int bits);

/*
 * pot_dequant -- stand-alone PoT de-quantisation (Sec. 4.2; value defined by
 * Sec. 3.1 Eq. (1) and Sec. 4.1 Eq. (11)).
 *   out[n,k] = bits16(scales[n, k/group]) + ((sign << 15) | (E << 10))   (16-bit integer add)
 * which equals (-1)^sign * 2^E * scale exactly whenever the scale is a positive
 * normal fp16 with biased exponent in [1, 30 - q_max], q_max = 2^(bits-1) - 1.
 * Outside that domain the result is, by definition of this library, the
 * wrap-around of that 16-bit add (pot_check_scales() finds such scales).
 *   codes   in   canonical layout, N rows of K*bits/8 bytes
 *   scales  in   N x (K/group) fp16
 *   out_f16 out  N x K fp16, row-major, fully overwritten
 */
int pot_dequant(const void *codes, const void *scales, void *out_f16,
                int64_t N, int64_t K, int bits, int group, void *hip_stream);

/*
 * int_dequant -- the uniform baseline (Sec. 4.1 Eq. (9)):
 *   out[n,k] = fp16_rne( (q[n,k] + zeros[n,k/group]) * scales[n,k/group] )
 * q is the unsigned `bits`-bit code (same canonical stream).  `zeros` must hold
 * integer-valued fp16 numbers in [-(2^bits - 1), 0]; for those q + Z is exact
 * and the result is the exact product rounded once, identically in int_dequant,
 * int_gemv and int_gemm.  Other zero-points are outside the contract: the sum
 * q + Z is then rounded at a point that differs between the entry points.
 */
int int_dequant(const void *codes, const void *scales, const void *zeros, void *out_f16,
                int64_t N, int64_t K, int bits, int group, void *hip_stream);

/*
 * pot_dequant_batch / int_dequant_batch -- the same operation on up to
 * POTQ_MAX_BATCH matrices (e.g. the seven projections of a decoder layer) in a
 * single kernel launch, so that the fixed start-up and drain time of a launch,
 * during which HBM idles, is paid once.  `items_host` is a HOST array of `count`
 * descriptors; it is copied into the launch and may be reused or freed as soon as
 * the call returns.  Every matrix obeys the rules of pot_dequant / int_dequant
 * (`zeros` is ignored by the PoT entry point); all share `bits` and `group`.
 * Results are identical, bit for bit, to `count` separate calls.
 */
#define POTQ_MAX_BATCH 16
typedef struct potq_dequant_item {
    const void *codes;      /* device, canonical layout */
    const void *scales;     /* device, N x (K/group) fp16 */
    const void *zeros;      /* device, N x (K/group) fp16; uniform baseline only */
    void *out_f16;          /* device, N x K fp16 */
    int64_t N, K;
} potq_dequant_item;

int pot_dequant_batch(const potq_dequant_item *items_host, int count, int bits, int group, void *hip_stream);
int int_dequant_batch(const potq_dequant_item *items_host, int count, int bits, int group, void *hip_stream);

/*
 * potq_repack -- permute packed codes between the two layouts (device to
 * device, src and dst must not overlap).  to_layout = POTQ_LAYOUT_TILE16
 * converts canonical -> tiled, POTQ_LAYOUT_CANONICAL converts tiled ->
 * canonical.  Bijective; the code values are untouched, so it serves PoT and
 * uniform codes alike.  N must be a multiple of 16.
 */
int potq_repack(const void *src, void *dst, int64_t N, int64_t K, int bits,
                int to_layout, void *hip_stream);

/*
 * pot_gemv -- fused de-quantise + matrix-vector product, batch-1 decode (the
 * consumer of Sec. 4.2's weights: Sec. 1 de-quantises to fp16 for the GEMM):
 *   y[n] = fp16( sum_k W~[n,k] * x[k] ),  W~ as defined by pot_dequant,
 * products exact, accumulation in fp32, one rounding to fp16 at the end.
 *   x_f16 in  K fp16;   y_f16 out  N fp16
 * `layout` names the layout `codes` is in.  POTQ_LAYOUT_TILE16 (needs N % 16 == 0;
 * potq_repack converts) is the fast path.  POTQ_LAYOUT_CANONICAL consumes the
 * boundary format as it is, any N, with more arithmetic per weight (about half
 * the speed on large matrices); there scales, zeros and y need only 2-byte
 * alignment.  The whole of x is held in on-chip memory: K <= 76672 (tiled) or
 * K <= 81920 (canonical), POTQ_ERR_SHAPE beyond.
 *
 * Large 2- and 3-bit matrices (potq_gemv_exponent_form() tells which) are served
 * in the exponent form of the product (Sec. 4.2, additivity of exponents):
 *   y[n] = sum_g scale[n,g] * sum_{k in g} (+-2^E[n,k]) x[k],
 * the inner sums in exact integer arithmetic on x in 32-bit fixed point, every
 * group of 128 activations against its own largest exponent (exact for every
 * x[k] within 2^19 of the largest |x| of its group, rounded to 2^-30 of it
 * below), one fp32 rounding per group.  For scales inside the domain of pot_dequant
 * this is the same sum; for scales outside it (pot_check_scales() finds them,
 * pot_quantize() never produces them) this form multiplies by 2^E where the
 * other adds into the exponent field, and the results differ.  Activations
 * with an infinity or a NaN among them have no fixed-point form and are
 * multiplied one by one in binary32, which gives what the definition gives:
 * the infinity whose sign all infinite terms of a row agree on, NaN otherwise.
 */
int pot_gemv(const void *codes, const void *scales, const void *x_f16, void *y_f16,
             int64_t N, int64_t K, int bits, int group, int layout, void *hip_stream);

/* int_gemv -- the same with W~ as defined by int_dequant (both layouts). */
int int_gemv(const void *codes, const void *scales, const void *zeros, const void *x_f16, void *y_f16,
             int64_t N, int64_t K, int bits, int group, int layout, void *hip_stream);

/*
 * 1 if pot_gemv (and pot_gemm with one token) serves an N x K matrix of this
 * width in the exponent form described above, else 0.  pot_gemm with two to
 * four tokens uses the same form (every token with its own fixed-point
 * exponents) on a subset of these shapes: group size 128 and more than 8192
 * rows (two tokens) or at least 16384 (three, four).
 */
int potq_gemv_exponent_form(int64_t N, int64_t K, int bits);

/*
 * The same question for pot_gemv_batch with `count` matrices of row length K:
 * matrices that share x share its conversion, so a batch takes the exponent
 * form at every size the form can serve (2 or 3 bits, 4096 <= K <= 32768).
 */
int potq_gemv_batch_exponent_form(int count, int64_t K, int bits);

/*
 * pot_gemv_batch / int_gemv_batch -- up to POTQ_MAX_BATCH matrices that consume
 * the SAME activation vector (the q/k/v or gate/up projections of a decoder
 * layer) in one kernel launch: y_i = W~_i x.  At batch 1 a 4096x4096 product is
 * a few-microsecond kernel dominated by launch and memory latency, so sharing a
 * launch is worth more than any tuning inside it.  `items_host` is a HOST array
 * (copied into the launch); all matrices share K, bits, group and layout, each
 * has its own N (a multiple of 16); only POTQ_LAYOUT_TILE16 is accepted here and
 * by pot_gemm / int_gemm.  Results equal `count` separate calls bit for bit.
 */
typedef struct potq_gemv_item {
    const void *codes;      /* device, POTQ_LAYOUT_TILE16 */
    const void *scales;     /* device, N x (K/group) fp16 */
    const void *zeros;      /* device, N x (K/group) fp16; uniform baseline only */
    void *y_f16;            /* device, N fp16 */
    int64_t N;
} potq_gemv_item;

int pot_gemv_batch(const potq_gemv_item *items_host, int count, const void *x_f16, int64_t K,
                   int bits, int group, int layout, void *hip_stream);
int int_gemv_batch(const potq_gemv_item *items_host, int count, const void *x_f16, int64_t K,
                   int bits, int group, int layout, void *hip_stream);

/*
 * pot_gemm -- fused de-quantise + GEMM on the matrix cores (Sec. 1: the weights
 * are de-quantised to fp16 for the GEMM that consumes them; W~ is Sec. 4.2's):
 *   Y[m,n] = fp16( sum_k X[m,k] * W~[n,k] ),   X: M x K fp16 row-major,
 *   Y: M x N fp16 row-major (Y = X . W~^T, the nn.Linear convention).
 * fp16 MFMA with fp32 accumulation (up to four tokens on large 2-/3-bit PoT
 * matrices: the exponent form described at pot_gemv, with its condition on
 * the scales).  `codes` must be in POTQ_LAYOUT_TILE16.
 *
 * `workspace` is optional device scratch memory (16-byte aligned) owned by the
 * caller.  Where the output tiles alone would not occupy the chip evenly, the
 * kernel splits K, writes fp32 partial sums to the workspace and adds them
 * in a fixed order in a second small kernel (results stay reproducible).
 * potq_gemm_workspace_bytes() returns the size that allows the preferred split
 * (0 when no split would be used); a NULL or smaller workspace is valid and
 * only means fewer splits.  With at most 16 tokens K is always split inside the
 * workgroups and the workspace is never touched (the size query returns 0).
 * The workspace may be reused by the next call on the
 * same stream; concurrent calls on different streams need separate workspaces.
 * The size query returns 0 for a shape pot_gemm would refuse (bits, K % 128,
 * N % 16, negative sizes); today the size depends on M, N and K.
 */
size_t potq_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K, int bits);

int pot_gemm(const void *codes, const void *scales, const void *X_f16, void *Y_f16,
             int64_t M, int64_t N, int64_t K, int bits, int group, int layout,
             void *workspace, size_t workspace_bytes, void *hip_stream);

/* int_gemm -- the same with W~ as defined by int_dequant. */
int int_gemm(const void *codes, const void *scales, const void *zeros, const void *X_f16, void *Y_f16,
             int64_t M, int64_t N, int64_t K, int bits, int group, int layout,
             void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * pot_gemm_noalloc -- pot_gemm for callers that cannot allocate device memory or
 * carry a workspace around: code running under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments and the same result,
 * bit for bit, as pot_gemm called with a workspace of
 * potq_gemm_workspace_bytes(M, N, K, bits) bytes; the split-K partial sums go to a
 * buffer of POTQ_STATIC_SCRATCH_BYTES built into the library's code object
 * (every GPU the library runs on holds its own copy until the process ends; its
 * address is looked up once per device, on the first call there).  The call
 * itself allocates and frees nothing and calls no allocating routine.
 *  - A shape whose preferred workspace exceeds the buffer is refused with
 *    POTQ_ERR_WORKSPACE and nothing is launched.  That can only happen with 17 to 64
 *    tokens and M * N above 2^20 elements; every other shape fits.
 *  - All calls on one GPU share that GPU's buffer: calls that overlap in time on
 *    different streams of one GPU race on it and must be serialised by the
 *    caller.  Calls on one stream are ordered and safe.  Nothing in the buffer
 *    has to start at zero (every partial sum that is read was written by the same
 *    call), so it is never cleared and keeps the last call's contents.
 */
#define POTQ_STATIC_SCRATCH_BYTES ((size_t)64 << 20)

int pot_gemm_noalloc(const void *codes, const void *scales, const void *X_f16, void *Y_f16,
                     int64_t M, int64_t N, int64_t K, int bits, int group, int layout,
                     void *hip_stream);

/*
 * pot_quantize -- Step 1 of the method, the data-agnostic scale search (Sec. 3.2,
 * Algorithm 1), producing the inputs of the entry points above from fp16 weights.
 * For every group of `group` consecutive weights of a row:
 *     s0 = max|w| / (2^qmax - 1),  qmax = 2^(bits-1) - 1
 *     for i = 1..200:  s = s0 * (0.01 i);  E_k = clamp(round(log2(|w_k|/s)), 0, qmax);
 *                      Q(i) = sum_k (w_k - sign(w_k) s 2^E_k)^2
 *     i* = the first i with the smallest Q;  scale = s(i*);  codes = (sign, E) under it.
 * The paper leaves the arithmetic open; it is fixed here as IEEE binary32, one
 * rounding per operation, no contraction: b_i = (float)i * 0.01f; s0 by a binary32
 * division; every candidate is taken as it would be stored and used at inference
 * (Sec. 4.2 keeps the scale as FP16): s = s0 * b_i rounded once to fp16 and clamped
 * into [2^-14, largest value with exponent field 30 - qmax], pot_dequant's exact
 * domain, so that Q(i) is the error of exactly what pot_dequant rebuilds and the
 * codes are the quantisation under the stored scale; E = number of e in 1..qmax with
 * |w| >= s * (float)2^(e-1/2) (a tie rounds up, |w| = 0 gives E = 0); w~ = s * 2^E
 * exactly; d = w - w~; Q = fma(d, d, Q) for k ascending; the sign bit is set only
 * for w < 0; an all-zero group gets the smallest scale, i* = 1 and E = 0 everywhere.
 *   W_f16      in   N x K fp16, row-major
 *   codes_out  out  canonical layout, N rows of K*bits/8 bytes
 *   scales_out out  N x (K/group) fp16
 */
int pot_quantize(const void *W_f16, void *codes_out, void *scales_out,
                 int64_t N, int64_t K, int bits, int group, void *hip_stream);

/*
 * pot_fakequant_forward / pot_fakequant_backward -- the weight path of one
 * iteration of Step 2, the data-dependent fine-tuning of the scales (Sec. 3.3,
 * Algorithm 2).  With the learnable residual Gamma (one value per group):
 *     S^   = S * (1 + Gamma)                                  refined scale
 *     E_k  = clamp(round(log2(|w_k| / S^)), 0, qmax)           exponent under S^
 *     w~_k = S^ * sign(w_k) * 2^E_k                            forward result
 * and, by the straight-through estimator (round() differentiated as the
 * identity, the clamp as it stands: derivative 1 on [0, qmax], 0 outside),
 *     dL/dGamma_g = S_g * sum over k in g with round(log2(|w_k|/S^)) outside [0, qmax]
 *                         of (dL/dw~_k) * sign(w_k) * 2^E_k
 * (inside the clamp's range the two terms of dw~/dS^ cancel).  The regulariser
 * (lambda/2)|Gamma|^2 and the update of Gamma are the caller's optimiser's.
 * Arithmetic as for pot_quantize: binary32, one rounding per operation, no
 * contraction; S^ = S * (1.0f + Gamma); E = number of e in 1..qmax with
 * |w| >= S^ * (float)2^(e-1/2); the clamp is active when |w| < S^ * (float)2^(-1/2)
 * or |w| >= S^ * (float)2^(qmax+1/2); |w| = 0 is below range with sign +.
 * Forward rounds the exact S^ * 2^E once to fp16.  Backward adds the (exact)
 * products in binary32, eight per lane in ascending k and then pairwise across
 * the lanes of a group, multiplies by S once; the order is fixed, results are
 * reproducible.  Gamma <= -1 (S^ <= 0) is outside the method; the thresholds
 * are then non-positive and the formulas above are applied as they stand.
 *   W_f16     in   N x K fp16 row-major, the original weights
 *   S_f16     in   N x (K/group) fp16, the Step 1 scales
 *   Gamma_f32 in   N x (K/group) binary32
 *   Wq_f16    out  N x K fp16                      (forward)
 *   dWq_f16   in   N x K fp16, dL/dw~              (backward)
 *   dGamma_f32 out N x (K/group) binary32          (backward)
 * W, Wq, dWq 16-byte aligned; N = 0 or K = 0 is valid and does nothing.
 */
int pot_fakequant_forward(const void *W_f16, const void *S_f16, const void *Gamma_f32, void *Wq_f16,
                          int64_t N, int64_t K, int bits, int group, void *hip_stream);

int pot_fakequant_backward(const void *W_f16, const void *S_f16, const void *Gamma_f32, const void *dWq_f16,
                           void *dGamma_f32, int64_t N, int64_t K, int bits, int group, void *hip_stream);

/*
 * pot_check_scales -- count the scales outside the domain on which the
 * integer-add recipe equals the definition (not positive, subnormal or zero,
 * exponent field above 30 - q_max, infinity, NaN).  The count is written, as
 * one int64, to `bad_count_dev` (device memory, 8-byte aligned) on the stream;
 * the caller copies it back.  Meant to be run once when weights are loaded.
 */
int pot_check_scales(const void *scales, int64_t count, int bits, void *bad_count_dev, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* POTQ_H */
