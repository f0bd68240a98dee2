/*
 * potq_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, scalar CPU statement of what the power-of-two (PoT) weight
 * de-quantisation path of PoT-PTQ (arXiv 2507.11959) computes, written from the
 * paper's definitions.  It exists so that the GPU library can be checked
 * against something that a reader can verify against the paper by eye.
 * Only the test-suite, the smoke check and the benchmark's CPU-baseline leg
 * may call it.  It shares no code, header, table or helper with the GPU
 * library and knows nothing about the GPU library's private layouts.
 *
 * Every floating-point quantity is evaluated in double precision and rounded
 * once to IEEE binary16 (round-to-nearest, ties-to-even) where the paper's
 * result is an fp16 number.  binary16 <-> double conversion is done in
 * software here (no compiler half type) so that the rounding is in plain view.
 *
 * What is defined where in the paper:
 *   - PoT value  w~ = S * P * 2^E, P in {-1,+1}, E in [0, q_max],
 *     q_max = 2^(n-1) - 1 for an n-bit code            : Sec. 3.1, Eq. (1)-(3)
 *   - one scale per group of G consecutive weights along the input dimension
 *                                                      : Sec. 3.1, Eq. (5)
 *   - code = sign bit (most significant) followed by the exponent bits
 *                                                      : Sec. 4.1 Eq. (11), Sec. 4.2 step 1(a)
 *   - fp16 = 1 sign, 5 exponent (bias 15), 10 mantissa bits : Sec. 4.1
 *   - bit recipe: (sign, 000, exponent bits) moved to the top six bits of a
 *     16-bit word and integer-added to the fp16 scale  : Sec. 4.2 steps 1-2
 *   - uniform baseline  w~ = (W_Q + Z) * S             : Sec. 4.1, Eq. (9)
 *
 * The paper does not say how codes are packed into memory beyond their density
 * (exactly n bits per weight, Table 2's "Avg Bits").  The layout used at this
 * library's boundary, and therefore here, is: each matrix row is a dense
 * little-endian bit stream along the input dimension; code k of a row occupies
 * stream bits [n*k, n*k+n); stream bit i is bit (i mod 8) of byte (i div 8);
 * within a code the exponent is the low n-1 bits and the sign the top bit.
 *
 * Parity pins (tests/test_oracle_*.py): all 65536 half->double values and all
 * rounding midpoints against numpy's float16; every code x every fp16 scale
 * pattern, definition vs bit recipe vs numpy ldexp; the closed-form grid;
 * brute-force pack/unpack; GEMV/GEMM special cases and numpy float64 matmul.
 * No function here is "parity unpinned".
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#if defined(_OPENMP)
#include <omp.h>
#endif

/* ------------------------------------------------------------------ fp16 -- */

/* Exact value of a binary16 bit pattern (Sec. 4.1: (-1)^S * 2^(E-15) * 1.M,
 * extended by the IEEE rules for E = 0 (subnormal: 2^-14 * 0.M) and E = 31). */
double orc_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int efield = (h >> 10) & 0x1F;
    int mant = h & 0x3FF;
    double v;
    if (efield == 0)
        v = ldexp((double)mant, -24);
    else if (efield == 31)
        v = mant ? NAN : INFINITY;
    else
        v = ldexp(1.0 + (double)mant / 1024.0, efield - 15);
    return sign ? -v : v;
}

/* Round a double to the nearest binary16, ties to even; overflow gives
 * infinity, NaN gives the quiet NaN 0x7E00 (sign kept). */
uint16_t orc_double_to_half(double v)
{
    uint16_t sign = signbit(v) ? 0x8000u : 0u;
    double a = fabs(v);
    int e2;
    double quantum, q, f, d;
    long r;
    int efield;

    if (isnan(v)) return (uint16_t)(sign | 0x7E00u);
    if (isinf(v)) return (uint16_t)(sign | 0x7C00u);
    if (a == 0.0) return sign;

    (void)frexp(a, &e2);          /* a = m * 2^e2, m in [0.5, 1)  =>  a in [2^(e2-1), 2^e2) */
    e2 -= 1;                      /* a = 1.f * 2^e2 */
    if (e2 < -14) e2 = -14;       /* subnormal range shares the spacing of the lowest binade */
    quantum = ldexp(1.0, e2 - 10);/* spacing of binary16 numbers around a */
    q = a / quantum;              /* exact: division by a power of two */
    f = floor(q);
    d = q - f;
    r = (long)f;
    if (d > 0.5 || (d == 0.5 && (r & 1))) r += 1;
    /* r counts quanta.  In the normal range r is in [1024, 2048]; 2048 carries
     * into the next binade, which the addition below does by itself. */
    if (e2 == -14 && r < 1024) {
        efield = 0;               /* subnormal or zero: bits are r itself */
        return (uint16_t)(sign | (uint16_t)r);
    }
    efield = e2 + 15;
    {
        long bits = ((long)efield << 10) + (r - 1024);
        if (bits >= 0x7C00) return (uint16_t)(sign | 0x7C00u);
        return (uint16_t)(sign | (uint16_t)bits);
    }
}

/* ----------------------------------------------------------- bit stream -- */

size_t orc_packed_row_bytes(int64_t K, int bits)
{
    return (size_t)((K * bits + 7) / 8);
}

/* Code k of one row, read one stream bit at a time. */
static unsigned get_code(const uint8_t *row, int64_t k, int bits)
{
    unsigned c = 0;
    for (int j = 0; j < bits; ++j) {
        int64_t pos = (int64_t)bits * k + j;
        unsigned bit = (row[pos >> 3] >> (pos & 7)) & 1u;
        c |= bit << j;
    }
    return c;
}

/* codes: N*K bytes, one code per byte (value < 2^bits).  packed: N rows of
 * orc_packed_row_bytes(K, bits) bytes, fully overwritten. */
void orc_pack_codes(const uint8_t *codes, uint8_t *packed, int64_t N, int64_t K, int bits)
{
    size_t rb = orc_packed_row_bytes(K, bits);
    memset(packed, 0, rb * (size_t)N);
    for (int64_t n = 0; n < N; ++n) {
        uint8_t *row = packed + rb * (size_t)n;
        for (int64_t k = 0; k < K; ++k) {
            unsigned c = codes[n * K + k];
            for (int j = 0; j < bits; ++j) {
                int64_t pos = (int64_t)bits * k + j;
                if ((c >> j) & 1u) row[pos >> 3] |= (uint8_t)(1u << (pos & 7));
            }
        }
    }
}

void orc_unpack_codes(const uint8_t *packed, uint8_t *codes, int64_t N, int64_t K, int bits)
{
    size_t rb = orc_packed_row_bytes(K, bits);
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k)
            codes[n * K + k] = (uint8_t)get_code(packed + rb * (size_t)n, k, bits);
}

/* --------------------------------------------------------------- decode -- */

/* The definition (Sec. 3.1 Eq. (1), Sec. 4.1 Eq. (11)): value = (-1)^sign *
 * 2^E * s, evaluated in real arithmetic and rounded once to binary16. */
uint16_t orc_decode_def(unsigned code, uint16_t scale_bits, int bits)
{
    unsigned sign = (code >> (bits - 1)) & 1u;
    int E = (int)(code & ((1u << (bits - 1)) - 1u));
    double s = orc_half_to_double(scale_bits);
    double w = (sign ? -1.0 : 1.0) * ldexp(s, E);
    return orc_double_to_half(w);
}

/* The bit recipe (Sec. 4.2): the six-bit field (sign, 0, 0, 0, exponent bits)
 * placed on the sign and exponent bits of a binary16 (a shift by ten places
 * towards the most significant bit) and added, as a 16-bit integer, to the bit
 * pattern of the scale. */
uint16_t orc_decode_bits(unsigned code, uint16_t scale_bits, int bits)
{
    unsigned sign = (code >> (bits - 1)) & 1u;
    unsigned E = code & ((1u << (bits - 1)) - 1u);
    unsigned field6 = (sign << 5) | E;
    return (uint16_t)(scale_bits + (uint16_t)(field6 << 10));
}

/* A scale is inside the domain on which the recipe equals the definition when
 * it is a positive normal binary16 whose biased exponent e satisfies
 * 1 <= e <= 30 - q_max, so that s * 2^q_max is still finite. */
int orc_scale_in_domain(uint16_t scale_bits, int bits)
{
    int qmax = (1 << (bits - 1)) - 1;
    int sign = (scale_bits >> 15) & 1;
    int efield = (scale_bits >> 10) & 0x1F;
    return !sign && efield >= 1 && efield <= 30 - qmax;
}

int64_t orc_check_scales(const uint16_t *scales, int64_t count, int bits)
{
    int64_t bad = 0;
    for (int64_t i = 0; i < count; ++i) bad += !orc_scale_in_domain(scales[i], bits);
    return bad;
}

/* -------------------------------------------------------------- dequant -- */

/* out[n,k] (row-major N x K binary16) = decode(code[n,k], scales[n, k div G]).
 * use_bit_recipe = 0: the definition; 1: the Sec. 4.2 integer-add recipe (they
 * are the same function on the scale domain above; the library's behaviour
 * outside that domain is, by its contract, the recipe's wrap-around). */
void orc_pot_dequant(const uint8_t *packed, const uint16_t *scales, uint16_t *out,
                     int64_t N, int64_t K, int bits, int group, int use_bit_recipe, int nthreads)
{
    size_t rb = orc_packed_row_bytes(K, bits);
    int64_t ngroups = K / group;
    (void)nthreads;
#if defined(_OPENMP)
#pragma omp parallel for num_threads(nthreads > 0 ? nthreads : 1) schedule(static)
#endif
    for (int64_t n = 0; n < N; ++n) {
        const uint8_t *row = packed + rb * (size_t)n;
        for (int64_t k = 0; k < K; ++k) {
            unsigned c = get_code(row, k, bits);
            uint16_t s = scales[n * ngroups + k / group];
            out[n * K + k] = use_bit_recipe ? orc_decode_bits(c, s, bits) : orc_decode_def(c, s, bits);
        }
    }
}

/* Uniform baseline (Sec. 4.1 Eq. (9)): W_Q is the unsigned code, Z the group's
 * zero-point and S the group's scale (both binary16); the exact real product
 * (W_Q + Z) * S is rounded once to binary16. */
uint16_t orc_int_decode(unsigned code, uint16_t scale_bits, uint16_t zero_bits)
{
    double S = orc_half_to_double(scale_bits);
    double Z = orc_half_to_double(zero_bits);
    return orc_double_to_half(((double)code + Z) * S);
}

void orc_int_dequant(const uint8_t *packed, const uint16_t *scales, const uint16_t *zeros, uint16_t *out,
                     int64_t N, int64_t K, int bits, int group, int nthreads)
{
    size_t rb = orc_packed_row_bytes(K, bits);
    int64_t ngroups = K / group;
    (void)nthreads;
#if defined(_OPENMP)
#pragma omp parallel for num_threads(nthreads > 0 ? nthreads : 1) schedule(static)
#endif
    for (int64_t n = 0; n < N; ++n) {
        const uint8_t *row = packed + rb * (size_t)n;
        for (int64_t k = 0; k < K; ++k) {
            int64_t g = n * ngroups + k / group;
            out[n * K + k] = orc_int_decode(get_code(row, k, bits), scales[g], zeros[g]);
        }
    }
}

/* ---------------------------------------------------------- GEMV / GEMM -- */

/* Y[m,n] = round_fp16( sum_k X[m,k] * W~[n,k] ), W~ the binary16 de-quantised
 * matrix above, the sum taken in double in ascending k (every product of two
 * binary16 numbers is exact in double).  zeros == NULL selects PoT (by the
 * definition), otherwise the uniform baseline.  Y_f64, when not NULL, also
 * receives the unrounded sums.  M = 1 is the GEMV. */
void orc_gemm(const uint8_t *packed, const uint16_t *scales, const uint16_t *zeros,
              const uint16_t *X, uint16_t *Y, double *Y_f64,
              int64_t M, int64_t N, int64_t K, int bits, int group, int nthreads)
{
    size_t rb = orc_packed_row_bytes(K, bits);
    int64_t ngroups = K / group;
    (void)nthreads;
#if defined(_OPENMP)
#pragma omp parallel for num_threads(nthreads > 0 ? nthreads : 1) schedule(static)
#endif
    for (int64_t n = 0; n < N; ++n) {
        const uint8_t *row = packed + rb * (size_t)n;
        /* row n of W~, first as binary16 bits and then as its exact double value */
        double *wrow = (double *)malloc(sizeof(double) * (size_t)K);
        for (int64_t k = 0; k < K; ++k) {
            unsigned c = get_code(row, k, bits);
            int64_t g = n * ngroups + k / group;
            uint16_t wbits = zeros ? orc_int_decode(c, scales[g], zeros[g])
                                   : orc_decode_def(c, scales[g], bits);
            wrow[k] = orc_half_to_double(wbits);
        }
        for (int64_t m = 0; m < M; ++m) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k)
                acc += wrow[k] * orc_half_to_double(X[m * K + k]);
            Y[m * N + n] = orc_double_to_half(acc);
            if (Y_f64) Y_f64[m * N + n] = acc;
        }
        free(wrow);
    }
}

int orc_max_threads(void)
{
#if defined(_OPENMP)
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------- Step 1 scale search (Alg. 1) -- */

/*
 * Data-agnostic scale initialisation, Sec. 3.2 / Algorithm 1, for one matrix of
 * binary16 weights: for every group of `group` consecutive weights of a row
 *     s0 = max|w| / (2^qmax - 1)
 *     for i = 1..200:  s = s0 * (0.01 * i)
 *         E_k = clamp(round(log2(|w_k| / s)), 0, qmax),   w~_k = sign(w_k) * s * 2^E_k
 *         Q(i) = sum_k (w_k - w~_k)^2 ;  keep i if Q(i) < best so far (strict: first minimum wins)
 *     scale = s0 * (0.01 * i*),  codes = (sign, E) under that scale.
 *
 * The paper leaves the arithmetic open.  So that the integer decisions (E, the
 * arg-min) are well defined and can be reproduced bit for bit, this oracle fixes
 * it as IEEE binary32 throughout, one rounding per operation, no contraction:
 *   - b_i = (float)i * 0.01f ; s0 by a binary32 division; the candidate scale is what would be
 *     stored and used at inference (Sec. 4.2 keeps the scale as FP16): s = s0 * b_i rounded once
 *     to binary16 and clamped into the domain on which the de-quantisation recipe is exact
 *     ([2^-14, largest value with exponent field 30 - qmax]); thresholds, reconstruction and
 *     error are taken from that value, so Q(i) is the error of exactly what pot_dequant rebuilds;
 *   - round(log2(|w|/s)) is taken through its decision thresholds: E = number of
 *     e in 1..qmax with |w| >= s * c_e, c_e = (float)2^(e - 1/2) (a tie on a
 *     threshold rounds up; |w| = 0 gives E = 0 as clamp(-inf) does);
 *   - w~ = s * 2^E is exact; d = w - w~ ; Q = fmaf(d, d, Q), k ascending;
 *   - sign(0) = +, i.e. the sign bit is set only for w < 0;
 *   - an all-zero group (s0 = 0) has every candidate clamped to 2^-14, equal errors, i* = 1
 *     and E = 0 everywhere.
 * codes: N*K bytes, one code per byte.  best_i (optional): N*(K/group) ints.
 */
static const float k_round_thresholds[8] = {
    0.0f, 1.41421356237309504880f, 2.82842712474619009760f, 5.65685424949238019521f,
    11.3137084989847603904f, 22.6274169979695207808f, 45.2548339959390415616f, 90.5096679918780831232f};

/* Candidate i of a group: binary16 pattern of the scale as it would be stored. */
static uint16_t quantize_candidate(float s0, int i, int qmax)
{
    const float s = s0 * ((float)i * 0.01f);
    uint16_t sb = orc_double_to_half((double)s);
    const uint16_t lo = 0x0400, hi = (uint16_t)(((30 - qmax) << 10) | 0x3FF);
    if (sb < lo) sb = lo;          /* positive patterns order like the values */
    if (sb > hi) sb = hi;
    return sb;
}

void orc_pot_quantize(const uint16_t *W, uint8_t *codes, uint16_t *scales, int32_t *best_i,
                      int64_t N, int64_t K, int bits, int group, int nthreads)
{
    const int qmax = (1 << (bits - 1)) - 1;
    const int64_t ngroups = K / group;
    const float denom = (float)((1 << qmax) - 1);
    (void)nthreads;
#if defined(_OPENMP)
#pragma omp parallel for num_threads(nthreads > 0 ? nthreads : 1) schedule(static)
#endif
    for (int64_t n = 0; n < N; ++n) {
        float *w = (float *)malloc(sizeof(float) * (size_t)group);
        for (int64_t g = 0; g < ngroups; ++g) {
            const uint16_t *src = W + n * K + g * group;
            uint8_t *dst = codes + n * K + g * group;
            float wmax = 0.0f;
            for (int k = 0; k < group; ++k) {
                w[k] = (float)orc_half_to_double(src[k]);      /* exact: binary16 is a subset of binary32 */
                if (fabsf(w[k]) > wmax) wmax = fabsf(w[k]);
            }
            const float s0 = wmax / denom;
            int ibest = 1;
            float qbest = INFINITY;
            for (int i = 1; i <= 200; ++i) {
                const float s = (float)orc_half_to_double(quantize_candidate(s0, i, qmax));
                float q = 0.0f;
                for (int k = 0; k < group; ++k) {
                    const float a = fabsf(w[k]);
                    int E = 0;
                    for (int e = 1; e <= qmax; ++e)
                        if (a >= s * k_round_thresholds[e]) E = e;
                    const float mag = ldexpf(s, E);
                    const float wq = w[k] < 0.0f ? -mag : mag;
                    const float d = w[k] - wq;
                    q = fmaf(d, d, q);
                }
                if (q < qbest) {
                    qbest = q;
                    ibest = i;
                }
            }
            const uint16_t sb = quantize_candidate(s0, ibest, qmax);
            const float sbest = (float)orc_half_to_double(sb);
            for (int k = 0; k < group; ++k) {
                const float a = fabsf(w[k]);
                int E = 0;
                for (int e = 1; e <= qmax; ++e)
                    if (a >= sbest * k_round_thresholds[e]) E = e;
                dst[k] = (uint8_t)((w[k] < 0.0f ? (1 << (bits - 1)) : 0) | E);
            }
            scales[n * ngroups + g] = sb;
            if (best_i) best_i[n * ngroups + g] = ibest;
        }
        free(w);
    }
}

/* --------------------------- Step 2 fake-quantisation op (Sec. 3.3, Alg. 2) -- */

/*
 * The weight path of one fine-tuning iteration, Sec. 3.3: with the learnable
 * residual Gamma (one binary32 per group) the scale becomes
 *     S^ = S * (1 + Gamma)                                   (refined scale)
 *     E_k = clamp(round(log2(|w_k| / S^)), 0, qmax)           (exponent under S^)
 *     w~_k = S^ * sign(w_k) * 2^E_k                           (reconstruction)
 * and the gradient of a loss L with respect to Gamma follows from the
 * straight-through estimator: round() is differentiated as the identity, so
 * inside the clamp dE/dS^ = -1 / (S^ ln 2) and the two terms of
 * dw~/dS^ = P 2^E + S^ P 2^E ln2 dE/dS^ cancel, while where the clamp is active
 * (round(log2(|w|/S^)) < 0 or > qmax) dE/dS^ = 0 and dw~/dS^ = P 2^E.  Hence
 *     dL/dGamma_g = S_g * sum_{k in g, clamp active at k} (dL/dw~_k) * sign(w_k) * 2^E_k .
 * (The paper states the estimator for round() only; the clamp is differentiated
 * as it stands, derivative 1 on the closed interval [0, qmax] and 0 outside.)
 *
 * Arithmetic, fixed as for the scale search so that the integer decisions can be
 * reproduced bit for bit: binary32, one rounding per operation, no contraction;
 * S^ = S * (1.0f + Gamma); round(log2(.)) through its thresholds S^ * (float)2^(e-1/2)
 * (a tie rounds up); below-range means |w| < S^ * (float)2^(-1/2), above-range
 * |w| >= S^ * (float)2^(qmax+1/2); |w| = 0 is below range, sign(0) = +.
 * The forward result S^ * 2^E is exact in binary32 and is rounded once to
 * binary16.  The backward sum is taken in binary64 (k ascending) and rounded
 * once to binary32; the incoming gradient is binary16.
 */
static const float k_inv_sqrt2 = 0.70710678118654752440f;

static int fq_exponent(float a, float shat, int qmax, int *clamped)
{
    int E = 0;
    for (int e = 1; e <= qmax; ++e)
        if (a >= shat * k_round_thresholds[e]) E = e;
    const float top = shat * (k_round_thresholds[qmax] * 2.0f);   /* (float)2^(qmax+1/2): doubling is exact */
    *clamped = (a < shat * k_inv_sqrt2) || (a >= top);
    return E;
}

void orc_fakequant_forward(const uint16_t *W, const uint16_t *S, const float *Gamma, uint16_t *Wq,
                           int64_t N, int64_t K, int bits, int group, int nthreads)
{
    const int qmax = (1 << (bits - 1)) - 1;
    const int64_t ngroups = K / group;
    (void)nthreads;
#if defined(_OPENMP)
#pragma omp parallel for num_threads(nthreads > 0 ? nthreads : 1) schedule(static)
#endif
    for (int64_t n = 0; n < N; ++n)
        for (int64_t g = 0; g < ngroups; ++g) {
            const float s = (float)orc_half_to_double(S[n * ngroups + g]);
            const float shat = s * (1.0f + Gamma[n * ngroups + g]);
            for (int k = 0; k < group; ++k) {
                const int64_t at = n * K + g * group + k;
                const float w = (float)orc_half_to_double(W[at]);
                int clamped;
                const int E = fq_exponent(fabsf(w), shat, qmax, &clamped);
                const float mag = ldexpf(shat, E);
                Wq[at] = orc_double_to_half((double)(w < 0.0f ? -mag : mag));
            }
        }
}

void orc_fakequant_backward(const uint16_t *W, const uint16_t *S, const float *Gamma, const uint16_t *dWq,
                            float *dGamma, int64_t N, int64_t K, int bits, int group, int nthreads)
{
    const int qmax = (1 << (bits - 1)) - 1;
    const int64_t ngroups = K / group;
    (void)nthreads;
#if defined(_OPENMP)
#pragma omp parallel for num_threads(nthreads > 0 ? nthreads : 1) schedule(static)
#endif
    for (int64_t n = 0; n < N; ++n)
        for (int64_t g = 0; g < ngroups; ++g) {
            const float s = (float)orc_half_to_double(S[n * ngroups + g]);
            const float shat = s * (1.0f + Gamma[n * ngroups + g]);
            double sum = 0.0;
            for (int k = 0; k < group; ++k) {
                const int64_t at = n * K + g * group + k;
                const float w = (float)orc_half_to_double(W[at]);
                int clamped;
                const int E = fq_exponent(fabsf(w), shat, qmax, &clamped);
                if (clamped) {
                    const double p = ldexp(1.0, E);
                    sum += orc_half_to_double(dWq[at]) * (w < 0.0f ? -p : p);
                }
            }
            dGamma[n * ngroups + g] = (float)((double)s * sum);
        }
}
