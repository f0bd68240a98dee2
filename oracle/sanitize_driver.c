/*
 * TEST INFRASTRUCTURE: runs every function of potq_oracle.c once on small inputs held in
 * heap blocks of exactly the size the function may touch, so that a build with
 * -fsanitize=address,undefined reports any access outside them or any undefined
 * arithmetic (tests/test_oracle_sanitizers.py builds and runs it).  It checks only a few
 * round trips itself; what the functions compute is pinned by the Python tests.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

double orc_half_to_double(uint16_t h);
uint16_t orc_double_to_half(double v);
size_t orc_packed_row_bytes(int64_t K, int bits);
void orc_pack_codes(const uint8_t *codes, uint8_t *packed, int64_t N, int64_t K, int bits);
void orc_unpack_codes(const uint8_t *packed, uint8_t *codes, int64_t N, int64_t K, int bits);
uint16_t orc_decode_def(unsigned code, uint16_t scale_bits, int bits);
uint16_t orc_decode_bits(unsigned code, uint16_t scale_bits, int bits);
int orc_scale_in_domain(uint16_t scale_bits, int bits);
int64_t orc_check_scales(const uint16_t *scales, int64_t count, int bits);
void orc_pot_dequant(const uint8_t *packed, const uint16_t *scales, uint16_t *out, int64_t N, int64_t K, int bits,
                     int group, int use_bit_recipe, int nthreads);
uint16_t orc_int_decode(unsigned code, uint16_t scale_bits, uint16_t zero_bits);
void orc_int_dequant(const uint8_t *packed, const uint16_t *scales, const uint16_t *zeros, uint16_t *out, int64_t N,
                     int64_t K, int bits, int group, int nthreads);
void orc_gemm(const uint8_t *packed, const uint16_t *scales, const uint16_t *zeros, const uint16_t *X, uint16_t *Y,
              double *Y64, int64_t M, int64_t N, int64_t K, int bits, int group, int nthreads);
void orc_pot_quantize(const uint16_t *W, uint8_t *codes, uint16_t *scales, int32_t *best_i, int64_t N, int64_t K,
                      int bits, int group, int nthreads);
void orc_fakequant_forward(const uint16_t *W, const uint16_t *S, const float *Gamma, uint16_t *Wq, int64_t N,
                           int64_t K, int bits, int group, int nthreads);
void orc_fakequant_backward(const uint16_t *W, const uint16_t *S, const float *Gamma, const uint16_t *dWq,
                            float *dGamma, int64_t N, int64_t K, int bits, int group, int nthreads);

static uint32_t rng_state = 12345u;
static uint32_t rnd(void)
{
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 17;
    rng_state ^= rng_state << 5;
    return rng_state;
}

static void *exact(size_t bytes) { return malloc(bytes ? bytes : 1); }

int main(void)
{
    /* conversions over every pattern and a spread of doubles, including the non-finite ones */
    for (unsigned h = 0; h < 65536u; ++h) {
        const double d = orc_half_to_double((uint16_t)h);
        const uint16_t back = orc_double_to_half(d);
        if (d == d && back != h) { printf("fp16 round trip failed at %04x\n", h); return 1; }
    }
    const double specials[] = {0.0, -0.0, 1e-30, -1e-30, 65504.0, 65520.0, 1e30, -1e30, INFINITY, -INFINITY, NAN, 6e-8, 2.98e-8};
    for (size_t i = 0; i < sizeof specials / sizeof specials[0]; ++i) (void)orc_double_to_half(specials[i]);

    for (int bits = 2; bits <= 4; ++bits) {
        for (unsigned code = 0; code < (1u << bits); ++code)
            for (unsigned s = 0; s < 65536u; s += 37) {
                (void)orc_decode_def(code, (uint16_t)s, bits);
                (void)orc_decode_bits(code, (uint16_t)s, bits);
                (void)orc_int_decode(code, (uint16_t)s, (uint16_t)(0xC000u | (code << 6)));
                (void)orc_scale_in_domain((uint16_t)s, bits);
            }
        for (int group = 64; group <= 128; group += 64) {
            const int64_t N = 5, K = 384, M = 3, G = K / group;
            const size_t rb = orc_packed_row_bytes(K, bits);
            uint8_t *codes = exact((size_t)(N * K)), *codes2 = exact((size_t)(N * K)), *packed = exact((size_t)N * rb);
            uint16_t *scales = exact(sizeof(uint16_t) * (size_t)(N * G)), *zeros = exact(sizeof(uint16_t) * (size_t)(N * G));
            uint16_t *out = exact(sizeof(uint16_t) * (size_t)(N * K)), *W = exact(sizeof(uint16_t) * (size_t)(N * K));
            uint16_t *X = exact(sizeof(uint16_t) * (size_t)(M * K)), *Y = exact(sizeof(uint16_t) * (size_t)(M * N));
            double *Y64 = exact(sizeof(double) * (size_t)(M * N));
            float *Gamma = exact(sizeof(float) * (size_t)(N * G)), *dGamma = exact(sizeof(float) * (size_t)(N * G));
            int32_t *best = exact(sizeof(int32_t) * (size_t)(N * G));
            for (int64_t i = 0; i < N * K; ++i) {
                codes[i] = (uint8_t)(rnd() & ((1u << bits) - 1u));
                W[i] = orc_double_to_half(((double)(rnd() % 20001u) - 10000.0) * 4e-6);
            }
            for (int64_t i = 0; i < N * G; ++i) {
                scales[i] = (uint16_t)(0x2800u + (rnd() & 0x7FFu));
                zeros[i] = orc_double_to_half(-(double)(rnd() % (1u << bits)));
                Gamma[i] = ((float)(rnd() % 2001u) - 1000.0f) * 2e-4f;
            }
            for (int64_t i = 0; i < M * K; ++i) X[i] = orc_double_to_half(((double)(rnd() % 8001u) - 4000.0) * 1e-3);
            X[7] = 0x7C00u;     /* an infinity and a NaN among the activations */
            X[K + 9] = 0x7E00u;
            orc_pack_codes(codes, packed, N, K, bits);
            orc_unpack_codes(packed, codes2, N, K, bits);
            if (memcmp(codes, codes2, (size_t)(N * K)) != 0) { printf("pack round trip failed\n"); return 1; }
            (void)orc_check_scales(scales, N * G, bits);
            orc_pot_dequant(packed, scales, out, N, K, bits, group, 0, 2);
            orc_pot_dequant(packed, scales, out, N, K, bits, group, 1, 1);
            orc_int_dequant(packed, scales, zeros, out, N, K, bits, group, 2);
            orc_gemm(packed, scales, NULL, X, Y, Y64, M, N, K, bits, group, 2);
            orc_gemm(packed, scales, zeros, X, Y, NULL, M, N, K, bits, group, 1);
            orc_pot_quantize(W, codes2, scales, best, N, K, bits, group, 2);
            memset(W, 0, sizeof(uint16_t) * (size_t)group);        /* an all-zero group */
            orc_pot_quantize(W, codes2, scales, NULL, N, K, bits, group, 1);
            orc_fakequant_forward(W, scales, Gamma, out, N, K, bits, group, 2);
            orc_fakequant_backward(W, scales, Gamma, out, dGamma, N, K, bits, group, 2);
            /* empty inputs touch nothing */
            orc_pot_dequant(packed, scales, out, 0, K, bits, group, 0, 1);
            orc_gemm(packed, scales, NULL, X, Y, NULL, 0, N, K, bits, group, 1);
            free(codes); free(codes2); free(packed); free(scales); free(zeros); free(out); free(W); free(X); free(Y);
            free(Y64); free(Gamma); free(dGamma); free(best);
        }
    }
    printf("oracle sanitizer driver: ok\n");
    return 0;
}
