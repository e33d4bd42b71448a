/* Driver for a host-sanitizer build of the CPU oracle (tests/test_oracle_sanitized.py compiles this
 * file together with oracle/goq_oracle.c under AddressSanitizer and UndefinedBehaviorSanitizer).
 * Every buffer is a heap allocation of exactly the size the interface states, so that an access one
 * element out of range is reported.  Besides running every entry point on both bit widths it checks
 * one identity that ties them together: y of gemm_a16 equals x times the dequantised matrix. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

double goq_oracle_half_to_double(uint16_t h);
uint16_t goq_oracle_double_to_half(double d);
int goq_oracle_quantize_geo(int bw, int64_t out, int64_t in, const float *w, uint8_t *codes, uint8_t *pattern,
                            uint8_t *signs, uint16_t *c1, uint16_t *c2, int threads);
int goq_oracle_dequant(int bw, int64_t out, int64_t in, const uint8_t *codes, const uint8_t *pattern,
                       const uint8_t *signs, const uint16_t *c1, const uint16_t *c2, double *B1, double *B2,
                       double *What);
int goq_oracle_gemm_a16(int bw, int64_t tokens, int64_t out, int64_t in, const uint8_t *codes,
                        const uint8_t *pattern, const uint8_t *signs, const uint16_t *c1, const uint16_t *c2,
                        const uint16_t *x, double *y, int threads);
int goq_oracle_gemm_a8(int bw, int64_t tokens, int64_t out, int64_t in, const uint8_t *codes,
                       const uint8_t *pattern, const uint8_t *signs, const uint16_t *c1, const uint16_t *c2,
                       const int8_t *x, const float *sx, double *y, int32_t *partials, int threads);
int goq_oracle_ref_coefficients(int bw, int64_t tokens, int64_t out, int64_t in, const float *w,
                                const uint8_t *codes, const uint8_t *pattern, const uint8_t *signs,
                                const uint16_t *x, double lambda, double *craw, uint16_t *c1, uint16_t *c2,
                                int threads);

static uint64_t state = 0x9E3779B97F4A7C15ull;
static double uniform(void)
{
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return (double)(state >> 11) / 9007199254740992.0 - 0.5;
}

int main(void)
{
    const int64_t out = 37, in = 384, tokens = 5, gn = in / 128;
    for (int bw = 3; bw <= 4; ++bw) {
        float *w = malloc(sizeof(float) * out * in);
        uint16_t *x = malloc(sizeof(uint16_t) * tokens * in);
        int8_t *xq = malloc(tokens * in);
        float *sx = malloc(sizeof(float) * tokens);
        for (int64_t i = 0; i < out * in; ++i) w[i] = (float)goq_oracle_half_to_double(goq_oracle_double_to_half(0.05 * uniform()));
        for (int64_t i = 0; i < 128; ++i) w[in + i] = 0.f;                      /* an all-zero macro-block */
        for (int64_t i = 0; i < tokens * in; ++i) { x[i] = goq_oracle_double_to_half(4.0 * uniform()); xq[i] = (int8_t)lrint(254.0 * uniform()); }
        for (int64_t t = 0; t < tokens; ++t) sx[t] = 0.01f * (float)(t + 1);
        uint8_t *codes = malloc(out * in), *pattern = malloc(out * in / 8), *signs = malloc(out * in / 8);
        uint16_t *c1 = malloc(sizeof(uint16_t) * out * gn), *c2 = malloc(sizeof(uint16_t) * out * gn);
        if (goq_oracle_quantize_geo(bw, out, in, w, codes, pattern, signs, c1, c2, 2)) return 1;
        double *What = malloc(sizeof(double) * out * in);
        if (goq_oracle_dequant(bw, out, in, codes, pattern, signs, c1, c2, NULL, NULL, What)) return 2;
        double *y = malloc(sizeof(double) * tokens * out);
        if (goq_oracle_gemm_a16(bw, tokens, out, in, codes, pattern, signs, c1, c2, x, y, 2)) return 3;
        for (int64_t t = 0; t < tokens; ++t)
            for (int64_t o = 0; o < out; ++o) {
                double ref = 0.0, scale = 0.0;
                for (int64_t k = 0; k < in; ++k) {
                    const double xv = goq_oracle_half_to_double(x[t * in + k]);
                    ref += xv * What[o * in + k];
                    scale += fabs(xv * What[o * in + k]);
                }
                if (fabs(ref - y[t * out + o]) > 1e-12 * (scale + 1e-30)) { printf("mismatch bw %d t %ld o %ld\n", bw, (long)t, (long)o); return 4; }
            }
        int32_t *partials = malloc(sizeof(int32_t) * tokens * out * gn * 2);
        if (goq_oracle_gemm_a8(bw, tokens, out, in, codes, pattern, signs, c1, c2, xq, sx, y, partials, 2)) return 5;
        if (goq_oracle_gemm_a8(bw, tokens, out, in, codes, pattern, signs, c1, c2, xq, sx, y, NULL, 1)) return 6;
        double *craw = malloc(sizeof(double) * out * gn * 2);
        uint16_t *r1 = malloc(sizeof(uint16_t) * out * gn), *r2 = malloc(sizeof(uint16_t) * out * gn);
        if (goq_oracle_ref_coefficients(bw, tokens, out, in, w, codes, pattern, signs, x, 1e-4, craw, r1, r2, 2)) return 7;
        if (goq_oracle_ref_coefficients(bw, tokens, out, in, w, codes, pattern, signs, x, 1e-4, NULL, r1, r2, 1)) return 8;
        /* argument errors are return codes, not accesses */
        if (goq_oracle_quantize_geo(5, out, in, w, codes, pattern, signs, c1, c2, 1) == 0) return 9;
        if (goq_oracle_gemm_a16(bw, tokens, out, in + 1, codes, pattern, signs, c1, c2, x, y, 1) == 0) return 10;
        free(w); free(x); free(xq); free(sx); free(codes); free(pattern); free(signs); free(c1); free(c2);
        free(What); free(y); free(partials); free(craw); free(r1); free(r2);
    }
    /* fp16 conversions over every bit pattern: round trip is the identity on non-NaN values */
    for (uint32_t h = 0; h < 65536; ++h) {
        const double d = goq_oracle_half_to_double((uint16_t)h);
        if (d == d && goq_oracle_double_to_half(d) != (uint16_t)h && !(d == 0.0)) { printf("half %u\n", h); return 11; }
    }
    printf("sanitized oracle run: ok\n");
    return 0;
}
