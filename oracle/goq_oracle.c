/*
 * GoQuant CPU oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, scalar fp64 implementation of
 *   (Q) the data-free GEO-mode analytical quantizer          (Sec. 3.2, 3.3, 3.4)
 *   (D) the dual power-of-two (PoT) inner product of a layer  (Sec. 3.5, Eq. 4)
 *   (R) the REF-mode activation-aware coefficients            (Sec. 3.4, Eq. 3)
 * written from the paper's equations in the paper's order.  It shares no code
 * with the HIP library; only tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it.
 *
 * Pins (tests/test_oracle_*.py): printed 3-bit lattice and pair sets, Theorem 1
 * orthogonality over all 64 (pattern, sign) choices, brute force over the
 * lattice per element and over the 64 exchange candidates per micro-block,
 * generic least squares for the coefficients, dense fp64 matmul of the
 * dequantised matrix, exact integer partials, a hand-derived worked example;
 * for (R): generic least squares on the ridge-augmented system, the closed form
 * for identity calibration inputs (which ties it to Eq. 2), exact recovery of
 * weights that lie in the span of the two bases.
 * Parity unpinned by the paper itself (pinned only by this build's readings):
 * the 4-bit lattice, rounding ties, the all-zero block, the code numbering and
 * the fp16 storage of coefficients.
 *
 * Notation follows the paper: N = 128 (macro-block), G = 8 (micro-block),
 * b1 primary basis, r_perp orthogonal residual, s in {1,2,3,4} exchange pattern,
 * eta pair sign, b2 secondary basis, c1/c2 block coefficients.
 *
 * Canonical arrays (row-major, a layer is W[out][in] like a linear layer's weight):
 *   codes   u8 [out][in]      code = sign << (bw-1) | e ; value (-1)^sign * 2^-e,
 *                             except (sign = 0, e = 2^(bw-1) - 1) which is exact zero
 *                             (the smallest positive bin is repurposed, Sec. 3.2)
 *   pattern u8 [out][in/8]    s - 1
 *   signs   u8 [out][in/8]    bit p = 1  <=>  eta of the p-th pair (ascending i) is -1
 *   c1, c2  u16 [out][in/128] IEEE binary16 bit patterns
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define GOQ_N 128
#define GOQ_G 8

/* ---------------------------------------------------------------- fp16 <-> fp64 */

double goq_oracle_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int exp = (h >> 10) & 0x1f;
    int man = h & 0x3ff;
    double v;
    if (exp == 0)
        v = ldexp((double)man, -24);          /* zero and subnormals */
    else if (exp == 31)
        v = man ? NAN : INFINITY;
    else
        v = ldexp((double)(man | 0x400), exp - 25);
    return sign ? -v : v;
}

/* round-to-nearest-even from fp64 straight to binary16 (no intermediate fp32) */
uint16_t goq_oracle_double_to_half(double d)
{
    uint16_t sign = signbit(d) ? 0x8000 : 0;
    double a = fabs(d);
    if (isnan(d)) return 0x7e00;
    if (a >= 65520.0) return sign | 0x7c00;   /* rounds to infinity */
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);                       /* a = f * 2^e, f in [0.5, 1) */
    int ex = e - 1;                           /* a in [2^ex, 2^(ex+1)) */
    if (ex < -14) ex = -14;                   /* subnormal range: fixed quantum 2^-24 */
    double q = ldexp(a, 10 - ex);             /* in units of the quantum 2^(ex-10); exact */
    double r = nearbyint(q);                  /* default rounding mode: ties to even */
    /* r in [0, 2048]; r == 2048 carries into the next binade */
    int m = (int)r;
    int be = ex + 15;                         /* biased exponent if normal */
    if (ex == -14 && m < 1024) return sign | (uint16_t)m;   /* subnormal (or zero) */
    if (m == 2048) { m = 1024; be += 1; }
    if (be >= 31) return sign | 0x7c00;
    return sign | (uint16_t)(be << 10) | (uint16_t)(m & 0x3ff);
}

/* ---------------------------------------------------------------- lattice (Sec. 3.2) */

/* number of magnitudes per sign */
static int lattice_E(int bw) { return 1 << (bw - 1); }

/* value of one canonical code */
double goq_oracle_code_value(int bw, int code)
{
    int E = lattice_E(bw);
    int sign = (code >> (bw - 1)) & 1;
    int e = code & (E - 1);
    if (!sign && e == E - 1) return 0.0;      /* smallest positive bin -> exact zero */
    double v = ldexp(1.0, -e);
    return sign ? -v : v;
}

/* L[0 .. 2^bw - 1] */
int goq_oracle_lattice(int bw, double *L)
{
    if (bw != 3 && bw != 4) return -1;
    for (int c = 0; c < (1 << bw); ++c) L[c] = goq_oracle_code_value(bw, c);
    return 0;
}

/* Q(.): nearest lattice state in linear distance; an exact tie goes to the state of
 * smaller magnitude (toward zero). */
static int nearest_code(int bw, double v)
{
    int best = 0;
    double bestd = INFINITY, bestabs = INFINITY;
    for (int c = 0; c < (1 << bw); ++c) {
        double l = goq_oracle_code_value(bw, c);
        double d = fabs(v - l);
        if (d < bestd || (d == bestd && fabs(l) < bestabs)) {
            best = c; bestd = d; bestabs = fabs(l);
        }
    }
    return best;
}

/* ---------------------------------------------------------------- exchange (Theorem 1) */

/* b2 micro-block from b1 micro-block x[0..7], pattern s in 1..4 and the sign nibble:
 * for every pair (i, j = i xor s), i < j, taken in ascending i,
 *     y_i = -eta * x_j ,  y_j = +eta * x_i ,   eta = -1 iff the pair's bit is set. */
void goq_oracle_exchange(const double *x, int s, int signs, double *y)
{
    int p = 0;
    for (int i = 0; i < GOQ_G; ++i) {
        int j = i ^ s;
        if (i < j) {
            double eta = ((signs >> p) & 1) ? -1.0 : 1.0;
            y[i] = -eta * x[j];
            y[j] = eta * x[i];
            ++p;
        }
    }
}

/* ---------------------------------------------------------------- Part Q: GEO quantizer */

/* One macro-block w[0..127] (fp16-valued weights held in double).
 * Outputs: codes[128], pattern[16], signs[16], c1, c2 (unrounded fp64). */
void goq_oracle_quantize_block(int bw, const double *w, uint8_t *codes, uint8_t *pattern,
                               uint8_t *signs, double *c1, double *c2)
{
    double b1[GOQ_N], b2[GOQ_N], r[GOQ_N];

    /* macro-block normalisation s_norm = ||w||_inf, v = w / s_norm */
    double snorm = 0.0;
    for (int k = 0; k < GOQ_N; ++k) if (fabs(w[k]) > snorm) snorm = fabs(w[k]);
    if (snorm == 0.0) {                        /* all-zero block: nothing to represent */
        int zero_code = lattice_E(bw) - 1;
        for (int k = 0; k < GOQ_N; ++k) codes[k] = (uint8_t)zero_code;
        memset(pattern, 0, GOQ_N / GOQ_G);
        memset(signs, 0, GOQ_N / GOQ_G);
        *c1 = 0.0; *c2 = 0.0;
        return;
    }
    /* primary projection b1 = Q(v) */
    for (int k = 0; k < GOQ_N; ++k) {
        double v = w[k] / snorm;
        codes[k] = (uint8_t)nearest_code(bw, v);
        b1[k] = goq_oracle_code_value(bw, codes[k]);
    }
    /* orthogonal residual, Eq. 1 */
    double wb1 = 0.0, n1 = 0.0;
    for (int k = 0; k < GOQ_N; ++k) { wb1 += w[k] * b1[k]; n1 += b1[k] * b1[k]; }
    for (int k = 0; k < GOQ_N; ++k) r[k] = (n1 > 0.0) ? w[k] - (wb1 / n1) * b1[k] : w[k];

    /* per micro-block: analytical signs, alignment score A_s, pattern argmax */
    for (int m = 0; m < GOQ_N / GOQ_G; ++m) {
        const double *x = b1 + GOQ_G * m;
        const double *rp = r + GOQ_G * m;
        int best_s = 1, best_signs = 0;
        double bestA = -1.0;
        for (int s = 1; s <= 4; ++s) {
            double A = 0.0;
            int sg = 0, p = 0;
            for (int i = 0; i < GOQ_G; ++i) {
                int j = i ^ s;
                if (i < j) {
                    double t = x[i] * rp[j] - x[j] * rp[i];
                    A += fabs(t);
                    if (t < 0.0) sg |= 1 << p;          /* eta = sgn(t); +1 when t == 0 */
                    ++p;
                }
            }
            if (A > bestA) { bestA = A; best_s = s; best_signs = sg; }   /* ties: smallest s */
        }
        pattern[m] = (uint8_t)(best_s - 1);
        signs[m] = (uint8_t)best_signs;
        goq_oracle_exchange(x, best_s, best_signs, b2 + GOQ_G * m);
    }
    /* GEO coefficients, Eq. 2 (diagonal normal equations) */
    double wb2 = 0.0, n2 = 0.0;
    for (int k = 0; k < GOQ_N; ++k) { wb2 += w[k] * b2[k]; n2 += b2[k] * b2[k]; }
    *c1 = (n1 > 0.0) ? wb1 / n1 : 0.0;
    *c2 = (n2 > 0.0) ? wb2 / n2 : 0.0;
}

/* Whole layer.  w is float32 holding fp16-representable values, [out][in]. */
int goq_oracle_quantize_geo(int bw, int64_t out, int64_t in, const float *w,
                            uint8_t *codes, uint8_t *pattern, uint8_t *signs,
                            uint16_t *c1, uint16_t *c2, int threads)
{
    if ((bw != 3 && bw != 4) || out <= 0 || in <= 0 || in % GOQ_N) return -1;
    int64_t gn = in / GOQ_N;
    (void)threads;
#pragma omp parallel for num_threads(threads > 0 ? threads : 1) schedule(static)
    for (int64_t o = 0; o < out; ++o) {
        for (int64_t g = 0; g < gn; ++g) {
            double wd[GOQ_N], a, b;
            const float *src = w + o * in + g * GOQ_N;
            for (int k = 0; k < GOQ_N; ++k) wd[k] = (double)src[k];
            goq_oracle_quantize_block(bw, wd, codes + o * in + g * GOQ_N,
                                      pattern + (o * in + g * GOQ_N) / GOQ_G,
                                      signs + (o * in + g * GOQ_N) / GOQ_G, &a, &b);
            c1[o * gn + g] = goq_oracle_double_to_half(a);
            c2[o * gn + g] = goq_oracle_double_to_half(b);
        }
    }
    return 0;
}

/* ---------------------------------------------------------------- Part D: dequantise */

/* b1, b2 of one row (length in) from the canonical arrays of that row */
static void row_bases(int bw, int64_t in, const uint8_t *codes, const uint8_t *pattern,
                      const uint8_t *signs, double *b1, double *b2)
{
    for (int64_t k = 0; k < in; ++k) b1[k] = goq_oracle_code_value(bw, codes[k]);
    for (int64_t m = 0; m < in / GOQ_G; ++m)
        goq_oracle_exchange(b1 + GOQ_G * m, pattern[m] + 1, signs[m], b2 + GOQ_G * m);
}

/* Dense bases and/or the dequantised matrix W^ = c1 b1 + c2 b2 (any output may be NULL) */
int goq_oracle_dequant(int bw, int64_t out, int64_t in, const uint8_t *codes,
                       const uint8_t *pattern, const uint8_t *signs, const uint16_t *c1,
                       const uint16_t *c2, double *B1, double *B2, double *What)
{
    if ((bw != 3 && bw != 4) || out <= 0 || in <= 0 || in % GOQ_N) return -1;
    int64_t gn = in / GOQ_N;
    double *b1 = (double *)malloc(sizeof(double) * in * 2), *b2 = b1 + in;
    if (!b1) return -2;
    for (int64_t o = 0; o < out; ++o) {
        row_bases(bw, in, codes + o * in, pattern + o * in / GOQ_G, signs + o * in / GOQ_G, b1, b2);
        for (int64_t k = 0; k < in; ++k) {
            int64_t g = k / GOQ_N;
            if (B1) B1[o * in + k] = b1[k];
            if (B2) B2[o * in + k] = b2[k];
            if (What)
                What[o * in + k] = goq_oracle_half_to_double(c1[o * gn + g]) * b1[k] +
                                   goq_oracle_half_to_double(c2[o * gn + g]) * b2[k];
        }
    }
    free(b1);
    return 0;
}

/* ---------------------------------------------------------------- Part D: layer output */

/* W/A16 (Eq. 4 read per 128-wide K slab, coefficients applied once per slab after the
 * slab's two dot products):
 *   P_m[t,o,g] = sum_{k in slab g} x[t,k] * b_m[o,k]
 *   y[t,o]     = sum_g ( c1[o,g] * P_1 + c2[o,g] * P_2 )
 * x: binary16 bit patterns [tokens][in]; y: fp64 [tokens][out]; everything in fp64. */
int goq_oracle_gemm_a16(int bw, int64_t tokens, int64_t out, int64_t in,
                        const uint8_t *codes, const uint8_t *pattern, const uint8_t *signs,
                        const uint16_t *c1, const uint16_t *c2, const uint16_t *x,
                        double *y, int threads)
{
    if ((bw != 3 && bw != 4) || tokens <= 0 || out <= 0 || in <= 0 || in % GOQ_N) return -1;
    int64_t gn = in / GOQ_N;
    double *xd = (double *)malloc(sizeof(double) * tokens * in);
    if (!xd) return -2;
    for (int64_t i = 0; i < tokens * in; ++i) xd[i] = goq_oracle_half_to_double(x[i]);
    int fail = 0;
#pragma omp parallel for num_threads(threads > 0 ? threads : 1) schedule(static)
    for (int64_t o = 0; o < out; ++o) {
        double *b1 = (double *)malloc(sizeof(double) * in * 2);
        if (!b1) { fail = 1; continue; }
        double *b2 = b1 + in;
        row_bases(bw, in, codes + o * in, pattern + o * in / GOQ_G, signs + o * in / GOQ_G, b1, b2);
        for (int64_t t = 0; t < tokens; ++t) {
            const double *xt = xd + t * in;
            double acc = 0.0;
            for (int64_t g = 0; g < gn; ++g) {
                double P1 = 0.0, P2 = 0.0;
                for (int64_t k = g * GOQ_N; k < (g + 1) * GOQ_N; ++k) {
                    P1 += xt[k] * b1[k];
                    P2 += xt[k] * b2[k];
                }
                acc += goq_oracle_half_to_double(c1[o * gn + g]) * P1 +
                       goq_oracle_half_to_double(c2[o * gn + g]) * P2;
            }
            y[t * out + o] = acc;
        }
        free(b1);
    }
    free(xd);
    return fail ? -2 : 0;
}

/* W/A8: the slab partials are exact integers on b_m * 2^(E-1):
 *   P_m[t,o,g] = sum_k x~[t,k] * (b_m[o,k] * 2^(E-1))            (int64 here, checked to fit int32)
 *   y[t,o]     = s_x[t] * 2^-(E-1) * sum_g ( c1 * P_1 + c2 * P_2 )  (fp64)
 * x: int8 [tokens][in]; sx: fp32 [tokens]; partials (may be NULL): int32 [tokens][out][in/128][2]. */
int goq_oracle_gemm_a8(int bw, int64_t tokens, int64_t out, int64_t in,
                       const uint8_t *codes, const uint8_t *pattern, const uint8_t *signs,
                       const uint16_t *c1, const uint16_t *c2, const int8_t *x, const float *sx,
                       double *y, int32_t *partials, int threads)
{
    if ((bw != 3 && bw != 4) || tokens <= 0 || out <= 0 || in <= 0 || in % GOQ_N) return -1;
    int64_t gn = in / GOQ_N;
    int E = lattice_E(bw);
    double scale = ldexp(1.0, E - 1);
    int fail = 0;
#pragma omp parallel for num_threads(threads > 0 ? threads : 1) schedule(static)
    for (int64_t o = 0; o < out; ++o) {
        double *b1 = (double *)malloc(sizeof(double) * in * 2);
        int64_t *i1 = (int64_t *)malloc(sizeof(int64_t) * in * 2);
        if (!b1 || !i1) { fail = 1; free(b1); free(i1); continue; }
        double *b2 = b1 + in;
        int64_t *i2 = i1 + in;
        row_bases(bw, in, codes + o * in, pattern + o * in / GOQ_G, signs + o * in / GOQ_G, b1, b2);
        for (int64_t k = 0; k < in; ++k) {      /* PoT * 2^(E-1) is an integer */
            i1[k] = (int64_t)(b1[k] * scale);
            i2[k] = (int64_t)(b2[k] * scale);
            if ((double)i1[k] != b1[k] * scale || (double)i2[k] != b2[k] * scale) fail = 2;
        }
        for (int64_t t = 0; t < tokens; ++t) {
            const int8_t *xt = x + t * in;
            double acc = 0.0;
            for (int64_t g = 0; g < gn; ++g) {
                int64_t P1 = 0, P2 = 0;
                for (int64_t k = g * GOQ_N; k < (g + 1) * GOQ_N; ++k) {
                    P1 += (int64_t)xt[k] * i1[k];
                    P2 += (int64_t)xt[k] * i2[k];
                }
                if (P1 > INT32_MAX || P1 < INT32_MIN || P2 > INT32_MAX || P2 < INT32_MIN) fail = 3;
                if (partials) {
                    partials[((t * out + o) * gn + g) * 2 + 0] = (int32_t)P1;
                    partials[((t * out + o) * gn + g) * 2 + 1] = (int32_t)P2;
                }
                acc += goq_oracle_half_to_double(c1[o * gn + g]) * (double)P1 +
                       goq_oracle_half_to_double(c2[o * gn + g]) * (double)P2;
            }
            y[t * out + o] = (double)sx[t] * (1.0 / scale) * acc;
        }
        free(b1);
        free(i1);
    }
    return fail ? -(10 + fail) : 0;
}

/* ---------------------------------------------------------------- Part R: REF mode (Sec. 3.4, Eq. 3)
 *
 * Activation-aware refinement of the two block coefficients.  The bases b1, b2 of every macro-block
 * are those of the canonical arrays (they are built without looking at activations); only c1, c2 are
 * re-solved.  For output channel o and macro-block g, with the M calibration rows
 * X_q = x[:, 128 g .. 128 g + 127] (M x 128):
 *     Y = X_q w                         the slab's output for the original weights
 *     A = [X_q b1, X_q b2]              (M x 2) the responses of the two bases
 *     c* = (A^T A + lambda I)^-1 A^T Y  ridge regression (the paper uses lambda = 1e-4)
 * w: float32 holding fp16-representable values [out][in]; x: fp16 bit patterns [tokens][in].
 * craw (optional): the unrounded solution [out][in/128][2]; c1, c2: rounded to fp16. */
int goq_oracle_ref_coefficients(int bw, int64_t tokens, int64_t out, int64_t in, const float *w,
                                const uint8_t *codes, const uint8_t *pattern, const uint8_t *signs,
                                const uint16_t *x, double lambda, double *craw,
                                uint16_t *c1, uint16_t *c2, int threads)
{
    if ((bw != 3 && bw != 4) || tokens <= 0 || out <= 0 || in <= 0 || in % GOQ_N || lambda < 0.0) return -1;
    int64_t gn = in / GOQ_N;
    int fail = 0;
#pragma omp parallel for num_threads(threads > 0 ? threads : 1) schedule(static)
    for (int64_t o = 0; o < out; ++o) {
        double *b1 = (double *)malloc(sizeof(double) * in * 2);
        if (!b1) { fail = 1; continue; }
        double *b2 = b1 + in;
        row_bases(bw, in, codes + o * in, pattern + o * in / GOQ_G, signs + o * in / GOQ_G, b1, b2);
        for (int64_t g = 0; g < gn; ++g) {
            double g11 = 0.0, g12 = 0.0, g22 = 0.0, r1 = 0.0, r2 = 0.0;      /* A^T A and A^T Y */
            for (int64_t t = 0; t < tokens; ++t) {
                double y = 0.0, a1 = 0.0, a2 = 0.0;
                for (int64_t k = g * GOQ_N; k < (g + 1) * GOQ_N; ++k) {
                    double xv = goq_oracle_half_to_double(x[t * in + k]);
                    y += xv * (double)w[o * in + k];
                    a1 += xv * b1[k];
                    a2 += xv * b2[k];
                }
                g11 += a1 * a1; g12 += a1 * a2; g22 += a2 * a2;
                r1 += a1 * y;   r2 += a2 * y;
            }
            g11 += lambda;
            g22 += lambda;
            double det = g11 * g22 - g12 * g12;
            double s1 = 0.0, s2 = 0.0;
            if (det != 0.0) {                       /* det = 0 only with lambda = 0 and dependent columns */
                s1 = (g22 * r1 - g12 * r2) / det;
                s2 = (g11 * r2 - g12 * r1) / det;
            }
            if (craw) { craw[(o * gn + g) * 2] = s1; craw[(o * gn + g) * 2 + 1] = s2; }
            c1[o * gn + g] = goq_oracle_double_to_half(s1);
            c2[o * gn + g] = goq_oracle_double_to_half(s2);
        }
        free(b1);
    }
    return fail ? -2 : 0;
}

int goq_oracle_max_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
