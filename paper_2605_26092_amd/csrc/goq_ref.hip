// goq_ref_coefficients: the REF-mode (activation-aware) block coefficients on the device
// (Sec. 3.4, Eq. 3).  The bases b1, b2 stay those of the canonical arrays; for every output channel
// o and macro-block g, with the M calibration rows X_q = X[:, 128 g .. 128 g + 127],
//     Y = X_q w,   A = [X_q b1, X_q b2],   c* = (A^T A + lambda I)^-1 A^T Y.
//
// A^T A and A^T Y are quadratic forms of the slab's Gram matrix S_g = X_q^T X_q (128 x 128), which
// all output channels share:
//     A^T A = [b1 b2]^T S_g [b1 b2],   A^T Y = [b1 b2]^T S_g w,
// so the tokens are reduced once per macro-block (kernel 1) instead of once per output channel, and
// kernel 2 needs, per (o, g), the two products S_g b1 and S_g b2 and five dot products.  Everything
// is fp64 with fixed summation orders (tokens ascending; columns, then rows ascending), so the
// result is a pure function of the inputs.  It differs from a token-by-token evaluation of Eq. 3
// only by fp64 rounding, far below the fp16 quantum of the stored coefficients.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "goq_layout.h"
#include "goq_internal.h"
#include "goq_f64.h"

namespace {

constexpr int RT = 256;                  // threads per workgroup (both kernels)
constexpr int TT = 16;                   // tokens per LDS tile of the Gram kernel
constexpr int OPT = 2;                   // output channels per thread of the solve kernel
constexpr int OB = 32 * OPT;             // output channels per workgroup of the solve kernel

// ---- kernel 1: S_g = X_q^T X_q, one workgroup per macro-block, thread (ti, tj) owns the 8 x 8
// block of rows 8 ti .., columns 8 tj ..
__global__ __launch_bounds__(RT) void gram_kernel(const uint16_t *__restrict__ X, int tokens, int64_t in,
                                                  double *__restrict__ S)
{
    __shared__ __attribute__((aligned(16))) uint16_t xt[TT][GOQ_N];
    const int g = blockIdx.x;
    const int tid = threadIdx.x;
    const int ti = tid >> 4, tj = tid & 15;
    double acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = 0.0;
    for (int t0 = 0; t0 < tokens; t0 += TT) {
        // 16 tokens x 128 halfs = 256 pieces of 16 bytes; rows past the end are zero
        const int r = tid >> 4, c = tid & 15;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (t0 + r < tokens) v = *reinterpret_cast<const uint4 *>(X + (int64_t)(t0 + r) * in + (int64_t)g * GOQ_N + c * 8);
        __syncthreads();                                       // the previous tile has been used
        *reinterpret_cast<uint4 *>(&xt[r][c * 8]) = v;
        __syncthreads();
        const int nt = min(TT, tokens - t0);
        for (int t = 0; t < nt; ++t) {
            const uint4 ra = *reinterpret_cast<const uint4 *>(&xt[t][8 * ti]);
            const uint4 rb = *reinterpret_cast<const uint4 *>(&xt[t][8 * tj]);
            const uint32_t wa[4] = {ra.x, ra.y, ra.z, ra.w}, wb[4] = {rb.x, rb.y, rb.z, rb.w};
            double a[8], b[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                a[k] = half_bits_to_double((wa[k >> 1] >> (16 * (k & 1))) & 0xffffu);
                b[k] = half_bits_to_double((wb[k >> 1] >> (16 * (k & 1))) & 0xffffu);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[i][j] = fma(a[i], b[j], acc[i][j]);
        }
    }
    double *Sg = S + (int64_t)g * GOQ_N * GOQ_N;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; j += 2)
            *reinterpret_cast<double2 *>(Sg + (8 * ti + i) * GOQ_N + 8 * tj + j) = make_double2(acc[i][j], acc[i][j + 1]);
}

// ---- kernel 2: per (g, block of OB output channels).  Thread (oo = tid % 32, ic = tid / 32) forms
// rows 16 ic .. 16 ic + 15 of u1 = S_g b1 and u2 = S_g b2 of the output channels oo, oo + 32, ..
// (S_g is symmetric, so column j of S_g is read as the contiguous row j, and one read serves all of
// a thread's channels), then its share of the five dot products; the eight shares of an output
// channel are added in order and the 2 x 2 system is solved.  b1, b2 and w are staged as fp16,
// which holds them exactly.
template <int BW>
__global__ __launch_bounds__(RT) void ref_solve_kernel(const uint16_t *__restrict__ w, const uint8_t *__restrict__ codes,
                                                       const uint8_t *__restrict__ pattern, const uint8_t *__restrict__ signs,
                                                       const double *__restrict__ S, int64_t out, int64_t in, double lambda,
                                                       double *__restrict__ craw, uint16_t *__restrict__ c1,
                                                       uint16_t *__restrict__ c2)
{
    __shared__ _Float16 vb1[OB][GOQ_N + 2], vb2[OB][GOQ_N + 2], vw[OB][GOQ_N + 2];
    __shared__ double red[8][OB][5];
    const int tid = threadIdx.x;
    const int g = blockIdx.x;
    const int64_t o0 = (int64_t)blockIdx.y * OB;
    const int64_t gn = in / GOQ_N;

    // stage b1, b2 (Theorem 1 exchange from pattern and pair signs) and w of the OB channels
    for (int it = tid; it < OB * 16; it += RT) {
        const int oo = it >> 4, m = it & 15;
        const int64_t o = min(o0 + oo, out - 1);               // channels past the end repeat the last one
        const int64_t k0 = o * in + (int64_t)g * GOQ_N + m * GOQ_G;
        const uint2 cw = *reinterpret_cast<const uint2 *>(codes + k0);
        const int s = pattern[k0 / GOQ_G] + 1;
        const int sg = signs[k0 / GOQ_G];
        float x[GOQ_G], y[GOQ_G];
#pragma unroll
        for (int i = 0; i < GOQ_G; ++i) x[i] = (float)code_value<BW>((int)(((i < 4 ? cw.x : cw.y) >> (8 * (i & 3))) & 0xffu));
        int p = 0;
#pragma unroll
        for (int i = 0; i < GOQ_G; ++i) {
            y[i] = 0.f;
        }
#pragma unroll
        for (int i = 0; i < GOQ_G; ++i) {
            const int j = i ^ s;
            if (i < j) {
                const float eta = ((sg >> p) & 1) ? -1.f : 1.f;
                y[i] = -eta * x[j];
                y[j] = eta * x[i];
                ++p;
            }
        }
#pragma unroll
        for (int i = 0; i < GOQ_G; ++i) { vb1[oo][m * GOQ_G + i] = (_Float16)x[i]; vb2[oo][m * GOQ_G + i] = (_Float16)y[i]; }
    }
    for (int it = tid; it < OB * GOQ_N; it += RT) {
        const int oo = it >> 7, k = it & 127;
        const int64_t o = min(o0 + oo, out - 1);
        vw[oo][k] = __builtin_bit_cast(_Float16, w[o * in + (int64_t)g * GOQ_N + k]);
    }
    __syncthreads();

    const int o32 = tid & 31, ic = tid >> 5;
    const double *Sg = S + (int64_t)g * GOQ_N * GOQ_N;
    double u1[OPT][16], u2[OPT][16];
#pragma unroll
    for (int c = 0; c < OPT; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) { u1[c][r] = 0.0; u2[c][r] = 0.0; }
    for (int j = 0; j < GOQ_N; ++j) {
        double bj1[OPT], bj2[OPT];
#pragma unroll
        for (int c = 0; c < OPT; ++c) { bj1[c] = (double)(float)vb1[o32 + 32 * c][j]; bj2[c] = (double)(float)vb2[o32 + 32 * c][j]; }
        const double *row = Sg + j * GOQ_N + 16 * ic;           // S[j][16 ic ..] = S[16 ic ..][j]
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
            const double2 sv = *reinterpret_cast<const double2 *>(row + r);
#pragma unroll
            for (int c = 0; c < OPT; ++c) {
                u1[c][r] = fma(sv.x, bj1[c], u1[c][r]);
                u1[c][r + 1] = fma(sv.y, bj1[c], u1[c][r + 1]);
                u2[c][r] = fma(sv.x, bj2[c], u2[c][r]);
                u2[c][r + 1] = fma(sv.y, bj2[c], u2[c][r + 1]);
            }
        }
    }
#pragma unroll
    for (int c = 0; c < OPT; ++c) {
        const int oo = o32 + 32 * c;
        double g11 = 0.0, g12 = 0.0, g22 = 0.0, r1 = 0.0, r2 = 0.0;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int i = 16 * ic + r;
            const double b1i = (double)(float)vb1[oo][i], b2i = (double)(float)vb2[oo][i], wi = (double)(float)vw[oo][i];
            g11 = fma(b1i, u1[c][r], g11);
            g12 = fma(b2i, u1[c][r], g12);
            g22 = fma(b2i, u2[c][r], g22);
            r1 = fma(wi, u1[c][r], r1);
            r2 = fma(wi, u2[c][r], r2);
        }
        red[ic][oo][0] = g11; red[ic][oo][1] = g12; red[ic][oo][2] = g22; red[ic][oo][3] = r1; red[ic][oo][4] = r2;
    }
    __syncthreads();
    for (int oo = tid; oo < OB; oo += RT) {
        if (o0 + oo >= out) continue;
        double q[5] = {0.0, 0.0, 0.0, 0.0, 0.0};
        for (int c = 0; c < 8; ++c)
#pragma unroll
            for (int k = 0; k < 5; ++k) q[k] += red[c][oo][k];
        const double a11 = q[0] + lambda, a22 = q[2] + lambda, a12 = q[1];
        const double det = a11 * a22 - a12 * a12;
        double s1 = 0.0, s2 = 0.0;
        if (det != 0.0) {                                       // det = 0 only without a ridge, dependent columns
            s1 = (a22 * q[3] - a12 * q[4]) / det;
            s2 = (a11 * q[4] - a12 * q[3]) / det;
        }
        const int64_t idx = (o0 + oo) * gn + g;
        if (craw) { craw[2 * idx] = s1; craw[2 * idx + 1] = s2; }
        c1[idx] = (uint16_t)double_to_half_bits(s1);
        c2[idx] = (uint16_t)double_to_half_bits(s2);
    }
}

}  // namespace

int goq_launch_ref(hipStream_t st, int bw, int64_t tokens, int64_t out, int64_t in, const uint16_t *w,
                   const uint8_t *codes, const uint8_t *pattern, const uint8_t *signs, const uint16_t *X,
                   double lambda, void *workspace, double *craw, uint16_t *c1, uint16_t *c2)
{
    const int64_t gn = in / GOQ_N;
    const int64_t ob = (out + OB - 1) / OB;
    if (gn > 0x7fffffff || ob > 65535 || tokens > 0x7fffffff)
        return goq_set_error(GOQ_ESHAPE, "goq_ref_coefficients: layer too large for one launch");
    double *S = reinterpret_cast<double *>(workspace);
    hipLaunchKernelGGL(gram_kernel, dim3((unsigned)gn), dim3(RT), 0, st, X, (int)tokens, in, S);
    int rc = goq_check_launch("goq_ref_coefficients");
    if (rc) return rc;
    if (bw == 3)
        hipLaunchKernelGGL(ref_solve_kernel<3>, dim3((unsigned)gn, (unsigned)ob), dim3(RT), 0, st, w, codes, pattern, signs,
                           S, out, in, lambda, craw, c1, c2);
    else
        hipLaunchKernelGGL(ref_solve_kernel<4>, dim3((unsigned)gn, (unsigned)ob), dim3(RT), 0, st, w, codes, pattern, signs,
                           S, out, in, lambda, craw, c1, c2);
    return goq_check_launch("goq_ref_coefficients");
}
