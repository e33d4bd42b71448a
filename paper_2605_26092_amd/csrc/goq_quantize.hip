// goq_quantize: the data-free GEO-mode quantizer on the device (Sec. 3.2 - 3.4): fp16 weights of a
// layer [out][in] -> canonical arrays (codes, pattern, signs, c1, c2), one macro-block of 128
// weights along `in` at a time.
//
// Steps per macro-block, in the paper's order: s_norm = ||w||_inf and v = w / s_norm (Sec. 3.2);
// b1 = nearest lattice state of v, linear distance, exact ties toward the smaller magnitude
// (decided by comparing |w| with the midpoints scaled by s_norm, see nearest_code);
// r = w - (<w, b1> / ||b1||^2) b1 (Eq. 1); per 8-weight micro-block the cross terms
// t = x_i r_j - x_j r_i of the pairs (i, j = i xor s) of the four patterns, A_s = sum |t|,
// s* = argmax (ties: smallest s), eta = sgn(t) (+1 at zero) (Sec. 3.3); b2 by the Theorem 1
// exchange; c1 = <w, b1> / ||b1||^2, c2 = <w, b2> / ||b2||^2 (Eq. 2), rounded to fp16.
//
// Arithmetic is fp64 and every sum runs over k in ascending order, so the result is a pure
// function of the weights (one rounding sequence): the stored codes, metadata and coefficient
// bits do not depend on the launch shape.  Every product has a power-of-two (or zero) factor and is
// therefore exact, so fused multiply-adds round exactly like separate operations.
//
// Work split: one THREAD per macro-block (the sums are sequential by definition); a 64-thread
// workgroup takes 64 consecutive macro-blocks = 16 KiB of contiguous weights, moved through LDS so
// that global loads and stores are coalesced (row stride 65 dwords: a lane's walk along its own
// macro-block hits its own bank).
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "goq_layout.h"
#include "goq_internal.h"
#include "goq_f64.h"

namespace {

constexpr int QT = 64;                       // macro-blocks (= threads) per workgroup
constexpr int WSTRIDE = 65;                  // dwords per macro-block row of the weight tile (64 + 1 pad)
constexpr int CSTRIDE = 33;                  // dwords per macro-block row of the code tile (32 + 1 pad)

// Nearest lattice state of v = w / s_norm in linear distance, an exact tie going to the state of
// smaller magnitude -- decided without the division.  Between neighbouring magnitudes 2^-e and
// 2^-(e+1) the midpoint is 0.75 * 2^-e; below the smallest magnitude m of a sign lies zero, with
// midpoint m / 2.  |v| > mid is the same as |w| > mid * s_norm, and mid * s_norm is exact (a two-bit
// number times an fp16 value).  The quotient's rounding cannot change a decision: |w| and
// mid * s_norm are multiples of 2^-33 below 2^16, so unless they are equal they differ by more than
// 2^-49 relative, a hundred times the quotient's rounding error, and v == mid exactly when they are
// equal.  (Zero is nearer to a value than any state of the opposite sign.)
template <int BW>
__device__ __forceinline__ int nearest_code(double w, double snorm)
{
    constexpr int E = 1 << (BW - 1);
    const bool neg = w < 0.0;
    const double a = fabs(w);
    const int emin = neg ? E - 1 : E - 2;          // exponent of the smallest magnitude of this sign
    int e = emin + 1;                              // emin + 1 stands for zero
    // largest magnitude whose lower midpoint a exceeds
    double mid = 0.75 * snorm;                     // between 2^0 and 2^-1
    int found = 0;
#pragma unroll
    for (int k = 0; k < E; ++k) {
        if (k < emin) {
            if (!found && a > mid) { e = k; found = 1; }
            mid *= 0.5;
        } else if (k == emin) {
            // below the smallest magnitude 2^-emin lies zero: midpoint 2^-(emin+1)
            const double mz = __longlong_as_double((long long)(1023 - emin - 1) << 52) * snorm;
            if (!found && a > mz) { e = k; found = 1; }
        }
    }
    if (e == emin + 1) return E - 1;               // the zero state (sign 0, e = E - 1)
    return (neg ? E : 0) | e;
}

template <int BW>
__global__ __launch_bounds__(QT) void quantize_kernel(const uint32_t *__restrict__ w, int64_t nblocks,
                                                      uint32_t *__restrict__ codes, uint32_t *__restrict__ pattern,
                                                      uint32_t *__restrict__ signs, uint16_t *__restrict__ c1,
                                                      uint16_t *__restrict__ c2)
{
    __shared__ uint32_t wt[QT * WSTRIDE];      // weights, two fp16 per dword
    __shared__ uint32_t ct[QT * CSTRIDE];      // codes, four per dword
    __shared__ uint32_t pt[QT * 5], st[QT * 5];  // pattern / sign bytes, 16 per macro-block (4 dwords + pad)

    const int t = threadIdx.x;
    const int64_t mb0 = (int64_t)blockIdx.x * QT;
    const int nb = (int)min((int64_t)QT, nblocks - mb0);

    // coalesced load of nb macro-blocks (64 dwords each)
    for (int i = t; i < nb * 64; i += QT) wt[(i >> 6) * WSTRIDE + (i & 63)] = w[mb0 * 64 + i];
    __syncthreads();

    if (t < nb) {
        const uint32_t *wr = wt + t * WSTRIDE;
        uint32_t *cr = ct + t * CSTRIDE;
        auto W = [&](int k) { return half_bits_to_double((wr[k >> 1] >> (16 * (k & 1))) & 0xffffu); };
        auto CODE = [&](int k) { return (int)((cr[k >> 2] >> (8 * (k & 3))) & 0xffu); };

        // macro-block normalisation s_norm = ||w||_inf
        double snorm = 0.0;
        for (int k = 0; k < GOQ_N; ++k) { const double a = fabs(W(k)); if (a > snorm) snorm = a; }
        double c1v = 0.0, c2v = 0.0;
        if (snorm == 0.0) {                                     // all-zero block: nothing to represent
            const uint32_t z = (uint32_t)goq_zero_code(BW) * 0x01010101u;
            for (int k = 0; k < 32; ++k) cr[k] = z;
            for (int m = 0; m < 4; ++m) { pt[t * 5 + m] = 0; st[t * 5 + m] = 0; }
        } else {
            // primary projection b1 = Q(v), <w, b1>, ||b1||^2
            double wb1 = 0.0, n1 = 0.0;
            for (int k4 = 0; k4 < 32; ++k4) {
                uint32_t pack = 0;
                for (int kk = 0; kk < 4; ++kk) {
                    const int k = 4 * k4 + kk;
                    const double wk = W(k);
                    const int c = nearest_code<BW>(wk, snorm);
                    pack |= (uint32_t)c << (8 * kk);
                    const double b = code_value<BW>(c);
                    wb1 += wk * b;
                    n1 += b * b;
                }
                cr[k4] = pack;
            }
            // orthogonal residual r = w - (<w,b1>/||b1||^2) b1 (Eq. 1), evaluated where it is used
            const double proj = wb1 / n1;
            auto R = [&](int k) { return (n1 > 0.0) ? W(k) - proj * code_value<BW>(CODE(k)) : W(k); };
            double wb2 = 0.0, n2 = 0.0;
            for (int m4 = 0; m4 < 4; ++m4) {
                uint32_t ppack = 0, spack = 0;
                for (int mm = 0; mm < 4; ++mm) {
                    const int m = 4 * m4 + mm;
                    double x[GOQ_G], r[GOQ_G];
#pragma unroll
                    for (int i = 0; i < GOQ_G; ++i) { x[i] = code_value<BW>(CODE(GOQ_G * m + i)); r[i] = R(GOQ_G * m + i); }
                    // analytical signs, alignment score A_s, pattern argmax
                    int best_s = 1, best_signs = 0;
                    double bestA = -1.0;
#pragma unroll
                    for (int s = 1; s <= 4; ++s) {
                        double A = 0.0;
                        int sg = 0, p = 0;
#pragma unroll
                        for (int i = 0; i < GOQ_G; ++i) {
                            const int j = i ^ s;
                            if (i < j) {
                                const double tt = x[i] * r[j] - x[j] * r[i];
                                A += fabs(tt);
                                if (tt < 0.0) sg |= 1 << p;              // eta = sgn(t); +1 when t == 0
                                ++p;
                            }
                        }
                        if (A > bestA) { bestA = A; best_s = s; best_signs = sg; }   // ties: smallest s
                    }
                    ppack |= (uint32_t)(best_s - 1) << (8 * mm);
                    spack |= (uint32_t)best_signs << (8 * mm);
                    // b2 by the Theorem 1 exchange, then its share of <w, b2> and ||b2||^2 in k order
                    double y[GOQ_G];
                    int p = 0;
#pragma unroll
                    for (int i = 0; i < GOQ_G; ++i) {
                        const int j = i ^ best_s;
                        if (i < j) {
                            const double eta = ((best_signs >> p) & 1) ? -1.0 : 1.0;
                            y[i] = -eta * x[j];
                            y[j] = eta * x[i];
                            ++p;
                        }
                    }
#pragma unroll
                    for (int i = 0; i < GOQ_G; ++i) { wb2 += W(GOQ_G * m + i) * y[i]; n2 += y[i] * y[i]; }
                }
                pt[t * 5 + m4] = ppack;
                st[t * 5 + m4] = spack;
            }
            // GEO coefficients, Eq. 2 (diagonal normal equations)
            c1v = (n1 > 0.0) ? wb1 / n1 : 0.0;
            c2v = (n2 > 0.0) ? wb2 / n2 : 0.0;
        }
        c1[mb0 + t] = (uint16_t)double_to_half_bits(c1v);
        c2[mb0 + t] = (uint16_t)double_to_half_bits(c2v);
    }
    __syncthreads();
    // coalesced stores: 32 code dwords and 4 + 4 metadata dwords per macro-block
    for (int i = t; i < nb * 32; i += QT) codes[mb0 * 32 + i] = ct[(i >> 5) * CSTRIDE + (i & 31)];
    for (int i = t; i < nb * 4; i += QT) {
        pattern[mb0 * 4 + i] = pt[(i >> 2) * 5 + (i & 3)];
        signs[mb0 * 4 + i] = st[(i >> 2) * 5 + (i & 3)];
    }
}

}  // namespace

int goq_launch_quantize(hipStream_t st, int bw, int64_t out, int64_t in, const uint16_t *w, uint8_t *codes,
                        uint8_t *pattern, uint8_t *signs, uint16_t *c1, uint16_t *c2)
{
    const int64_t nblocks = out * (in / GOQ_N);
    const int64_t grid = (nblocks + QT - 1) / QT;
    if (grid > 0x7fffffff) return goq_set_error(GOQ_ESHAPE, "goq_quantize: layer too large for one launch");
    if (bw == 3)
        hipLaunchKernelGGL(quantize_kernel<3>, dim3((unsigned)grid), dim3(QT), 0, st, (const uint32_t *)w, nblocks,
                           (uint32_t *)codes, (uint32_t *)pattern, (uint32_t *)signs, c1, c2);
    else
        hipLaunchKernelGGL(quantize_kernel<4>, dim3((unsigned)grid), dim3(QT), 0, st, (const uint32_t *)w, nblocks,
                           (uint32_t *)codes, (uint32_t *)pattern, (uint32_t *)signs, c1, c2);
    return goq_check_launch("goq_quantize");
}
