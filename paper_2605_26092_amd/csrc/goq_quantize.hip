// goq_quantize: the data-free GEO-mode quantizer on the device (Sec. 3.2 - 3.4): fp16 weights of a
// layer [out][in] -> canonical arrays (codes, pattern, signs, c1, c2).
//
// One LANE per micro-block of 8 weights, one ROW of 16 lanes per macro-block of 128 weights, four
// macro-blocks per wavefront.  Everything that belongs to a micro-block -- nearest states, the 16
// cross terms of the four exchange patterns, scores, argmax, pair signs, the exchange itself -- is
// lane-local and lives in registers; what belongs to the macro-block -- the norm s_norm and the
// four sums of Eq. 1 and Eq. 2 -- is reduced across the 16 lanes of a row with data-parallel-
// primitive (DPP) moves, which stay inside a row by construction.  No LDS, no barriers.  The
// arithmetic is laid out around what is exact:
//
//   products    A lattice state is a signed power of two, so every product with a state (w b1,
//               w b2, c b1, x r) is exact in fp64.
//   sums        <w, b1> and <w, b2> (Eq. 1, Eq. 2) are sums of multiples of 2^-31 below 2^23: every
//               partial sum is exactly representable in fp64 whatever the order (always for
//               bw = 3; for bw = 4 unless |<w, b>| reaches 2^22, i.e. more than 64 weights of the
//               block at the fp16 maximum), so the reduction tree is free.  ||b1||^2 and ||b2||^2
//               are small integers (units of 4^-(E-1)).
//   nearest     Q(v), v = w / s_norm (Sec. 3.2), is decided without the division: |v| lies above
//               the midpoint 0.75 * 2^-k of the states 2^-k and 2^-(k+1) exactly when
//               |w| > 0.75 * 2^-k * s_norm, and above the midpoint to zero, 2^-(emin+1), when
//               |w| > 2^-(emin+1) * s_norm.  The thresholds fall with k, so the exponent of the
//               nearest state is the NUMBER of thresholds |w| does not exceed, and that number is
//               a difference of fp64 exponent fields (see the loop); an exact tie goes to the
//               smaller magnitude.
//   roundings   Only what the method defines as real arithmetic rounds: the projection
//               coefficient <w,b1> / ||b1||^2 (one correctly rounded division of two exact
//               numbers), the residual r = w - c b1 (Eq. 1; one rounding), the cross terms
//               t = x_i r_j - x_j r_i (Sec. 3.3; one rounding) and the four-term score
//               A_s = |t_0| + |t_1| + |t_2| + |t_3|, added in pair order.  eta = sgn(t)
//               (+1 at zero), s* = argmax A_s (ties: smallest s).
//
// The results are a pure function of the weights and equal those of a sequential fp64 evaluation
// of the same formulas bit for bit under the condition on the sums stated above.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "goq_layout.h"
#include "goq_internal.h"
#include "goq_f64.h"

namespace {

constexpr int QW = 4;                        // wavefronts per workgroup
constexpr int ROWS = 4;                      // macro-blocks (rows of 16 lanes) per wavefront

// ---- DPP moves inside a row of 16 lanes -------------------------------------------------------
// quad_perm [a, b, c, d]: lane 4 m + i reads lane 4 m + (a, b, c, d)[i]
constexpr int QUAD_SWAP1 = 1 | (0 << 2) | (3 << 4) | (2 << 6);      // i xor 1
constexpr int QUAD_SWAP2 = 2 | (3 << 2) | (0 << 4) | (1 << 6);      // i xor 2
constexpr int ROW_HALF_MIRROR = 0x141;                              // i -> 7 - i within 8 lanes
constexpr int ROW_MIRROR = 0x140;                                   // i -> 15 - i within 16 lanes

template <int CTRL>
__device__ __forceinline__ uint32_t dpp32(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, false);
}
template <int CTRL>
__device__ __forceinline__ double dpp_double(double v)
{
    const uint64_t u = __builtin_bit_cast(uint64_t, v);
    const uint64_t m = ((uint64_t)dpp32<CTRL>((uint32_t)(u >> 32)) << 32) | dpp32<CTRL>((uint32_t)u);
    return __builtin_bit_cast(double, m);
}
// After the four steps every lane of a row holds the row's result: the partners are i xor 1,
// i xor 2 (a quad holds one value), 7 - i (a group of eight does), 15 - i.
__device__ __forceinline__ double row_sum(double v)
{
    v += dpp_double<QUAD_SWAP1>(v);
    v += dpp_double<QUAD_SWAP2>(v);
    v += dpp_double<ROW_HALF_MIRROR>(v);
    v += dpp_double<ROW_MIRROR>(v);
    return v;
}
__device__ __forceinline__ uint32_t row_sum(uint32_t v)
{
    v += dpp32<QUAD_SWAP1>(v);
    v += dpp32<QUAD_SWAP2>(v);
    v += dpp32<ROW_HALF_MIRROR>(v);
    v += dpp32<ROW_MIRROR>(v);
    return v;
}
__device__ __forceinline__ uint32_t row_max(uint32_t v)
{
    v = max(v, dpp32<QUAD_SWAP1>(v));
    v = max(v, dpp32<QUAD_SWAP2>(v));
    v = max(v, dpp32<ROW_HALF_MIRROR>(v));
    v = max(v, dpp32<ROW_MIRROR>(v));
    return v;
}

// 2^-e as fp64, e >= 0 small
__device__ __forceinline__ double pow2_neg(int e) { return __longlong_as_double((long long)(1023 - e) << 52); }

template <int BW>
__global__ __launch_bounds__(64 * QW) void quantize_kernel(const uint4 *__restrict__ w, int64_t nblocks,
                                                           uint2 *__restrict__ codes, uint8_t *__restrict__ pattern,
                                                           uint8_t *__restrict__ signs, uint16_t *__restrict__ c1,
                                                           uint16_t *__restrict__ c2)
{
    constexpr int E = 1 << (BW - 1);
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int row = lane >> 4, m = lane & 15;        // macro-block of the wavefront, micro-block of the macro-block
    const int64_t groups = (nblocks + ROWS - 1) / ROWS;

    for (int64_t grp = (int64_t)blockIdx.x * QW + wave; grp < groups; grp += (int64_t)gridDim.x * QW) {
        const int64_t mb_raw = grp * ROWS + row;
        const bool valid = mb_raw < nblocks;         // rows past the end repeat the last macro-block, store nothing
        const int64_t mb = valid ? mb_raw : nblocks - 1;
        const uint4 q = w[mb * 16 + m];
        const uint32_t pk[4] = {q.x, q.y, q.z, q.w};
        uint32_t h[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) { h[2 * i] = pk[i] & 0xffffu; h[2 * i + 1] = pk[i] >> 16; }

        // macro-block normalisation s_norm = ||w||_inf: magnitude bits order like magnitudes
        uint32_t amax = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) amax = max(amax, h[i] & 0x7fffu);
        amax = row_max(amax);
        const bool zero_block = amax == 0;           // nothing to represent: zero codes, c1 = c2 = 0
        const double sn = half_bits_to_double(amax);

        // nearest states.  Thresholds common to both signs: 0.75 2^-k s_norm, k = 0 .. E-3; then a
        // negative weight has the state 2^-(E-1) (midpoints 0.75 2^-(E-2) s_norm and, to zero,
        // 2^-E s_norm), a positive one ends at 2^-(E-2) (midpoint to zero 2^-(E-1) s_norm).
        const int T075 = __double2hiint(0.75 * sn), Tsn = __double2hiint(sn);
        double wv[8], x[8];
        uint32_t code_lo = 0, code_hi = 0, n1 = 0;
        double s1 = 0.0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            wv[i] = half_bits_to_double(h[i]);
            const double wa = fabs(wv[i]);
            const uint32_t neg = h[i] >> 15;                         // 1 for a negative weight
            // Number of thresholds |w| does not exceed.  |w| (11 significant bits) and 0.75 s_norm
            // (13) are positive fp64 numbers whose low words are zero, so they order like their high
            // words, and a factor 2^k is k units of the exponent field (bit 20 of the high word):
            // |w| 2^k <= 0.75 s_norm  <=>  A + (k << 20) <= T.  That holds for k = 0 .. (T - A) >> 20
            // when T >= A and for no k otherwise; a negative weight has E - 1 such thresholds, a
            // positive one E - 2, and the midpoint to zero is one more comparison.
            const int A = __double2hiint(wa);
            const int nth = min(max(((T075 - A) >> 20) + 1, 0), E - 2 + (int)neg);
            const int e = nth + ((A <= Tsn - ((E - 1 + (int)neg) << 20)) ? 1 : 0);
            const bool is_zero = zero_block || e == E - 1 + (int)neg;
            const uint32_t code = is_zero ? (uint32_t)(E - 1) : ((neg << (BW - 1)) | (uint32_t)e);
            if (i < 4) code_lo |= code << (8 * i);
            else code_hi |= code << (8 * (i - 4));
            // b1_i = (-1)^neg 2^-e assembled from sign and exponent field (low word zero)
            const uint32_t xhi = is_zero ? 0u : (((uint32_t)(1023 - e) << 20) | (neg << 31));
            x[i] = __hiloint2double((int)xhi, 0);
            s1 += wa * fabs(x[i]);                                  // a weight and its state share the sign
            n1 += is_zero ? 0u : (1u << (2 * (E - 1 - e)));         // |b1_i|^2 in units of 4^-(E-1)
        }
        if (valid) codes[mb * 16 + m] = make_uint2(code_lo, code_hi);
        const double S1 = row_sum(s1);
        const uint32_t N1 = row_sum(n1);             // > 0 unless the block is zero: the largest weight maps to +-1
        // projection coefficient <w,b1> / ||b1||^2 and the residual r = w - c b1 (Eq. 1)
        const double proj = zero_block ? 0.0 : S1 / ((double)N1 * pow2_neg(2 * (E - 1)));
        double r[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) r[i] = wv[i] - proj * x[i];

        // Sec. 3.3: the four patterns s, pairs (i, i xor s) in ascending lower index; cross term,
        // score in pair order, sign bits (eta = -1 where t < 0).  The pair's share of <w, b2> under
        // the Theorem 1 exchange (b2_i = -eta x_j for the lower index, b2_j = +eta x_i for the upper
        // one) is eta (w_j x_i - w_i x_j): exact, and summed for every pattern alongside its score,
        // so that choosing the pattern chooses the sum.
        int best_s = 1;
        uint32_t best_signs = 0;
        double bestA = -1.0, best_d = 0.0;
#pragma unroll
        for (int s = 1; s <= 4; ++s) {
            double A = 0.0, d = 0.0;
            uint32_t sg = 0;
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const int i = (s == 1) ? 2 * p : (s == 4) ? p : ((p & 1) | ((p >> 1) << 2));
                const int j = i ^ s;
                const double t = x[i] * r[j] - x[j] * r[i];
                const double u = wv[j] * x[i] - wv[i] * x[j];
                const bool eta_neg = t < 0.0;
                A = (p == 0) ? fabs(t) : A + fabs(t);
                sg |= (eta_neg ? 1u : 0u) << p;
                d += eta_neg ? -u : u;
            }
            const bool better = A > bestA;                           // ties: the smaller s stays
            bestA = better ? A : bestA;
            best_s = better ? s : best_s;
            best_signs = better ? sg : best_signs;
            best_d = better ? d : best_d;
        }
        if (zero_block) { best_s = 1; best_signs = 0; }
        if (valid) {
            pattern[mb * 16 + m] = (uint8_t)(best_s - 1);
            signs[mb * 16 + m] = (uint8_t)best_signs;
        }
        // <w, b2> of the macro-block; ||b2||^2 = ||b1||^2 (b2 is a signed permutation of b1)
        const double S2 = row_sum(best_d);
        const uint32_t N2 = N1;
        if (valid && m == 0) {
            // GEO coefficients, Eq. 2 (the normal equations are diagonal: <b1, b2> = 0)
            const double c2v = N2 ? S2 / ((double)N2 * pow2_neg(2 * (E - 1))) : 0.0;
            c1[mb] = (uint16_t)double_to_half_bits(proj);
            c2[mb] = (uint16_t)double_to_half_bits(c2v);
        }
    }
}

}  // namespace

int goq_launch_quantize(hipStream_t st, int bw, int64_t out, int64_t in, const uint16_t *w, uint8_t *codes,
                        uint8_t *pattern, uint8_t *signs, uint16_t *c1, uint16_t *c2)
{
    const int64_t nblocks = out * (in / GOQ_N);
    int64_t grid = (nblocks + QW * ROWS - 1) / (QW * ROWS);
    if (grid > 256 * 32) grid = 256 * 32;            // every wavefront walks its share of the row groups
    if (bw == 3)
        hipLaunchKernelGGL(quantize_kernel<3>, dim3((unsigned)grid), dim3(64 * QW), 0, st, (const uint4 *)w, nblocks,
                           (uint2 *)codes, pattern, signs, c1, c2);
    else
        hipLaunchKernelGGL(quantize_kernel<4>, dim3((unsigned)grid), dim3(64 * QW), 0, st, (const uint4 *)w, nblocks,
                           (uint2 *)codes, pattern, signs, c1, c2);
    return goq_check_launch("goq_quantize");
}
