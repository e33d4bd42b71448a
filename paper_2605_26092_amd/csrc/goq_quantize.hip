// goq_quantize: the data-free GEO-mode quantizer on the device (Sec. 3.2 - 3.4): fp16 weights of a
// layer [out][in] -> canonical arrays (codes, pattern, signs, c1, c2).
//
// One WAVEFRONT per macro-block of 128 weights: lane l owns the weights k = 2l and 2l + 1, a
// micro-block of 8 weights is a group of 4 consecutive lanes, and pair p of every exchange pattern
// of a micro-block belongs to lane p of its group.  The arithmetic is laid out around what is
// exact:
//
//   fixed point  An fp16 weight is an integer W (up to 41 bits) times 2^-24; a lattice state is a
//                signed power of two B times 2^-(E-1), E = 2^(bw-1).  So <w, b1>, ||b1||^2,
//                <w, b2> and ||b2||^2 (Eq. 1, Eq. 2) are INTEGER sums -- 64-bit adds across the
//                wavefront, no rounding and therefore no summation order -- and s_norm = ||w||_inf
//                is an integer maximum of the fp16 magnitude bits.
//   nearest      Q(v), v = w / s_norm (Sec. 3.2), is decided without the division: |v| lies above
//                the midpoint 0.75 * 2^-e of the states 2^-e and 2^-(e+1) exactly when
//                W * 2^(e+2) > 3 S (S the integer of s_norm), and above the midpoint to zero,
//                2^-(emin+1), when W * 2^(emin+1) > S: integer comparisons, an exact tie going to
//                the smaller magnitude.
//   fp64         Only what the method defines as real arithmetic: the projection coefficient
//                <w,b1> / ||b1||^2 (one correctly rounded division of two exact integers), the
//                residual r = w - c b1 (Eq. 1; c b1 is exact, one rounding), the cross terms
//                t = x_i r_j - x_j r_i (Sec. 3.3; both products exact, one rounding) and the four
//                term score A_s = |t_0| + |t_1| + |t_2| + |t_3|, added in pair order.  eta = sgn(t)
//                (+1 at zero), s* = argmax A_s (ties: smallest s).
//
// The results are a pure function of the weights: no sum depends on the launch shape.  They equal
// those of a sequential fp64 evaluation of the same formulas bit for bit as long as the integer
// sums fit the 53-bit significand, which they do for bw = 3 always and for bw = 4 unless
// |<w, b>| reaches 2^22 (more than 64 weights of the block at the fp16 maximum).
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "goq_layout.h"
#include "goq_internal.h"
#include "goq_f64.h"

namespace {

constexpr int QW = 4;                        // wavefronts (= macro-blocks in flight) per workgroup

// fp16 magnitude bits (sign removed) -> integer multiple of 2^-24
__device__ __forceinline__ uint64_t half_magnitude(uint32_t a)
{
    const uint32_t e = a >> 10, m = a & 0x3ffu;
    return e ? (uint64_t)(1024u + m) << (e - 1) : (uint64_t)m;
}

// fp16 bits -> fp64 (exact): sign, magnitude integer, scale 2^-24
__device__ __forceinline__ double half_value(uint32_t h)
{
    const double v = __builtin_ldexp((double)(int64_t)half_magnitude(h & 0x7fffu), -24);
    return (h & 0x8000u) ? -v : v;
}

template <typename T>
__device__ __forceinline__ T wave_sum(T v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// code of one weight: sign bit | exponent, (sign 0, e = E - 1) is zero (Sec. 3.2)
template <int BW>
__device__ __forceinline__ int nearest_state(uint32_t h, uint64_t S)
{
    constexpr int E = 1 << (BW - 1);
    const bool neg = (h & 0x8000u) != 0;
    const uint64_t W = half_magnitude(h & 0x7fffu);
    const int emin = neg ? E - 1 : E - 2;            // exponent of the smallest magnitude of this sign
    const uint64_t S3 = 3 * S;
    int e = -1;
#pragma unroll
    for (int k = E - 1; k >= 0; --k) {               // descending: the smallest qualifying k wins
        const bool above = (k < emin) ? ((W << (k + 2)) > S3) : ((W << (k + 1)) > S);
        if (k <= emin && above) e = k;
    }
    if (e < 0) return E - 1;                         // zero
    return (neg ? E : 0) | e;
}

// signed integer value of a code in units of 2^-(E-1)
template <int BW>
__device__ __forceinline__ int state_integer(int code)
{
    constexpr int E = 1 << (BW - 1);
    const int s = code >> (BW - 1), e = code & (E - 1);
    if (!s && e == E - 1) return 0;
    const int mag = 1 << (E - 1 - e);
    return s ? -mag : mag;
}

template <int BW>
__global__ __launch_bounds__(64 * QW) void quantize_kernel(const uint32_t *__restrict__ w, int64_t nblocks,
                                                           uint16_t *__restrict__ codes, uint8_t *__restrict__ pattern,
                                                           uint8_t *__restrict__ signs, uint16_t *__restrict__ c1,
                                                           uint16_t *__restrict__ c2)
{
    constexpr int E = 1 << (BW - 1);
    __shared__ double rs[QW][GOQ_N];                 // residual r
    __shared__ double xs[QW][GOQ_N];                 // primary basis b1 (real value)
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int grp = lane >> 2, p = lane & 3;         // micro-block of this lane, its pair index
    double *r = rs[wave], *x = xs[wave];

    for (int64_t mb = (int64_t)blockIdx.x * QW + wave; mb < nblocks; mb += (int64_t)gridDim.x * QW) {
        const uint32_t pair = w[mb * 64 + lane];
        const uint32_t h[2] = {pair & 0xffffu, pair >> 16};
        // macro-block normalisation: magnitude bits order like magnitudes
        uint32_t amax = max(h[0] & 0x7fffu, h[1] & 0x7fffu);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) amax = max(amax, (uint32_t)__shfl_xor((int)amax, o));
        if (amax == 0) {                             // all-zero block: nothing to represent
            codes[mb * 64 + lane] = (uint16_t)((E - 1) * 0x0101);
            if (p == 0) { pattern[mb * 16 + grp] = 0; signs[mb * 16 + grp] = 0; }
            if (lane == 0) { c1[mb] = 0; c2[mb] = 0; }
            continue;
        }
        const uint64_t S = half_magnitude(amax);

        // primary projection; <w, b1> and ||b1||^2 as integers (a weight and its state share the sign)
        int code[2], B[2];
        uint64_t s1 = 0;
        uint32_t n1 = 0;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            code[i] = nearest_state<BW>(h[i], S);
            B[i] = state_integer<BW>(code[i]);
            const uint32_t mag = (uint32_t)(B[i] < 0 ? -B[i] : B[i]);
            s1 += half_magnitude(h[i] & 0x7fffu) * mag;
            n1 += mag * mag;
        }
        codes[mb * 64 + lane] = (uint16_t)(code[0] | (code[1] << 8));
        const uint64_t S1 = wave_sum(s1);
        const uint32_t N1 = wave_sum(n1);            // > 0: the largest weight maps to +-1
        // projection coefficient <w,b1> / ||b1||^2 = (S1 / N1) 2^(E-1-24); residual (Eq. 1)
        const double proj = __builtin_ldexp((double)S1 / (double)N1, E - 1 - 24);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const double b = __builtin_ldexp((double)B[i], -(E - 1));
            x[2 * lane + i] = b;
            r[2 * lane + i] = half_value(h[i]) - proj * b;
        }
        __builtin_amdgcn_wave_barrier();             // LDS accesses of one wavefront execute in order

        // pair p of pattern s of this lane's micro-block: (i, i xor s), i the p-th lower index
        const double *xm = x + 8 * grp, *rm = r + 8 * grp;
        int best_s = 1;
        uint32_t best_signs = 0;
        double bestA = -1.0;
#pragma unroll
        for (int s = 1; s <= 4; ++s) {
            const int i = (s == 1) ? 2 * p : (s == 4) ? p : ((p & 1) | ((p >> 1) << 2));
            const int j = i ^ s;
            const double t = xm[i] * rm[j] - xm[j] * rm[i];
            const double at = fabs(t);
            // alignment score: the four terms in pair order
            double A = __shfl(at, 0, 4);
            A += __shfl(at, 1, 4);
            A += __shfl(at, 2, 4);
            A += __shfl(at, 3, 4);
            const uint64_t negs = __ballot(t < 0.0);                 // eta = -1 where t < 0
            const uint32_t sg = (uint32_t)(negs >> (4 * grp)) & 15u;
            if (A > bestA) { bestA = A; best_s = s; best_signs = sg; }   // ties: the smaller s stays
        }
        if (p == 0) {
            pattern[mb * 16 + grp] = (uint8_t)(best_s - 1);
            signs[mb * 16 + grp] = (uint8_t)best_signs;
        }

        // b2 by the Theorem 1 exchange: y_i = -eta x_j for the lower index of a pair, +eta x_i for
        // the upper one; <w, b2> and ||b2||^2 as integers
        int64_t s2 = 0;
        uint32_t n2 = 0;
#pragma unroll
        for (int ii = 0; ii < 2; ++ii) {
            const int i = 2 * p + ii, j = i ^ best_s;
            const int lower = i < j ? i : j;
            const int rank = (best_s == 1) ? (lower >> 1) : (best_s == 4) ? lower : ((lower & 1) | ((lower >> 2) << 1));
            const bool eta_neg = (best_signs >> rank) & 1u;
            const int Bj = (int)__builtin_ldexp(xm[j], E - 1);       // the partner's state as an integer
            const int Y = ((i < j) != eta_neg) ? -Bj : Bj;
            const int64_t Wi = (int64_t)half_magnitude(h[ii] & 0x7fffu);
            s2 += ((h[ii] & 0x8000u) ? -Wi : Wi) * Y;
            n2 += (uint32_t)(Y * Y);
        }
        const int64_t S2 = wave_sum(s2);
        const uint32_t N2 = wave_sum(n2);
        if (lane == 0) {
            // GEO coefficients, Eq. 2 (the normal equations are diagonal: <b1, b2> = 0)
            const double c1v = proj;
            const double c2v = N2 ? __builtin_ldexp((double)S2 / (double)N2, E - 1 - 24) : 0.0;
            c1[mb] = (uint16_t)double_to_half_bits(c1v);
            c2[mb] = (uint16_t)double_to_half_bits(c2v);
        }
        __builtin_amdgcn_wave_barrier();             // the next block overwrites x and r
    }
}

}  // namespace

int goq_launch_quantize(hipStream_t st, int bw, int64_t out, int64_t in, const uint16_t *w, uint8_t *codes,
                        uint8_t *pattern, uint8_t *signs, uint16_t *c1, uint16_t *c2)
{
    const int64_t nblocks = out * (in / GOQ_N);
    int64_t grid = (nblocks + QW - 1) / QW;
    if (grid > 256 * 16) grid = 256 * 16;            // 16 workgroups per CU, each wavefront walks its share
    if (bw == 3)
        hipLaunchKernelGGL(quantize_kernel<3>, dim3((unsigned)grid), dim3(64 * QW), 0, st, (const uint32_t *)w, nblocks,
                           (uint16_t *)codes, pattern, signs, c1, c2);
    else
        hipLaunchKernelGGL(quantize_kernel<4>, dim3((unsigned)grid), dim3(64 * QW), 0, st, (const uint32_t *)w, nblocks,
                           (uint16_t *)codes, pattern, signs, c1, c2);
    return goq_check_launch("goq_quantize");
}
