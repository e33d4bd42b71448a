// fp64 helpers shared by the calibration-time kernels (quantizer, REF coefficients): exact
// fp16 <-> fp64 conversion and the value of a canonical lattice code.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// fp16 -> fp64 is exact; the two hardware conversions (fp16 -> fp32 -> fp64) keep subnormals
__device__ __forceinline__ double half_bits_to_double(uint32_t h)
{
    return (double)(float)__builtin_bit_cast(_Float16, (unsigned short)h);
}

// round-to-nearest-even from fp64 straight to binary16 (no intermediate fp32)
__device__ __forceinline__ uint32_t double_to_half_bits(double d)
{
    const uint32_t sign = (__double_as_longlong(d) < 0) ? 0x8000u : 0u;
    const double a = fabs(d);
    if (d != d) return 0x7e00u;
    if (a >= 65520.0) return sign | 0x7c00u;                    // rounds to infinity
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);                                         // a = f 2^e, f in [0.5, 1)
    int ex = e - 1;
    if (ex < -14) ex = -14;                                     // subnormal range: fixed quantum 2^-24
    const double q = ldexp(a, 10 - ex);                         // in units of 2^(ex-10); exact
    int m = (int)rint(q);                                       // ties to even; in [0, 2048]
    int be = ex + 15;
    if (ex == -14 && m < 1024) return sign | (uint32_t)m;       // subnormal (or zero)
    if (m == 2048) { m = 1024; be += 1; }
    if (be >= 31) return sign | 0x7c00u;
    return sign | (uint32_t)(be << 10) | (uint32_t)(m & 0x3ff);
}

// value of one canonical code: (-1)^sign 2^-e, (sign 0, e = E - 1) is exact zero (Sec. 3.2)
template <int BW>
__device__ __forceinline__ double code_value(int code)
{
    constexpr int E = 1 << (BW - 1);
    const int sign = (code >> (BW - 1)) & 1;
    const int e = code & (E - 1);
    if (!sign && e == E - 1) return 0.0;
    // 2^-e assembled from its exponent field
    return __longlong_as_double(((long long)sign << 63) | ((long long)(1023 - e) << 52));
}

