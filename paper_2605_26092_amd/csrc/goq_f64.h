// fp64 helpers shared by the calibration-time kernels (quantizer, REF coefficients): exact
// fp16 -> fp64 conversion, fp64 -> fp16 rounding and the value of a canonical lattice code.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// fp16 -> fp64 is exact; the two hardware conversions (fp16 -> fp32 -> fp64) keep subnormals
__device__ __forceinline__ double half_bits_to_double(uint32_t h)
{
    return (double)(float)__builtin_bit_cast(_Float16, (unsigned short)h);
}

// fp64 -> IEEE binary16 bits, round to nearest even, straight from the bit pattern (no
// intermediate fp32): the 53-bit significand is cut at the binary16 quantum of its binade (2^-24
// below 2^-14) and the cut-off part is compared with half a quantum.
__device__ __forceinline__ uint32_t double_to_half_bits(double d)
{
    const uint64_t u = (uint64_t)__double_as_longlong(d);
    const uint32_t sign = (uint32_t)(u >> 48) & 0x8000u;
    const int ex = (int)((u >> 52) & 0x7ff);
    const uint64_t frac = u & 0xfffffffffffffull;
    if (ex == 0x7ff) return sign | (frac ? 0x7e00u : 0x7c00u);
    if (ex == 0) return sign;                                   // fp64 subnormals are far below 2^-25
    const int e = ex - 1023;
    if (e > 15) return sign | 0x7c00u;
    const uint64_t sig = frac | (1ull << 52);                   // 1.f as a 53-bit integer, value sig 2^(e-52)
    int drop = 42;                                              // bits below the quantum 2^(e-10)
    if (e < -14) drop += -14 - e;                               // subnormal range: quantum 2^-24
    if (drop > 54) return sign;                                 // below a quarter quantum: zero
    const uint64_t q = sig >> drop;
    const uint64_t rem = sig & ((1ull << drop) - 1), halfq = 1ull << (drop - 1);
    const uint32_t up = (rem > halfq || (rem == halfq && (q & 1))) ? 1u : 0u;
    // normal: q in [1024, 2047] carries the implicit bit, which lands on the exponent field;
    // subnormal: q < 1024 is the fraction itself.  A carry out of the fraction bumps the exponent
    // by plain addition (2047 + 1 -> next binade, 1023 + 1 -> smallest normal, 31 << 10 -> infinity).
    const uint32_t base = (e < -14) ? 0u : (uint32_t)(e + 14) << 10;
    return sign | (base + (uint32_t)q + up);
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

