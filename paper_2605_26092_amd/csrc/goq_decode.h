// Device helpers: primary-code decode (Sec. 3.2 lattice) with byte look-up permutes.
//
// A decoded micro-block is kept as eight BYTES in two registers, elements 0..3 in `lo` and
// 4..7 in `hi`:
//   A16: the byte is the HIGH byte of the fp16 power of two (sign, exponent, two zero mantissa
//        bits) -- the low byte of any fp16 power of two is zero, so widening byte -> fp16 is a
//        byte shuffle, no arithmetic.  The multiply x * 2^-e then runs as an fp16 dot product
//        whose weight operand has a zero mantissa: an exponent add.
//   A8 : the byte is the int8 value b * 2^(E-1) (a signed power of two): x * b is a shift.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef _Float16 goq_half2 __attribute__((ext_vector_type(2)));

// v_perm_b32: byte i of the result = byte sel[i] of the 8-byte value {hi, lo}; selector 0x0c = 0x00
__device__ __forceinline__ uint32_t goq_perm(uint32_t hi, uint32_t lo, uint32_t sel)
{
    return __builtin_amdgcn_perm(hi, lo, sel);
}

__device__ __forceinline__ float goq_dot2(uint32_t a, uint32_t b, float c)
{
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(goq_half2, a), __builtin_bit_cast(goq_half2, b), c, false);
}

__device__ __forceinline__ int goq_dot4(uint32_t a, uint32_t b, int c)
{
    return __builtin_amdgcn_sdot4((int)a, (int)b, c, false);
}

// bytes -> two fp16 with zero low bytes: (b0, b1) and (b2, b3)
__device__ __forceinline__ uint32_t goq_widen01(uint32_t bytes) { return goq_perm(0u, bytes, 0x010c000cu); }
__device__ __forceinline__ uint32_t goq_widen23(uint32_t bytes) { return goq_perm(0u, bytes, 0x030c020cu); }

template <int BW, int ACT>
struct GoqLut;

// bw = 3, codes 0..7 = +1 +.5 +.25 0 -1 -.5 -.25 -.125
template <>
struct GoqLut<3, 0> {   // fp16 high bytes
    static constexpr uint32_t lo = 0x0034383Cu, hi = 0xB0B4B8BCu;
};
template <>
struct GoqLut<3, 1> {   // int8 b * 8
    static constexpr uint32_t lo = 0x00020408u, hi = 0xFFFEFCF8u;
};

// Decode one packed code dword into element bytes.
template <int BW, int ACT>
__device__ __forceinline__ void goq_decode_bytes(uint32_t w, uint32_t &lo, uint32_t &hi)
{
    if constexpr (BW == 3) {
        const uint32_t clo = w & 0x07070707u;
        const uint32_t chi = (w >> 3) & 0x07070707u;
        lo = goq_perm(GoqLut<3, ACT>::hi, GoqLut<3, ACT>::lo, clo);
        hi = goq_perm(GoqLut<3, ACT>::hi, GoqLut<3, ACT>::lo, chi);
    } else {
        static_assert(ACT == 0, "bw = 4 with int8 activations: b * 128 does not fit int8");
        // nibble = sign << 3 | e ; fp16 high byte = sign << 7 | (15 - e) << 2 ; (0, 7) -> 0x00.
        // Both lattice halves are looked up by e; a third permute picks per byte by the sign bit
        // (selector byte i = i for the positive, 4 + i for the negative look-up).
        constexpr uint32_t PL = 0x3034383Cu, PH = 0x0024282Cu;   // +2^0 .. +2^-6, zero
        constexpr uint32_t NL = 0xB0B4B8BCu, NH = 0xA0A4A8ACu;   // -2^0 .. -2^-7
        {
            const uint32_t e = w & 0x07070707u;
            const uint32_t pick = ((w >> 1) & 0x04040404u) | 0x03020100u;
            lo = goq_perm(goq_perm(NH, NL, e), goq_perm(PH, PL, e), pick);
        }
        {
            const uint32_t e = (w >> 4) & 0x07070707u;
            const uint32_t pick = ((w >> 5) & 0x04040404u) | 0x03020100u;
            hi = goq_perm(goq_perm(NH, NL, e), goq_perm(PH, PL, e), pick);
        }
    }
}

// Exchange table entry of variant v = pattern | signs << 2 (Theorem 1) for decoded BYTES:
//   x, y : v_perm selectors, byte i of b2 = byte (i xor s) of b1 (s = pattern + 1)
//   z, w : FLIP in the bytes whose sign flips: b2_i = -eta b1_j for the lower index of a pair,
//          +eta b1_i for the upper one.  FLIP = 0x80 flips the sign bit of a float byte (fp16 high
//          byte, E5M2); 0xFF marks the byte for a two's complement negation (int8).
// Sign bit p of the descriptor belongs to the p-th pair in ascending lower index (the printed order
// of the pair sets P_s).
template <uint32_t FLIP>
__device__ __forceinline__ uint4 goq_exchange_entry(int v)
{
    const int s = (v & 3) + 1;
    const int sg = v >> 2;
    uint32_t mlo = 0, mhi = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int j = i ^ s;
        const int l = i < j ? i : j;
        const int p = (s == 1) ? (l >> 1) : (s == 4) ? l : ((l & 1) | ((l >> 2) << 1));
        const int eta_neg = (sg >> p) & 1;
        const int lower = i < j;
        const uint32_t flip = (uint32_t)(eta_neg ^ lower) * FLIP;
        if (i < 4) mlo |= flip << (8 * i);
        else mhi |= flip << (8 * (i - 4));
    }
    const uint32_t srep = (uint32_t)s * 0x01010101u;
    return make_uint4(0x03020100u ^ srep, 0x07060504u ^ srep, mlo, mhi);
}
