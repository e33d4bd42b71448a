// goq_gemv / goq_gemv_batch: batch-1 dual-PoT layer output (Eq. 4 with one token).
//
// Why the matrix cores appear in a bandwidth-bound kernel.  A batch-1 product streams 4 (bw = 3)
// or 5 (bw = 4) bits per weight and has to retire two multiply-accumulates per weight (b1 and b2).
// On the vector ALU that is, all in, 3.5 lane-instructions per weight (decode, widen to fp16,
// two-term dot products): more issue time than the HBM stream takes, so the vector ALU, not HBM,
// was the limit.  Here the vector ALU only DECODES: a 3-bit code becomes, with one byte look-up
// permute, the 8-bit float (E5M2) of its power of two -- E5M2 is exactly the high byte of the
// fp16 value, and a power of two has no other nonzero byte -- and b2 is rebuilt from b1 by the
// Theorem 1 exchange as one more byte permute plus a sign XOR (what Sec. 3.3 builds from a
// four-way exchange multiplexer and an XOR gate per lane, driven by the 6 stored metadata bits).  The multiply-accumulates
// run on v_mfma_f32_16x16x128_f8f6f4 as a 16-row x 128-deep product per instruction:
//
//   B operand (weights): lane l = (column c = l % 16, k-group q = l / 16) supplies the 32 decoded
//       weights k = 32 q .. 32 q + 31 of output row 16 j + c of the row block (j = 0..3: four
//       instructions per basis cover the 64 rows of a row block times one macro-block).  That is
//       exactly the 16-byte quad (chunk q, row 16 j + c) of the packed layout.
//   A operand (activations): eight of the 16 rows hold the eight digits of the macro-block's
//       128 activations (digit d in row 4 (d / 2) + d % 2, the other rows are zero).
//       Activations are handed over as block fixed point, see stage_run.
//   D[row][c] = sum_k digit(x_k) b[row c][k]: lane (c, q) receives rows 4q .. 4q + 3, i.e. two
//       digit sums, so the slab dot product of a row is spread over four lanes and is put
//       together once, when the row is stored.
//
// Work decomposition.  The unit of work is (row group, macro-block g): a ROW GROUP is 8 row
// blocks of 64 output channels, one row block per wavefront of a 512-thread workgroup.  All units
// of all problems of a launch form one linear sequence (problem, row group, g) cut into equal
// contiguous pieces, one per workgroup (two workgroups per CU), so every workgroup streams the
// same number of bytes whatever the matrix shapes are.  The coefficient rescale (H5) is two FMAs
// per row and slab, after the slab's dot products.
//
// (Launches of a few hundred 16-row tiles at most -- single layers -- take the second kernel of this
// file instead, gemv_rows_kernel: one workgroup per 16 rows over the whole depth, no combine.)
//
// Where a piece boundary falls inside a row group, each wavefront publishes the partial sums of
// its 64 rows to a workspace and the LAST wavefront to arrive (an atomic counter per boundary
// and row block) adds the parts in workgroup order and stores y: no zero-fill pass, no
// floating-point atomics, and the result does not depend on timing.  The workspace is the
// caller's (goq_gemv_batch_ws, goq_gemv_stream) or one of the library's static regions, one per
// stream (goq_gemv, goq_gemv_batch).
//
// The same kernel body runs in two forms: with up to GOQ_MAX_BATCH problems in the kernel
// arguments (goq_gemv_batch: the lowest start-up latency), and with a problem table in device
// memory (goq_gemv_stream: thousands of problems -- e.g. every projection of every decoder block
// of a model -- as ONE unit sequence, so that start-up and tail are paid once per stream).
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <mutex>
#include <string.h>
#include <stddef.h>
#include <stdio.h>
#include <type_traits>
#include "goq_layout.h"
#include "goq_decode.h"
#include "goq_internal.h"


namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
// (explicitly global-memory pointers: generic ones would turn loads into flat loads, which the LDS
// wait counter has to wait for as well)
typedef const __attribute__((address_space(1))) uint32_t *gptr;
typedef const __attribute__((address_space(1))) u32x4 *gptr4;

#ifndef GOQ_WAVES
#define GOQ_WAVES 8
#define GOQ_WGS 512
#define GOQ_WPE 4
#endif
constexpr int WAVES = GOQ_WAVES;                 // wavefronts (= row blocks) per workgroup
constexpr int NT = WAVES * 64;           // threads per workgroup
constexpr int MAX_WG = GOQ_WGS;              // workgroups per launch (two per CU)
constexpr int SW = 16;                   // units whose activation digits are resident in LDS
constexpr int XG = 1024;                 // bytes of digits per macro-block: 4 k-groups x 8 digits x 32
constexpr int XZ = 256;                  // zero bytes in front of the digit table
#ifndef GOQ_CB
#define GOQ_CB 16
#endif
#ifndef GOQ_VCOPIES
#define GOQ_VCOPIES 16
#endif
constexpr int VC = GOQ_VCOPIES;          // copies of the exchange table in LDS (a lane uses copy lane % VC)
constexpr int VS = VC * 16;              // bytes from one entry to the next
constexpr int CB = GOQ_CB;               // parts a combining wavefront requests at a time
constexpr int REGIONS = 8;               // static scratch regions: one per stream that launches

// Workspace of one launch: the parts of the row groups cut by a piece boundary.
struct Region {
    float partials[MAX_WG][2][NT];       // [workgroup][head | tail][row of the row group]
    unsigned counters[MAX_WG][WAVES];    // arrivals per boundary (first contributor) and row block
};
// The library's own regions, for the entry points that take no workspace.  Host code never uses
// this name as an address: region_of_stream() resolves the device address once per device.
static __device__ __align__(256) Region scratch[REGIONS];

struct GemvProblem {
    const uint32_t *packed;
    const void *x;
    const float *sx;
    void *y;
    int out;
    int gn;          // macro-blocks per row
    int ytype;
    int rbn;         // row blocks
    int rgroups;     // row groups
    int begin;       // first unit of this problem in the linear unit sequence
    int bb;          // first 16-row block of this problem in the grid of the row-owner kernel
    int pad;
};

struct GemvArgs {
    int n;
    int total;       // units in the launch
    int pq, pr;      // total / workgroups, total % workgroups
    Region *scratch;
    GemvProblem p[GOQ_MAX_BATCH];
};

// Problem table of goq_gemv_stream (built on the host by goq_gemv_stream_table, copied to the
// device by the caller): this header, then the n problems.
constexpr uint32_t TABLE_MAGIC = 0x51544247u;
struct GemvTable {
    uint32_t magic;
    int bw, act;
    int n;
    int total;       // units of the whole stream
    int nwg;         // workgroups (= pieces) of the launch
    int pq, pr;      // total / nwg, total % nwg
    int pad[8];
    int first[MAX_WG];   // the problem that holds the first unit of each piece
};

// Where the problems of a launch live: in the kernel arguments (up to GOQ_MAX_BATCH) or in a
// table in device memory.
template <bool TABLE>
struct Problems;
// (Kernel arguments are read through the kernel-argument segment pointer: indexing the by-value
// argument struct with a run-time index inside loops makes the compiler copy it to scratch.)
template <>
struct Problems<false> {
    typedef const __attribute__((address_space(4))) GemvProblem Entry;
    Entry *t;
    int cnt;
    __device__ __forceinline__ Entry &operator[](int i) const { return t[i]; }
    __device__ __forceinline__ int n() const { return cnt; }
};
template <>
struct Problems<true> {
    const GemvProblem *__restrict__ t;
    int cnt;
    __device__ __forceinline__ const GemvProblem &operator[](int i) const { return t[i]; }
    __device__ __forceinline__ int n() const { return cnt; }
};

// The piece decomposition of a launch and its workspace.
struct Pieces {
    int pq, pr;
    Region *scratch;
};

// What one lane holds of one unit: for j = 0..3 the quad (chunk q, row 16 j + c); for bw = 4
// also the metadata dword of chunk q of that row.
template <int BW>
struct UnitBuf {
    uint4 q[4];
    uint32_t md[(BW == 4) ? 4 : 1];
};

template <int BW>
__device__ __forceinline__ void load_unit(const uint32_t *__restrict__ packed, int64_t gn, int64_t R, int64_t g,
                                          int lane, UnitBuf<BW> &u)
{
    constexpr int CH = (BW == 3) ? 4 : 5;
    const int c = lane & 15, q = lane >> 4;
    // (explicitly a global-memory pointer: a generic one would turn the loads into flat loads,
    // which the LDS wait counter has to wait for as well)
    typedef const __attribute__((address_space(1))) uint32_t *gptr;
    typedef const __attribute__((address_space(1))) u32x4 *gptr4;
    gptr base = (gptr)packed + (R * gn + g) * (CH * GOQ_ROWS * 4);
    gptr4 pq = (gptr4)(base + q * (GOQ_ROWS * 4) + c * 4);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const u32x4 v = __builtin_nontemporal_load(pq + 16 * j);       // streamed once: no reuse
        u.q[j] = make_uint4(v.x, v.y, v.z, v.w);
    }
    if constexpr (BW == 4) {
        gptr pm = base + 4 * (GOQ_ROWS * 4) + c * 4 + q;
#pragma unroll
        for (int j = 0; j < 4; ++j) u.md[j] = __builtin_nontemporal_load(pm + 64 * j);
    }
}

// ---- activation digits ----------------------------------------------------------------------
// The 8-bit-float matrix instruction adds the products of 8 consecutive k on a grid that ends 13
// binary places below the largest exponent sum of the 8 (measured); anything lower is cut off.
// Floating-point pieces of x (own exponent per element) would therefore lose bits whenever a
// micro-block mixes large and small activations.  So x is handed over as block FIXED point: for
// each block of 32 activations that share an MFMA block scale, with largest exponent E, |x_k| is
// written with 24 bits below 2^(E+1) -- every fp16 value within 2^13 of the block maximum exactly,
// smaller ones truncated at 2^(E-23), the same footing as an fp32 sum -- and cut into 8 digits of
// 3 bits.  Digit i of the block is an E5M2 operand (0..7 are exact in E5M2) with the block scale
// 2^(E-2-3i), applied by the MFMA's per-lane E8M0 scale.  Inside a micro-block all products are
// now (3-bit digit) x (power of two >= 2^-7): at most 13 binary places, so the instruction's grid
// keeps every bit, and D = sum_k digit_k b_k is exact.
//
// Which 32 activations share a block scale is fixed by the instruction (measured): the scale a
// lane of lane-group Q supplies covers, of the A row it holds, register halves (bytes 0..15 for
// Q = 0, 1; bytes 16..31 for Q = 2, 3) of the two k-groups 2 (Q % 2) and 2 (Q % 2) + 1.  In
// micro-blocks m = 0..15 of the macro-block that is block Q = {m : m / 8 == Q % 2, (m / 2) % 2 ==
// Q / 2}, i.e. micro-blocks b, b+1, b+4, b+5 with b = 0, 8, 2, 10.
//
// One run = 8 consecutive activations (one micro-block), handled by one thread.  Digit table of a
// macro-block: the 32 bytes of (k-group h, digit i) at h * 256 + i * 32; scale byte (E + 110) of
// block Q at st[Q], where E + 15 is the largest biased fp16 exponent of the block (subnormals
// count as 1).
// The 8 activations of run r as four registers of two fp16 each, from the run's raw words:
// raw[0..3] (fp16), raw[0..1] (int8), raw[0] (packed int4: element i in nibble i) or the low 48
// bits of raw[1]:raw[0] (packed int6: element i in bits 6 i .. 6 i + 5) or the low 24 bits of raw[0]
// (packed int3: element i in bits 3 i .. 3 i + 2).  Integer activations are exact in fp16.
template <int ACT>
__device__ __forceinline__ void run_as_half(const uint32_t (&raw)[4], uint32_t (&v)[4])
{
    if constexpr (ACT == 0) {
        v[0] = raw[0]; v[1] = raw[1]; v[2] = raw[2]; v[3] = raw[3];
    } else if constexpr (ACT == 1) {
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const int e0 = (int)(int8_t)(raw[d >> 1] >> (16 * (d & 1)));
            const int e1 = (int)(int8_t)(raw[d >> 1] >> (16 * (d & 1) + 8));
            const goq_half2 hv = {(_Float16)e0, (_Float16)e1};     // exact: |e| <= 128
            v[d] = __builtin_bit_cast(uint32_t, hv);
        }
    } else if constexpr (ACT == 2) {
        const uint32_t q = raw[0];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const int e0 = (int)(q << (28 - 8 * d)) >> 28;         // sign-extended nibble 2 d
            const int e1 = (int)(q << (24 - 8 * d)) >> 28;         // nibble 2 d + 1
            const goq_half2 hv = {(_Float16)e0, (_Float16)e1};
            v[d] = __builtin_bit_cast(uint32_t, hv);
        }
    } else if constexpr (ACT == 4) {
        const uint32_t q = raw[0];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const int e0 = (int)(q << (29 - 6 * d)) >> 29;         // sign-extended field 2 d
            const int e1 = (int)(q << (26 - 6 * d)) >> 29;         // field 2 d + 1
            const goq_half2 hv = {(_Float16)e0, (_Float16)e1};
            v[d] = __builtin_bit_cast(uint32_t, hv);
        }
    } else {
        // fields 0..4 lie in raw[0], field 5 straddles the two words, 6 and 7 lie in raw[1]
        const uint32_t lo = raw[0], hi = (raw[0] >> 30) | (raw[1] << 2);     // hi: fields 5, 6, 7 from bit 0
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const int k0 = 2 * d, k1 = 2 * d + 1;
            const int e0 = k0 < 5 ? (int)(lo << (26 - 6 * k0)) >> 26 : (int)(hi << (26 - 6 * (k0 - 5))) >> 26;
            const int e1 = k1 < 5 ? (int)(lo << (26 - 6 * k1)) >> 26 : (int)(hi << (26 - 6 * (k1 - 5))) >> 26;
            const goq_half2 hv = {(_Float16)e0, (_Float16)e1};
            v[d] = __builtin_bit_cast(uint32_t, hv);
        }
    }
}

// run r of macro-block g of x in global memory
template <int ACT>
__device__ __forceinline__ void load_run(const void *x, int g, int r, uint32_t (&raw)[4])
{
    raw[0] = raw[1] = raw[2] = raw[3] = 0u;
    if constexpr (ACT == 0) {
        const u32x4 q = ((gptr4)x)[(int64_t)g * 16 + r];
        raw[0] = q.x; raw[1] = q.y; raw[2] = q.z; raw[3] = q.w;
    } else if constexpr (ACT == 1) {
        raw[0] = ((gptr)x)[(int64_t)g * 32 + 2 * r];
        raw[1] = ((gptr)x)[(int64_t)g * 32 + 2 * r + 1];
    } else if constexpr (ACT == 2) {
        raw[0] = ((gptr)x)[(int64_t)g * 16 + r];
    } else if constexpr (ACT == 4) {
        // the run's 3 bytes start at byte 3 r of the macro-block's 48; they reach into the next
        // dword only when they start at byte 2 or 3 of theirs (never for the last run)
        const gptr p = (gptr)x + ((int64_t)g * 12 + ((3 * r) >> 2));
        const uint32_t sh = (uint32_t)((3 * r) & 3) * 8u;
        const uint32_t d0 = p[0], d1 = sh > 8u ? p[1] : 0u;
        raw[0] = sh ? __builtin_amdgcn_alignbit(d1, d0, sh) : d0;
    } else {
        // the run's 6 bytes start at byte 6 r of the macro-block's 96: in the two dwords from dword
        // 3 r / 2, at byte offset 0 (r even) or 2 (r odd)
        const gptr p = (gptr)x + ((int64_t)g * 24 + ((3 * r) >> 1));
        const uint32_t d0 = p[0], d1 = p[1];
        raw[0] = (r & 1) ? __builtin_amdgcn_alignbit(d1, d0, 16) : d0;
        raw[1] = (r & 1) ? (d1 >> 16) : d1;
    }
}

template <int ACT>
__device__ __forceinline__ void stage_digits(unsigned char *xt, unsigned char *st, const uint32_t (&raw)[4], int r);

template <int ACT>
__device__ __forceinline__ void stage_run(unsigned char *xt, unsigned char *st, const void *x, int g, int r)
{
    uint32_t raw[4];
    load_run<ACT>(x, g, r, raw);
    stage_digits<ACT>(xt, st, raw, r);
}

// digit table and block scales of one run (see above) from its raw words
template <int ACT>
__device__ __forceinline__ void stage_digits(unsigned char *xt, unsigned char *st, const uint32_t (&raw)[4], int r)
{
    uint32_t v[4];
    run_as_half<ACT>(raw, v);
    // largest biased exponent of the run (subnormals count as 1), then of the scale block
    int emax = 1;
#pragma unroll
    for (int d = 0; d < 4; ++d)
        emax = max(emax, max((int)((v[d] >> 10) & 31u), (int)((v[d] >> 26) & 31u)));
    emax = max(emax, __shfl_xor(emax, 1));              // runs r, r^1, r^4, r^5 form one scale block
    emax = max(emax, __shfl_xor(emax, 4));
    // 24-bit fixed point below 2^(emax - 14), truncated: |x| 2^(38 - emax) is an integer part of at
    // most 24 bits, exact in fp32, and the conversion to integer truncates
    uint32_t fx[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const unsigned short hb = (unsigned short)((v[k >> 1] >> (16 * (k & 1))) & 0x7FFFu);
        fx[k] = (uint32_t)ldexpf((float)__builtin_bit_cast(_Float16, hb), 38 - emax);
    }
    // sign bytes of elements 0..3 and 4..7
    const uint32_t slo = goq_perm(v[1], v[0], 0x07050301u) & 0x80808080u;
    const uint32_t shi = goq_perm(v[3], v[2], 0x07050301u) & 0x80808080u;
    unsigned char *dst = xt + (r >> 2) * 256 + (r & 3) * 8;
    // Digit i of an element is bits 23 - 3 i .. 21 - 3 i of its fixed-point value.  The three bytes
    // of the values are first gathered across four elements (one element per byte), so that a digit
    // of four elements is a shift and a mask of one register.
    uint32_t dg[2][8];
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) {
        uint32_t pl[3];
#pragma unroll
        for (int b = 0; b < 3; ++b) {
            const uint32_t sel = 0x0c0c0400u + (uint32_t)b * 0x0101u;              // byte b of both sources
            pl[b] = goq_perm(goq_perm(fx[4 * hf + 3], fx[4 * hf + 2], sel), goq_perm(fx[4 * hf + 1], fx[4 * hf], sel), 0x05040100u);
        }
        const uint32_t M = 0x07070707u;
        dg[hf][0] = (pl[2] >> 5) & M;
        dg[hf][1] = (pl[2] >> 2) & M;
        dg[hf][2] = ((pl[2] << 1) & 0x06060606u) | ((pl[1] >> 7) & 0x01010101u);
        dg[hf][3] = (pl[1] >> 4) & M;
        dg[hf][4] = (pl[1] >> 1) & M;
        dg[hf][5] = ((pl[1] << 2) & 0x04040404u) | ((pl[0] >> 6) & 0x03030303u);
        dg[hf][6] = (pl[0] >> 3) & M;
        dg[hf][7] = pl[0] & M;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        // E5M2 of 0..7: 00 3C 40 42 44 45 46 47
        const uint32_t lo = goq_perm(0x47464544u, 0x42403C00u, dg[0][i]) | slo;
        const uint32_t hi = goq_perm(0x47464544u, 0x42403C00u, dg[1][i]) | shi;
        *reinterpret_cast<uint2 *>(dst + i * 32) = make_uint2(lo, hi);
    }
    if ((r & 5) == 0) st[(r & 2) | (r >> 3)] = (unsigned char)(emax + 110);
}

// Position in the linear unit sequence.
struct Cursor {
    int pi, rg, g;
};

// The few fields of a problem the streaming loop needs, read once per problem and kept in scalar
// registers.  end: first unit of the next problem.
struct Stream {
    const uint32_t *packed;
    void *y;
    const float *sx;
    int gn, rbn, rgroups, begin, end, out, ytype;
};

__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

template <typename Fields>
__device__ __forceinline__ void output_fields(Stream &s, const Fields &P)
{
    const uint64_t py = (uint64_t)P.y, ps = (uint64_t)P.sx;
    s.y = (void *)(((uint64_t)(uint32_t)uniform((int)(py >> 32)) << 32) | (uint32_t)uniform((int)py));
    s.sx = (const float *)(((uint64_t)(uint32_t)uniform((int)(ps >> 32)) << 32) | (uint32_t)uniform((int)ps));
    s.out = uniform(P.out);
    s.ytype = uniform(P.ytype);
}

// OUTPUT: also the fields the end of a row group needs (bw = 3 keeps them in scalar registers for
// the whole problem, so that a row group ends without a memory round trip; bw = 4 has no registers
// to spare and reads them when a row group ends).
template <bool OUTPUT, bool TABLE>
__device__ __forceinline__ Stream stream_of(const Problems<TABLE> &pb, int pi)
{
    Stream s;
    const auto &P = pb[pi];
    if constexpr (OUTPUT) output_fields(s, P);
    const uint64_t pk = (uint64_t)P.packed;
    s.packed = (const uint32_t *)(((uint64_t)(uint32_t)uniform((int)(pk >> 32)) << 32) | (uint32_t)uniform((int)pk));
    s.gn = uniform(P.gn);
    s.rbn = uniform(P.rbn);
    s.rgroups = uniform(P.rgroups);
    s.begin = uniform(P.begin);
    s.end = uniform(P.begin + P.rgroups * P.gn);
    return s;
}

// Digits of the units [u0, u0 + ns) of the sequence, unit s into table slot s.  Thread
// (slot = tid / 16, run = tid % 16); ns <= SW = NT / 32.  u0 lies in problem pi0, whose units end
// at end0; units past it belong to the following problems.
template <int ACT, bool TABLE>
__device__ __forceinline__ void stage_window(const Problems<TABLE> &pb, int pi0, int end0, int u0, int ns,
                                             unsigned char *xt, unsigned char *st, int tid)
{
    if (tid < ns * 16) {
        const int slot = tid >> 4;
        const int u = u0 + slot;
        int pi = pi0;
        if (u >= end0) {
            ++pi;
            while (pi + 1 < pb.n() && u >= pb[pi + 1].begin) ++pi;
        }
        const auto &P = pb[pi];
        stage_run<ACT>(xt + slot * XG, st + slot * 4, P.x, (u - P.begin) % P.gn, tid & 15);
    }
}

// ---- one 16-row slice of a macro-block (decode, exchange, the two slab dot products) ---------
// quad: the lane's quad (chunk q, row c of the slice); md (bw = 4): the metadata dword of that
// chunk and row; vt: LDS address of this lane's copy of the exchange table; A, sa: the
// macro-block's digits (this lane's A row and k-group) and their block scale.  D1, D2: the
// matrix instruction's results against b1 and b2; this lane group's two digit sums of row c are
// elements 0 and 1.
template <int BW>
__device__ __forceinline__ void slice_products(const uint4 &quad, uint32_t md, uint32_t vt,
                                               const v8i &A, int sa, v4f &D1, v4f &D2)
{
    const v4f zero = {0.f, 0.f, 0.f, 0.f};
    const uint32_t dw[4] = {quad.x, quad.y, quad.z, quad.w};
    // LA exchange-table entries are requested ahead, so that the look-ups are in flight while the
    // primary codes are decoded (bw = 4 has fewer registers to spare)
    constexpr int LA = (BW == 3) ? 4 : 2;
    u32x4 ev[4];
    auto address = [&](int k) {            // LDS address of the entry: vt + VS * (pattern | signs << 2)
        if constexpr (BW == 3) {
            // a_0 (bits 6..7), a_1 (14..15), a_2 (22..23) are the top two bits of bytes 0..2: a
            // byte dot product with weights 1, 4, 16 gives 64 (a_0 + 4 a_1 + 16 a_2); the weights
            // are scaled to the entry stride VS
            return __builtin_amdgcn_udot4(dw[k] & 0x00C0C0C0u, 0x00100401u * (VS / 64), vt, false);
        } else {
            return vt + ((md >> (6 * k)) & 63u) * VS;
        }
    };
    auto fetch = [&](int k, uint32_t eo) {
        ev[k] = *reinterpret_cast<const __attribute__((address_space(3))) u32x4 *>(eo);
    };
    auto request = [&](int k) { fetch(k, address(k)); };
    {
        // the addresses first, then the reads: a dot-product result needs a few cycles before an
        // LDS instruction may use it as address, which the other address computations cover
        uint32_t eo[LA];
#pragma unroll
        for (int k = 0; k < LA; ++k) eo[k] = address(k);
#pragma unroll
        for (int k = 0; k < LA; ++k) __builtin_amdgcn_sched_group_barrier(0x002, BW == 3 ? 2 : 3, 0);   // VALU
        __builtin_amdgcn_sched_group_barrier(0x100, LA, 0);                                            // DS read
#pragma unroll
        for (int k = 0; k < LA; ++k) fetch(k, eo[k]);
    }
    v8i B1, B2;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        uint32_t lo, hi;
        goq_decode_bytes<BW, 0>(dw[k], lo, hi);                      // code -> E5M2 byte
        B1[2 * k] = (int)lo;
        B1[2 * k + 1] = (int)hi;
    }
    // E5M2 x E5M2, fp32 accumulation; block scale sa on the activation side, 2^0 on the weight side
    D1 = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(A, B1, zero, 1, 1, 0, sa, 0, 127);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint32_t lo = (uint32_t)B1[2 * k], hi = (uint32_t)B1[2 * k + 1];
        B2[2 * k] = (int)(goq_perm(hi, lo, ev[k].x) ^ ev[k].z);       // Theorem 1 exchange + sign XOR
        B2[2 * k + 1] = (int)(goq_perm(hi, lo, ev[k].y) ^ ev[k].w);
        if (k + LA < 4) request(k + LA);
    }
    D2 = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(A, B2, zero, 1, 1, 0, sa, 0, 127);
}

// A row's coefficient word is spread over what its four lanes (c, 0..3) load, one byte each: two
// bits in each of the quad's dwords (bw = 3), the top byte of the metadata dword (bw = 4).
// position: the byte of the word this lane holds.
template <int BW>
__device__ __forceinline__ uint32_t coefficient_byte(const uint4 &quad, uint32_t md)
{
    if constexpr (BW == 3) {
        uint32_t cw = quad.x >> 30;
        cw = __builtin_amdgcn_alignbit(cw, quad.y, 30);
        cw = __builtin_amdgcn_alignbit(cw, quad.z, 30);
        cw = __builtin_amdgcn_alignbit(cw, quad.w, 30);
        return cw;
    } else {
        return md >> 24;
    }
}
template <int BW>
__device__ __forceinline__ int coefficient_byte_position(int q) { return BW == 3 ? 3 - q : q; }

// Coefficient rescale (Eq. 4), once per slab, outside the dot-product loop: the two digit sums
// this lane group received for each basis, times the slab's coefficient pair.
__device__ __forceinline__ float rescale(uint32_t cword, const v4f &D1, const v4f &D2, float acc)
{
    const float c1 = __half2float(__ushort_as_half((unsigned short)(cword & 0xffffu)));
    const float c2 = __half2float(__ushort_as_half((unsigned short)(cword >> 16)));
    return fmaf(c2, D2[0] + D2[1], fmaf(c1, D1[0] + D1[1], acc));
}

// ---- one unit of one wavefront: 64 rows x one macro-block --------------------------------------
// buf: the lane's quads; cwx: this wavefront's 256-byte exchange area for coefficient bytes;
// acc[j]: running sum of row 16 j + c over the digits this lane receives.
template <int BW>
__device__ __forceinline__ void compute_unit(const UnitBuf<BW> &buf, uint32_t vt, const v8i &A, int sa,
                                             unsigned char *cwx, int lane, float (&acc)[4])
{
    const int c = lane & 15, q = lane >> 4;
    // The four lanes (c, 0..3) each hold one byte of the coefficient word of row 16 j + c; they
    // swap bytes through LDS, for all four sub-steps at once.  (LDS operations of one wavefront
    // execute in order; the empty asm only keeps the compiler from moving the reads above the
    // writes.)
    const int cpos = coefficient_byte_position<BW>(q);
#pragma unroll
    for (int j = 0; j < 4; ++j)
        cwx[j * 64 + c * 4 + cpos] = (unsigned char)coefficient_byte<BW>(buf.q[j], buf.md[BW == 4 ? j : 0]);
    asm volatile("" ::: "memory");
    // bw = 3: the rescale of slice j is issued after the matrix instructions of slice j + 1, whose
    // decode covers the latency of slice j's results (bw = 4 has no registers to spare for that).
    constexpr bool DEFER = (BW == 3);
    v4f D1[2], D2[2];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        slice_products<BW>(buf.q[j], buf.md[BW == 4 ? j : 0], vt, A, sa, D1[j & 1], D2[j & 1]);
        const int jr = DEFER ? j - 1 : j;
        if (jr >= 0) {
            const uint32_t cword = *reinterpret_cast<const uint32_t *>(cwx + jr * 64 + c * 4);
            acc[jr] = rescale(cword, D1[jr & 1], D2[jr & 1], acc[jr]);
        }
    }
    if constexpr (DEFER) {
        const uint32_t cword = *reinterpret_cast<const uint32_t *>(cwx + 3 * 64 + c * 4);
        acc[3] = rescale(cword, D1[1], D2[1], acc[3]);
    }
}

// The unit sequence is cut into nwg pieces: the first `pr` workgroups take pq + 1 units, the others
// pq (pq = total / nwg and pr = total % nwg come from the host).
// first unit of workgroup b's piece
__device__ __forceinline__ int piece_begin(const Pieces &pc, int b)
{
    return b * pc.pq + min(b, pc.pr);
}

// the workgroup whose piece holds unit u
__device__ __forceinline__ int piece_of(const Pieces &pc, int u)
{
    const int big = pc.pr * (pc.pq + 1);                    // units held by the larger pieces
    return u < big ? u / (pc.pq + 1) : pc.pr + (u - big) / pc.pq;
}

// Reduce + store for the 64 rows of one wavefront: acc[j] of lanes (c, 0..3) add up to the sum of
// row 16 j + c over the units [max(u0, i0), min(u1, i1)) of its row group.
//
// Split row groups.  Every contributor writes its 64 parts with agent-scope atomic stores (they go
// through to memory, past the L2 of its XCD), waits until they have been acknowledged
// (s_waitcnt vmcnt(0): the hardware form of "these stores happen before what follows"), and then
// counts itself in with an agent-scope atomic add on the boundary's counter.  The contributor whose
// add returns the last count reads all parts with agent-scope atomic loads (which do not hit in a
// stale L2 line) -- every one of them was acknowledged before its writer's add, and the adds are
// totally ordered at the counter, so the reader's loads come after all the stores.  This is a
// release (stores, wait, add) / acquire (add, loads) pair built from per-access scopes instead of
// fences: an agent-scope release FENCE would write back the whole L2 for 256 bytes of parts.
// P: the problem's fields, from the table (GemvProblem) or from scalar registers (Stream).
template <int ACT, typename Fields>
__device__ __forceinline__ void flush(const Fields &P, const Pieces &pc, const Cursor &cur, float (&acc)[4],
                                      int i0, int i1, int wave, int lane)
{
    const int u0 = P.begin + cur.rg * P.gn, u1 = u0 + P.gn;
    // lane l takes over row l of the row block: the sum of row 16 j + c is spread over the four
    // lanes c, c + 16, c + 32, c + 48 (two digits each)
    float mine = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float t = acc[j] + __shfl_xor(acc[j], 16);
        t += __shfl_xor(t, 32);
        const float r = __shfl(t, lane & 15);
        if ((lane >> 4) == j) mine = r;
    }
    if constexpr (ACT != 0) mine *= ((const __attribute__((address_space(1))) float *)P.sx)[0];
    const int rl = wave * GOQ_ROWS + lane;                 // row inside the row group
    const int row = cur.rg * (WAVES * GOQ_ROWS) + rl;
    auto store = [&](float s) {
        if (row < P.out) {
            // (global-memory pointers, said explicitly: a generic store may hit LDS as far as the
            // compiler knows, and every later LDS read would wait for it)
            if (P.ytype == GOQ_F32) ((__attribute__((address_space(1))) float *)P.y)[row] = s;
            else ((__attribute__((address_space(1))) unsigned short *)P.y)[row] = __half_as_ushort(__float2half(s));
        }
    };
    if (i0 <= u0 && u1 <= i1) {                            // the whole row group was ours
        store(mine);
        return;
    }
    // Of the contributors bf..bl only the first can hold the row group as the tail of its piece
    // (slot 1); for the others it is the head.
    Region *S = pc.scratch;
    const int b = blockIdx.x;
    __hip_atomic_store(&S->partials[b][i0 > u0 ? 0 : 1][rl], mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int bf = piece_of(pc, u0), bl = piece_of(pc, u1 - 1);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    unsigned old = 0;
    if (lane == 0) {
        old = __hip_atomic_fetch_add(&S->counters[bf][wave], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (old == (unsigned)(bl - bf))                    // back to zero for the next launch
            __hip_atomic_store(&S->counters[bf][wave], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    old = (unsigned)uniform((int)old);
    if (old == (unsigned)(bl - bf)) {
        float s = __hip_atomic_load(&S->partials[bf][1][rl], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        for (int w = bf + 1; w <= bl; w += CB) {           // CB independent loads at a time
            float t[CB];
#pragma unroll
            for (int i = 0; i < CB; ++i)
                t[i] = __hip_atomic_load(&S->partials[min(w + i, bl)][0][rl], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
            for (int i = 0; i < CB; ++i)
                if (w + i <= bl) s += t[i];
        }
        store(s);
    }
}

// ---- the streaming loop of one workgroup over its piece [i0, i1) ------------------------------
// cur: the position of unit i0.  LDS: xtab = zeros (the A rows without a digit), then the digit
// table of the resident units; stab = its block scales; vtab = exchange table, entry v at
// VS v + 16 r, VC copies r (lane l reads copy l % 16: the 16 lanes of a 128-bit LDS read then hit 16
// different bank groups whatever their entries v are); cwx = coefficient-byte exchange.
template <int BW, int ACT, bool TABLE>
__device__ __forceinline__ void stream_piece(const Problems<TABLE> &pb, const Pieces &pc, int i0, int i1, Cursor cur,
                                             unsigned char *xtab, unsigned char *stab, unsigned char *vtab,
                                             unsigned char *cwx)
{
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = uniform(tid >> 6);

    // the first unit's weights are requested before anything else
    UnitBuf<BW> bufA, bufB;
    constexpr bool KEEP = (BW == 3);
    Stream S = stream_of<KEEP>(pb, cur.pi);
    load_unit<BW>(S.packed, S.gn, min(cur.rg * WAVES + wave, S.rbn - 1), cur.g, lane, bufA);

    for (int t = tid; t < 64 * VC; t += NT) *reinterpret_cast<uint4 *>(vtab + t * 16) = goq_exchange_entry<0x80u>(t / VC);
    if (tid < XZ / 4) reinterpret_cast<uint32_t *>(xtab)[tid] = 0u;

    // A operand of this lane: row = lane % 16, k-group q = lane / 16.  Digit d sits in row
    // 4 (d / 2) + d % 2, so that every lane group receives two digit sums (D rows 4q, 4q + 1) and
    // rows 4q + 2, 4q + 3 are zero.
    const int arow = lane & 15, q = lane >> 4;
    const bool arow_live = (arow & 3) < 2;
    const int digit = 2 * (arow >> 2) + (arow & 1);
    const uint32_t abase = arow_live ? (uint32_t)(XZ + q * 256 + digit * 32) : 0u;
    const uint32_t amask = arow_live ? ~0u : 0u;
    const uint32_t vt_lane = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)vtab + (lane % VC) * 16;

    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    int idx = i0;
    // One unit: (re)stage the digits when the resident window is used up, request the next unit's
    // weights (MORE), compute this unit, flush at the end of a row group.  The request is
    // unconditional inside a MORE step -- a wavefront without rows of its own in the next row
    // group re-reads that group's last row block -- so that the compiler's wait counts stay
    // exact: this unit's registers wait for exactly the loads older than the new request.
    auto step = [&](UnitBuf<BW> &bcur, UnitBuf<BW> &bnxt, auto more_tag) {
        constexpr bool MORE = decltype(more_tag)::value;
        const int slot = (idx - i0) % SW;
        if (slot == 0) {
            if (idx != i0) __syncthreads();                    // everyone is done with the old window
            stage_window<ACT, TABLE>(pb, cur.pi, S.end, idx, min(SW, i1 - idx), xtab + XZ, stab, tid);
            __syncthreads();
        }
        Cursor nxt = cur;
        if (++nxt.g == S.gn) { nxt.g = 0; if (++nxt.rg == S.rgroups) { nxt.rg = 0; ++nxt.pi; } }
        Stream Sn = S;
        if constexpr (MORE) {
            if (nxt.pi != cur.pi) Sn = stream_of<KEEP>(pb, nxt.pi);
            load_unit<BW>(Sn.packed, Sn.gn, min(nxt.rg * WAVES + wave, Sn.rbn - 1), nxt.g, lane, bnxt);
        }
        const int R = cur.rg * WAVES + wave;
        const bool live = R < S.rbn;
        if (live) {
            const v8i A = *reinterpret_cast<const v8i *>(xtab + abase + ((uint32_t)(slot * XG) & amask));
            const uint32_t sc = *reinterpret_cast<const uint32_t *>(stab + slot * 4);
            const int sa = (int)((sc >> (8 * q)) & 0xFFu) - 3 * digit;    // digit i sits 3 i places lower
            compute_unit<BW>(bcur, vt_lane, A, sa, cwx + wave * 256, lane, acc);
        }
        if (!MORE || nxt.rg != cur.rg || nxt.pi != cur.pi) {
            if (live) {
                if constexpr (KEEP) flush<ACT>(S, pc, cur, acc, i0, i1, wave, lane);
                else flush<ACT>(pb[cur.pi], pc, cur, acc, i0, i1, wave, lane);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[j] = 0.f;
        }
        cur = nxt;
        S = Sn;
        ++idx;
    };
    while (true) {
        if (idx + 1 < i1) step(bufA, bufB, std::true_type{});
        else { step(bufA, bufB, std::false_type{}); break; }
        if (idx + 1 < i1) step(bufB, bufA, std::true_type{});
        else { step(bufB, bufA, std::false_type{}); break; }
    }
}

// LDS of the streaming kernels
#define GOQ_GEMV_LDS                                                                     \
    __shared__ __attribute__((aligned(16))) unsigned char xtab[XZ + SW * XG];            \
    __shared__ __attribute__((aligned(16))) unsigned char stab[SW * 4];                  \
    __shared__ __attribute__((aligned(256))) unsigned char vtab[64 * VS];                \
    __shared__ __attribute__((aligned(16))) unsigned char cwx[WAVES * 256]

// Problems in the kernel arguments.  The leading scalar arguments repeat what the first
// instructions of a workgroup need -- the piece sizes and the first unit of every problem -- as
// separate kernel arguments, so that they can be preloaded into scalar registers at wavefront
// launch (-amdgpu-kernarg-preload-count): finding the workgroup's first unit then costs no memory
// round trip, and its weights are requested one round trip (the problem's fields) after the
// wavefront starts.
template <int BW, int ACT>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(GOQ_WPE, GOQ_WPE)))
void gemv_kernel(int pq, int pr, int bg1, int bg2, int bg3, int bg4, int bg5, int bg6, int bg7, GemvArgs a)
{
    GOQ_GEMV_LDS;
    // this workgroup's piece [i0, i1) of the unit sequence
    const int bid = blockIdx.x;
    const int i0 = uniform(bid * pq + min(bid, pr));
    const int i1 = uniform((bid + 1) * pq + min(bid + 1, pr));
    if (i0 >= i1) return;

    // the problem that holds unit i0, by compares with the (preloaded) first units: unused
    // problems start at INT_MAX
    Cursor cur;
    {
        const int bg[GOQ_MAX_BATCH] = {0, bg1, bg2, bg3, bg4, bg5, bg6, bg7};
        int pi = 0, b0 = 0;
#pragma unroll
        for (int i = 1; i < GOQ_MAX_BATCH; ++i) {
            const bool ge = i0 >= bg[i];
            pi += ge ? 1 : 0;
            b0 = ge ? bg[i] : b0;
        }
        const int gn = a.p[pi].gn;
        cur.pi = uniform(pi);
        cur.rg = uniform((i0 - b0) / gn);
        cur.g = uniform((i0 - b0) % gn);
    }
    // `a` follows the nine leading ints (36 bytes) at the next 8-byte boundary of the segment
    constexpr int KARG_P = 40 + (int)offsetof(GemvArgs, p);
    const __attribute__((address_space(4))) char *kseg =
        (const __attribute__((address_space(4))) char *)__builtin_amdgcn_kernarg_segment_ptr();
    const Problems<false> pb{(const __attribute__((address_space(4))) GemvProblem *)(kseg + KARG_P), a.n};
    const Pieces pc{pq, pr, a.scratch};
    stream_piece<BW, ACT, false>(pb, pc, i0, i1, cur, xtab, stab, vtab, cwx);
}

// Problems in a table in device memory (goq_gemv_stream).
template <int BW, int ACT>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(GOQ_WPE, GOQ_WPE)))
void gemv_stream_kernel(const GemvTable *__restrict__ T, Region *ws)
{
    GOQ_GEMV_LDS;
    const int bid = blockIdx.x;
    const int pq = uniform(T->pq), pr = uniform(T->pr);
    const int i0 = uniform(bid * pq + min(bid, pr));
    const int i1 = uniform((bid + 1) * pq + min(bid + 1, pr));
    if (i0 >= i1) return;
    const Problems<true> pb{reinterpret_cast<const GemvProblem *>(T + 1), uniform(T->n)};
    Cursor cur;
    cur.pi = uniform(T->first[bid]);
    {
        const GemvProblem &P = pb[cur.pi];
        const int local = i0 - P.begin, gn = P.gn;
        cur.rg = uniform(local / gn);
        cur.g = uniform(local % gn);
    }
    const Pieces pc{pq, pr, ws};
    stream_piece<BW, ACT, true>(pb, pc, i0, i1, cur, xtab, stab, vtab, cwx);
}

// Zero-fill of a caller-owned workspace (a kernel, not a memset node, so that a caller may
// capture it).
__global__ __launch_bounds__(256) void workspace_init_kernel(Region *ws)
{
    unsigned *c = &ws->counters[0][0];
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < MAX_WG * WAVES; i += gridDim.x * blockDim.x) c[i] = 0u;
}


// ---- small layers: one workgroup per 16 output rows ------------------------------------------
// When a launch has few units per workgroup of the kernel above, each row group is cut among up
// to gn workgroups and the combine through the scratch area -- a device-scope round trip per
// batch of contributors -- costs more than the streaming.  This kernel cuts the
// other way: a workgroup owns 16 output rows (one matrix-instruction tile: sub-step j of row block
// R) over the whole depth, its eight wavefronts take the macro-blocks round-robin, and the 32
// partial sums of a row (8 wavefronts x 4 lane groups) meet in LDS, added in a fixed order.  No
// scratch, no atomics.  Measured against the streaming kernel it is the faster one as long as the
// grid fits the chip in one go and the launch is small (layers up to about 8192 x 4096 or
// 4096 x 11008); beyond that the streaming kernel's equal pieces win.
constexpr int RW = NT / 16;              // macro-blocks staged per window: one run per thread
constexpr int RS = RW / WAVES;           // slices per wavefront and window
constexpr int ROWS_MAX_TILES = 512;      // automatic choice: largest grid ...
constexpr int ROWS_MAX_SLICES = 24576;   // ... and most (tile, macro-block) slices per launch

struct Slice {
    uint4 q;
    uint32_t md;
};

template <int BW, int ACT>
__global__ __launch_bounds__(NT)
void gemv_rows_kernel(GemvArgs a)
{
    __shared__ __attribute__((aligned(16))) unsigned char xtab[XZ + RW * XG];
    __shared__ __attribute__((aligned(16))) unsigned char stab[RW * 4];
    __shared__ __attribute__((aligned(16))) unsigned char vtab[64 * VS];
    __shared__ __attribute__((aligned(16))) unsigned char cwx[WAVES * 256];
    __shared__ float red[NT];
    constexpr int CH = (BW == 3) ? 4 : 5;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 15, q = lane >> 4;

    int pi = 0;
#pragma unroll
    for (int i = 1; i < GOQ_MAX_BATCH; ++i) pi += ((int)blockIdx.x >= a.p[i].bb) ? 1 : 0;   // unused: INT_MAX
    pi = __builtin_amdgcn_readfirstlane(pi);
    const GemvProblem &P = a.p[pi];
    const int lb = (int)blockIdx.x - P.bb;
    const int R = lb >> 2, j = lb & 3;
    const int gn = P.gn;

    typedef const __attribute__((address_space(1))) uint32_t *gptr;
    typedef const __attribute__((address_space(1))) u32x4 *gptr4;
    gptr rowbase = (gptr)P.packed + (int64_t)R * gn * (CH * GOQ_ROWS * 4) + (16 * j + c) * 4;
    // slices of macro-blocks w0 + wave + WAVES i (past the end: the last one again, not used)
    auto request = [&](int w0, Slice (&s)[RS]) {
#pragma unroll
        for (int i = 0; i < RS; ++i) {
            const int g = min(w0 + wave + WAVES * i, gn - 1);
            gptr base = rowbase + (int64_t)g * (CH * GOQ_ROWS * 4);
            const u32x4 v = __builtin_nontemporal_load((gptr4)(base + q * (GOQ_ROWS * 4)));
            s[i].q = make_uint4(v.x, v.y, v.z, v.w);
            s[i].md = 0u;
            if constexpr (BW == 4) s[i].md = __builtin_nontemporal_load(base + 4 * (GOQ_ROWS * 4) + q);
        }
    };
    Slice cur[RS], nxt[RS];
    request(0, cur);

    for (int t = tid; t < 64 * VC; t += NT) *reinterpret_cast<uint4 *>(vtab + t * 16) = goq_exchange_entry<0x80u>(t / VC);
    if (tid < XZ / 4) reinterpret_cast<uint32_t *>(xtab)[tid] = 0u;

    // A operand of this lane, as in the kernel above
    const bool arow_live = (c & 3) < 2;
    const int digit = 2 * (c >> 2) + (c & 1);
    const uint32_t abase = arow_live ? (uint32_t)(XZ + q * 256 + digit * 32) : 0u;
    const uint32_t amask = arow_live ? ~0u : 0u;
    const uint32_t vt_lane = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)vtab + (lane % VC) * 16;
    unsigned char *cw = cwx + wave * 256;

    float acc = 0.f;
    for (int w0 = 0; w0 < gn; w0 += RW) {
        if (w0) __syncthreads();                               // everyone is done with the old window
        if (tid < min(RW, gn - w0) * 16)
            stage_run<ACT>(xtab + XZ + (tid >> 4) * XG, stab + (tid >> 4) * 4, P.x, w0 + (tid >> 4), tid & 15);
        __syncthreads();
        if (w0 + RW < gn) request(w0 + RW, nxt);
#pragma unroll
        for (int i = 0; i < RS; ++i)
            cw[i * 64 + c * 4 + coefficient_byte_position<BW>(q)] = (unsigned char)coefficient_byte<BW>(cur[i].q, cur[i].md);
        asm volatile("" ::: "memory");
#pragma unroll
        for (int i = 0; i < RS; ++i) {
            const int slot = wave + WAVES * i;
            if (w0 + slot < gn) {
                const v8i A = *reinterpret_cast<const v8i *>(xtab + abase + ((uint32_t)(slot * XG) & amask));
                const uint32_t sc = *reinterpret_cast<const uint32_t *>(stab + slot * 4);
                const int sa = (int)((sc >> (8 * q)) & 0xFFu) - 3 * digit;
                v4f D1, D2;
                slice_products<BW>(cur[i].q, cur[i].md, vt_lane, A, sa, D1, D2);
                acc = rescale(*reinterpret_cast<const uint32_t *>(cw + i * 64 + c * 4), D1, D2, acc);
            }
        }
#pragma unroll
        for (int i = 0; i < RS; ++i) cur[i] = nxt[i];
    }
    // H6: the 32 partial sums of row c, in wavefront and lane-group order
    red[tid] = acc;
    __syncthreads();
    if (tid < 16) {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < NT / 16; ++i) s += red[i * 16 + tid];
        if constexpr (ACT != 0) s *= ((const __attribute__((address_space(1))) float *)P.sx)[0];
        const int row = R * GOQ_ROWS + 16 * j + tid;
        if (row < P.out) {
            // (global-memory pointers, said explicitly: a generic store may hit LDS as far as the
            // compiler knows, and every later LDS read would wait for it)
            if (P.ytype == GOQ_F32) ((__attribute__((address_space(1))) float *)P.y)[row] = s;
            else ((__attribute__((address_space(1))) unsigned short *)P.y)[row] = __half_as_ushort(__float2half(s));
        }
    }
}

template <int BW, int ACT>
int launch_rows(hipStream_t st, const GemvArgs &a, int nblocks)
{
    hipLaunchKernelGGL((gemv_rows_kernel<BW, ACT>), dim3(nblocks), dim3(NT), 0, st, a);
    return goq_check_launch("goq_gemv");
}

template <int BW, int ACT>
int launch(hipStream_t st, const GemvArgs &a, int nwg)
{
    static_assert(GOQ_MAX_BATCH == 8, "the kernel takes the first units of problems 1..7 as arguments");
    hipLaunchKernelGGL((gemv_kernel<BW, ACT>), dim3(nwg), dim3(NT), 0, st, a.pq, a.pr, a.p[1].begin, a.p[2].begin,
                       a.p[3].begin, a.p[4].begin, a.p[5].begin, a.p[6].begin, a.p[7].begin, a);
    return goq_check_launch("goq_gemv");
}

template <int BW, int ACT>
int launch_stream(hipStream_t st, const GemvTable *dev, Region *ws, int nwg)
{
    hipLaunchKernelGGL((gemv_stream_kernel<BW, ACT>), dim3(nwg), dim3(NT), 0, st, dev, ws);
    return goq_check_launch("goq_gemv_stream");
}

// ---- the library's static regions ---------------------------------------------------------------
// Launches on one stream run one after the other, so a region per stream is never shared by two
// launches in flight.  Per device: the device address of `scratch` (looked up once, with that
// device current) and which stream owns which region.
constexpr int MAXDEV = 64;
struct DeviceRegions {
    Region *base = nullptr;
    hipStream_t owner[REGIONS] = {};
    bool used[REGIONS] = {};
    unsigned long long stamp[REGIONS] = {};
};
DeviceRegions g_regions[MAXDEV];
unsigned long long g_clock = 0;
std::mutex g_regions_mutex;

// Region of stream st on the current device, or nullptr with *rc set.
Region *region_of_stream(hipStream_t st, int *rc)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAXDEV) {
        *rc = goq_set_error(GOQ_EHIP, "goq_gemv: cannot tell the current device");
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_regions_mutex);
    DeviceRegions &D = g_regions[dev];
    if (!D.base) {
        void *sym = nullptr;
        const hipError_t e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !sym) {
            *rc = goq_set_error(GOQ_EHIP, "goq_gemv: cannot resolve the scratch area on device %d: %s", dev,
                                hipGetErrorString(e));
            return nullptr;
        }
        D.base = reinterpret_cast<Region *>(sym);
    }
    ++g_clock;
    int free_slot = -1;
    for (int i = 0; i < REGIONS; ++i) {
        if (D.used[i] && D.owner[i] == st) { D.stamp[i] = g_clock; return D.base + i; }
        if (!D.used[i] && free_slot < 0) free_slot = i;
    }
    if (free_slot < 0) {
        // All regions have an owner: take over the least recently used one, after waiting on the
        // host until its stream has drained (the only call of this library that may block; a
        // stream that no longer exists counts as drained).  Not possible while either stream is
        // being captured.
        int lru = 0;
        for (int i = 1; i < REGIONS; ++i)
            if (D.stamp[i] < D.stamp[lru]) lru = i;
        hipStreamCaptureStatus mine = hipStreamCaptureStatusNone, theirs = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(st, &mine) != hipSuccess) (void)hipGetLastError();
        const bool gone = hipStreamIsCapturing(D.owner[lru], &theirs) != hipSuccess;
        if (gone) (void)hipGetLastError();
        if (mine != hipStreamCaptureStatusNone || (!gone && theirs != hipStreamCaptureStatusNone)) {
            *rc = goq_set_error(GOQ_EUNSUPPORTED,
                                "goq_gemv: all %d scratch regions of device %d belong to other streams and one of the "
                                "streams involved is being captured; use goq_gemv_batch_ws with a workspace of your own",
                                REGIONS, dev);
            return nullptr;
        }
        if (!gone && hipStreamSynchronize(D.owner[lru]) != hipSuccess) (void)hipGetLastError();
        free_slot = lru;
    }
    D.used[free_slot] = true;
    D.owner[free_slot] = st;
    D.stamp[free_slot] = g_clock;
    return D.base + free_slot;
}

// selection of goq_gemv_select: a property of the calling thread, so that one caller's experiment
// or test cannot change what another thread of the process launches
thread_local int g_kernel = GOQ_GEMV_AUTO;

void fill_problem(GemvProblem &P, const goq_gemv_desc &d)
{
    P.packed = (const uint32_t *)d.packed;
    P.x = d.x;
    P.sx = d.sx;
    P.y = d.y;
    P.out = (int)d.out;
    P.gn = (int)(d.in / GOQ_N);
    P.ytype = d.ytype;
    P.rbn = (int)goq_row_blocks(d.out);
    P.rgroups = (P.rbn + WAVES - 1) / WAVES;
    P.begin = 0;
    P.bb = 0;
    P.pad = 0;
}

}  // namespace

void goq_gemv_set_kernel(int kernel) { g_kernel = kernel; }

size_t goq_gemv_workspace_size() { return sizeof(Region); }

int goq_launch_gemv_workspace_init(hipStream_t st, void *workspace)
{
    hipLaunchKernelGGL(workspace_init_kernel, dim3(16), dim3(256), 0, st, reinterpret_cast<Region *>(workspace));
    return goq_check_launch("goq_gemv_workspace_init");
}

// Which kernel a launch of these problems takes under the current selection, and with how many
// workgroups (host logic only).
int goq_gemv_plan_launch(int n, const goq_gemv_desc *descs, int *kernel, int *workgroups)
{
    int64_t units = 0, blocks = 0, slices = 0;
    for (int i = 0; i < n; ++i) {
        const int64_t gn = descs[i].in / GOQ_N;
        units += (goq_row_blocks(descs[i].out) + WAVES - 1) / WAVES * gn;
        blocks += (descs[i].out + 15) / 16;
        slices += (descs[i].out + 15) / 16 * gn;
        if (units > 0x3fffffff || blocks > 0x3fffffff)
            return goq_set_error(GOQ_ESHAPE, "goq_gemv: too much work for one launch");
    }
    const int which = g_kernel;
    const bool rows = which == GOQ_GEMV_ROWS ||
                      (which == GOQ_GEMV_AUTO && blocks <= ROWS_MAX_TILES && slices <= ROWS_MAX_SLICES);
    *kernel = rows ? GOQ_GEMV_ROWS : GOQ_GEMV_STREAM;
    *workgroups = rows ? (int)blocks : (int)(units < MAX_WG ? units : MAX_WG);
    return GOQ_OK;
}

// workspace: the caller's, or NULL for the library's region of this stream
int goq_launch_gemv(hipStream_t st, int bw, int act, int n, const goq_gemv_desc *descs, void *workspace)
{
    int kernel = 0, workgroups = 0;
    int rc = goq_gemv_plan_launch(n, descs, &kernel, &workgroups);
    if (rc) return rc;
    GemvArgs a;
    a.n = n;
    a.scratch = nullptr;
    int64_t total = 0, blocks = 0;
    for (int i = 0; i < n; ++i) {
        GemvProblem &P = a.p[i];
        fill_problem(P, descs[i]);
        P.begin = (int)total;
        total += (int64_t)P.rgroups * P.gn;
        P.bb = (int)blocks;
        blocks += (descs[i].out + 15) / 16;
    }
    for (int i = n; i < GOQ_MAX_BATCH; ++i) { a.p[i] = a.p[0]; a.p[i].begin = 0x7fffffff; a.p[i].bb = 0x7fffffff; }
    a.total = (int)total;
    a.pq = a.pr = 0;
    // Small launches go to the row-owner kernel: one workgroup per 16 output rows, no workspace.
    if (kernel == GOQ_GEMV_ROWS) {
        const int nb = workgroups;
        if (bw == 3 && act == GOQ_A16) return launch_rows<3, 0>(st, a, nb);
        if (bw == 3 && act == GOQ_A8) return launch_rows<3, 1>(st, a, nb);
        if (bw == 4 && act == GOQ_A8) return launch_rows<4, 1>(st, a, nb);
        if (bw == 3 && act == GOQ_A4) return launch_rows<3, 2>(st, a, nb);
        if (bw == 4 && act == GOQ_A4) return launch_rows<4, 2>(st, a, nb);
        if (bw == 3 && act == GOQ_A6) return launch_rows<3, 3>(st, a, nb);
        if (bw == 4 && act == GOQ_A6) return launch_rows<4, 3>(st, a, nb);
        if (bw == 3 && act == GOQ_A3) return launch_rows<3, 4>(st, a, nb);
        if (bw == 4 && act == GOQ_A3) return launch_rows<4, 4>(st, a, nb);
        return launch_rows<4, 0>(st, a, nb);
    }
    a.scratch = reinterpret_cast<Region *>(workspace);
    if (!a.scratch) {
        a.scratch = region_of_stream(st, &rc);
        if (!a.scratch) return rc;
    }
    // two 512-thread workgroups per CU (4 wavefronts per SIMD)
    const int nwg = workgroups;
    a.pq = a.total / nwg;
    a.pr = a.total % nwg;
    if (bw == 3 && act == GOQ_A16) return launch<3, 0>(st, a, nwg);
    if (bw == 3 && act == GOQ_A8) return launch<3, 1>(st, a, nwg);
    if (bw == 4 && act == GOQ_A8) return launch<4, 1>(st, a, nwg);
    if (bw == 3 && act == GOQ_A4) return launch<3, 2>(st, a, nwg);
    if (bw == 4 && act == GOQ_A4) return launch<4, 2>(st, a, nwg);
    if (bw == 3 && act == GOQ_A6) return launch<3, 3>(st, a, nwg);
    if (bw == 4 && act == GOQ_A6) return launch<4, 3>(st, a, nwg);
    if (bw == 3 && act == GOQ_A3) return launch<3, 4>(st, a, nwg);
    if (bw == 4 && act == GOQ_A3) return launch<4, 4>(st, a, nwg);
    return launch<4, 0>(st, a, nwg);
}

// ---- goq_gemv_stream: the problem table ---------------------------------------------------------
size_t goq_gemv_stream_table_size(int n) { return sizeof(GemvTable) + (size_t)n * sizeof(GemvProblem); }

int goq_gemv_stream_build_table(int bw, int act, int n, const goq_gemv_desc *descs, void *table)
{
    GemvTable *T = reinterpret_cast<GemvTable *>(table);
    GemvProblem *P = reinterpret_cast<GemvProblem *>(T + 1);
    memset(T, 0, sizeof(GemvTable));
    int64_t total = 0;
    for (int i = 0; i < n; ++i) {
        fill_problem(P[i], descs[i]);
        P[i].begin = (int)total;
        total += (int64_t)P[i].rgroups * P[i].gn;
        if (total > 0x3fffffff) return goq_set_error(GOQ_ESHAPE, "goq_gemv_stream_table: too much work for one stream");
    }
    T->magic = TABLE_MAGIC;
    T->bw = bw;
    T->act = act;
    T->n = n;
    T->total = (int)total;
    T->nwg = (int)(total < MAX_WG ? total : MAX_WG);
    T->pq = T->total / T->nwg;
    T->pr = T->total % T->nwg;
    int pi = 0;
    for (int b = 0; b < MAX_WG; ++b) {
        const int64_t i0 = (int64_t)b * T->pq + (b < T->pr ? b : T->pr);
        if (b >= T->nwg) { T->first[b] = 0; continue; }
        while (pi + 1 < n && i0 >= P[pi + 1].begin) ++pi;
        T->first[b] = pi;
    }
    return GOQ_OK;
}

int goq_launch_gemv_stream(hipStream_t st, const void *table_host, const void *table_dev, void *workspace)
{
    const GemvTable *T = reinterpret_cast<const GemvTable *>(table_host);
    if (T->magic != TABLE_MAGIC || T->n < 1 || T->nwg < 1 || T->nwg > MAX_WG)
        return goq_set_error(GOQ_EINVAL, "goq_gemv_stream: table_host was not written by goq_gemv_stream_table");
    const GemvTable *dev = reinterpret_cast<const GemvTable *>(table_dev);
    Region *ws = reinterpret_cast<Region *>(workspace);
    const int bw = T->bw, act = T->act, nwg = T->nwg;
    if (bw == 3 && act == GOQ_A16) return launch_stream<3, 0>(st, dev, ws, nwg);
    if (bw == 3 && act == GOQ_A8) return launch_stream<3, 1>(st, dev, ws, nwg);
    if (bw == 4 && act == GOQ_A8) return launch_stream<4, 1>(st, dev, ws, nwg);
    if (bw == 3 && act == GOQ_A4) return launch_stream<3, 2>(st, dev, ws, nwg);
    if (bw == 4 && act == GOQ_A4) return launch_stream<4, 2>(st, dev, ws, nwg);
    if (bw == 3 && act == GOQ_A6) return launch_stream<3, 3>(st, dev, ws, nwg);
    if (bw == 4 && act == GOQ_A6) return launch_stream<4, 3>(st, dev, ws, nwg);
    if (bw == 3 && act == GOQ_A3) return launch_stream<3, 4>(st, dev, ws, nwg);
    if (bw == 4 && act == GOQ_A3) return launch_stream<4, 4>(st, dev, ws, nwg);
    return launch_stream<4, 0>(st, dev, ws, nwg);
}
