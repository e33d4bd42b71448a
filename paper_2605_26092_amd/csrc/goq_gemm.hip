// goq_gemm: many-token dual-PoT layer output, Y[tokens][out] = X[tokens][in] * W^T (Eq. 4).
//
// The contraction is dense (hundreds to thousands of tokens), so it runs on the matrix cores:
//   A16: v_mfma_f32_16x16x32_f16, operands fp16, fp32 accumulation
//   A8 : v_mfma_i32_16x16x64_i8,  operands int8, exact int32 accumulation
// The weight side is the MFMA B operand.  Its register layout -- lane (n = lane % 16,
// kg = lane / 16) holds 8 (fp16) or 16 (int8) consecutive k of output channel n -- is exactly
// one (two) 8-weight micro-block(s) of one row, which is the unit the packed layout stores in a
// dword.  A lane therefore loads its 16-byte quad (4 micro-blocks of its row), decodes each
// micro-block in registers with the byte LUT (H2), and rebuilds the residual basis b2 of the same
// micro-block in registers too (H4): a byte permute by i xor s plus sign flips, both looked up by
// the 6 metadata bits in a 1 KiB LDS table built at kernel start.  No decoded weight ever goes
// through memory.  The activation tile of the current 128-wide slab is staged in LDS (XOR-swizzled
// 16-byte pieces against bank conflicts) and read as the MFMA A operand.
//
// Tiling: workgroup = 4 wavefronts, tile 64 tokens x 128 outputs; each wavefront owns
// 64 tokens x 32 outputs = 4 x 2 MFMA tiles, with three accumulator sets: the slab partials
// P1, P2 (restarted every slab by feeding C = 0 to the slab's first MFMA) and the output Y.
// That fits two wavefronts per SIMD, which measured faster than a 128-token tile at one.
// The next slab's weights (registers) and activations (global_load_lds straight into the other
// LDS buffer) are requested before the current slab's MFMAs; one barrier per slab.
// Coefficient rescale (H5) once per slab: Y += c1[n,g] * P1 + c2[n,g] * P2 in fp32, after the
// slab's MFMAs; a lane needs one (c1, c2) pair per MFMA tile column because every accumulator
// register of a lane belongs to the same output channel.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <type_traits>
#include "goq_layout.h"
#include "goq_decode.h"
#include "goq_internal.h"

namespace {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

#ifndef GOQ_GEMM_TM
#define GOQ_GEMM_TM 64
#endif
constexpr int TM = GOQ_GEMM_TM;   // tokens per workgroup tile
constexpr int TN = 128;       // outputs per workgroup tile
constexpr int WN = 32;        // outputs per wavefront
constexpr int MS = TM / 16;   // MFMA tiles along tokens per wavefront
constexpr int NS = WN / 16;   // MFMA tiles along outputs per wavefront

struct GemmArgs {
    const uint32_t *packed;
    const void *X;
    const float *sx;
    void *Y;
    int32_t *partials;
    int tokens, out, in, gn, rbn, ytype;
};

// Exchange table entry of variant v = pattern | signs << 2 (Theorem 1):
//   x, y : v_perm selectors, byte i of b2 = byte (i xor s) of b1
//   z, w : per-byte masks of the elements whose sign flips (0x80 for fp16 high bytes, 0xFF for
//          int8): b2_i = -eta b1_j for the lower index of a pair, +eta b1_i for the upper one.
template <int ACT>
__device__ __forceinline__ uint4 exchange_entry(int v)
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
        const uint32_t flip = (uint32_t)(eta_neg ^ lower) * (ACT == 0 ? 0x80u : 0xFFu);
        if (i < 4) mlo |= flip << (8 * i);
        else mhi |= flip << (8 * (i - 4));
    }
    const uint32_t srep = (uint32_t)s * 0x01010101u;
    return make_uint4(0x03020100u ^ srep, 0x07060504u ^ srep, mlo, mhi);
}

// 16 * (pattern | signs << 2) of micro-block q (0..3) of a lane's quad
template <int BW>
__device__ __forceinline__ uint32_t exchange_offset(uint32_t w, const uint4 &meta, int m)
{
    if constexpr (BW == 3) {
        const uint32_t t = w & 0x00C0C0C0u;
        const uint32_t u = __umul24(t, 0x1041u);
        return (u >> 14) & 0x3F0u;
    } else {
        const uint32_t pat = (meta.x >> (2 * m)) & 3u;
        const uint32_t sg = (meta.y >> (4 * (m & 7))) & 15u;   // meta.y already holds this lane's half
        return (pat | (sg << 2)) << 4;
    }
}

// per-byte two's complement negation of the bytes selected by mask (0xFF per selected byte)
__device__ __forceinline__ uint32_t negate_bytes(uint32_t x, uint32_t mask)
{
    const uint32_t a = x ^ mask;
    const uint32_t one = mask & 0x01010101u;
    return ((a & 0x7F7F7F7Fu) + one) ^ (a & 0x80808080u);
}

// Decode one micro-block dword into the bytes of b1 and b2 (elements 0..3 in lo, 4..7 in hi).
template <int BW, int ACT>
__device__ __forceinline__ void decode_pair(uint32_t w, const uint4 &meta, int m, const unsigned char *xtab,
                                            uint32_t &b1lo, uint32_t &b1hi, uint32_t &b2lo, uint32_t &b2hi)
{
    goq_decode_bytes<BW, ACT>(w, b1lo, b1hi);
    const uint4 e = *reinterpret_cast<const uint4 *>(xtab + exchange_offset<BW>(w, meta, m));
    const uint32_t tlo = goq_perm(b1hi, b1lo, e.x);
    const uint32_t thi = goq_perm(b1hi, b1lo, e.y);
    if constexpr (ACT == 0) {
        b2lo = tlo ^ e.z;
        b2hi = thi ^ e.w;
    } else {
        b2lo = negate_bytes(tlo, e.z);
        b2hi = negate_bytes(thi, e.w);
    }
}

__device__ __forceinline__ f16x8 widen8(uint32_t lo, uint32_t hi)
{
    const uint4 v = make_uint4(goq_widen01(lo), goq_widen23(lo), goq_widen01(hi), goq_widen23(hi));
    return __builtin_bit_cast(f16x8, v);
}

template <int BW, int ACT, bool PART>
#ifndef GOQ_GEMM_MINWAVES
#define GOQ_GEMM_MINWAVES 2
#endif
__global__ __launch_bounds__(256, GOQ_GEMM_MINWAVES) void gemm_kernel(GemmArgs a)
{
    constexpr int CH = (BW == 3) ? 4 : 5;
    constexpr int XB = (ACT == 0) ? 2 : 1;             // bytes per activation
    constexpr int ROWB = GOQ_N * XB;                   // LDS row stride (XOR-swizzled, not padded)
    constexpr int KSTEPS = (ACT == 0) ? 4 : 2;         // MFMA k-steps per slab
    using AccT = typename std::conditional<ACT == 0, f32x4, i32x4>::type;

    __shared__ __attribute__((aligned(16))) unsigned char xs0[TM * ROWB];
    __shared__ __attribute__((aligned(16))) unsigned char xs1[TM * ROWB];
    __shared__ __attribute__((aligned(16))) unsigned char xtab[64 * 16];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ln = lane & 15;     // MFMA column (output channel) / A row (token)
    const int lh = lane >> 4;     // k-group

    const int mtiles = (a.tokens + TM - 1) / TM;
    const int mt = blockIdx.x % mtiles;
    const int nt = blockIdx.x / mtiles;
    const int m0 = mt * TM;
    const int n0 = nt * TN + wave * WN;

    if (tid < 64) *reinterpret_cast<uint4 *>(xtab + tid * 16) = exchange_entry<ACT>(tid);

    f32x4 Yacc[MS][NS];
#pragma unroll
    for (int i = 0; i < MS; ++i)
#pragma unroll
        for (int j = 0; j < NS; ++j) Yacc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    // the quad this lane reads for MFMA column tile j: row n0 + 16 j + ln, chunk lh
    bool live[NS];
    const uint32_t *wq[NS];
#pragma unroll
    for (int j = 0; j < NS; ++j) {
        const int row = n0 + 16 * j + ln;
        live[j] = (row / GOQ_ROWS) < a.rbn;
        wq[j] = a.packed + goq_quad_index(CH, a.gn, row / GOQ_ROWS, 0, lh, row % GOQ_ROWS);
    }
    const int64_t gstride = (int64_t)CH * GOQ_ROWS * 4;     // dwords between macro-blocks

    // 16-byte pieces of the activation slab this thread moves from HBM to LDS
    constexpr int PIECES = TM * GOQ_N * XB / 16;
    constexpr int PER_ROW = GOQ_N * XB / 16;
    constexpr int NP = PIECES / 256;
    auto swz = [](int row) { return (ACT == 0) ? (row & 15) : ((row >> 1) & 7); };
    auto load_weights = [&](int g, uint4 (&wd)[NS], uint4 (&meta)[NS]) {
#pragma unroll
        for (int j = 0; j < NS; ++j) {
            wd[j] = make_uint4(0, 0, 0, 0);
            meta[j] = make_uint4(0, 0, 0, 0);
            if (live[j]) {
                wd[j] = *reinterpret_cast<const uint4 *>(wq[j] + g * gstride);
                if constexpr (BW == 4) {
                    // chunk 4 of the same row: patterns, signs lo, signs hi, coefficient word
                    const uint4 mq = *reinterpret_cast<const uint4 *>(wq[j] + g * gstride + (4 - lh) * GOQ_ROWS * 4);
                    meta[j] = make_uint4(mq.x >> (8 * lh), (lh < 2 ? mq.y : mq.z) >> (16 * (lh & 1)), 0, mq.w);
                }
            }
        }
    };
    // Activation slab -> LDS without passing through registers (global_load_lds_dwordx4): each
    // instruction fills 64 consecutive 16-byte LDS slots, one per lane, from per-lane addresses.
    // Slot (row, cs) holds k-piece cs ^ f(row): the XOR swizzle makes the 16 rows an MFMA A
    // operand read touches fall into 16 different bank groups (row stride is 256 / 128 bytes).
    // per-thread byte offsets (inside the token tile) of the pieces this thread requests: constant
    // over the slabs, so a slab's request is one uniform base plus these 32-bit offsets
    uint32_t xoff[NP];
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        const int S = i * 256 + tid;
        const int row = S / PER_ROW, cs = S % PER_ROW;
        const int c = cs ^ swz(row);
        int m = m0 + row;
        m = m < a.tokens ? m : a.tokens - 1;          // rows past the end are never stored
        xoff[i] = (uint32_t)(m - m0) * (uint32_t)a.in * XB + c * 16;
    }
    const unsigned char *xtile = reinterpret_cast<const unsigned char *>(a.X) + (int64_t)m0 * a.in * XB;
    auto stage_x = [&](int g, unsigned char *buf) {
        const unsigned char *base = xtile + (int64_t)g * GOQ_N * XB;
#pragma unroll
        for (int i = 0; i < NP; ++i)
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void *)(base + xoff[i]),
                (__attribute__((address_space(3))) void *)(buf + (i * 256 + wave * 64) * 16), 16, 0, 0);
    };

    // slab 0 is staged up front; afterwards the next slab's weights and activations are requested
    // from HBM before the current slab's MFMAs (activations land in the other LDS buffer)
    uint4 wd[NS], meta[NS], wdn[NS], metan[NS];
    load_weights(0, wd, meta);
    stage_x(0, xs0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    for (int g = 0; g < a.gn; ++g) {
        const unsigned char *xs = (g & 1) ? xs1 : xs0;
        if (g + 1 < a.gn) {
            load_weights(g + 1, wdn, metan);
            stage_x(g + 1, (g & 1) ? xs0 : xs1);
        }

        // ---- coefficient pair of this lane's column in every column tile
        float c1[NS], c2[NS];
#pragma unroll
        for (int j = 0; j < NS; ++j) {
            uint32_t cw;
            if constexpr (BW == 3) {
                // this lane's 4 dwords carry 8 of the 32 bits; the 4 k-group lanes of a column
                // (lane, lane^16, lane^32, lane^48) carry the rest
                uint32_t part = ((wd[j].x >> 30) << 6) | ((wd[j].y >> 30) << 4) | ((wd[j].z >> 30) << 2) | (wd[j].w >> 30);
                part <<= (24 - 8 * lh);
                part |= __shfl_xor(part, 16);
                part |= __shfl_xor(part, 32);
                cw = part;
            } else {
                cw = meta[j].w;
            }
            c1[j] = __half2float(__ushort_as_half((unsigned short)(cw & 0xffffu)));
            c2[j] = __half2float(__ushort_as_half((unsigned short)(cw >> 16)));
        }

        // ---- the slab's MFMAs: every A operand read from LDS feeds the b1 and b2 MFMAs of both
        //      column tiles
        AccT P1[MS][NS], P2[MS][NS];
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            if constexpr (ACT == 0) {
                f16x8 B1[NS], B2[NS];
#pragma unroll
                for (int j = 0; j < NS; ++j) {
                    const uint32_t w = ks == 0 ? wd[j].x : ks == 1 ? wd[j].y : ks == 2 ? wd[j].z : wd[j].w;
                    uint32_t l1, h1, l2, h2;
                    decode_pair<BW, ACT>(w, meta[j], ks, xtab, l1, h1, l2, h2);
                    B1[j] = widen8(l1, h1);
                    B2[j] = widen8(l2, h2);
                }
#pragma unroll
                for (int i = 0; i < MS; ++i) {
                    // A operand: token 16 i + ln, k = 8 (4 lh + ks) .. + 7 of the slab
                    const f16x8 A = *reinterpret_cast<const f16x8 *>(xs + (16 * i + ln) * ROWB + (((4 * lh + ks) ^ swz(16 * i + ln)) * 16));
                    const f32x4 z = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int j = 0; j < NS; ++j) {
                        P1[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(A, B1[j], ks == 0 ? z : P1[i][j], 0, 0, 0);
                        P2[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(A, B2[j], ks == 0 ? z : P2[i][j], 0, 0, 0);
                    }
                }
            } else {
                i32x4 B1[NS], B2[NS];
#pragma unroll
                for (int j = 0; j < NS; ++j) {
                    const uint32_t wa = ks == 0 ? wd[j].x : wd[j].z;
                    const uint32_t wb = ks == 0 ? wd[j].y : wd[j].w;
                    uint32_t l1, h1, l2, h2, l3, h3, l4, h4;
                    decode_pair<BW, ACT>(wa, meta[j], 2 * ks, xtab, l1, h1, l2, h2);
                    decode_pair<BW, ACT>(wb, meta[j], 2 * ks + 1, xtab, l3, h3, l4, h4);
                    B1[j] = i32x4{(int)l1, (int)h1, (int)l3, (int)h3};
                    B2[j] = i32x4{(int)l2, (int)h2, (int)l4, (int)h4};
                }
#pragma unroll
                for (int i = 0; i < MS; ++i) {
                    // A operand: token 16 i + ln, k = 32 lh + 16 ks .. + 15 of the slab
                    const i32x4 A = *reinterpret_cast<const i32x4 *>(xs + (16 * i + ln) * ROWB + (((2 * lh + ks) ^ swz(16 * i + ln)) * 16));
                    const i32x4 z = i32x4{0, 0, 0, 0};
#pragma unroll
                    for (int j = 0; j < NS; ++j) {
                        P1[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(A, B1[j], ks == 0 ? z : P1[i][j], 0, 0, 0);
                        P2[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(A, B2[j], ks == 0 ? z : P2[i][j], 0, 0, 0);
                    }
                }
            }
#ifdef GOQ_GEMM_SCHEDBAR
            __builtin_amdgcn_sched_barrier(0);
#endif
        }
        // ---- coefficient rescale, once per slab, outside the dot-product loop (H5)
#pragma unroll
        for (int i = 0; i < MS; ++i)
#pragma unroll
            for (int j = 0; j < NS; ++j) {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    Yacc[i][j][v] = fmaf(c1[j], (float)P1[i][j][v], Yacc[i][j][v]);
                    Yacc[i][j][v] = fmaf(c2[j], (float)P2[i][j][v], Yacc[i][j][v]);
                }
                if constexpr (PART) {
                    // exact int32 slab partials [tokens][out][in/128][2] (verification output)
                    const int n = n0 + 16 * j + ln;
                    int32_t *pp = a.partials + (((int64_t)(m0 + 16 * i + 4 * lh) * a.out + n) * a.gn + g) * 2;
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int m = m0 + 16 * i + 4 * lh + v;
                        if (m < a.tokens && n < a.out)
                            *reinterpret_cast<int2 *>(pp + (int64_t)v * a.out * a.gn * 2) = make_int2(P1[i][j][v], P2[i][j][v]);
                    }
                }
            }
        if (g + 1 < a.gn) {
#pragma unroll
            for (int j = 0; j < NS; ++j) { wd[j] = wdn[j]; meta[j] = metan[j]; }
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the next slab's activations are in LDS
        __syncthreads();
    }

    // ---- store the tile (H6): lane holds Y[m0 + 16 i + 4 lh + v][n0 + 16 j + ln]
#pragma unroll
    for (int i = 0; i < MS; ++i)
#pragma unroll
        for (int j = 0; j < NS; ++j) {
            const int n = n0 + 16 * j + ln;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int m = m0 + 16 * i + 4 * lh + v;
                if (m >= a.tokens || n >= a.out) continue;
                float y = Yacc[i][j][v];
                if constexpr (ACT == 1) y *= a.sx[m] * (1.f / (float)(1 << ((1 << (BW - 1)) - 1)));
                if (a.ytype == GOQ_F32) reinterpret_cast<float *>(a.Y)[(int64_t)m * a.out + n] = y;
                else reinterpret_cast<__half *>(a.Y)[(int64_t)m * a.out + n] = __float2half(y);
            }
        }
}

template <int BW, int ACT>
int launch(hipStream_t st, const GemmArgs &a)
{
    const int mtiles = (a.tokens + TM - 1) / TM;
    const int ntiles = (a.out + TN - 1) / TN;
    if (ACT == 1 && a.partials)
        hipLaunchKernelGGL((gemm_kernel<BW, ACT, (ACT == 1)>), dim3(mtiles * ntiles), dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL((gemm_kernel<BW, ACT, false>), dim3(mtiles * ntiles), dim3(256), 0, st, a);
    return goq_check_launch("goq_gemm");
}

}  // namespace

int goq_launch_gemm(hipStream_t st, int bw, int act, int64_t tokens, int64_t out, int64_t in,
                    const void *packed, const void *X, const float *sx, void *Y, int ytype,
                    int32_t *partials)
{
    GemmArgs a;
    a.packed = (const uint32_t *)packed;
    a.X = X;
    a.sx = sx;
    a.Y = Y;
    a.partials = partials;
    a.tokens = (int)tokens;
    a.out = (int)out;
    a.in = (int)in;
    a.gn = (int)(in / GOQ_N);
    a.rbn = (int)goq_row_blocks(out);
    a.ytype = ytype;
    if (bw == 3 && act == GOQ_A16) return launch<3, 0>(st, a);
    if (bw == 3 && act == GOQ_A8) return launch<3, 1>(st, a);
    if (bw == 4 && act == GOQ_A16) return launch<4, 0>(st, a);
    return goq_set_error(GOQ_EUNSUPPORTED, "goq_gemm: bw=4 with int8 activations is not implemented");
}
