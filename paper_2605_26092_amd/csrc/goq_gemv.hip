// goq_gemv / goq_gemv_batch: batch-1 dual-PoT layer output (Eq. 4 with one token).
//
// Work decomposition.  A workgroup of 4 wavefronts takes a ROW GROUP of 4*NRB row blocks
// (a row block = 64 output channels, one per lane) and a range of macro-blocks g.  For every
// g the lane that owns row r loads that row's whole macro-block (CH coalesced 16-byte quads,
// see goq_layout.h) and keeps both slab dot products P1, P2 and the coefficient pair in its own
// registers, so the slab needs no cross-lane traffic at all; the coefficient rescale (H5) is two
// FMAs per 128 weights, after the slab's dot products.
//
// Residual basis without rebuilding it: x . b2 = b1 . (T x), where T is the signed exchange
// of the micro-block (Theorem 1).  T depends only on the micro-block's 6 metadata bits, and
// x is shared by all rows, so the workgroup stages, per macro-block, the 64 possible T x for
// each of the 16 micro-block positions in LDS (16 KiB for fp16 x) and a lane fetches the
// variant its metadata selects with one 16-byte LDS read.  P1 uses x itself, which is uniform
// across the wavefront (scalar registers).  Per micro-block a lane then spends: 2 byte-LUT
// permutes (decode), 4 byte shuffles (widen to fp16), 8 two-term fp16 dot products.
//
// Output: a workgroup that covers all macro-blocks of its rows stores y directly; otherwise
// the macro-block ranges are combined with fp32 atomic adds into a y that a fill kernel zeroed.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include "goq_layout.h"
#include "goq_decode.h"
#include "goq_internal.h"

namespace {

struct GemvProblem {
    const uint32_t *packed;
    const void *x;
    const float *sx;
    void *y;
    int out;
    int gn;          // macro-blocks per row
    int ytype;
    int rbn;         // row blocks
    int gper;        // macro-blocks per task
    int gsplits;     // tasks along g
    int task_begin;  // first blockIdx of this problem
    int atomic;      // combine with atomics (y is fp32 and pre-zeroed)
};

struct GemvArgs {
    int n;
    GemvProblem p[GOQ_MAX_BATCH];
};

constexpr int WAVES = 4;
constexpr int NRB_DEFAULT = 2;   // row blocks per wavefront

// Per-thread constants of the exchange variant v = pattern | signs << 2 this thread stages:
// for output register t (elements 2t, 2t+1): which x register holds the partners, whether the
// halves swap, and the sign mask (x'_i = +eta x_j for the lower index of a pair, -eta x_i for
// the upper one).
struct Variant {
    int src[4];        // element index of the partner of element 2t (its register is src >> 1)
    uint32_t swapsel;  // v_perm selector: identity or swap halves
    uint32_t sign[4];  // fp16 sign masks for (element 2t, element 2t+1)
    int8_t sgn8[8];    // +1 / -1 per element (int8 path)
    int part[8];       // partner element
};

__device__ __forceinline__ Variant make_variant(int v)
{
    Variant V;
    const int s = (v & 3) + 1;
    const int sg = v >> 2;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int j = i ^ s;
        const int l = i < j ? i : j;                      // lower index of the pair
        // rank of the pair in ascending-lower-index order (the printed order of P_s)
        const int p = (s == 1) ? (l >> 1) : (s == 4) ? l : ((l & 1) | ((l >> 2) << 1));
        const int eta_neg = (sg >> p) & 1;
        const int upper = i > j;
        V.part[i] = j;
        V.sgn8[i] = (int8_t)((eta_neg ^ upper) ? -1 : 1);
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        V.src[t] = (2 * t) ^ s;
        V.sign[t] = (V.sgn8[2 * t] < 0 ? 0x00008000u : 0u) | (V.sgn8[2 * t + 1] < 0 ? 0x80000000u : 0u);
    }
    V.swapsel = (s & 1) ? 0x01000302u : 0x03020100u;
    return V;
}

template <int BW>
__device__ __forceinline__ void load_block(const uint32_t *__restrict__ packed, int64_t gn, int64_t R,
                                           int64_t g, int lane, uint4 (&d)[(BW == 3) ? 4 : 5])
{
    constexpr int CH = (BW == 3) ? 4 : 5;
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 *base = reinterpret_cast<const u32x4 *>(packed + goq_quad_index(CH, gn, R, g, 0, lane));
#pragma unroll
    for (int h = 0; h < CH; ++h) {
        const u32x4 v = __builtin_nontemporal_load(base + h * GOQ_ROWS);   // streamed once: no reuse
        d[h] = make_uint4(v.x, v.y, v.z, v.w);
    }
}

// byte offset of the variant inside one micro-block position's table (16-byte entries for fp16 x,
// 8-byte entries for int8 x)
template <int BW, int ACT>
__device__ __forceinline__ uint32_t variant_offset(uint32_t w, const uint4 &meta, int m)
{
    constexpr int SH = (ACT == 0) ? 4 : 3;
    if constexpr (BW == 3) {
        // a_0 (bits 6..7) a_1 (14..15) a_2 (22..23) -> contiguous 6-bit index at bits 18..23
        const uint32_t t = w & 0x00C0C0C0u;
        const uint32_t u = __umul24(t, 0x1041u);
        return (u >> (18 - SH)) & (0x3Fu << SH);
    } else {
        const uint32_t pat = (meta.x >> (2 * m)) & 3u;
        const uint32_t sg = ((m < 8 ? meta.y >> (4 * m) : meta.z >> (4 * (m - 8)))) & 15u;
        return (pat | (sg << 2)) << SH;
    }
}

// Stage, for macro-block g, the 64 exchanged copies T x of each of the 16 micro-block positions.
// Thread (wave, lane) writes variant `lane` of positions wave, wave + 4, ...
template <int ACT>
__device__ __forceinline__ void stage_table(unsigned char *tb, const void *x, int g, int wave, int lane,
                                            const Variant &V)
{
#pragma unroll
    for (int j = 0; j < 16 / WAVES; ++j) {
        const int m = wave + WAVES * j;
        if constexpr (ACT == 0) {
            const uint32_t *xm = reinterpret_cast<const uint32_t *>(x) + (int64_t)g * 64 + 4 * m;
            uint4 e;
            e.x = goq_perm(0u, xm[V.src[0] >> 1], V.swapsel) ^ V.sign[0];
            e.y = goq_perm(0u, xm[V.src[1] >> 1], V.swapsel) ^ V.sign[1];
            e.z = goq_perm(0u, xm[V.src[2] >> 1], V.swapsel) ^ V.sign[2];
            e.w = goq_perm(0u, xm[V.src[3] >> 1], V.swapsel) ^ V.sign[3];
            *reinterpret_cast<uint4 *>(tb + (m * 64 + lane) * 16) = e;
        } else {
            const int8_t *xm = reinterpret_cast<const int8_t *>(x) + (int64_t)g * 128 + 8 * m;
            uint32_t lo = 0, hi = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                lo |= (uint32_t)(uint8_t)(int8_t)(V.sgn8[i] * xm[V.part[i]]) << (8 * i);
                hi |= (uint32_t)(uint8_t)(int8_t)(V.sgn8[i + 4] * xm[V.part[i + 4]]) << (8 * i);
            }
            *reinterpret_cast<uint2 *>(tb + (m * 64 + lane) * 8) = make_uint2(lo, hi);
        }
    }
}

// One slab of one row: P1 = x . b1, P2 = (T x) . b1 (H2..H4), then acc += c1 P1 + c2 P2 (H5).
template <int BW, int ACT>
__device__ __forceinline__ void slab(const uint4 (&d)[(BW == 3) ? 4 : 5], const unsigned char *tb,
                                     const void *x, int g, float &acc)
{
    uint32_t cw = 0;
    uint4 meta = make_uint4(0, 0, 0, 0);
    if constexpr (BW == 4) { meta = d[4]; cw = meta.w; }
    if constexpr (ACT == 0) {
        const uint32_t *xs = reinterpret_cast<const uint32_t *>(x) + (int64_t)g * 64;
        float P1 = 0.f, P2 = 0.f;
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            const uint32_t dw[4] = {d[h].x, d[h].y, d[h].z, d[h].w};
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int m = 4 * h + q;
                const uint32_t w = dw[q];
                uint32_t lo, hi;
                goq_decode_bytes<BW, ACT>(w, lo, hi);
                const uint32_t b0 = goq_widen01(lo), b1 = goq_widen23(lo);
                const uint32_t b2 = goq_widen01(hi), b3 = goq_widen23(hi);
                const uint4 e = *reinterpret_cast<const uint4 *>(tb + m * 1024 + variant_offset<BW, ACT>(w, meta, m));
                P1 = goq_dot2(b0, xs[4 * m + 0], P1);
                P1 = goq_dot2(b1, xs[4 * m + 1], P1);
                P1 = goq_dot2(b2, xs[4 * m + 2], P1);
                P1 = goq_dot2(b3, xs[4 * m + 3], P1);
                P2 = goq_dot2(b0, e.x, P2);
                P2 = goq_dot2(b1, e.y, P2);
                P2 = goq_dot2(b2, e.z, P2);
                P2 = goq_dot2(b3, e.w, P2);
                if constexpr (BW == 3) cw = __builtin_amdgcn_alignbit(cw, w, 30);
            }
        }
        const float c1 = __half2float(__ushort_as_half((unsigned short)(cw & 0xffffu)));
        const float c2 = __half2float(__ushort_as_half((unsigned short)(cw >> 16)));
        acc = fmaf(c1, P1, acc);
        acc = fmaf(c2, P2, acc);
    } else {
        const uint32_t *xs = reinterpret_cast<const uint32_t *>(x) + (int64_t)g * 32;
        int P1 = 0, P2 = 0;
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            const uint32_t dw[4] = {d[h].x, d[h].y, d[h].z, d[h].w};
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int m = 4 * h + q;
                const uint32_t w = dw[q];
                uint32_t lo, hi;
                goq_decode_bytes<BW, ACT>(w, lo, hi);
                const uint2 e = *reinterpret_cast<const uint2 *>(tb + m * 512 + variant_offset<BW, ACT>(w, meta, m));
                P1 = goq_dot4(lo, xs[2 * m + 0], P1);
                P1 = goq_dot4(hi, xs[2 * m + 1], P1);
                P2 = goq_dot4(lo, e.x, P2);
                P2 = goq_dot4(hi, e.y, P2);
                if constexpr (BW == 3) cw = __builtin_amdgcn_alignbit(cw, w, 30);
            }
        }
        const float c1 = __half2float(__ushort_as_half((unsigned short)(cw & 0xffffu)));
        const float c2 = __half2float(__ushort_as_half((unsigned short)(cw >> 16)));
        acc = fmaf(c1, (float)P1, acc);
        acc = fmaf(c2, (float)P2, acc);
    }
}

template <int BW, int ACT, int NRB>
__global__ __launch_bounds__(WAVES * 64) void gemv_kernel(GemvArgs a)
{
    constexpr int CH = (BW == 3) ? 4 : 5;
    constexpr int ENTRY = (ACT == 0) ? 16 : 8;                  // bytes per table entry
    constexpr int TBL = 16 * 64 * ENTRY;                        // one macro-block's table
    __shared__ __attribute__((aligned(16))) unsigned char table[2][TBL];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    int pi = 0;
    while (pi + 1 < a.n && (int)blockIdx.x >= a.p[pi + 1].task_begin) ++pi;
    const GemvProblem P = a.p[pi];
    const int task = blockIdx.x - P.task_begin;
    const int gs = task % P.gsplits;
    const int rg = task / P.gsplits;
    const int g0 = gs * P.gper;
    const int g1 = min(g0 + P.gper, P.gn);
    const int Rbase = (rg * WAVES + wave) * NRB;
    const int64_t gn = P.gn;

    const Variant V = make_variant(lane);

    float acc[NRB];
#pragma unroll
    for (int i = 0; i < NRB; ++i) acc[i] = 0.f;

    // two register buffers per row block: one being consumed, one being filled from HBM
    uint4 bufA[NRB][CH], bufB[NRB][CH];
#pragma unroll
    for (int i = 0; i < NRB; ++i)
        if (Rbase + i < P.rbn) load_block<BW>(P.packed, gn, Rbase + i, g0, lane, bufA[i]);

    for (int g = g0; g < g1; g += 2) {
        stage_table<ACT>(table[0], P.x, g, wave, lane, V);
        if (g + 1 < g1) {
#pragma unroll
            for (int i = 0; i < NRB; ++i)
                if (Rbase + i < P.rbn) load_block<BW>(P.packed, gn, Rbase + i, g + 1, lane, bufB[i]);
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < NRB; ++i)
            if (Rbase + i < P.rbn) slab<BW, ACT>(bufA[i], table[0], P.x, g, acc[i]);
        if (g + 1 < g1) {
            stage_table<ACT>(table[1], P.x, g + 1, wave, lane, V);
            if (g + 2 < g1) {
#pragma unroll
                for (int i = 0; i < NRB; ++i)
                    if (Rbase + i < P.rbn) load_block<BW>(P.packed, gn, Rbase + i, g + 2, lane, bufA[i]);
            }
            __syncthreads();
#pragma unroll
            for (int i = 0; i < NRB; ++i)
                if (Rbase + i < P.rbn) slab<BW, ACT>(bufB[i], table[1], P.x, g + 1, acc[i]);
        }
    }

    // ---- reduce + store (H6): the lane owns the row, nothing to reduce inside the wave
    float post = 1.f;
    if constexpr (ACT == 1) post = P.sx[0] * (1.f / (float)(1 << ((1 << (BW - 1)) - 1)));
#pragma unroll
    for (int i = 0; i < NRB; ++i) {
        const int row = (Rbase + i) * GOQ_ROWS + lane;
        if (Rbase + i >= P.rbn || row >= P.out) continue;
        const float v = acc[i] * post;
        if (P.atomic) {
            atomicAdd(reinterpret_cast<float *>(P.y) + row, v);
        } else if (P.ytype == GOQ_F32) {
            reinterpret_cast<float *>(P.y)[row] = v;
        } else {
            reinterpret_cast<__half *>(P.y)[row] = __float2half(v);
        }
    }
}

__global__ __launch_bounds__(256) void zero_kernel(GemvArgs a)
{
    const GemvProblem &P = a.p[blockIdx.y];
    if (!P.atomic) return;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < P.out; i += gridDim.x * blockDim.x)
        reinterpret_cast<float *>(P.y)[i] = 0.f;
}

template <int BW, int ACT>
int launch(hipStream_t st, const GemvArgs &a, int total, bool any_atomic)
{
    constexpr int NRB = NRB_DEFAULT;
    if (any_atomic) hipLaunchKernelGGL(zero_kernel, dim3(16, a.n), dim3(256), 0, st, a);
    hipLaunchKernelGGL((gemv_kernel<BW, ACT, NRB>), dim3(total), dim3(WAVES * 64), 0, st, a);
    return goq_check_launch("goq_gemv");
}

}  // namespace

int goq_launch_gemv(hipStream_t st, int bw, int act, int n, const goq_gemv_desc *descs)
{
    constexpr int NRB = NRB_DEFAULT;
    GemvArgs a;
    a.n = n;
    int total = 0;
    bool any_atomic = false;
    // how finely to split the macro-block range: enough workgroups to fill 256 CUs a few times
    int64_t rowgroups_total = 0;
    for (int i = 0; i < n; ++i)
        rowgroups_total += (goq_row_blocks(descs[i].out) + WAVES * NRB - 1) / (WAVES * NRB);
    for (int i = 0; i < n; ++i) {
        GemvProblem &P = a.p[i];
        P.packed = (const uint32_t *)descs[i].packed;
        P.x = descs[i].x;
        P.sx = descs[i].sx;
        P.y = descs[i].y;
        P.out = (int)descs[i].out;
        P.gn = (int)(descs[i].in / GOQ_N);
        P.ytype = descs[i].ytype;
        P.rbn = (int)goq_row_blocks(descs[i].out);
        const int rgroups = (P.rbn + WAVES * NRB - 1) / (WAVES * NRB);
        int gper = P.gn;
        if (descs[i].ytype == GOQ_F32) {
            // aim at >= 1024 workgroups per launch, at least 2 macro-blocks per task
            const int64_t want_splits = (1024 + rowgroups_total - 1) / rowgroups_total;
            gper = (int)((P.gn + want_splits - 1) / want_splits);
            if (gper < 2) gper = P.gn < 2 ? P.gn : 2;
        }
        P.gper = gper;
        P.gsplits = (P.gn + gper - 1) / gper;
        P.atomic = P.gsplits > 1 ? 1 : 0;
        any_atomic |= P.atomic != 0;
        P.task_begin = total;
        total += rgroups * P.gsplits;
    }
    for (int i = n; i < GOQ_MAX_BATCH; ++i) { a.p[i] = a.p[0]; a.p[i].task_begin = 0x7fffffff; }
    if (bw == 3 && act == GOQ_A16) return launch<3, 0>(st, a, total, any_atomic);
    if (bw == 3 && act == GOQ_A8) return launch<3, 1>(st, a, total, any_atomic);
    if (bw == 4 && act == GOQ_A16) return launch<4, 0>(st, a, total, any_atomic);
    return goq_set_error(GOQ_EUNSUPPORTED, "goq_gemv: bw=4 with int8 activations is not implemented");
}
