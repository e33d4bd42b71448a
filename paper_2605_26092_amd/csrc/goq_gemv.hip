// goq_gemv / goq_gemv_batch: batch-1 dual-PoT layer output (Eq. 4 with one token).
//
// Work decomposition.  The unit of work is (row group, macro-block g): a ROW GROUP is 8 row
// blocks of 64 output channels, one row block per wavefront of a 512-thread workgroup, one row
// per lane.  The lane that owns row r loads that row's whole macro-block (CH coalesced 16-byte
// quads, see goq_layout.h) and keeps both slab dot products P1, P2 and the coefficient pair in
// its own registers, so a slab needs no cross-lane traffic; the coefficient rescale (H5) is two
// FMAs per 128 weights, after the slab's dot products.
//
// All units of all problems of a launch form one linear sequence (problem, row group, g) that
// is cut into equal contiguous pieces, one per workgroup (two workgroups per CU), so the weight
// stream of a workgroup is one long prefetched sequence and every workgroup gets the same
// amount of work whatever the matrix shapes are.  Where a piece ends inside a row group the
// partial y is combined with fp32 atomic adds (y zeroed by a fill kernel first); when fp16
// output is requested the pieces are aligned to row groups instead and y is stored directly.
//
// Residual basis without rebuilding it: x . b2 = b1 . (T x), where T is the signed exchange
// of the micro-block (Theorem 1).  T depends only on the micro-block's 6 metadata bits, and
// x is shared by all rows, so the workgroup stages, per macro-block, the 64 possible T x for
// each of the 16 micro-block positions in LDS (16 KiB for fp16 x) and a lane fetches the
// variant its metadata selects with one 16-byte LDS read.  P1 uses x itself, which is uniform
// across the wavefront (scalar registers).  Per micro-block a lane then spends: 2 byte-LUT
// permutes (decode), 4 byte shuffles (widen to fp16), 8 two-term fp16 dot products.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <type_traits>
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
    int rgroups;     // row groups
    int begin;       // first piece-space index of this problem (units, or row groups when !split)
};

struct GemvArgs {
    int n;
    int split;       // 1: pieces are unit ranges, combine with atomics; 0: pieces are whole row groups
    int total;       // size of the piece space
    GemvProblem p[GOQ_MAX_BATCH];
};

#ifndef GOQ_EXP_WAVES
#define GOQ_EXP_WAVES 8
#endif
constexpr int WAVES = GOQ_EXP_WAVES;   // wavefronts (= row blocks) per workgroup

// x is read-only for the whole kernel: reading it through the constant address space lets the
// wave-uniform chunk of x live in scalar registers (s_load) instead of 64 identical lanes.
typedef __attribute__((address_space(4))) uint32_t goq_const_u32;

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
#ifdef GOQ_EXP_NONT
        const u32x4 v = base[h * GOQ_ROWS];
#else
        const u32x4 v = __builtin_nontemporal_load(base + h * GOQ_ROWS);   // streamed once: no reuse
#endif
        d[h] = make_uint4(v.x, v.y, v.z, v.w);
    }
}

// byte offset of the variant inside one micro-block position's table (16-byte entries for fp16 x,
// 8-byte entries for int8 x)
template <int BW, int ACT>
__device__ __forceinline__ uint32_t variant_offset(uint32_t w, const uint4 &meta, int m)
{
    constexpr int SH = (ACT == 0) ? 4 : 3;
#ifdef GOQ_EXP_UNIFORM_LDS
    return 0;
#endif
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

// Staging of the exchanged copies T x of macro-block g, split in two so that the loads of x can
// be issued a whole slab before they are needed.  Thread (wave, lane) produces variant `lane`
// of micro-block positions wave and wave + 8.
template <int ACT>
struct StageRegs {
    uint32_t v[16 / WAVES][(ACT == 0) ? 4 : 8];
};

template <int ACT>
__device__ __forceinline__ void stage_load(StageRegs<ACT> &sr, const void *x, int g, int wave, const Variant &V)
{
#pragma unroll
    for (int j = 0; j < 16 / WAVES; ++j) {
        const int m = wave + WAVES * j;
        if constexpr (ACT == 0) {
            const uint32_t *xm = reinterpret_cast<const uint32_t *>(x) + (int64_t)g * 64 + 4 * m;
#pragma unroll
            for (int t = 0; t < 4; ++t) sr.v[j][t] = xm[V.src[t] >> 1];
        } else {
            const int8_t *xm = reinterpret_cast<const int8_t *>(x) + (int64_t)g * 128 + 8 * m;
#pragma unroll
            for (int i = 0; i < 8; ++i) sr.v[j][i] = (uint32_t)(int32_t)xm[V.part[i]];
        }
    }
}

template <int ACT>
__device__ __forceinline__ void stage_write(unsigned char *tb, const StageRegs<ACT> &sr, int wave, int lane,
                                            const Variant &V)
{
#pragma unroll
    for (int j = 0; j < 16 / WAVES; ++j) {
        const int m = wave + WAVES * j;
        if constexpr (ACT == 0) {
            uint4 e;
            e.x = goq_perm(0u, sr.v[j][0], V.swapsel) ^ V.sign[0];
            e.y = goq_perm(0u, sr.v[j][1], V.swapsel) ^ V.sign[1];
            e.z = goq_perm(0u, sr.v[j][2], V.swapsel) ^ V.sign[2];
            e.w = goq_perm(0u, sr.v[j][3], V.swapsel) ^ V.sign[3];
            *reinterpret_cast<uint4 *>(tb + (m * 64 + lane) * 16) = e;
        } else {
            uint32_t lo = 0, hi = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                lo |= (uint32_t)(uint8_t)(int8_t)(V.sgn8[i] * (int32_t)sr.v[j][i]) << (8 * i);
                hi |= (uint32_t)(uint8_t)(int8_t)(V.sgn8[i + 4] * (int32_t)sr.v[j][i + 4]) << (8 * i);
            }
            *reinterpret_cast<uint2 *>(tb + (m * 64 + lane) * 8) = make_uint2(lo, hi);
        }
    }
}

// Operands of one pipeline stage = one chunk of 4 micro-blocks of one row: the chunk's x
// (uniform, scalar registers) and the 4 exchanged copies the lane's metadata selects (LDS).
template <int ACT>
struct StageOps {
    uint32_t xs[(ACT == 0) ? 16 : 8];
    uint4 e[(ACT == 0) ? 4 : 2];
};

template <int BW, int ACT>
__device__ __forceinline__ void fetch_stage(StageOps<ACT> &o, const uint4 &d, const uint4 &meta, int h,
                                            const unsigned char *tb, const void *x, int g)
{
    const uint32_t dw[4] = {d.x, d.y, d.z, d.w};
    if constexpr (ACT == 0) {
        const goq_const_u32 *xs = reinterpret_cast<const goq_const_u32 *>((uintptr_t)x) + (int64_t)g * 64 + 16 * h;
#pragma unroll
        for (int i = 0; i < 16; ++i) o.xs[i] = xs[i];
#pragma unroll
        for (int q = 0; q < 4; ++q)
            o.e[q] = *reinterpret_cast<const uint4 *>(tb + (4 * h + q) * 1024 +
                                                     variant_offset<BW, ACT>(dw[q], meta, 4 * h + q));
    } else {
        const goq_const_u32 *xs = reinterpret_cast<const goq_const_u32 *>((uintptr_t)x) + (int64_t)g * 32 + 8 * h;
#pragma unroll
        for (int i = 0; i < 8; ++i) o.xs[i] = xs[i];
        uint2 t[4];
#pragma unroll
        for (int q = 0; q < 4; ++q)
            t[q] = *reinterpret_cast<const uint2 *>(tb + (4 * h + q) * 512 +
                                                    variant_offset<BW, ACT>(dw[q], meta, 4 * h + q));
        o.e[0] = make_uint4(t[0].x, t[0].y, t[1].x, t[1].y);
        o.e[1] = make_uint4(t[2].x, t[2].y, t[3].x, t[3].y);
    }
}

// H2..H4 for one chunk: decode, P1 += x . b1, P2 += (T x) . b1; gathers the coefficient bits.
template <int BW, int ACT, typename AccT>
__device__ __forceinline__ void compute_stage(const StageOps<ACT> &o, uint4 &d, AccT &P1, AccT &P2,
                                              uint32_t &cw)
{
    // pin the chunk's decode to this pipeline stage (in place, no copies): without it the compiler
    // hoists the pure decode arithmetic of all 16 micro-blocks to the top of the slab and runs out
    // of registers
    asm volatile("" : "+v"(d.x), "+v"(d.y), "+v"(d.z), "+v"(d.w));
    const uint32_t dw[4] = {d.x, d.y, d.z, d.w};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const uint32_t w = dw[q];
        uint32_t lo, hi;
        goq_decode_bytes<BW, ACT>(w, lo, hi);
        if constexpr (ACT == 0) {
            const uint32_t b0 = goq_widen01(lo), b1 = goq_widen23(lo);
            const uint32_t b2 = goq_widen01(hi), b3 = goq_widen23(hi);
            P1 = goq_dot2(b0, o.xs[4 * q + 0], P1);
            P1 = goq_dot2(b1, o.xs[4 * q + 1], P1);
            P1 = goq_dot2(b2, o.xs[4 * q + 2], P1);
            P1 = goq_dot2(b3, o.xs[4 * q + 3], P1);
#ifndef GOQ_EXP_NOP2
            P2 = goq_dot2(b0, o.e[q].x, P2);
            P2 = goq_dot2(b1, o.e[q].y, P2);
            P2 = goq_dot2(b2, o.e[q].z, P2);
            P2 = goq_dot2(b3, o.e[q].w, P2);
#endif
        } else {
            const uint32_t ex = (q & 1) ? o.e[q >> 1].z : o.e[q >> 1].x;
            const uint32_t ey = (q & 1) ? o.e[q >> 1].w : o.e[q >> 1].y;
            P1 = goq_dot4(lo, o.xs[2 * q + 0], P1);
            P1 = goq_dot4(hi, o.xs[2 * q + 1], P1);
            P2 = goq_dot4(lo, ex, P2);
            P2 = goq_dot4(hi, ey, P2);
        }
        if constexpr (BW == 3) cw = __builtin_amdgcn_alignbit(cw, w, 30);
    }
}

// One slab of one row, software pipelined over its 4 chunks: the operands of chunk h+1 are
// requested (scalar load of x, LDS reads of the exchanged copies) before chunk h is computed.
// Ends with the coefficient rescale (H5): acc += c1 P1 + c2 P2.
template <int BW, int ACT>
__device__ __forceinline__ void slab(uint4 (&d)[(BW == 3) ? 4 : 5], const unsigned char *tb,
                                     const void *x, int g, float &acc)
{
    using AccT = typename std::conditional<ACT == 0, float, int>::type;
    uint32_t cw = 0;
    uint4 meta = make_uint4(0, 0, 0, 0);
    if constexpr (BW == 4) { meta = d[4]; cw = meta.w; }
    AccT P1 = 0, P2 = 0;
    // Scalar loads return out of order, so any use of one waits for ALL outstanding scalar and
    // LDS requests.  Each stage therefore first touches its own operands (the wait lands here),
    // then requests the next stage's, then computes.
#define GOQ_TOUCH(o) asm volatile("" ::"s"((o).xs[0]), "v"((o).e[0].x))
    StageOps<ACT> o0, o1;
    fetch_stage<BW, ACT>(o0, d[0], meta, 0, tb, x, g);
    GOQ_TOUCH(o0);
    fetch_stage<BW, ACT>(o1, d[1], meta, 1, tb, x, g);
    __builtin_amdgcn_sched_barrier(0);
    compute_stage<BW, ACT>(o0, d[0], P1, P2, cw);
    __builtin_amdgcn_sched_barrier(0);
    GOQ_TOUCH(o1);
    fetch_stage<BW, ACT>(o0, d[2], meta, 2, tb, x, g);
    __builtin_amdgcn_sched_barrier(0);
    compute_stage<BW, ACT>(o1, d[1], P1, P2, cw);
    __builtin_amdgcn_sched_barrier(0);
    GOQ_TOUCH(o0);
    fetch_stage<BW, ACT>(o1, d[3], meta, 3, tb, x, g);
    __builtin_amdgcn_sched_barrier(0);
    compute_stage<BW, ACT>(o0, d[2], P1, P2, cw);
    __builtin_amdgcn_sched_barrier(0);
    GOQ_TOUCH(o1);
    compute_stage<BW, ACT>(o1, d[3], P1, P2, cw);
#undef GOQ_TOUCH
    const float c1 = __half2float(__ushort_as_half((unsigned short)(cw & 0xffffu)));
    const float c2 = __half2float(__ushort_as_half((unsigned short)(cw >> 16)));
    acc = fmaf(c1, (float)P1, acc);
    acc = fmaf(c2, (float)P2, acc);
}

// Position in the linear unit sequence.
struct Cursor {
    int pi, rg, g;
};

__device__ __forceinline__ Cursor locate(const GemvArgs &a, int idx)
{
    Cursor c;
    if (idx >= a.total) { c.pi = a.n; c.rg = 0; c.g = 0; return c; }
    int pi = 0;
    while (pi + 1 < a.n && idx >= a.p[pi + 1].begin) ++pi;
    const int local = idx - a.p[pi].begin;
    c.pi = pi;
    if (a.split) { c.rg = local / a.p[pi].gn; c.g = local % a.p[pi].gn; }
    else { c.rg = local; c.g = 0; }
    // the divisions run on the vector ALU: move the (uniform) results back to scalar registers
    // so that all later cursor and address arithmetic is scalar
    c.rg = __builtin_amdgcn_readfirstlane(c.rg);
    c.g = __builtin_amdgcn_readfirstlane(c.g);
    return c;
}

__device__ __forceinline__ bool same(const Cursor &a, const Cursor &b)
{
    return a.pi == b.pi && a.rg == b.rg && a.g == b.g;
}

// The few fields of a problem the streaming loop needs (kept in scalar registers); the output
// side (y, out, sx, ytype) is re-read from the kernel arguments only when a row group is flushed.
struct Stream {
    const uint32_t *packed;
    const void *x;
    int gn, rbn, rgroups;
};

__device__ __forceinline__ Stream stream_of(const GemvArgs &a, int pi)
{
    Stream s;
    const uint64_t pk = (uint64_t)a.p[pi].packed, px = (uint64_t)a.p[pi].x;
    s.packed = (const uint32_t *)(((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(pk >> 32)) << 32) |
                                  (uint32_t)__builtin_amdgcn_readfirstlane((int)pk));
    s.x = (const void *)(((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(px >> 32)) << 32) |
                         (uint32_t)__builtin_amdgcn_readfirstlane((int)px));
    s.gn = __builtin_amdgcn_readfirstlane(a.p[pi].gn);
    s.rbn = __builtin_amdgcn_readfirstlane(a.p[pi].rbn);
    s.rgroups = __builtin_amdgcn_readfirstlane(a.p[pi].rgroups);
    return s;
}

// One unit: prefetch the next unit's weights and x, compute this unit's slab, publish the next
// unit's table.  Invariant on entry: tcur holds this unit's exchanged copies and every wave has
// passed the barrier after they were written.  Returns false after the piece's last unit.
template <int BW, int ACT>
__device__ __forceinline__ bool gemv_unit(const GemvArgs &a, Cursor &cur, const Cursor &end, Stream &S,
                                          uint4 (&bcur)[(BW == 3) ? 4 : 5], uint4 (&bnxt)[(BW == 3) ? 4 : 5],
                                          unsigned char *tcur, unsigned char *tnxt, StageRegs<ACT> &sr,
                                          const Variant &V, float &acc, int wave, int lane)
{
    Cursor nxt = cur;
    if (++nxt.g == S.gn) { nxt.g = 0; if (++nxt.rg == S.rgroups) { nxt.rg = 0; ++nxt.pi; } }
    // the cursor is wave-uniform: keep it (and everything derived from it) in scalar registers
    nxt.pi = __builtin_amdgcn_readfirstlane(nxt.pi);
    nxt.rg = __builtin_amdgcn_readfirstlane(nxt.rg);
    nxt.g = __builtin_amdgcn_readfirstlane(nxt.g);
    const bool more = !same(nxt, end);
    const bool new_problem = more && nxt.pi != cur.pi;
    Stream Sn = S;
    if (new_problem) Sn = stream_of(a, nxt.pi);
    if (more) {
        const int Rn = nxt.rg * WAVES + wave;
#ifndef GOQ_EXP_NOMEM
        if (Rn < Sn.rbn) load_block<BW>(Sn.packed, Sn.gn, Rn, nxt.g, lane, bnxt);
#endif
        stage_load<ACT>(sr, Sn.x, nxt.g, wave, V);
    }
    const int R = cur.rg * WAVES + wave;
#ifdef GOQ_EXP_READONLY
    if (R < S.rbn) {
        uint32_t t = 0;
        for (int h = 0; h < ((BW == 3) ? 4 : 5); ++h) t ^= bcur[h].x ^ bcur[h].y ^ bcur[h].z ^ bcur[h].w;
        acc += (float)t;
    }
#else
    if (R < S.rbn) slab<BW, ACT>(bcur, tcur, S.x, cur.g, acc);
#endif
    if (!more || nxt.rg != cur.rg || new_problem) {
        // ---- reduce + store (H6): the lane owns the row, nothing to reduce inside the wave
        const GemvProblem &P = a.p[cur.pi];
        float v = acc;
        if constexpr (ACT == 1) v *= P.sx[0] * (1.f / (float)(1 << ((1 << (BW - 1)) - 1)));
        const int row = R * GOQ_ROWS + lane;
        if (R < S.rbn && row < P.out) {
            if (a.split) atomicAdd(reinterpret_cast<float *>(P.y) + row, v);
            else if (P.ytype == GOQ_F32) reinterpret_cast<float *>(P.y)[row] = v;
            else reinterpret_cast<__half *>(P.y)[row] = __float2half(v);
        }
        acc = 0.f;
    }
    if (more) {
        stage_write<ACT>(tnxt, sr, wave, lane, V);
#ifndef GOQ_EXP_NOBARRIER
        __syncthreads();
#endif
    }
    cur = nxt;
    S = Sn;
    return more;
}

template <int BW, int ACT>
__global__ __launch_bounds__(WAVES * 64) void gemv_kernel(GemvArgs a)
{
    constexpr int CH = (BW == 3) ? 4 : 5;
    constexpr int ENTRY = (ACT == 0) ? 16 : 8;                  // bytes per table entry
    constexpr int TBL = 16 * 64 * ENTRY;                        // one macro-block's table
    __shared__ __attribute__((aligned(16))) unsigned char table[2][TBL];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    // this workgroup's piece [i0, i1) of the piece space
    const int64_t nwg = gridDim.x;
    const int i0 = __builtin_amdgcn_readfirstlane((int)((int64_t)a.total * blockIdx.x / nwg));
    const int i1 = __builtin_amdgcn_readfirstlane((int)((int64_t)a.total * (blockIdx.x + 1) / nwg));
    if (i0 >= i1) return;
    Cursor cur = locate(a, i0);
    const Cursor end = locate(a, i1);
    Stream S = stream_of(a, cur.pi);

    const Variant V = make_variant(lane);
    float acc = 0.f;
    uint4 bufA[CH], bufB[CH];
#ifdef GOQ_EXP_NOMEM
    for (int h = 0; h < CH; ++h)
        bufA[h] = bufB[h] = make_uint4(lane * 0x01234567u, lane * 0x89abcdefu + h, lane ^ 0x5a5a5a5au, h * 0x11111111u);
#endif
    StageRegs<ACT> sr;

    {
        const int R = cur.rg * WAVES + wave;
#ifndef GOQ_EXP_NOMEM
        if (R < S.rbn) load_block<BW>(S.packed, S.gn, R, cur.g, lane, bufA);
#endif
        stage_load<ACT>(sr, S.x, cur.g, wave, V);
        stage_write<ACT>(table[0], sr, wave, lane, V);
        __syncthreads();
    }
    while (true) {
        if (!gemv_unit<BW, ACT>(a, cur, end, S, bufA, bufB, table[0], table[1], sr, V, acc, wave, lane)) break;
        if (!gemv_unit<BW, ACT>(a, cur, end, S, bufB, bufA, table[1], table[0], sr, V, acc, wave, lane)) break;
    }
}

__global__ __launch_bounds__(256) void zero_kernel(GemvArgs a)
{
    const GemvProblem &P = a.p[blockIdx.y];
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < P.out; i += gridDim.x * blockDim.x)
        reinterpret_cast<float *>(P.y)[i] = 0.f;
}

template <int BW, int ACT>
int launch(hipStream_t st, const GemvArgs &a, int nwg)
{
    if (a.split) hipLaunchKernelGGL(zero_kernel, dim3(8, a.n), dim3(256), 0, st, a);
    hipLaunchKernelGGL((gemv_kernel<BW, ACT>), dim3(nwg), dim3(WAVES * 64), 0, st, a);
    return goq_check_launch("goq_gemv");
}

}  // namespace

int goq_launch_gemv(hipStream_t st, int bw, int act, int n, const goq_gemv_desc *descs)
{
    GemvArgs a;
    a.n = n;
    a.split = 1;
    for (int i = 0; i < n; ++i)
        if (descs[i].ytype != GOQ_F32) a.split = 0;     // fp16 y cannot take atomic partial sums
    int total = 0;
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
        P.rgroups = (P.rbn + WAVES - 1) / WAVES;
        P.begin = total;
        total += a.split ? P.rgroups * P.gn : P.rgroups;
    }
    for (int i = n; i < GOQ_MAX_BATCH; ++i) { a.p[i] = a.p[0]; a.p[i].begin = 0x7fffffff; }
    a.total = total;
    // two 512-thread workgroups per CU fill the register file (4 wavefronts per SIMD)
    int nwg = 2 * 256;
#ifdef GOQ_EXP_NWG
    nwg = GOQ_EXP_NWG;
#endif
    if (nwg > total) nwg = total;
    if (bw == 3 && act == GOQ_A16) return launch<3, 0>(st, a, nwg);
    if (bw == 3 && act == GOQ_A8) return launch<3, 1>(st, a, nwg);
    if (bw == 4 && act == GOQ_A16) return launch<4, 0>(st, a, nwg);
    return goq_set_error(GOQ_EUNSUPPORTED, "goq_gemv: bw=4 with int8 activations is not implemented");
}
