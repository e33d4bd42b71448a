// goq_gemm: many-token dual-PoT layer output, Y[tokens][out] = X[tokens][in] * W^T (Eq. 4).
//
// The contraction is dense (hundreds to thousands of tokens), so it runs on the matrix cores:
//   A16: v_mfma_f32_32x32x16_f16, operands fp16, fp32 accumulation
//   A8 : v_mfma_i32_32x32x32_i8,  operands int8, exact int32 accumulation (bw = 3)
//   A8 with bw = 4: b * 2^7 reaches +128, which is no int8.  The int8 activations are widened to
//        fp16 on their way into LDS and the fp16 instruction is used: int8 values and powers of
//        two down to 2^-7 are exact in fp16, every product is exact, and a slab sum needs at most
//        22 bits, so the fp32 accumulators hold the exact integers (in units of 2^-7).
// The weight side is the MFMA B operand.  Its register layout -- lane (n = lane % 32,
// kg = lane / 32) holds 8 (fp16) or 16 (int8) consecutive k of output channel n -- is one (two)
// 8-weight micro-block(s) of one row, which is the unit the packed layout stores in a dword.  A
// lane loads two 16-byte quads of its row per slab (micro-blocks 8 kg .. 8 kg + 7), decodes a
// micro-block in registers with the byte LUT (H2), and rebuilds the residual basis b2 of the same
// micro-block in registers too (H4): a byte permute by i xor s plus sign flips, both looked up by
// the 6 metadata bits in a 1 KiB LDS table built at kernel start.  No decoded weight ever goes
// through memory.  The order of k inside a slab is free as long as both operands agree: k-step t
// takes micro-block 8 kg + t of lane group kg.  The activation tile of the slab is staged in LDS
// (XOR-swizzled 16-byte pieces against bank conflicts) and read as the MFMA A operand.
//
// Tiling: workgroup = 4 wavefronts, tile 64 tokens x 128 outputs; each wavefront owns 64 tokens x
// 32 outputs = two MFMA tiles of 32 x 32, with three accumulator sets: the slab partials P1, P2
// (restarted every slab by feeding C = 0 to the slab's first MFMA) and the output Y.  That fits
// three wavefronts per SIMD.  Measured on this chip with a probe of the same instruction mix:
// vector-ALU instructions hide only to a small extent behind matrix instructions, whatever the
// program order (about five per 32x32x16 instruction; every further one costs nearly its full
// four cycles), so the rate is set by vector-ALU and LDS instructions per matrix instruction.
// The 32x32x16 instruction halves both per flop compared with 16x16x32 at the same tile.  A
// 128-token tile (one wavefront per SIMD) spreads the decode over more matrix instructions but
// needs the partials in accumulator registers, which the rescale can only read through copies:
// it measured slower.
// Pipeline: activations of slab g + 2 are requested (global_load_lds, straight into one of three
// LDS buffers) and the weights of slab g + 1 (registers) at the start of slab g; inside a slab
// every k-step's MFMAs run on operands prepared during the previous k-step; one barrier per slab.
// One launch covers up to GOQ_MAX_BATCH layers (goq_gemm_batch): their tiles form one grid, the
// layers with the deepest rows first, so that a block of matrices has one tail, not one per matrix.
// Coefficient rescale (H5) once per slab: Y += c1[n,g] * P1 + c2[n,g] * P2 in fp32, after the
// slab's MFMAs; a lane needs one (c1, c2) pair because every accumulator register of a lane
// belongs to the same output channel.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <type_traits>
#include "goq_layout.h"
#include "goq_decode.h"
#include "goq_internal.h"

namespace {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x16 __attribute__((ext_vector_type(16)));

#ifndef GOQ_GEMM_TM
#define GOQ_GEMM_TM 64
#endif
constexpr int TM = GOQ_GEMM_TM;   // tokens per workgroup tile
constexpr int TN = 128;       // outputs per workgroup tile
constexpr int WN = 32;        // outputs per wavefront
constexpr int MS = TM / 32;   // MFMA tiles along tokens per wavefront

struct GemmArgs {
    const uint32_t *packed;
    const void *X;
    const float *sx;
    void *Y;
    int32_t *partials;
    int tokens, out, in, gn, rbn, ytype;
};

// The problems of one launch: workgroups first[i] .. first[i + 1] - 1 own the tiles of problem i
// (unused problems start at INT_MAX).
struct GemmBatch {
    int first[GOQ_MAX_BATCH];
    GemmArgs p[GOQ_MAX_BATCH];
};

// LDS address of the exchange table entry of a micro-block: vt + 16 * (pattern | signs << 2)
template <int BW>
__device__ __forceinline__ uint32_t exchange_address(uint32_t w, const uint4 &meta, int m, uint32_t vt)
{
    if constexpr (BW == 3) {
        // a_0 (bits 6..7), a_1 (14..15), a_2 (22..23) -> contiguous 6-bit index at bits 18..23
        const uint32_t u = __umul24(w & 0x00C0C0C0u, 0x1041u);
        return vt + ((u >> 14) & 0x3F0u);
    } else {
        // meta.x, meta.y: the metadata dwords of this lane's two chunks (6 bits per micro-block)
        const uint32_t md = m < 4 ? meta.x : meta.y;
        return vt + (((md >> (6 * (m & 3))) & 63u) << 4);
    }
}

// Decode one micro-block dword into the bytes of b1 and b2 (elements 0..3 in lo, 4..7 in hi).
template <int BW, int ACT>
__device__ __forceinline__ void decode_pair(uint32_t w, const uint4 &meta, int m, uint32_t vt,
                                            uint32_t &b1lo, uint32_t &b1hi, uint32_t &b2lo, uint32_t &b2hi)
{
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 e = *reinterpret_cast<const __attribute__((address_space(3))) u32x4 *>(exchange_address<BW>(w, meta, m, vt));
    if constexpr (ACT == 0) {
        // fp16 high bytes: exchange the decoded bytes, flip sign bits
        goq_decode_bytes<BW, ACT>(w, b1lo, b1hi);
        b2lo = goq_perm(b1hi, b1lo, e.x) ^ e.z;
        b2hi = goq_perm(b1hi, b1lo, e.y) ^ e.w;
    } else {
        // int8 (bw = 3): a sign flip is no bit flip, so the CODES are exchanged and looked up in
        // the lattice and in the negated lattice; the mask picks per byte
        static_assert(BW == 3, "int8 operands exist for bw = 3 only");
        const uint32_t clo = w & 0x07070707u;
        const uint32_t chi = (w >> 3) & 0x07070707u;
        constexpr uint32_t PL = GoqLut<3, 1>::lo, PH = GoqLut<3, 1>::hi;
        constexpr uint32_t NL = 0x00FEFCF8u, NH = 0x01020408u;       // -(b * 8) for codes 0..7
        b1lo = goq_perm(PH, PL, clo);
        b1hi = goq_perm(PH, PL, chi);
        const uint32_t xlo = goq_perm(chi, clo, e.x);
        const uint32_t xhi = goq_perm(chi, clo, e.y);
        b2lo = (goq_perm(NH, NL, xlo) & e.z) | (goq_perm(PH, PL, xlo) & ~e.z);
        b2hi = (goq_perm(NH, NL, xhi) & e.w) | (goq_perm(PH, PL, xhi) & ~e.w);
    }
}

__device__ __forceinline__ f16x8 widen8(uint32_t lo, uint32_t hi)
{
    const uint4 v = make_uint4(goq_widen01(lo), goq_widen23(lo), goq_widen01(hi), goq_widen23(hi));
    return __builtin_bit_cast(f16x8, v);
}

#ifndef GOQ_GEMM_MINWAVES
#define GOQ_GEMM_MINWAVES 2
#endif
// FOLD (fp16 activations only) is the ablation of the method's two-basis product: the decoded
// operands are combined in registers to the fp16 weight c1 b1 + c2 b2 (two packed fp16 operations
// per register) and ONE matrix instruction per k-step and tile accumulates straight into Y.  Half
// the matrix instructions and no rescale, but the operand is no power of two any more: every
// weight is rounded to fp16 (2^-11 relative), which the two-basis path avoids.
template <int BW, int ACT, bool PART, bool FOLD = false>
__global__ __launch_bounds__(256, GOQ_GEMM_MINWAVES) void gemm_kernel(GemmBatch batch)
{
    int pi = 0;
#pragma unroll
    for (int i = 1; i < GOQ_MAX_BATCH; ++i) pi += ((int)blockIdx.x >= batch.first[i]) ? 1 : 0;
    pi = __builtin_amdgcn_readfirstlane(pi);
    const GemmArgs &a = batch.p[pi];
    const int tile = (int)blockIdx.x - batch.first[pi];
    static_assert(!FOLD || (ACT == 0 && !PART), "the folded product exists for fp16 activations only");
    constexpr int CH = (BW == 3) ? 4 : 5;
    // ACT: 0 fp16 x; 1 int8 x, int8 MFMA; 2 int8 x widened to fp16; 3 packed int4 x unpacked to
    // int8, int8 MFMA; 4 packed int4 x widened to fp16; 5 packed int6 x unpacked to int8, int8
    // MFMA; 6 packed int6 x widened to fp16; 7 packed int3 x unpacked to int8, int8 MFMA; 8 packed
    // int3 x widened to fp16.  2..8 stage x through registers.
    constexpr bool F16 = (ACT == 0 || ACT == 2 || ACT == 4 || ACT == 6 || ACT == 8);   // fp16 MFMA
    constexpr bool REGSTAGE = (ACT >= 2);
    constexpr bool X4 = (ACT == 3 || ACT == 4);                    // two activations per byte
    constexpr bool X6 = (ACT == 5 || ACT == 6);                    // four activations per three bytes
    constexpr bool X3 = (ACT == 7 || ACT == 8);                    // eight activations per three bytes
    constexpr bool I8OUT = (ACT == 3 || ACT == 5 || ACT == 7);     // staged as int8 (else widened to fp16)
    constexpr int WACT = F16 ? 0 : 1;                  // how the weights are decoded
    constexpr int XB = F16 ? 2 : 1;                    // bytes per activation in LDS
    constexpr int ROWB = GOQ_N * XB;                   // LDS row stride (XOR-swizzled, not padded)
    constexpr int KSTEPS = F16 ? 8 : 4;                // MFMA k-steps per slab (16 / 32 k each)
    constexpr int NBUF = 3;                            // activation slabs resident in LDS
    using AccT = typename std::conditional<F16, f32x16, i32x16>::type;
    using OpT = typename std::conditional<F16, f16x8, i32x4>::type;          // one MFMA operand

    __shared__ __attribute__((aligned(16))) unsigned char xsb[NBUF][TM * ROWB];
    __shared__ __attribute__((aligned(16))) unsigned char xtab[64 * 16];        // exchange table

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ln = lane & 31;     // MFMA column (output channel) / A row (token)
    const int kg = lane >> 5;     // k-group

    const int mtiles = (a.tokens + TM - 1) / TM;
    const int mt = tile % mtiles;
    const int nt = tile / mtiles;
    const int m0 = mt * TM;
    const int n0 = nt * TN + wave * WN;

    if (tid < 64) *reinterpret_cast<uint4 *>(xtab + tid * 16) = goq_exchange_entry<(WACT == 0 ? 0x80u : 0xFFu)>(tid);
    const uint32_t vt = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)xtab;

    f32x16 Yacc[MS];
#pragma unroll
    for (int i = 0; i < MS; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) Yacc[i][v] = 0.f;

    // the two quads this lane reads per slab: row n0 + ln, chunks 2 kg and 2 kg + 1 (micro-blocks
    // 8 kg .. 8 kg + 7).  Rows past the last row block are redirected to the last one (their
    // outputs are never stored), so that every lane always issues the same loads.
    int wrow = n0 + ln;
    wrow = (wrow / GOQ_ROWS) < a.rbn ? wrow : a.rbn * GOQ_ROWS - 1;
    const uint32_t *wq = a.packed + goq_quad_index(CH, a.gn, wrow / GOQ_ROWS, 0, 2 * kg, wrow % GOQ_ROWS);
    const int64_t gstride = (int64_t)CH * GOQ_ROWS * 4;     // dwords between macro-blocks

    struct Weights {
        uint4 q0, q1;     // micro-blocks 8 kg .. 8 kg + 3 and 8 kg + 4 .. 8 kg + 7
        uint4 meta;       // bw = 4: metadata dwords of the two chunks (x, y), coefficient word (w)
    };
    auto load_weights = [&](int g, Weights &w) {
        const uint32_t *p = wq + g * gstride;
        w.q0 = *reinterpret_cast<const uint4 *>(p);
        w.q1 = *reinterpret_cast<const uint4 *>(p + GOQ_ROWS * 4);
        w.meta = make_uint4(0, 0, 0, 0);
        if constexpr (BW == 4) {
            // chunk 4 of the same row: one metadata dword per chunk, each with a byte of the
            // coefficient word on top
            const uint4 mq = *reinterpret_cast<const uint4 *>(p + (4 - 2 * kg) * GOQ_ROWS * 4);
            const uint32_t cw = goq_perm(mq.y, mq.x, 0x0c0c0703u) | goq_perm(mq.w, mq.z, 0x07030c0cu);
            w.meta = make_uint4(kg ? mq.z : mq.x, kg ? mq.w : mq.y, 0, cw);
        }
    };
    auto word_of = [](const Weights &w, int t) {
        return t == 0 ? w.q0.x : t == 1 ? w.q0.y : t == 2 ? w.q0.z : t == 3 ? w.q0.w
             : t == 4 ? w.q1.x : t == 5 ? w.q1.y : t == 6 ? w.q1.z : w.q1.w;
    };

    // Activation slab -> LDS without passing through registers (global_load_lds_dwordx4): each
    // instruction fills 64 consecutive 16-byte LDS slots, one per lane, from per-lane addresses.
    // Slot (row, cs) holds k-piece cs ^ f(row): the XOR swizzle makes the 16 rows a quarter of an
    // MFMA A operand read touches fall into 16 different bank groups (row stride 256 / 128 bytes).
    // The per-thread byte offsets (inside the token tile) of the pieces a thread requests are
    // constant over the slabs: a slab's request is one uniform base plus these 32-bit offsets.
    constexpr int PIECES = TM * GOQ_N * XB / 16;
    constexpr int PER_ROW = GOQ_N * XB / 16;
    constexpr int NP = PIECES / 256;
    auto swz = [](int row) { return F16 ? (row & 15) : ((row >> 1) & 7); };
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
    auto stage_x = [&](int g) {          // exactly NP vector-memory instructions
        const unsigned char *base = xtile + (int64_t)g * GOQ_N * XB;
        unsigned char *buf = xsb[g % NBUF];
#pragma unroll
        for (int i = 0; i < NP; ++i)
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void *)(base + xoff[i]),
                (__attribute__((address_space(3))) void *)(buf + (i * 256 + wave * 64) * 16), 16, 0, 0);
    };
    // Register staging (ACT >= 2): integer activations pass through registers and are unpacked /
    // widened on their way into LDS.  A thread moves NPS 16-byte pieces per slab; a piece holds
    // 16 int8 or 32 int4 activations and becomes OUTP 16-byte pieces of the LDS row.
    // int -> fp16 without a conversion instruction: 0x6400 | u is the fp16 number 1024 + u.
    // (int6 / int3: a source piece is 24 / 12 bytes = 32 activations = two 16-byte LDS pieces of
    // int8, fetched as three 8-byte / 4-byte loads)
    constexpr int SRCROW = X4 ? GOQ_N / 2 : X6 ? GOQ_N * 3 / 4 : X3 ? GOQ_N * 3 / 8 : GOQ_N;   // bytes of a slab row in memory
    constexpr int SRCP = X6 ? 24 : X3 ? 12 : 16;                   // bytes of a source piece
    constexpr int SPR = SRCROW / SRCP;                             // source pieces per row
    constexpr int NPS = (TM * SPR + 255) / 256;
    constexpr int NQ = X6 ? 2 : 1;                                 // uint4 registers per source piece (int6: 6 of 8 words used)
    constexpr int OUTP = ROWB / SPR / 16;                          // LDS pieces per source piece
    const int64_t xpitch = X4 ? a.in / 2 : X6 ? a.in / 4 * 3 : X3 ? a.in / 8 * 3 : a.in;   // bytes of a token row in memory
    uint32_t soff[NPS];
#pragma unroll
    for (int i = 0; i < NPS; ++i) {
        const int S = i * 256 + tid;
        int m = m0 + S / SPR;
        m = m < a.tokens ? m : a.tokens - 1;
        soff[i] = (uint32_t)(m - m0) * (uint32_t)xpitch + (S % SPR) * SRCP;
    }
    auto fetch_x = [&](int g, uint4 (&r)[NPS * NQ]) {
        const unsigned char *base = reinterpret_cast<const unsigned char *>(a.X) + (int64_t)m0 * xpitch + (int64_t)g * SRCROW;
#pragma unroll
        for (int i = 0; i < NPS; ++i) {
            if constexpr (X6) {
                const uint2 a0 = *reinterpret_cast<const uint2 *>(base + soff[i]);
                const uint2 a1 = *reinterpret_cast<const uint2 *>(base + soff[i] + 8);
                const uint2 a2 = *reinterpret_cast<const uint2 *>(base + soff[i] + 16);
                r[2 * i] = make_uint4(a0.x, a0.y, a1.x, a1.y);
                r[2 * i + 1] = make_uint4(a2.x, a2.y, 0u, 0u);
            } else if constexpr (X3) {
                const uint32_t *p3 = reinterpret_cast<const uint32_t *>(base + soff[i]);
                r[i] = make_uint4(p3[0], p3[1], p3[2], 0u);
            } else {
                r[i] = *reinterpret_cast<const uint4 *>(base + soff[i]);
            }
        }
    };
    // four int8 -> two registers of two fp16
    auto widen_i8 = [](uint32_t d, uint32_t &h0, uint32_t &h1) {
        const goq_half2 off = {(_Float16)1152.f, (_Float16)1152.f};
        const uint32_t u = d ^ 0x80808080u;                        // x + 128
        h0 = __builtin_bit_cast(uint32_t, __builtin_bit_cast(goq_half2, goq_perm(0x64646464u, u, 0x04010400u)) - off);
        h1 = __builtin_bit_cast(uint32_t, __builtin_bit_cast(goq_half2, goq_perm(0x64646464u, u, 0x04030402u)) - off);
    };
    // eight int4 (element i in nibble i) -> two registers of four int8
    auto unpack_i4 = [](uint32_t d, uint32_t &b0, uint32_t &b1) {
        auto sext = [](uint32_t v) {      // per byte: low nibble, two's complement -> int8
            return ((((v ^ 0x08080808u) | 0x80808080u) - 0x08080808u) ^ 0x80808080u);
        };
        const uint32_t ev = sext(d & 0x0F0F0F0Fu);                 // elements 0, 2, 4, 6
        const uint32_t od = sext((d >> 4) & 0x0F0F0F0Fu);          // elements 1, 3, 5, 7
        b0 = goq_perm(od, ev, 0x05010400u);                        // elements 0, 1, 2, 3
        b1 = goq_perm(od, ev, 0x07030602u);                        // elements 4, 5, 6, 7
    };
    // four int6 (24 bits, element i in bits 6 i .. 6 i + 5) -> one register of four int8
    auto unpack_i6 = [](uint32_t v) {
        const uint32_t b = (v & 0x3Fu) | ((v << 2) & 0x3F00u) | ((v << 4) & 0x3F0000u) | ((v << 6) & 0x3F000000u);
        return ((((b ^ 0x20202020u) | 0x80808080u) - 0x20202020u) ^ 0x80808080u);   // per byte: 6 -> 8 bits, signed
    };
    // eight int3 (24 bits, element i in bits 3 i .. 3 i + 2) -> two registers of four int8
    auto unpack_i3 = [](uint32_t v, uint32_t &b0, uint32_t &b1) {
        auto spread = [](uint32_t t) {
            const uint32_t b = (t & 0x7u) | ((t << 5) & 0x700u) | ((t << 10) & 0x70000u) | ((t << 15) & 0x7000000u);
            return ((((b ^ 0x04040404u) | 0x80808080u) - 0x04040404u) ^ 0x80808080u);   // per byte: 3 -> 8 bits, signed
        };
        b0 = spread(v);
        b1 = spread(v >> 12);
    };
    auto write_x = [&](int g, const uint4 (&r)[NPS * NQ]) {
        unsigned char *buf = xsb[g % NBUF];
#pragma unroll
        for (int i = 0; i < NPS; ++i) {
            const int S = i * 256 + tid;
            const int row = S / SPR, cs = S % SPR;
            if (NPS * 256 > TM * SPR && S >= TM * SPR) continue;
            uint32_t o[16];                                        // the source piece's LDS pieces
            if constexpr (X6) {
                // 6 dwords = 8 groups of 24 bits; group j starts at bit 24 j
                const uint32_t w[6] = {r[i * 2].x, r[i * 2].y, r[i * 2].z, r[i * 2].w, r[i * 2 + 1].x, r[i * 2 + 1].y};
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int dwi = (24 * j) >> 5, sh = (24 * j) & 31;
                    const uint32_t v = sh == 0 ? w[dwi] : sh == 8 ? (w[dwi] >> 8) : __builtin_amdgcn_alignbit(w[dwi + 1], w[dwi], sh);
                    const uint32_t b = unpack_i6(v);
                    if constexpr (I8OUT) o[j] = b;
                    else widen_i8(b, o[2 * j], o[2 * j + 1]);
                }
            } else if constexpr (X3) {
                // 3 dwords = 4 groups of 24 bits = 32 activations
                const uint32_t w[3] = {r[i].x, r[i].y, r[i].z};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int dwi = (24 * j) >> 5, sh = (24 * j) & 31;
                    const uint32_t v = sh == 0 ? w[dwi] : sh == 8 ? (w[dwi] >> 8) : __builtin_amdgcn_alignbit(w[dwi + 1], w[dwi], sh);
                    uint32_t b0, b1;
                    unpack_i3(v, b0, b1);
                    if constexpr (I8OUT) { o[2 * j] = b0; o[2 * j + 1] = b1; }
                    else { widen_i8(b0, o[4 * j], o[4 * j + 1]); widen_i8(b1, o[4 * j + 2], o[4 * j + 3]); }
                }
            }
            const uint32_t d[4] = {r[i * NQ].x, r[i * NQ].y, r[i * NQ].z, r[i * NQ].w};
            if constexpr (X6 || X3) {
                (void)d;
            } else if constexpr (ACT == 2) {
#pragma unroll
                for (int k = 0; k < 4; ++k) widen_i8(d[k], o[2 * k], o[2 * k + 1]);
            } else if constexpr (ACT == 3) {
#pragma unroll
                for (int k = 0; k < 4; ++k) unpack_i4(d[k], o[2 * k], o[2 * k + 1]);
            } else {
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    uint32_t b0, b1;
                    unpack_i4(d[k], b0, b1);
                    widen_i8(b0, o[4 * k], o[4 * k + 1]);
                    widen_i8(b1, o[4 * k + 2], o[4 * k + 3]);
                }
            }
            unsigned char *dst = buf + row * ROWB;
#pragma unroll
            for (int q = 0; q < OUTP; ++q)
                *reinterpret_cast<uint4 *>(dst + (((OUTP * cs + q) ^ swz(row)) * 16)) =
                    make_uint4(o[4 * q], o[4 * q + 1], o[4 * q + 2], o[4 * q + 3]);
        }
    };
    // decoded B operands (b1 and b2) of k-step t of a slab (H2, H4); cf (FOLD): the slab's
    // coefficients (c1, c2) as fp16, both halves of a register alike
    f16x8 cf1, cf2;
    auto decode_step = [&](const Weights &w, int t, OpT &B1, OpT &B2) {
        if constexpr (F16) {
            uint32_t l1, h1, l2, h2;
            decode_pair<BW, WACT>(word_of(w, t), w.meta, t, vt, l1, h1, l2, h2);
            B1 = widen8(l1, h1);
            B2 = widen8(l2, h2);
            if constexpr (FOLD) B1 = cf1 * B1 + cf2 * B2;
        } else {
            uint32_t l1, h1, l2, h2, l3, h3, l4, h4;
            decode_pair<BW, WACT>(word_of(w, 2 * t), w.meta, 2 * t, vt, l1, h1, l2, h2);
            decode_pair<BW, WACT>(word_of(w, 2 * t + 1), w.meta, 2 * t + 1, vt, l3, h3, l4, h4);
            B1 = i32x4{(int)l1, (int)h1, (int)l3, (int)h3};
            B2 = i32x4{(int)l2, (int)h2, (int)l4, (int)h4};
        }
    };
    // A operands of k-step t: token 32 i + ln, the 16-byte piece that holds the k of micro-block(s)
    // 8 kg + MPK t .. of the slab
    auto read_a = [&](const unsigned char *xs, int t, OpT (&A)[MS]) {
        const int piece = KSTEPS * kg + t;
#pragma unroll
        for (int i = 0; i < MS; ++i)
            A[i] = *reinterpret_cast<const OpT *>(xs + (32 * i + ln) * ROWB + ((piece ^ swz(32 * i + ln)) * 16));
    };
    // coefficient pair of this lane's output channel
    auto coefficients = [&](const Weights &w, float &c1, float &c2) {
        uint32_t cw;
        if constexpr (BW == 3) {
            // a lane's 8 dwords carry 16 of the 32 bits (lane group 0: c2, lane group 1: c1)
            uint32_t part = 0;
#pragma unroll
            for (int t = 0; t < 8; ++t) part = __builtin_amdgcn_alignbit(part, word_of(w, t), 30);
            const uint32_t other = __shfl_xor(part, 32);
            cw = kg ? (part | (other << 16)) : (other | (part << 16));
        } else {
            cw = w.meta.w;
        }
        c1 = __half2float(__ushort_as_half((unsigned short)(cw & 0xffffu)));
        c2 = __half2float(__ushort_as_half((unsigned short)(cw >> 16)));
    };

    // Prologue: slabs 0 and 1 are requested and waited for.
    Weights wd, wn;
    uint4 xr[NPS * NQ];
    load_weights(0, wd);
    if constexpr (REGSTAGE) {
        fetch_x(0, xr);
        write_x(0, xr);
        if (a.gn > 1) {
            fetch_x(1, xr);
            write_x(1, xr);
        }
    } else {
        stage_x(0);
        if (a.gn > 1) stage_x(1);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    auto fold_coefficients = [&](const Weights &w) {
        float c1, c2;
        coefficients(w, c1, c2);
#pragma unroll
        for (int k = 0; k < 8; ++k) { cf1[k] = (_Float16)c1; cf2[k] = (_Float16)c2; }
    };
    OpT B1, B2, A[MS];
    if constexpr (FOLD) fold_coefficients(wd);
    decode_step(wd, 0, B1, B2);
    read_a(xsb[0], 0, A);

    for (int g = 0; g < a.gn; ++g) {
        const unsigned char *xs = xsb[g % NBUF];
        const bool more2 = g + 2 < a.gn;
        // (the weight request is unconditional, on a clamped slab index: past the last slab the
        // result is not used; the activation request comes last so that the wait below is exact)
        load_weights(min(g + 1, a.gn - 1), wn);
        if constexpr (REGSTAGE) {
            if (more2) fetch_x(g + 2, xr);
        } else {
            if (more2) stage_x(g + 2);
        }

        float c1 = 0.f, c2 = 0.f;
        if constexpr (!FOLD) coefficients(wd, c1, c2);

        AccT P1[MS], P2[MS];
#pragma unroll
        for (int t = 0; t < KSTEPS; ++t) {
            const OpT B1c = B1, B2c = B2;
            OpT Ac[MS];
#pragma unroll
            for (int i = 0; i < MS; ++i) Ac[i] = A[i];
            if (t + 1 < KSTEPS) {
                decode_step(wd, t + 1, B1, B2);
                read_a(xs, t + 1, A);
            } else {
                // last k-step of the slab.  Everything older than this slab's activation request
                // has landed once at most NP vector-memory operations are outstanding (they return
                // in order): slab g + 1's activations, requested a slab ago, and its weights.
                if constexpr (REGSTAGE) {
                    // (register path: slab g + 2 is written here; its buffer was last read before
                    // the previous slab's barrier, and it is first read after the next one)
                    if (more2) write_x(g + 2, xr);
                } else {
                    if (more2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NP) : "memory");
                    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                }
                __syncthreads();
                if constexpr (FOLD) fold_coefficients(wn);
                decode_step(wn, 0, B1, B2);
                read_a(xsb[min(g + 1, a.gn - 1) % NBUF], 0, A);
            }
#pragma unroll
            for (int i = 0; i < MS; ++i) {
                AccT z;
#pragma unroll
                for (int v = 0; v < 16; ++v) z[v] = 0;
                if constexpr (FOLD) {
                    Yacc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(Ac[i], B1c, Yacc[i], 0, 0, 0);
                } else if constexpr (F16) {
                    P1[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(Ac[i], B1c, t == 0 ? z : P1[i], 0, 0, 0);
                    P2[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(Ac[i], B2c, t == 0 ? z : P2[i], 0, 0, 0);
                } else {
                    P1[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(Ac[i], B1c, t == 0 ? z : P1[i], 0, 0, 0);
                    P2[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(Ac[i], B2c, t == 0 ? z : P2[i], 0, 0, 0);
                }
            }
        }
        // ---- coefficient rescale, once per slab, outside the dot-product loop (H5).  Register v
        //      of a 32 x 32 tile: token 8 (v / 4) + 4 kg + v % 4, output ln.
#pragma unroll
        for (int i = 0; i < MS; ++i) {
            if constexpr (!FOLD) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    Yacc[i][v] = fmaf(c1, (float)P1[i][v], Yacc[i][v]);
                    Yacc[i][v] = fmaf(c2, (float)P2[i][v], Yacc[i][v]);
                }
            }
            if constexpr (PART) {
                // exact int32 slab partials [tokens][out][in/128][2] (verification output)
                const int n = n0 + ln;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = m0 + 32 * i + 8 * (v / 4) + 4 * kg + (v % 4);
                    if (m < a.tokens && n < a.out && a.partials)
                        *reinterpret_cast<int2 *>(a.partials + (((int64_t)m * a.out + n) * a.gn + g) * 2) =
                            F16 ? make_int2((int)((float)P1[i][v] * (float)(1 << ((1 << (BW - 1)) - 1))),
                                            (int)((float)P2[i][v] * (float)(1 << ((1 << (BW - 1)) - 1))))
                                : make_int2((int)P1[i][v], (int)P2[i][v]);
                }
            }
        }
        wd = wn;
    }

    // ---- store the tile (H6)
    const int n = n0 + ln;
#pragma unroll
    for (int i = 0; i < MS; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int m = m0 + 32 * i + 8 * (v / 4) + 4 * kg + (v % 4);
            if (m >= a.tokens || n >= a.out) continue;
            float y = Yacc[i][v];
            if constexpr (ACT != 0 && !F16) y *= a.sx[m] * (1.f / (float)(1 << ((1 << (BW - 1)) - 1)));
            if constexpr (ACT != 0 && F16) y *= a.sx[m];
            if (a.ytype == GOQ_F32) reinterpret_cast<float *>(a.Y)[(int64_t)m * a.out + n] = y;
            else reinterpret_cast<__half *>(a.Y)[(int64_t)m * a.out + n] = __float2half(y);
        }
}

// tiles of the problems, in launch order; returns the grid size (0: too large).  The problems with
// the deepest rows go first: their tiles take longest, and the launch should end with short ones.
int64_t lay_out(GemmBatch &b, int n)
{
    for (int i = 1; i < n; ++i)
        for (int j = i; j > 0 && b.p[j].gn > b.p[j - 1].gn; --j) {
            const GemmArgs t = b.p[j];
            b.p[j] = b.p[j - 1];
            b.p[j - 1] = t;
        }
    int64_t tiles = 0;
    for (int i = 0; i < GOQ_MAX_BATCH; ++i) {
        if (i >= n) { b.first[i] = 0x7fffffff; b.p[i] = b.p[0]; continue; }
        b.first[i] = (int)tiles;
        tiles += (int64_t)((b.p[i].tokens + TM - 1) / TM) * ((b.p[i].out + TN - 1) / TN);
        if (tiles > 0x3fffffff) return 0;
    }
    return tiles;
}

template <int BW, int ACT>
int launch(hipStream_t st, GemmBatch &b, int n)
{
    const int64_t grid = lay_out(b, n);
    if (!grid) return goq_set_error(GOQ_ESHAPE, "goq_gemm: too much work for one launch");
    bool part = false;
    for (int i = 0; i < n; ++i) part = part || b.p[i].partials;
    if (ACT != 0 && part)
        hipLaunchKernelGGL((gemm_kernel<BW, ACT, (ACT != 0)>), dim3((unsigned)grid), dim3(256), 0, st, b);
    else
        hipLaunchKernelGGL((gemm_kernel<BW, ACT, false>), dim3((unsigned)grid), dim3(256), 0, st, b);
    return goq_check_launch("goq_gemm");
}

template <int BW>
int launch_folded(hipStream_t st, GemmBatch &b, int n)
{
    const int64_t grid = lay_out(b, n);
    if (!grid) return goq_set_error(GOQ_ESHAPE, "goq_gemm_folded: too much work for one launch");
    hipLaunchKernelGGL((gemm_kernel<BW, 0, false, true>), dim3((unsigned)grid), dim3(256), 0, st, b);
    return goq_check_launch("goq_gemm_folded");
}

GemmArgs make_args(const goq_gemm_desc &d)
{
    GemmArgs a;
    a.packed = (const uint32_t *)d.packed;
    a.X = d.X;
    a.sx = d.sx;
    a.Y = d.Y;
    a.partials = d.partials;
    a.tokens = (int)d.tokens;
    a.out = (int)d.out;
    a.in = (int)d.in;
    a.gn = (int)(d.in / GOQ_N);
    a.rbn = (int)goq_row_blocks(d.out);
    a.ytype = d.ytype;
    return a;
}

}  // namespace

int goq_launch_gemm_folded(hipStream_t st, int bw, int64_t tokens, int64_t out, int64_t in, const void *packed,
                           const void *X, void *Y, int ytype)
{
    goq_gemm_desc d;
    d.tokens = tokens; d.out = out; d.in = in; d.packed = packed; d.X = X; d.sx = nullptr; d.Y = Y;
    d.ytype = ytype; d.partials = nullptr;
    GemmBatch b;
    b.p[0] = make_args(d);
    return bw == 3 ? launch_folded<3>(st, b, 1) : launch_folded<4>(st, b, 1);
}

int goq_launch_gemm(hipStream_t st, int bw, int act, int n, const goq_gemm_desc *descs)
{
    GemmBatch b;
    for (int i = 0; i < n; ++i) b.p[i] = make_args(descs[i]);
    if (bw == 3 && act == GOQ_A16) return launch<3, 0>(st, b, n);
    if (bw == 3 && act == GOQ_A8) return launch<3, 1>(st, b, n);
    if (bw == 4 && act == GOQ_A16) return launch<4, 0>(st, b, n);
    if (bw == 4 && act == GOQ_A8) return launch<4, 2>(st, b, n);
    if (bw == 3 && act == GOQ_A4) return launch<3, 3>(st, b, n);
    if (bw == 4 && act == GOQ_A4) return launch<4, 4>(st, b, n);
    if (bw == 3 && act == GOQ_A6) return launch<3, 5>(st, b, n);
    if (bw == 4 && act == GOQ_A6) return launch<4, 6>(st, b, n);
    if (bw == 3 && act == GOQ_A3) return launch<3, 7>(st, b, n);
    return launch<4, 8>(st, b, n);
}
