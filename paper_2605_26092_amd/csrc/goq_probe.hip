// goq_mfma_probe: measures the two properties of v_mfma_scale_f32_16x16x128_f8f6f4 that the
// batch-1 kernels (goq_gemv.hip) build their exactness on, so that a change of hardware,
// microcode or compiler is caught by name instead of by a drifting result:
//
//   depth       With E5M2 operands the instruction adds the products of 8 consecutive k on a
//               fixed-point grid below the largest product of the 8.  The kernels hand x over as
//               3-bit digits against powers of two 2^0 .. 2^-7, so a group's products span at
//               most 10 binary places below the leading bit of the largest one; the grid must
//               keep them all.  Measured: the largest s for which 1 * 1 + 2^-s (k = 0 and k = 1 of
//               one group) is returned exactly.
//   membership  Which of the 128 k of an A row the E8M0 scale supplied by lane (row, Q) applies
//               to.  The digit tables give every block of 32 activations that share a scale its
//               own exponent; they assume: k-groups 2 (Q % 2) and 2 (Q % 2) + 1, bytes
//               16 (Q / 2) .. 16 (Q / 2) + 15 of each.
//
// One wavefront, 16 + 4 * 128 matrix instructions.  Operand layout as in goq_gemv.hip: lane
// (row = l % 16, k-group = l / 16) holds the 32 bytes k = 32 (l / 16) .. + 31 of A row / B
// column l % 16; lane (c, q) receives D[4 q + i][c], i = 0..3.
#include <hip/hip_runtime.h>
#include "goq_internal.h"

namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));

__device__ __forceinline__ unsigned char e5m2_pot(int e) { return (unsigned char)((e + 15) << 2); }   // 2^e

// register vector with byte `pos` (0..31) set to v, everything else zero
__device__ __forceinline__ v8i one_byte(int pos, unsigned char v)
{
    v8i r = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < 8; ++i)
        if (i == (pos >> 2)) r[i] = (int)((uint32_t)v << (8 * (pos & 3)));
    return r;
}

__global__ __launch_bounds__(64) void mfma_probe_kernel(int32_t *report)
{
    const int lane = threadIdx.x;
    const int c = lane & 15, q = lane >> 4;
    const v4f zero = {0.f, 0.f, 0.f, 0.f};

    // depth: A[0][0] = B[0][0] = 1; A[0][1] = 2^-(s / 2), B[1][0] = 2^-(s - s / 2)
    int depth = 0;
    for (int s = 1; s <= 16; ++s) {
        v8i A = {0, 0, 0, 0, 0, 0, 0, 0}, B = {0, 0, 0, 0, 0, 0, 0, 0};
        if (lane == 0) {
            A[0] = (int)((uint32_t)e5m2_pot(0) | ((uint32_t)e5m2_pot(-(s / 2)) << 8));
            B[0] = (int)((uint32_t)e5m2_pot(0) | ((uint32_t)e5m2_pot(-(s - s / 2)) << 8));
        }
        const v4f D = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(A, B, zero, 1, 1, 0, 127, 0, 127);
        // Lane 0 holds D[0][0].  The broadcast makes every lane a consumer of the result: the
        // matrix instruction must run with all lanes active, and the compiler may otherwise sink
        // it into the lane-0-only code that stores the report.
        const float d00 = __shfl(D[0], 0);
        if (d00 == 1.0f + __builtin_ldexpf(1.0f, -s)) depth = s;
    }
    if (lane == 0) report[0] = depth;

    // membership: A row 0 = 1 for all k, B column 0 = 1 at one k; lane (0, Q) supplies the scale
    // 2^1, every other lane 2^0: D[0][0] = 2 exactly when k is covered by that lane's scale
    for (int Q = 0; Q < 4; ++Q) {
        uint32_t mask[4] = {0u, 0u, 0u, 0u};
        for (int k = 0; k < 128; ++k) {
            v8i A = {0, 0, 0, 0, 0, 0, 0, 0};
            if (c == 0)
#pragma unroll
                for (int i = 0; i < 8; ++i) A[i] = 0x3C3C3C3C;
            v8i B = {0, 0, 0, 0, 0, 0, 0, 0};
            if (c == 0 && q == (k >> 5)) B = one_byte(k & 31, e5m2_pot(0));
            const int sa = 127 + ((c == 0 && q == Q) ? 1 : 0);
            const v4f D = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(A, B, zero, 1, 1, 0, sa, 0, 127);
            const float d00 = __shfl(D[0], 0);
            if (d00 == 2.0f) mask[k >> 5] |= 1u << (k & 31);
        }
        if (lane == 0)
            for (int i = 0; i < 4; ++i) report[1 + 4 * Q + i] = (int32_t)mask[i];
    }
}

// ---- measured ceilings (bench.py reports them beside the nominal peaks) -------------------------
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef int v4i __attribute__((ext_vector_type(4)));

// Pure read stream: every workgroup reads one contiguous piece of the buffer, 8 x 16 bytes per lane
// in flight (what the batch-1 kernel keeps in flight), nontemporal, nothing else.
__global__ __launch_bounds__(512) void read_probe_kernel(const u32x4 *__restrict__ p, size_t n16, uint32_t *sink)
{
    const size_t per = n16 / gridDim.x;
    const u32x4 *q = p + per * blockIdx.x;
    uint32_t acc = 0;
    size_t i = threadIdx.x;
    for (; i + 7 * 512 < per; i += 8 * 512) {
        u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(q + i + u * 512);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (; i < per; i += 512) {
        const u32x4 v = __builtin_nontemporal_load(q + i);
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    if (acc == 0x9E3779B9u) sink[0] = acc;                     // keeps the loads alive
}

// Pure matrix-instruction loop: four independent accumulator chains per wavefront, operands in
// registers, nothing else.  KIND 0: v_mfma_f32_32x32x16_f16, 1: v_mfma_i32_32x32x32_i8,
// 2: v_mfma_scale_f32_16x16x128_f8f6f4 with E5M2 operands.
template <int KIND>
__global__ __launch_bounds__(256) void mfma_rate_kernel(int iters, float *sink)
{
    const int lane = threadIdx.x & 63;
    float out = 0.f;
    if constexpr (KIND == 0) {
        v8h a, b;
        for (int i = 0; i < 8; ++i) { a[i] = (_Float16)(lane * 0.001f + i); b[i] = (_Float16)(1.0f - i * 0.01f); }
        v16f c[4] = {};
        for (int it = 0; it < iters; ++it)
#pragma unroll
            for (int k = 0; k < 4; ++k) c[k] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c[k], 0, 0, 0);
        for (int k = 0; k < 4; ++k) out += c[k][0];
    } else if constexpr (KIND == 1) {
        v4i a = {lane, lane + 1, lane + 2, lane + 3}, b = {0x01010101, 0x02020202, 0x01010101, 0x03030303};
        v16i c[4] = {};
        for (int it = 0; it < iters; ++it)
#pragma unroll
            for (int k = 0; k < 4; ++k) c[k] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c[k], 0, 0, 0);
        for (int k = 0; k < 4; ++k) out += (float)c[k][0];
    } else {
        v8i a, b;
        for (int i = 0; i < 8; ++i) { a[i] = 0x3C383C34; b[i] = 0x3C3C3834; }
        v4f c[4] = {};
        for (int it = 0; it < iters; ++it)
#pragma unroll
            for (int k = 0; k < 4; ++k)
                c[k] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c[k], 1, 1, 0, 127, 0, 127);
        for (int k = 0; k < 4; ++k) out += c[k][0];
    }
    if (out == 123.456f) sink[0] = out;
}

}  // namespace

int goq_launch_read_probe(hipStream_t st, const void *buf, size_t bytes, uint32_t *sink)
{
    hipLaunchKernelGGL(read_probe_kernel, dim3(512), dim3(512), 0, st, reinterpret_cast<const u32x4 *>(buf), bytes / 16, sink);
    return goq_check_launch("goq_read_probe");
}

// workgroups x 4 wavefronts x iters x 4 matrix instructions; *ops receives the multiply-add
// operations (2 per MAC) of the launch
int goq_launch_mfma_rate_probe(hipStream_t st, int kind, int workgroups, int iters, float *sink, double *ops)
{
    const double per = kind == 0 ? 2.0 * 32 * 32 * 16 : kind == 1 ? 2.0 * 32 * 32 * 32 : 2.0 * 16 * 16 * 128;
    *ops = per * 4.0 * iters * 4.0 * workgroups;
    if (kind == 0) hipLaunchKernelGGL(mfma_rate_kernel<0>, dim3(workgroups), dim3(256), 0, st, iters, sink);
    else if (kind == 1) hipLaunchKernelGGL(mfma_rate_kernel<1>, dim3(workgroups), dim3(256), 0, st, iters, sink);
    else hipLaunchKernelGGL(mfma_rate_kernel<2>, dim3(workgroups), dim3(256), 0, st, iters, sink);
    return goq_check_launch("goq_mfma_rate_probe");
}

int goq_launch_mfma_probe(hipStream_t st, int32_t *report)
{
    hipLaunchKernelGGL(mfma_probe_kernel, dim3(1), dim3(64), 0, st, report);
    return goq_check_launch("goq_mfma_probe");
}
