// goq_pack / goq_unpack: canonical arrays <-> packed device layout (see goq_layout.h).
// One thread per (row, macro-block).  Off the timed path.
#include <hip/hip_runtime.h>
#include "goq_layout.h"
#include "goq_internal.h"

namespace {

template <int BW>
__global__ __launch_bounds__(256) void pack_kernel(int64_t out, int64_t in,
                                                   const uint8_t *__restrict__ codes,
                                                   const uint8_t *__restrict__ pattern,
                                                   const uint8_t *__restrict__ signs,
                                                   const uint16_t *__restrict__ c1,
                                                   const uint16_t *__restrict__ c2,
                                                   uint32_t *__restrict__ packed)
{
    constexpr int CH = (BW == 3) ? 4 : 5;
    const int64_t gn = in / GOQ_N;
    const int64_t rows = goq_row_blocks(out) * GOQ_ROWS;
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (tid >= rows * gn) return;
    // consecutive threads = consecutive rows of one macro-block column: coalesced writes
    const int64_t g = tid / rows % gn;   // tid = g * rows + row
    const int64_t row = tid % rows;
    const int64_t R = row / GOQ_ROWS;
    const int r = (int)(row % GOQ_ROWS);
    const bool live = row < out;

    uint32_t cw = 0;
    if (live) cw = (uint32_t)c1[row * gn + g] | ((uint32_t)c2[row * gn + g] << 16);
    const uint8_t *cp = codes + row * in + g * GOQ_N;
    const uint8_t *pp = pattern + (row * in + g * GOQ_N) / GOQ_G;
    const uint8_t *sp = signs + (row * in + g * GOQ_N) / GOQ_G;

    uint32_t meta[4] = {0, 0, 0, 0};
    for (int h = 0; h < 4; ++h) {
        uint32_t d[4];
        for (int q = 0; q < 4; ++q) {
            const int m = 4 * h + q;
            uint32_t w = 0;
            uint32_t pat = 0, sg = 0;
            if (live) { pat = pp[m] & 3u; sg = sp[m] & 15u; }
            for (int j = 0; j < 4; ++j) {
                uint32_t lo = goq_zero_code(BW), hi = goq_zero_code(BW);
                if (live) { lo = cp[8 * m + j]; hi = cp[8 * m + j + 4]; }
                if (BW == 3) {
                    w |= ((lo & 7u) | ((hi & 7u) << 3)) << (8 * j);
                } else {
                    w |= ((lo & 15u) | ((hi & 15u) << 4)) << (8 * j);
                }
            }
            if (BW == 3) {
                w |= pat << 6;
                w |= (sg & 3u) << 14;
                w |= (sg >> 2) << 22;
                w |= ((cw >> (30 - 2 * m)) & 3u) << 30;
            } else {
                meta[h] |= (pat | (sg << 2)) << (6 * q);
            }
            d[q] = w;
        }
        uint4 *dst = reinterpret_cast<uint4 *>(packed + goq_quad_index(CH, gn, R, g, h, r));
        *dst = make_uint4(d[0], d[1], d[2], d[3]);
    }
    if (BW == 4) {
        uint4 *dst = reinterpret_cast<uint4 *>(packed + goq_quad_index(CH, gn, R, g, 4, r));
        for (int h = 0; h < 4; ++h) meta[h] |= ((cw >> (8 * h)) & 0xffu) << 24;
        *dst = make_uint4(meta[0], meta[1], meta[2], meta[3]);
    }
}

template <int BW>
__global__ __launch_bounds__(256) void unpack_kernel(int64_t out, int64_t in,
                                                     const uint32_t *__restrict__ packed,
                                                     uint8_t *__restrict__ codes,
                                                     uint8_t *__restrict__ pattern,
                                                     uint8_t *__restrict__ signs,
                                                     uint16_t *__restrict__ c1,
                                                     uint16_t *__restrict__ c2)
{
    constexpr int CH = (BW == 3) ? 4 : 5;
    const int64_t gn = in / GOQ_N;
    const int64_t rows = goq_row_blocks(out) * GOQ_ROWS;
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (tid >= rows * gn) return;
    const int64_t g = tid / rows % gn;
    const int64_t row = tid % rows;
    if (row >= out) return;
    const int64_t R = row / GOQ_ROWS;
    const int r = (int)(row % GOQ_ROWS);

    uint8_t *cp = codes + row * in + g * GOQ_N;
    uint8_t *pp = pattern + (row * in + g * GOQ_N) / GOQ_G;
    uint8_t *sp = signs + (row * in + g * GOQ_N) / GOQ_G;
    uint32_t cw = 0;
    uint4 meta = make_uint4(0, 0, 0, 0);
    if (BW == 4) meta = *reinterpret_cast<const uint4 *>(packed + goq_quad_index(CH, gn, R, g, 4, r));
    for (int h = 0; h < 4; ++h) {
        const uint4 v = *reinterpret_cast<const uint4 *>(packed + goq_quad_index(CH, gn, R, g, h, r));
        const uint32_t d[4] = {v.x, v.y, v.z, v.w};
        for (int q = 0; q < 4; ++q) {
            const int m = 4 * h + q;
            const uint32_t w = d[q];
            for (int j = 0; j < 4; ++j) {
                const uint32_t b = (w >> (8 * j)) & 0xffu;
                if (BW == 3) {
                    cp[8 * m + j] = (uint8_t)(b & 7u);
                    cp[8 * m + j + 4] = (uint8_t)((b >> 3) & 7u);
                } else {
                    cp[8 * m + j] = (uint8_t)(b & 15u);
                    cp[8 * m + j + 4] = (uint8_t)(b >> 4);
                }
            }
            if (BW == 3) {
                pp[m] = (uint8_t)((w >> 6) & 3u);
                sp[m] = (uint8_t)(((w >> 14) & 3u) | (((w >> 22) & 3u) << 2));
                cw = (cw << 2) | (w >> 30);
            } else {
                const uint32_t md = h == 0 ? meta.x : h == 1 ? meta.y : h == 2 ? meta.z : meta.w;
                const uint32_t v = (md >> (6 * q)) & 63u;
                pp[m] = (uint8_t)(v & 3u);
                sp[m] = (uint8_t)(v >> 2);
            }
        }
    }
    if (BW == 4) cw = (meta.x >> 24) | ((meta.y >> 24) << 8) | ((meta.z >> 24) << 16) | ((meta.w >> 24) << 24);
    c1[row * gn + g] = (uint16_t)(cw & 0xffffu);
    c2[row * gn + g] = (uint16_t)(cw >> 16);
}

}  // namespace

int goq_launch_pack(hipStream_t st, int bw, int64_t out, int64_t in, const uint8_t *codes,
                    const uint8_t *pattern, const uint8_t *signs, const uint16_t *c1,
                    const uint16_t *c2, void *packed)
{
    const int64_t n = goq_row_blocks(out) * GOQ_ROWS * (in / GOQ_N);
    const unsigned grid = (unsigned)((n + 255) / 256);
    if (bw == 3)
        hipLaunchKernelGGL(pack_kernel<3>, dim3(grid), dim3(256), 0, st, out, in, codes, pattern, signs,
                           c1, c2, (uint32_t *)packed);
    else
        hipLaunchKernelGGL(pack_kernel<4>, dim3(grid), dim3(256), 0, st, out, in, codes, pattern, signs,
                           c1, c2, (uint32_t *)packed);
    return goq_check_launch("goq_pack");
}

int goq_launch_unpack(hipStream_t st, int bw, int64_t out, int64_t in, const void *packed,
                      uint8_t *codes, uint8_t *pattern, uint8_t *signs, uint16_t *c1, uint16_t *c2)
{
    const int64_t n = goq_row_blocks(out) * GOQ_ROWS * (in / GOQ_N);
    const unsigned grid = (unsigned)((n + 255) / 256);
    if (bw == 3)
        hipLaunchKernelGGL(unpack_kernel<3>, dim3(grid), dim3(256), 0, st, out, in,
                           (const uint32_t *)packed, codes, pattern, signs, c1, c2);
    else
        hipLaunchKernelGGL(unpack_kernel<4>, dim3(grid), dim3(256), 0, st, out, in,
                           (const uint32_t *)packed, codes, pattern, signs, c1, c2);
    return goq_check_launch("goq_unpack");
}
