// Internal (non-ABI) declarations shared by the library's translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/goq.h"

// records the message of a failed launch / HIP call; returns GOQ_OK or GOQ_EHIP
int goq_check_launch(const char *what);
int goq_set_error(int code, const char *fmt, ...);

int goq_launch_pack(hipStream_t st, int bw, int64_t out, int64_t in, const uint8_t *codes,
                    const uint8_t *pattern, const uint8_t *signs, const uint16_t *c1,
                    const uint16_t *c2, void *packed);
int goq_launch_unpack(hipStream_t st, int bw, int64_t out, int64_t in, const void *packed,
                      uint8_t *codes, uint8_t *pattern, uint8_t *signs, uint16_t *c1, uint16_t *c2);
int goq_launch_quantize(hipStream_t st, int bw, int64_t out, int64_t in, const uint16_t *w, uint8_t *codes,
                        uint8_t *pattern, uint8_t *signs, uint16_t *c1, uint16_t *c2);
int goq_launch_ref(hipStream_t st, int bw, int64_t tokens, int64_t out, int64_t in, const uint16_t *w,
                   const uint8_t *codes, const uint8_t *pattern, const uint8_t *signs, const uint16_t *X,
                   double lambda, void *workspace, double *craw, uint16_t *c1, uint16_t *c2);
// workspace: caller-owned (goq_gemv_workspace_size() bytes), or NULL for the library's static
// region of this stream
int goq_launch_gemv(hipStream_t st, int bw, int act, int n, const goq_gemv_desc *descs, void *workspace);
size_t goq_gemv_workspace_size();
int goq_launch_gemv_workspace_init(hipStream_t st, void *workspace);
size_t goq_gemv_stream_table_size(int n);
int goq_gemv_stream_build_table(int bw, int act, int n, const goq_gemv_desc *descs, void *table);
int goq_launch_gemv_stream(hipStream_t st, const void *table_host, const void *table_dev, void *workspace);
void goq_gemv_set_kernel(int kernel);
int goq_gemv_plan_launch(int n, const goq_gemv_desc *descs, int *kernel, int *workgroups);
int goq_launch_gemm_folded(hipStream_t st, int bw, int64_t tokens, int64_t out, int64_t in, const void *packed,
                           const void *X, void *Y, int ytype);
int goq_launch_gemm(hipStream_t st, int bw, int act, int n, const goq_gemm_desc *descs);
int goq_launch_mfma_probe(hipStream_t st, int32_t *report);
int goq_launch_read_probe(hipStream_t st, const void *buf, size_t bytes, uint32_t *sink);
int goq_launch_mfma_rate_probe(hipStream_t st, int kind, int workgroups, int iters, float *sink, double *ops);
