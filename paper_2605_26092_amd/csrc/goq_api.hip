// C ABI entry points (include/goq.h): host-side validation, then dispatch to the launchers.
#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdio.h>
#include "goq_internal.h"
#include "goq_layout.h"

namespace {
thread_local char g_err[512] = "";
inline bool misaligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }
}  // namespace

int goq_set_error(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int goq_check_launch(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return goq_set_error(GOQ_EHIP, "%s: %s", what, hipGetErrorString(e));
    return GOQ_OK;
}

static int check_shape(const char *fn, int bw, int64_t out, int64_t in)
{
    if (bw != 3 && bw != 4) return goq_set_error(GOQ_EINVAL, "%s: bw must be 3 or 4 (got %d)", fn, bw);
    if (out <= 0 || out > (1 << 24)) return goq_set_error(GOQ_ESHAPE, "%s: out = %lld out of range", fn, (long long)out);
    if (in <= 0 || in % GOQ_N != 0 || in > (1 << 24))
        return goq_set_error(GOQ_ESHAPE, "%s: in = %lld must be a positive multiple of 128", fn, (long long)in);
    return GOQ_OK;
}

extern "C" {

int goq_version(void) { return 1001; }

const char *goq_last_error(void) { return g_err; }

int goq_packed_bytes(int bw, int64_t out, int64_t in, size_t *bytes)
{
    if (!bytes) return goq_set_error(GOQ_EINVAL, "goq_packed_bytes: bytes is NULL");
    int rc = check_shape("goq_packed_bytes", bw, out, in);
    if (rc) return rc;
    *bytes = (size_t)goq_packed_dwords(bw, out, in) * 4;
    return GOQ_OK;
}

int goq_quantize(void *stream, int bw, int64_t out, int64_t in, const uint16_t *w, uint8_t *codes,
                 uint8_t *pattern, uint8_t *signs, uint16_t *c1, uint16_t *c2)
{
    int rc = check_shape("goq_quantize", bw, out, in);
    if (rc) return rc;
    if (!w || !codes || !pattern || !signs || !c1 || !c2) return goq_set_error(GOQ_EINVAL, "goq_quantize: NULL pointer");
    if (misaligned(w, 16) || misaligned(codes, 8) || misaligned(c1, 2) || misaligned(c2, 2))
        return goq_set_error(GOQ_EINVAL, "goq_quantize: w must be 16-byte, codes 8-byte, c1 and c2 2-byte aligned");
    return goq_launch_quantize((hipStream_t)stream, bw, out, in, w, codes, pattern, signs, c1, c2);
}

int goq_ref_workspace_bytes(int64_t in, size_t *bytes)
{
    if (!bytes) return goq_set_error(GOQ_EINVAL, "goq_ref_workspace_bytes: bytes is NULL");
    if (in <= 0 || in % GOQ_N) return goq_set_error(GOQ_ESHAPE, "goq_ref_workspace_bytes: in = %lld must be a positive multiple of 128", (long long)in);
    *bytes = (size_t)(in / GOQ_N) * GOQ_N * GOQ_N * sizeof(double);
    return GOQ_OK;
}

int goq_ref_coefficients(void *stream, int bw, int64_t tokens, int64_t out, int64_t in, const uint16_t *w,
                         const uint8_t *codes, const uint8_t *pattern, const uint8_t *signs, const uint16_t *X,
                         double lambda, void *workspace, double *craw, uint16_t *c1, uint16_t *c2)
{
    int rc = check_shape("goq_ref_coefficients", bw, out, in);
    if (rc) return rc;
    if (tokens <= 0 || tokens > (1 << 24))
        return goq_set_error(GOQ_ESHAPE, "goq_ref_coefficients: tokens = %lld out of range", (long long)tokens);
    if (!(lambda >= 0.0) || lambda > 1e300)
        return goq_set_error(GOQ_EINVAL, "goq_ref_coefficients: lambda must be finite and >= 0");
    if (!w || !codes || !pattern || !signs || !X || !workspace || !c1 || !c2)
        return goq_set_error(GOQ_EINVAL, "goq_ref_coefficients: NULL pointer");
    if (misaligned(X, 16) || misaligned(workspace, 16) || misaligned(codes, 8) || misaligned(w, 2) ||
        misaligned(c1, 2) || misaligned(c2, 2) || misaligned(craw, 8))
        return goq_set_error(GOQ_EINVAL, "goq_ref_coefficients: X and workspace must be 16-byte aligned, codes 8-byte");
    return goq_launch_ref((hipStream_t)stream, bw, tokens, out, in, w, codes, pattern, signs, X, lambda, workspace,
                          craw, c1, c2);
}

int goq_pack(void *stream, int bw, int64_t out, int64_t in, const uint8_t *codes, const uint8_t *pattern,
             const uint8_t *signs, const uint16_t *c1, const uint16_t *c2, void *packed)
{
    int rc = check_shape("goq_pack", bw, out, in);
    if (rc) return rc;
    if (!codes || !pattern || !signs || !c1 || !c2 || !packed)
        return goq_set_error(GOQ_EINVAL, "goq_pack: NULL pointer");
    if (misaligned(packed, 16)) return goq_set_error(GOQ_EINVAL, "goq_pack: packed must be 16-byte aligned");
    return goq_launch_pack((hipStream_t)stream, bw, out, in, codes, pattern, signs, c1, c2, packed);
}

int goq_unpack(void *stream, int bw, int64_t out, int64_t in, const void *packed, uint8_t *codes,
               uint8_t *pattern, uint8_t *signs, uint16_t *c1, uint16_t *c2)
{
    int rc = check_shape("goq_unpack", bw, out, in);
    if (rc) return rc;
    if (!codes || !pattern || !signs || !c1 || !c2 || !packed)
        return goq_set_error(GOQ_EINVAL, "goq_unpack: NULL pointer");
    if (misaligned(packed, 16)) return goq_set_error(GOQ_EINVAL, "goq_unpack: packed must be 16-byte aligned");
    return goq_launch_unpack((hipStream_t)stream, bw, out, in, packed, codes, pattern, signs, c1, c2);
}

static int check_gemv_desc(const char *fn, int bw, int act, const goq_gemv_desc &d)
{
    int rc = check_shape(fn, bw, d.out, d.in);
    if (rc) return rc;
    if (act != GOQ_A16 && act != GOQ_A8 && act != GOQ_A4 && act != GOQ_A6 && act != GOQ_A3) return goq_set_error(GOQ_EINVAL, "%s: bad activation type %d", fn, act);
    if (d.ytype != GOQ_F16 && d.ytype != GOQ_F32) return goq_set_error(GOQ_EINVAL, "%s: bad output type %d", fn, d.ytype);
    if (!d.packed || !d.x || !d.y) return goq_set_error(GOQ_EINVAL, "%s: NULL pointer", fn);
    if (act != GOQ_A16 && !d.sx) return goq_set_error(GOQ_EINVAL, "%s: integer activations need sx", fn);
    if (act == GOQ_A16 && d.sx) return goq_set_error(GOQ_EINVAL, "%s: sx must be NULL for fp16 activations", fn);
    if (misaligned(d.packed, 16) || misaligned(d.x, 16) || misaligned(d.y, 16))
        return goq_set_error(GOQ_EINVAL, "%s: packed, x and y must be 16-byte aligned", fn);
    return GOQ_OK;
}

int goq_gemv(void *stream, int bw, int act, int64_t out, int64_t in, const void *packed, const void *x,
             const float *sx, void *y, int ytype)
{
    goq_gemv_desc d;
    d.out = out; d.in = in; d.packed = packed; d.x = x; d.sx = sx; d.y = y; d.ytype = ytype;
    int rc = check_gemv_desc("goq_gemv", bw, act, d);
    if (rc) return rc;
    return goq_launch_gemv((hipStream_t)stream, bw, act, 1, &d, nullptr);
}

int goq_mfma_probe(void *stream, int32_t *report)
{
    if (!report || misaligned(report, 4)) return goq_set_error(GOQ_EINVAL, "goq_mfma_probe: report must be a 4-byte aligned device pointer");
    return goq_launch_mfma_probe((hipStream_t)stream, report);
}

int goq_read_probe(void *stream, const void *buf, size_t bytes, uint32_t *sink)
{
    if (!buf || !sink || misaligned(buf, 16) || misaligned(sink, 4))
        return goq_set_error(GOQ_EINVAL, "goq_read_probe: buf must be 16-byte aligned, sink 4-byte");
    if (bytes < (size_t)512 * 512 * 16 || bytes % 16)
        return goq_set_error(GOQ_ESHAPE, "goq_read_probe: bytes must be a multiple of 16 and at least 4 MiB");
    return goq_launch_read_probe((hipStream_t)stream, buf, bytes, sink);
}

int goq_mfma_rate_probe(void *stream, int kind, int workgroups, int iters, float *sink, double *ops)
{
    if (!sink || !ops || misaligned(sink, 4)) return goq_set_error(GOQ_EINVAL, "goq_mfma_rate_probe: NULL or misaligned pointer");
    if (kind < 0 || kind > 2) return goq_set_error(GOQ_EINVAL, "goq_mfma_rate_probe: kind = %d must be 0, 1 or 2", kind);
    if (workgroups < 1 || workgroups > (1 << 20) || iters < 1 || iters > (1 << 24))
        return goq_set_error(GOQ_ESHAPE, "goq_mfma_rate_probe: workgroups or iters out of range");
    return goq_launch_mfma_rate_probe((hipStream_t)stream, kind, workgroups, iters, sink, ops);
}

int goq_gemv_select(int kernel)
{
    if (kernel != GOQ_GEMV_AUTO && kernel != GOQ_GEMV_STREAM && kernel != GOQ_GEMV_ROWS)
        return goq_set_error(GOQ_EINVAL, "goq_gemv_select: kernel = %d is none of GOQ_GEMV_AUTO/STREAM/ROWS", kernel);
    goq_gemv_set_kernel(kernel);
    return GOQ_OK;
}

int goq_gemv_plan(int bw, int act, int n, const goq_gemv_desc *descs, int *kernel, int *workgroups)
{
    if (!descs || !kernel || !workgroups) return goq_set_error(GOQ_EINVAL, "goq_gemv_plan: NULL pointer");
    if (n < 1 || n > GOQ_MAX_BATCH)
        return goq_set_error(GOQ_ESHAPE, "goq_gemv_plan: n = %d must be in 1..%d", n, GOQ_MAX_BATCH);
    if (act != GOQ_A16 && act != GOQ_A8 && act != GOQ_A4 && act != GOQ_A6 && act != GOQ_A3) return goq_set_error(GOQ_EINVAL, "goq_gemv_plan: bad activation type %d", act);
    for (int i = 0; i < n; ++i) {
        int rc = check_shape("goq_gemv_plan", bw, descs[i].out, descs[i].in);
        if (rc) return rc;
    }
    return goq_gemv_plan_launch(n, descs, kernel, workgroups);
}

int goq_gemv_batch(void *stream, int bw, int act, int n, const goq_gemv_desc *descs)
{
    if (!descs) return goq_set_error(GOQ_EINVAL, "goq_gemv_batch: descs is NULL");
    if (n <= 0 || n > GOQ_MAX_BATCH)
        return goq_set_error(GOQ_ESHAPE, "goq_gemv_batch: n = %d must be in 1..%d", n, GOQ_MAX_BATCH);
    for (int i = 0; i < n; ++i) {
        int rc = check_gemv_desc("goq_gemv_batch", bw, act, descs[i]);
        if (rc) return rc;
    }
    return goq_launch_gemv((hipStream_t)stream, bw, act, n, descs, nullptr);
}

int goq_gemv_workspace_bytes(size_t *bytes)
{
    if (!bytes) return goq_set_error(GOQ_EINVAL, "goq_gemv_workspace_bytes: bytes is NULL");
    *bytes = goq_gemv_workspace_size();
    return GOQ_OK;
}

int goq_gemv_workspace_init(void *stream, void *workspace)
{
    if (!workspace || misaligned(workspace, 256))
        return goq_set_error(GOQ_EINVAL, "goq_gemv_workspace_init: workspace must be a 256-byte aligned device pointer");
    return goq_launch_gemv_workspace_init((hipStream_t)stream, workspace);
}

int goq_gemv_batch_ws(void *stream, int bw, int act, int n, const goq_gemv_desc *descs, void *workspace)
{
    if (!descs) return goq_set_error(GOQ_EINVAL, "goq_gemv_batch_ws: descs is NULL");
    if (!workspace || misaligned(workspace, 256))
        return goq_set_error(GOQ_EINVAL, "goq_gemv_batch_ws: workspace must be a 256-byte aligned device pointer");
    if (n <= 0 || n > GOQ_MAX_BATCH)
        return goq_set_error(GOQ_ESHAPE, "goq_gemv_batch_ws: n = %d must be in 1..%d", n, GOQ_MAX_BATCH);
    for (int i = 0; i < n; ++i) {
        int rc = check_gemv_desc("goq_gemv_batch_ws", bw, act, descs[i]);
        if (rc) return rc;
    }
    return goq_launch_gemv((hipStream_t)stream, bw, act, n, descs, workspace);
}

int goq_gemv_stream_table_bytes(int n, size_t *bytes)
{
    if (!bytes) return goq_set_error(GOQ_EINVAL, "goq_gemv_stream_table_bytes: bytes is NULL");
    if (n < 1 || n > GOQ_MAX_STREAM)
        return goq_set_error(GOQ_ESHAPE, "goq_gemv_stream_table_bytes: n = %d must be in 1..%d", n, GOQ_MAX_STREAM);
    *bytes = goq_gemv_stream_table_size(n);
    return GOQ_OK;
}

int goq_gemv_stream_table(int bw, int act, int n, const goq_gemv_desc *descs, void *table)
{
    if (!descs || !table) return goq_set_error(GOQ_EINVAL, "goq_gemv_stream_table: NULL pointer");
    if (misaligned(table, 8)) return goq_set_error(GOQ_EINVAL, "goq_gemv_stream_table: table must be 8-byte aligned");
    if (n < 1 || n > GOQ_MAX_STREAM)
        return goq_set_error(GOQ_ESHAPE, "goq_gemv_stream_table: n = %d must be in 1..%d", n, GOQ_MAX_STREAM);
    for (int i = 0; i < n; ++i) {
        int rc = check_gemv_desc("goq_gemv_stream_table", bw, act, descs[i]);
        if (rc) return rc;
    }
    return goq_gemv_stream_build_table(bw, act, n, descs, table);
}

int goq_gemv_stream(void *stream, const void *table_host, const void *table_dev, void *workspace)
{
    if (!table_host || !table_dev || !workspace) return goq_set_error(GOQ_EINVAL, "goq_gemv_stream: NULL pointer");
    if (misaligned(table_host, 8) || misaligned(table_dev, 16) || misaligned(workspace, 256))
        return goq_set_error(GOQ_EINVAL, "goq_gemv_stream: table_dev must be 16-byte, workspace 256-byte aligned");
    return goq_launch_gemv_stream((hipStream_t)stream, table_host, table_dev, workspace);
}

static int check_gemm_desc(const char *fn, int bw, int act, const goq_gemm_desc &d)
{
    int rc = check_shape(fn, bw, d.out, d.in);
    if (rc) return rc;
    if (d.tokens <= 0 || d.tokens > (1 << 24)) return goq_set_error(GOQ_ESHAPE, "%s: tokens = %lld out of range", fn, (long long)d.tokens);
    if (act != GOQ_A16 && act != GOQ_A8 && act != GOQ_A4 && act != GOQ_A6 && act != GOQ_A3) return goq_set_error(GOQ_EINVAL, "%s: bad activation type %d", fn, act);
    if (d.ytype != GOQ_F16 && d.ytype != GOQ_F32) return goq_set_error(GOQ_EINVAL, "%s: bad output type %d", fn, d.ytype);
    if (!d.packed || !d.X || !d.Y) return goq_set_error(GOQ_EINVAL, "%s: NULL pointer", fn);
    if (act != GOQ_A16 && !d.sx) return goq_set_error(GOQ_EINVAL, "%s: integer activations need sx", fn);
    if (act == GOQ_A16 && d.sx) return goq_set_error(GOQ_EINVAL, "%s: sx must be NULL for fp16 activations", fn);
    if (act == GOQ_A16 && d.partials) return goq_set_error(GOQ_EINVAL, "%s: partials is only defined for int8 activations", fn);
    if (misaligned(d.packed, 16) || misaligned(d.X, 16) || misaligned(d.Y, 16))
        return goq_set_error(GOQ_EINVAL, "%s: packed, X and Y must be 16-byte aligned", fn);
    return GOQ_OK;
}

int goq_gemm(void *stream, int bw, int act, int64_t tokens, int64_t out, int64_t in, const void *packed,
             const void *X, const float *sx, void *Y, int ytype, int32_t *partials)
{
    goq_gemm_desc d;
    d.tokens = tokens; d.out = out; d.in = in; d.packed = packed; d.X = X; d.sx = sx; d.Y = Y;
    d.ytype = ytype; d.partials = partials;
    int rc = check_gemm_desc("goq_gemm", bw, act, d);
    if (rc) return rc;
    return goq_launch_gemm((hipStream_t)stream, bw, act, 1, &d);
}

int goq_gemm_batch(void *stream, int bw, int act, int n, const goq_gemm_desc *descs)
{
    if (!descs) return goq_set_error(GOQ_EINVAL, "goq_gemm_batch: descs is NULL");
    if (n < 1 || n > GOQ_MAX_BATCH)
        return goq_set_error(GOQ_ESHAPE, "goq_gemm_batch: n = %d must be in 1..%d", n, GOQ_MAX_BATCH);
    for (int i = 0; i < n; ++i) {
        int rc = check_gemm_desc("goq_gemm_batch", bw, act, descs[i]);
        if (rc) return rc;
    }
    return goq_launch_gemm((hipStream_t)stream, bw, act, n, descs);
}

int goq_gemm_folded(void *stream, int bw, int64_t tokens, int64_t out, int64_t in, const void *packed,
                    const void *X, void *Y, int ytype)
{
    int rc = check_shape("goq_gemm_folded", bw, out, in);
    if (rc) return rc;
    if (tokens <= 0 || tokens > (1 << 24)) return goq_set_error(GOQ_ESHAPE, "goq_gemm_folded: tokens = %lld out of range", (long long)tokens);
    if (ytype != GOQ_F16 && ytype != GOQ_F32) return goq_set_error(GOQ_EINVAL, "goq_gemm_folded: bad output type %d", ytype);
    if (!packed || !X || !Y) return goq_set_error(GOQ_EINVAL, "goq_gemm_folded: NULL pointer");
    if (misaligned(packed, 16) || misaligned(X, 16) || misaligned(Y, 16))
        return goq_set_error(GOQ_EINVAL, "goq_gemm_folded: packed, X and Y must be 16-byte aligned");
    return goq_launch_gemm_folded((hipStream_t)stream, bw, tokens, out, in, packed, X, Y, ytype);
}

}  // extern "C"
