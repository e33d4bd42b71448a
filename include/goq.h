/*
 * goq.h -- C ABI of the MI355X (gfx950) dual power-of-two linear-layer library.
 *
 * What the library computes (GoQuant, "Fully Quantized Inference Dataflow", Eq. 4, read per
 * 128-wide slab of the input dimension):
 *
 *     P_m[t,o,g] = sum_{k in slab g} x[t,k] * b_m[o,k]            m = 1, 2
 *     y[t,o]     = sum_g ( c1[o,g] * P_1[t,o,g] + c2[o,g] * P_2[t,o,g] )   ( * s_x[t] * 2^-(E-1) for int8 x )
 *
 * b_1[o,k] is the power-of-two value of the stored 3- or 4-bit code (asymmetric lattice of
 * Sec. 3.2: sign + exponent, the smallest positive bin repurposed as exact zero).  b_2 is never
 * stored: inside every 8-weight micro-block it is rebuilt from b_1 by the Strided Dual-Exchange
 * of Theorem 1 (partner i xor s, s in 1..4; y_i = -eta x_j, y_j = +eta x_i), configured by the
 * micro-block's 2-bit pattern index and 4 pair-sign bits (Sec. 3.3 item 3).  c1, c2 are the two
 * fp16 coefficients of a 128-weight macro-block (Sec. 3.4); they are applied once per slab after
 * the two dot products, outside the multiply-free core.
 *
 * Conventions
 *   - every function returns GOQ_OK (0) or a negative error; goq_last_error() gives the text of
 *     the calling thread's last error.  Arguments are validated on the host before any launch.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work is
 *     enqueued on it; no call synchronises, allocates or frees.
 *   - every pointer named below is a DEVICE pointer unless it says "host".  The caller owns all
 *     buffers and keeps them alive until the stream has passed the call.  x / X / y / Y and the
 *     packed buffer must be 16-byte aligned.
 *   - canonical (logical) weight format, row-major like a linear layer's weight [out][in]:
 *       codes   u8  [out][in]       code = sign << (bw-1) | e, value (-1)^sign 2^-e,
 *                                   (sign 0, e = 2^(bw-1)-1) is exact zero
 *       pattern u8  [out][in/8]     s - 1
 *       signs   u8  [out][in/8]     bit p = 1  <=>  eta of the p-th pair (ascending i) is -1
 *       c1, c2  u16 [out][in/128]   IEEE binary16 bit patterns
 *   - the packed buffer is opaque, position independent (it may be copied or saved) and holds
 *     exactly 4.0 (bw = 3) or 5.0 (bw = 4) bits per weight, rows padded to a multiple of 64.  Its
 *     arrangement belongs to the library version that wrote it (goq_version): a saved buffer is
 *     read back with goq_unpack of the same version, or repacked from the canonical arrays.
 */
#ifndef GOQ_H
#define GOQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    GOQ_OK = 0,
    GOQ_EINVAL = -1,        /* null / misaligned pointer, bad enum                      */
    GOQ_ESHAPE = -2,        /* in % 128 != 0, out <= 0, tokens <= 0, too many problems  */
    GOQ_EUNSUPPORTED = -3,  /* a combination this build does not implement             */
    GOQ_EHIP = -4           /* a HIP runtime call failed (text in goq_last_error)       */
};

/* activation type (b_a-bit integer activations with scale s_x of Eq. 4): fp16 | int8 with a per-token
 * scale | int4, two per byte (element 2 i in the low nibble of byte i, two's complement), with a
 * per-token scale | int6, four per three bytes (element k in bits 6 k .. 6 k + 5 of the token's
 * row read as a little-endian bit string, two's complement), with a per-token scale | int3, eight
 * per three bytes (element k in bits 3 k .. 3 k + 2 of the same bit string).  Integer activations
 * of any other width go in the next larger container. */
enum { GOQ_A16 = 0, GOQ_A8 = 1, GOQ_A4 = 2, GOQ_A6 = 3, GOQ_A3 = 4 };
enum { GOQ_F16 = 0, GOQ_F32 = 1 };  /* output type                                      */

#define GOQ_MAX_BATCH 8             /* problems per goq_gemv_batch / goq_gemm_batch call */
#define GOQ_MAX_STREAM 65536        /* problems per goq_gemv_stream table               */

/* library version, major * 1000 + minor */
int goq_version(void);

/* text of the calling thread's last error (host pointer, valid until the thread's next call) */
const char *goq_last_error(void);

/* size in bytes of the packed buffer of a [out][in] layer: the stored representation of Sec. 3.3
 * item 3 (code bits + 6 metadata bits per 8 weights + two fp16 coefficients per 128 weights) with
 * rows padded to a multiple of 64.  *bytes is a host pointer. */
int goq_packed_bytes(int bw, int64_t out, int64_t in, size_t *bytes);

/* Data-free GEO-mode quantizer (Sec. 3.2 - 3.4) on the device: fp16 weights w [out][in] (IEEE
 * binary16 bit patterns, row-major, 16-byte aligned) -> canonical arrays.  Per 128-weight
 * macro-block along `in`: s_norm = max |w|; codes = nearest lattice state of w / s_norm (linear
 * distance, exact ties toward the smaller magnitude); residual r = w - (<w,b1>/||b1||^2) b1
 * (Eq. 1); per 8-weight micro-block the pattern s* = argmax_s sum_pairs |x_i r_j - x_j r_i| (ties:
 * smallest s) with pair signs eta = sgn(x_i r_j - x_j r_i) (+1 at zero) (Sec. 3.3); b2 by the
 * Theorem 1 exchange; c1 = <w,b1>/||b1||^2, c2 = <w,b2>/||b2||^2 (Eq. 2) rounded to fp16.  An
 * all-zero macro-block gets zero codes, pattern 0, signs 0, c1 = c2 = 0.  Arithmetic is fp64; the
 * sums are exact (every term is a multiple of 2^-31 and the totals stay below 2^22), so the
 * outputs are a pure function of w and equal a sequential evaluation in ascending k.  codes must be
 * 8-byte aligned.  Weights must be finite. */
int goq_quantize(void *stream, int bw, int64_t out, int64_t in, const uint16_t *w,
                 uint8_t *codes, uint8_t *pattern, uint8_t *signs, uint16_t *c1, uint16_t *c2);

/* REF-mode (activation-aware) block coefficients (Sec. 3.4, Eq. 3) on the device.  The bases b1, b2
 * are those of the canonical arrays (codes, pattern, signs: from goq_quantize or elsewhere); for
 * every output channel and 128-wide macro-block the pair (c1, c2) is re-solved by ridge regression
 * on the calibration inputs X (fp16 [tokens][in], row-major, 16-byte aligned):
 *     Y = X_q w,  A = [X_q b1, X_q b2],  c* = (A^T A + lambda I)^-1 A^T Y        (the paper: lambda = 1e-4)
 * with X_q the macro-block's 128 columns of X and w the fp16 weights [out][in].  Computed in fp64
 * through the macro-block's Gram matrix X_q^T X_q, which all output channels share; `workspace` is
 * caller-owned device memory of goq_ref_workspace_bytes(in) bytes (16-byte aligned), used only
 * during the call.  c1, c2 [out][in/128] receive the fp16 bit patterns; craw (optional, may be
 * NULL) receives the unrounded pairs as double [out][in/128][2].  lambda >= 0; a singular system
 * (possible only at lambda = 0) gives c1 = c2 = 0.  codes must be 8-byte aligned. */
int goq_ref_workspace_bytes(int64_t in, size_t *bytes);      /* *bytes is a host pointer */
int goq_ref_coefficients(void *stream, int bw, int64_t tokens, int64_t out, int64_t in, const uint16_t *w,
                         const uint8_t *codes, const uint8_t *pattern, const uint8_t *signs,
                         const uint16_t *X, double lambda, void *workspace, double *craw,
                         uint16_t *c1, uint16_t *c2);

/* Stored representation (Sec. 3.3 item 3): canonical arrays -> packed buffer, on the device. */
int goq_pack(void *stream, int bw, int64_t out, int64_t in,
             const uint8_t *codes, const uint8_t *pattern, const uint8_t *signs,
             const uint16_t *c1, const uint16_t *c2, void *packed);

/* Inverse of goq_pack (test hook): packed buffer -> the canonical arrays of Sec. 3.3 item 3. */
int goq_unpack(void *stream, int bw, int64_t out, int64_t in, const void *packed,
               uint8_t *codes, uint8_t *pattern, uint8_t *signs, uint16_t *c1, uint16_t *c2);

/* Batch-1 layer output (Eq. 4 with one token).
 *   act = GOQ_A16: x is fp16 [in], sx must be NULL.
 *   act = GOQ_A8 : x is int8 [in], sx points to one fp32 scale (device).  Both bit widths.
 *   act = GOQ_A4 : x is packed int4 [in / 2 bytes], sx as for GOQ_A8.
 *   act = GOQ_A6 : x is packed int6 [3 in / 4 bytes], sx as for GOQ_A8.
 *   act = GOQ_A3 : x is packed int3 [3 in / 8 bytes], sx as for GOQ_A8.
 *   y is [out] of ytype.  The PoT codes are decoded to 8-bit floats (a power of two is exact in
 *   E5M2) and b2 is rebuilt from b1 by a byte permute and a sign flip; the two slab dot products
 *   run on the 8-bit-float matrix instruction against x written as block fixed point (24 bits
 *   below the largest exponent of each 32-activation block: exact for int8 x, and for fp16 x up
 *   to a truncation at 2^-24 of the block maximum), accumulate in fp32; coefficients are applied
 *   per slab in fp32.  Results are deterministic (no floating-point atomics).  x must be finite
 *   (Inf / NaN inputs give unspecified finite or non-finite outputs).
 *   Row groups split over several workgroups are combined through one of the library's 8 static
 *   scratch regions on the device (2.1 MB each), one region per stream: launches on one stream run
 *   one after the other and may follow each other without limit.  A 9th stream takes over the
 *   region of the least recently used stream after waiting ON THE HOST until that stream has
 *   drained (the one case in which a call of this library blocks); if one of the two streams is
 *   being captured the call returns GOQ_EUNSUPPORTED instead.  A captured graph bakes the region
 *   of its capture stream in: replay it on that stream only, or capture goq_gemv_batch_ws. */
int goq_gemv(void *stream, int bw, int act, int64_t out, int64_t in,
             const void *packed, const void *x, const float *sx, void *y, int ytype);

/* Several independent batch-1 layers in ONE launch (e.g. the projections of a decoder block).
 * descs is a HOST array of n <= GOQ_MAX_BATCH descriptors; all must share bw and act.
 * This is the entry point for callers that cannot allocate device memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid it): like goq_gemv it allocates nothing and
 * takes no workspace -- its scratch for split row groups is the library's static device array
 * described at goq_gemv (8 regions of 2.1 MB, held on every device the library runs on until the
 * process ends; its device address is resolved once per device on the first call).  The array
 * suffices for every accepted shape (the launch never has more than 512 workgroups, whatever the
 * layers' sizes), so no size is rejected on its account.  It keeps the previous launch's contents:
 * the arrival counters are back at zero when a launch has completed, the parts are overwritten
 * before they are read.  Launches that overlap on one region would race: the library gives every
 * stream a region of its own (see goq_gemv for the limit of 8 streams). */
typedef struct goq_gemv_desc {
    int64_t out, in;
    const void *packed;
    const void *x;
    const float *sx;
    void *y;
    int ytype;
} goq_gemv_desc;
int goq_gemv_batch(void *stream, int bw, int act, int n, const goq_gemv_desc *descs);

/* goq_gemv_batch for callers that cannot allocate and want no library-side state: the
 * workspace for split row groups is the caller's.  For: launches under HIP graph capture that are
 * replayed on any stream, serving loops with more than 8 streams in flight, harnesses that forbid
 * library-owned device state.  workspace: goq_gemv_workspace_bytes() bytes of device memory,
 * 256-byte aligned, zero-filled once by goq_gemv_workspace_init (a kernel launch on `stream`, no
 * memset node) before its first use; every completed launch leaves it ready for the next.  One
 * workspace serves one launch at a time: launches that share it must be ordered (same stream, or
 * events).  The workspace size does not depend on the problem sizes.  Results are bit-identical
 * to goq_gemv_batch. */
int goq_gemv_workspace_bytes(size_t *bytes);                 /* *bytes is a host pointer */
int goq_gemv_workspace_init(void *stream, void *workspace);
int goq_gemv_batch_ws(void *stream, int bw, int act, int n, const goq_gemv_desc *descs, void *workspace);

/* A whole stream of batch-1 layers in ONE launch (Eq. 4 with one token, for every layer of the
 * stream): e.g. all projections of all decoder blocks of a model.  The units (512 output rows x
 * one 128-wide slab) of all n <= GOQ_MAX_STREAM problems form one sequence that is cut into equal
 * contiguous pieces, one per workgroup, so start-up and tail of the launch are paid once per
 * stream instead of once per block.  The problems are independent: the library orders nothing
 * between them (x of every problem must be ready before the launch).
 *   goq_gemv_stream_table writes the problem table (goq_gemv_stream_table_bytes(n) bytes) into a
 *   HOST buffer, 8-byte aligned; the caller copies those bytes to device memory (16-byte aligned)
 *   and passes both copies to goq_gemv_stream: the host copy tells the library the launch shape,
 *   the device copy feeds the kernel.  The table holds the descriptors' device pointers: it stays
 *   valid as long as they do.  All problems share bw and act.
 *   workspace: as for goq_gemv_batch_ws.
 * A stream of the problems of one goq_gemv_batch call gives that call's streaming-kernel results
 * bit for bit; in general the split points, hence the fp32 summation order, depend on the stream. */
int goq_gemv_stream_table_bytes(int n, size_t *bytes);       /* *bytes is a host pointer */
int goq_gemv_stream_table(int bw, int act, int n, const goq_gemv_desc *descs, void *table /* host */);
int goq_gemv_stream(void *stream, const void *table_host, const void *table_dev, void *workspace);

/* Test hook: measures, on the device, the two properties of the 8-bit-float matrix instruction
 * that the exactness of the batch-1 path (Eq. 4 with integer activations: exact slab sums)
 * rests on.  report: 17 int32 in device memory.
 *   report[0]        depth of the fixed-point grid on which the products of 8 consecutive k are
 *                    added, in binary places below the largest product (the library needs >= 10:
 *                    3-bit digits against powers of two 2^0 .. 2^-7; gfx950 gives 13)
 *   report[1 + 4 Q + i], Q = 0..3, i = 0..3: bit b set <=> the block scale supplied by lane
 *                    (row, Q) applies to k = 32 i + b of that A row.  The library assumes
 *                    k-groups 2 (Q % 2) and 2 (Q % 2) + 1 (i.e. i), bits 16 (Q / 2) .. + 15. */
int goq_mfma_probe(void *stream, int32_t *report);

/* Measurement hooks: the ceilings of this device as a kernel of this library's launch shape sees
 * them, reported by bench.py beside the nominal peaks (they compute nothing of the method).
 *   goq_read_probe       streams buf [bytes] (device, 16-byte aligned, >= 4 MiB) once with
 *                        nontemporal 16-byte loads, 512 workgroups of 512 threads, one contiguous
 *                        piece each: the read rate a batch-1 launch of that size could reach at best.
 *   goq_mfma_rate_probe  `workgroups` x 4 wavefronts, each issuing iters x 4 matrix instructions
 *                        on four accumulator chains and nothing else.  kind 0: fp16 32x32x16,
 *                        1: int8 32x32x32, 2: 8-bit float 16x16x128.  *ops (host) receives the
 *                        operations of the launch (2 per multiply-add).
 * sink: 4 bytes of device memory (written only if the data happen to hash to a magic value). */
int goq_read_probe(void *stream, const void *buf, size_t bytes, uint32_t *sink);
int goq_mfma_rate_probe(void *stream, int kind, int workgroups, int iters, float *sink, double *ops);

/* Which of the two batch-1 kernels goq_gemv / goq_gemv_batch launch when called from THIS thread
 * (a per-thread setting, takes effect with the thread's next call; both kernels compute the same sums of Eq. 4 and both accept every shape):
 *   GOQ_GEMV_AUTO   (default) by size: launches of at most 512 tiles of 16 output rows (each
 *                   problem's rows rounded up to 16) and at most 24576 (tile, macro-block)
 *                   pairs -- 48 Mi weights -- go to the row-owner kernel, everything else streams;
 *   GOQ_GEMV_STREAM the streaming kernel: equal contiguous pieces of the launch's weight bytes
 *                   per workgroup, split row groups combined through the scratch area;
 *   GOQ_GEMV_ROWS   the row-owner kernel: one workgroup per 16 output rows over the whole depth,
 *                   partial sums combined in LDS (no scratch).
 * Returns GOQ_EINVAL for any other value. */
enum { GOQ_GEMV_AUTO = 0, GOQ_GEMV_STREAM = 1, GOQ_GEMV_ROWS = 2 };
int goq_gemv_select(int kernel);

/* What a goq_gemv_batch call with these shapes would launch under the current selection: *kernel
 * receives GOQ_GEMV_STREAM or GOQ_GEMV_ROWS, *workgroups the grid size (both host pointers).
 * Only out and in of the descriptors are read; nothing is launched and no device is touched. */
int goq_gemv_plan(int bw, int act, int n, const goq_gemv_desc *descs, int *kernel, int *workgroups);

/* Many-token layer output (Eq. 4), Y[tokens][out] = X[tokens][in] * W^T.
 *   act = GOQ_A16: X fp16, sx NULL; PoT codes are decoded to fp16 operands of the fp16 MFMA,
 *                  fp32 accumulation.
 *   act = GOQ_A8 : X int8, sx fp32 [tokens].  bw = 3: PoT codes are decoded to int8 (b * 2^(E-1))
 *                  operands of the int8 MFMA, exact int32 slab partials.  bw = 4: b * 2^7 reaches
 *                  +128, which is no int8; the int8 activations are widened to fp16 on their way
 *                  into LDS and the fp16 MFMA is used -- every product is exact and a slab sum
 *                  needs at most 22 bits, so the fp32 accumulators hold the same exact integers.
 *   act = GOQ_A4 : X packed int4 [tokens][in / 2 bytes], sx fp32 [tokens]; unpacked to int8 (bw = 3)
 *                  or widened to fp16 (bw = 4) on the way into LDS, then as GOQ_A8.
 *   act = GOQ_A6 : X packed int6 [tokens][3 in / 4 bytes], otherwise as GOQ_A4.
 *   act = GOQ_A3 : X packed int3 [tokens][3 in / 8 bytes], otherwise as GOQ_A4.
 *   partials (optional, integer activations only, else NULL): int32 [tokens][out][in/128][2] receives
 *   the exact slab partials P_1, P_2 (in units of 2^-(E-1)). */
int goq_gemm(void *stream, int bw, int act, int64_t tokens, int64_t out, int64_t in,
             const void *packed, const void *X, const float *sx, void *Y, int ytype,
             int32_t *partials);

/* Several independent many-token layers in ONE launch (e.g. q, k, v or gate, up of a decoder block,
 * which share X): the tiles of all problems form one grid, so a small matrix does not leave the
 * chip half empty and there is one tail instead of n.  descs is a HOST array of n <= GOQ_MAX_BATCH
 * descriptors with the arguments of goq_gemm; all share bw and act.  Results are those of n
 * goq_gemm calls, bit for bit. */
typedef struct goq_gemm_desc {
    int64_t tokens, out, in;
    const void *packed;
    const void *X;
    const float *sx;
    void *Y;
    int ytype;
    int32_t *partials;
} goq_gemm_desc;
int goq_gemm_batch(void *stream, int bw, int act, int n, const goq_gemm_desc *descs);

/* Ablation of the two-basis product (not the method's path; it measures what keeping the PoT
 * operands native costs on matrix-core hardware).  Same result as goq_gemm with GOQ_A16 up to
 * rounding, computed differently: the decoded bases are combined in registers to the fp16 weight
 * c1 b1 + c2 b2 of Eq. 4's slab and ONE fp16 matrix instruction per k-step accumulates into Y in
 * fp32 -- half the matrix instructions, no per-slab rescale, but every weight is rounded to fp16
 * (relative 2^-11), so the result is held to 1e-3 normalised backward error
 * |y - y^| / sum_k |x_k| |W^_k| only, not to the element-wise bound of goq_gemm.  X fp16
 * [tokens][in], Y [tokens][out] of ytype; arguments and errors as for goq_gemm. */
int goq_gemm_folded(void *stream, int bw, int64_t tokens, int64_t out, int64_t in,
                    const void *packed, const void *X, void *Y, int ytype);

#ifdef __cplusplus
}
#endif
#endif /* GOQ_H */
