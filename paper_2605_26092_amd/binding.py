"""ctypes binding of include/goq.h: same names, argument marshalling only.

Tensors are torch tensors on the GPU (or anything with .data_ptr()); the current torch stream is
passed as the hipStream_t.  The library is loaded on first use and a missing build is an error:
there is no fallback path."""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libgoq.so")
_lib = None

A16, A8, A4, A6, A3 = 0, 1, 2, 3, 4
F16, F32 = 0, 1
OK, EINVAL, ESHAPE, EUNSUPPORTED, EHIP = 0, -1, -2, -3, -4
MAX_BATCH = 8
GEMV_AUTO, GEMV_STREAM, GEMV_ROWS = 0, 1, 2

EXPORTS = ["goq_version", "goq_last_error", "goq_packed_bytes", "goq_quantize", "goq_ref_workspace_bytes",
           "goq_ref_coefficients", "goq_pack", "goq_unpack",
           "goq_gemv", "goq_gemv_batch", "goq_gemv_workspace_bytes", "goq_gemv_workspace_init", "goq_gemv_batch_ws",
           "goq_gemv_stream_table_bytes", "goq_gemv_stream_table", "goq_gemv_stream", "goq_mfma_probe", "goq_read_probe", "goq_mfma_rate_probe", "goq_gemv_select", "goq_gemv_plan", "goq_gemm", "goq_gemm_batch", "goq_gemm_folded"]


class GoqError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("goq error %d: %s" % (code, msg))
        self.code = code


class _GemmDesc(ctypes.Structure):
    _fields_ = [("tokens", ctypes.c_int64), ("out", ctypes.c_int64), ("in_", ctypes.c_int64),
                ("packed", ctypes.c_void_p), ("X", ctypes.c_void_p), ("sx", ctypes.c_void_p),
                ("Y", ctypes.c_void_p), ("ytype", ctypes.c_int), ("partials", ctypes.c_void_p)]


class _Desc(ctypes.Structure):
    _fields_ = [("out", ctypes.c_int64), ("in_", ctypes.c_int64), ("packed", ctypes.c_void_p),
                ("x", ctypes.c_void_p), ("sx", ctypes.c_void_p), ("y", ctypes.c_void_p),
                ("ytype", ctypes.c_int)]


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError("libgoq.so is not built: run `python -m paper_2605_26092_amd.build` "
                              "(or __graft_entry__.build()) first; there is no fallback path")
        # torch first: libgoq.so binds to the HIP runtime already in the process (same soname), and
        # that must be the one that owns the caller's tensors and streams, i.e. the one torch ships
        import torch  # noqa: F401
        L = ctypes.CDLL(_LIB_PATH)
        vp, i, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
        L.goq_version.restype = i
        L.goq_last_error.restype = ctypes.c_char_p
        L.goq_packed_bytes.argtypes = [i, i64, i64, ctypes.POINTER(ctypes.c_size_t)]
        L.goq_quantize.argtypes = [vp, i, i64, i64, vp, vp, vp, vp, vp, vp]
        L.goq_ref_workspace_bytes.argtypes = [i64, ctypes.POINTER(ctypes.c_size_t)]
        L.goq_ref_coefficients.argtypes = [vp, i, i64, i64, i64, vp, vp, vp, vp, vp, ctypes.c_double, vp, vp, vp, vp]
        L.goq_pack.argtypes = [vp, i, i64, i64, vp, vp, vp, vp, vp, vp]
        L.goq_unpack.argtypes = [vp, i, i64, i64, vp, vp, vp, vp, vp, vp]
        L.goq_gemv.argtypes = [vp, i, i, i64, i64, vp, vp, vp, vp, i]
        L.goq_gemv_batch.argtypes = [vp, i, i, i, ctypes.POINTER(_Desc)]
        L.goq_gemv_workspace_bytes.argtypes = [ctypes.POINTER(ctypes.c_size_t)]
        L.goq_gemv_workspace_init.argtypes = [vp, vp]
        L.goq_gemv_batch_ws.argtypes = [vp, i, i, i, ctypes.POINTER(_Desc), vp]
        L.goq_gemv_stream_table_bytes.argtypes = [i, ctypes.POINTER(ctypes.c_size_t)]
        L.goq_gemv_stream_table.argtypes = [i, i, i, ctypes.POINTER(_Desc), vp]
        L.goq_gemv_stream.argtypes = [vp, vp, vp, vp]
        L.goq_mfma_probe.argtypes = [vp, vp]
        L.goq_read_probe.argtypes = [vp, vp, ctypes.c_size_t, vp]
        L.goq_mfma_rate_probe.argtypes = [vp, i, i, i, vp, ctypes.POINTER(ctypes.c_double)]
        L.goq_gemv_select.argtypes = [i]
        L.goq_gemv_plan.argtypes = [i, i, i, ctypes.POINTER(_Desc), ctypes.POINTER(i), ctypes.POINTER(i)]
        L.goq_gemm.argtypes = [vp, i, i, i64, i64, i64, vp, vp, vp, vp, i, vp]
        L.goq_gemm_batch.argtypes = [vp, i, i, i, ctypes.POINTER(_GemmDesc)]
        L.goq_gemm_folded.argtypes = [vp, i, i64, i64, i64, vp, vp, vp, i]
        _lib = L
    return _lib


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is not None:
        return stream if isinstance(stream, int) else stream.cuda_stream
    import torch
    return torch.cuda.current_stream().cuda_stream


def _check(rc):
    if rc != 0:
        raise GoqError(rc, last_error())


def version():
    return lib().goq_version()


def last_error():
    return lib().goq_last_error().decode()


def packed_bytes(bw, out, inn):
    n = ctypes.c_size_t(0)
    _check(lib().goq_packed_bytes(bw, out, inn, ctypes.byref(n)))
    return n.value


def quantize(bw, out, inn, w, codes, pattern, signs, c1, c2, stream=None):
    _check(lib().goq_quantize(_stream(stream), bw, out, inn, _ptr(w), _ptr(codes), _ptr(pattern), _ptr(signs),
                              _ptr(c1), _ptr(c2)))


def ref_workspace_bytes(inn):
    n = ctypes.c_size_t(0)
    _check(lib().goq_ref_workspace_bytes(inn, ctypes.byref(n)))
    return n.value


def ref_coefficients(bw, tokens, out, inn, w, codes, pattern, signs, X, lam, workspace, craw, c1, c2, stream=None):
    _check(lib().goq_ref_coefficients(_stream(stream), bw, tokens, out, inn, _ptr(w), _ptr(codes), _ptr(pattern),
                                      _ptr(signs), _ptr(X), float(lam), _ptr(workspace), _ptr(craw), _ptr(c1), _ptr(c2)))


def pack(bw, out, inn, codes, pattern, signs, c1, c2, packed, stream=None):
    _check(lib().goq_pack(_stream(stream), bw, out, inn, _ptr(codes), _ptr(pattern), _ptr(signs),
                          _ptr(c1), _ptr(c2), _ptr(packed)))


def unpack(bw, out, inn, packed, codes, pattern, signs, c1, c2, stream=None):
    _check(lib().goq_unpack(_stream(stream), bw, out, inn, _ptr(packed), _ptr(codes), _ptr(pattern),
                            _ptr(signs), _ptr(c1), _ptr(c2)))


def gemv(bw, act, out, inn, packed, x, sx, y, ytype, stream=None):
    _check(lib().goq_gemv(_stream(stream), bw, act, out, inn, _ptr(packed), _ptr(x), _ptr(sx), _ptr(y), ytype))


def make_descs(problems):
    """problems: list of (out, in, packed, x, sx, y, ytype) -> ctypes array (host memory)."""
    arr = (_Desc * len(problems))()
    for d, (out, inn, packed, x, sx, y, ytype) in zip(arr, problems):
        d.out, d.in_, d.packed, d.x, d.sx, d.y, d.ytype = out, inn, _ptr(packed), _ptr(x), _ptr(sx), _ptr(y), ytype
    return arr


def mfma_probe(report, stream=None):
    _check(lib().goq_mfma_probe(_stream(stream), _ptr(report)))


def read_probe(buf, nbytes, sink, stream=None):
    _check(lib().goq_read_probe(_stream(stream), _ptr(buf), nbytes, _ptr(sink)))


def mfma_rate_probe(kind, workgroups, iters, sink, stream=None):
    """-> operations (2 per multiply-add) of the launch."""
    ops = ctypes.c_double(0.0)
    _check(lib().goq_mfma_rate_probe(_stream(stream), kind, workgroups, iters, _ptr(sink), ctypes.byref(ops)))
    return ops.value


def gemv_select(kernel):
    _check(lib().goq_gemv_select(kernel))


def gemv_plan(bw, act, shapes):
    """shapes: list of (out, in) -> (kernel, workgroups) a gemv_batch call of these layers would launch."""
    arr = (_Desc * len(shapes))()
    for d, (out, inn) in zip(arr, shapes):
        d.out, d.in_ = out, inn
    k, w = ctypes.c_int(0), ctypes.c_int(0)
    _check(lib().goq_gemv_plan(bw, act, len(arr), arr, ctypes.byref(k), ctypes.byref(w)))
    return k.value, w.value


def gemv_batch(bw, act, problems, stream=None):
    arr = problems if isinstance(problems, ctypes.Array) else make_descs(problems)
    _check(lib().goq_gemv_batch(_stream(stream), bw, act, len(arr), arr))


def gemv_workspace_bytes():
    n = ctypes.c_size_t(0)
    _check(lib().goq_gemv_workspace_bytes(ctypes.byref(n)))
    return n.value


def gemv_workspace_init(workspace, stream=None):
    _check(lib().goq_gemv_workspace_init(_stream(stream), _ptr(workspace)))


def gemv_batch_ws(bw, act, problems, workspace, stream=None):
    arr = problems if isinstance(problems, ctypes.Array) else make_descs(problems)
    _check(lib().goq_gemv_batch_ws(_stream(stream), bw, act, len(arr), arr, _ptr(workspace)))


def gemv_stream_table(bw, act, problems):
    """problems (list of (out, in, packed, x, sx, y, ytype) or a ctypes array from make_descs) -> the
    problem table as a host buffer (a ctypes char array); the caller copies it to the device."""
    arr = problems if isinstance(problems, ctypes.Array) else make_descs(problems)
    n = ctypes.c_size_t(0)
    _check(lib().goq_gemv_stream_table_bytes(len(arr), ctypes.byref(n)))
    buf = (ctypes.c_uint64 * ((n.value + 7) // 8))()
    _check(lib().goq_gemv_stream_table(bw, act, len(arr), arr, ctypes.addressof(buf)))
    return buf, n.value


def gemv_stream(table_host, table_dev, workspace, stream=None):
    _check(lib().goq_gemv_stream(_stream(stream), ctypes.addressof(table_host), _ptr(table_dev), _ptr(workspace)))


def bind_gemv_stream(table_host, table_dev, workspace, stream=None):
    """A zero-argument callable that launches goq_gemv_stream on pre-marshalled arguments."""
    fn, s, th, td, ws = lib().goq_gemv_stream, _stream(stream), ctypes.addressof(table_host), _ptr(table_dev), _ptr(workspace)

    def call():
        rc = fn(s, th, td, ws)
        if rc:
            _check(rc)
    return call


def bind_gemv_batch(bw, act, descs, stream=None):
    """A zero-argument callable that launches goq_gemv_batch on pre-marshalled arguments (descs from
    make_descs): for callers that launch the same problems many times and want no per-call
    marshalling."""
    fn, s, n = lib().goq_gemv_batch, _stream(stream), len(descs)

    def call():
        rc = fn(s, bw, act, n, descs)
        if rc:
            _check(rc)
    return call


def gemm(bw, act, tokens, out, inn, packed, X, sx, Y, ytype, partials=None, stream=None):
    _check(lib().goq_gemm(_stream(stream), bw, act, tokens, out, inn, _ptr(packed), _ptr(X), _ptr(sx),
                          _ptr(Y), ytype, _ptr(partials)))


def gemm_folded(bw, tokens, out, inn, packed, X, Y, ytype, stream=None):
    _check(lib().goq_gemm_folded(_stream(stream), bw, tokens, out, inn, _ptr(packed), _ptr(X), _ptr(Y), ytype))


def make_gemm_descs(problems):
    """problems: list of (tokens, out, in, packed, X, sx, Y, ytype[, partials]) -> ctypes array (host memory)."""
    arr = (_GemmDesc * len(problems))()
    for d, p in zip(arr, problems):
        tokens, out, inn, packed, X, sx, Y, ytype = p[:8]
        d.tokens, d.out, d.in_, d.packed, d.X, d.sx, d.Y, d.ytype = tokens, out, inn, _ptr(packed), _ptr(X), _ptr(sx), _ptr(Y), ytype
        d.partials = _ptr(p[8]) if len(p) > 8 else None
    return arr


def gemm_batch(bw, act, problems, stream=None):
    arr = problems if isinstance(problems, ctypes.Array) else make_gemm_descs(problems)
    _check(lib().goq_gemm_batch(_stream(stream), bw, act, len(arr), arr))
