"""ctypes front end of the CPU oracle (goq_oracle.c) -- TEST INFRASTRUCTURE, NOT THE PRODUCT.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this module.
It marshals numpy arrays into the plain-C oracle and performs no arithmetic of its own.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libgoq_oracle.so")
_lib = None

N = 128   # macro-block (Sec. 3.1)
G = 8     # micro-block (Sec. 3.3)


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            from oracle import build as _b
            _b.build(force=True)
        L = ctypes.CDLL(_LIB_PATH)
        L.goq_oracle_half_to_double.restype = ctypes.c_double
        L.goq_oracle_half_to_double.argtypes = [ctypes.c_uint16]
        L.goq_oracle_double_to_half.restype = ctypes.c_uint16
        L.goq_oracle_double_to_half.argtypes = [ctypes.c_double]
        L.goq_oracle_code_value.restype = ctypes.c_double
        L.goq_oracle_code_value.argtypes = [ctypes.c_int, ctypes.c_int]
        L.goq_oracle_max_threads.restype = ctypes.c_int
        _lib = L
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct)) if a is not None else None


def _c(a, dt):
    a = np.ascontiguousarray(a, dtype=dt)
    return a


def max_threads():
    return int(lib().goq_oracle_max_threads())


def lattice(bw):
    L = np.zeros(1 << bw, dtype=np.float64)
    rc = lib().goq_oracle_lattice(ctypes.c_int(bw), _p(L, ctypes.c_double))
    if rc:
        raise ValueError("bad bit width")
    return L


def half_to_double(bits):
    return float(lib().goq_oracle_half_to_double(int(bits)))


def double_to_half(x):
    return int(lib().goq_oracle_double_to_half(float(x)))


def exchange(x, s, signs):
    x = _c(x, np.float64)
    assert x.shape == (G,)
    y = np.zeros(G, dtype=np.float64)
    lib().goq_oracle_exchange(_p(x, ctypes.c_double), ctypes.c_int(s), ctypes.c_int(signs),
                              _p(y, ctypes.c_double))
    return y


def quantize_block(bw, w):
    """One macro-block (128 fp16-valued weights) -> codes, pattern, signs, c1, c2 (fp64, unrounded)."""
    w = _c(w, np.float64)
    assert w.shape == (N,)
    codes = np.zeros(N, np.uint8)
    pat = np.zeros(N // G, np.uint8)
    sg = np.zeros(N // G, np.uint8)
    c1 = ctypes.c_double(0)
    c2 = ctypes.c_double(0)
    lib().goq_oracle_quantize_block(ctypes.c_int(bw), _p(w, ctypes.c_double), _p(codes, ctypes.c_uint8),
                                    _p(pat, ctypes.c_uint8), _p(sg, ctypes.c_uint8),
                                    ctypes.byref(c1), ctypes.byref(c2))
    return codes, pat, sg, c1.value, c2.value


def quantize_geo(bw, w, threads=1):
    """Layer weights [out, in] (fp16-valued) -> canonical arrays dict."""
    w32 = _c(np.asarray(w, dtype=np.float32), np.float32)
    out, inn = w32.shape
    gn = inn // N
    codes = np.zeros((out, inn), np.uint8)
    pat = np.zeros((out, inn // G), np.uint8)
    sg = np.zeros((out, inn // G), np.uint8)
    c1 = np.zeros((out, gn), np.uint16)
    c2 = np.zeros((out, gn), np.uint16)
    rc = lib().goq_oracle_quantize_geo(ctypes.c_int(bw), ctypes.c_int64(out), ctypes.c_int64(inn),
                                       _p(w32, ctypes.c_float), _p(codes, ctypes.c_uint8),
                                       _p(pat, ctypes.c_uint8), _p(sg, ctypes.c_uint8),
                                       _p(c1, ctypes.c_uint16), _p(c2, ctypes.c_uint16),
                                       ctypes.c_int(threads))
    if rc:
        raise ValueError("goq_oracle_quantize_geo failed: %d" % rc)
    return {"bw": bw, "codes": codes, "pattern": pat, "signs": sg, "c1": c1, "c2": c2}


def dequant(q, want=("b1", "b2", "what")):
    out, inn = q["codes"].shape
    B1 = np.zeros((out, inn)) if "b1" in want else None
    B2 = np.zeros((out, inn)) if "b2" in want else None
    Wh = np.zeros((out, inn)) if "what" in want else None
    rc = lib().goq_oracle_dequant(ctypes.c_int(q["bw"]), ctypes.c_int64(out), ctypes.c_int64(inn),
                                  _p(_c(q["codes"], np.uint8), ctypes.c_uint8),
                                  _p(_c(q["pattern"], np.uint8), ctypes.c_uint8),
                                  _p(_c(q["signs"], np.uint8), ctypes.c_uint8),
                                  _p(_c(q["c1"], np.uint16), ctypes.c_uint16),
                                  _p(_c(q["c2"], np.uint16), ctypes.c_uint16),
                                  _p(B1, ctypes.c_double), _p(B2, ctypes.c_double), _p(Wh, ctypes.c_double))
    if rc:
        raise ValueError("goq_oracle_dequant failed: %d" % rc)
    return {"b1": B1, "b2": B2, "what": Wh}


def gemm_a16(q, x_f16, threads=1):
    """x_f16: float16 [tokens, in] -> y fp64 [tokens, out]."""
    x = _c(np.asarray(x_f16, dtype=np.float16), np.float16)
    if x.ndim == 1:
        x = x[None, :]
    tokens, inn = x.shape
    out = q["codes"].shape[0]
    assert q["codes"].shape[1] == inn
    y = np.zeros((tokens, out), np.float64)
    xb = x.view(np.uint16)
    rc = lib().goq_oracle_gemm_a16(ctypes.c_int(q["bw"]), ctypes.c_int64(tokens), ctypes.c_int64(out),
                                   ctypes.c_int64(inn),
                                   _p(_c(q["codes"], np.uint8), ctypes.c_uint8),
                                   _p(_c(q["pattern"], np.uint8), ctypes.c_uint8),
                                   _p(_c(q["signs"], np.uint8), ctypes.c_uint8),
                                   _p(_c(q["c1"], np.uint16), ctypes.c_uint16),
                                   _p(_c(q["c2"], np.uint16), ctypes.c_uint16),
                                   _p(xb, ctypes.c_uint16), _p(y, ctypes.c_double), ctypes.c_int(threads))
    if rc:
        raise ValueError("goq_oracle_gemm_a16 failed: %d" % rc)
    return y


def gemm_a8(q, x_i8, sx, threads=1, want_partials=False):
    """x_i8: int8 [tokens, in]; sx: float32 [tokens] -> (y fp64 [tokens,out], partials int32 or None)."""
    x = _c(np.asarray(x_i8, dtype=np.int8), np.int8)
    if x.ndim == 1:
        x = x[None, :]
    tokens, inn = x.shape
    out = q["codes"].shape[0]
    gn = inn // N
    sxa = _c(np.asarray(sx, dtype=np.float32).reshape(-1), np.float32)
    assert sxa.shape[0] == tokens
    y = np.zeros((tokens, out), np.float64)
    parts = np.zeros((tokens, out, gn, 2), np.int32) if want_partials else None
    rc = lib().goq_oracle_gemm_a8(ctypes.c_int(q["bw"]), ctypes.c_int64(tokens), ctypes.c_int64(out),
                                  ctypes.c_int64(inn),
                                  _p(_c(q["codes"], np.uint8), ctypes.c_uint8),
                                  _p(_c(q["pattern"], np.uint8), ctypes.c_uint8),
                                  _p(_c(q["signs"], np.uint8), ctypes.c_uint8),
                                  _p(_c(q["c1"], np.uint16), ctypes.c_uint16),
                                  _p(_c(q["c2"], np.uint16), ctypes.c_uint16),
                                  _p(x, ctypes.c_int8), _p(sxa, ctypes.c_float), _p(y, ctypes.c_double),
                                  _p(parts, ctypes.c_int32), ctypes.c_int(threads))
    if rc:
        raise ValueError("goq_oracle_gemm_a8 failed: %d" % rc)
    return y, parts


def ref_coefficients(q, w, x_f16, lam=1e-4, threads=1):
    """REF mode (Eq. 3): canonical arrays q (bases), fp16-valued weights w [out, in], calibration
    inputs x_f16 [tokens, in] -> (dict like q with the re-solved c1, c2, unrounded c [out, gn, 2])."""
    w32 = _c(np.asarray(w, dtype=np.float32), np.float32)
    x = _c(np.asarray(x_f16, dtype=np.float16), np.float16)
    tokens, inn = x.shape
    out = q["codes"].shape[0]
    assert w32.shape == (out, inn) and q["codes"].shape[1] == inn
    gn = inn // N
    craw = np.zeros((out, gn, 2), np.float64)
    c1 = np.zeros((out, gn), np.uint16)
    c2 = np.zeros((out, gn), np.uint16)
    rc = lib().goq_oracle_ref_coefficients(ctypes.c_int(q["bw"]), ctypes.c_int64(tokens), ctypes.c_int64(out),
                                           ctypes.c_int64(inn), _p(w32, ctypes.c_float),
                                           _p(_c(q["codes"], np.uint8), ctypes.c_uint8),
                                           _p(_c(q["pattern"], np.uint8), ctypes.c_uint8),
                                           _p(_c(q["signs"], np.uint8), ctypes.c_uint8),
                                           _p(x.view(np.uint16), ctypes.c_uint16), ctypes.c_double(lam),
                                           _p(craw, ctypes.c_double), _p(c1, ctypes.c_uint16),
                                           _p(c2, ctypes.c_uint16), ctypes.c_int(threads))
    if rc:
        raise ValueError("goq_oracle_ref_coefficients failed: %d" % rc)
    r = dict(q)
    r["c1"], r["c2"] = c1, c2
    return r, craw
