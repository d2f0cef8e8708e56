"""ctypes front end of the C++ oracle (numpy arrays in, numpy arrays out).

TEST INFRASTRUCTURE ONLY: used by tests, the smoke check and the benchmark's
CPU-baseline leg.  Formats are named "p8", "p16", "p32" (posit<8,0>, <16,1>,
<32,2>, Table 1) and "p8_1", "p8_2", "p10_1", "p10_2", "p12_1", "p12_2" (Sec. 4)."""
import ctypes
import os

import numpy as np

from . import build as _build

CODES = {"p8": 0, "p16": 1, "p32": 2, "p8_1": 3, "p8_2": 4, "p10_1": 5, "p10_2": 6, "p12_1": 7, "p12_2": 8}
DTYPES = {"p8": np.uint8, "p16": np.uint16, "p32": np.uint32, "p8_1": np.uint8, "p8_2": np.uint8, "p10_1": np.uint16,
          "p10_2": np.uint16, "p12_1": np.uint16, "p12_2": np.uint16}

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = ctypes.CDLL(path)
        i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        L.oracle_gemm.argtypes = [ci, ci, ci, ci, i64, i64, i64, vp, i64, vp, i64, vp, vp, i64, i64, i64, ci, ctypes.POINTER(i64), ci]
        L.oracle_conv2d_fwd.argtypes = [ci, ci, ctypes.POINTER(i64), vp, vp, vp, vp, ci, ci]
        L.oracle_conv2d_bwd_data.argtypes = [ci, ci, ctypes.POINTER(i64), vp, vp, vp, ci, ci]
        L.oracle_conv2d_bwd_weight.argtypes = [ci, ci, ctypes.POINTER(i64), vp, vp, vp, vp, ci, ci]
        L.oracle_round_f32.argtypes = [ci, i64, vp, vp]
        L.oracle_round_f64.argtypes = [ci, i64, vp, vp]
        L.oracle_convert.argtypes = [ci, ci, i64, vp, vp]
        L.oracle_to_f32.argtypes = [ci, i64, vp, vp]
        L.oracle_to_f64.argtypes = [ci, i64, vp, vp]
        L.oracle_axpy.argtypes = [ci, ci, ctypes.c_uint32, i64, vp, vp, ci, vp]
        _lib = L
    return _lib


def hw_threads():
    return int(lib().oracle_hw_threads())


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _arr(a, fmt):
    a = np.ascontiguousarray(a, dtype=DTYPES[fmt])
    return a


def gemm(A, B, fin, fout, trans_a=False, trans_b=False, bias=None, rows=None, threads=None, noquire=False):
    """Returns C (and the number of outputs whose exact sum left the quire range).

    noquire (here and in the convolutions): no quire; every product and partial sum is rounded to fin, terms in
    order of the reduction index, bias last (Sec. 3.3: the quire is an option; Table 2)."""
    A, B = _arr(A, fin), _arr(B, fin)
    M, K = (A.shape[1], A.shape[0]) if trans_a else A.shape
    N = B.shape[0] if trans_b else B.shape[1]
    assert (B.shape[1] if trans_b else B.shape[0]) == K
    bias = None if bias is None else _arr(bias, fin)
    C = np.zeros((M, N), dtype=DTYPES[fout])
    lo, hi = (0, M) if rows is None else rows
    ovf = ctypes.c_int64(0)
    rc = lib().oracle_gemm(CODES[fin], CODES[fout], int(trans_a), int(trans_b), M, N, K, _ptr(A), A.shape[1],
                           _ptr(B), B.shape[1], _ptr(bias), _ptr(C), N, lo, hi, threads or hw_threads(), ctypes.byref(ovf), int(noquire))
    assert rc == 0
    return C, ovf.value


def _desc(d):
    vals = [d["N"], d["C"], d["H"], d["W"], d["K"], d["R"], d["S"], d.get("pad_h", 0), d.get("pad_w", 0),
            d.get("stride_h", 1), d.get("stride_w", 1)]
    return (ctypes.c_int64 * 11)(*vals)


def out_hw(d):
    oh = (d["H"] + 2 * d.get("pad_h", 0) - d["R"]) // d.get("stride_h", 1) + 1
    ow = (d["W"] + 2 * d.get("pad_w", 0) - d["S"]) // d.get("stride_w", 1) + 1
    return oh, ow


def conv2d_fwd(x, w, d, fin, fout, bias=None, threads=None, noquire=False):
    x, w = _arr(x, fin), _arr(w, fin)
    bias = None if bias is None else _arr(bias, fin)
    oh, ow = out_hw(d)
    y = np.zeros((d["N"], d["K"], oh, ow), dtype=DTYPES[fout])
    rc = lib().oracle_conv2d_fwd(CODES[fin], CODES[fout], _desc(d), _ptr(x), _ptr(w), _ptr(bias), _ptr(y), threads or hw_threads(), int(noquire))
    assert rc == 0
    return y


def conv2d_bwd_data(dy, w, d, fin, fout, threads=None, noquire=False):
    dy, w = _arr(dy, fin), _arr(w, fin)
    dx = np.zeros((d["N"], d["C"], d["H"], d["W"]), dtype=DTYPES[fout])
    rc = lib().oracle_conv2d_bwd_data(CODES[fin], CODES[fout], _desc(d), _ptr(dy), _ptr(w), _ptr(dx), threads or hw_threads(), int(noquire))
    assert rc == 0
    return dx


def conv2d_bwd_weight(dy, x, d, fin, fout, with_bias=False, threads=None, noquire=False):
    dy, x = _arr(dy, fin), _arr(x, fin)
    dw = np.zeros((d["K"], d["C"], d["R"], d["S"]), dtype=DTYPES[fout])
    db = np.zeros((d["K"],), dtype=DTYPES[fout]) if with_bias else None
    rc = lib().oracle_conv2d_bwd_weight(CODES[fin], CODES[fout], _desc(d), _ptr(dy), _ptr(x), _ptr(dw), _ptr(db), threads or hw_threads(), int(noquire))
    assert rc == 0
    return (dw, db) if with_bias else dw


def round_from_float(src, fdst):
    src = np.ascontiguousarray(src)
    out = np.zeros(src.shape, dtype=DTYPES[fdst])
    if src.dtype == np.float32:
        rc = lib().oracle_round_f32(CODES[fdst], src.size, _ptr(src), _ptr(out))
    elif src.dtype == np.float64:
        rc = lib().oracle_round_f64(CODES[fdst], src.size, _ptr(src), _ptr(out))
    else:
        raise TypeError(src.dtype)
    assert rc == 0
    return out


def convert(src, fsrc, fdst):
    src = _arr(src, fsrc)
    out = np.zeros(src.shape, dtype=DTYPES[fdst])
    assert lib().oracle_convert(CODES[fsrc], CODES[fdst], src.size, _ptr(src), _ptr(out)) == 0
    return out


def to_float(src, fsrc, kind="f32"):
    src = _arr(src, fsrc)
    if kind == "f32":
        out = np.zeros(src.shape, dtype=np.float32)
        assert lib().oracle_to_f32(CODES[fsrc], src.size, _ptr(src), _ptr(out)) == 0
    else:
        out = np.zeros(src.shape, dtype=np.float64)
        assert lib().oracle_to_f64(CODES[fsrc], src.size, _ptr(src), _ptr(out)) == 0
    return out


def axpy(alpha, x, y, fx, fy, fcopy=None):
    """Returns new y (and the narrowed copy when fcopy is given); inputs are not modified."""
    x = _arr(x, fx)
    ynew = np.array(_arr(y, fy), copy=True)
    cp = np.zeros(ynew.shape, dtype=DTYPES[fcopy]) if fcopy else None
    rc = lib().oracle_axpy(CODES[fx], CODES[fy], int(alpha), x.size, _ptr(x), _ptr(ynew), CODES[fcopy] if fcopy else -1, _ptr(cp))
    assert rc == 0
    return (ynew, cp) if fcopy else ynew
