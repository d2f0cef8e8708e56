"""Thin Python binding of the C ABI declared in include/positnn.h.

Argument marshalling only: torch tensors provide device memory and the current
HIP stream; every computation happens inside libpositnn_hip.so.  There is no
CPU fallback: a missing library or a non-device tensor is an error.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libpositnn_hip.so")

P8, P16, P32, F32, F64 = 0, 1, 2, 100, 101
P8_1, P8_2, P10_1, P10_2, P12_1, P12_2 = 3, 4, 5, 6, 7, 8  # formats of the paper's experiments outside Table 1
FORMAT_BITS = {"p8": 8, "p16": 16, "p32": 32, "p8_1": 8, "p8_2": 8, "p10_1": 10, "p10_2": 10, "p12_1": 12, "p12_2": 12}
FORMAT_CODES = {"p8": P8, "p16": P16, "p32": P32, "f32": F32, "f64": F64, "p8_1": P8_1, "p8_2": P8_2, "p10_1": P10_1,
                "p10_2": P10_2, "p12_1": P12_1, "p12_2": P12_2}
TORCH_DTYPE = {P8: torch.uint8, P16: torch.uint16, P32: torch.uint32, F32: torch.float32, F64: torch.float64,
               P8_1: torch.uint8, P8_2: torch.uint8, P10_1: torch.uint16, P10_2: torch.uint16, P12_1: torch.uint16, P12_2: torch.uint16}
ELEM_SIZE = {P8: 1, P16: 2, P32: 4, F32: 4, F64: 8, P8_1: 1, P8_2: 1, P10_1: 2, P10_2: 2, P12_1: 2, P12_2: 2}
# signed views are accepted too (same bits)
_SAME_SIZE = {1: (torch.uint8, torch.int8), 2: (torch.uint16, torch.int16), 4: (torch.uint32, torch.int32, torch.float32),
              8: (torch.float64, torch.int64, torch.uint64)}


class AxpyItem(ctypes.Structure):
    _fields_ = [("x", ctypes.c_void_p), ("y", ctypes.c_void_p), ("y_copy", ctypes.c_void_p), ("n", ctypes.c_int64)]


class ConvDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int64) for n in ("N", "C", "H", "W", "K", "R", "S", "pad_h", "pad_w", "stride_h", "stride_w")]


class PositError(RuntimeError):
    pass


_lib = None


def load():
    """Load the shared library (built by paper_2105_00053_amd.build); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise PositError("libpositnn_hip.so is not built: run `python -m paper_2105_00053_amd.build`")
    L = ctypes.CDLL(_LIB_PATH)
    vp, i64, ci, sz, u32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t, ctypes.c_uint32
    L.posit_gemm.argtypes = [vp, ci, ci, ci, ci, i64, i64, i64, vp, i64, vp, i64, vp, vp, i64, vp, sz]
    L.posit_gemm.restype = ci
    L.posit_gemm_static.argtypes = [vp, ci, ci, ci, ci, i64, i64, i64, vp, i64, vp, i64, vp, vp, i64]
    L.posit_gemm_static.restype = ci
    L.posit_gemm_workspace.argtypes = [ci, ci, ci, ci, i64, i64, i64]
    L.posit_gemm_workspace.restype = sz
    dp = ctypes.POINTER(ConvDesc)
    L.posit_conv2d_fwd.argtypes = [vp, ci, ci, dp, vp, vp, vp, vp, vp, sz]
    L.posit_conv2d_bwd_data.argtypes = [vp, ci, ci, dp, vp, vp, vp, vp, sz]
    L.posit_conv2d_bwd_weight.argtypes = [vp, ci, ci, dp, vp, vp, vp, vp, vp, sz]
    L.posit_conv2d_workspace.argtypes = [ci, ci, ci, dp]
    L.posit_conv2d_workspace.restype = sz
    L.posit_round.argtypes = [vp, ci, ci, i64, vp, vp]
    L.posit_convert.argtypes = [vp, ci, ci, i64, vp, vp]
    L.posit_axpy.argtypes = [vp, ci, ci, u32, i64, vp, vp, ci, vp]
    L.posit_relu.argtypes = [vp, ci, i64, vp, vp]
    L.posit_relu_bwd.argtypes = [vp, ci, ci, i64, vp, vp, vp]
    L.posit_maxpool2d_fwd.argtypes = [vp, ci, i64, i64, i64, i64, i64, vp, vp, vp]
    L.posit_maxpool2d_bwd.argtypes = [vp, ci, i64, i64, i64, i64, i64, vp, vp, vp]
    L.posit_avgpool2d_fwd.argtypes = [vp, ci, ci, i64, i64, i64, i64, i64, vp, vp]
    L.posit_avgpool2d_bwd.argtypes = [vp, ci, ci, i64, i64, i64, i64, i64, vp, vp]
    L.posit_gemm_noquire.argtypes = [vp, ci, ci, ci, ci, i64, i64, i64, vp, i64, vp, i64, vp, vp, i64]
    L.posit_conv2d_fwd_noquire.argtypes = [vp, ci, ci, dp, vp, vp, vp, vp]
    L.posit_conv2d_bwd_data_noquire.argtypes = [vp, ci, ci, dp, vp, vp, vp]
    L.posit_conv2d_bwd_weight_noquire.argtypes = [vp, ci, ci, dp, vp, vp, vp, vp]
    L.posit_axpy_multi.argtypes = [vp, ci, ci, u32, ci, ctypes.POINTER(AxpyItem), ci]
    L.posit_unary.argtypes = [vp, ci, ci, i64, vp, vp]
    L.posit_unary_bwd.argtypes = [vp, ci, ci, ci, i64, vp, vp, vp]
    L.posit_cross_entropy.argtypes = [vp, ci, ci, ci, i64, i64, vp, vp, vp, vp]
    L.posit_mse.argtypes = [vp, ci, ci, ci, i64, vp, vp, vp, vp]
    L.posit_status_string.argtypes = [ci]
    L.posit_status_string.restype = ctypes.c_char_p
    for name in ("posit_conv2d_fwd", "posit_conv2d_bwd_data", "posit_conv2d_bwd_weight", "posit_round", "posit_convert", "posit_axpy",
                 "posit_gemm_noquire", "posit_conv2d_fwd_noquire", "posit_conv2d_bwd_data_noquire", "posit_conv2d_bwd_weight_noquire",
                 "posit_axpy_multi", "posit_unary", "posit_unary_bwd", "posit_cross_entropy", "posit_mse",
                 "posit_relu", "posit_relu_bwd", "posit_maxpool2d_fwd", "posit_maxpool2d_bwd", "posit_avgpool2d_fwd", "posit_avgpool2d_bwd"):
        getattr(L, name).restype = ci
    _lib = L
    return L


def _code(f):
    return FORMAT_CODES[f] if isinstance(f, str) else int(f)


def _check(status):
    if status != 0:
        raise PositError("positnn: %s (status %d)" % (load().posit_status_string(status).decode(), status))


def _dev(t, fmt, name):
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise PositError("%s must be a device tensor" % name)
    if not t.is_contiguous():
        raise PositError("%s must be contiguous" % name)
    if t.dtype not in _SAME_SIZE[ELEM_SIZE[fmt]]:
        raise PositError("%s has dtype %s, expected %d-byte elements" % (name, t.dtype, ELEM_SIZE[fmt]))
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _workspace(nbytes, device, workspace):
    if nbytes == 0:
        return None, 0, None
    if workspace is None:
        workspace = torch.empty(nbytes, dtype=torch.uint8, device=device)
    elif workspace.numel() * workspace.element_size() < nbytes:
        raise PositError("workspace too small: need %d bytes" % nbytes)
    return ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size(), workspace


def posit_gemm_workspace(fin, fout, trans_a, trans_b, M, N, K):
    return int(load().posit_gemm_workspace(_code(fin), _code(fout), int(trans_a), int(trans_b), M, N, K))


def posit_gemm(A, B, fin, fout, trans_a=False, trans_b=False, bias=None, out=None, workspace=None):
    """C = round_fout(op(A) @ op(B) (+ bias)), 2-D row-major device tensors of patterns."""
    fin, fout = _code(fin), _code(fout)
    if A.dim() != 2 or B.dim() != 2:
        raise PositError("A and B must be 2-D")
    M, K = (A.shape[1], A.shape[0]) if trans_a else (A.shape[0], A.shape[1])
    N, Kb = (B.shape[0], B.shape[1]) if trans_b else (B.shape[1], B.shape[0])
    if K != Kb:
        raise PositError("inner dimensions differ: %d vs %d" % (K, Kb))
    if bias is not None and bias.numel() != N:
        raise PositError("bias must have N elements")
    if out is None:
        out = torch.empty((M, N), dtype=TORCH_DTYPE[fout], device=A.device)
    need = posit_gemm_workspace(fin, fout, trans_a, trans_b, M, N, K)
    wp, wbytes, _keep = _workspace(need, A.device, workspace)
    _check(load().posit_gemm(_stream(), fin, fout, int(trans_a), int(trans_b), M, N, K,
                             _dev(A, fin, "A"), A.shape[1], _dev(B, fin, "B"), B.shape[1], _dev(bias, fin, "bias"),
                             _dev(out, fout, "out"), out.shape[1], wp, wbytes))
    return out


def posit_gemm_static(A, B, fin, fout, trans_a=False, trans_b=False, bias=None, out=None):
    """posit_gemm with the library's own fixed scratch array as workspace: the call allocates nothing
    when `out` is given.  Calls that overlap in time on one GPU race on that array."""
    fin, fout = _code(fin), _code(fout)
    if A.dim() != 2 or B.dim() != 2:
        raise PositError("A and B must be 2-D")
    M, K = (A.shape[1], A.shape[0]) if trans_a else (A.shape[0], A.shape[1])
    N, Kb = (B.shape[0], B.shape[1]) if trans_b else (B.shape[1], B.shape[0])
    if K != Kb:
        raise PositError("inner dimensions differ: %d vs %d" % (K, Kb))
    if bias is not None and bias.numel() != N:
        raise PositError("bias must have N elements")
    if out is None:
        out = torch.empty((M, N), dtype=TORCH_DTYPE[fout], device=A.device)
    _check(load().posit_gemm_static(_stream(), fin, fout, int(trans_a), int(trans_b), M, N, K,
                                    _dev(A, fin, "A"), A.shape[1], _dev(B, fin, "B"), B.shape[1], _dev(bias, fin, "bias"),
                                    _dev(out, fout, "out"), out.shape[1]))
    return out


def conv_desc(x_shape, w_shape, padding=(0, 0), stride=(1, 1)):
    n, c, h, w = x_shape
    k, c2, r, s = w_shape
    if c != c2:
        raise PositError("channel mismatch")
    return ConvDesc(n, c, h, w, k, r, s, padding[0], padding[1], stride[0], stride[1])


def conv_out_hw(d):
    return (d.H + 2 * d.pad_h - d.R) // d.stride_h + 1, (d.W + 2 * d.pad_w - d.S) // d.stride_w + 1


def posit_conv2d_workspace(which, fin, fout, desc):
    return int(load().posit_conv2d_workspace(int(which), _code(fin), _code(fout), ctypes.byref(desc)))


def posit_conv2d_fwd(x, w, desc, fin, fout, bias=None, out=None, workspace=None):
    fin, fout = _code(fin), _code(fout)
    oh, ow = conv_out_hw(desc)
    if out is None:
        out = torch.empty((desc.N, desc.K, oh, ow), dtype=TORCH_DTYPE[fout], device=x.device)
    wp, wbytes, _keep = _workspace(posit_conv2d_workspace(0, fin, fout, desc), x.device, workspace)
    _check(load().posit_conv2d_fwd(_stream(), fin, fout, ctypes.byref(desc), _dev(x, fin, "x"), _dev(w, fin, "w"),
                                   _dev(bias, fin, "bias"), _dev(out, fout, "y"), wp, wbytes))
    return out


def posit_conv2d_bwd_data(dy, w, desc, fin, fout, out=None, workspace=None):
    fin, fout = _code(fin), _code(fout)
    if out is None:
        out = torch.empty((desc.N, desc.C, desc.H, desc.W), dtype=TORCH_DTYPE[fout], device=dy.device)
    wp, wbytes, _keep = _workspace(posit_conv2d_workspace(1, fin, fout, desc), dy.device, workspace)
    _check(load().posit_conv2d_bwd_data(_stream(), fin, fout, ctypes.byref(desc), _dev(dy, fin, "dy"), _dev(w, fin, "w"),
                                        _dev(out, fout, "dx"), wp, wbytes))
    return out


def posit_conv2d_bwd_weight(dy, x, desc, fin, fout, with_bias=False, out=None, out_bias=None, workspace=None):
    fin, fout = _code(fin), _code(fout)
    if out is None:
        out = torch.empty((desc.K, desc.C, desc.R, desc.S), dtype=TORCH_DTYPE[fout], device=dy.device)
    if with_bias and out_bias is None:
        out_bias = torch.empty((desc.K,), dtype=TORCH_DTYPE[fout], device=dy.device)
    wp, wbytes, _keep = _workspace(posit_conv2d_workspace(2, fin, fout, desc), dy.device, workspace)
    _check(load().posit_conv2d_bwd_weight(_stream(), fin, fout, ctypes.byref(desc), _dev(dy, fin, "dy"), _dev(x, fin, "x"),
                                          _dev(out, fout, "dw"), _dev(out_bias, fout, "dbias") if with_bias else None, wp, wbytes))
    return (out, out_bias) if with_bias else out


def posit_gemm_noquire(A, B, fin, fout, trans_a=False, trans_b=False, bias=None, out=None):
    """As posit_gemm with the quire switched off: every product and running sum rounded to fin, k ascending, bias last."""
    fin, fout = _code(fin), _code(fout)
    if A.dim() != 2 or B.dim() != 2:
        raise PositError("A and B must be 2-D")
    M, K = (A.shape[1], A.shape[0]) if trans_a else (A.shape[0], A.shape[1])
    N, Kb = (B.shape[0], B.shape[1]) if trans_b else (B.shape[1], B.shape[0])
    if K != Kb:
        raise PositError("inner dimensions differ: %d vs %d" % (K, Kb))
    if bias is not None and bias.numel() != N:
        raise PositError("bias must have N elements")
    if out is None:
        out = torch.empty((M, N), dtype=TORCH_DTYPE[fout], device=A.device)
    _check(load().posit_gemm_noquire(_stream(), fin, fout, int(trans_a), int(trans_b), M, N, K,
                                     _dev(A, fin, "A"), A.shape[1], _dev(B, fin, "B"), B.shape[1], _dev(bias, fin, "bias"),
                                     _dev(out, fout, "out"), out.shape[1]))
    return out


def posit_conv2d_fwd_noquire(x, w, desc, fin, fout, bias=None, out=None):
    fin, fout = _code(fin), _code(fout)
    oh, ow = conv_out_hw(desc)
    if out is None:
        out = torch.empty((desc.N, desc.K, oh, ow), dtype=TORCH_DTYPE[fout], device=x.device)
    _check(load().posit_conv2d_fwd_noquire(_stream(), fin, fout, ctypes.byref(desc), _dev(x, fin, "x"), _dev(w, fin, "w"),
                                           _dev(bias, fin, "bias"), _dev(out, fout, "y")))
    return out


def posit_conv2d_bwd_data_noquire(dy, w, desc, fin, fout, out=None):
    fin, fout = _code(fin), _code(fout)
    if out is None:
        out = torch.empty((desc.N, desc.C, desc.H, desc.W), dtype=TORCH_DTYPE[fout], device=dy.device)
    _check(load().posit_conv2d_bwd_data_noquire(_stream(), fin, fout, ctypes.byref(desc), _dev(dy, fin, "dy"), _dev(w, fin, "w"),
                                                _dev(out, fout, "dx")))
    return out


def posit_conv2d_bwd_weight_noquire(dy, x, desc, fin, fout, with_bias=False, out=None, out_bias=None):
    fin, fout = _code(fin), _code(fout)
    if out is None:
        out = torch.empty((desc.K, desc.C, desc.R, desc.S), dtype=TORCH_DTYPE[fout], device=dy.device)
    if with_bias and out_bias is None:
        out_bias = torch.empty((desc.K,), dtype=TORCH_DTYPE[fout], device=dy.device)
    _check(load().posit_conv2d_bwd_weight_noquire(_stream(), fin, fout, ctypes.byref(desc), _dev(dy, fin, "dy"), _dev(x, fin, "x"),
                                                  _dev(out, fout, "dw"), _dev(out_bias, fout, "dbias") if with_bias else None))
    return (out, out_bias) if with_bias else out


def posit_axpy_multi(alpha_bits, xs, ys, fx, fy, fcopy=None, y_copies=None):
    """posit_axpy over lists of tensors in one launch (in place on ys; y_copies entries may be None)."""
    fx, fy = _code(fx), _code(fy)
    fc = _code(fcopy) if fcopy is not None else fy
    if len(xs) != len(ys) or (y_copies is not None and len(y_copies) != len(ys)):
        raise PositError("lists of different lengths")
    items = (AxpyItem * max(1, len(xs)))()
    for i, (x, y) in enumerate(zip(xs, ys)):
        if x.numel() != y.numel():
            raise PositError("x and y of item %d differ in size" % i)
        c = y_copies[i] if y_copies is not None else None
        if c is not None and c.numel() != y.numel():
            raise PositError("copy of item %d differs in size" % i)
        items[i].x = _dev(x, fx, "x").value
        items[i].y = _dev(y, fy, "y").value
        items[i].y_copy = _dev(c, fc, "y_copy").value if c is not None else None
        items[i].n = y.numel()
    _check(load().posit_axpy_multi(_stream(), fx, fy, int(alpha_bits) & 0xFFFFFFFF, len(xs), items, fc))


FUNCTIONS = {"sigmoid": 0, "tanh": 1, "exp": 2, "log": 3}


def posit_unary(fn, x, fmt, out=None):
    """y = correctly rounded fn(x) elementwise; fn in "sigmoid", "tanh", "exp", "log"."""
    fmt = _code(fmt)
    if out is None:
        out = torch.empty_like(x)
    _check(load().posit_unary(_stream(), FUNCTIONS[fn], fmt, x.numel(), _dev(x, fmt, "x"), _dev(out, fmt, "y")))
    return out


def posit_unary_bwd(fn, y_fwd, dy, fmt_y, fmt_d, out=None):
    fmt_y, fmt_d = _code(fmt_y), _code(fmt_d)
    if out is None:
        out = torch.empty_like(dy)
    _check(load().posit_unary_bwd(_stream(), FUNCTIONS[fn], fmt_y, fmt_d, dy.numel(), _dev(y_fwd, fmt_y, "y_fwd"),
                                  _dev(dy, fmt_d, "dy"), _dev(out, fmt_d, "dx")))
    return out


def posit_cross_entropy(logits, labels, f_logits, f_loss, f_grad, want_loss=True, want_grad=True):
    """Returns (loss, dlogits): loss a 1-element tensor of f_loss, dlogits [batch][classes] of f_grad (None when not wanted).
    labels: int32 device tensor."""
    f_logits, f_loss, f_grad = _code(f_logits), _code(f_loss), _code(f_grad)
    if logits.dim() != 2 or labels.dtype != torch.int32 or labels.numel() != logits.shape[0] or not labels.is_contiguous() or not labels.is_cuda:
        raise PositError("logits must be [batch][classes] and labels a contiguous int32 device tensor with one entry per row")
    loss = torch.empty((1,), dtype=TORCH_DTYPE[f_loss], device=logits.device) if want_loss else None
    grad = torch.empty(tuple(logits.shape), dtype=TORCH_DTYPE[f_grad], device=logits.device) if want_grad else None
    _check(load().posit_cross_entropy(_stream(), f_logits, f_loss, f_grad, logits.shape[0], logits.shape[1], _dev(logits, f_logits, "logits"),
                                      labels.data_ptr(), _dev(loss, f_loss, "loss") if want_loss else None,
                                      _dev(grad, f_grad, "dlogits") if want_grad else None))
    return loss, grad


def posit_mse(pred, target, f_pred, f_loss, f_grad, want_loss=True, want_grad=True):
    f_pred, f_loss, f_grad = _code(f_pred), _code(f_loss), _code(f_grad)
    loss = torch.empty((1,), dtype=TORCH_DTYPE[f_loss], device=pred.device) if want_loss else None
    grad = torch.empty(tuple(pred.shape), dtype=TORCH_DTYPE[f_grad], device=pred.device) if want_grad else None
    _check(load().posit_mse(_stream(), f_pred, f_loss, f_grad, pred.numel(), _dev(pred, f_pred, "pred"), _dev(target, f_pred, "target"),
                            _dev(loss, f_loss, "loss") if want_loss else None, _dev(grad, f_grad, "dpred") if want_grad else None))
    return loss, grad


def posit_round(src, fdst, out=None):
    """float32 / float64 device tensor -> tensor of posit patterns."""
    fdst = _code(fdst)
    fsrc = F32 if src.dtype == torch.float32 else F64 if src.dtype == torch.float64 else None
    if fsrc is None:
        raise PositError("posit_round takes float32 or float64")
    if out is None:
        out = torch.empty(src.shape, dtype=TORCH_DTYPE[fdst], device=src.device)
    _check(load().posit_round(_stream(), fsrc, fdst, src.numel(), _dev(src, fsrc, "src"), _dev(out, fdst, "dst")))
    return out


def posit_convert(src, fsrc, fdst, out=None):
    """posit -> posit of another format, or posit -> float32 / float64."""
    fsrc, fdst = _code(fsrc), _code(fdst)
    if out is None:
        out = torch.empty(src.shape, dtype=TORCH_DTYPE[fdst], device=src.device)
    _check(load().posit_convert(_stream(), fsrc, fdst, src.numel(), _dev(src, fsrc, "src"), _dev(out, fdst, "dst")))
    return out


def posit_axpy(alpha_bits, x, y, fx, fy, fcopy=None, y_copy=None):
    """In place y <- round(y + alpha * x); optionally also writes the narrowed copy of the new y."""
    fx, fy = _code(fx), _code(fy)
    if x.numel() != y.numel():
        raise PositError("x and y differ in size")
    fc = -1
    if fcopy is not None:
        fc = _code(fcopy)
        if y_copy is None:
            y_copy = torch.empty(y.shape, dtype=TORCH_DTYPE[fc], device=y.device)
    _check(load().posit_axpy(_stream(), fx, fy, int(alpha_bits) & 0xFFFFFFFF, y.numel(), _dev(x, fx, "x"), _dev(y, fy, "y"),
                             fc, _dev(y_copy, fc, "y_copy") if fcopy is not None else None))
    return (y, y_copy) if fcopy is not None else y


def posit_relu(x, fmt, out=None):
    fmt = _code(fmt)
    if out is None:
        out = torch.empty_like(x)
    _check(load().posit_relu(_stream(), fmt, x.numel(), _dev(x, fmt, "x"), _dev(out, fmt, "y")))
    return out


def posit_relu_bwd(y_fwd, dy, fmt_y, fmt_d, out=None):
    fmt_y, fmt_d = _code(fmt_y), _code(fmt_d)
    if y_fwd.numel() != dy.numel():
        raise PositError("y_fwd and dy differ in size")
    if out is None:
        out = torch.empty_like(dy)
    _check(load().posit_relu_bwd(_stream(), fmt_y, fmt_d, dy.numel(), _dev(y_fwd, fmt_y, "y_fwd"), _dev(dy, fmt_d, "dy"), _dev(out, fmt_d, "dx")))
    return out


def _planes(x):
    if x.dim() < 2:
        raise PositError("pooling takes [..., H, W] tensors")
    h, w = x.shape[-2], x.shape[-1]
    return x.numel() // (h * w) if h * w else 0, h, w


def posit_maxpool2d_fwd(x, fmt, kh=2, kw=2):
    """Returns (y, idx): idx is the uint8 window position of the first maximum."""
    fmt = _code(fmt)
    planes, h, w = _planes(x)
    shape = tuple(x.shape[:-2]) + (h // kh, w // kw)
    y = torch.empty(shape, dtype=x.dtype, device=x.device)
    idx = torch.empty(shape, dtype=torch.uint8, device=x.device)
    _check(load().posit_maxpool2d_fwd(_stream(), fmt, planes, h, w, kh, kw, _dev(x, fmt, "x"), _dev(y, fmt, "y"), _dev(idx, P8, "idx")))
    return y, idx


def posit_maxpool2d_bwd(dy, idx, fmt, kh=2, kw=2):
    fmt = _code(fmt)
    planes, oh, ow = _planes(dy)
    shape = tuple(dy.shape[:-2]) + (oh * kh, ow * kw)
    dx = torch.empty(shape, dtype=dy.dtype, device=dy.device)
    _check(load().posit_maxpool2d_bwd(_stream(), fmt, planes, oh * kh, ow * kw, kh, kw, _dev(dy, fmt, "dy"), _dev(idx, P8, "idx"), _dev(dx, fmt, "dx")))
    return dx


def posit_avgpool2d_fwd(x, fin, fout, kh=2, kw=2):
    fin, fout = _code(fin), _code(fout)
    planes, h, w = _planes(x)
    y = torch.empty(tuple(x.shape[:-2]) + (h // kh, w // kw), dtype=TORCH_DTYPE[fout], device=x.device)
    _check(load().posit_avgpool2d_fwd(_stream(), fin, fout, planes, h, w, kh, kw, _dev(x, fin, "x"), _dev(y, fout, "y")))
    return y


def posit_avgpool2d_bwd(dy, fin, fout, kh=2, kw=2):
    fin, fout = _code(fin), _code(fout)
    planes, oh, ow = _planes(dy)
    dx = torch.empty(tuple(dy.shape[:-2]) + (oh * kh, ow * kw), dtype=TORCH_DTYPE[fout], device=dy.device)
    _check(load().posit_avgpool2d_bwd(_stream(), fin, fout, planes, oh * kh, ow * kw, kh, kw, _dev(dy, fin, "dy"), _dev(dx, fout, "dx")))
    return dx
