"""Layer-by-layer training step for the LeNet-5-shaped and CifarNet-shaped configs.

Every quire dot product (convolutions, linear layers, their two backward passes, bias
gradients, average pooling as a convolution with four weights of 1/4, the SGD update) is
run twice on identical inputs: through the GPU library and through the C++ oracle, and
compared bit for bit; so is the softmax cross-entropy gradient (library against the
Python oracle).  The glue that is not arithmetic (ReLU, max-pool routing) is evaluated
once on the host and its result is fed to both sides, so the chain stays comparable layer
by layer.

Formats (Sec. 3.3 mixed precision, stages of Fig. 3), as the triple fmts = (compute, master,
loss): activations, weight copies and back-propagated errors in `compute` (an 8-bit format);
weight gradients rounded from the quire straight to `master`, which also holds the master
weights and runs the optimizer (learning rate 0.1, i.e. 0x14CD in posit<16,1>); the loss in
`loss`.  Default posit<8,0> / <16,1> / <16,1>; ("p8_2", "p12_2", "p10_2") is the paper's final
configuration (Sec. 4, Table 4).
"""
import numpy as np
import torch

import paper_2105_00053_amd as pn
from oracle import fast
from oracle import posit_oracle as po

from gpu_util import to_dev, to_np

ALPHA = 0xEB33  # posit<16,1> pattern of -(0x14CD) = -0.1 rounded
DEFAULT_FORMATS = ("p8", "p16", "p16")


class Mismatch(AssertionError):
    pass


def _check(name, got, want, log):
    got = np.asarray(got)
    want = np.asarray(want)
    bad = int((got.astype(np.int64) != want.astype(np.int64)).sum())
    log.append((name, got.size, bad))
    if bad:
        raise Mismatch("%s: %d of %d outputs differ from the oracle" % (name, bad, got.size))


def relu(p8):
    out = p8.copy()
    out[p8 > 0x80] = 0  # negative patterns (NaR 0x80 stays)
    return out


def maxpool_fwd(p8):
    n, c, h, w = p8.shape
    s = p8.view(np.int8).reshape(n, c, h // 2, 2, w // 2, 2).transpose(0, 1, 2, 4, 3, 5).reshape(n, c, h // 2, w // 2, 4)
    idx = s.argmax(axis=-1)  # first maximum in row-major window order
    out = np.take_along_axis(s, idx[..., None], axis=-1)[..., 0]
    return out.view(np.uint8), idx


def maxpool_bwd(dy8, idx, in_shape):
    n, c, h, w = in_shape
    dx = np.zeros((n, c, h // 2, w // 2, 4), dtype=np.uint8)
    np.put_along_axis(dx, idx[..., None], dy8[..., None], axis=-1)
    return dx.reshape(n, c, h // 2, w // 2, 2, 2).transpose(0, 1, 2, 4, 3, 5).reshape(n, c, h, w)


def _conv_desc(n, cin, h, w, cout, k, pad, stride=1):
    return dict(N=n, C=cin, H=h, W=w, K=cout, R=k, S=k, pad_h=pad, pad_w=pad, stride_h=stride, stride_w=stride)


def _pn_desc(d):
    return pn.ConvDesc(d["N"], d["C"], d["H"], d["W"], d["K"], d["R"], d["S"], d["pad_h"], d["pad_w"], d["stride_h"], d["stride_w"])


def quarter(fc):
    """Pattern of 1/4 in the compute format (0x10 in posit<8,0>)."""
    return int(fast.round_from_float(np.array([0.25], dtype=np.float32), fc)[0])


def avgpool_desc(shape):
    n, c, h, w = shape
    return _conv_desc(n * c, 1, h, w, 1, 2, 0, 2)


def training_step(net, batch, x_f32, params_f32, labels, check=True, timers=None, final_state=None, fmts=DEFAULT_FORMATS):
    """Runs forward, backward and update.  Returns the log [(name, outputs, mismatches)]."""
    fc, fm, fl = fmts
    assert po.FORMATS[fc].n == 8, "the host glue (ReLU, max-pool routing) works on 8-bit patterns"
    alpha = int(fast.round_from_float(np.array([-0.1], dtype=np.float32), fm)[0])
    log = []
    # master weights and compute copies
    W16, B16, W8, B8 = [], [], [], []
    for w, b in params_f32:
        w16 = to_np(pn.posit_round(to_dev(w), fm), fm)
        b16 = to_np(pn.posit_round(to_dev(b), fm), fm)
        if check:
            _check("round w->master", w16, fast.round_from_float(w, fm), log)
        W16.append(w16)
        B16.append(b16)
        W8.append(to_np(pn.posit_convert(to_dev(w16), fm, fc), fc))
        B8.append(to_np(pn.posit_convert(to_dev(b16), fm, fc), fc))
        if check:
            _check("convert w->compute", W8[-1], fast.convert(w16, fm, fc), log)
    x = to_np(pn.posit_round(to_dev(x_f32), fc), fc)
    if check:
        _check("round x->compute", x, fast.round_from_float(x_f32, fc), log)

    # ---------------- forward ----------------
    tape = []
    li = 0
    for layer in net["layers"]:
        kind = layer[0]
        if kind == "conv":
            _, cin, cout, k, pad = layer
            d = _conv_desc(x.shape[0], cin, x.shape[2], x.shape[3], cout, k, pad)
            y = to_np(pn.posit_conv2d_fwd(to_dev(x), to_dev(W8[li]), _pn_desc(d), fc, fc, bias=to_dev(B8[li])), fc)
            if check:
                _check("conv%d fwd" % li, y, fast.conv2d_fwd(x, W8[li], d, fc, fc, bias=B8[li]), log)
            tape.append(("conv", li, d, x))
            x = y
            li += 1
        elif kind == "fc":
            y = to_np(pn.posit_gemm(to_dev(x), to_dev(W8[li]), fc, fc, trans_b=True, bias=to_dev(B8[li])), fc)
            if check:
                _check("fc%d fwd" % li, y, fast.gemm(x, W8[li], fc, fc, trans_b=True, bias=B8[li])[0], log)
            tape.append(("fc", li, None, x))
            x = y
            li += 1
        elif kind == "relu":
            y = relu(x)
            tape.append(("relu", None, None, y))
            x = y
        elif kind == "avgpool":
            d = avgpool_desc(x.shape)
            xin = x.reshape(d["N"], 1, d["H"], d["W"])
            wq = np.full((1, 1, 2, 2), quarter(fc), dtype=np.uint8)
            y = to_np(pn.posit_conv2d_fwd(to_dev(xin), to_dev(wq), _pn_desc(d), fc, fc), fc)
            if check:
                _check("avgpool fwd", y, fast.conv2d_fwd(xin, wq, d, fc, fc), log)
            tape.append(("avgpool", None, d, x.shape))
            x = y.reshape(x.shape[0], x.shape[1], x.shape[2] // 2, x.shape[3] // 2)
        elif kind == "maxpool":
            y, idx = maxpool_fwd(x)
            tape.append(("maxpool", None, idx, x.shape))
            x = y
        elif kind == "flatten":
            tape.append(("flatten", None, None, x.shape))
            x = np.ascontiguousarray(x.reshape(x.shape[0], -1))
    logits = x

    # ---------------- loss gradient: softmax cross entropy in the loss format ----------------
    lab32 = torch.from_numpy(np.asarray(labels, dtype=np.int32)).cuda()
    loss_d, g16_d = pn.posit_cross_entropy(to_dev(logits), lab32, fc, fl, fl)
    want_loss, want_g = po.cross_entropy(logits.tolist(), [int(v) for v in labels], po.FORMATS[fc], po.FORMATS[fl], po.FORMATS[fl])
    g16 = np.array(want_g, dtype=np.uint8 if po.FORMATS[fl].n <= 8 else np.uint16 if po.FORMATS[fl].n <= 16 else np.uint32)
    if check:
        _check("cross entropy dlogits", to_np(g16_d, fl), g16, log)
        _check("cross entropy loss", to_np(loss_d, fl), np.array([want_loss]), log)
    dy = to_np(pn.posit_convert(to_dev(g16), fl, fc), fc)
    if check:
        _check("dlogits loss->compute", dy, fast.convert(g16, fl, fc), log)

    # ---------------- backward + update ----------------
    for kind, li, d, saved in reversed(tape):
        if kind == "fc":
            xin = saved
            dw = to_np(pn.posit_gemm(to_dev(dy), to_dev(xin), fc, fm, trans_a=True), fm)
            ones = np.full((dy.shape[0], 1), 0x40, dtype=np.uint8)
            db = to_np(pn.posit_gemm(to_dev(dy), to_dev(ones), fc, fm, trans_a=True), fm).reshape(-1)
            dx = to_np(pn.posit_gemm(to_dev(dy), to_dev(W8[li]), fc, fc), fc)
            if check:
                _check("fc%d bwd_weight" % li, dw, fast.gemm(dy, xin, fc, fm, trans_a=True)[0], log)
                _check("fc%d bwd_bias" % li, db, fast.gemm(dy, ones, fc, fm, trans_a=True)[0].reshape(-1), log)
                _check("fc%d bwd_data" % li, dx, fast.gemm(dy, W8[li], fc, fc)[0], log)
            _update(li, dw, db, W16, B16, W8, B8, check, log, alpha, fm, fc)
            dy = dx
        elif kind == "conv":
            xin = saved
            desc = _pn_desc(d)
            dw, db = pn.posit_conv2d_bwd_weight(to_dev(dy), to_dev(xin), desc, fc, fm, with_bias=True)
            dw, db = to_np(dw, fm), to_np(db, fm)
            if check:
                wdw, wdb = fast.conv2d_bwd_weight(dy, xin, d, fc, fm, with_bias=True)
                _check("conv%d bwd_weight" % li, dw, wdw, log)
                _check("conv%d bwd_bias" % li, db, wdb, log)
            if li > 0:
                dx = to_np(pn.posit_conv2d_bwd_data(to_dev(dy), to_dev(W8[li]), desc, fc, fc), fc)
                if check:
                    _check("conv%d bwd_data" % li, dx, fast.conv2d_bwd_data(dy, W8[li], d, fc, fc), log)
            else:
                dx = None  # the input needs no gradient
            _update(li, dw, db, W16, B16, W8, B8, check, log, alpha, fm, fc)
            dy = dx
        elif kind == "relu":
            dy = dy.copy()
            dy[(saved == 0) | (saved > 0x80)] = 0
        elif kind == "avgpool":
            shape = saved
            dyin = dy.reshape(d["N"], 1, d["H"] // 2, d["W"] // 2)
            wq = np.full((1, 1, 2, 2), quarter(fc), dtype=np.uint8)
            dx = to_np(pn.posit_conv2d_bwd_data(to_dev(dyin), to_dev(wq), _pn_desc(d), fc, fc), fc)
            if check:
                _check("avgpool bwd", dx, fast.conv2d_bwd_data(dyin, wq, d, fc, fc), log)
            dy = dx.reshape(shape)
        elif kind == "maxpool":
            dy = maxpool_bwd(dy, d, saved)
        elif kind == "flatten":
            dy = np.ascontiguousarray(dy.reshape(saved))
    if final_state is not None:
        final_state.update(dict(logits=logits, W16=W16, B16=B16, W8=W8, B8=B8))
    return log


def _update(li, dw, db, W16, B16, W8, B8, check, log, alpha=ALPHA, fm="p16", fc="p8"):
    for grads, masters, copies, tag in ((dw, W16, W8, "w"), (db, B16, B8, "b")):
        yd = to_dev(masters[li].reshape(-1))
        ynew, ycopy = pn.posit_axpy(alpha, to_dev(grads.reshape(-1)), yd, fm, fm, fcopy=fc)
        ynew, ycopy = to_np(ynew, fm), to_np(ycopy, fc)
        if check:
            want, wantc = fast.axpy(alpha, grads.reshape(-1), masters[li].reshape(-1), fm, fm, fc)
            _check("sgd %s%d" % (tag, li), ynew, want, log)
            _check("sgd %s%d copy" % (tag, li), ycopy, wantc, log)
        masters[li] = ynew.reshape(masters[li].shape)
        copies[li] = ycopy.reshape(copies[li].shape)
