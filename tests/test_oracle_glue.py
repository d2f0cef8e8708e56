"""Pins for the oracle's layer glue (ReLU, max / average pooling).

The oracle works on decoded values; these checks redo the same operations on the raw
patterns as signed integers (posit order is the two's-complement order of the patterns,
Sec. 2, pinned exhaustively in test_oracle_scalar) and, for average pooling, through the
oracle's convolution with a constant kernel and stride equal to the window."""
import random

import numpy as np
import pytest

from oracle import posit_oracle as po

FMT = {"p8": (po.P8, np.uint8, np.int8), "p16": (po.P16, np.uint16, np.int16)}


@pytest.mark.parametrize("name", ["p8", "p16"])
def test_relu_and_backward_on_patterns(name):
    fmt, ut, st = FMT[name]
    rng = np.random.default_rng(3)
    x = rng.integers(0, 1 << fmt.n, size=4000).astype(ut)
    x[:4] = [0, fmt.nar, 1, fmt.mask]
    y = np.array(po.relu(x.tolist(), fmt), dtype=ut)
    want = np.where((x.view(st) > 0) | (x == fmt.nar), x, 0).astype(ut)
    assert np.array_equal(y, want)
    dy = rng.integers(0, 1 << 16, size=4000).astype(np.uint16)
    dx = np.array(po.relu_bwd(y.tolist(), dy.tolist(), fmt, po.P16), dtype=np.uint16)
    want = np.where(y == fmt.nar, 0x8000, np.where(y.view(st) > 0, dy, 0)).astype(np.uint16)
    assert np.array_equal(dx, want)


@pytest.mark.parametrize("name", ["p8", "p16"])
@pytest.mark.parametrize("kh,kw", [(2, 2), (3, 2)])
def test_maxpool_on_patterns(name, kh, kw):
    fmt, ut, st = FMT[name]
    rng = np.random.default_rng(kh * 10 + kw)
    planes, H, W = 5, 6, 8
    x = rng.integers(0, 1 << fmt.n, size=(planes, H, W)).astype(ut)
    x[0, 0, :4] = [7, 7, fmt.nar, 7]  # ties and a NaR
    x[1, :2, :2] = fmt.nar             # all-NaR window
    y, idx = po.maxpool2d_fwd(x.flatten().tolist(), planes, H, W, kh, kw, fmt)
    win = x.view(st).reshape(planes, H // kh, kh, W // kw, kw).transpose(0, 1, 3, 2, 4).reshape(planes, H // kh, W // kw, kh * kw)
    wi = win.argmax(axis=-1)  # numpy returns the first maximum
    assert np.array_equal(np.array(idx).reshape(wi.shape), wi)
    assert np.array_equal(np.array(y, dtype=ut).view(st).reshape(wi.shape), np.take_along_axis(win, wi[..., None], -1)[..., 0])
    dy = rng.integers(1, 1 << fmt.n, size=len(y)).astype(ut)
    dx = np.array(po.maxpool2d_bwd(dy.tolist(), idx, planes, H, W, kh, kw), dtype=ut).reshape(planes, H, W)
    back = dx.reshape(planes, H // kh, kh, W // kw, kw).transpose(0, 1, 3, 2, 4).reshape(planes, H // kh, W // kw, kh * kw)
    assert np.array_equal(np.take_along_axis(back, wi[..., None], -1)[..., 0].flatten(), dy)
    assert (back != 0).sum() == len(y)


@pytest.mark.parametrize("fin,fout", [(po.P8, po.P8), (po.P16, po.P8), (po.P8, po.P16)])
def test_avgpool_is_a_strided_convolution_with_constant_kernel(fin, fout):
    rng = random.Random(fin.n + fout.n)
    planes, H, W, kh, kw = 3, 4, 8, 2, 4
    x = [rng.getrandbits(fin.n) for _ in range(planes * H * W)]
    x[5] = fin.nar
    wpat = po.round_to_posit(po.Fraction(1, kh * kw), fin)
    sh = po.ConvShape(planes, 1, H, W, 1, kh, kw, 0, 0, kh, kw)
    assert po.avgpool2d_fwd(x, planes, H, W, kh, kw, fin, fout) == po.conv2d_fwd(x, [wpat] * (kh * kw), sh, fin, fout)
    dy = [rng.getrandbits(fin.n) for _ in range(planes * (H // kh) * (W // kw))]
    assert po.avgpool2d_bwd(dy, planes, H, W, kh, kw, fin, fout) == po.conv2d_bwd_data(dy, [wpat] * (kh * kw), sh, fin, fout)
    # a window of equal values averages to that value exactly
    same = [0x48] * (kh * kw)
    assert po.avgpool2d_fwd(same, 1, kh, kw, kh, kw, po.P8, po.P8) == [0x48]
