"""GPU parity of the activation and loss entry points (paper Fig. 2: Sigmoid, TanH, Cross Entropy, MSE)
against the Python oracle, bit for bit.  The elementary functions are checked on EVERY pattern of every
supported format: that is what shows the binary64 evaluation in the kernel to be correctly rounded."""
import numpy as np
import pytest
import torch

import paper_2105_00053_amd as pn
from oracle import posit_oracle as po

from gpu_util import BITS, NP_DTYPE, rand_patterns, to_dev, to_np

pytestmark = pytest.mark.gpu
SMALL = ["p8", "p8_1", "p8_2", "p10_1", "p10_2", "p12_1", "p12_2", "p16"]


@pytest.mark.parametrize("fmt", SMALL)
def test_unary_all_patterns(fmt):
    f = po.FORMATS[fmt]
    pats = np.arange(1 << f.n, dtype=np.uint32).astype(NP_DTYPE[fmt])
    x = to_dev(pats)
    for fn in po.UNARY:
        got = to_np(pn.posit_unary(fn, x, fmt), fmt).astype(np.int64)
        want = np.array([po.unary(fn, int(p), f) for p in pats], dtype=np.int64)
        bad = np.nonzero(got != want)[0]
        assert len(bad) == 0, "%s %s: %d mismatches, first pattern %#x got %#x want %#x" % (fn, fmt, len(bad), bad[0], got[bad[0]], want[bad[0]])


@pytest.mark.parametrize("fy,fd", [("p8", "p8"), ("p8_2", "p12_2"), ("p16", "p16"), ("p12_2", "p8_2"), ("p10_1", "p16")])
def test_unary_bwd(fy, fd):
    f_y, f_d = po.FORMATS[fy], po.FORMATS[fd]
    rng = np.random.default_rng(BITS[fy] + BITS[fd])
    n = 3001
    dy = rand_patterns(rng, n, fd, special=0.05)
    for fn in ("sigmoid", "tanh"):
        x = rand_patterns(rng, n, fy, special=0.05)
        y = to_np(pn.posit_unary(fn, to_dev(x), fy), fy)   # genuine forward outputs ...
        y[: n // 4] = rand_patterns(rng, n // 4, fy, special=0.1)  # ... and arbitrary patterns
        got = to_np(pn.posit_unary_bwd(fn, to_dev(y), to_dev(dy), fy, fd), fd)
        want = np.array([po.unary_bwd(fn, int(a), int(b), f_y, f_d) for a, b in zip(y, dy)])
        assert np.array_equal(got.astype(np.int64), want), fn


def _logits(rng, B, C, fmt, scale):
    z = rng.normal(0, scale, (B, C))
    return np.array([[po.from_float(v, po.FORMATS[fmt]) for v in row] for row in z], dtype=NP_DTYPE[fmt])


@pytest.mark.parametrize("fz,fl,fg,B,C,scale", [("p8", "p16", "p16", 64, 10, 2.0), ("p8_2", "p12_2", "p12_2", 128, 10, 3.0), ("p8_2", "p10_2", "p12_2", 37, 10, 1.0),
                                                 ("p16", "p16", "p8", 300, 7, 5.0), ("p8_2", "p8_2", "p8_2", 16, 3, 1.0), ("p12_1", "p12_1", "p16", 5, 100, 2.0), ("p8_2", "p12_2", "p12_2", 9, 256, 2.0),
                                                 ("p8", "p16", "p16", 3, 300, 2.0), ("p10_2", "p10_2", "p10_2", 70, 16, 2.0),
                                                 ("p8", "p8", "p8", 1, 1, 1.0)])
def test_cross_entropy(fz, fl, fg, B, C, scale):
    rng = np.random.default_rng(B * 31 + C)
    logits = _logits(rng, B, C, fz, scale)
    labels = rng.integers(0, C, B).astype(np.int32)
    loss, grad = pn.posit_cross_entropy(to_dev(logits), torch.from_numpy(labels).cuda(), fz, fl, fg)
    wl, wg = po.cross_entropy(logits.tolist(), labels.tolist(), po.FORMATS[fz], po.FORMATS[fl], po.FORMATS[fg])
    assert np.array_equal(to_np(grad, fg).astype(np.int64), np.array(wg)), "dlogits"
    assert int(to_np(loss, fl)[0]) == wl, "loss"
    # only one of the two outputs requested
    loss2, none = pn.posit_cross_entropy(to_dev(logits), torch.from_numpy(labels).cuda(), fz, fl, fg, want_grad=False)
    assert none is None and int(to_np(loss2, fl)[0]) == wl
    none, grad2 = pn.posit_cross_entropy(to_dev(logits), torch.from_numpy(labels).cuda(), fz, fl, fg, want_loss=False)
    assert none is None and np.array_equal(to_np(grad2, fg).astype(np.int64), np.array(wg))


def test_cross_entropy_nar_rows_and_bad_labels():
    rng = np.random.default_rng(5)
    B, C = 40, 10
    logits = _logits(rng, B, C, "p8_2", 2.0)
    labels = rng.integers(0, C, B).astype(np.int32)
    logits[3, 4] = 0x80
    labels[17] = C
    labels[20] = -1
    loss, grad = pn.posit_cross_entropy(to_dev(logits), torch.from_numpy(labels).cuda(), "p8_2", "p12_2", "p12_2")
    wl, wg = po.cross_entropy(logits.tolist(), labels.tolist(), po.FORMATS["p8_2"], po.FORMATS["p12_2"], po.FORMATS["p12_2"])
    assert wl == po.FORMATS["p12_2"].nar and int(to_np(loss, "p12_2")[0]) == wl
    assert np.array_equal(to_np(grad, "p12_2").astype(np.int64), np.array(wg))


@pytest.mark.parametrize("fp,fl,fg,n", [("p8", "p16", "p16", 1280), ("p8_2", "p12_2", "p12_2", 640), ("p16", "p16", "p8", 1001), ("p10_2", "p10_2", "p10_2", 3),
                                        ("p8_1", "p8_1", "p16", 1)])
def test_mse(fp, fl, fg, n):
    rng = np.random.default_rng(n)
    pred = rand_patterns(rng, n, fp, special=0.0, allow_nar=False)
    target = rand_patterns(rng, n, fp, special=0.0, allow_nar=False)
    if n > 100:  # mostly moderate values, as network outputs are
        f = po.FORMATS[fp]
        pred[: n - 20] = [po.from_float(v, f) for v in rng.normal(0, 1, n - 20)]
        target[: n - 20] = [po.from_float(v, f) for v in rng.normal(0, 1, n - 20)]
    for with_nar in (False, True):
        if with_nar:
            pred[n // 2] = po.FORMATS[fp].nar
        loss, grad = pn.posit_mse(to_dev(pred), to_dev(target), fp, fl, fg)
        wl, wg = po.mse(pred.tolist(), target.tolist(), po.FORMATS[fp], po.FORMATS[fl], po.FORMATS[fg])
        assert int(to_np(loss, fl)[0]) == wl, with_nar
        assert np.array_equal(to_np(grad, fg).astype(np.int64), np.array(wg)), with_nar
