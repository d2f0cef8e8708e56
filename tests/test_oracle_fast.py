"""The C++ oracle must reproduce the Python oracle on every entry point."""
import random

import numpy as np
import pytest

from oracle import fast
from oracle import posit_oracle as po

F = dict(po.FORMATS)
GENERAL = ["p8_1", "p8_2", "p10_1", "p10_2", "p12_1", "p12_2"]


def _rand_patterns(rng, shape, fmt, special=0.02):
    bits = F[fmt].n
    a = rng.integers(0, 1 << bits, size=shape, dtype=np.uint64)
    m = rng.random(size=shape) < special
    sp = rng.choice(np.array([0, 1, F[fmt].maxpos_pattern, F[fmt].mask, F[fmt].nar + 1], dtype=np.uint64), size=shape)
    a = np.where(m, sp, a)
    return a.astype(fast.DTYPES[fmt])


@pytest.mark.parametrize("fmt", ["p8", "p16"] + GENERAL)
def test_convert_and_float_exhaustive(fmt):
    pats = np.arange(1 << F[fmt].n, dtype=np.uint32).astype(fast.DTYPES[fmt])
    f64 = fast.to_float(pats, fmt, "f64")
    f32 = fast.to_float(pats, fmt, "f32")
    for p in range(0, 1 << F[fmt].n, 1 if F[fmt].n == 8 else 3):
        want = po.to_float(p, F[fmt], "f64")
        if p == F[fmt].nar:
            assert np.isnan(f64[p]) and np.isnan(f32[p])
        else:
            assert f64[p] == want and float(f32[p]) == want
    assert np.array_equal(fast.round_from_float(f64, fmt)[np.arange(len(pats)) != F[fmt].nar], pats[np.arange(len(pats)) != F[fmt].nar])
    for dst in ("p8", "p16", "p32", "p8_2", "p12_2", "p10_1"):
        got = fast.convert(pats, fmt, dst)
        step = 1 if F[fmt].n == 8 else 11
        for p in range(0, 1 << F[fmt].n, step):
            assert int(got[p]) == po.convert(p, F[fmt], F[dst])


def test_p32_conversions_sample():
    rng = np.random.default_rng(0)
    pats = _rand_patterns(rng, 3000, "p32")
    f32 = fast.to_float(pats, "p32", "f32")
    f64 = fast.to_float(pats, "p32", "f64")
    c16 = fast.convert(pats, "p32", "p16")
    c8 = fast.convert(pats, "p32", "p8")
    for i, p in enumerate(pats.tolist()):
        assert float(f32[i]) == po.to_float(p, po.P32, "f32")
        assert float(f64[i]) == po.to_float(p, po.P32, "f64")
        assert int(c16[i]) == po.convert(p, po.P32, po.P16)
        assert int(c8[i]) == po.convert(p, po.P32, po.P8)


@pytest.mark.parametrize("dst", ["p8", "p16", "p32"] + GENERAL)
def test_round_from_float(dst):
    rng = np.random.default_rng(5)
    x = (rng.standard_normal(4000) * np.exp2(rng.uniform(-40, 40, 4000))).astype(np.float32)
    x[:8] = [0.0, -0.0, np.inf, -np.inf, np.nan, 1e-45, 3.4e38, -1.0]
    got = fast.round_from_float(x, dst)
    for i in range(len(x)):
        assert int(got[i]) == po.from_float(float(x[i]), F[dst])
    xd = rng.standard_normal(2000) * np.exp2(rng.uniform(-200, 200, 2000))
    xd[:3] = [5e-324, 1.7e308, -2.2e-308]
    got = fast.round_from_float(xd, dst)
    for i in range(len(xd)):
        assert int(got[i]) == po.from_float(float(xd[i]), F[dst])


@pytest.mark.parametrize("fin,fout,M,N,K", [("p8", "p8", 7, 9, 40), ("p8", "p16", 5, 6, 300), ("p16", "p16", 6, 5, 50),
                                             ("p16", "p8", 4, 4, 33), ("p32", "p32", 4, 5, 20), ("p32", "p16", 3, 3, 9),
                                             ("p8_2", "p8_2", 5, 4, 60), ("p8_2", "p12_2", 4, 4, 30), ("p8_1", "p8_1", 4, 5, 40),
                                             ("p10_1", "p10_1", 4, 3, 30), ("p12_1", "p8_2", 3, 4, 25), ("p12_2", "p12_2", 3, 3, 20),
                                             ("p10_2", "p16", 3, 3, 15)])
def test_gemm_matches_python_oracle(fin, fout, M, N, K):
    rng = np.random.default_rng(M * 100 + K)
    A = _rand_patterns(rng, (M, K), fin)
    B = _rand_patterns(rng, (K, N), fin)
    bias = _rand_patterns(rng, (N,), fin)
    want = np.array(po.gemm(A.tolist(), B.tolist(), F[fin], F[fout], bias=bias.tolist()))
    got, _ = fast.gemm(A, B, fin, fout, bias=bias, threads=3)
    assert np.array_equal(got.astype(np.int64), want)
    got, _ = fast.gemm(np.ascontiguousarray(A.T), np.ascontiguousarray(B.T), fin, fout, trans_a=True, trans_b=True, bias=bias)
    assert np.array_equal(got.astype(np.int64), want)
    want = np.array(po.gemm(A.tolist(), B.tolist(), F[fin], F[fout]))
    got, _ = fast.gemm(A, B, fin, fout)
    assert np.array_equal(got.astype(np.int64), want)


def test_gemm_wrap_and_overflow_count():
    A = np.full((1, 128), 0x7F, dtype=np.uint8)
    B = np.full((128, 1), 0x7F, dtype=np.uint8)
    C, ovf = fast.gemm(A, B, "p8", "p8")
    assert C[0, 0] == 0x81 and ovf == 1
    C, ovf = fast.gemm(A[:, :127], B[:127], "p8", "p8")
    assert C[0, 0] == 0x7F and ovf == 0


@pytest.mark.parametrize("fin,fout", [("p8", "p8"), ("p8", "p16"), ("p16", "p16"), ("p32", "p32"), ("p8_2", "p8_2"), ("p8_2", "p12_2")])
def test_conv_matches_python_oracle(fin, fout):
    rng = np.random.default_rng(F[fin].n + F[fout].n)
    for d in (dict(N=2, C=3, H=6, W=5, K=4, R=3, S=3, pad_h=1, pad_w=1),
              dict(N=1, C=2, H=7, W=8, K=3, R=5, S=2, pad_h=2, pad_w=0, stride_h=2, stride_w=1),
              dict(N=2, C=1, H=5, W=5, K=2, R=2, S=3, pad_h=0, pad_w=2, stride_h=1, stride_w=2)):
        sh = po.ConvShape(d["N"], d["C"], d["H"], d["W"], d["K"], d["R"], d["S"], d.get("pad_h", 0), d.get("pad_w", 0),
                          d.get("stride_h", 1), d.get("stride_w", 1))
        x = _rand_patterns(rng, (sh.N, sh.C, sh.H, sh.W), fin)
        w = _rand_patterns(rng, (sh.K, sh.C, sh.R, sh.S), fin)
        dy = _rand_patterns(rng, (sh.N, sh.K, sh.OH, sh.OW), fin)
        bias = _rand_patterns(rng, (sh.K,), fin)
        y = fast.conv2d_fwd(x, w, d, fin, fout, bias=bias, threads=2)
        assert y.flatten().tolist() == po.conv2d_fwd(x.flatten().tolist(), w.flatten().tolist(), sh, F[fin], F[fout], bias.tolist())
        dx = fast.conv2d_bwd_data(dy, w, d, fin, fout)
        assert dx.flatten().tolist() == po.conv2d_bwd_data(dy.flatten().tolist(), w.flatten().tolist(), sh, F[fin], F[fout])
        # a NaR weight at a corner tap: NaR only at the input positions that tap reaches (both quire and no-quire chains)
        wn = w.copy()
        wn[0, 0, 0, 0] = F[fin].nar
        dxn = fast.conv2d_bwd_data(dy, wn, d, fin, fout)
        assert dxn.flatten().tolist() == po.conv2d_bwd_data(dy.flatten().tolist(), wn.flatten().tolist(), sh, F[fin], F[fout])
        assert (dxn[:, 0] == F[fout].nar).any() and not (dxn[:, 0] == F[fout].nar).all()
        dxq = fast.conv2d_bwd_data(dy, wn, d, fin, fout, noquire=True)
        assert dxq.flatten().tolist() == po.conv2d_bwd_data_noquire(dy.flatten().tolist(), wn.flatten().tolist(), sh, F[fin], F[fout])
        dw, db = fast.conv2d_bwd_weight(dy, x, d, fin, fout, with_bias=True)
        assert dw.flatten().tolist() == po.conv2d_bwd_weight(dy.flatten().tolist(), x.flatten().tolist(), sh, F[fin], F[fout])
        assert db.tolist() == po.conv2d_bias_grad(dy.flatten().tolist(), sh, F[fin], F[fout])


@pytest.mark.parametrize("fx,fy,fc", [("p8", "p16", "p8"), ("p16", "p16", None), ("p8", "p8", None), ("p16", "p32", "p16"), ("p32", "p32", "p8"),
                                      ("p12_2", "p12_2", "p8_2"), ("p8_2", "p12_2", None), ("p10_1", "p12_1", "p8_1")])
def test_axpy_matches_python_oracle(fx, fy, fc):
    rng = np.random.default_rng(F[fx].n * 3 + F[fy].n)
    n = 1500
    x = _rand_patterns(rng, n, fx)
    y = _rand_patterns(rng, n, fy)
    for alpha in (po.from_float(-0.1, F[fy]), po.from_float(1.0, F[fy]), 0, int(_rand_patterns(rng, 1, fy)[0])):
        res = fast.axpy(alpha, x, y, fx, fy, fc)
        for i in range(n):
            want = po.axpy(alpha, int(x[i]), int(y[i]), F[fx], F[fy], F[fc] if fc else None)
            if fc:
                assert (int(res[0][i]), int(res[1][i])) == want
            else:
                assert int(res[i]) == want
