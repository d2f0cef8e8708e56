"""Pins for the quire part of the oracle: dot, gemm, convolution and its adjoints, axpy.

Checks come from outside the oracle's own formulas: Table 1's dot-product limit,
brute-force rational sums, numpy's integer matmul and torch's float64
convolution routines (exact for posit<8,0>, whose values are small multiples of
2^-6), and algebraic identities (1x1 convolution == matrix product, adjointness).
"""
import math
import random
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import posit_oracle as po


def _p8_float_table():
    """posit<8,0> values written from the structure of the format, not via the
    oracle: patterns below 0x40 are the integer itself over 64; from 0x40 up a run
    of m ones gives 2^(m-1) * (1 + f / 2^(6-m))."""
    t = np.zeros(256, dtype=np.float64)
    for x in range(1, 128):
        if x < 64:
            v = x / 64.0
        else:
            m = 0
            while m < 7 and (x >> (6 - m)) & 1:
                m += 1
            nf = max(6 - m, 0)
            f = x & ((1 << nf) - 1)
            v = 2.0 ** (m - 1) * (1.0 + f / (1 << nf))
        t[x] = v
        t[256 - x] = -v
    t[128] = np.nan
    return t


P8F = _p8_float_table()


def test_p8_structure_table_matches_decode():
    for p in range(256):
        v = po.decode(p, po.P8)
        if p == 128:
            assert v is po.NaR
        else:
            assert Fraction(float(P8F[p])) == v


def test_dot_product_limit_table1():
    # K = limit products of maxpos*maxpos still fit; the sum rounds to maxpos, no wrap
    for fmt, limit in ((po.P8, 127), (po.P16, 32767)):
        mp = fmt.maxpos_pattern
        u = po.to_minpos_units(mp, fmt)
        total = limit * u * u
        assert po.quire_fits(total, fmt)
        assert not po.quire_fits(total + u * u, fmt)
        assert po.quire_round(total, fmt, fmt) == mp
    assert po.dot([0x7F] * 127, [0x7F] * 127, po.P8, po.P8) == 0x7F
    # one more product wraps the 32-bit quire to -2^31 units: the reading "modular quire"
    assert po.dot([0x7F] * 128, [0x7F] * 128, po.P8, po.P8) == 0x81
    assert po.quire_wrap(128 * 4096 * 4096, po.P8) == -(1 << 31)
    u32 = po.to_minpos_units(po.P32.maxpos_pattern, po.P32)
    assert po.quire_fits((2 ** 31 - 1) * u32 * u32, po.P32)
    assert not po.quire_fits((2 ** 31) * u32 * u32, po.P32)


def test_p8_full_multiplication_table():
    for a in range(256):
        va = po.decode(a, po.P8)
        for b in range(256):
            vb = po.decode(b, po.P8)
            got = po.dot([a], [b], po.P8, po.P8)
            if va is po.NaR or vb is po.NaR:
                assert got == 0x80
            else:
                assert got == po.round_by_search(va * vb, po.P8)


@pytest.mark.parametrize("fmt", [po.P8, po.P16, po.P32])
def test_dot_bruteforce_rationals(fmt):
    rng = random.Random(fmt.n)
    for trial in range(400):
        K = rng.randint(0, 8)
        a = [rng.getrandbits(fmt.n) for _ in range(K)]
        b = [rng.getrandbits(fmt.n) for _ in range(K)]
        if trial % 5 == 0 and K:
            a[rng.randrange(K)] = rng.choice([1, fmt.maxpos_pattern, fmt.mask, fmt.nar + 1])
        bias = rng.getrandbits(fmt.n) if trial % 3 == 0 else None
        vals = [po.decode(p, fmt) for p in a + b + ([bias] if bias is not None else [])]
        got = po.dot(a, b, fmt, fmt, bias)
        if any(v is po.NaR for v in vals):
            assert got == fmt.nar
            continue
        s = sum((po.decode(x, fmt) * po.decode(y, fmt) for x, y in zip(a, b)), Fraction(0))
        if bias is not None:
            s += po.decode(bias, fmt)
        # K <= 8 (+bias) is far inside the dot-product limit: no wrap possible
        assert got == po.round_by_search(s, fmt)
        if K == 0 and bias is None:
            assert got == 0


def test_nar_times_zero_is_nar():
    assert po.dot([0x80, 0x40], [0x00, 0x40], po.P8, po.P8) == 0x80
    assert po.dot([0x40], [0x40], po.P8, po.P8, bias=0x80) == 0x80


def test_p8_quire_equals_numpy_integer_matmul():
    rng = np.random.default_rng(1)
    M, N, K = 9, 7, 33
    A = rng.integers(0, 256, size=(M, K), dtype=np.uint8)
    B = rng.integers(0, 256, size=(K, N), dtype=np.uint8)
    A[A == 128] = 0
    B[B == 128] = 0
    Ai = np.rint(P8F[A] * 64).astype(np.int64)
    Bi = np.rint(P8F[B] * 64).astype(np.int64)
    Q = Ai @ Bi
    for i in range(M):
        for j in range(N):
            assert po.quire_dot(A[i].tolist(), B[:, j].tolist(), po.P8) == int(Q[i, j])


def test_gemm_transposes_and_mixed_output_format():
    rng = random.Random(9)
    M, N, K = 5, 4, 6
    A = [[rng.getrandbits(8) for _ in range(K)] for _ in range(M)]
    B = [[rng.getrandbits(8) for _ in range(N)] for _ in range(K)]
    bias = [rng.getrandbits(8) for _ in range(N)]
    C = po.gemm(A, B, po.P8, po.P16, bias=bias)
    At = [list(r) for r in zip(*A)]
    Bt = [list(r) for r in zip(*B)]
    assert po.gemm(At, B, po.P8, po.P16, trans_a=True, bias=bias) == C
    assert po.gemm(A, Bt, po.P8, po.P16, trans_b=True, bias=bias) == C
    assert po.gemm(At, Bt, po.P8, po.P16, trans_a=True, trans_b=True, bias=bias) == C
    for i in range(M):
        for j in range(N):
            vals = [po.decode(A[i][k], po.P8) for k in range(K)] + [po.decode(B[k][j], po.P8) for k in range(K)] + [po.decode(bias[j], po.P8)]
            if any(v is po.NaR for v in vals):
                assert C[i][j] == po.P16.nar
            else:
                s = sum(vals[k] * vals[K + k] for k in range(K)) + vals[-1]
                assert C[i][j] == po.round_by_search(s, po.P16)


CONV_SHAPES = [
    po.ConvShape(2, 3, 6, 5, 4, 3, 3, 1, 1, 1, 1),
    po.ConvShape(1, 2, 7, 8, 3, 5, 2, 2, 0, 2, 1),
    po.ConvShape(2, 1, 5, 5, 2, 2, 3, 0, 2, 1, 2),
    po.ConvShape(1, 4, 4, 4, 5, 1, 1, 0, 0, 1, 1),
]


def _rand_p8(rng, n):
    a = rng.integers(0, 256, size=n, dtype=np.uint8)
    a[a == 128] = 64
    return a


@pytest.mark.parametrize("sh", CONV_SHAPES)
def test_p8_conv_quires_equal_torch_float64(sh):
    """posit<8,0> products are multiples of 2^-12 below 2^12, so float64 library
    convolutions are exact: they pin forward, backward-data and backward-weight."""
    rng = np.random.default_rng(sh.H * 31 + sh.R)
    x = _rand_p8(rng, sh.N * sh.C * sh.H * sh.W)
    w = _rand_p8(rng, sh.K * sh.C * sh.R * sh.S)
    dy = _rand_p8(rng, sh.N * sh.K * sh.OH * sh.OW)
    bias = _rand_p8(rng, sh.K)
    xt = torch.tensor(P8F[x]).reshape(sh.N, sh.C, sh.H, sh.W)
    wt = torch.tensor(P8F[w]).reshape(sh.K, sh.C, sh.R, sh.S)
    dyt = torch.tensor(P8F[dy]).reshape(sh.N, sh.K, sh.OH, sh.OW)
    bt = torch.tensor(P8F[bias])
    stride, pad = (sh.stride_h, sh.stride_w), (sh.pad_h, sh.pad_w)
    y = torch.nn.functional.conv2d(xt, wt, bt, stride=stride, padding=pad)
    assert tuple(y.shape) == (sh.N, sh.K, sh.OH, sh.OW)
    got = po.conv2d_fwd_quire(x.tolist(), w.tolist(), sh, po.P8, bias.tolist())
    assert got == [int(v) for v in (y * 4096).flatten().tolist()]
    dx = torch.nn.grad.conv2d_input(xt.shape, wt, dyt, stride=stride, padding=pad)
    got = po.conv2d_bwd_data_quire(dy.tolist(), w.tolist(), sh, po.P8)
    assert got == [int(v) for v in (dx * 4096).flatten().tolist()]
    dw = torch.nn.grad.conv2d_weight(xt, wt.shape, dyt, stride=stride, padding=pad)
    got = po.conv2d_bwd_weight_quire(dy.tolist(), x.tolist(), sh, po.P8)
    assert got == [int(v) for v in (dw * 4096).flatten().tolist()]
    db = dyt.sum(dim=(0, 2, 3))
    got = po.conv2d_bias_grad_quire(dy.tolist(), sh, po.P8)
    assert got == [int(v) for v in (db * 4096).tolist()]


def test_conv_1x1_is_gemm_and_ones_kernel_is_window_sum():
    rng = random.Random(4)
    sh = po.ConvShape(2, 3, 4, 5, 6, 1, 1)
    x = [rng.getrandbits(16) for _ in range(sh.N * sh.C * sh.H * sh.W)]
    w = [rng.getrandbits(16) for _ in range(sh.K * sh.C)]
    y = po.conv2d_fwd(x, w, sh, po.P16, po.P16)
    # as a matrix product: rows = (n, h, w), columns = k, reduction over c
    for n in range(sh.N):
        A = [[x[((n * sh.C + c) * sh.H + h) * sh.W + ww] for c in range(sh.C)] for h in range(sh.H) for ww in range(sh.W)]
        Wm = [w[k * sh.C:(k + 1) * sh.C] for k in range(sh.K)]
        Cm = po.gemm(A, Wm, po.P16, po.P16, trans_b=True)
        for hw in range(sh.H * sh.W):
            for k in range(sh.K):
                assert y[(n * sh.K + k) * sh.H * sh.W + hw] == Cm[hw][k]
    # all-ones 2x2 kernel: each output is the exact sum of its window
    sh2 = po.ConvShape(1, 1, 4, 4, 1, 2, 2)
    x2 = [rng.getrandbits(16) | 1 for _ in range(16)]
    x2 = [p if p != 0x8000 else 1 for p in x2]
    y2 = po.conv2d_fwd(x2, [0x4000] * 4, sh2, po.P16, po.P16)
    for oh in range(3):
        for ow in range(3):
            s = sum(po.decode(x2[(oh + r) * 4 + ow + c], po.P16) for r in range(2) for c in range(2))
            assert y2[oh * 3 + ow] == po.round_by_search(s, po.P16)


@pytest.mark.parametrize("fmt", [po.P16, po.P32])
def test_conv_adjoint_identities_exact(fmt):
    """<conv(x,w), dy> == <x, bwd_data(dy,w)> == <w, bwd_weight(dy,x)> before any rounding."""
    rng = random.Random(fmt.n + 1)
    sh = po.ConvShape(2, 2, 5, 4, 3, 3, 2, 1, 1, 2, 1)

    def rnd(n):
        out = []
        for _ in range(n):
            p = rng.getrandbits(fmt.n)
            out.append(p if p != fmt.nar else 1)
        return out

    x = rnd(sh.N * sh.C * sh.H * sh.W)
    w = rnd(sh.K * sh.C * sh.R * sh.S)
    dy = rnd(sh.N * sh.K * sh.OH * sh.OW)
    units = lambda v: [po.to_minpos_units(p, fmt) for p in v]
    yq = po.conv2d_fwd_quire(x, w, sh, fmt)
    dxq = po.conv2d_bwd_data_quire(dy, w, sh, fmt)
    dwq = po.conv2d_bwd_weight_quire(dy, x, sh, fmt)
    lhs = sum(a * b for a, b in zip(yq, units(dy)))
    assert lhs == sum(a * b for a, b in zip(dxq, units(x)))
    assert lhs == sum(a * b for a, b in zip(dwq, units(w)))
    assert lhs != 0


def test_axpy():
    rng = random.Random(2)
    lr = po.from_float(-0.1, po.P16)
    for _ in range(2000):
        x = rng.getrandbits(8)
        y = rng.getrandbits(16)
        got, cp = po.axpy(lr, x, y, po.P8, po.P16, po.P8)
        vx, vy = po.decode(x, po.P8), po.decode(y, po.P16)
        if vx is po.NaR or vy is po.NaR:
            assert got == 0x8000 and cp == 0x80
        else:
            want = po.round_by_search(vy + po.decode(lr, po.P16) * vx, po.P16)
            assert got == want
            assert cp == po.round_by_search(po.decode(want, po.P16), po.P8)
    for _ in range(500):
        y = rng.getrandbits(16)
        if y == 0x8000:
            continue
        assert po.axpy(0, rng.getrandbits(15), y, po.P16, po.P16) == y  # alpha = 0
        assert po.axpy(0x4000, (-y) & 0xFFFF, y, po.P16, po.P16) == 0  # y + 1*(-y)
    assert po.axpy(0x8000, 0x4000, 0x4000, po.P16, po.P16) == 0x8000


def test_conv_is_the_matrix_product_of_its_unfolded_form_including_nar():
    """Forward and weight gradient: zero padding materialised (pattern 0) and the pass written as a plain
    gemm over the unfolded input: same bits, NaR included (NaR * 0 = NaR).  Input gradient: the sum of
    what the unfolded columns scatter back to each input position."""
    rng = random.Random(12)
    sh = po.ConvShape(2, 2, 4, 5, 3, 3, 2, 1, 1, 2, 1)
    fmt = po.P8

    def rnd(n, nar_at=()):
        v = [rng.getrandbits(8) for _ in range(n)]
        v = [p if p != 0x80 else 0x40 for p in v]
        for i in nar_at:
            v[i] = 0x80
        return v

    x = rnd(sh.N * sh.C * sh.H * sh.W, nar_at=(7,))
    w = rnd(sh.K * sh.C * sh.R * sh.S, nar_at=(5,))  # NaR in output channel 0
    dy = rnd(sh.N * sh.K * sh.OH * sh.OW, nar_at=(3,))

    def xat(n, c, ih, iw):
        return x[((n * sh.C + c) * sh.H + ih) * sh.W + iw] if 0 <= ih < sh.H and 0 <= iw < sh.W else 0

    # forward: rows (n,oh,ow), reduction (c,r,s)
    cols = [[xat(n, c, oh * sh.stride_h + r - sh.pad_h, ow * sh.stride_w + s - sh.pad_w)
             for c in range(sh.C) for r in range(sh.R) for s in range(sh.S)]
            for n in range(sh.N) for oh in range(sh.OH) for ow in range(sh.OW)]
    Wm = [w[k * sh.C * sh.R * sh.S:(k + 1) * sh.C * sh.R * sh.S] for k in range(sh.K)]
    Y = po.gemm(cols, Wm, fmt, fmt, trans_b=True)
    y = po.conv2d_fwd(x, w, sh, fmt, fmt)
    for n in range(sh.N):
        for k in range(sh.K):
            for i in range(sh.OH * sh.OW):
                assert y[(n * sh.K + k) * sh.OH * sh.OW + i] == Y[n * sh.OH * sh.OW + i][k]
    assert all(y[(n * sh.K + 0) * sh.OH * sh.OW + i] == 0x80 for n in range(sh.N) for i in range(sh.OH * sh.OW))
    # backward-weight: rows k, columns (c,r,s), reduction (n,oh,ow)
    dyT = [[dy[(n * sh.K + k) * sh.OH * sh.OW + i] for n in range(sh.N) for i in range(sh.OH * sh.OW)] for k in range(sh.K)]
    DW = po.gemm(dyT, cols, fmt, po.P16)
    dw = po.conv2d_bwd_weight(dy, x, sh, fmt, po.P16)
    assert dw == [DW[k][j] for k in range(sh.K) for j in range(sh.C * sh.R * sh.S)]
    # backward-data follows the scatter of LibTorch's flow (W^T times dY, every column entry sent back to
    # the input position it was unfolded from): the terms of a position are collected by walking the
    # FORWARD index map, the opposite loop order of the oracle's gather
    terms = {}
    for n in range(sh.N):
        for k in range(sh.K):
            for oh in range(sh.OH):
                for ow in range(sh.OW):
                    for c in range(sh.C):
                        for r in range(sh.R):
                            for s in range(sh.S):
                                h, ww = oh * sh.stride_h + r - sh.pad_h, ow * sh.stride_w + s - sh.pad_w
                                if 0 <= h < sh.H and 0 <= ww < sh.W:
                                    a, b = terms.setdefault((n, c, h, ww), ([], []))
                                    a.append(dy[((n * sh.K + k) * sh.OH + oh) * sh.OW + ow])
                                    b.append(w[((k * sh.C + c) * sh.R + r) * sh.S + s])
    dx = po.conv2d_bwd_data(dy, w, sh, fmt, fmt)
    for n in range(sh.N):
        for c in range(sh.C):
            for h in range(sh.H):
                for ww in range(sh.W):
                    a, b = terms.get((n, c, h, ww), ([], []))
                    assert dx[((n * sh.C + c) * sh.H + h) * sh.W + ww] == po.dot(a, b, fmt, fmt), (n, c, h, ww)
    # the NaR weight w[5] = w[k=0][c=0][r=2][s=1] reaches input row h from output row oh only when
    # 2*oh + 2 - 1 == h, i.e. odd h, and column ww from ow = ww: channel 0 is NaR on rows 1 and 3 only
    # (for every n and ww), apart from what the one NaR entry of dy adds
    assert (sh.stride_h, sh.pad_h, sh.R, sh.S) == (2, 1, 3, 2)
    dy_clean = [p if p != 0x80 else 0x40 for p in dy]
    dxc = po.conv2d_bwd_data(dy_clean, w, sh, fmt, fmt)
    for n in range(sh.N):
        for c in range(sh.C):
            for h in range(sh.H):
                for ww in range(sh.W):
                    is_nar = dxc[((n * sh.C + c) * sh.H + h) * sh.W + ww] == 0x80
                    assert is_nar == (c == 0 and h % 2 == 1 and ww - 1 + sh.pad_w >= 0 and ww - 1 + sh.pad_w < sh.OW), (n, c, h, ww)
