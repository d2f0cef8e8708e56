"""Pins of the oracle's accumulation without the quire (paper Sec. 3.3: the quire is an option;
Table 2 trains "without quire"): the two rounded operations and the order of the terms."""
import bisect
from fractions import Fraction

import numpy as np
import pytest

from oracle import fast
from oracle import posit_oracle as po

GENERAL = ["p8_1", "p8_2", "p10_1", "p10_2", "p12_1", "p12_2"]


def _nearest_by_search(x, fmt, values, patterns):
    """Nearest posit to the exact rational x by looking through the sorted value table: never 0 or NaR for
    x != 0, beyond maxpos clamps; a tie goes to the even pattern.  Valid where nearest in the encoding and
    nearest in value coincide, which for posit<8,0> is everywhere."""
    if x == 0:
        return 0
    i = bisect.bisect_left(values, x)
    cands = [j for j in (i - 1, i, i + 1) if 0 <= j < len(values) and values[j] != 0]
    best = min(abs(values[j] - x) for j in cands)
    tied = [patterns[j] for j in cands if abs(values[j] - x) == best]
    if len(tied) == 1:
        return tied[0]
    even = [p for p in tied if p % 2 == 0]
    assert len(even) == 1
    return even[0]


def test_posit8_add_and_mul_are_nearest_exhaustively():
    fmt = po.P8
    real = sorted((po.decode(p, fmt), p) for p in range(256) if p != fmt.nar)
    values = [v for v, _ in real]
    patterns = [p for _, p in real]
    for a in range(256):
        for b in range(a, 256):
            if a == fmt.nar or b == fmt.nar:
                assert po.add(a, b, fmt) == fmt.nar and po.mul(a, b, fmt) == fmt.nar
                continue
            va, vb = po.decode(a, fmt), po.decode(b, fmt)
            assert po.add(a, b, fmt) == _nearest_by_search(va + vb, fmt, values, patterns), (a, b)
            assert po.mul(a, b, fmt) == _nearest_by_search(va * vb, fmt, values, patterns), (a, b)


@pytest.mark.parametrize("name", ["p8", "p16", "p32"] + GENERAL)
def test_algebraic_identities_of_the_rounded_operations(name):
    fmt = po.FORMATS[name]
    rng = np.random.default_rng(fmt.n * 5 + fmt.es)
    one = 1 << (fmt.n - 2)
    neg = lambda p: (-p) & fmt.mask
    for _ in range(400):
        a, b = (int(v) for v in rng.integers(0, 1 << fmt.n, 2))
        assert po.add(a, b, fmt) == po.add(b, a, fmt)
        assert po.mul(a, b, fmt) == po.mul(b, a, fmt)
        assert po.add(a, 0, fmt) == a and po.mul(a, one, fmt) == a
        if a != fmt.nar:
            assert po.add(a, neg(a), fmt) == 0
            assert po.mul(a, 0, fmt) == 0
        if a != fmt.nar and b != fmt.nar:
            assert po.mul(neg(a), b, fmt) == neg(po.mul(a, b, fmt))  # rounding is symmetric in the sign
            assert po.add(neg(a), neg(b), fmt) == neg(po.add(a, b, fmt))
    assert po.mul(fmt.nar, 0, fmt) == fmt.nar and po.add(fmt.nar, one, fmt) == fmt.nar


def test_sum_is_monotone_in_each_term_posit8():
    """x -> add(a, x) never decreases as x runs through the posits in value order."""
    fmt = po.P8
    order = sorted((p for p in range(256) if p != fmt.nar), key=lambda p: po.decode(p, fmt))
    for a in (0x01, 0x20, 0x40, 0x55, 0x7F, 0xC0, 0xFF):
        sums = [po.decode(po.add(a, x, fmt), fmt) for x in order]
        assert all(s0 <= s1 for s0, s1 in zip(sums, sums[1:]))


def test_worked_example_where_the_quire_matters():
    """posit<8,0> has 5 fraction bits next to one, so 1 + 1/64 lies halfway between the patterns 0x40 (1) and
    0x41 (1 + 1/32) and goes to the even one, 0x40: forty terms of 1/64 added one at a time never move the
    sum, while the exact sum 1 + 40/64 = 1.625 = 1 + 20/32 is the pattern 0x40 + 20."""
    fmt = po.P8
    assert po.decode(0x01, fmt) == Fraction(1, 64) and po.decode(0x40, fmt) == 1
    a = [0x40] + [0x01] * 40
    b = [0x40] * 41
    assert po.dot_noquire(a, b, fmt, fmt) == 0x40
    assert po.dot(a, b, fmt, fmt) == 0x54
    # and the order matters: the small terms first reach 40/64 = 0.625 exactly, then + 1 = 1.625
    assert po.dot_noquire(a[::-1], b, fmt, fmt) == 0x54


def test_noquire_equals_quire_when_nothing_is_rounded():
    """Small integers in posit<16,1>: every product and partial sum is representable, so both modes agree."""
    fmt = po.P16
    rng = np.random.default_rng(4)
    ints = [po.round_to_posit(Fraction(int(v)), fmt) for v in range(-8, 9)]
    for _ in range(20):
        a = [ints[i] for i in rng.integers(0, len(ints), 12)]
        b = [ints[i] for i in rng.integers(0, len(ints), 12)]
        assert po.dot_noquire(a, b, fmt, fmt) == po.dot(a, b, fmt, fmt)


def test_bias_is_added_last_and_final_conversion():
    fmt = po.P8
    # thirty-two terms of 1/64 reach 0.5 exactly; the bias 1 added after them gives 1.5 = pattern 0x50.
    # Had the bias come first, the sum would have stuck at 1 (see the worked example above): 0x40.
    a, b = [0x01] * 32, [0x40] * 32
    assert po.dot_noquire(a, b, fmt, fmt, bias=0x40) == 0x50
    assert po.dot_noquire([0x40] + a, [0x40] + b, fmt, fmt) == 0x40
    # the running posit is converted, not re-derived: posit<8,0> result widened exactly
    assert po.dot_noquire(a, b, fmt, po.P16, bias=0x40) == po.round_to_posit(Fraction(3, 2), po.P16)
    assert po.dot_noquire([fmt.nar], [0], fmt, po.P16) == po.P16.nar


CONVS = [
    po.ConvShape(2, 3, 6, 5, 4, 3, 3, 1, 1, 1, 1),
    po.ConvShape(2, 2, 7, 6, 3, 3, 2, 1, 0, 2, 1),
    po.ConvShape(1, 2, 5, 5, 2, 2, 2, 0, 1, 1, 2),
]


@pytest.mark.parametrize("ci", range(len(CONVS)))
def test_term_sequences_reproduce_the_quire_convolutions(ci):
    """The operand sequences that the no-quire convolutions fold over, summed exactly instead, are the
    (separately pinned) quire convolutions: same terms, so only the order is new."""
    sh = CONVS[ci]
    fmt = po.P8
    rng = np.random.default_rng(ci)
    x = [int(v) for v in rng.integers(0, 256, sh.N * sh.C * sh.H * sh.W)]
    w = [int(v) for v in rng.integers(0, 256, sh.K * sh.C * sh.R * sh.S)]
    dy = [int(v) for v in rng.integers(0, 256, sh.N * sh.K * sh.OH * sh.OW)]
    assert [po.dot(a, b, fmt, po.P16) for a, b in po.conv2d_fwd_terms(x, w, sh)] == po.conv2d_fwd(x, w, sh, fmt, po.P16)
    assert [po.dot(a, b, fmt, po.P16) for a, b in po.conv2d_bwd_data_terms(dy, w, sh)] == po.conv2d_bwd_data(dy, w, sh, fmt, po.P16)
    assert [po.dot(a, b, fmt, po.P16) for a, b in po.conv2d_bwd_weight_terms(dy, x, sh)] == po.conv2d_bwd_weight(dy, x, sh, fmt, po.P16)
    assert [po.dot(a, b, fmt, po.P16) for a, b in po.conv2d_bias_grad_terms(dy, sh, fmt)] == po.conv2d_bias_grad(dy, sh, fmt, po.P16)


def test_term_order_is_that_of_the_unfolded_matrix():
    """Forward terms run over (c, r, s) with s fastest: the flattened weight of one output channel, in order."""
    sh = po.ConvShape(1, 2, 4, 4, 2, 2, 3, 0, 0, 1, 1)
    x = list(range(1, 1 + sh.C * sh.H * sh.W))
    w = list(range(100, 100 + sh.K * sh.C * sh.R * sh.S))
    terms = po.conv2d_fwd_terms(x, w, sh)
    per = sh.C * sh.R * sh.S
    a0, b0 = terms[0]
    assert b0 == w[:per]
    assert a0 == [x[(c * sh.H + r) * sh.W + s] for c in range(sh.C) for r in range(sh.R) for s in range(sh.S)]
    # backward-weight terms run over (n, oh, ow): the flattened output gradient of one channel per image
    sh2 = po.ConvShape(2, 1, 3, 3, 2, 2, 2, 0, 0, 1, 1)
    dy = list(range(1, 1 + sh2.N * sh2.K * sh2.OH * sh2.OW))
    xx = list(range(50, 50 + sh2.N * sh2.C * sh2.H * sh2.W))
    a, _ = po.conv2d_bwd_weight_terms(dy, xx, sh2)[0]
    assert a == [dy[(n * sh2.K + 0) * 4 + i] for n in range(2) for i in range(4)]


# ---- the C++ oracle against the Python one ----

@pytest.mark.parametrize("fin,fout", [("p8", "p8"), ("p8", "p16"), ("p16", "p16"), ("p32", "p32"), ("p8_2", "p12_2"), ("p10_1", "p10_1"),
                                      ("p12_2", "p8_2"), ("p8_1", "p8_1")])
def test_fast_gemm_noquire_matches_python(fin, fout):
    f_in, f_out = po.FORMATS[fin], po.FORMATS[fout]
    rng = np.random.default_rng(f_in.n + 3 * f_out.n)
    M, N, K = 5, 6, 23
    A = rng.integers(0, 1 << f_in.n, (M, K), dtype=np.uint64)
    B = rng.integers(0, 1 << f_in.n, (K, N), dtype=np.uint64)
    A[1, 3] = f_in.nar
    B[4, 2] = 0
    bias = rng.integers(0, 1 << f_in.n, N, dtype=np.uint64)
    got, _ = fast.gemm(A, B, fin, fout, bias=bias, noquire=True, threads=2)
    want = po.gemm_noquire(A.tolist(), B.tolist(), f_in, f_out, bias=bias.tolist())
    assert got.tolist() == want
    got, _ = fast.gemm(A.T.copy(), B.T.copy(), fin, fout, trans_a=True, trans_b=True, noquire=True, threads=1)
    assert got.tolist() == po.gemm_noquire(A.tolist(), B.tolist(), f_in, f_out)
    # differs from the quire result somewhere (otherwise the mode flag is not being honoured)
    ref, _ = fast.gemm(A, B, fin, fout, bias=bias, threads=1)
    if fin != "p32":
        assert (ref != np.array(want)).any()


@pytest.mark.parametrize("ci", range(len(CONVS)))
@pytest.mark.parametrize("fin,fout", [("p8", "p8"), ("p16", "p8"), ("p8_2", "p12_2")])
def test_fast_conv_noquire_matches_python(ci, fin, fout):
    sh = CONVS[ci]
    f_in, f_out = po.FORMATS[fin], po.FORMATS[fout]
    d = dict(N=sh.N, C=sh.C, H=sh.H, W=sh.W, K=sh.K, R=sh.R, S=sh.S, pad_h=sh.pad_h, pad_w=sh.pad_w, stride_h=sh.stride_h, stride_w=sh.stride_w)
    rng = np.random.default_rng(ci + f_in.n)
    x = rng.integers(0, 1 << f_in.n, (sh.N, sh.C, sh.H, sh.W), dtype=np.uint64)
    w = rng.integers(0, 1 << f_in.n, (sh.K, sh.C, sh.R, sh.S), dtype=np.uint64)
    dy = rng.integers(0, 1 << f_in.n, (sh.N, sh.K, sh.OH, sh.OW), dtype=np.uint64)
    bias = rng.integers(0, 1 << f_in.n, sh.K, dtype=np.uint64)
    xf, wf, dyf = x.flatten().tolist(), w.flatten().tolist(), dy.flatten().tolist()
    assert fast.conv2d_fwd(x, w, d, fin, fout, bias=bias, noquire=True).flatten().tolist() == po.conv2d_fwd_noquire(xf, wf, sh, f_in, f_out, bias.tolist())
    assert fast.conv2d_bwd_data(dy, w, d, fin, fout, noquire=True).flatten().tolist() == po.conv2d_bwd_data_noquire(dyf, wf, sh, f_in, f_out)
    dw, db = fast.conv2d_bwd_weight(dy, x, d, fin, fout, with_bias=True, noquire=True)
    assert dw.flatten().tolist() == po.conv2d_bwd_weight_noquire(dyf, xf, sh, f_in, f_out)
    assert db.tolist() == po.conv2d_bias_grad_noquire(dyf, sh, f_in, f_out)
