"""Pins of the oracle's elementary functions, division and losses (paper Fig. 2: Sigmoid, TanH, Cross
Entropy, MSE; Sec. 4 Table 4: loss in posit(10,2) / posit(12,2))."""
import bisect
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import posit_oracle as po

LOSS_FORMATS = ["p8", "p16", "p8_2", "p10_2", "p12_2", "p12_1"]
LIBM = {"exp": math.exp, "log": math.log, "tanh": math.tanh, "sigmoid": lambda x: 1.0 / (1.0 + math.exp(-x))}


def _libm_candidates(fn, x, fmt):
    """Patterns that the correctly rounded result may be, given libm's double (a few ulp off at most):
    the roundings of the two ends of a 2^-45 relative bracket around it."""
    try:
        v = LIBM[fn](x)
    except OverflowError:
        return None
    if v == 0.0 or math.isinf(v):
        return None
    f = Fraction(v)
    eps = Fraction(1, 1 << 45)
    return {po.round_to_posit(f * (1 - eps), fmt), po.round_to_posit(f * (1 + eps), fmt)}


@pytest.mark.parametrize("name", ["p8", "p8_2", "p10_2", "p12_2"])
@pytest.mark.parametrize("fn", po.UNARY)
def test_unary_agrees_with_libm_within_one_rounding(fn, name):
    fmt = po.FORMATS[name]
    checked = 0
    for p in range(1 << fmt.n):
        if p == fmt.nar:
            assert po.unary(fn, p, fmt) == fmt.nar
            continue
        x = po.decode(p, fmt)
        if fn == "log" and x <= 0:
            assert po.unary(fn, p, fmt) == fmt.nar
            continue
        if abs(x) > 700 or (fn == "sigmoid" and abs(x) > 30) or (fn == "tanh" and abs(x) < 1e-5):
            continue  # libm overflows, or loses the last bits of 1 - tiny / of x - x^3/3
        cands = _libm_candidates(fn, float(x), fmt)
        if cands is None:
            continue
        assert po.unary(fn, p, fmt) in cands, (fn, p)
        checked += 1
    assert checked > (1 << fmt.n) // 4


@pytest.mark.parametrize("name", LOSS_FORMATS)
def test_unary_exact_cases_clamps_and_symmetry(name):
    fmt = po.FORMATS[name]
    one = 1 << (fmt.n - 2)
    half = po.round_to_posit(Fraction(1, 2), fmt)
    maxpos, minpos = fmt.nar - 1, 1
    assert po.unary("exp", 0, fmt) == one and po.unary("log", one, fmt) == 0
    assert po.unary("tanh", 0, fmt) == 0 and po.unary("sigmoid", 0, fmt) == half
    # saturation: e^maxpos clamps to maxpos, e^-maxpos and sigmoid(-maxpos) to minpos (never zero)
    assert po.unary("exp", maxpos, fmt) == maxpos and po.unary("exp", po.neg(maxpos, fmt), fmt) == minpos
    assert po.unary("sigmoid", po.neg(maxpos, fmt), fmt) == minpos and po.unary("sigmoid", maxpos, fmt) == one
    assert po.unary("tanh", maxpos, fmt) == one and po.unary("tanh", po.neg(maxpos, fmt), fmt) == po.neg(one, fmt)
    assert po.unary("log", 0, fmt) == fmt.nar and po.unary("log", po.neg(one, fmt), fmt) == fmt.nar
    rng = np.random.default_rng(fmt.n)
    pats = sorted((int(v) for v in rng.integers(0, 1 << fmt.n, 300) if int(v) != fmt.nar), key=lambda p: po.decode(p, fmt))
    for fn in ("exp", "sigmoid", "tanh"):
        vals = [po.decode(po.unary(fn, p, fmt), fmt) for p in pats]
        assert all(a <= b for a, b in zip(vals, vals[1:])), fn  # monotone
    for p in pats[:100]:
        assert po.unary("tanh", po.neg(p, fmt), fmt) == po.neg(po.unary("tanh", p, fmt), fmt)  # odd
        s = po.decode(po.unary("sigmoid", p, fmt), fmt)
        assert 0 < s <= 1


def test_division_is_nearest_exhaustively_posit8():
    fmt = po.P8
    real = sorted((po.decode(p, fmt), p) for p in range(256) if p != fmt.nar)
    values, patterns = [v for v, _ in real], [p for _, p in real]

    def nearest(x):
        if x == 0:
            return 0
        i = bisect.bisect_left(values, x)
        cands = [j for j in (i - 1, i, i + 1) if 0 <= j < len(values) and values[j] != 0]
        best = min(abs(values[j] - x) for j in cands)
        tied = [patterns[j] for j in cands if abs(values[j] - x) == best]
        return tied[0] if len(tied) == 1 else [p for p in tied if p % 2 == 0][0]

    for a in range(256):
        for b in range(256):
            if a == fmt.nar or b == fmt.nar or b == 0:
                assert po.div(a, b, fmt) == fmt.nar
            else:
                assert po.div(a, b, fmt) == nearest(po.decode(a, fmt) / po.decode(b, fmt)), (a, b)


@pytest.mark.parametrize("name", LOSS_FORMATS)
def test_division_identities(name):
    fmt = po.FORMATS[name]
    one = 1 << (fmt.n - 2)
    rng = np.random.default_rng(fmt.n + 1)
    for a in (int(v) for v in rng.integers(0, 1 << fmt.n, 300)):
        if a in (0, fmt.nar):
            continue
        assert po.div(a, a, fmt) == one and po.div(a, one, fmt) == a and po.div(0, a, fmt) == 0
        assert po.div(po.neg(a, fmt), a, fmt) == po.neg(one, fmt)


def test_unary_bwd_closed_forms():
    f = po.P16
    r = lambda x: po.round_to_posit(Fraction(x), f)
    # sigmoid: y = 1/2, dy = 1 -> 1/4 ; y = 1/4, dy = -2 -> -2 * 3/16 = -3/8
    assert po.unary_bwd("sigmoid", r(Fraction(1, 2)), r(1), f, f) == r(Fraction(1, 4))
    assert po.unary_bwd("sigmoid", r(Fraction(1, 4)), r(-2), f, f) == r(Fraction(-3, 8))
    # tanh: y = 1/2, dy = 4 -> 4 * 3/4 = 3 ; y = 1 -> 0 ; y = 0 -> dy
    assert po.unary_bwd("tanh", r(Fraction(1, 2)), r(4), f, f) == r(3)
    assert po.unary_bwd("tanh", r(1), r(4), f, f) == 0 and po.unary_bwd("tanh", 0, r(4), f, f) == r(4)
    assert po.unary_bwd("tanh", f.nar, r(4), f, f) == f.nar


def test_cross_entropy_closed_forms():
    f8, f16 = po.P8, po.P16
    ln = lambda c: po.round_to_posit(Fraction(math.log(c)), f16)  # ln 2, ln 4 are far from any posit<16,1> boundary
    # C equal logits: e_j = 1, S = C, p_j = 1/C (exact for C = 2, 4), loss = ln C
    q = lambda x: po.round_to_posit(Fraction(x), f16)
    loss, g = po.cross_entropy([[0x40, 0x40]], [0], f8, f16, f16)
    assert loss == ln(2) and g == [[q(Fraction(-1, 2)), q(Fraction(1, 2))]]
    assert q(Fraction(1, 2)) == 0x3000 and q(Fraction(-1, 2)) == 0xD000  # 0 | 01 | 1 | 0..: regime k=-1, exponent 1
    loss, g = po.cross_entropy([[0x30] * 4, [0x55] * 4], [1, 3], f8, f16, f16)
    assert loss == ln(4)
    assert g == [[q(Fraction(1, 8)), q(Fraction(-3, 8)), q(Fraction(1, 8)), q(Fraction(1, 8))],
                 [q(Fraction(1, 8)), q(Fraction(1, 8)), q(Fraction(1, 8)), q(Fraction(-3, 8))]]
    # NaR logit or bad label: that row's gradient and the loss are NaR, other rows unaffected
    loss, g = po.cross_entropy([[0x40, 0x80], [0x40, 0x40]], [0, 1], f8, f16, f16)
    assert loss == f16.nar and g[0] == [f16.nar, f16.nar] and g[1] == [q(Fraction(1, 4)), q(Fraction(-1, 4))]
    loss, g = po.cross_entropy([[0x40, 0x40]], [2], f8, f16, f16)
    assert loss == f16.nar and g[0] == [f16.nar, f16.nar]


@pytest.mark.parametrize("fl", ["p16", "p12_2", "p10_2"])
def test_cross_entropy_close_to_float64(fl):
    """Sanity against the float64 definition (softmax - onehot) / B and mean(-log softmax): a wrong sign,
    index or scale is far outside the few-ulp band that rounding in a 10..16-bit loss format allows."""
    f_in, f_l = po.FORMATS["p8_2"], po.FORMATS[fl]
    rng = np.random.default_rng(7)
    B, C = 8, 10
    z = rng.normal(0, 2, (B, C))
    logits = [[po.from_float(v, f_in) for v in row] for row in z]
    labels = [int(v) for v in rng.integers(0, C, B)]
    zq = np.array([[float(po.decode(p, f_in)) for p in row] for row in logits])
    sm = np.exp(zq - zq.max(1, keepdims=True))
    sm /= sm.sum(1, keepdims=True)
    want_g = sm.copy()
    want_g[np.arange(B), labels] -= 1
    want_g /= B
    want_loss = float(np.mean(-np.log(sm[np.arange(B), labels])))
    loss, g = po.cross_entropy(logits, labels, f_in, f_l, f_l)
    tol = 2.0 ** -(f_l.n - 7)  # relative: a handful of roundings at the precision the format has near these magnitudes
    assert abs(float(po.decode(loss, f_l)) - want_loss) <= tol * want_loss
    got = np.array([[float(po.decode(p, f_l)) for p in row] for row in g])
    assert np.all(np.abs(got - want_g) <= tol * np.abs(want_g) + 2.0 ** -(f_l.n + 2))
    assert np.all(np.sign(got) == np.sign(want_g))


def test_mse_closed_forms():
    f8, f16 = po.P8, po.P16
    q = lambda x: po.round_to_posit(Fraction(x), f16)
    p8 = lambda x: po.round_to_posit(Fraction(x), f8)
    pred = [p8(1), p8(Fraction(3, 2)), p8(-2), p8(0)]
    target = [p8(Fraction(3, 4)), p8(Fraction(3, 2)), p8(1), p8(-1)]
    # d = (1/4, 0, -3, 1): loss = (1/16 + 9 + 1) / 4, dpred = 2 d / 4
    loss, g = po.mse(pred, target, f8, f16, f16)
    assert loss == q(Fraction(161, 64)) and g == [q(Fraction(1, 8)), 0, q(Fraction(-3, 2)), q(Fraction(1, 2))]
    loss, g = po.mse([p8(1), 0x80], [p8(1), p8(1)], f8, f16, f16)
    assert loss == f16.nar and g == [0, f16.nar]
