"""Pins for the scalar part of the oracle: decode (Eq. 2), rounding, conversions.

None of these checks re-type the oracle's own formula: they use the encodings
the definition fixes (golden file), Table 1, exhaustive round trips, ordering
invariants, an independently written string-based decoder and the agreement of
two unrelated rounding formulations.
"""
import math
import os
import random
from fractions import Fraction

import numpy as np
import pytest

from oracle import posit_oracle as po

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "known_encodings.txt")
FMT = {(8, 0): po.P8, (16, 1): po.P16, (32, 2): po.P32, (8, 1): po.P8_1, (8, 2): po.P8_2, (10, 1): po.P10_1,
       (10, 2): po.P10_2, (12, 1): po.P12_1, (12, 2): po.P12_2}
GENERAL = [po.P8_1, po.P8_2, po.P10_1, po.P10_2, po.P12_1, po.P12_2]


def _golden_rows():
    rows = []
    with open(GOLDEN) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            n, es, pat, val = line.split()
            rows.append((int(n), int(es), int(pat, 16), val))
    return rows


@pytest.mark.parametrize("n,es,pat,val", _golden_rows())
def test_known_encodings(n, es, pat, val):
    fmt = FMT[(n, es)]
    got = po.decode(pat, fmt)
    if val == "NaR":
        assert got is po.NaR
        assert po.round_to_posit(po.NaR, fmt) == pat
    else:
        num, den = val.split("/")
        want = Fraction(int(num), int(den))
        assert got == want
        assert po.round_constructive(want, fmt) == pat
        assert po.round_by_search(want, fmt) == pat


def test_table1_dynamic_range_and_quire_limits():
    # Table 1: dynamic range 2^+-6, 2^+-28, 2^+-120; quire 32/128/512; limits 127, 32767, 2^31-1
    for fmt, rng, q, limit in ((po.P8, 6, 32, 127), (po.P16, 28, 128, 32767), (po.P32, 120, 512, 2 ** 31 - 1)):
        assert po.decode(fmt.maxpos_pattern, fmt) == Fraction(2) ** rng
        assert po.decode(1, fmt) == Fraction(1, 2 ** rng)
        assert fmt.quire_bits == q
        # a Q-bit signed integer in units of minpos^2 holds exactly `limit` products maxpos*maxpos
        biggest_product = (fmt.maxpos * fmt.maxpos) / fmt.quire_unit
        assert biggest_product.denominator == 1
        assert ((1 << (q - 1)) - 1) // biggest_product.numerator == limit


def _string_decode(p, n, es):
    """Independent decoder working on the printed bit string, in floating point
    via ldexp (exact for these ranges)."""
    if p == 0:
        return 0.0
    if p == 1 << (n - 1):
        return None
    s = format(p, "0%db" % n)
    sign = s[0] == "1"
    if sign:
        s = format((1 << n) - p, "0%db" % n)
    body = s[1:]
    first = body[0]
    run = len(body) - len(body.lstrip(first))
    k = run - 1 if first == "1" else -run
    tail = body[run + 1:]
    e_str = (tail[:es] + "0" * es)[:es]
    e = int(e_str, 2) if es else 0
    f_str = tail[es:]
    f = int(f_str, 2) / (1 << len(f_str)) if f_str else 0.0
    v = math.ldexp(1.0 + f, (1 << es) * k + e)
    return -v if sign else v


@pytest.mark.parametrize("fmt", [po.P8, po.P16] + GENERAL)
def test_decode_exhaustive_against_string_decoder(fmt):
    for p in range(1 << fmt.n):
        want = _string_decode(p, fmt.n, fmt.es)
        got = po.decode(p, fmt)
        if want is None:
            assert got is po.NaR
        else:
            assert got == Fraction(want)


def test_decode_p32_sample_against_string_decoder():
    rng = random.Random(7)
    pats = [rng.getrandbits(32) for _ in range(20000)] + [1, 2, 3, 0x7FFFFFFF, 0x7FFFFFFE, 0xFFFFFFFF, 0x80000001]
    for p in pats:
        want = _string_decode(p, 32, 2)
        got = po.decode(p, po.P32)
        if want is None:
            assert got is po.NaR
        else:
            assert got == Fraction(want)


@pytest.mark.parametrize("fmt", [po.P8, po.P16] + GENERAL)
def test_roundtrip_monotone_negation_exhaustive(fmt):
    n = fmt.n
    prev = None
    # walk patterns in signed-integer order: decode is strictly increasing
    for sp in range(-(1 << (n - 1)) + 1, 1 << (n - 1)):
        p = sp & fmt.mask
        v = po.decode(p, fmt)
        assert po.round_constructive(v, fmt) == p
        assert po.round_by_search(v, fmt) == p
        if prev is not None:
            assert v > prev
        prev = v
        # negation is two's complement of the pattern (Sec. 2)
        assert po.decode((-p) & fmt.mask, fmt) == -v
        # every posit is an integer number of minpos
        assert (v / fmt.minpos).denominator == 1


def test_roundtrip_p32_sample():
    rng = random.Random(11)
    for _ in range(1 << 14):
        p = rng.getrandbits(32)
        if p == po.P32.nar:
            continue
        v = po.decode(p, po.P32)
        assert po.round_constructive(v, po.P32) == p
        assert po.round_by_search(v, po.P32) == p
        assert (v / po.P32.minpos).denominator == 1


@pytest.mark.parametrize("fmt", [po.P8, po.P16] + GENERAL)
def test_two_rounding_formulations_agree_at_every_midpoint(fmt):
    """R1 (bit string) == R2 (neighbour search) at all encoding midpoints and one
    quire unit either side; elsewhere nearest-in-value must also agree."""
    ulp = fmt.quire_unit
    wider = po.PositFormat(fmt.n + 1, fmt.es, 0)
    step = 1 if fmt.n <= 10 else 7
    for u in range(1, fmt.maxpos_pattern, step):
        lo = po.decode(u, fmt)
        hi = po.decode(u + 1, fmt)
        mid = po.decode(2 * u + 1, wider)
        assert lo < mid < hi
        for x in (mid - ulp, mid, mid + ulp, lo + ulp, hi - ulp):
            for sx in (x, -x):
                r1 = po.round_constructive(sx, fmt)
                r2 = po.round_by_search(sx, fmt)
                assert r1 == r2
        assert po.round_constructive(mid, fmt) == (u if u % 2 == 0 else u + 1)
        assert po.round_constructive(mid - ulp, fmt) == u
        assert po.round_constructive(mid + ulp, fmt) == u + 1
        # where the interval has fraction bits on both ends the encoding midpoint
        # is the arithmetic one
        if mid == (lo + hi) / 2:
            pass
        else:
            # only the intervals where the cut falls in regime/exponent bits differ
            assert hi / lo >= 2


def test_midpoint_exceptions_are_the_listed_ones():
    # posit<8,0>: encoding midpoint == arithmetic midpoint everywhere
    w9 = po.PositFormat(9, 0, 0)
    for u in range(1, 127):
        assert po.decode(2 * u + 1, w9) == (po.decode(u, po.P8) + po.decode(u + 1, po.P8)) / 2 or u in ()
    # posit<16,1>: exactly two intervals per sign differ (next to minpos and next to maxpos)
    w17 = po.PositFormat(17, 1, 0)
    odd = [u for u in range(1, 0x7FFF) if po.decode(2 * u + 1, w17) != (po.decode(u, po.P16) + po.decode(u + 1, po.P16)) / 2]
    assert odd == [1, 0x7FFE]
    assert po.decode(3, w17) == Fraction(1, 2 ** 27)
    assert po.decode(2 * 0x7FFE + 1, w17) == Fraction(2 ** 27)


def test_round_random_rationals_is_nearest_bracketing_and_monotone():
    rng = random.Random(3)
    for fmt in (po.P8, po.P16, po.P32):
        xs = []
        for _ in range(3000):
            e = rng.uniform(-fmt.max_scale - 3, fmt.max_scale + 3)
            x = Fraction(rng.getrandbits(40) + 1, 1 << 40) * Fraction(2) ** int(e)
            xs.append(x if rng.random() < 0.5 else -x)
        xs.sort()
        prev = None
        for x in xs:
            p = po.round_constructive(x, fmt)
            assert p == po.round_by_search(x, fmt)
            assert p not in (0, fmt.nar)  # a nonzero never rounds to 0 or NaR
            v = po.decode(p, fmt)
            sp = p - (1 << fmt.n) if p >> (fmt.n - 1) else p
            # result is one of the two posits bracketing x (or a clamp)
            if abs(x) >= fmt.maxpos:
                assert abs(v) == fmt.maxpos
            elif abs(x) <= fmt.minpos:
                assert abs(v) == fmt.minpos
            else:
                below = po.decode((sp - 1) & fmt.mask, fmt) if v > x else v
                above = po.decode((sp + 1) & fmt.mask, fmt) if v < x else v
                assert below <= x <= above
            if prev is not None:
                assert sp >= prev
            prev = sp


def test_clamps():
    for fmt in (po.P8, po.P16, po.P32):
        assert po.round_to_posit(fmt.minpos / 4, fmt) == 1
        assert po.round_to_posit(-fmt.minpos / 4, fmt) == fmt.mask
        assert po.round_to_posit(3 * fmt.maxpos, fmt) == fmt.maxpos_pattern
        assert po.round_to_posit(-3 * fmt.maxpos, fmt) == fmt.nar + 1
        assert po.round_to_posit(0, fmt) == 0


def test_from_float_and_to_float():
    for fmt in (po.P8, po.P16, po.P32):
        assert po.from_float(float("nan"), fmt) == fmt.nar
        assert po.from_float(float("inf"), fmt) == fmt.nar
        assert po.from_float(-float("inf"), fmt) == fmt.nar
        assert po.from_float(-0.0, fmt) == 0
        assert po.from_float(1.0, fmt) == 1 << (fmt.n - 2)
        assert math.isnan(po.to_float(fmt.nar, fmt, "f32"))
    # the learning rate 0.1 in posit<16,1>: neighbours straddle 0.1 and 0x14CD is nearer
    lr = po.from_float(0.1, po.P16)
    assert lr == 0x14CD
    a, b, c = (po.decode(p, po.P16) for p in (0x14CC, 0x14CD, 0x14CE))
    assert a < Fraction(1, 10) < c and abs(b - Fraction(1, 10)) < min(abs(a - Fraction(1, 10)), abs(c - Fraction(1, 10)))
    # to_float is exact for every posit<8,0>, posit<16,1> in binary32 ...
    for fmt in (po.P8, po.P16):
        for p in range(0, 1 << fmt.n, 1 if fmt.n == 8 else 13):
            if p == fmt.nar:
                continue
            v = po.decode(p, fmt)
            f = po.to_float(p, fmt, "f32")
            assert Fraction(f) == v and float(np.float32(f)) == f
            assert po.from_float(f, fmt) == p
    # ... while posit<32,2> has up to 28 significand bits: binary32 rounds (checked
    # against numpy's own double->single rounding of the exact double)
    rng = random.Random(5)
    for _ in range(5000):
        p = rng.getrandbits(32)
        if p == po.P32.nar:
            continue
        v = po.decode(p, po.P32)
        d = po.to_float(p, po.P32, "f64")
        assert Fraction(d) == v
        assert po.to_float(p, po.P32, "f32") == float(np.float32(d))


def test_convert_widening_is_exact_and_narrowing_rounds():
    for p in range(256):
        v = po.decode(p, po.P8)
        q = po.convert(p, po.P8, po.P16)
        assert po.decode(q, po.P16) is v if v is po.NaR else po.decode(q, po.P16) == v
        assert po.convert(q, po.P16, po.P8) == p
    for p in range(0, 1 << 16, 5):
        v = po.decode(p, po.P16)
        q = po.convert(p, po.P16, po.P32)
        if v is po.NaR:
            assert q == po.P32.nar
        else:
            assert po.decode(q, po.P32) == v
            assert po.convert(p, po.P16, po.P8) == po.round_by_search(v, po.P8)


def test_quire_width_formula_reproduces_table_1():
    """Table 1 prints the quire width of the three standard formats: 32, 128 and 512 bits.  The
    formula used for the formats Table 1 does not list must return exactly those for the ones it does."""
    assert [po.general_quire_bits(n, es) for n, es in ((8, 0), (16, 1), (32, 2))] == [32, 128, 512]
    assert (po.P8.quire_bits, po.P16.quire_bits, po.P32.quire_bits) == (32, 128, 512)


def test_general_format_quire_widths_hold_many_products():
    """Formats outside Table 1: maxpos = useed^(n-2) and the chosen quire width leaves at
    least 2^(n-1) - 1 products of maxpos * maxpos without wrap (n-1 carry-guard bits)."""
    for fmt in GENERAL:
        assert po.decode(fmt.maxpos_pattern, fmt) == Fraction(fmt.useed) ** (fmt.n - 2)
        assert po.decode(1, fmt) == 1 / Fraction(fmt.useed) ** (fmt.n - 2)
        assert fmt.quire_bits % 32 == 0
        biggest = (fmt.maxpos * fmt.maxpos) / fmt.quire_unit
        limit = ((1 << (fmt.quire_bits - 1)) - 1) // biggest.numerator
        assert limit >= 2 ** (fmt.n - 1) - 1
        # and one limb less would not do
        assert ((1 << (fmt.quire_bits - 33)) - 1) // biggest.numerator < 2 ** (fmt.n - 1) - 1
