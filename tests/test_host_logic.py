"""The library's scalar device functions (decode, encode, quire limbs, exact add),
compiled for the host, against the oracle.  Runs without a GPU; the kernels
call exactly these functions."""
import ctypes
from fractions import Fraction
import os

import numpy as np
import pytest

from oracle import fast
from oracle import posit_oracle as po

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2105_00053_amd", "libpositnn_hostcheck.so")
CODE = {"p8": 0, "p16": 1, "p32": 2, "f32": 100, "f64": 101, "p8_1": 3, "p8_2": 4, "p10_1": 5, "p10_2": 6, "p12_1": 7, "p12_2": 8}
BITS = {"p8": 8, "p16": 16, "p32": 32, "p8_1": 8, "p8_2": 8, "p10_1": 10, "p10_2": 10, "p12_1": 12, "p12_2": 12}
GENERAL = ["p8_1", "p8_2", "p10_1", "p10_2", "p12_1", "p12_2"]


@pytest.fixture(scope="module")
def hc():
    if not os.path.exists(LIB):
        from paper_2105_00053_amd import build
        build.build()
    L = ctypes.CDLL(LIB)
    vp, i64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
    L.hostcheck_round.argtypes = [ci, ci, i64, vp, vp]
    L.hostcheck_convert.argtypes = [ci, ci, i64, vp, vp]
    L.hostcheck_axpy.argtypes = [ci, ci, ctypes.c_uint32, i64, vp, vp, vp]
    L.hostcheck_dot.argtypes = [ci, ci, i64, vp, vp, ci, ctypes.c_uint32]
    L.hostcheck_dot.restype = ctypes.c_uint32
    L.hostcheck_conv_gather.argtypes = [ci, vp, ci, i64, i64, vp, vp, vp]
    L.hostcheck_dot_noquire.restype = ctypes.c_uint32
    L.hostcheck_dot_noquire.argtypes = [ci, ci, i64, vp, vp, ci, ctypes.c_uint32]
    L.hostcheck_dot_bucket.restype = ctypes.c_uint32
    L.hostcheck_dot_bucket.argtypes = [ci, ci, i64, vp, vp, ci, ctypes.c_uint32]
    L.hostcheck_dot_cascade.restype = ctypes.c_uint32
    L.hostcheck_dot_cascade.argtypes = [ci, ci, i64, vp, vp, ci, ctypes.c_uint32]
    L.hostcheck_bucket_config.argtypes = [ci, vp, vp, vp]
    L.hostcheck_bucket_flush.argtypes = [ci, ci, ctypes.c_double, vp]
    L.hostcheck_bucket_split.argtypes = [ci, ctypes.c_uint32, ctypes.c_uint32, vp, vp]
    L.hostcheck_posit_op.restype = ctypes.c_uint32
    L.hostcheck_posit_op.argtypes = [ci, ci, ctypes.c_uint32, ctypes.c_uint32]
    L.hostcheck_div_int.restype = ctypes.c_uint32
    L.hostcheck_div_int.argtypes = [ci, ci, ctypes.c_uint32, ci, ctypes.c_uint32]
    L.hostcheck_map_rt.argtypes = [ci, ci, i64, vp, vp]
    L.hostcheck_axpy_rt.argtypes = [ci, ci, ctypes.c_uint32, i64, vp, vp, vp]
    L.hostcheck_axpy_f64.argtypes = [ci, ci, ctypes.c_uint32, i64, vp, vp, vp]
    L.hostcheck_narrow_step.argtypes = [i64, vp, vp]
    L.hostcheck_p8_round_quire.argtypes = [i64, vp, vp]
    L.hostcheck_round_f64.restype = ctypes.c_uint32
    L.hostcheck_round_f64.argtypes = [ci, ctypes.c_double, ci, ci]
    return L


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _patterns(rng, n, fmt, special=0.03):
    b = BITS[fmt]
    a = rng.integers(0, 1 << b, size=n, dtype=np.uint64)
    sp = rng.choice(np.array([0, 1, 2, (1 << (b - 1)) - 1, (1 << (b - 1)) - 2, (1 << b) - 1, (1 << (b - 1)) + 1, 1 << (b - 1), 1 << (b - 2)],
                             dtype=np.uint64), size=n)
    return np.where(rng.random(n) < special, sp, a)


@pytest.mark.parametrize("dst", ["p8", "p16", "p32"])
def test_round_from_floats(hc, dst):
    rng = np.random.default_rng(1)
    x = (rng.standard_normal(200000) * np.exp2(rng.uniform(-70, 70, 200000))).astype(np.float32)
    x[:10] = [0.0, -0.0, np.inf, -np.inf, np.nan, 1e-45, -1e-45, 3.4e38, 1.0, -1.0]
    bits = x.view(np.uint32).astype(np.uint64)
    out = np.zeros_like(bits)
    hc.hostcheck_round(100, CODE[dst], len(bits), _p(bits), _p(out))
    assert np.array_equal(out, fast.round_from_float(x, dst).astype(np.uint64))
    xd = rng.standard_normal(200000) * np.exp2(rng.uniform(-300, 300, 200000))
    xd[:6] = [5e-324, -5e-324, 1.7e308, np.nan, -np.inf, 2.0 ** -120]
    bits = xd.view(np.uint64).copy()
    hc.hostcheck_round(101, CODE[dst], len(bits), _p(bits), _p(out))
    assert np.array_equal(out, fast.round_from_float(xd, dst).astype(np.uint64))


@pytest.mark.parametrize("src", ["p8", "p16", "p32"])
@pytest.mark.parametrize("dst", ["p8", "p16", "p32", "f32", "f64"])
def test_convert(hc, src, dst):
    if src == "p32":
        pats = _patterns(np.random.default_rng(2), 300000, "p32")
    else:
        pats = np.arange(1 << BITS[src], dtype=np.uint64)
    out = np.zeros_like(pats)
    assert hc.hostcheck_convert(CODE[src], CODE[dst], len(pats), _p(pats), _p(out)) == 0
    if dst in ("f32", "f64"):
        want = fast.to_float(pats, src, dst)
        got = out.astype(np.uint32).view(np.float32) if dst == "f32" else out.view(np.float64)
        nan = np.isnan(want)
        assert np.array_equal(np.isnan(got), nan)
        assert np.array_equal(got[~nan], want[~nan])
    else:
        assert np.array_equal(out, fast.convert(pats, src, dst).astype(np.uint64))


@pytest.mark.parametrize("fx", ["p8", "p16", "p32"])
@pytest.mark.parametrize("fy", ["p8", "p16", "p32"])
def test_axpy(hc, fx, fy):
    rng = np.random.default_rng(BITS[fx] + 7 * BITS[fy])
    n = 60000
    x = _patterns(rng, n, fx)
    y = _patterns(rng, n, fy)
    # near-cancelling cases: y close to -alpha*x
    alphas = [int(fast.round_from_float(np.array([-0.1], dtype=np.float32), fy)[0]), 1 << (BITS[fy] - 2),
              int(_patterns(rng, 1, fy, 0)[0]), 0, 1 << (BITS[fy] - 1), (1 << (BITS[fy] - 2)) | (1 << (BITS[fy] - 1))]
    for alpha in alphas:
        out = np.zeros(n, dtype=np.uint64)
        assert hc.hostcheck_axpy(CODE[fx], CODE[fy], alpha, n, _p(x), _p(y), _p(out)) == 0
        want = fast.axpy(alpha, x, y, fx, fy)
        assert np.array_equal(out, want.astype(np.uint64)), alpha
    # y = -x in the same format with alpha = 1 cancels exactly; y = -x +- 1 pattern nearly cancels
    if fx == fy:
        one = 1 << (BITS[fy] - 2)
        mask = (1 << BITS[fy]) - 1
        for delta in (0, 1, -1, 2):
            y2 = ((-x.astype(np.int64) + delta) & mask).astype(np.uint64)
            out = np.zeros(n, dtype=np.uint64)
            hc.hostcheck_axpy(CODE[fx], CODE[fy], one, n, _p(x), _p(y2), _p(out))
            assert np.array_equal(out, fast.axpy(one, x, y2, fx, fy).astype(np.uint64))


@pytest.mark.parametrize("fx,fy", [("p8", "p16"), ("p16", "p16"), ("p8", "p8"), ("p16", "p8"), ("p32", "p32"), ("p16", "p32")])
def test_axpy_near_cancellation(hc, fx, fy):
    """y chosen as the rounded value of -alpha*x, then nudged by a few patterns: the sum
    cancels almost completely, which is where an inexact alignment would show."""
    rng = np.random.default_rng(BITS[fx] * 5 + BITS[fy])
    n = 40000
    x = _patterns(rng, n, fx, special=0.0)
    mask = (1 << BITS[fy]) - 1
    for alpha in (int(fast.round_from_float(np.array([-0.1], dtype=np.float32), fy)[0]), int(_patterns(rng, 1, fy, 0)[0]) | 1):
        zero = np.zeros(n, dtype=np.uint64)
        t = fast.axpy(alpha, x, zero, fx, fy).astype(np.int64)  # round(alpha * x)
        for delta in (0, 1, -1, 3, -7, 64):
            y = ((-t + delta) & mask).astype(np.uint64)
            out = np.zeros(n, dtype=np.uint64)
            assert hc.hostcheck_axpy(CODE[fx], CODE[fy], alpha, n, _p(x), _p(y), _p(out)) == 0
            assert np.array_equal(out, fast.axpy(alpha, x, y, fx, fy).astype(np.uint64)), (alpha, delta)


F64_PAIRS = [("p16", "p16"), ("p8", "p16"), ("p12_2", "p12_2"), ("p8_2", "p12_2"), ("p8", "p8"), ("p10_1", "p12_1")]


@pytest.mark.parametrize("fx,fy", F64_PAIRS)
def test_axpy_through_binary64_with_error_free_sum(hc, fx, fy):
    """The arithmetic of the large-tensor update kernel: product in binary64, sum with its exact error term, one
    rounding.  Random patterns, special patterns, sums that cancel almost completely, and terms so far apart that
    the smaller one lies wholly below the larger one's last bit (where the error term alone decides a tie)."""
    rng = np.random.default_rng(BITS[fx] * 3 + BITS[fy] + CODE[fy])
    n = 80000
    mask = (1 << BITS[fy]) - 1
    x = _patterns(rng, n, fx)
    y = _patterns(rng, n, fy)
    lr = int(fast.round_from_float(np.array([-0.1], dtype=np.float32), fy)[0])
    alphas = [lr, 1 << (BITS[fy] - 2), int(_patterns(rng, 1, fy, 0)[0]), 0, 1 << (BITS[fy] - 1), 1, mask, (1 << (BITS[fy] - 1)) - 1,
              (1 << (BITS[fy] - 2)) | (1 << (BITS[fy] - 1))]
    for alpha in alphas:
        out = np.zeros(n, dtype=np.uint64)
        assert hc.hostcheck_axpy_f64(CODE[fx], CODE[fy], alpha, n, _p(x), _p(y), _p(out)) == 0
        assert np.array_equal(out, fast.axpy(alpha, x, y, fx, fy).astype(np.uint64)), alpha
    # near cancellation: y = -round(alpha x) nudged by a few patterns
    xs = _patterns(rng, n, fx, special=0.0)
    for alpha in (lr, int(_patterns(rng, 1, fy, 0)[0]) | 1):
        t = fast.axpy(alpha, xs, np.zeros(n, dtype=np.uint64), fx, fy).astype(np.int64)
        for delta in (0, 1, -1, 3, -7, 64):
            y2 = ((-t + delta) & mask).astype(np.uint64)
            out = np.zeros(n, dtype=np.uint64)
            hc.hostcheck_axpy_f64(CODE[fx], CODE[fy], alpha, n, _p(xs), _p(y2), _p(out))
            assert np.array_equal(out, fast.axpy(alpha, xs, y2, fx, fy).astype(np.uint64)), (alpha, delta)
    # far apart: huge y with tiny alpha x and the other way round, both signs: every y that sits exactly on a tie of the
    # coarser neighbourhood is decided by the sign of the tiny term
    big = np.array([p for p in range(1, 1 << (BITS[fy] - 1))] * 2, dtype=np.uint64)
    big[len(big) // 2:] = ((-big[len(big) // 2:].astype(np.int64)) & mask).astype(np.uint64)
    for tiny_x, alpha in ((1, 1), (1, mask), ((1 << BITS[fx]) - 1, 3), (3, lr)):
        xt = np.full(len(big), tiny_x, dtype=np.uint64)
        out = np.zeros(len(big), dtype=np.uint64)
        hc.hostcheck_axpy_f64(CODE[fx], CODE[fy], alpha, len(big), _p(xt), _p(big), _p(out))
        assert np.array_equal(out, fast.axpy(alpha, xt, big, fx, fy).astype(np.uint64)), (tiny_x, alpha)


def test_posit8_quire_rounding_of_the_kernel_epilogues(hc):
    """p8_round_quire (32-bit quire in units of 2^-12 -> posit<8,0>) against the oracle's rounding of the exact rational:
    every sum up to 2^14 units, every tie between neighbouring patterns and its two neighbours, powers of two and their
    neighbours, the extremes of the 32-bit range, random sums; both signs."""
    f = po.P8
    wide = po.PositFormat(9, 0, 0)
    vals = set(range(0, 1 << 14))
    for p in range(1, 256):   # values of posit<9,0>: the patterns of posit<8,0> and the ties between them
        v = po.decode(p, wide) * 4096
        if v.denominator == 1:
            vals.update((int(v) - 1, int(v), int(v) + 1))
    for e in range(31):
        vals.update(((1 << e) - 1, 1 << e, (1 << e) + 1, 3 << max(e - 1, 0)))
    rng = np.random.default_rng(8)
    vals.update(int(v) for v in rng.integers(0, 1 << 31, 20000))
    vals.update(int(v) >> int(s) for v, s in zip(rng.integers(0, 1 << 31, 20000), rng.integers(0, 31, 20000)))
    vals.update(((1 << 31) - 1, (1 << 31) - 2))
    qs = sorted(v for v in vals if 0 <= v < (1 << 31))
    q = np.array(qs + [-v for v in qs] + [-(1 << 31)], dtype=np.int64).astype(np.int32)
    out = np.zeros(len(q), dtype=np.uint32)
    assert hc.hostcheck_p8_round_quire(len(q), _p(q), _p(out)) == 0
    for qi, got in zip(q.tolist(), out.tolist()):
        assert got == po.round_to_posit(Fraction(qi, 4096), f), qi


def _pw_dot(hc, a, b):
    a = np.ascontiguousarray(a, dtype=np.uint32)
    b = np.ascontiguousarray(b, dtype=np.uint32)
    q = np.zeros(4, dtype=np.uint32)
    outl = np.zeros(2, dtype=np.int32)
    assert hc.hostcheck_pw_dot(len(a), _p(a), _p(b), _p(q), _p(outl)) == 0
    got = sum(int(w) << (32 * i) for i, w in enumerate(q))
    want = sum(po.decode(int(x), po.P16) * po.decode(int(y), po.P16) for x, y in zip(a, b)
               if int(x) != 0x8000 and int(y) != 0x8000) * (1 << 56)  # quire units: minpos^2 = 2^-56
    assert want.denominator == 1
    assert got == int(want) % (1 << 128), (got, int(want))
    return outl


def test_posit16_two_bucket_window_dot_product_at_its_bounds(hc):
    """The posit<16,1> GEMM keeps operands that are multiples of 2^-24 below 2^19 in two fp64 buckets for up to 1024
    products and takes every other operand through integer arithmetic.  Against exact rationals: the classification
    itself (every pattern: an operand counts as main exactly when it lies in that band), 1024 and more products of the
    largest and of the smallest main operands (the guard bits of both buckets filled, either sign), sums that cancel
    down to one unit, random patterns over the whole range (a few outliers each), and vectors of outliers only."""
    P = po.P16
    main = []
    for p in range(1, 1 << 16):
        if p == 0x8000:
            continue
        v = abs(po.decode(p, P)) * (1 << 28)        # scaled value, an integer
        assert v.denominator == 1
        iv = int(v)
        # the kernel's rule looks at the weight of the pattern's last fraction bit (set or not), which depends on the
        # regime only: 15 body bits = regime run + its terminating bit + one exponent bit + fraction
        mag = p if p < 0x8000 else 0x10000 - p
        body = format(mag, "015b")
        run = len(body) - len(body.lstrip(body[0]))
        nf = max(0, 15 - run - 1 - 1)
        last_bit_weight = (iv.bit_length() - 1) - nf
        is_main = last_bit_weight >= 4 and iv < (1 << 47)
        if is_main:
            assert iv % 16 == 0      # what the arithmetic needs: a multiple of 2^4 below 2^47
            main.append(p)
    assert len(main) > 0.95 * 65534  # the band covers all but the longest regimes
    # classification of every pattern through one-element dot products with 1.0 (itself a main operand)
    allp = np.arange(1, 1 << 16, dtype=np.uint32)
    allp = allp[allp != 0x8000]
    for chunk in np.array_split(allp, 64):
        outl = _pw_dot(hc, chunk, np.full(len(chunk), 0x4000, dtype=np.uint32))
        assert outl[0] == len(set(chunk.tolist()) - set(main)) and outl[1] == 0
    pos = [p for p in main if p < 0x8000]
    big, small = max(pos), min(pos)
    neg = lambda p: (0x10000 - p) & 0xFFFF
    rng = np.random.default_rng(16)
    for n in (1024, 2048, 5000):
        _pw_dot(hc, [big] * n, [big] * n)                       # hi bucket to its last guard bit
        _pw_dot(hc, [big] * n, [neg(big)] * n)
        _pw_dot(hc, [small] * n, [small] * n)
        # largest rests in the lo bucket: products just below a tie of the cut
        a = rng.choice(pos, n)
        b = rng.choice(pos, n)
        _pw_dot(hc, a, b)
        # cancellation: every product twice with opposite sign, then one small unit
        a2 = np.concatenate([a, a, [small]])
        b2 = np.concatenate([b, [neg(int(x)) for x in b], [small]])
        perm = rng.permutation(len(a2))
        _pw_dot(hc, a2[perm], b2[perm])
    for _ in range(20):
        n = int(rng.integers(1, 3000))
        a = rng.integers(0, 1 << 16, n)
        b = rng.integers(0, 1 << 16, n)
        _pw_dot(hc, a, b)
    outliers = [p for p in range(1, 1 << 16) if p != 0x8000 and p not in set(main)]
    a = rng.choice(outliers, 500)
    b = rng.choice(outliers, 500)
    outl = _pw_dot(hc, a, b)
    assert outl[0] == 500 and outl[1] == 500
    _pw_dot(hc, a, rng.choice(pos, 500))


def test_narrowing_step_table_posit16_to_posit8_all_patterns(hc):
    pats = np.arange(1 << 16, dtype=np.uint64)
    out = np.zeros_like(pats)
    assert hc.hostcheck_narrow_step(len(pats), _p(pats), _p(out)) == 0
    assert np.array_equal(out, fast.convert(pats, "p16", "p8").astype(np.uint64))


@pytest.mark.parametrize("fmt", ["p8", "p16", "p8_1", "p8_2", "p10_1", "p10_2", "p12_1", "p12_2"])
def test_round_binary64_to_posit_with_sticky_flags(hc, fmt):
    """round_f64_to_posit against the oracle's rounding of exact rationals: every tie point and every pattern value of
    the format as the binary64 s, exact, with 'a little more' and 'a little less' (the two flag settings), both signs;
    random binary64 values with all 52 fraction bits in use; values beyond maxpos and below minpos."""
    f = po.FORMATS[fmt]
    wide = po.PositFormat(f.n + 1, f.es, 0)
    eps = Fraction(1, 1 << 300)
    cases = []
    for p in range(1, 1 << f.n):  # values of the (n+1)-bit format: the patterns of fmt and the ties between them
        v = po.decode(p, wide)
        if v is po.NaR:
            continue
        cases.append(v)
    rng = np.random.default_rng(f.n * 7 + f.es)
    maxs = (f.n - 2) << f.es
    for _ in range(3000):
        m = 1 + Fraction(int(rng.integers(0, 1 << 52)), 1 << 52)
        e = int(rng.integers(-maxs - 4, maxs + 4))
        cases.append((m * Fraction(2) ** e) * (1 if rng.random() < 0.5 else -1))
    cases += [Fraction(2) ** (maxs + 40), -Fraction(2) ** (maxs + 40), Fraction(2) ** (-maxs - 40), -Fraction(2) ** (-maxs - 40)]
    for v in cases:
        s = float(v)
        assert Fraction(s) == v
        assert hc.hostcheck_round_f64(CODE[fmt], s, 0, 0) == po.round_to_posit(v, f), v
        up = v + eps if v > 0 else v - eps    # magnitude a little larger
        dn = v - eps if v > 0 else v + eps    # magnitude a little smaller
        assert hc.hostcheck_round_f64(CODE[fmt], s, 1, 0) == po.round_to_posit(up, f), ("more", v)
        assert hc.hostcheck_round_f64(CODE[fmt], s, 1, 1) == po.round_to_posit(dn, f), ("less", v)
    assert hc.hostcheck_round_f64(CODE[fmt], 0.0, 0, 0) == 0
    assert hc.hostcheck_round_f64(CODE[fmt], -0.0, 0, 0) == 0
    assert hc.hostcheck_round_f64(CODE[fmt], float("nan"), 0, 0) == f.nar


@pytest.mark.parametrize("fin,fout", [(f, f) for f in GENERAL] + [("p8_2", "p12_2"), ("p8_2", "p10_2"), ("p12_1", "p8"), ("p8_1", "p16"), ("p16", "p12_2")])
def test_quire_dot_general_formats(hc, fin, fout):
    test_quire_dot(hc, fin, fout)


def test_general_quire_wraps_like_the_oracle(hc):
    """posit<8,1> has a 64-bit quire that maxpos^2 = 2^48 minpos^2 leaves after 2^15 terms; the wrap is then
    modulo 2^64 on both sides.  (The 96-bit quires would need 2^31 terms: out of any test's reach.)"""
    fmt = "p8_1"
    mp = (1 << (BITS[fmt] - 1)) - 1
    a = np.full(70000, mp, dtype=np.uint32)
    seen = 0
    for K in (30000, 40000, 70000):
        want, ovf = fast.gemm(a[:K].reshape(1, K), a[:K].reshape(K, 1), fmt, fmt, threads=1)
        seen += ovf
        assert hc.hostcheck_dot(CODE[fmt], CODE[fmt], K, _p(a), _p(a), 0, 0) == int(want[0, 0]), K
    assert seen == 2  # the two longest runs did leave the quire range, so the wrap was exercised


@pytest.mark.parametrize("src", GENERAL + ["p8", "p16", "f32", "f64"])
@pytest.mark.parametrize("dst", GENERAL + ["p16", "f32"])
def test_runtime_format_conversions(hc, src, dst):
    rng = np.random.default_rng(len(src) * 7 + len(dst))
    if src == "f32":
        x = (rng.standard_normal(50000) * np.exp2(rng.uniform(-50, 50, 50000))).astype(np.float32)
        x[:5] = [0.0, -0.0, np.inf, np.nan, 1e-45]
        bits = x.view(np.uint32).astype(np.uint64)
        want = fast.round_from_float(x, dst).astype(np.uint64) if dst != "f32" else None
    elif src == "f64":
        x = rng.standard_normal(50000) * np.exp2(rng.uniform(-200, 200, 50000))
        bits = x.view(np.uint64).copy()
        want = fast.round_from_float(x, dst).astype(np.uint64) if dst != "f32" else None
    else:
        bits = np.arange(1 << BITS[src], dtype=np.uint64)
        want = None
    if dst == "f32" and src in ("f32", "f64"):
        pytest.skip("float to float is not a library operation")
    out = np.zeros_like(bits)
    assert hc.hostcheck_map_rt(CODE[src], CODE[dst], len(bits), _p(bits), _p(out)) == 0
    if src in ("f32", "f64"):
        assert np.array_equal(out, want)
    elif dst == "f32":
        ref = fast.to_float(bits, src, "f32")
        got = out.astype(np.uint32).view(np.float32)
        nan = np.isnan(ref)
        assert np.array_equal(np.isnan(got), nan) and np.array_equal(got[~nan], ref[~nan])
    else:
        assert np.array_equal(out, fast.convert(bits, src, dst).astype(np.uint64))


@pytest.mark.parametrize("fx,fy", [("p12_2", "p12_2"), ("p8_2", "p12_2"), ("p8_2", "p8_2"), ("p10_1", "p12_1"), ("p8_1", "p10_2"), ("p16", "p12_2")])
def test_runtime_format_axpy(hc, fx, fy):
    rng = np.random.default_rng(BITS[fx] * 11 + BITS[fy])
    n = 50000
    x = _patterns(rng, n, fx)
    y = _patterns(rng, n, fy)
    mask = (1 << BITS[fy]) - 1
    lr = int(fast.round_from_float(np.array([-0.1], dtype=np.float32), fy)[0])
    for alpha in (lr, 1 << (BITS[fy] - 2), 0, int(_patterns(rng, 1, fy, 0)[0])):
        out = np.zeros(n, dtype=np.uint64)
        assert hc.hostcheck_axpy_rt(CODE[fx], CODE[fy], alpha, n, _p(x), _p(y), _p(out)) == 0
        assert np.array_equal(out, fast.axpy(alpha, x, y, fx, fy).astype(np.uint64)), alpha
    t = fast.axpy(lr, x, np.zeros(n, dtype=np.uint64), fx, fy).astype(np.int64)
    for delta in (0, 1, -1, 5):
        y2 = ((-t + delta) & mask).astype(np.uint64)
        out = np.zeros(n, dtype=np.uint64)
        hc.hostcheck_axpy_rt(CODE[fx], CODE[fy], lr, n, _p(x), _p(y2), _p(out))
        assert np.array_equal(out, fast.axpy(lr, x, y2, fx, fy).astype(np.uint64))


@pytest.mark.parametrize("fin", ["p8", "p16", "p32"])
@pytest.mark.parametrize("fout", ["p8", "p16", "p32"])
def test_quire_dot(hc, fin, fout):
    rng = np.random.default_rng(BITS[fin] * 3 + BITS[fout])
    for trial in range(300):
        K = int(rng.integers(0, 40))
        special = [0.0, 0.05, 0.5][trial % 3]
        a = _patterns(rng, K, fin, special).astype(np.uint32)
        b = _patterns(rng, K, fin, special).astype(np.uint32)
        if trial % 4:
            nar = 1 << (BITS[fin] - 1)
            a[a == nar] = 1
            b[b == nar] = 1
        if trial % 7 == 3 and K >= 2:
            # exact cancellation of the two largest terms leaves only small ones
            a[1] = a[0]
            b[1] = (-b[0].astype(np.int64)) & ((1 << BITS[fin]) - 1)
        has_bias = trial % 2
        bias = int(_patterns(rng, 1, fin, 0.1)[0])
        got = hc.hostcheck_dot(CODE[fin], CODE[fout], K, _p(a), _p(b), has_bias, bias)
        want, _ = fast.gemm(a.reshape(1, K), b.reshape(K, 1), fin, fout,
                            bias=np.array([bias]) if has_bias else None, threads=1)
        assert got == int(want[0, 0]), (trial, K)


def test_quire_dot_wraps_like_the_oracle(hc):
    a = np.full(128, 0x7F, dtype=np.uint32)
    assert hc.hostcheck_dot(0, 0, 128, _p(a), _p(a), 0, 0) == 0x81
    assert hc.hostcheck_dot(0, 0, 127, _p(a), _p(a), 0, 0) == 0x7F
    a16 = np.full(40000, 0x7FFF, dtype=np.uint32)
    for K in (32767, 32768, 40000):
        want, _ = fast.gemm(a16[:K].reshape(1, K), a16[:K].reshape(K, 1), "p16", "p16", threads=1)
        assert hc.hostcheck_dot(1, 1, K, _p(a16), _p(a16), 0, 0) == int(want[0, 0])


BUCKETED = ["p16", "p8_1", "p8_2", "p10_1", "p10_2", "p12_1", "p12_2"]


def _bucket_config(hc, fmt):
    vals = [ctypes.c_int(0) for _ in range(3)]
    hc.hostcheck_bucket_config(CODE[fmt], *[ctypes.byref(v) for v in vals])
    return tuple(v.value for v in vals)


@pytest.mark.parametrize("fmt", BUCKETED)
def test_bucket_bounds_hold_for_the_format(hc, fmt):
    """The inequalities that make the fp64 buckets exact, re-derived here from the format alone: with
    R = 4 (n-2) 2^es the bit length of the largest product in quire units, B buckets cut at multiples
    of 54-G, 2^G products of magnitude 2^R must not push the top bucket past 2^53 of its units, and
    the rounding constant 1.5 * 2^(52+T1) must dominate a product."""
    f = po.FORMATS[fmt]
    R = 4 * (f.n - 2) * (1 << f.es)
    B, G, T1 = _bucket_config(hc, fmt)
    assert B >= 1 and G >= 5 and (1 << G) >= 16
    assert T1 == (B - 1) * (54 - G)
    assert R + G - T1 <= 53
    assert R <= 51 + T1 or B == 1
    assert 2 * (f.n - 2 - f.es) + 2 <= 53  # a product's significand is a double


@pytest.mark.parametrize("fmt", BUCKETED)
def test_bucket_split_of_a_product_is_error_free_and_not_folded_away(hc, fmt):
    """One product cut into its bucket parts: every part is a whole multiple of its bucket's unit 2^T_j, at most half
    a unit of the bucket above, and the parts add up to the product exactly.  A build that re-associated
    (r + C) - C into r (fast-math) would leave bits below 2^T_j in bucket j and fail the first property."""
    f = po.FORMATS[fmt]
    B, G, T1 = _bucket_config(hc, fmt)
    rng = np.random.default_rng(CODE[fmt])
    parts = (ctypes.c_double * 4)()
    cuts = (ctypes.c_int * 4)()
    pats = [int(p) for p in _patterns(rng, 300, fmt, 0.0)] + [1, (1 << (f.n - 1)) - 1, 3, (1 << (f.n - 1)) - 2, (1 << (f.n - 2)) + 1]
    straddles = 0
    for a in pats:
        for b in pats[::7]:
            if a in (0, f.nar) or b in (0, f.nar):
                continue
            nb = hc.hostcheck_bucket_split(CODE[fmt], a, b, parts, cuts)
            assert nb == max(B, 1)
            exact = po.decode(a, f) * po.decode(b, f) / f.quire_unit
            assert exact.denominator == 1
            total = 0
            for j in range(nb):
                v = Fraction(parts[j])
                assert v.denominator == 1 and int(v) % (1 << cuts[j]) == 0, (fmt, a, b, j)
                if j > 0:
                    assert abs(int(v)) <= 1 << (cuts[j - 1] - 1)
                total += int(v)
            assert total == exact.numerator
            straddles += sum(1 for j in range(nb) if parts[j] != 0.0) > 1
    if B > 1:
        assert straddles > 0, "some product must have bits on both sides of a cut"


def test_build_states_the_floating_point_model():
    from paper_2105_00053_amd import build
    assert "-fno-fast-math" in build.DEVICE_FLAGS and "-ffp-contract=off" in build.DEVICE_FLAGS
    assert not any(f in build.DEVICE_FLAGS for f in ("-ffast-math", "-Ofast", "-funsafe-math-optimizations", "-ffp-contract=fast"))


@pytest.mark.parametrize("fmt", BUCKETED)
def test_bucket_dot_random(hc, fmt):
    rng = np.random.default_rng(BITS[fmt] * 11 + CODE[fmt])
    fouts = [fmt, "p16", "p8"]
    for trial in range(240):
        K = int(rng.integers(0, 100)) if trial % 6 else int(rng.integers(100, 3000))
        special = [0.0, 0.05, 0.5][trial % 3]
        a = _patterns(rng, K, fmt, special).astype(np.uint32)
        b = _patterns(rng, K, fmt, special).astype(np.uint32)
        if trial % 4:
            nar = 1 << (BITS[fmt] - 1)
            a[a == nar] = 1
            b[b == nar] = 1
        if trial % 7 == 3 and K >= 2:
            a[1] = a[0]
            b[1] = (-b[0].astype(np.int64)) & ((1 << BITS[fmt]) - 1)
        has_bias = trial % 2
        bias = int(_patterns(rng, 1, fmt, 0.1)[0])
        fout = fouts[trial % 3]
        got = hc.hostcheck_dot_bucket(CODE[fmt], CODE[fout], K, _p(a), _p(b), has_bias, bias)
        want, _ = fast.gemm(a.reshape(1, K), b.reshape(K, 1), fmt, fout, bias=np.array([bias]) if has_bias else None, threads=1)
        assert got == int(want[0, 0]), (trial, K, fout)


@pytest.mark.parametrize("fmt", BUCKETED)
def test_bucket_dot_at_the_bounds(hc, fmt):
    """Inputs that fill the guard bits of every bucket: runs of maxpos^2 of one sign as long as several
    flush intervals, minpos^2 terms underneath them, products just below / at / above every cut
    position, and exact cancellation that leaves one unit of the quire."""
    n = BITS[fmt]
    full = (1 << n) - 1
    maxpos, minpos, one = (1 << (n - 1)) - 1, 1, 1 << (n - 2)
    neg = lambda p: (-p) & full
    B, G, T1 = _bucket_config(hc, fmt)
    flush = 1 << G
    cases = []
    for K in (flush - 1, flush, flush + 1, 2 * flush + 17, 5000):
        cases.append((np.full(K, maxpos), np.full(K, maxpos)))                      # + maxpos^2 each
        cases.append((np.full(K, maxpos), np.full(K, neg(maxpos))))                 # - maxpos^2 each
        a = np.full(K, maxpos); b = np.full(K, maxpos); a[1::2] = minpos; b[1::2] = neg(minpos)
        cases.append((a, b))                                                        # maxpos^2 - minpos^2 alternating
        a = np.full(K, maxpos); b = np.full(K, maxpos); b[K // 2:] = neg(maxpos); a[-1] = minpos; b[-1] = minpos
        cases.append((a, b))                                                        # cancels down to (K odd: +maxpos^2) + minpos^2
    rng = np.random.default_rng(CODE[fmt])
    # every pair of "power of two with full fraction" neighbours: products land on all bit positions, cut positions included
    pos = np.arange(1, 1 << (n - 1), dtype=np.int64)
    for rep in range(6):
        K = 4096
        a = rng.choice(pos, K); b = rng.choice(pos, K)
        sgn = rng.random(K) < 0.5
        a = np.where(sgn, a, (-a) & full)
        # sort by magnitude so that long runs of similar scale hit one bucket
        if rep % 2:
            order = np.argsort(a & (full >> 1)); a, b = a[order], b[order]
        cases.append((a, b))
    for a, b in cases:
        a = np.asarray(a).astype(np.uint32); b = np.asarray(b).astype(np.uint32)
        K = len(a)
        for fout in (fmt, "p32"):
            got = hc.hostcheck_dot_bucket(CODE[fmt], CODE[fout], K, _p(a), _p(b), 0, 0)
            want, _ = fast.gemm(a.reshape(1, K), b.reshape(K, 1), fmt, fout, threads=1)
            assert got == int(want[0, 0]), (K, fout)
            assert got == hc.hostcheck_dot(CODE[fmt], CODE[fout], K, _p(a), _p(b), 0, 0)


@pytest.mark.parametrize("fmt", BUCKETED)
def test_bucket_flush_converts_every_integer_exactly(hc, fmt):
    """Emptying a bucket holding m * 2^T adds exactly m << T (two's complement) to the limbs: ties of
    the high / low split (m = k 2^32 +- 2^31), the extremes +-2^53, small and random m."""
    B, G, _ = _bucket_config(hc, fmt)
    rng = np.random.default_rng(5)
    ms = [0, 1, -1, 2**31, -2**31, 2**31 - 1, -2**31 - 1, 2**32, -2**32, 3 * 2**31, -3 * 2**31, 5 * 2**31, -5 * 2**31,
          2**53, -2**53, 2**53 - 1, -(2**53 - 1), 2**52 + 2**31, -(2**52 + 2**31), (2**20 + 1) * 2**32 + 2**31, -((2**20 + 2) * 2**32 + 2**31)]
    ms += [int(v) for v in rng.integers(-2**53, 2**53, 300)]
    ms += [int(k) * 2**32 + int(r) for k, r in zip(rng.integers(-2**20, 2**20, 100), rng.choice([2**31, -2**31, 2**31 - 1, -2**31 + 1, 0], 100))]
    out = (ctypes.c_uint32 * 16)()
    for j in range(1, B + 1):
        T = (B - j) * (54 - G)
        for m in ms:
            L = hc.hostcheck_bucket_flush(CODE[fmt], j, float(m), out)
            assert L > 0 and float(m) == m
            got = sum(int(out[l]) << (32 * l) for l in range(L))
            assert got == (m << T) % (1 << (32 * L)), (fmt, j, m)


@pytest.mark.parametrize("fmt", BUCKETED)
def test_bucket_guard_bits_are_needed_and_enough(hc, fmt):
    """For every bucket: as many copies of the largest product that lands wholly in it as fit
    between two flushes (and 2x, 4x, 8x that many, which only stay exact because the buckets are
    emptied in between), then one product worth a single unit of that bucket, then the copies again
    with the other sign.  The exact sum is that one unit; any lost bit shows in the result."""
    import bucket_cases
    B, G, T1 = _bucket_config(hc, fmt)
    lay = bucket_cases.bucket_layout(fmt)
    assert (B, G, T1) == (lay[0], lay[1], lay[2][0])  # the test's own derivation agrees with the library's constants
    checked = 0
    for a, b, (sa, sb) in bucket_cases.guard_cases(fmt):
        K = len(a)
        got = hc.hostcheck_dot_bucket(CODE[fmt], CODE["p32"], K, _p(a), _p(b), 0, 0)
        want, _ = fast.gemm(np.array([[sa]]), np.array([[sb]]), fmt, "p32", threads=1)  # the one surviving product
        assert got == int(want[0, 0]), (fmt, K)
        checked += 1
    assert checked >= 3 * B


@pytest.mark.parametrize("fmt", ["p8_1", "p8_2"])
def test_cascade_dot_random_and_at_the_bounds(hc, fmt):
    """The 8-bit kernels keep the whole sum in doubles (carries between them every 16 and 32 products) and form the
    integer quire once: random vectors, the guard-filling vectors of the buckets, and long runs of maxpos^2 of one
    sign (the top level grows to K * maxpos^2) with minpos^2 terms and sign flips in between."""
    import bucket_cases
    n = BITS[fmt]
    full = (1 << n) - 1
    maxpos, minpos = (1 << (n - 1)) - 1, 1
    neg = lambda p: (-p) & full
    rng = np.random.default_rng(CODE[fmt] + 100)
    cases = []
    for trial in range(150):
        K = int(rng.integers(0, 100)) if trial % 5 else int(rng.integers(100, 4000))
        a = _patterns(rng, K, fmt, [0.0, 0.05, 0.5][trial % 3]).astype(np.uint32)
        b = _patterns(rng, K, fmt, [0.0, 0.05, 0.5][trial % 3]).astype(np.uint32)
        if trial % 4:
            a[a == 1 << (n - 1)] = 1
            b[b == 1 << (n - 1)] = 1
        cases.append((a, b))
    for a, b, _ in bucket_cases.guard_cases(fmt, mults=(1, 2, 4, 8), leads=(0, 5, 11, 16, 27)):
        cases.append((a, b))
    for K in (15, 16, 17, 31, 32, 33, 1000, 40000, 70000):
        cases.append((np.full(K, maxpos), np.full(K, maxpos)))
        cases.append((np.full(K, maxpos), np.full(K, neg(maxpos))))
        a = np.full(K, maxpos); b = np.full(K, maxpos); a[1::2] = minpos; b[1::2] = neg(minpos)
        cases.append((a, b))
        a = np.full(K, maxpos); b = np.full(K, maxpos); b[K // 2:] = neg(maxpos); a[-1] = minpos; b[-1] = minpos
        cases.append((a, b))
    for a, b in cases:
        a = np.asarray(a).astype(np.uint32); b = np.asarray(b).astype(np.uint32)
        K = len(a)
        for fout in (fmt, "p32"):
            got = hc.hostcheck_dot_cascade(CODE[fmt], CODE[fout], K, _p(a), _p(b), 1, 3)
            want, _ = fast.gemm(a.reshape(1, K), b.reshape(K, 1), fmt, fout, bias=np.array([3]), threads=1)
            assert got == int(want[0, 0]), (fmt, K, fout)


def test_bucket_dot_wraps_like_the_quire(hc):
    """posit<8,1>: 56 quire bits in a 64-bit word; 2^16 products of maxpos^2 = 2^48 quire units overflow it."""
    for K in (30000, 40000, 70000):
        a = np.full(K, 0x7F, dtype=np.uint32)
        want, _ = fast.gemm(a.reshape(1, K), a.reshape(K, 1), "p8_1", "p8_1", threads=1)
        assert hc.hostcheck_dot_bucket(CODE["p8_1"], CODE["p8_1"], K, _p(a), _p(a), 0, 0) == int(want[0, 0])


def test_conv_gather_descriptors_match_direct_indexing(hc):
    """The run-time affine descriptors of the posit<8,0> implicit-GEMM convolution (row / k
    decompositions by multiply-high division, separable offsets and bounds) against the direct
    NCHW / KCRS index formulas, for random geometries, all three passes, both operands, and
    the output index map."""
    import random
    rng = random.Random(5)
    i64 = ctypes.c_int64
    for trial in range(40):
        N, C, H, W, K = rng.randint(1, 3), rng.randint(1, 4), rng.randint(3, 9), rng.randint(3, 9), rng.randint(1, 4)
        R, S = rng.randint(1, min(4, H)), rng.randint(1, min(4, W))
        ph, pw, sh, sw = rng.randint(0, 2), rng.randint(0, 2), rng.randint(1, 2), rng.randint(1, 2)
        OH, OW = (H + 2 * ph - R) // sh + 1, (W + 2 * pw - S) // sw + 1
        geom = (i64 * 11)(N, C, H, W, K, R, S, ph, pw, sh, sw)

        def query(which, b, row, k, want_out=False):
            off, dims, oidx = i64(0), (i64 * 3)(), i64(0)
            ok = hc.hostcheck_conv_gather(which, geom, b, row, k, ctypes.byref(off), dims, ctypes.byref(oidx))
            return ok, off.value, tuple(dims), oidx.value

        def xoff(n, c, ih, iw):
            return ((n * C + c) * H + ih) * W + iw if 0 <= ih < H and 0 <= iw < W else None

        # forward: A rows (n,oh,ow) x k (c,r,s) on x ; B rows ko on w ; output y[n,ko,oh,ow]
        M, Nn, Kk = N * OH * OW, K, C * R * S
        for _ in range(200):
            m, k, ko = rng.randrange(M), rng.randrange(Kk), rng.randrange(Nn)
            n, rem = divmod(m, OH * OW); oh, ow = divmod(rem, OW)
            c, rs = divmod(k, R * S); r, s = divmod(rs, S)
            ok, off, dims, _ = query(0, 0, m, k)
            assert dims == (M, Nn, Kk)
            want = xoff(n, c, oh * sh + r - ph, ow * sw + s - pw)
            assert (off if ok else None) == want
            ok, off, _, _ = query(0, 1, ko, k)
            assert ok and off == ko * Kk + k
            _, _, _, oidx = query(0, 0, m, ko)
            assert oidx == ((n * K + ko) * OH + oh) * OW + ow
        # backward-weight (transposed): A rows (c,r,s) x k (n,oh,ow) on x ; B rows ko on dy ; output dw[ko,(c,r,s)]
        M, Nn, Kk = C * R * S, K, N * OH * OW
        for _ in range(200):
            m, k, ko = rng.randrange(M), rng.randrange(Kk), rng.randrange(Nn)
            c, rs = divmod(m, R * S); r, s = divmod(rs, S)
            n, rem = divmod(k, OH * OW); oh, ow = divmod(rem, OW)
            ok, off, dims, _ = query(2, 0, m, k)
            assert dims == (M, Nn, Kk)
            assert (off if ok else None) == xoff(n, c, oh * sh + r - ph, ow * sw + s - pw)
            ok, off, _, _ = query(2, 1, ko, k)
            assert ok and off == ((n * K + ko) * OH + oh) * OW + ow
            _, _, _, oidx = query(2, 0, m, ko)
            assert oidx == ko * M + m
        if sh == 1 and sw == 1:
            # backward-data: A rows (n,h,w) x k (ko,r,s) on dy ; B rows c on w ; output dx[n,c,h,w]
            M, Nn, Kk = N * H * W, C, K * R * S
            for _ in range(200):
                m, k, c = rng.randrange(M), rng.randrange(Kk), rng.randrange(Nn)
                n, rem = divmod(m, H * W); h, w = divmod(rem, W)
                ko, rs = divmod(k, R * S); r, s = divmod(rs, S)
                oh, ow = h + ph - r, w + pw - s
                ok, off, dims, _ = query(1, 0, m, k)
                assert dims == (M, Nn, Kk)
                want = ((n * K + ko) * OH + oh) * OW + ow if 0 <= oh < OH and 0 <= ow < OW else None
                assert (off if ok else None) == want
                ok, off, _, _ = query(1, 1, c, k)
                assert ok and off == ((ko * C + c) * R + r) * S + s
                _, _, _, oidx = query(1, 0, m, c)
                assert oidx == ((n * C + c) * H + h) * W + w


# ---------------- accumulation without the quire ----------------

@pytest.mark.parametrize("fmt", ["p8", "p8_1", "p8_2"])
def test_rounded_mul_add_exhaustive_8bit(hc, fmt):
    """All 65536 pairs of an 8-bit format, both operations, against the Python oracle's mul / add."""
    f = po.FORMATS[fmt]
    for op, ref in ((0, po.mul), (1, po.add)):
        for a in range(256):
            for b in range(256):
                assert hc.hostcheck_posit_op(CODE[fmt], op, a, b) == ref(a, b, f), (op, a, b)


@pytest.mark.parametrize("fmt", ["p16", "p32", "p10_1", "p10_2", "p12_1", "p12_2"])
def test_rounded_mul_add_sampled(hc, fmt):
    f = po.FORMATS[fmt]
    rng = np.random.default_rng(BITS[fmt])
    n = 3000
    a = _patterns(rng, n, fmt)
    b = _patterns(rng, n, fmt)
    # near-cancellation and neighbouring magnitudes, where the alignment window is exercised
    b[: n // 3] = ((-a[: n // 3].astype(np.int64) + rng.integers(-3, 4, n // 3)) & f.mask).astype(np.uint64)
    for x, y in zip(a.tolist(), b.tolist()):
        assert hc.hostcheck_posit_op(CODE[fmt], 0, x, y) == po.mul(x, y, f), (x, y)
        assert hc.hostcheck_posit_op(CODE[fmt], 1, x, y) == po.add(x, y, f), (x, y)


@pytest.mark.parametrize("fin,fout", [("p8", "p8"), ("p8", "p16"), ("p16", "p16"), ("p16", "p8"), ("p32", "p32"), ("p8_2", "p12_2"), ("p10_1", "p10_1"),
                                      ("p12_2", "p8_2"), ("p8_1", "p8_1"), ("p12_1", "p16"), ("p10_2", "p10_2")])
def test_noquire_dot_matches_oracle(hc, fin, fout):
    rng = np.random.default_rng(BITS[fin] + 5 * BITS[fout])
    for K in (1, 2, 17, 300):
        for trial in range(6):
            a = _patterns(rng, K, fin, special=0.03).astype(np.uint32)
            b = _patterns(rng, K, fin, special=0.03).astype(np.uint32)
            bias = int(_patterns(rng, 1, fin)[0])
            want, _ = fast.gemm(a.reshape(1, K), b.reshape(K, 1), fin, fout, bias=np.array([bias]), noquire=True, threads=1)
            got = hc.hostcheck_dot_noquire(CODE[fin], CODE[fout], K, _p(a), _p(b), 1, bias)
            assert got == int(want[0, 0]), (K, trial)
    # the worked example of the oracle's pin: 1 + forty times 1/64 sticks at 1 in posit<8,0>
    if fin == "p8" and fout == "p8":
        a = np.array([0x40] + [0x01] * 40, dtype=np.uint32)
        b = np.full(41, 0x40, dtype=np.uint32)
        assert hc.hostcheck_dot_noquire(0, 0, 41, _p(a), _p(b), 0, 0) == 0x40
        assert hc.hostcheck_dot(0, 0, 41, _p(a), _p(b), 0, 0) == 0x54


# ---------------- division and the scaling step of the losses ----------------

@pytest.mark.parametrize("fmt", ["p8", "p8_1", "p8_2"])
def test_division_exhaustive_8bit(hc, fmt):
    f = po.FORMATS[fmt]
    for a in range(256):
        for b in range(256):
            assert hc.hostcheck_posit_op(CODE[fmt], 2, a, b) == po.div(a, b, f), (a, b)


@pytest.mark.parametrize("fmt", ["p16", "p10_1", "p10_2", "p12_1", "p12_2"])
def test_division_sampled(hc, fmt):
    f = po.FORMATS[fmt]
    rng = np.random.default_rng(BITS[fmt] + 9)
    a = _patterns(rng, 4000, fmt)
    b = _patterns(rng, 4000, fmt)
    b[:500] = a[:500] + rng.integers(-2, 3, 500).astype(np.uint64) & f.mask  # quotients next to one
    for x, y in zip(a.tolist(), b.tolist()):
        assert hc.hostcheck_posit_op(CODE[fmt], 2, x, y) == po.div(x, y, f), (x, y)


@pytest.mark.parametrize("fin,fout", [("p16", "p16"), ("p12_2", "p12_2"), ("p10_2", "p8_2"), ("p8", "p16"), ("p16", "p8"), ("p32", "p16")])
def test_value_over_integer_rounds_once(hc, fin, fout):
    """posit * 2^k / d rounded once (gradient scaling 1/batch, 2/n): against the exact rational."""
    from fractions import Fraction
    fi, fo = po.FORMATS[fin], po.FORMATS[fout]
    rng = np.random.default_rng(BITS[fin] * 3 + BITS[fout])
    pats = _patterns(rng, 1500, fin).tolist()
    divs = [1, 2, 3, 7, 10, 64, 100, 128, 1000, 1280, 65537, 2 ** 31 - 1, 2 ** 32 - 1] + [int(v) for v in rng.integers(1, 2 ** 32, 20)]
    for i, p in enumerate(pats):
        d = divs[i % len(divs)]
        k = (i // len(divs)) % 3 - 1
        v = po.decode(p, fi)
        want = fo.nar if p == fi.nar else po.round_to_posit(v * Fraction(2) ** k / d, fo)
        assert hc.hostcheck_div_int(CODE[fin], CODE[fout], p, k, d) == want, (p, k, d)
    # quotients that land exactly on a rounding tie: 3 * minpos-spacing cases, e.g. (1 + 3 ulp) / 2 in posit<8,0>
    for p in range(1, 128):
        for d in (2, 4, 8, 3, 6):
            assert hc.hostcheck_div_int(0, 0, p, 0, d) == po.round_to_posit(po.decode(p, po.P8) / d, po.P8), (p, d)
