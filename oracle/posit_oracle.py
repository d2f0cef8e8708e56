"""Plain CPU oracle for quire-exact posit arithmetic (PositNN, arXiv 2105.00053).

TEST INFRASTRUCTURE ONLY.  This module is the slow, obviously-correct definition
that the GPU library is compared against.  It is imported by the tests, by the
smoke check and by the CPU-baseline leg of the benchmark, never by the product
path, and it shares no code with the HIP sources.

Everything here is exact integer / rational arithmetic (Python ``int`` and
``fractions.Fraction``): no floats take part in any result.

What each function follows
--------------------------
* ``decode``            : Sec. 2, Eq. 2 (sign, regime run-length k, exponent,
                          fraction; two's complement first when negative).
* ``PositFormat``       : Sec. 3.1, Table 1 (nbits/es pairs, dynamic range,
                          quire width).
* ``round_to_posit``    : the single rounding the paper delegates to the Posit
                          Standard (Sec. 3.2): nearest, ties to the even
                          encoding, never to zero or NaR.  Two independent
                          formulations, ``round_constructive`` and
                          ``round_by_search``, must agree.
* ``quire_*`` / ``gemm``: Sec. 2 (quire = exact sum of products) and Sec. 3.3
                          (quire accumulation in matrix products and
                          convolutions, one rounding at the end).
* ``mul`` / ``add`` / ``*_noquire``: Sec. 3.3 makes the quire an option and
                          Table 2 reports training "without quire": every
                          product and every running sum is then a posit, rounded
                          as it is produced, terms taken in order of the
                          reduction index.
* ``unary`` / ``unary_bwd`` / ``div`` / ``cross_entropy`` / ``mse``: Fig. 2 lists
                          Sigmoid and TanH activations and the Cross Entropy and
                          MSE losses, Sec. 3.3 / Fig. 3 give the loss its own posit
                          precision and Sec. 4 (Table 4) uses posit(10,2) and
                          posit(12,2) for it; no algorithm is printed.  Each
                          elementary function is taken as the correctly rounded
                          posit of the real function (``decimal``'s exp / ln at 120
                          digits bracket the value), the losses as the chain of such
                          operations written out in their docstrings.
* ``conv2d_*``          : Sec. 3.1 (layers inherit LibTorch semantics:
                          cross-correlation, NCHW / OIHW, zero padding) and its
                          two adjoints, which the framework writes by hand
                          because it has no automatic differentiation.
* ``from_float`` / ``to_float`` / ``convert``: Fig. 2 utilities (tensor
                          conversion, copies of a tensor in several formats).
* ``axpy``              : Fig. 2 optimizer (SGD), y <- round(y + alpha*x).
* ``relu`` / ``maxpool2d_*`` / ``avgpool2d_*``: Fig. 2 activation and pooling
                          layers, by value (max is taken on decoded values;
                          average pooling is a quire dot with 1/window).

Readings of points the paper leaves open (all listed in the design notes):
the quire is a Q-bit two's-complement integer whose unit is minpos^2 and which
wraps modulo 2^Q; NaR is absorbing (NaR * 0 = NaR); a bias is added inside the
quire; missing exponent bits read as zero; the forward convolution and its
weight gradient are matrix products over the unfolded (im2col) input, whose
padded entries are zero OPERANDS (a NaR weight makes its whole output channel
NaR, a NaR gradient entry its whole filter); the input gradient is the sum of
what the unfolded columns scatter back to each input position, so a filter tap
that reaches no output position from there is no term of that position's sum.

Parity pins: every function here is pinned by tests that do not reuse its own
formula (exhaustive round trips, encodings fixed by the definition, Table 1's
dot-product limits, brute-force rational sums, integer matmul and float64
library convolutions for posit<8,0>).  The choices "bias inside the quire",
"one quire over the whole batch reduction" and "single rounding in the SGD
update" cannot be pinned to the paper's own framework: parity unpinned for
those three readings (the definition here is the contract).  The same holds
for the order of the terms and the position of the bias (last) in the
``*_noquire`` functions: parity unpinned against the paper's framework; their
arithmetic (``mul``, ``add``) is pinned exhaustively for posit<8,0>.  The order
of operations inside ``cross_entropy`` and ``mse`` is likewise a reading (parity
unpinned against the paper's framework); their building blocks are pinned to
libm within one rounding, to closed forms and to symmetries.
"""

from fractions import Fraction
import decimal
import math


class _NaRType:
    """Not-a-Real: the pattern 10...0."""

    _inst = None

    def __new__(cls):
        if cls._inst is None:
            cls._inst = super().__new__(cls)
        return cls._inst

    def __repr__(self):
        return "NaR"


NaR = _NaRType()


class PositFormat:
    """posit<n, es> with its quire (Table 1)."""

    def __init__(self, n, es, quire_bits):
        self.n = n
        self.es = es
        self.quire_bits = quire_bits
        self.mask = (1 << n) - 1
        self.nar = 1 << (n - 1)
        self.useed = 2 ** (2 ** es)
        # maxpos = useed^(n-2); minpos = 1/maxpos  (Table 1, "dynamic range")
        self.max_scale = (n - 2) * (2 ** es)
        self.maxpos = Fraction(2) ** self.max_scale
        self.minpos = 1 / self.maxpos
        self.maxpos_pattern = self.nar - 1
        self.minpos_pattern = 1
        # unit of the quire's least significant bit
        self.quire_unit = self.minpos * self.minpos

    def __repr__(self):
        return "posit<%d,%d>" % (self.n, self.es)


P8 = PositFormat(8, 0, 32)
P16 = PositFormat(16, 1, 128)
P32 = PositFormat(32, 2, 512)


def general_quire_bits(n, es):
    """Quire width for (n, es) pairs Table 1 does not list (the paper's experiments use
    posit(8,1), (8,2), (10,x), (12,x), Sec. 4): room for the largest product over the
    smallest, 4(n-2)2^es bits, a sign bit and n-1 carry-guard bits, rounded up to a
    whole number of 32-bit limbs.  A reading: the paper gives no width for these."""
    return -(-(4 * (n - 2) * 2 ** es + 1 + (n - 1)) // 32) * 32


P8_1 = PositFormat(8, 1, general_quire_bits(8, 1))     # 64
P8_2 = PositFormat(8, 2, general_quire_bits(8, 2))     # 128
P10_1 = PositFormat(10, 1, general_quire_bits(10, 1))  # 96
P10_2 = PositFormat(10, 2, general_quire_bits(10, 2))  # 160
P12_1 = PositFormat(12, 1, general_quire_bits(12, 1))  # 96
P12_2 = PositFormat(12, 2, general_quire_bits(12, 2))  # 192
FORMATS = {"p8": P8, "p16": P16, "p32": P32, "p8_1": P8_1, "p8_2": P8_2, "p10_1": P10_1, "p10_2": P10_2,
           "p12_1": P12_1, "p12_2": P12_2}


# --------------------------------------------------------------------------
# decode (Eq. 2)
# --------------------------------------------------------------------------

def decode(p, fmt):
    """Pattern -> exact value as a Fraction, or NaR."""
    n, es = fmt.n, fmt.es
    p &= fmt.mask
    if p == 0:
        return Fraction(0)
    if p == fmt.nar:
        return NaR
    negative = (p >> (n - 1)) & 1
    if negative:
        p = (-p) & fmt.mask  # two's complement before reading the fields
    bits = [(p >> i) & 1 for i in range(n - 2, -1, -1)]  # below the sign, MSB first
    r = bits[0]
    m = 1
    while m < len(bits) and bits[m] == r:
        m += 1
    k = (m - 1) if r == 1 else -m
    rest = bits[m + 1:]  # drop the bit that ended the run, if there was room for it
    exp_bits = rest[:es]
    exp_bits = exp_bits + [0] * (es - len(exp_bits))  # truncated exponent bits are zeros
    e = 0
    for b in exp_bits:
        e = 2 * e + b
    frac_bits = rest[es:]
    f_num = 0
    for b in frac_bits:
        f_num = 2 * f_num + b
    f = Fraction(f_num, 2 ** len(frac_bits))
    value = Fraction(2) ** ((2 ** es) * k + e) * (1 + f)
    return -value if negative else value


_tables = {}


def decode_table(fmt):
    """All 2^n decoded values (n <= 16 only); built by calling ``decode``."""
    key = (fmt.n, fmt.es)
    if key not in _tables:
        if fmt.n > 16:
            raise ValueError("table only for n <= 16")
        _tables[key] = [decode(p, fmt) for p in range(1 << fmt.n)]
    return _tables[key]


def _value(p, fmt):
    p = int(p) & fmt.mask
    if fmt.n <= 16:
        return decode_table(fmt)[p]
    return decode(p, fmt)


def to_minpos_units(p, fmt):
    """Integer v with value = v * minpos (every posit is such a multiple), or NaR."""
    v = _value(p, fmt)
    if v is NaR:
        return NaR
    u = v / fmt.minpos
    assert u.denominator == 1
    return u.numerator


# --------------------------------------------------------------------------
# rounding: exact rational -> posit<n,es>
# --------------------------------------------------------------------------

def _floor_log2(x):
    """floor(log2(x)) for a positive Fraction."""
    s = x.numerator.bit_length() - x.denominator.bit_length()
    if Fraction(2) ** s > x:
        s -= 1
    assert Fraction(2) ** s <= x < Fraction(2) ** (s + 1)
    return s


def round_constructive(x, fmt):
    """Write out regime | exponent | fraction, keep n-1 bits, nearest-even."""
    x = Fraction(x)
    n, es = fmt.n, fmt.es
    if x == 0:
        return 0
    negative = x < 0
    a = -x if negative else x
    if a >= fmt.maxpos:
        body = fmt.maxpos_pattern
    elif a <= fmt.minpos:
        body = fmt.minpos_pattern
    else:
        scale = _floor_log2(a)
        f = a / Fraction(2) ** scale - 1  # in [0, 1)
        k = scale >> es  # floor division
        e = scale - (k << es)
        if k >= 0:
            regime = ((1 << (k + 1)) - 1) << 1  # k+1 ones, then a zero
            rlen = k + 2
        else:
            regime = 1  # -k zeros, then a one
            rlen = -k + 1
        prefix = (regime << es) | e
        plen = rlen + es
        keep = n - 1
        # the unbounded string, read as a binary number with `keep` integer bits
        exact = (prefix + f) * Fraction(2) ** (keep - plen)
        body = exact.numerator // exact.denominator
        rem = exact - body
        if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (body & 1)):
            body += 1
        assert 1 <= body <= fmt.maxpos_pattern
    return (-body) & fmt.mask if negative else body


def round_by_search(x, fmt):
    """Find the two neighbouring patterns; their midpoint is the (n+1)-bit posit between."""
    x = Fraction(x)
    if x == 0:
        return 0
    negative = x < 0
    a = -x if negative else x
    if a >= fmt.maxpos:
        body = fmt.maxpos_pattern
    elif a <= fmt.minpos:
        body = fmt.minpos_pattern
    else:
        lo, hi = 1, fmt.maxpos_pattern  # decode(lo) < a < decode(hi), patterns are monotone
        while hi - lo > 1:
            mid = (lo + hi) // 2
            vm = decode(mid, fmt)
            if vm == a:
                lo = hi = mid
                break
            if vm < a:
                lo = mid
            else:
                hi = mid
        if lo == hi:
            body = lo
        else:
            wider = PositFormat(fmt.n + 1, fmt.es, 0)
            midpoint = decode(2 * lo + 1, wider)
            if a < midpoint:
                body = lo
            elif a > midpoint:
                body = hi
            else:
                body = lo if (lo & 1) == 0 else hi
    return (-body) & fmt.mask if negative else body


def round_to_posit(x, fmt):
    """The rounding every result goes through exactly once."""
    if x is NaR:
        return fmt.nar
    return round_constructive(x, fmt)


# --------------------------------------------------------------------------
# quire: exact sum of products, Q-bit two's complement in units of minpos^2
# --------------------------------------------------------------------------

def quire_wrap(total, fmt):
    """Reduce an exact integer (units of minpos^2) to the Q-bit signed range."""
    q = fmt.quire_bits
    t = total & ((1 << q) - 1)
    if t >> (q - 1):
        t -= 1 << q
    return t


def quire_fits(total, fmt):
    q = fmt.quire_bits
    return -(1 << (q - 1)) <= total <= (1 << (q - 1)) - 1


def quire_round(total, fin, fout):
    """Wrapped quire integer -> posit in fout."""
    return round_to_posit(Fraction(quire_wrap(total, fin)) * fin.quire_unit, fout)


def quire_dot(a, b, fin, bias=None):
    """Exact sum_k a[k]*b[k] (+ bias*1) as an integer in units of minpos^2, or NaR."""
    total = 0
    nar = False
    for pa, pb in zip(a, b):
        ua = to_minpos_units(pa, fin)
        ub = to_minpos_units(pb, fin)
        if ua is NaR or ub is NaR:
            nar = True
            continue
        total += ua * ub
    if bias is not None:
        ubias = to_minpos_units(bias, fin)
        if ubias is NaR:
            nar = True
        else:
            total += ubias * (1 << fin.max_scale)  # bias times the value one
    return NaR if nar else total


def dot(a, b, fin, fout, bias=None):
    t = quire_dot(a, b, fin, bias)
    if t is NaR:
        return fout.nar
    return quire_round(t, fin, fout)


def gemm(A, B, fin, fout, trans_a=False, trans_b=False, bias=None):
    """C[i][j] = round_fout( sum_k op(A)[i][k] * op(B)[k][j] (+ bias[j]) ).

    A, B are lists of rows of patterns (as stored, before op()).  Returns rows.
    """
    if trans_a:
        A = [list(r) for r in zip(*A)] if A and A[0] else []
    Bt = B if trans_b else ([list(r) for r in zip(*B)] if B and len(B[0]) else [])
    # Bt[j] is column j of op(B)
    C = []
    for i in range(len(A)):
        row = []
        for j in range(len(Bt)):
            row.append(dot(A[i], Bt[j], fin, fout, None if bias is None else bias[j]))
        C.append(row)
    return C


# --------------------------------------------------------------------------
# convolution (cross-correlation, NCHW / OIHW, zero padding, stride) and adjoints
# --------------------------------------------------------------------------

class ConvShape:
    def __init__(self, N, C, H, W, K, R, S, pad_h=0, pad_w=0, stride_h=1, stride_w=1):
        self.N, self.C, self.H, self.W = N, C, H, W
        self.K, self.R, self.S = K, R, S
        self.pad_h, self.pad_w = pad_h, pad_w
        self.stride_h, self.stride_w = stride_h, stride_w
        self.OH = (H + 2 * pad_h - R) // stride_h + 1
        self.OW = (W + 2 * pad_w - S) // stride_w + 1


def _units_list(flat, fmt):
    return [to_minpos_units(p, fmt) for p in flat]


def conv2d_fwd_quire(x, w, sh, fin, bias=None):
    """Exact y[n][k][oh][ow] = sum_{c,r,s} x[n][c][oh*sh+r-ph][ow*sw+s-pw] * w[k][c][r][s] (+bias[k]).

    x, w, bias are flat sequences of patterns (NCHW, OIHW).  Returns a flat list
    of integers in units of minpos^2 (or NaR).
    """
    xu = _units_list(x, fin)
    wu = _units_list(w, fin)
    bu = None if bias is None else _units_list(bias, fin)
    one = 1 << fin.max_scale
    out = []
    for n in range(sh.N):
        for k in range(sh.K):
            for oh in range(sh.OH):
                for ow in range(sh.OW):
                    total = 0
                    nar = False
                    for c in range(sh.C):
                        for r in range(sh.R):
                            ih = oh * sh.stride_h + r - sh.pad_h
                            for s in range(sh.S):
                                iw = ow * sh.stride_w + s - sh.pad_w
                                inside = 0 <= ih < sh.H and 0 <= iw < sh.W
                                # a padded position holds the value zero and is an operand like any other
                                a = xu[((n * sh.C + c) * sh.H + ih) * sh.W + iw] if inside else 0
                                b = wu[((k * sh.C + c) * sh.R + r) * sh.S + s]
                                if a is NaR or b is NaR:
                                    nar = True
                                else:
                                    total += a * b
                    if bu is not None:
                        if bu[k] is NaR:
                            nar = True
                        else:
                            total += bu[k] * one
                    out.append(NaR if nar else total)
    return out


def conv2d_bwd_data_quire(dy, w, sh, fin):
    """Exact dx[n][c][h][w] = sum of dy[n][k][oh][ow]*w[k][c][r][s] over the (k,r,s,oh,ow) with
    oh*sh+r-ph == h and ow*sw+s-pw == w: the adjoint of the forward pass with respect to x.  It is
    what LibTorch's data flow (Sec. 3.1) accumulates when it multiplies W^T by dY and scatters every
    column entry back to the input position it was unfolded from: a (k,r,s) that reaches no output
    position from (h,w) sends nothing there, so it is no term of that sum (and a NaR weight at
    such a tap does not touch that position)."""
    dyu = _units_list(dy, fin)
    wu = _units_list(w, fin)
    out = []
    for n in range(sh.N):
        for c in range(sh.C):
            for h in range(sh.H):
                for ww in range(sh.W):
                    total = 0
                    nar = False
                    for k in range(sh.K):
                        for r in range(sh.R):
                            t = h + sh.pad_h - r
                            oh = t // sh.stride_h
                            row_ok = t >= 0 and t % sh.stride_h == 0 and oh < sh.OH
                            for s in range(sh.S):
                                u = ww + sh.pad_w - s
                                ow = u // sh.stride_w
                                if not (row_ok and u >= 0 and u % sh.stride_w == 0 and ow < sh.OW):
                                    continue  # no output position reads x[n][c][h][w] through this tap
                                a = dyu[((n * sh.K + k) * sh.OH + oh) * sh.OW + ow]
                                b = wu[((k * sh.C + c) * sh.R + r) * sh.S + s]
                                if a is NaR or b is NaR:
                                    nar = True
                                else:
                                    total += a * b
                    out.append(NaR if nar else total)
    return out


def conv2d_bwd_weight_quire(dy, x, sh, fin):
    """Exact dw[k][c][r][s] = sum_{n,oh,ow} dy[n][k][oh][ow] * x[n][c][oh*sh+r-ph][ow*sw+s-pw]."""
    dyu = _units_list(dy, fin)
    xu = _units_list(x, fin)
    out = []
    for k in range(sh.K):
        for c in range(sh.C):
            for r in range(sh.R):
                for s in range(sh.S):
                    total = 0
                    nar = False
                    for n in range(sh.N):
                        for oh in range(sh.OH):
                            ih = oh * sh.stride_h + r - sh.pad_h
                            for ow in range(sh.OW):
                                iw = ow * sh.stride_w + s - sh.pad_w
                                inside = 0 <= ih < sh.H and 0 <= iw < sh.W
                                a = dyu[((n * sh.K + k) * sh.OH + oh) * sh.OW + ow]
                                b = xu[((n * sh.C + c) * sh.H + ih) * sh.W + iw] if inside else 0
                                if a is NaR or b is NaR:
                                    nar = True
                                else:
                                    total += a * b
                    out.append(NaR if nar else total)
    return out


def conv2d_bias_grad_quire(dy, sh, fin):
    """Exact dbias[k] = sum_{n,oh,ow} dy[n][k][oh][ow] * 1."""
    dyu = _units_list(dy, fin)
    one = 1 << fin.max_scale
    out = []
    for k in range(sh.K):
        total = 0
        nar = False
        for n in range(sh.N):
            for i in range(sh.OH * sh.OW):
                a = dyu[(n * sh.K + k) * sh.OH * sh.OW + i]
                if a is NaR:
                    nar = True
                else:
                    total += a * one
        out.append(NaR if nar else total)
    return out


def _round_quires(qs, fin, fout):
    return [fout.nar if t is NaR else quire_round(t, fin, fout) for t in qs]


def conv2d_fwd(x, w, sh, fin, fout, bias=None):
    return _round_quires(conv2d_fwd_quire(x, w, sh, fin, bias), fin, fout)


def conv2d_bwd_data(dy, w, sh, fin, fout):
    return _round_quires(conv2d_bwd_data_quire(dy, w, sh, fin), fin, fout)


def conv2d_bwd_weight(dy, x, sh, fin, fout):
    return _round_quires(conv2d_bwd_weight_quire(dy, x, sh, fin), fin, fout)


def conv2d_bias_grad(dy, sh, fin, fout):
    return _round_quires(conv2d_bias_grad_quire(dy, sh, fin), fin, fout)


# --------------------------------------------------------------------------
# accumulation without the quire (Sec. 3.3: the quire is an option; Table 2)
# --------------------------------------------------------------------------

def mul(pa, pb, fmt):
    """posit x posit -> posit: the exact product rounded once."""
    va, vb = _value(pa, fmt), _value(pb, fmt)
    if va is NaR or vb is NaR:
        return fmt.nar
    return round_to_posit(va * vb, fmt)


def add(pa, pb, fmt):
    """posit + posit -> posit: the exact sum rounded once."""
    va, vb = _value(pa, fmt), _value(pb, fmt)
    if va is NaR or vb is NaR:
        return fmt.nar
    return round_to_posit(va + vb, fmt)


def dot_noquire(a, b, fin, fout, bias=None):
    """s_0 = 0, s_k = add(s_{k-1}, mul(a_k, b_k)) for k in order, then the bias, all in fin;
    the final posit is converted to fout."""
    acc = 0
    for pa, pb in zip(a, b):
        acc = add(acc, mul(pa, pb, fin), fin)
    if bias is not None:
        acc = add(acc, bias, fin)
    return convert(acc, fin, fout) if acc != fin.nar else fout.nar


def gemm_noquire(A, B, fin, fout, trans_a=False, trans_b=False, bias=None):
    """As ``gemm`` with every dot product taken by ``dot_noquire`` (k ascending)."""
    if trans_a:
        A = [list(r) for r in zip(*A)] if A and A[0] else []
    Bt = B if trans_b else ([list(r) for r in zip(*B)] if B and len(B[0]) else [])
    return [[dot_noquire(A[i], Bt[j], fin, fout, None if bias is None else bias[j]) for j in range(len(Bt))]
            for i in range(len(A))]


def conv2d_fwd_terms(x, w, sh):
    """For every output (n,k,oh,ow) in NCHW order: the two operand sequences of its dot product, terms
    ordered by (c,r,s) as in the unfolded matrix; a padded position is the pattern 0."""
    out = []
    for n in range(sh.N):
        for k in range(sh.K):
            for oh in range(sh.OH):
                for ow in range(sh.OW):
                    a, b = [], []
                    for c in range(sh.C):
                        for r in range(sh.R):
                            ih = oh * sh.stride_h + r - sh.pad_h
                            for s in range(sh.S):
                                iw = ow * sh.stride_w + s - sh.pad_w
                                inside = 0 <= ih < sh.H and 0 <= iw < sh.W
                                a.append(x[((n * sh.C + c) * sh.H + ih) * sh.W + iw] if inside else 0)
                                b.append(w[((k * sh.C + c) * sh.R + r) * sh.S + s])
                    out.append((a, b))
    return out


def conv2d_bwd_data_terms(dy, w, sh):
    """For every dx[n,c,h,w]: operand sequences ordered by (k,r,s); only the taps that reach an output
    position from (h,w) are terms."""
    out = []
    for n in range(sh.N):
        for c in range(sh.C):
            for h in range(sh.H):
                for ww in range(sh.W):
                    a, b = [], []
                    for k in range(sh.K):
                        for r in range(sh.R):
                            t = h + sh.pad_h - r
                            for s in range(sh.S):
                                u = ww + sh.pad_w - s
                                ok = (t >= 0 and t % sh.stride_h == 0 and t // sh.stride_h < sh.OH and
                                      u >= 0 and u % sh.stride_w == 0 and u // sh.stride_w < sh.OW)
                                if not ok:
                                    continue
                                a.append(dy[((n * sh.K + k) * sh.OH + t // sh.stride_h) * sh.OW + u // sh.stride_w])
                                b.append(w[((k * sh.C + c) * sh.R + r) * sh.S + s])
                    out.append((a, b))
    return out


def conv2d_bwd_weight_terms(dy, x, sh):
    """For every dw[k,c,r,s]: operand sequences ordered by (n,oh,ow)."""
    out = []
    for k in range(sh.K):
        for c in range(sh.C):
            for r in range(sh.R):
                for s in range(sh.S):
                    a, b = [], []
                    for n in range(sh.N):
                        for oh in range(sh.OH):
                            ih = oh * sh.stride_h + r - sh.pad_h
                            for ow in range(sh.OW):
                                iw = ow * sh.stride_w + s - sh.pad_w
                                inside = 0 <= ih < sh.H and 0 <= iw < sh.W
                                a.append(dy[((n * sh.K + k) * sh.OH + oh) * sh.OW + ow])
                                b.append(x[((n * sh.C + c) * sh.H + ih) * sh.W + iw] if inside else 0)
                    out.append((a, b))
    return out


def conv2d_bias_grad_terms(dy, sh, fin):
    """For every dbias[k]: dy[n,k,:,:] ordered by (n,oh,ow), each against the value one."""
    one = 1 << (fin.n - 2)
    out = []
    for k in range(sh.K):
        a = [dy[(n * sh.K + k) * sh.OH * sh.OW + i] for n in range(sh.N) for i in range(sh.OH * sh.OW)]
        out.append((a, [one] * len(a)))
    return out


def conv2d_fwd_noquire(x, w, sh, fin, fout, bias=None):
    terms = conv2d_fwd_terms(x, w, sh)
    per_k = sh.OH * sh.OW
    return [dot_noquire(a, b, fin, fout, None if bias is None else bias[(i // per_k) % sh.K]) for i, (a, b) in enumerate(terms)]


def conv2d_bwd_data_noquire(dy, w, sh, fin, fout):
    return [dot_noquire(a, b, fin, fout) for a, b in conv2d_bwd_data_terms(dy, w, sh)]


def conv2d_bwd_weight_noquire(dy, x, sh, fin, fout):
    return [dot_noquire(a, b, fin, fout) for a, b in conv2d_bwd_weight_terms(dy, x, sh)]


def conv2d_bias_grad_noquire(dy, sh, fin, fout):
    return [dot_noquire(a, b, fin, fout) for a, b in conv2d_bias_grad_terms(dy, sh, fin)]


# --------------------------------------------------------------------------
# elementary functions, division, losses (Fig. 2: Sigmoid, TanH, Cross Entropy, MSE)
# --------------------------------------------------------------------------

_DEC = decimal.Context(prec=120, Emax=decimal.MAX_EMAX, Emin=decimal.MIN_EMIN, rounding=decimal.ROUND_HALF_EVEN)
_DEC_SLACK = Fraction(1, 10 ** 100)  # far above the error of a few 120-digit operations


def _to_decimal(x):
    """Exact: posit values are dyadic rationals with short decimal expansions."""
    x = Fraction(x)
    d = _DEC.divide(decimal.Decimal(x.numerator), decimal.Decimal(x.denominator))
    assert Fraction(d) == x
    return d


def _round_decimal(d, fmt):
    """Round the real number that the 120-digit decimal d approximates (relative error far below
    10^-100): both ends of the bracket must give the same pattern, which is then the correctly
    rounded one.  Magnitudes beyond 10^+-60 lie outside every format here and clamp."""
    if d == 0:
        return 0
    sign = -1 if d < 0 else 1
    if d.adjusted() > 60:
        return round_to_posit(sign * fmt.maxpos * 2, fmt)
    if d.adjusted() < -60:
        return round_to_posit(sign * fmt.minpos / 2, fmt)
    v = Fraction(d)
    lo, hi = round_to_posit(v * (1 - _DEC_SLACK), fmt), round_to_posit(v * (1 + _DEC_SLACK), fmt)
    if lo != hi:
        raise ArithmeticError("value too close to a rounding boundary for 120 digits")
    return lo


UNARY = ("sigmoid", "tanh", "exp", "log")


def unary(fn, p, fmt):
    """Correctly rounded posit of sigmoid(x) = 1/(1+e^-x), tanh(x), e^x or ln(x) at the value x of pattern p.
    NaR gives NaR; ln of zero or of a negative value gives NaR; exact cases: tanh(0) = 0, ln(1) = 0."""
    x = _value(p, fmt)
    if x is NaR:
        return fmt.nar
    one = decimal.Decimal(1)
    if fn == "exp":
        return _round_decimal(_DEC.exp(_to_decimal(x)), fmt)
    if fn == "log":
        if x <= 0:
            return fmt.nar
        return 0 if x == 1 else _round_decimal(_DEC.ln(_to_decimal(x)), fmt)
    if fn == "sigmoid":
        return _round_decimal(_DEC.divide(one, _DEC.add(one, _DEC.exp(_to_decimal(-x)))), fmt)
    if fn == "tanh":
        if x == 0:
            return 0
        e2 = _DEC.exp(_to_decimal(2 * x))  # tanh = (e^2x - 1) / (e^2x + 1)
        if e2.adjusted() > 200:
            return _round_decimal(one, fmt)
        if e2.adjusted() < -200:
            return _round_decimal(-one, fmt)
        return _round_decimal(_DEC.divide(_DEC.subtract(e2, one), _DEC.add(e2, one)), fmt)
    raise ValueError(fn)


def unary_bwd(fn, y, dy, fmt_y, fmt_d):
    """Gradient through an activation from its forward OUTPUT y, in posit operations of the gradient's
    format fmt_d, each rounded: with y' = convert(y), sigmoid: mul(dy, mul(y', add(1, -y'))); tanh:
    mul(dy, add(1, -mul(y', y')))."""
    yc = convert(y, fmt_y, fmt_d)
    one = 1 << (fmt_d.n - 2)
    if fn == "sigmoid":
        return mul(dy, mul(yc, add(one, neg(yc, fmt_d), fmt_d), fmt_d), fmt_d)
    if fn == "tanh":
        return mul(dy, add(one, neg(mul(yc, yc, fmt_d), fmt_d), fmt_d), fmt_d)
    raise ValueError(fn)


def div(pa, pb, fmt):
    """posit / posit -> posit: the exact quotient rounded once; a zero divisor gives NaR."""
    va, vb = _value(pa, fmt), _value(pb, fmt)
    if va is NaR or vb is NaR or vb == 0:
        return fmt.nar
    return round_to_posit(va / vb, fmt)


def neg(p, fmt):
    return (-int(p)) & fmt.mask


def _exact_sum_rounded(values, fmt, divisor=1):
    """round( wrap_Q( sum of exact values ) / divisor ): the values are whole multiples of minpos^2 of fmt,
    held in fmt's quire (which wraps modulo 2^Q like every quire here), then divided exactly."""
    unit = fmt.minpos * fmt.minpos
    total = sum(values, Fraction(0)) / unit
    assert total.denominator == 1
    return round_to_posit(Fraction(quire_wrap(total.numerator, fmt)) * unit / divisor, fmt)


def cross_entropy(logits, labels, f_logits, f_loss, f_grad):
    """Softmax cross entropy with mean reduction over the batch, computed in the loss format f_loss.

    logits: rows of patterns in f_logits; labels: one class index per row.  Per row, with every operation
    rounded to f_loss:  z_j = convert(logit_j);  m = max_j z_j;  t_j = add(z_j, -m);  e_j = exp(t_j);
    S = round(sum_j e_j) (exact sum, one rounding);  p_j = div(e_j, S);  g_j = add(p_j, -[j == label]);
    row loss = add(log(S), -t_label).  Outputs: dlogits[b][j] = round_f_grad(g_j / B) (exact division by the
    batch size B, one rounding) and loss = round_f_loss((sum_b row loss_b) / B) (exact sum and division).
    A NaR logit or a label outside 0..C-1 makes its row's gradient and the loss NaR."""
    B = len(logits)
    grads, row_losses, any_nar = [], [], False
    for row, label in zip(logits, labels):
        C = len(row)
        z = [convert(p, f_logits, f_loss) for p in row]
        if any(p == f_loss.nar for p in z) or not (0 <= label < C):
            grads.append([f_grad.nar] * C)
            any_nar = True
            continue
        m = max(z, key=lambda p: _value(p, f_loss))
        t = [add(p, neg(m, f_loss), f_loss) for p in z]
        e = [unary("exp", p, f_loss) for p in t]
        S = _exact_sum_rounded([_value(p, f_loss) for p in e], f_loss)
        prob = [div(p, S, f_loss) for p in e]
        one = 1 << (f_loss.n - 2)
        g = [add(prob[j], neg(one, f_loss) if j == label else 0, f_loss) for j in range(C)]
        grads.append([round_to_posit(_value(p, f_loss) / B, f_grad) for p in g])
        row_losses.append(add(unary("log", S, f_loss), neg(t[label], f_loss), f_loss))
    if any_nar:
        return f_loss.nar, grads
    return _exact_sum_rounded([_value(p, f_loss) for p in row_losses], f_loss, divisor=B), grads


def mse(pred, target, f_pred, f_loss, f_grad):
    """Mean squared error over n elements in the loss format: d_i = add(convert(pred_i), -convert(target_i))
    rounded to f_loss; loss = round_f_loss((sum_i d_i^2) / n), the squares summed exactly in f_loss's quire;
    dpred_i = round_f_grad(2 d_i / n), exact inside.  NaR anywhere makes the loss NaR and that element's gradient NaR."""
    n = len(pred)
    d = [add(convert(p, f_pred, f_loss), neg(convert(t, f_pred, f_loss), f_loss), f_loss) for p, t in zip(pred, target)]
    grads = [f_grad.nar if x == f_loss.nar else round_to_posit(2 * _value(x, f_loss) / n, f_grad) for x in d]
    if any(x == f_loss.nar for x in d):
        return f_loss.nar, grads
    return _exact_sum_rounded([_value(x, f_loss) ** 2 for x in d], f_loss, divisor=n), grads


# --------------------------------------------------------------------------
# conversions
# --------------------------------------------------------------------------

def from_float(x, fmt):
    """IEEE value (a Python float holding the f32/f64 exactly) -> posit; NaN, +-Inf -> NaR."""
    x = float(x)
    if math.isnan(x) or math.isinf(x):
        return fmt.nar
    return round_to_posit(Fraction(x), fmt)  # Fraction(float) is exact; -0.0 -> 0


def ieee_round(x, precision, emin):
    """Exact rational -> nearest-even binary float with `precision` significand bits
    and minimum normal exponent `emin` (subnormals below).  Returns a Fraction."""
    x = Fraction(x)
    if x == 0:
        return Fraction(0)
    negative = x < 0
    a = -x if negative else x
    e = max(_floor_log2(a), emin)
    ulp = Fraction(2) ** (e - (precision - 1))
    q = a / ulp
    body = q.numerator // q.denominator
    rem = q - body
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (body & 1)):
        body += 1
    r = body * ulp
    return -r if negative else r


def to_float(p, fmt, kind="f64"):
    """posit -> IEEE binary32 / binary64 value (as a Python float); NaR -> NaN.

    All three standard formats fit both IEEE types without overflow, so only
    the significand rounding of ieee_round matters."""
    v = _value(p, fmt)
    if v is NaR:
        return float("nan")
    if kind == "f32":
        r = ieee_round(v, 24, -126)
    elif kind == "f64":
        r = ieee_round(v, 53, -1022)
    else:
        raise ValueError(kind)
    out = r.numerator / r.denominator  # exact: r is representable
    assert Fraction(out) == r
    return out


def convert(p, fsrc, fdst):
    """posit<a> -> posit<b>: round the exact value once."""
    return round_to_posit(_value(p, fsrc), fdst)


# --------------------------------------------------------------------------
# axpy (SGD update): y <- round(y + alpha * x)
# --------------------------------------------------------------------------

def axpy(alpha, x, y, fx, fy, fcopy=None):
    """alpha and y are patterns in fy, x in fx.  Exact inside, one rounding.

    Returns new y, or (new y, narrowed copy of new y in fcopy)."""
    va = _value(alpha, fy)
    vx = _value(x, fx)
    vy = _value(y, fy)
    if va is NaR or vx is NaR or vy is NaR:
        ynew = fy.nar
    else:
        ynew = round_to_posit(vy + va * vx, fy)
    if fcopy is None:
        return ynew
    return ynew, convert(ynew, fy, fcopy)


# --------------------------------------------------------------------------
# layer glue with exact definitions (Fig. 2: ReLU, maximum / average pooling)
# --------------------------------------------------------------------------

def relu(x, fmt):
    """max(x, 0) element by element; NaR stays NaR."""
    out = []
    for p in x:
        v = _value(p, fmt)
        out.append(fmt.nar if v is NaR else (int(p) & fmt.mask if v > 0 else 0))
    return out


def relu_bwd(y_fwd, dy, fmt_y, fmt_d):
    """dy where the forward output is positive, 0 elsewhere, NaR where the output was NaR."""
    out = []
    for py, pd in zip(y_fwd, dy):
        v = _value(py, fmt_y)
        out.append(fmt_d.nar if v is NaR else (int(pd) & fmt_d.mask if v > 0 else 0))
    return out


def _less(a, b):
    """value order with NaR below every real"""
    if b is NaR:
        return False
    if a is NaR:
        return True
    return a < b


def maxpool2d_fwd(x, planes, H, W, kh, kw, fmt):
    """Non-overlapping windows; returns (values, index of the first maximum in row-major window order)."""
    OH, OW = H // kh, W // kw
    ys, idx = [], []
    for p in range(planes):
        for oh in range(OH):
            for ow in range(OW):
                best, bi = None, 0
                for r in range(kh):
                    for c in range(kw):
                        pat = int(x[(p * H + oh * kh + r) * W + ow * kw + c]) & fmt.mask
                        v = _value(pat, fmt)
                        if best is None or _less(best[0], v):
                            best, bi = (v, pat), r * kw + c
                ys.append(best[1])
                idx.append(bi)
    return ys, idx


def maxpool2d_bwd(dy, idx, planes, H, W, kh, kw):
    OH, OW = H // kh, W // kw
    dx = [0] * (planes * H * W)
    for p in range(planes):
        for oh in range(OH):
            for ow in range(OW):
                o = (p * OH + oh) * OW + ow
                r, c = divmod(idx[o], kw)
                dx[(p * H + oh * kh + r) * W + ow * kw + c] = int(dy[o])
    return dx


def avgpool2d_fwd(x, planes, H, W, kh, kw, fin, fout):
    """Exact quire dot product of each window with the weight 1/(kh*kw) (a power of two), one rounding."""
    wpat = round_to_posit(Fraction(1, kh * kw), fin)
    assert decode(wpat, fin) == Fraction(1, kh * kw)
    OH, OW = H // kh, W // kw
    out = []
    for p in range(planes):
        for oh in range(OH):
            for ow in range(OW):
                win = [x[(p * H + oh * kh + r) * W + ow * kw + c] for r in range(kh) for c in range(kw)]
                out.append(dot(win, [wpat] * len(win), fin, fout))
    return out


def avgpool2d_bwd(dy, planes, H, W, kh, kw, fin, fout):
    wpat = round_to_posit(Fraction(1, kh * kw), fin)
    OH, OW = H // kh, W // kw
    out = []
    for p in range(planes):
        for h in range(H):
            for w in range(W):
                out.append(dot([dy[(p * OH + h // kh) * OW + w // kw]], [wpat], fin, fout))
    return out
