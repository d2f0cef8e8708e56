"""GPU parity: every entry point of the C ABI against the CPU oracle, bit for bit.

All calls go through paper_2105_00053_amd (ctypes over libpositnn_hip.so).
Inputs are seeded and synthetic (workloads module); expected values come only
from oracle/.
"""
import numpy as np
import pytest
import torch

import paper_2105_00053_amd as pn
import workloads
from oracle import fast
from oracle import posit_oracle as po

from gpu_util import BITS, GENERAL, NP_DTYPE, mismatches, oracle_axpy_chunked, rand_patterns, to_dev, to_np

pytestmark = pytest.mark.gpu
PF = {k: po.FORMATS[k] for k in BITS}


def _assert_equal(got, want, what):
    bad = mismatches(got, want)
    assert len(bad) == 0, "%s: %d mismatches, first at %s: got %s want %s" % (
        what, len(bad), bad[0], np.asarray(got)[tuple(bad[0])], np.asarray(want)[tuple(bad[0])])


# ---------------- elementwise ----------------

@pytest.mark.parametrize("dst", ["p8", "p16", "p32"])
@pytest.mark.parametrize("n", [0, 1, 5, 100003])
def test_round_f32(dst, n):
    rng = np.random.default_rng(n + 1)
    x = (rng.standard_normal(n) * np.exp2(rng.uniform(-70, 70, n))).astype(np.float32)
    if n >= 5:
        x[:5] = [0.0, -0.0, np.inf, np.nan, 1e-45]
    got = to_np(pn.posit_round(to_dev(x), dst), dst)
    _assert_equal(got, fast.round_from_float(x, dst), "round f32->" + dst)


@pytest.mark.parametrize("dst", ["p8", "p16", "p32"])
def test_round_f64_and_unaligned(dst):
    rng = np.random.default_rng(3)
    n = 50001
    x = rng.standard_normal(n) * np.exp2(rng.uniform(-300, 300, n))
    x[:4] = [5e-324, -1.7e308, np.nan, -np.inf]
    got = to_np(pn.posit_round(to_dev(x), dst), dst)
    _assert_equal(got, fast.round_from_float(x, dst), "round f64->" + dst)
    # a source pointer that is not 16-byte aligned takes the scalar kernel
    xf = x.astype(np.float32)
    base = to_dev(np.concatenate([np.zeros(1, np.float32), xf]))
    got = to_np(pn.posit_round(base[1:], dst), dst)
    _assert_equal(got, fast.round_from_float(xf, dst), "round f32 (offset)->" + dst)


@pytest.mark.parametrize("src", ["p8", "p16", "p32"])
@pytest.mark.parametrize("dst", ["p8", "p16", "p32", "f32", "f64"])
def test_convert(src, dst):
    if src == "p32":
        pats = rand_patterns(np.random.default_rng(5), 200001, "p32")
    else:
        pats = np.arange(1 << BITS[src], dtype=np.uint32).astype(NP_DTYPE[src])
    out = pn.posit_convert(to_dev(pats), src, dst)
    want = fast.to_float(pats, src, dst) if dst in ("f32", "f64") else fast.convert(pats, src, dst)
    if dst in ("f32", "f64"):
        got = out.cpu().numpy()
        nan = np.isnan(want)
        assert np.array_equal(np.isnan(got), nan)
        assert np.array_equal(got[~nan], want[~nan])
    else:
        _assert_equal(to_np(out, dst), want, "convert %s->%s" % (src, dst))


@pytest.mark.parametrize("fx,fy,fc", [("p8", "p16", "p8"), ("p16", "p16", None), ("p16", "p16", "p8"), ("p8", "p8", None),
                                      ("p16", "p32", "p16"), ("p32", "p32", "p8"), ("p32", "p16", None)])
def test_axpy(fx, fy, fc):
    rng = np.random.default_rng(BITS[fx] + BITS[fy])
    n = 70001
    x = rand_patterns(rng, n, fx)
    y = rand_patterns(rng, n, fy)
    lr = int(fast.round_from_float(np.array([-0.1], np.float32), fy)[0])
    for alpha in (lr, 1 << (BITS[fy] - 2), 0, int(rand_patterns(rng, 1, fy, 0)[0])):
        yd = to_dev(y)
        res = pn.posit_axpy(alpha, to_dev(x), yd, fx, fy, fc)
        want = fast.axpy(alpha, x, y, fx, fy, fc)
        if fc:
            _assert_equal(to_np(res[0], fy), want[0], "axpy y")
            _assert_equal(to_np(res[1], fc), want[1], "axpy copy")
        else:
            _assert_equal(to_np(res, fy), want, "axpy y")


@pytest.mark.parametrize("fx,fy,fc,n", [("p16", "p16", "p8", (1 << 22) + 13), ("p16", "p16", None, 1 << 22), ("p8", "p16", "p8", (1 << 22) + 8),
                                        ("p8", "p16", None, (1 << 22) + 1), ("p12_2", "p12_2", "p8_2", (1 << 19) + 5),
                                        ("p12_2", "p12_2", None, 1 << 19), ("p8_2", "p12_2", "p8_2", (1 << 19) + 7), ("p8_2", "p12_2", None, (1 << 20) + 3)])
def test_axpy_large_tensors_take_the_binary64_kernel(fx, fy, fc, n):
    """Sizes from which posit_axpy switches to the kernel with LDS decode tables and binary64 arithmetic (whole vectors
    of 8, the generic kernel on the ragged tail): every pattern of y occurs, against random x, with special patterns,
    near-cancelling pairs and pairs far apart; two values of alpha."""
    rng = np.random.default_rng(n % 1000 + BITS[fx])
    mask = (1 << BITS[fy]) - 1
    x = rand_patterns(rng, n, fx, special=0.01)
    y = rand_patterns(rng, n, fy, special=0.01)
    y[: 1 << BITS[fy]] = np.arange(1 << BITS[fy], dtype=np.uint32).astype(NP_DTYPE[fy])
    lr = int(fast.round_from_float(np.array([-0.1], np.float32), fy)[0])
    # a stretch where y nearly cancels alpha * x
    m = 200000
    t = fast.axpy(lr, x[-m:], np.zeros(m, dtype=NP_DTYPE[fy]), fx, fy).astype(np.int64)
    y[-m:] = ((-t + rng.integers(-2, 3, m)) & mask).astype(NP_DTYPE[fy])
    for alpha in (lr, int(rand_patterns(rng, 1, fy, 0, allow_nar=False)[0])):
        yd = to_dev(y)
        res = pn.posit_axpy(alpha, to_dev(x), yd, fx, fy, fc)
        want = oracle_axpy_chunked(alpha, x, y, fx, fy, fc)
        if fc:
            _assert_equal(to_np(res[0], fy), want[0], "axpy y")
            _assert_equal(to_np(res[1], fc), want[1], "axpy copy")
        else:
            _assert_equal(to_np(res, fy), want, "axpy y")


def test_convert_posit16_to_posit8_large_takes_the_step_table_kernel():
    n = (1 << 21) + 11
    rng = np.random.default_rng(5)
    pats = rng.integers(0, 1 << 16, n, dtype=np.uint32).astype(np.uint16)
    pats[: 1 << 16] = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    got = to_np(pn.posit_convert(to_dev(pats), "p16", "p8"), "p8")
    _assert_equal(got, fast.convert(pats, "p16", "p8"), "convert p16->p8, large")


@pytest.mark.parametrize("fx,fy,fc", [("p16", "p16", "p8"), ("p8_2", "p12_2", "p8_2"), ("p32", "p32", None), ("p8", "p16", None)])
def test_axpy_multi(fx, fy, fc):
    """Twenty tensors of assorted sizes (more than one launch holds, some empty, some without a copy) updated at once."""
    rng = np.random.default_rng(BITS[fx] * 3 + BITS[fy])
    sizes = [1, 0, 7, 300, 4097, 25, 0, 10, 64, 70001, 3, 864, 32, 9216, 5, 0, 129, 2, 1000, 31]
    lr = int(fast.round_from_float(np.array([-0.1], np.float32), fy)[0])
    xs = [rand_patterns(rng, n, fx) for n in sizes]
    ys = [rand_patterns(rng, n, fy) for n in sizes]
    xd, yd = [to_dev(a) for a in xs], [to_dev(a) for a in ys]
    copies = None
    if fc:
        copies = [torch.zeros(n, dtype=pn.binding.TORCH_DTYPE[pn.binding.FORMAT_CODES[fc]], device="cuda") if i % 3 else None
                  for i, n in enumerate(sizes)]
    pn.posit_axpy_multi(lr, xd, yd, fx, fy, fcopy=fc, y_copies=copies)
    for i, n in enumerate(sizes):
        if n == 0:
            continue
        want = fast.axpy(lr, xs[i], ys[i], fx, fy, fc if fc else None)
        wy = want[0] if fc else want
        _assert_equal(to_np(yd[i], fy), wy, "tensor %d" % i)
        if fc and copies[i] is not None:
            _assert_equal(to_np(copies[i], fc), want[1], "copy %d" % i)


# ---------------- GEMM ----------------

def test_config1_p8_gemm_64_against_python_oracle():
    A, B = workloads.gemm_operands(1, 64)
    Ap = to_np(pn.posit_round(to_dev(A), "p8"), "p8")
    Bp = to_np(pn.posit_round(to_dev(B), "p8"), "p8")
    _assert_equal(Ap, fast.round_from_float(A, "p8"), "A patterns")
    C = to_np(pn.posit_gemm(to_dev(Ap), to_dev(Bp), "p8", "p8"), "p8")
    want = np.array(po.gemm(Ap.tolist(), Bp.tolist(), po.P8, po.P8))
    _assert_equal(C, want, "config 1")


GEMM_CASES = [
    # fin, fout, M, N, K, transA, transB, bias, nar
    ("p8", "p8", 130, 70, 100, 0, 0, 0, 0),
    ("p8", "p8", 64, 64, 64, 1, 0, 1, 1),
    ("p8", "p16", 33, 129, 257, 0, 1, 1, 1),
    ("p8", "p32", 17, 5, 31, 1, 1, 0, 0),
    ("p8", "p8", 1, 1, 1, 0, 0, 0, 0),
    ("p8", "p8", 256, 256, 512, 0, 0, 0, 0),
    ("p16", "p16", 70, 130, 100, 0, 0, 1, 1),
    ("p16", "p8", 65, 63, 129, 1, 0, 0, 0),
    ("p16", "p32", 20, 33, 64, 0, 1, 1, 0),
    ("p16", "p16", 128, 128, 256, 1, 1, 0, 1),
    ("p32", "p32", 40, 35, 50, 0, 0, 1, 1),
    ("p32", "p16", 33, 31, 40, 1, 1, 0, 0),
    ("p32", "p8", 16, 16, 33, 0, 1, 0, 0),
    # many outputs, a reduction of at most two slices: the one-thread-per-output kernel, not the tiled ones
    ("p8", "p8", 128, 2048, 10, 0, 0, 1, 1),
    ("p8", "p16", 300, 400, 40, 1, 1, 0, 1),
    ("p8", "p8", 1000, 700, 64, 0, 1, 1, 0),
]


@pytest.mark.parametrize("fin,fout,M,N,K,ta,tb,use_bias,nar", GEMM_CASES)
def test_gemm_random_patterns(fin, fout, M, N, K, ta, tb, use_bias, nar):
    rng = np.random.default_rng(M * 7 + N * 3 + K)
    A = rand_patterns(rng, (K, M) if ta else (M, K), fin, allow_nar=bool(nar), special=0.01)
    B = rand_patterns(rng, (N, K) if tb else (K, N), fin, allow_nar=bool(nar), special=0.01)
    bias = rand_patterns(rng, (N,), fin, allow_nar=bool(nar)) if use_bias else None
    got = pn.posit_gemm(to_dev(A), to_dev(B), fin, fout, trans_a=ta, trans_b=tb, bias=None if bias is None else to_dev(bias))
    want, _ = fast.gemm(A, B, fin, fout, trans_a=ta, trans_b=tb, bias=bias)
    _assert_equal(to_np(got, fout), want, "gemm %s->%s %dx%dx%d" % (fin, fout, M, N, K))


@pytest.mark.parametrize("M,N,K,ta,tb,fout,use_bias", [
    (65, 65, 128, 0, 0, "p8", 0), (130, 257, 1000, 0, 1, "p16", 1), (200, 150, 4096, 1, 0, "p8", 1), (129, 300, 555, 1, 1, "p8", 0),
    (256, 192, 2048, 0, 0, "p32", 1), (70, 2000, 130, 0, 0, "p8", 0), (1000, 66, 129, 1, 0, "p8", 1), (384, 320, 1056, 0, 1, "p8", 0),
    (1280, 1152, 160, 1, 1, "p16", 0), (300, 260, 9000, 0, 0, "p8", 1)])
def test_p8_gemm_reduction_cut_inside_the_workgroup(M, N, K, ta, tb, fout, use_bias):
    """posit<8,0> products with too few 128 x 128 tiles to fill the chip: 64 x 64 tiles, the four waves of a workgroup
    each take a quarter of the reduction and merge in LDS.  Ragged edges in all three dimensions, quarters that are no
    whole number of slices (and waves left with nothing: K = 128 .. 160), unaligned pitches (K = 555, 129: byte-wise
    fetch), the four transposition cases, NaR in both operands near the edges, bias, three output formats."""
    # a long reduction over few tiles is cut across workgroups as well (workspace + merge kernel)
    assert (pn.posit_gemm_workspace("p8", fout, ta, tb, M, N, K) > 0) == ((M, N, K) in ((200, 150, 4096), (256, 192, 2048), (300, 260, 9000)))
    rng = np.random.default_rng(M + 3 * N + 7 * K)
    A = rand_patterns(rng, (M, K), "p8", special=0.002, allow_nar=False)
    B = rand_patterns(rng, (K, N), "p8", special=0.002, allow_nar=False)
    A[M - 1, K - 1] = 0x80   # last row of C is NaR
    A[min(M - 1, 70), 0] = 0x80
    B[0, N - 1] = 0x80       # last column of C is NaR
    B[K - 1, min(N - 1, 65)] = 0x80
    bias = rand_patterns(rng, (N,), "p8", allow_nar=False) if use_bias else None
    if use_bias:
        bias[1] = 0x80
    Ain, Bin = (np.ascontiguousarray(A.T) if ta else A), (np.ascontiguousarray(B.T) if tb else B)
    got = to_np(pn.posit_gemm(to_dev(Ain), to_dev(Bin), "p8", fout, trans_a=ta, trans_b=tb, bias=None if bias is None else to_dev(bias)), fout)
    want, _ = fast.gemm(Ain, Bin, "p8", fout, trans_a=ta, trans_b=tb, bias=bias)
    _assert_equal(got, want, "w4 gemm %dx%dx%d" % (M, N, K))
    nar = 1 << (BITS[fout] - 1)
    assert (want[M - 1] == nar).all() and (want[:, N - 1] == nar).all()


@pytest.mark.parametrize("fin,fout,M,N,K,ta,tb,use_bias", [
    ("p16", "p16", 96, 96, 64, 0, 0, 0), ("p16", "p8", 100, 130, 200, 1, 0, 1), ("p16", "p16", 200, 150, 1100, 0, 1, 1),
    ("p16", "p32", 129, 257, 333, 1, 1, 0), ("p16", "p16", 128, 128, 2048, 0, 0, 1), ("p16", "p16", 97, 99, 70000, 0, 0, 0),
    ("p16", "p16", 1700, 1600, 130, 0, 0, 1), ("p12_2", "p12_2", 130, 140, 520, 0, 1, 1), ("p12_2", "p8_2", 1700, 1600, 90, 1, 0, 0),
    ("p10_1", "p10_1", 300, 200, 777, 1, 1, 1), ("p10_2", "p12_2", 111, 222, 4096, 0, 0, 0), ("p12_1", "p12_1", 2000, 1400, 100, 0, 0, 0),
    ("p10_2", "p10_2", 900, 900, 2500, 0, 0, 0)])  # enough tiles, but more products per output than the buckets' guard bits allow: cut anyway
def test_bucket_formats_gemm_with_operands_decoded_once(fin, fout, M, N, K, ta, tb, use_bias):
    """posit<16,1> and the 10- / 12-bit formats beyond 96 x 96 outputs: both operands are decoded into the workspace
    first (so the call always needs one), 32 x 32 or 64 x 64 tiles, the reduction cut across workgroups for few tiles
    or beyond 2^16 products per output.  Ragged edges in all three dimensions, the four transposition cases, NaR in
    both operands at the edges, bias with a NaR entry, several output formats; random patterns over the whole
    regime range, so sums span all buckets."""
    assert pn.posit_gemm_workspace(fin, fout, ta, tb, M, N, K) >= 8 * K * (M + N)
    rng = np.random.default_rng(M + 3 * N + 7 * K)
    A = rand_patterns(rng, (M, K), fin, special=0.002, allow_nar=False)
    B = rand_patterns(rng, (K, N), fin, special=0.002, allow_nar=False)
    nar_in = 1 << (BITS[fin] - 1)
    A[M - 1, K - 1] = nar_in   # last row of C is NaR
    A[min(M - 1, 70), 0] = nar_in
    B[0, N - 1] = nar_in       # last column of C is NaR
    B[K - 1, min(N - 1, 65)] = nar_in
    bias = rand_patterns(rng, (N,), fin, allow_nar=False) if use_bias else None
    if use_bias:
        bias[1] = nar_in
    Ain, Bin = (np.ascontiguousarray(A.T) if ta else A), (np.ascontiguousarray(B.T) if tb else B)
    got = to_np(pn.posit_gemm(to_dev(Ain), to_dev(Bin), fin, fout, trans_a=ta, trans_b=tb, bias=None if bias is None else to_dev(bias)), fout)
    want, _ = fast.gemm(Ain, Bin, fin, fout, trans_a=ta, trans_b=tb, bias=bias)
    _assert_equal(got, want, "decoded-once gemm %s %dx%dx%d" % (fin, M, N, K))
    nar = 1 << (BITS[fout] - 1)
    assert (want[M - 1] == nar).all() and (want[:, N - 1] == nar).all() and (want[70, :N - 1] == nar).all()
    assert (want[:M - 1, :N - 1] != nar).sum() > (M - 3) * (N - 3)


@pytest.mark.parametrize("share,M,N,K,ta,tb", [(0.0, 130, 140, 1300, 0, 0), (0.3, 130, 140, 1300, 0, 1), (1.0, 100, 97, 300, 1, 0),
                                               (0.05, 200, 300, 2500, 1, 1), (0.5, 1100, 1050, 96, 0, 0)])
def test_p16_gemm_long_regime_operands_take_the_integer_correction(share, M, N, K, ta, tb):
    """posit<16,1> operands outside the band the two fp64 buckets cover (|x| below about 2^-23 or above 2^18) are
    multiplied in integer arithmetic by the owner of each output.  A given share of both operands is replaced by
    such values (either sign, down to minpos and up to maxpos), from none to all of them; where an outlier of A
    meets an outlier of B the product must be counted once."""
    rng = np.random.default_rng(int(share * 100) + K)
    A = fast.round_from_float(rng.standard_normal((M, K)).astype(np.float32), "p16")
    B = fast.round_from_float((rng.standard_normal((K, N)) * 0.05).astype(np.float32), "p16")
    for X in (A, B):
        pick = rng.random(X.shape) < share
        n = int(pick.sum())
        tiny = rng.integers(1, 0x0040, n)          # minpos .. about 2^-22
        huge = rng.integers(0x7F00, 0x8000, n)     # about 2^14 .. maxpos
        mag = np.where(rng.random(n) < 0.5, tiny, huge)
        pat = np.where(rng.random(n) < 0.5, mag, (0x10000 - mag) & 0xFFFF)
        X[pick] = pat.astype(np.uint16)
    A[3, 5] = 0x8000  # NaR row
    Ain, Bin = (np.ascontiguousarray(A.T) if ta else A), (np.ascontiguousarray(B.T) if tb else B)
    got = to_np(pn.posit_gemm(to_dev(Ain), to_dev(Bin), "p16", "p16", trans_a=ta, trans_b=tb), "p16")
    want, _ = fast.gemm(Ain, Bin, "p16", "p16", trans_a=ta, trans_b=tb)
    _assert_equal(got, want, "p16 gemm, outlier share %.2f" % share)
    assert (want[3] == 0x8000).all() and (want[4] != 0x8000).all()


@pytest.mark.parametrize("M,N,K,ta,tb,fout,use_bias", [(450, 470, 77, 0, 0, "p32", 1), (449, 433, 130, 1, 0, "p16", 0), (600, 330, 40, 0, 1, "p32", 1),
                                                       (400, 500, 1, 1, 1, "p8", 1)])
def test_p32_gemm_quire_in_lds(M, N, K, ta, tb, fout, use_bias):
    """posit<32,2> products with at least 768 tiles of 16 x 16 outputs: one output per thread, its 512-bit quire in LDS
    as lazily carried 64-bit limbs.  Random patterns over the whole regime range (products land on every limb, both
    signs), ragged edges, the four transposition cases, NaR rows and columns, bias, three output formats; no workspace."""
    assert pn.posit_gemm_workspace("p32", fout, ta, tb, M, N, K) == 0
    rng = np.random.default_rng(M + 3 * N + 7 * K)
    A = rand_patterns(rng, (M, K), "p32", special=0.002, allow_nar=False)
    B = rand_patterns(rng, (K, N), "p32", special=0.002, allow_nar=False)
    A[M - 1, K - 1] = 1 << 31   # last row of C is NaR
    B[0, N - 1] = 1 << 31       # last column of C is NaR
    # extreme products: maxpos^2, minpos^2 and their negatives in one dot product
    A[0, 0], B[0, 0] = 0x7FFFFFFF, 0x7FFFFFFF
    if K > 2:
        A[0, 1], B[1, 0] = 0x00000001, 0x00000001
        A[0, 2], B[2, 0] = 0x80000001, 0x7FFFFFFF   # -maxpos * maxpos: cancels the first term exactly
    bias = rand_patterns(rng, (N,), "p32", allow_nar=False) if use_bias else None
    if use_bias:
        bias[1] = 1 << 31
    Ain, Bin = (np.ascontiguousarray(A.T) if ta else A), (np.ascontiguousarray(B.T) if tb else B)
    got = to_np(pn.posit_gemm(to_dev(Ain), to_dev(Bin), "p32", fout, trans_a=ta, trans_b=tb, bias=None if bias is None else to_dev(bias)), fout)
    want, _ = fast.gemm(Ain, Bin, "p32", fout, trans_a=ta, trans_b=tb, bias=bias)
    _assert_equal(got, want, "p32 gemm with the quire in LDS %dx%dx%d" % (M, N, K))
    nar = 1 << (BITS[fout] - 1)
    assert (want[M - 1] == nar).all() and (want[:, N - 1] == nar).all() and (want[:M - 1, 2:N - 1] != nar).all()


def test_gemm_padded_leading_dimensions_and_k0():
    rng = np.random.default_rng(8)
    M, N, K = 37, 29, 41
    Abig = rand_patterns(rng, (M, K + 5), "p8")
    Bbig = rand_patterns(rng, (K, N + 3), "p8")
    Cbig = np.full((M, N + 7), 0x55, dtype=np.uint8)
    L = pn.load()
    import ctypes
    Ad, Bd, Cd = to_dev(Abig), to_dev(Bbig), to_dev(Cbig)
    rc = L.posit_gemm(None, 0, 0, 0, 0, M, N, K, ctypes.c_void_p(Ad.data_ptr()), K + 5, ctypes.c_void_p(Bd.data_ptr()), N + 3,
                      None, ctypes.c_void_p(Cd.data_ptr()), N + 7, None, 0)
    assert rc == 0
    torch.cuda.synchronize()
    got = Cd.cpu().numpy()
    want, _ = fast.gemm(np.ascontiguousarray(Abig[:, :K]), np.ascontiguousarray(Bbig[:, :N]), "p8", "p8")
    _assert_equal(got[:, :N], want, "padded ld")
    assert (got[:, N:] == 0x55).all()  # padding columns untouched
    # K = 0: the rounded bias (or zero)
    bias = rand_patterns(rng, (N,), "p16", allow_nar=False)
    A0 = torch.empty((M, 0), dtype=torch.int16, device="cuda")
    B0 = torch.empty((0, N), dtype=torch.int16, device="cuda")
    got = to_np(pn.posit_gemm(A0, B0, "p16", "p8", bias=to_dev(bias)), "p8")
    _assert_equal(got, np.tile(fast.convert(bias, "p16", "p8"), (M, 1)), "K=0 with bias")
    got = to_np(pn.posit_gemm(A0, B0, "p16", "p16"), "p16")
    assert (got == 0).all()


@pytest.mark.parametrize("fin,fout,M,N,K", [("p8", "p16", 32, 288, 8192), ("p16", "p16", 16, 50, 4096), ("p32", "p32", 8, 20, 2048),
                                            ("p8", "p8", 6, 25, 50176)])
def test_gemm_split_reduction(fin, fout, M, N, K):
    """Small outputs with a long reduction: the reduction is split over workgroups (needs workspace) or, for the
    smallest posit<8,0> problems, over the threads of an output; the merged quires must give the same bits."""
    small_p8 = fin == "p8" and M * N * K <= 1 << 26
    assert (pn.posit_gemm_workspace(fin, fout, 1, 0, M, N, K) > 0) != small_p8
    rng = np.random.default_rng(K)
    A = rand_patterns(rng, (K, M), fin, special=0.001)
    B = rand_patterns(rng, (K, N), fin, special=0.001)
    A[5, 3] = 1 << (BITS[fin] - 1)  # one NaR: row 3 of the product is NaR
    bias = rand_patterns(rng, (N,), fin, allow_nar=False)
    got = pn.posit_gemm(to_dev(A), to_dev(B), fin, fout, trans_a=True, bias=to_dev(bias))
    want, _ = fast.gemm(A, B, fin, fout, trans_a=True, bias=bias)
    _assert_equal(to_np(got, fout), want, "split gemm")
    assert (want[3] == (1 << (BITS[fout] - 1))).all()


def test_config2_p16_gemm_1024_with_regime_extremes():
    A, B = workloads.gemm_operands(2, 1024, sigma=0.1, extremes=True)
    Ap = to_np(pn.posit_round(to_dev(A), "p16"), "p16")
    Bp = to_np(pn.posit_round(to_dev(B), "p16"), "p16")
    _assert_equal(Ap, fast.round_from_float(A, "p16"), "A patterns")
    _assert_equal(Bp, fast.round_from_float(B, "p16"), "B patterns")
    C = to_np(pn.posit_gemm(to_dev(Ap), to_dev(Bp), "p16", "p16"), "p16")
    want, overflowed = fast.gemm(Ap, Bp, "p16", "p16")
    assert overflowed == 0
    _assert_equal(C, want, "config 2")
    # a few entries again through the Python oracle
    rng = np.random.default_rng(0)
    for _ in range(16):
        i, j = int(rng.integers(1024)), int(rng.integers(1024))
        assert int(C[i, j]) == po.dot(Ap[i].tolist(), Bp[:, j].tolist(), po.P16, po.P16)


def test_config5_p8_gemm_1024_full_and_p32_wide_quire():
    A, B = workloads.gemm_operands(5, 1024)
    Ap, Bp = fast.round_from_float(A, "p8"), fast.round_from_float(B, "p8")
    C = to_np(pn.posit_gemm(to_dev(Ap), to_dev(Bp), "p8", "p8"), "p8")
    want, overflowed = fast.gemm(Ap, Bp, "p8", "p8")
    assert overflowed == 0
    _assert_equal(C, want, "config 5, 1024")
    # posit<32,2>, 512-bit quire, 1024^3: the whole product against the C++ oracle, entries against Python
    A32, B32 = fast.round_from_float(A, "p32"), fast.round_from_float(B, "p32")
    C32 = to_np(pn.posit_gemm(to_dev(A32), to_dev(B32), "p32", "p32"), "p32")
    want, overflowed = fast.gemm(A32, B32, "p32", "p32")
    assert overflowed == 0
    _assert_equal(C32, want, "config 5, posit<32,2> 1024")
    rng = np.random.default_rng(1)
    for _ in range(8):
        i, j = int(rng.integers(1024)), int(rng.integers(1024))
        assert int(C32[i, j]) == po.dot(A32[i].tolist(), B32[:, j].tolist(), po.P32, po.P32)


@pytest.mark.timeout(400)
@pytest.mark.parametrize("S", [2048, 4096])
def test_config5_p8_gemm_large_full(S):
    """Full benchmark size, same launch path as bench.py (the integer-matrix-core kernel the headline figure is
    timed on: two int8 digits per operand, three int32 sums per output): every one of the S x S outputs against the
    C++ oracle (about 45 s of host time at 4096), a few entries again through the Python oracle."""
    A, B = workloads.gemm_operands(5, S)
    Ap, Bp = fast.round_from_float(A, "p8"), fast.round_from_float(B, "p8")
    C = to_np(pn.posit_gemm(to_dev(Ap), to_dev(Bp), "p8", "p8"), "p8")
    want, overflowed = fast.gemm(Ap, Bp, "p8", "p8")
    assert overflowed == 0
    _assert_equal(C, want, "config 5, %d" % S)
    rng = np.random.default_rng(S)
    for _ in range(8):
        i, j = int(rng.integers(S)), int(rng.integers(S))
        assert int(C[i, j]) == po.dot(Ap[i].tolist(), Bp[:, j].tolist(), po.P8, po.P8)
    # property that holds at any size: negating A negates C pattern-wise (two's complement)
    An = ((-Ap.astype(np.int16)) & 0xFF).astype(np.uint8)
    Cn = to_np(pn.posit_gemm(to_dev(An), to_dev(Bp), "p8", "p8"), "p8")
    assert np.array_equal(Cn, ((-C.astype(np.int16)) & 0xFF).astype(np.uint8))


@pytest.mark.parametrize("M,N,K,ta,tb,fout", [(2100, 2050, 4000, 0, 0, "p8"), (2048, 2176, 4100, 1, 0, "p16"), (2300, 2048, 3999, 0, 1, "p8"),
                                              (2050, 2100, 4033, 1, 1, "p8"), (1100, 1030, 16400, 0, 0, "p8"),
                                              (600, 540, 1700, 0, 0, "p8"), (2200, 1900, 300, 1, 0, "p8"), (1900, 2200, 290, 0, 1, "p16"),
                                              (1030, 1025, 1024, 1, 1, "p8"), (200, 300, 9000, 0, 1, "p8"), (384, 640, 2100, 1, 0, "p16"),
                                              (130, 4100, 600, 0, 0, "p8")])
def test_p8_gemm_packed_operands_path(M, N, K, ta, tb, fout):
    """Products of 2^28 MACs and more (outputs at least 128 each way) first rewrite both operands into the workspace (int8 digit planes in the lane
    order of the matrix instruction, NaR as a marker digit) and run on the matrix cores: ragged sizes, the four
    transposition cases (an operand stored reduction-index-major is transposed through LDS), NaR in rows and columns
    near the edges, a bias, a workspace full of ones; the cases after the first five take the 64 x 64, 128 x 64 and
    64 x 128 tiles chosen when 128 x 128 would leave compute units idle, two of them (fewer than 81 tiles of 64 x 64) the
    split form: slices of the reduction per tile, merged by a second launch; the last is 130 rows thin.  Sampled rows against the oracle, the NaR rows and columns in full."""
    assert M * N * K >= 1 << 28 and min(M, N) >= 128
    assert pn.posit_gemm_workspace("p8", fout, ta, tb, M, N, K) >= 4 * (K // 2) * (M + N)
    rng = np.random.default_rng(M + K)
    A = rand_patterns(rng, (K, M) if ta else (M, K), "p8", special=0.001, allow_nar=False)
    B = rand_patterns(rng, (N, K) if tb else (K, N), "p8", special=0.001, allow_nar=False)
    bias = rand_patterns(rng, (N,), "p8", allow_nar=False)
    nar_rows, nar_cols = [5, M - 1], [0, N - 2]
    for i, r in enumerate(nar_rows):
        k = [K - 1, 17][i]
        if ta: A[k, r] = 0x80
        else: A[r, k] = 0x80
    for i, c in enumerate(nar_cols):
        k = [3, K - 2][i]
        if tb: B[c, k] = 0x80
        else: B[k, c] = 0x80
    ws = torch.full((pn.posit_gemm_workspace("p8", fout, ta, tb, M, N, K) + 64,), 0xFF, dtype=torch.uint8, device="cuda")
    got = to_np(pn.posit_gemm(to_dev(A), to_dev(B), "p8", fout, trans_a=ta, trans_b=tb, bias=to_dev(bias), workspace=ws), fout)
    onar = 1 << (BITS[fout] - 1)
    for r in nar_rows:
        assert (got[r] == onar).all()
    for c in nar_cols:
        assert (got[:, c] == onar).all()
    assert (got == onar).sum() == 2 * N + 2 * M - 4
    rows = sorted(set([0, 4, 6, 127, 128, M - 2] + [int(r) for r in rng.integers(0, M, size=4)]) - set(nar_rows))
    for r in rows:
        want, _ = fast.gemm(A, B, "p8", fout, trans_a=ta, trans_b=tb, bias=bias, rows=(r, r + 1))
        _assert_equal(got[r], want[r], "packed path row %d" % r)


@pytest.mark.parametrize("fin", ["p8_2", "p8_1"])
@pytest.mark.parametrize("M,N,K,ta,tb,fout", [(520, 1000, 700, 0, 0, None), (600, 900, 1030, 1, 0, "p16"), (900, 530, 999, 0, 1, None),
                                              (515, 1100, 800, 1, 1, "p12_2"), (1024, 1024, 1024, 0, 0, None)])
def test_b8_gemm_on_the_integer_matrix_cores(fin, M, N, K, ta, tb, fout):
    """posit(8,1) / posit(8,2) products of 2^28 MACs and more (128 outputs each way, reductions up to 8192) rewrite both
    operands as signed base-128 digit planes over the whole range of the format (4 / 8 planes) and run on the integer
    matrix cores, skipping the digit planes a block does not use.  Patterns uniform over the whole format (every plane
    in use), the four transposition cases, ragged sizes, NaR in rows and columns near the edges, a bias, a workspace full
    of ones; the last case is Gaussian data (few planes in use: the skipping at work).  Sampled rows against the oracle,
    the NaR rows and columns in full."""
    fout = fout or fin
    assert pn.posit_gemm_workspace(fin, fout, ta, tb, M, N, K) >= 4 * K * (M + N)   # at least four planes per operand
    rng = np.random.default_rng(M + K + BITS[fin])
    if M == 1024:
        A = fast.round_from_float(rng.standard_normal((M, K)).astype(np.float32), fin)
        B = fast.round_from_float((0.05 * rng.standard_normal((K, N))).astype(np.float32), fin)
    else:
        A = rand_patterns(rng, (K, M) if ta else (M, K), fin, special=0.001, allow_nar=False)
        B = rand_patterns(rng, (N, K) if tb else (K, N), fin, special=0.001, allow_nar=False)
    bias = rand_patterns(rng, (N,), fin, allow_nar=False)
    nar_rows, nar_cols = [5, M - 1], [0, N - 2]
    for i, r in enumerate(nar_rows):
        k = [K - 1, 17][i]
        if ta: A[k, r] = 0x80
        else: A[r, k] = 0x80
    for i, c in enumerate(nar_cols):
        k = [3, K - 2][i]
        if tb: B[c, k] = 0x80
        else: B[k, c] = 0x80
    ws = torch.full((pn.posit_gemm_workspace(fin, fout, ta, tb, M, N, K) + 64,), 0xFF, dtype=torch.uint8, device="cuda")
    got = to_np(pn.posit_gemm(to_dev(A), to_dev(B), fin, fout, trans_a=ta, trans_b=tb, bias=to_dev(bias), workspace=ws), fout)
    onar = 1 << (BITS[fout] - 1)
    for r in nar_rows:
        assert (got[r] == onar).all()
    for c in nar_cols:
        assert (got[:, c] == onar).all()
    assert (got == onar).sum() == 2 * N + 2 * M - 4
    rows = sorted(set([0, 4, 6, 31, 32, 63, 64, M - 2] + [int(r) for r in rng.integers(0, M, size=6)]) - set(nar_rows))
    for r in rows:
        want, _ = fast.gemm(A, B, fin, fout, trans_a=ta, trans_b=tb, bias=bias, rows=(r, r + 1))
        _assert_equal(got[r], want[r], "matrix-core path of %s, row %d" % (fin, r))


@pytest.mark.parametrize("fin", ["p8_2", "p8_1"])
@pytest.mark.parametrize("case", ["gaussian", "offset", "offset and NaR", "wide", "five planes", "gaussian, large", "zero"])
def test_b8_gemm_matrix_cores_narrow_and_wide_operands(fin, case):
    """posit(8,2) operands whose digits all lie in four (five, from 2^31 products on) adjacent planes take a product
    kernel with seven (nine) sums, counted from the lowest plane each operand uses; anything wider takes the one over
    all planes.  posit(8,1) has a three-plane kernel, used from 2^32 products on.
    gaussian: planes from 0 up.  offset: A in +-[1, 64), B in +-[2^-10, 2^-4): both windows start above plane 0.
    offset and NaR: values from 1/8 up and NaR, whose marker in the top plane is then inside the window.  wide: Gaussian
    data plus a few huge and a few tiny values.  five planes: A over 2^-13 .. 2^16 in a product large enough for the
    nine-sum kernel.  gaussian, large: the size at which posit(8,1) takes its narrow kernel.  zero: A is all zeros (no plane in use).  Sampled rows and the NaR rows / columns against the oracle."""
    M, N, K, ta, tb = (1664, 1700, 1536, 0, 1) if case in ("five planes", "gaussian, large") else (640, 520, 1100, 0, 1)
    rng = np.random.default_rng(len(case) + BITS[fin] + int(fin[-1]))

    def signed_log_uniform(shape, lo, hi):
        mag = np.exp2(rng.uniform(lo, hi, size=shape))
        return (mag * rng.choice([-1.0, 1.0], size=shape)).astype(np.float32)

    if case in ("gaussian", "gaussian, large"):
        Af, Bf = rng.standard_normal((M, K)), 0.05 * rng.standard_normal((N, K))
    elif case == "offset":
        Af, Bf = signed_log_uniform((M, K), 0, 6), signed_log_uniform((N, K), -10, -4)
    elif case == "offset and NaR":
        Af, Bf = signed_log_uniform((M, K), 0, 6), signed_log_uniform((N, K), -3, 3)
    elif case == "five planes":
        Af, Bf = signed_log_uniform((M, K), -13, 16), rng.standard_normal((N, K))
    elif case == "zero":
        Af, Bf = np.zeros((M, K)), rng.standard_normal((N, K))
    else:
        Af, Bf = rng.standard_normal((M, K)), rng.standard_normal((N, K))
        Af[rng.integers(0, M, 5), rng.integers(0, K, 5)] = 3000.0
        Bf[rng.integers(0, N, 5), rng.integers(0, K, 5)] = 1e-6
    A = fast.round_from_float(np.asarray(Af, dtype=np.float32), fin)
    B = fast.round_from_float(np.asarray(Bf, dtype=np.float32), fin)
    nar_rows, nar_cols = [], []
    if case == "offset and NaR":
        nar_rows, nar_cols = [7, M - 1], [N - 3]
        A[7, K - 1] = A[M - 1, 40] = 0x80
        B[N - 3, 0] = 0x80
    ws = torch.full((pn.posit_gemm_workspace(fin, fin, ta, tb, M, N, K) + 64,), 0xFF, dtype=torch.uint8, device="cuda")
    got = to_np(pn.posit_gemm(to_dev(A), to_dev(B), fin, fin, trans_a=ta, trans_b=tb, workspace=ws), fin)
    for r in nar_rows:
        assert (got[r] == 0x80).all()
    for c in nar_cols:
        assert (got[:, c] == 0x80).all()
    assert (got == 0x80).sum() == len(nar_rows) * N + len(nar_cols) * (M - len(nar_rows))
    rows = sorted(set([0, 31, 32, 63, 64, M - 2] + [int(r) for r in rng.integers(0, M, size=6)]) - set(nar_rows))
    for r in rows:
        want, _ = fast.gemm(A, B, fin, fin, trans_a=ta, trans_b=tb, rows=(r, r + 1))
        _assert_equal(got[r], want[r], "%s, %s operands, row %d" % (fin, case, r))
    if case == "zero":
        assert (got == 0).all()
    else:
        assert len(set(got[rows].ravel().tolist())) > 8   # not a constant


def test_b8_gemm_graph_replay_follows_the_data():
    """Which posit(8,2) product kernel does the work is decided on the device, from the operands' plane masks, so a
    captured call must follow the data of each replay: narrow operands, then operands over the whole range, then NaR,
    then narrow ones again, every replay compared with an eager call on the same operands (bit for bit) and the first
    one with the oracle on sampled rows."""
    fin, M, N, K = "p8_2", 384, 448, 1024
    rng = np.random.default_rng(82)
    narrow = lambda shape, s: fast.round_from_float((s * rng.standard_normal(shape)).astype(np.float32), fin)
    fills = [(narrow((M, K), 1.0), narrow((K, N), 0.05)),
             (rand_patterns(rng, (M, K), fin, allow_nar=False), rand_patterns(rng, (K, N), fin, allow_nar=False)),
             (narrow((M, K), 1.0), narrow((K, N), 1.0)),
             (narrow((M, K), 0.01), narrow((K, N), 8.0))]
    fills[2][0][17, 5] = 0x80
    A = torch.zeros((M, K), dtype=torch.uint8, device="cuda")
    B = torch.zeros((K, N), dtype=torch.uint8, device="cuda")
    C = torch.zeros((M, N), dtype=torch.uint8, device="cuda")
    ws = torch.full((pn.posit_gemm_workspace(fin, fin, 0, 0, M, N, K),), 0xFF, dtype=torch.uint8, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        pn.posit_gemm(A, B, fin, fin, out=C, workspace=ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        pn.posit_gemm(A, B, fin, fin, out=C, workspace=ws)
    for i, (a, b) in enumerate(fills):
        A.copy_(to_dev(a)); B.copy_(to_dev(b))
        C.fill_(0x55)
        graph.replay()
        torch.cuda.synchronize()
        got = to_np(C, fin).copy()
        eager = to_np(pn.posit_gemm(to_dev(a), to_dev(b), fin, fin), fin)
        assert np.array_equal(got, eager), "replay %d" % i
        if i == 2:
            assert (got[17] == 0x80).all() and (got == 0x80).sum() == N
        if i == 0:
            for r in (0, 100, M - 1):
                want, _ = fast.gemm(a, b, fin, fin, rows=(r, r + 1))
                _assert_equal(got[r], want[r], "replay 0, row %d" % r)


@pytest.mark.parametrize("M,N,K,ta,tb,kernel", [(130, 130, 259, 0, 0, "tiled dot2"), (131, 140, 300, 1, 1, "tiled dot2, transposed"),
                                                (40, 300, 8200, 0, 0, "byte gather"), (20, 30, 300, 0, 1, "small problem"),
                                                (1100, 1030, 16400, 0, 0, "packed operands")])
def test_p8_quire_wraps_modulo_2_32_in_every_dot_product_kernel(M, N, K, ta, tb, kernel):
    """Past Table 1's limit of 127 products the 32-bit quire wraps (two's complement): a row of A and a column of B
    full of maxpos push several outputs beyond 2^31 units; the kernels must wrap, not saturate, like the oracle."""
    rng = np.random.default_rng(K)
    A = rand_patterns(rng, (M, K), "p8", special=0.0, allow_nar=False)
    B = rand_patterns(rng, (K, N), "p8", special=0.0, allow_nar=False)
    A[0, :] = 0x7F
    A[1, :] = 0x81            # -maxpos: wraps the other way
    B[:, 0] = 0x7F
    B[:, 1] = 0x7F
    B[: K // 2, 1] = 0x7E      # half the products 2^23 units: a different multiple of 2^32 is dropped
    Ain, Bin = (np.ascontiguousarray(A.T) if ta else A), (np.ascontiguousarray(B.T) if tb else B)
    got = to_np(pn.posit_gemm(to_dev(Ain), to_dev(Bin), "p8", "p8", trans_a=ta, trans_b=tb), "p8")
    rows = (0, min(M, 4))
    want, ovf = fast.gemm(Ain, Bin, "p8", "p8", trans_a=ta, trans_b=tb, rows=rows)
    assert ovf >= 4, "the case must leave the quire range"
    _assert_equal(got[rows[0]:rows[1]], want[rows[0]:rows[1]], "wrapped quire, %s" % kernel)


@pytest.mark.parametrize("stride", [1, 2])
def test_p8_conv_bwd_weight_quire_wraps(stride):
    """The same through the convolution kernels (stride 1: operands rewritten first; stride 2: byte gather): the weight
    gradient of a filter sums N*OH*OW = 512 / 128 products of maxpos * maxpos and wraps."""
    d = dict(N=8, C=2, H=8 * stride, W=8 * stride, K=3, R=1, S=1, stride_h=stride, stride_w=stride)
    x = np.full((8, 2, 8 * stride, 8 * stride), 0x7F, dtype=np.uint8)
    dy = np.full((8, 3, 8, 8), 0x7F, dtype=np.uint8)
    dy[:, 1] = 0x81
    dy[:, 2, :, ::2] = 0x7E
    dw, db = pn.posit_conv2d_bwd_weight(to_dev(dy), to_dev(x), _desc(d), "p8", "p16", with_bias=True)
    wdw, wdb = fast.conv2d_bwd_weight(dy, x, d, "p8", "p16", with_bias=True)
    _assert_equal(to_np(dw, "p16"), wdw, "wrapped weight gradient")
    _assert_equal(to_np(db, "p16"), wdb, "bias gradient")
    # 512 products of 2^24 units are 2^33 = 0 modulo 2^32: the first filter's gradient is exactly zero
    assert (wdw[0] == 0).all() and (wdw[1] == 0).all()


def test_gemm_is_deterministic():
    rng = np.random.default_rng(77)
    A = to_dev(rand_patterns(rng, (300, 500), "p16"))
    B = to_dev(rand_patterns(rng, (500, 200), "p16"))
    c1 = pn.posit_gemm(A, B, "p16", "p16").cpu()
    c2 = pn.posit_gemm(A, B, "p16", "p16").cpu()
    assert torch.equal(c1.view(torch.int16), c2.view(torch.int16))


# ---------------- convolution ----------------

CONV_CASES = [
    dict(N=2, C=3, H=9, W=7, K=5, R=3, S=3, pad_h=1, pad_w=1),
    dict(N=3, C=2, H=11, W=10, K=4, R=5, S=2, pad_h=2, pad_w=0, stride_h=2, stride_w=1),
    dict(N=2, C=1, H=8, W=8, K=3, R=2, S=3, pad_h=0, pad_w=2, stride_h=1, stride_w=2),
    dict(N=4, C=6, H=14, W=14, K=16, R=5, S=5),           # LeNet conv2 shape, small batch
    dict(N=2, C=32, H=16, W=16, K=32, R=3, S=3, pad_h=1, pad_w=1),
    dict(N=1, C=4, H=5, W=5, K=7, R=1, S=1),
    # output widths that are multiples of 8: the image operands are fetched as 8-byte runs trimmed at the borders
    dict(N=2, C=3, H=8, W=16, K=5, R=3, S=3, pad_h=1, pad_w=1),
    dict(N=3, C=2, H=12, W=8, K=4, R=5, S=5, pad_h=2, pad_w=2),
    dict(N=2, C=4, H=6, W=24, K=9, R=1, S=1),
    dict(N=1, C=2, H=10, W=18, K=3, R=3, S=3),
    dict(N=2, C=2, H=9, W=16, K=3, R=3, S=1, pad_h=1, stride_h=2),
    dict(N=5, C=3, H=16, W=16, K=70, R=3, S=3, pad_h=1, pad_w=1),   # more than one column tile
]


def _desc(d):
    return pn.ConvDesc(d["N"], d["C"], d["H"], d["W"], d["K"], d["R"], d["S"], d.get("pad_h", 0), d.get("pad_w", 0),
                       d.get("stride_h", 1), d.get("stride_w", 1))


@pytest.mark.parametrize("ci", range(len(CONV_CASES)))
@pytest.mark.parametrize("fin,fout", [("p8", "p8"), ("p8", "p16"), ("p16", "p16"), ("p32", "p32")])
def test_conv_all_three_passes(ci, fin, fout):
    d = CONV_CASES[ci]
    rng = np.random.default_rng(ci * 10 + BITS[fin])
    oh, ow = fast.out_hw(d)
    x = rand_patterns(rng, (d["N"], d["C"], d["H"], d["W"]), fin, special=0.005)
    w = rand_patterns(rng, (d["K"], d["C"], d["R"], d["S"]), fin, special=0.005)
    dy = rand_patterns(rng, (d["N"], d["K"], oh, ow), fin, special=0.005)
    bias = rand_patterns(rng, (d["K"],), fin, allow_nar=False)
    desc = _desc(d)
    y = pn.posit_conv2d_fwd(to_dev(x), to_dev(w), desc, fin, fout, bias=to_dev(bias))
    _assert_equal(to_np(y, fout), fast.conv2d_fwd(x, w, d, fin, fout, bias=bias), "conv fwd")
    dx = pn.posit_conv2d_bwd_data(to_dev(dy), to_dev(w), desc, fin, fout)
    _assert_equal(to_np(dx, fout), fast.conv2d_bwd_data(dy, w, d, fin, fout), "conv bwd_data")
    dw, db = pn.posit_conv2d_bwd_weight(to_dev(dy), to_dev(x), desc, fin, fout, with_bias=True)
    wdw, wdb = fast.conv2d_bwd_weight(dy, x, d, fin, fout, with_bias=True)
    _assert_equal(to_np(dw, fout), wdw, "conv bwd_weight")
    _assert_equal(to_np(db, fout), wdb, "conv dbias")


@pytest.mark.parametrize("geom", [dict(N=37, C=8, H=33, W=33, K=16, R=3, S=3, pad_h=1, pad_w=1),
                                  dict(N=29, C=6, H=30, W=40, K=27, R=3, S=3, pad_h=1, pad_w=1)])
def test_p8_conv_many_rows_few_channels(geom):
    """Tens of thousands of output positions and at most 32 channels: the 128 x 32 tile (four waves per SIMD instead of
    two), ragged in rows and columns, through the byte-gather kernel (width 33) and the pre-decoded one (width 40)."""
    d = geom
    rng = np.random.default_rng(d["W"])
    oh, ow = fast.out_hw(d)
    x = rand_patterns(rng, (d["N"], d["C"], d["H"], d["W"]), "p8", special=0.001)
    w = rand_patterns(rng, (d["K"], d["C"], d["R"], d["S"]), "p8", special=0.001, allow_nar=False)
    dy = rand_patterns(rng, (d["N"], d["K"], oh, ow), "p8", special=0.001)
    bias = rand_patterns(rng, (d["K"],), "p8", allow_nar=False)
    desc = _desc(d)
    y = pn.posit_conv2d_fwd(to_dev(x), to_dev(w), desc, "p8", "p8", bias=to_dev(bias))
    _assert_equal(to_np(y, "p8"), fast.conv2d_fwd(x, w, d, "p8", "p8", bias=bias), "conv fwd")
    dx = pn.posit_conv2d_bwd_data(to_dev(dy), to_dev(w), desc, "p8", "p8")
    _assert_equal(to_np(dx, "p8"), fast.conv2d_bwd_data(dy, w, d, "p8", "p8"), "conv bwd_data")
    dw, db = pn.posit_conv2d_bwd_weight(to_dev(dy), to_dev(x), desc, "p8", "p16", with_bias=True)
    wdw, wdb = fast.conv2d_bwd_weight(dy, x, d, "p8", "p16", with_bias=True)
    _assert_equal(to_np(dw, "p16"), wdw, "conv bwd_weight")
    _assert_equal(to_np(db, "p16"), wdb, "conv bias gradient")


@pytest.mark.parametrize("geom,fout", [(dict(N=10, C=20, H=31, W=33, K=40, R=3, S=3, pad_h=1, pad_w=1), "p8"),
                                       (dict(N=17, C=8, H=64, W=64, K=40, R=3, S=3, pad_h=1, pad_w=1), "p8"),
                                       (dict(N=8, C=24, H=20, W=52, K=72, R=2, S=3, pad_h=1, pad_w=1), "p16"),
                                       (dict(N=13, C=16, H=30, W=30, K=32, R=5, S=5, pad_h=0, pad_w=0), "p32"),
                                       (dict(N=9, C=33, H=32, W=32, K=64, R=3, S=3, pad_h=2, pad_w=0), "p8"),
                                       (dict(N=16, C=16, H=32, W=32, K=80, R=3, S=3, pad_h=1, pad_w=1), "p8")])
def test_p8_conv_on_the_integer_matrix_cores(geom, fout):
    """Unit-stride posit<8,0> forward and backward-data convolutions of 2^26 products and more (8192 output positions,
    16 output channels) run as implicit matrix products on the integer matrix cores: the input rewritten as int8 digit
    planes pixel-major in groups of 16 channels, gathered tap by tap.  Channel counts that do not fill a group, 32 x 128,
    64 x 64, 64 x 128 and (last case: 80 output channels over 16384 positions) 128 x 64 tiles, ragged position counts, filters 2 x 3 and 5 x 5, no padding and padding beyond the
    filter's half, NaR in the input (every output whose window holds it), a NaR weight (forward: its whole output
    channel, padding counts as an operand; backward-data: the positions its tap reaches), a NaR bias.  Backward-weight
    runs there too, as a matrix product over unfolded digit planes with the positions cut into slices."""
    d = geom
    rng = np.random.default_rng(d["C"] * 7 + d["K"])
    oh, ow = fast.out_hw(d)
    x = rand_patterns(rng, (d["N"], d["C"], d["H"], d["W"]), "p8", special=0.0005)
    w = rand_patterns(rng, (d["K"], d["C"], d["R"], d["S"]), "p8", special=0.001, allow_nar=False)
    dy = rand_patterns(rng, (d["N"], d["K"], oh, ow), "p8", special=0.0005)
    bias = rand_patterns(rng, (d["K"],), "p8", allow_nar=False)
    desc = _desc(d)
    assert pn.posit_conv2d_workspace(0, "p8", fout, desc) >= 2 * x.size  # the digit planes of the input
    y = pn.posit_conv2d_fwd(to_dev(x), to_dev(w), desc, "p8", fout, bias=to_dev(bias))
    _assert_equal(to_np(y, fout), fast.conv2d_fwd(x, w, d, "p8", fout, bias=bias), "conv fwd")
    dx = pn.posit_conv2d_bwd_data(to_dev(dy), to_dev(w), desc, "p8", fout)
    _assert_equal(to_np(dx, fout), fast.conv2d_bwd_data(dy, w, d, "p8", fout), "conv bwd_data")
    # backward-weight: the positions are the reduction, cut into slices; dy and the unfolded input as digit planes
    # (every output sums over all positions: one NaR each in dy and x, or nothing but NaR would come out)
    dyw, xw = dy.copy(), x.copy()
    dyw[dyw == 0x80] = 0x41
    xw[xw == 0x80] = 0xC3
    dyw[0, 3, 1, 1] = 0x80
    xw[1, 2, 5, 5] = 0x80
    dw, db = pn.posit_conv2d_bwd_weight(to_dev(dyw), to_dev(xw), desc, "p8", "p16", with_bias=True)
    wdw, wdb = fast.conv2d_bwd_weight(dyw, xw, d, "p8", "p16", with_bias=True)
    _assert_equal(to_np(dw, "p16"), wdw, "conv bwd_weight")
    _assert_equal(to_np(db, "p16"), wdb, "conv bias gradient")
    assert (wdw[3] == 0x8000).all() and (wdw[:, 2] == 0x8000).any() and not (wdw[4] == 0x8000).all()
    # NaR among the weights and in the bias
    w2, b2 = w.copy(), bias.copy()
    w2[1, d["C"] - 1, d["R"] - 1, 0] = 0x80
    w2[d["K"] - 1, 0, 0, d["S"] - 1] = 0x80
    b2[2] = 0x80
    y2 = to_np(pn.posit_conv2d_fwd(to_dev(x), to_dev(w2), desc, "p8", fout, bias=to_dev(b2)), fout)
    _assert_equal(y2, fast.conv2d_fwd(x, w2, d, "p8", fout, bias=b2), "conv fwd, NaR weights")
    onar = 1 << (BITS[fout] - 1)
    assert (y2[:, 1] == onar).all() and (y2[:, 2] == onar).all() and (y2[:, d["K"] - 1] == onar).all()
    dx2 = pn.posit_conv2d_bwd_data(to_dev(dy), to_dev(w2), desc, "p8", fout)
    _assert_equal(to_np(dx2, fout), fast.conv2d_bwd_data(dy, w2, d, "p8", fout), "conv bwd_data, NaR weights")


@pytest.mark.parametrize("geom", [dict(N=64, C=1, H=28, W=28, K=6, R=5, S=5, pad_h=2, pad_w=2),
                                  dict(N=64, C=6, H=14, W=14, K=16, R=5, S=5),
                                  dict(N=40, C=16, H=15, W=15, K=5, R=3, S=3, pad_h=1, pad_w=1)])
def test_p8_conv_matrix_cores_small_layers(geom):
    """The LeNet-5-shaped layers and one more with 5 output channels: a few million products, 4 to 16 channels.  Backward-weight
    runs on the matrix cores from 2^22 products and 4 output channels on (most of a 64-row tile is padding: the launches, not
    the multiplies, set the time), backward-data and forward from 2^24 products, 4 output and 8 input channels on."""
    d = geom
    rng = np.random.default_rng(d["C"] * 31 + d["K"])
    oh, ow = fast.out_hw(d)
    x = rand_patterns(rng, (d["N"], d["C"], d["H"], d["W"]), "p8", special=0.0002)
    w = rand_patterns(rng, (d["K"], d["C"], d["R"], d["S"]), "p8", special=0.001, allow_nar=False)
    dy = rand_patterns(rng, (d["N"], d["K"], oh, ow), "p8", special=0.0002)
    bias = rand_patterns(rng, (d["K"],), "p8", allow_nar=False)
    desc = _desc(d)
    fo = "p32" if d["K"] == 5 else "p8"   # the 32-bit container through the tile-in-LDS epilogue as well
    y = pn.posit_conv2d_fwd(to_dev(x), to_dev(w), desc, "p8", fo, bias=to_dev(bias))
    _assert_equal(to_np(y, fo), fast.conv2d_fwd(x, w, d, "p8", fo, bias=bias), "conv fwd")
    dx = pn.posit_conv2d_bwd_data(to_dev(dy), to_dev(w), desc, "p8", fo)
    _assert_equal(to_np(dx, fo), fast.conv2d_bwd_data(dy, w, d, "p8", fo), "conv bwd_data")
    dyw, xw = dy.copy(), x.copy()
    dyw[dyw == 0x80] = 0x3F
    xw[xw == 0x80] = 0xC1
    dyw[3, d["K"] - 1, 0, ow - 1] = 0x80
    xw[d["N"] - 1, 0, d["H"] - 1, 1] = 0x80
    dw, db = pn.posit_conv2d_bwd_weight(to_dev(dyw), to_dev(xw), desc, "p8", "p16", with_bias=True)
    wdw, wdb = fast.conv2d_bwd_weight(dyw, xw, d, "p8", "p16", with_bias=True)
    _assert_equal(to_np(dw, "p16"), wdw, "conv bwd_weight")
    _assert_equal(to_np(db, "p16"), wdb, "conv bias gradient")


@pytest.mark.parametrize("seed", range(8))
def test_p8_conv_matrix_core_random_geometries(seed):
    """Random geometries large enough for the matrix-core convolutions (2^26 products, 8192 positions): filters 1 x 1 to
    5 x 4, padding from none to the filter size, odd channel and batch counts (groups of 16 partly filled), strides 1 and
    2 (at stride 2 only backward-weight runs there).  All three passes against the oracle, bias and bias gradient included."""
    rng = np.random.default_rng(1000 + seed)
    while True:
        R, S = int(rng.integers(1, 6)), int(rng.integers(1, 5))
        d = dict(C=int(rng.integers(8, 41)), K=int(rng.integers(16, 81)), H=int(rng.integers(12, 41)), W=int(rng.integers(12, 41)), R=R, S=S,
                 pad_h=int(rng.integers(0, R + 1)), pad_w=int(rng.integers(0, S + 1)))
        if seed % 4 == 3:
            d["stride_h"], d["stride_w"] = 2, int(rng.integers(1, 3))
        d["N"] = 1
        oh, ow = fast.out_hw(d)
        if oh < 1 or ow < 1:
            continue
        need = max(-(-8192 // (oh * ow)), -(-(1 << 26) // (oh * ow * d["K"] * d["C"] * R * S)))
        d["N"] = need + int(rng.integers(0, 3))
        if d["N"] <= 96 and d["N"] * oh * ow * d["K"] * d["C"] * R * S < 3 << 27:
            break
    x = rand_patterns(rng, (d["N"], d["C"], d["H"], d["W"]), "p8", special=0.0002)
    w = rand_patterns(rng, (d["K"], d["C"], d["R"], d["S"]), "p8", special=0.001, allow_nar=False)
    dy = rand_patterns(rng, (d["N"], d["K"], oh, ow), "p8", special=0.0002)
    bias = rand_patterns(rng, (d["K"],), "p8", allow_nar=False)
    desc = _desc(d)
    y = pn.posit_conv2d_fwd(to_dev(x), to_dev(w), desc, "p8", "p8", bias=to_dev(bias))
    _assert_equal(to_np(y, "p8"), fast.conv2d_fwd(x, w, d, "p8", "p8", bias=bias), "conv fwd %r" % d)
    dx = pn.posit_conv2d_bwd_data(to_dev(dy), to_dev(w), desc, "p8", "p16")
    _assert_equal(to_np(dx, "p16"), fast.conv2d_bwd_data(dy, w, d, "p8", "p16"), "conv bwd_data %r" % d)
    dyw, xw = dy.copy(), x.copy()   # every output of this pass sums over all positions: keep a few NaR only
    dyw[dyw == 0x80] = 0x3F
    xw[xw == 0x80] = 0xC1
    dyw[d["N"] - 1, 1, oh - 1, 0] = 0x80
    xw[0, d["C"] - 1, d["H"] // 2, d["W"] // 2] = 0x80
    dw, db = pn.posit_conv2d_bwd_weight(to_dev(dyw), to_dev(xw), desc, "p8", "p16", with_bias=True)
    wdw, wdb = fast.conv2d_bwd_weight(dyw, xw, d, "p8", "p16", with_bias=True)
    _assert_equal(to_np(dw, "p16"), wdw, "conv bwd_weight %r" % d)
    _assert_equal(to_np(db, "p16"), wdb, "conv bias gradient %r" % d)
    dw2 = pn.posit_conv2d_bwd_weight(to_dev(dyw), to_dev(xw), desc, "p8", "p8")   # without the bias gradient's column
    dw2 = dw2[0] if isinstance(dw2, tuple) else dw2
    _assert_equal(to_np(dw2, "p8"), fast.conv2d_bwd_weight(dyw, xw, d, "p8", "p8"), "conv bwd_weight, no bias gradient %r" % d)


@pytest.mark.parametrize("fin,fout", [("p8", "p8"), ("p8", "p16"), ("p8_2", "p8_2"), ("p8_1", "p12_2"), ("p16", "p16"), ("p12_2", "p8_2"), ("p32", "p32")])
@pytest.mark.parametrize("geom", ["unit stride (operands rewritten)", "pad beyond the filter (byte gather)", "strided (generic kernel)"])
def test_conv_bwd_data_nar_weight_reaches_only_its_taps_positions(fin, fout, geom):
    """One NaR weight at a corner tap: the input gradient is NaR exactly where that tap reaches an output position (the
    scatter of LibTorch's flow), not over the whole channel; through every kernel family that serves this pass, and
    through the chain without quire."""
    d = {"unit stride (operands rewritten)": dict(N=2, C=3, H=9, W=16, K=4, R=3, S=3, pad_h=1, pad_w=1),
         "pad beyond the filter (byte gather)": dict(N=2, C=3, H=7, W=9, K=4, R=2, S=3, pad_h=3, pad_w=0),
         "strided (generic kernel)": dict(N=2, C=3, H=11, W=10, K=4, R=3, S=2, pad_h=1, pad_w=0, stride_h=2, stride_w=3)}[geom]
    rng = np.random.default_rng(BITS[fin] * 5 + len(geom))
    oh, ow = fast.out_hw(d)
    w = rand_patterns(rng, (d["K"], d["C"], d["R"], d["S"]), fin, allow_nar=False)
    dy = rand_patterns(rng, (d["N"], d["K"], oh, ow), fin, allow_nar=False)
    w[1, 2, 0, 0] = 1 << (BITS[fin] - 1)
    w[3, 0, d["R"] - 1, d["S"] - 1] = 1 << (BITS[fin] - 1)
    desc = _desc(d)
    nar_out = 1 << (BITS[fout] - 1)
    want = fast.conv2d_bwd_data(dy, w, d, fin, fout)
    for c in (0, 2):  # the footprint is a proper, non-empty part of the channel; channel 1 holds no NaR at all
        assert (want[:, c] == nar_out).any() and not (want[:, c] == nar_out).all()
    assert not (want[:, 1] == nar_out).any()
    dx = pn.posit_conv2d_bwd_data(to_dev(dy), to_dev(w), desc, fin, fout)
    _assert_equal(to_np(dx, fout), want, "bwd_data with NaR weights")
    dxq = pn.posit_conv2d_bwd_data_noquire(to_dev(dy), to_dev(w), desc, fin, fout)
    _assert_equal(to_np(dxq, fout), fast.conv2d_bwd_data(dy, w, d, fin, fout, noquire=True), "bwd_data without quire, NaR weights")


def test_conv_bwd_weight_long_reduction_splits():
    d = dict(N=16, C=3, H=32, W=32, K=8, R=3, S=3, pad_h=1, pad_w=1)
    desc = _desc(d)
    assert pn.posit_conv2d_workspace(2, "p8", "p16", desc) > 0
    rng = np.random.default_rng(21)
    x = rand_patterns(rng, (16, 3, 32, 32), "p8", special=0.0)
    dy = rand_patterns(rng, (16, 8, 32, 32), "p8", special=0.0)
    dw, db = pn.posit_conv2d_bwd_weight(to_dev(dy), to_dev(x), desc, "p8", "p16", with_bias=True)
    wdw, wdb = fast.conv2d_bwd_weight(dy, x, d, "p8", "p16", with_bias=True)
    _assert_equal(to_np(dw, "p16"), wdw, "split bwd_weight")
    _assert_equal(to_np(db, "p16"), wdb, "split dbias")


@pytest.mark.parametrize("fin,fout", [("p8", "p8"), ("p8", "p16"), ("p16", "p16")])
def test_conv_empty_reductions(fin, fout):
    """No input channels: y is the rounded bias.  No images: dw and dbias are zero.  No output channels: dx is zero."""
    rng = np.random.default_rng(3)
    d = dict(N=2, C=0, H=8, W=8, K=3, R=3, S=3, pad_h=1, pad_w=1)
    x = np.zeros((2, 0, 8, 8), dtype=NP_DTYPE[fin])
    w = np.zeros((3, 0, 3, 3), dtype=NP_DTYPE[fin])
    bias = rand_patterns(rng, (3,), fin, allow_nar=False)
    y = pn.posit_conv2d_fwd(to_dev(x), to_dev(w), _desc(d), fin, fout, bias=to_dev(bias))
    _assert_equal(to_np(y, fout), fast.conv2d_fwd(x, w, d, fin, fout, bias=bias), "fwd without input channels")
    assert (to_np(y, fout)[:, 1] == fast.convert(bias[1:2], fin, fout)[0]).all()
    d = dict(N=0, C=2, H=8, W=8, K=3, R=3, S=3, pad_h=1, pad_w=1)
    dw, db = pn.posit_conv2d_bwd_weight(to_dev(np.zeros((0, 3, 8, 8), dtype=NP_DTYPE[fin])), to_dev(np.zeros((0, 2, 8, 8), dtype=NP_DTYPE[fin])),
                                        _desc(d), fin, fout, with_bias=True)
    assert not to_np(dw, fout).any() and not to_np(db, fout).any()
    d = dict(N=2, C=2, H=8, W=8, K=0, R=3, S=3, pad_h=1, pad_w=1)
    dx = pn.posit_conv2d_bwd_data(to_dev(np.zeros((2, 0, 8, 8), dtype=NP_DTYPE[fin])), to_dev(np.zeros((0, 2, 3, 3), dtype=NP_DTYPE[fin])),
                                  _desc(d), fin, fout)
    assert dx.shape == (2, 2, 8, 8) and not to_np(dx, fout).any()


def _random_geometries(count, seed):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        R, S = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        ph, pw = int(rng.integers(0, 4)), int(rng.integers(0, 4))
        H, W = int(rng.integers(1, 21)), int(rng.integers(1, 21))
        if H + 2 * ph < R or W + 2 * pw < S:
            continue
        unit = rng.random() < 0.75  # mostly unit stride: the pre-decoded path
        out.append(dict(N=int(rng.integers(1, 4)), C=int(rng.integers(1, 6)), H=H, W=W, K=int(rng.integers(1, 7)), R=R, S=S, pad_h=ph, pad_w=pw,
                        stride_h=1 if unit else int(rng.integers(1, 4)), stride_w=1 if unit else int(rng.integers(1, 4))))
    return out


@pytest.mark.parametrize("gi", range(40))
def test_conv_random_geometries_posit8(gi):
    """Seeded random shapes, pads larger than the filter allows for a border, one-pixel images, widths of every
    residue modulo 8: all three passes and the bias gradient of the posit<8,0> paths."""
    d = _random_geometries(40, 2105)[gi]
    rng = np.random.default_rng(1000 + gi)
    oh, ow = fast.out_hw(d)
    fout = "p8" if gi % 2 else "p16"
    x = rand_patterns(rng, (d["N"], d["C"], d["H"], d["W"]), "p8", special=0.01)
    w = rand_patterns(rng, (d["K"], d["C"], d["R"], d["S"]), "p8", special=0.01, allow_nar=gi % 3 == 0)
    dy = rand_patterns(rng, (d["N"], d["K"], oh, ow), "p8", special=0.01)
    bias = rand_patterns(rng, (d["K"],), "p8", allow_nar=False)
    desc = _desc(d)
    y = pn.posit_conv2d_fwd(to_dev(x), to_dev(w), desc, "p8", fout, bias=to_dev(bias))
    _assert_equal(to_np(y, fout), fast.conv2d_fwd(x, w, d, "p8", fout, bias=bias), "fwd %s" % d)
    dx = pn.posit_conv2d_bwd_data(to_dev(dy), to_dev(w), desc, "p8", fout)
    _assert_equal(to_np(dx, fout), fast.conv2d_bwd_data(dy, w, d, "p8", fout), "bwd_data %s" % d)
    dw, db = pn.posit_conv2d_bwd_weight(to_dev(dy), to_dev(x), desc, "p8", fout, with_bias=True)
    wdw, wdb = fast.conv2d_bwd_weight(dy, x, d, "p8", fout, with_bias=True)
    _assert_equal(to_np(dw, fout), wdw, "bwd_weight %s" % d)
    _assert_equal(to_np(db, fout), wdb, "dbias %s" % d)


@pytest.mark.parametrize("gi", range(24))
def test_conv_random_geometries_posit8_es(gi):
    """The same seeded random shapes through the byte-gather kernel of posit(8,1) / posit(8,2) (every tile
    variant, every gather mode, strided backward-data falling back to the generic kernel)."""
    d = _random_geometries(40, 2105)[gi + 8]
    rng = np.random.default_rng(3000 + gi)
    oh, ow = fast.out_hw(d)
    fin = "p8_2" if gi % 2 else "p8_1"
    fout = [fin, "p12_2", "p16"][gi % 3]
    x = rand_patterns(rng, (d["N"], d["C"], d["H"], d["W"]), fin, special=0.01)
    w = rand_patterns(rng, (d["K"], d["C"], d["R"], d["S"]), fin, special=0.01, allow_nar=gi % 3 == 0)
    dy = rand_patterns(rng, (d["N"], d["K"], oh, ow), fin, special=0.01)
    bias = rand_patterns(rng, (d["K"],), fin, allow_nar=False)
    desc = _desc(d)
    y = pn.posit_conv2d_fwd(to_dev(x), to_dev(w), desc, fin, fout, bias=to_dev(bias))
    _assert_equal(to_np(y, fout), fast.conv2d_fwd(x, w, d, fin, fout, bias=bias), "fwd %s" % d)
    dx = pn.posit_conv2d_bwd_data(to_dev(dy), to_dev(w), desc, fin, fout)
    _assert_equal(to_np(dx, fout), fast.conv2d_bwd_data(dy, w, d, fin, fout), "bwd_data %s" % d)
    dw, db = pn.posit_conv2d_bwd_weight(to_dev(dy), to_dev(x), desc, fin, fout, with_bias=True)
    wdw, wdb = fast.conv2d_bwd_weight(dy, x, d, fin, fout, with_bias=True)
    _assert_equal(to_np(dw, fout), wdw, "bwd_weight %s" % d)
    _assert_equal(to_np(db, fout), wdb, "dbias %s" % d)


@pytest.mark.parametrize("fin,fout", [("p8", "p16"), ("p16", "p16"), ("p8_2", "p12_2"), ("p32", "p32")])
def test_bias_gradient_over_batch_slices(fin, fout):
    """Enough images that the bias-gradient reduction is cut into slices of the batch and merged;
    one channel carries a NaR, one sums to a large value."""
    d = dict(N=24, C=1, H=32, W=32, K=3, R=1, S=1)
    desc = _desc(d)
    rng = np.random.default_rng(BITS[fin] + 77)
    x = rand_patterns(rng, (24, 1, 32, 32), fin, special=0.0, allow_nar=False)
    dy = rand_patterns(rng, (24, 3, 32, 32), fin, special=0.0, allow_nar=False)
    dy[17, 1, 5, 9] = 1 << (BITS[fin] - 1)
    dy[:, 2] = (1 << (BITS[fin] - 2)) + 3  # all slightly above one: the sum is about N * OH * OW
    dw, db = pn.posit_conv2d_bwd_weight(to_dev(dy), to_dev(x), desc, fin, fout, with_bias=True)
    wdw, wdb = fast.conv2d_bwd_weight(dy, x, d, fin, fout, with_bias=True)
    _assert_equal(to_np(db, fout), wdb, "sliced dbias")
    _assert_equal(to_np(dw, fout), wdw, "bwd_weight")


# ---------------- layer glue ----------------

@pytest.mark.parametrize("fmt", ["p8", "p16", "p32"])
def test_relu_forward_backward(fmt):
    rng = np.random.default_rng(BITS[fmt])
    n = 30001
    x = rand_patterns(rng, n, fmt, special=0.05)
    y = to_np(pn.posit_relu(to_dev(x), fmt), fmt)
    _assert_equal(y, np.array(po.relu(x.tolist(), PF[fmt])), "relu")
    dy = rand_patterns(rng, n, "p16")
    dx = to_np(pn.posit_relu_bwd(to_dev(y), to_dev(dy), fmt, "p16"), "p16")
    _assert_equal(dx, np.array(po.relu_bwd(y.tolist(), dy.tolist(), PF[fmt], po.P16)), "relu bwd")


@pytest.mark.parametrize("fmt", ["p8", "p16", "p32"])
@pytest.mark.parametrize("kh,kw,W", [(2, 2, 10), (3, 2, 10), (2, 2, 12), (3, 4, 12), (2, 3, 12)])
def test_maxpool_forward_backward(fmt, kh, kw, W):
    """Width 10: one element per thread; width 12: the backward kernel that handles four elements of a row per thread."""
    rng = np.random.default_rng(kh + kw + BITS[fmt])
    planes, H = 14, 12
    x = rand_patterns(rng, (2, 7, H, W), fmt, special=0.1)
    y, idx = pn.posit_maxpool2d_fwd(to_dev(x), fmt, kh, kw)
    wy, widx = po.maxpool2d_fwd(x.flatten().tolist(), planes, H, W, kh, kw, PF[fmt])
    _assert_equal(to_np(y, fmt).flatten(), np.array(wy), "maxpool fwd")
    _assert_equal(idx.cpu().numpy().flatten(), np.array(widx), "maxpool idx")
    dy = rand_patterns(rng, tuple(y.shape), fmt)
    dx = pn.posit_maxpool2d_bwd(to_dev(dy), idx, fmt, kh, kw)
    _assert_equal(to_np(dx, fmt).flatten(), np.array(po.maxpool2d_bwd(dy.flatten().tolist(), widx, planes, H, W, kh, kw)), "maxpool bwd")


@pytest.mark.parametrize("fin,fout", [("p8", "p8"), ("p16", "p8"), ("p8", "p16"), ("p32", "p32")])
def test_avgpool_forward_backward(fin, fout):
    rng = np.random.default_rng(BITS[fin] + 3 * BITS[fout])
    planes, H, W, kh, kw = 6, 8, 12, 2, 2
    x = rand_patterns(rng, (planes, H, W), fin, special=0.05)
    y = pn.posit_avgpool2d_fwd(to_dev(x), fin, fout, kh, kw)
    _assert_equal(to_np(y, fout).flatten(), np.array(po.avgpool2d_fwd(x.flatten().tolist(), planes, H, W, kh, kw, PF[fin], PF[fout])), "avgpool fwd")
    dy = rand_patterns(rng, (planes, H // kh, W // kw), fin, special=0.05)
    dx = pn.posit_avgpool2d_bwd(to_dev(dy), fin, fout, kh, kw)
    _assert_equal(to_np(dx, fout).flatten(), np.array(po.avgpool2d_bwd(dy.flatten().tolist(), planes, H, W, kh, kw, PF[fin], PF[fout])), "avgpool bwd")


# ---------------- the formats of the paper's experiments outside Table 1 (Sec. 4: posit<8..12, 1..2>) ----------------

@pytest.mark.parametrize("fmt", GENERAL)
def test_general_formats_round_convert(fmt):
    rng = np.random.default_rng(BITS[fmt] * 3 + len(fmt))
    n = 60001
    x = (rng.standard_normal(n) * np.exp2(rng.uniform(-60, 60, n))).astype(np.float32)
    x[:5] = [0.0, -0.0, np.inf, np.nan, 1e-45]
    _assert_equal(to_np(pn.posit_round(to_dev(x), fmt), fmt), fast.round_from_float(x, fmt), "round f32->" + fmt)
    x64 = rng.standard_normal(n) * np.exp2(rng.uniform(-300, 300, n))
    _assert_equal(to_np(pn.posit_round(to_dev(x64), fmt), fmt), fast.round_from_float(x64, fmt), "round f64->" + fmt)
    pats = np.arange(1 << BITS[fmt], dtype=np.uint32).astype(NP_DTYPE[fmt])
    for dst in GENERAL + ["p8", "p16", "p32"]:
        _assert_equal(to_np(pn.posit_convert(to_dev(pats), fmt, dst), dst), fast.convert(pats, fmt, dst), "convert %s->%s" % (fmt, dst))
    for src in ("p16", "p32"):
        sp = rand_patterns(rng, 100001, src)
        _assert_equal(to_np(pn.posit_convert(to_dev(sp), src, fmt), fmt), fast.convert(sp, src, fmt), "convert %s->%s" % (src, fmt))
    for dst in ("f32", "f64"):
        got = pn.posit_convert(to_dev(pats), fmt, dst).cpu().numpy()
        want = fast.to_float(pats, fmt, dst)
        nan = np.isnan(want)
        assert np.array_equal(np.isnan(got), nan) and np.array_equal(got[~nan], want[~nan])


@pytest.mark.parametrize("fx,fy,fc", [("p12_2", "p12_2", "p8_2"), ("p8_2", "p12_2", None), ("p8_2", "p8_2", None), ("p10_1", "p12_1", "p8_1"),
                                      ("p8_1", "p10_2", "p8"), ("p16", "p12_2", "p10_2"), ("p12_1", "p16", "p12_1")])
def test_general_formats_axpy(fx, fy, fc):
    test_axpy(fx, fy, fc)


GENERAL_GEMM_CASES = [
    ("p8_1", "p8_1", 70, 130, 100, 0, 0, 1, 1),
    ("p8_2", "p8_2", 65, 63, 129, 1, 0, 0, 1),
    ("p8_2", "p12_2", 130, 70, 300, 0, 1, 1, 0),
    ("p10_1", "p10_1", 33, 129, 257, 1, 1, 1, 1),
    ("p10_2", "p10_2", 64, 64, 200, 0, 0, 0, 1),
    ("p12_1", "p12_1", 100, 50, 96, 0, 0, 1, 0),
    ("p12_2", "p12_2", 130, 70, 100, 0, 0, 1, 1),
    ("p12_2", "p8_2", 20, 33, 64, 0, 1, 0, 0),
    ("p16", "p12_2", 40, 35, 50, 0, 0, 1, 1),
    ("p8", "p10_1", 150, 140, 70, 0, 0, 0, 1),   # posit<8,0> packed-dot kernel, general output format
    ("p8_1", "p32", 17, 5, 31, 1, 1, 0, 0),
    # beyond the small-problem kernel of the 8-bit formats: the tiled byte-gather kernel, all four transposition cases
    ("p8_2", "p8_2", 300, 260, 900, 1, 1, 1, 1),
    ("p8_2", "p12_2", 270, 300, 333, 0, 0, 1, 1),
    ("p8_1", "p16", 520, 130, 700, 0, 1, 1, 1),
    ("p8_1", "p8_1", 129, 520, 519, 1, 0, 0, 1),
]


@pytest.mark.parametrize("fin,fout,M,N,K,ta,tb,use_bias,nar", GENERAL_GEMM_CASES)
def test_general_formats_gemm(fin, fout, M, N, K, ta, tb, use_bias, nar):
    test_gemm_random_patterns(fin, fout, M, N, K, ta, tb, use_bias, nar)


@pytest.mark.parametrize("fin,fout,M,N,K", [("p8_2", "p12_2", 32, 96, 8192), ("p12_2", "p12_2", 16, 50, 4096), ("p10_1", "p10_1", 24, 40, 4096),
                                            ("p8_1", "p8_1", 8, 24, 70000), ("p8_2", "p12_2", 64, 288, 8192), ("p8_1", "p8_1", 40, 70, 70000)])
def test_general_formats_gemm_split_reduction(fin, fout, M, N, K):
    """Long reductions take the split-K path (the smallest 8-bit problems split over the threads of an output
    instead, without workspace); posit<8,1> with maxpos operands in one row wraps its 64-bit quire."""
    rng = np.random.default_rng(K + M)
    A = rand_patterns(rng, (M, K), fin, special=0.0, allow_nar=False)
    B = rand_patterns(rng, (K, N), fin, special=0.0, allow_nar=False)
    if fin == "p8_1":
        A[0, :] = 0x7F
        B[:, 0] = 0x7F
    small8 = BITS[fin] == 8 and M * N <= 65536 and M * N * K <= 1 << 26
    assert (pn.posit_gemm_workspace(fin, fout, False, False, M, N, K) > 0) != small8
    got = pn.posit_gemm(to_dev(A), to_dev(B), fin, fout)
    want, ovf = fast.gemm(A, B, fin, fout)
    if fin == "p8_1":
        assert ovf >= 1
    _assert_equal(to_np(got, fout), want, "split gemm %s" % fin)


@pytest.mark.parametrize("ci", [0, 1, 3])
@pytest.mark.parametrize("fin,fout", [("p8_2", "p8_2"), ("p8_2", "p12_2"), ("p12_2", "p12_2"), ("p10_1", "p10_1"), ("p8_1", "p12_1"), ("p10_2", "p8_2")])
def test_general_formats_conv(ci, fin, fout):
    test_conv_all_three_passes(ci, fin, fout)


@pytest.mark.parametrize("fmt", GENERAL)
def test_general_formats_glue(fmt):
    rng = np.random.default_rng(BITS[fmt] + len(fmt))
    n = 20001
    x = rand_patterns(rng, n, fmt, special=0.05)
    y = to_np(pn.posit_relu(to_dev(x), fmt), fmt)
    _assert_equal(y, np.array(po.relu(x.tolist(), PF[fmt])), "relu")
    dy = rand_patterns(rng, n, "p12_2")
    dx = to_np(pn.posit_relu_bwd(to_dev(y), to_dev(dy), fmt, "p12_2"), "p12_2")
    _assert_equal(dx, np.array(po.relu_bwd(y.tolist(), dy.tolist(), PF[fmt], po.FORMATS["p12_2"])), "relu bwd")
    planes, H, W = 6, 12, 10
    for kh, kw in ((2, 2), (3, 2)):
        xp = rand_patterns(rng, (planes, H, W), fmt, special=0.1)
        yp, idx = pn.posit_maxpool2d_fwd(to_dev(xp), fmt, kh, kw)
        wy, widx = po.maxpool2d_fwd(xp.flatten().tolist(), planes, H, W, kh, kw, PF[fmt])
        _assert_equal(to_np(yp, fmt).flatten(), np.array(wy), "maxpool fwd")
        _assert_equal(idx.cpu().numpy().flatten(), np.array(widx), "maxpool idx")
        dyp = rand_patterns(rng, tuple(yp.shape), fmt)
        dxp = pn.posit_maxpool2d_bwd(to_dev(dyp), idx, fmt, kh, kw)
        _assert_equal(to_np(dxp, fmt).flatten(), np.array(po.maxpool2d_bwd(dyp.flatten().tolist(), widx, planes, H, W, kh, kw)), "maxpool bwd")
    for fout, (kh, kw) in ((fmt, (2, 2)), ("p12_2", (2, 4)), ("p8", (2, 2))):
        xp = rand_patterns(rng, (planes, 8, 12), fmt, special=0.05)
        ya = pn.posit_avgpool2d_fwd(to_dev(xp), fmt, fout, kh, kw)
        _assert_equal(to_np(ya, fout).flatten(), np.array(po.avgpool2d_fwd(xp.flatten().tolist(), planes, 8, 12, kh, kw, PF[fmt], PF[fout])), "avgpool fwd")
        dya = rand_patterns(rng, (planes, 8 // kh, 12 // kw), fmt, special=0.05)
        dxa = pn.posit_avgpool2d_bwd(to_dev(dya), fmt, fout, kh, kw)
        _assert_equal(to_np(dxa, fout).flatten(), np.array(po.avgpool2d_bwd(dya.flatten().tolist(), planes, 8, 12, kh, kw, PF[fmt], PF[fout])), "avgpool bwd")


# ---------------- accumulation without the quire (Sec. 3.3 option; Table 2) ----------------

NOQUIRE_GEMM_CASES = [
    ("p8", "p8", 70, 130, 100, 0, 0, 1, 1),
    ("p8", "p16", 33, 40, 257, 1, 1, 1, 0),
    ("p16", "p16", 65, 63, 129, 1, 0, 1, 1),
    ("p16", "p8", 40, 35, 300, 0, 1, 0, 0),
    ("p32", "p32", 33, 31, 70, 0, 0, 1, 1),
    ("p8_2", "p8_2", 64, 64, 200, 0, 0, 1, 1),
    ("p8_2", "p12_2", 30, 70, 150, 0, 1, 0, 0),
    ("p10_1", "p10_1", 50, 20, 96, 0, 0, 1, 0),
    ("p12_1", "p12_1", 20, 50, 96, 1, 0, 0, 1),
    ("p12_2", "p8_2", 35, 33, 64, 0, 0, 1, 0),
    ("p8_1", "p8_1", 1, 1, 1, 0, 0, 0, 0),
    ("p10_2", "p16", 17, 5, 31, 1, 1, 0, 0),
]


@pytest.mark.parametrize("fin,fout,M,N,K,ta,tb,use_bias,nar", NOQUIRE_GEMM_CASES)
def test_noquire_gemm(fin, fout, M, N, K, ta, tb, use_bias, nar):
    rng = np.random.default_rng(M * 5 + N * 3 + K)
    A = rand_patterns(rng, (K, M) if ta else (M, K), fin, allow_nar=bool(nar), special=0.01)
    B = rand_patterns(rng, (N, K) if tb else (K, N), fin, allow_nar=bool(nar), special=0.01)
    bias = rand_patterns(rng, (N,), fin, allow_nar=bool(nar)) if use_bias else None
    got = pn.posit_gemm_noquire(to_dev(A), to_dev(B), fin, fout, trans_a=ta, trans_b=tb, bias=None if bias is None else to_dev(bias))
    want, _ = fast.gemm(A, B, fin, fout, trans_a=ta, trans_b=tb, bias=bias, noquire=True)
    _assert_equal(to_np(got, fout), want, "noquire gemm %s->%s %dx%dx%d" % (fin, fout, M, N, K))


def test_noquire_gemm_small_values_long_reduction_differs_from_quire():
    """Weights-times-activations-like data, K = 2048: the mode must follow the oracle term by term over a long
    chain (never split), and it does differ from the quire result."""
    A32, B32 = workloads.gemm_operands(2, 2048, sigma=0.1, extremes=False)
    A = fast.round_from_float(A32[:96], "p16")
    B = fast.round_from_float(B32[:, :80], "p16")
    got = to_np(pn.posit_gemm_noquire(to_dev(A), to_dev(B), "p16", "p16"), "p16")
    want, _ = fast.gemm(A, B, "p16", "p16", noquire=True)
    _assert_equal(got, want, "noquire gemm K=2048")
    quire, _ = fast.gemm(A, B, "p16", "p16")
    assert (quire != want).any()
    assert pn.posit_gemm_workspace("p16", "p16", False, False, 96, 80, 2048) > 0  # the quire path would split this reduction


@pytest.mark.parametrize("ci", [0, 1, 2, 3])
@pytest.mark.parametrize("fin,fout", [("p8", "p8"), ("p16", "p16"), ("p8_2", "p12_2"), ("p10_1", "p8_1"), ("p32", "p32")])
def test_noquire_conv_all_three_passes(ci, fin, fout):
    d = CONV_CASES[ci]
    rng = np.random.default_rng(ci * 10 + BITS[fin] + 1)
    oh, ow = fast.out_hw(d)
    x = rand_patterns(rng, (d["N"], d["C"], d["H"], d["W"]), fin, special=0.005)
    w = rand_patterns(rng, (d["K"], d["C"], d["R"], d["S"]), fin, special=0.005)
    dy = rand_patterns(rng, (d["N"], d["K"], oh, ow), fin, special=0.005)
    bias = rand_patterns(rng, (d["K"],), fin, allow_nar=False)
    desc = _desc(d)
    y = pn.posit_conv2d_fwd_noquire(to_dev(x), to_dev(w), desc, fin, fout, bias=to_dev(bias))
    _assert_equal(to_np(y, fout), fast.conv2d_fwd(x, w, d, fin, fout, bias=bias, noquire=True), "noquire conv fwd")
    dx = pn.posit_conv2d_bwd_data_noquire(to_dev(dy), to_dev(w), desc, fin, fout)
    _assert_equal(to_np(dx, fout), fast.conv2d_bwd_data(dy, w, d, fin, fout, noquire=True), "noquire conv bwd_data")
    dw, db = pn.posit_conv2d_bwd_weight_noquire(to_dev(dy), to_dev(x), desc, fin, fout, with_bias=True)
    wdw, wdb = fast.conv2d_bwd_weight(dy, x, d, fin, fout, with_bias=True, noquire=True)
    _assert_equal(to_np(dw, fout), wdw, "noquire conv bwd_weight")
    _assert_equal(to_np(db, fout), wdb, "noquire conv dbias")


@pytest.mark.parametrize("fin,fout,M,N,K", [("p8", "p8", 200, 300, 4096), ("p8", "p16", 40, 300, 8192), ("p16", "p16", 150, 200, 2048),
                                            ("p8_2", "p8_2", 150, 200, 4096), ("p8_1", "p16", 100, 200, 8192), ("p12_1", "p12_1", 70, 130, 2048),
                                            ("p32", "p32", 40, 70, 1024)])
def test_split_reduction_nar_flags_on_a_dirty_workspace(fin, fout, M, N, K):
    """A split reduction over several tile rows and columns, NaR patterns in a few rows of A and columns
    of B that only some slices of the reduction see, and a workspace full of ones: the flags of every
    slice are stored afresh by the kernels, nothing depends on what the workspace held."""
    need = pn.posit_gemm_workspace(fin, fout, False, False, M, N, K)
    assert need > 0
    rng = np.random.default_rng(M + N + K)
    A = rand_patterns(rng, (M, K), fin, special=0.001, allow_nar=False)
    B = rand_patterns(rng, (K, N), fin, special=0.001, allow_nar=False)
    nar = 1 << (BITS[fin] - 1)
    A[3, 7] = nar; A[M - 1, K - 1] = nar; A[M // 2, K // 2] = nar
    B[11, 5] = nar; B[K - 2, N - 1] = nar
    for fill in (0xFF, 0x00):
        ws = torch.full((need + 64,), fill, dtype=torch.uint8, device="cuda")
        got = pn.posit_gemm(to_dev(A), to_dev(B), fin, fout, workspace=ws)
        want, _ = fast.gemm(A, B, fin, fout)
        _assert_equal(to_np(got, fout), want, "split gemm with NaR, workspace filled with %#x" % fill)
    onar = 1 << (BITS[fout] - 1)
    assert (want[3] == onar).all() and (want[:, 5] == onar).all() and (want[:, N - 1] == onar).all()
    assert (want == onar).sum() == 3 * N + 2 * M - 6


@pytest.mark.parametrize("fin,fout", [("p8", "p16"), ("p8_2", "p12_2"), ("p16", "p16")])
def test_conv_bwd_weight_split_nar_on_a_dirty_workspace(fin, fout):
    """The backward-weight pass is computed transposed and splits its long reduction: NaR in dy (one
    output channel) and in x (the taps that read that pixel), workspace full of ones."""
    d = dict(N=16, C=5, H=20, W=20, K=70, R=3, S=3, pad_h=1, pad_w=1)
    desc = _desc(d)
    need = pn.posit_conv2d_workspace(2, fin, fout, desc)
    assert need > 0
    rng = np.random.default_rng(77)
    x = rand_patterns(rng, (16, 5, 20, 20), fin, special=0.0, allow_nar=False)
    dy = rand_patterns(rng, (16, 70, 20, 20), fin, special=0.0, allow_nar=False)
    nar = 1 << (BITS[fin] - 1)
    dy[9, 66, 4, 4] = nar
    x[2, 3, 0, 19] = nar
    ws = torch.full((need + 64,), 0xFF, dtype=torch.uint8, device="cuda")
    dw, db = pn.posit_conv2d_bwd_weight(to_dev(dy), to_dev(x), desc, fin, fout, with_bias=True, workspace=ws)
    wdw, wdb = fast.conv2d_bwd_weight(dy, x, d, fin, fout, with_bias=True)
    _assert_equal(to_np(dw, fout), wdw, "split bwd_weight with NaR")
    _assert_equal(to_np(db, fout), wdb, "dbias with NaR")
    onar = 1 << (BITS[fout] - 1)
    assert (wdw[66] == onar).all() and 0 < (wdw[0] == onar).sum() < wdw[0].size
