"""GPU parity of the kernels that gather products in fp64 buckets (formats of at most 16 bits other
than posit<8,0>) on inputs that use up the buckets' guard bits: see bucket_cases.  Expected values
come from the oracle only."""
import numpy as np
import pytest

import paper_2105_00053_amd as pn
from oracle import fast

import bucket_cases
from gpu_util import NP_DTYPE, mismatches, rand_patterns, to_dev, to_np

pytestmark = pytest.mark.gpu
BUCKETED = ["p16", "p8_1", "p8_2", "p10_1", "p10_2", "p12_1", "p12_2"]


def _assert_equal(got, want, what):
    bad = mismatches(got, want)
    assert len(bad) == 0, "%s: %d mismatches, first at %s: got %s want %s" % (
        what, len(bad), bad[0], np.asarray(got)[tuple(bad[0])], np.asarray(want)[tuple(bad[0])])


def _stack(fmt, cases):
    """Rows of A and columns of B from the cases, zero-padded at the end to one length."""
    K = max(len(a) for a, _, _ in cases)
    A = np.zeros((len(cases), K), dtype=NP_DTYPE[fmt])
    B = np.zeros((K, len(cases)), dtype=NP_DTYPE[fmt])
    for i, (a, b, _) in enumerate(cases):
        A[i, :len(a)] = a
        B[:len(b), i] = b
    return A, B


@pytest.mark.parametrize("fmt", BUCKETED)
def test_guard_filling_vectors_small_problem(fmt):
    """Few outputs, long reduction: the launch splits the reduction; every pairing of a case's row
    with a case's column is compared, the diagonal being the single surviving product."""
    cases = list(bucket_cases.guard_cases(fmt, mults=(1, 2, 4), leads=(0, 5, 16), max_len=140000))
    assert len(cases) >= 3
    A, B = _stack(fmt, cases)
    for fout in (fmt, "p32"):
        got = to_np(pn.posit_gemm(to_dev(A), to_dev(B), fmt, fout), fout)
        want, _ = fast.gemm(A, B, fmt, fout)
        _assert_equal(got, want, "guard cases %s->%s" % (fmt, fout))
        for i, (_, _, (sa, sb)) in enumerate(cases):
            one, _ = fast.gemm(np.array([[sa]], dtype=A.dtype), np.array([[sb]], dtype=A.dtype), fmt, fout, threads=1)
            assert got[i, i] == one[0, 0]


@pytest.mark.parametrize("fmt", BUCKETED)
def test_guard_filling_vectors_unsplit_long_reduction(fmt):
    """2048 x 2048 outputs, so that no workgroup shares its reduction: one workgroup runs through
    more than two flush intervals of the buckets.  The cases sit in the first rows and columns of
    random operands; the first rows of the result are compared in full."""
    B_, G, _, _ = bucket_cases.bucket_layout(fmt)
    rng = np.random.default_rng(G * 31 + B_)
    cases = list(bucket_cases.guard_cases(fmt, mults=(2,), leads=(0, 5), max_len=1 << 20))
    A_c, B_c = _stack(fmt, cases)
    nc, K = A_c.shape
    K += 37  # a ragged tail after the last case
    M = N = 2048
    # each workgroup runs through a long stretch of the reduction: the workspace holds the operands decoded once
    # (8 bytes per element, padded, plus bitmaps) and the partial quires of at most 8 slices, not of K / 2^G
    assert pn.posit_gemm_workspace(fmt, fmt, False, False, M, N, K) < 8.2 * (K + 64) * (M + N) + 8 * 25 * M * N
    reps = (K + 1023) // 1024  # a random block repeated along the reduction (cheap to generate at K = 2^18)
    A = np.ascontiguousarray(np.tile(rand_patterns(rng, (M, 1024), fmt, special=0.0, allow_nar=False), (1, reps))[:, :K])
    B = np.ascontiguousarray(np.tile(rand_patterns(rng, (1024, N), fmt, special=0.0, allow_nar=False), (reps, 1))[:K, :])
    A[:nc, :] = 0
    A[:nc, :K - 37] = A_c
    B[:, :nc] = 0
    B[:K - 37, :nc] = B_c
    rows = nc + 2
    got = to_np(pn.posit_gemm(to_dev(A), to_dev(B), fmt, fmt), fmt)
    want, _ = fast.gemm(A, B, fmt, fmt, rows=(0, rows))
    _assert_equal(got[:rows], want[:rows], "unsplit long reduction " + fmt)
    # the cases' columns against every row of a sample further down
    sample = np.array([rows, 777, 2047])
    want_s, _ = fast.gemm(A[sample], B[:, :nc], fmt, fmt)
    _assert_equal(got[sample][:, :nc], want_s, "case columns " + fmt)
