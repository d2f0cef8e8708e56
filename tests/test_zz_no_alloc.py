"""posit_gemm_static (the entry point for callers that cannot allocate): through the C ABI, against
posit_gemm with a caller's workspace, bit for bit, on calls in a row that share the library's one
scratch array -- each followed by a smaller problem, so stale contents of the array from the larger
call lie where the smaller one works."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2105_00053_amd as pn
from oracle import fast

from gpu_util import BITS, rand_patterns, to_dev, to_np

pytestmark = pytest.mark.gpu

TORCH = {"p8": torch.uint8, "p16": torch.int16, "p32": torch.int32, "p8_2": torch.uint8, "p12_2": torch.int16}
CODE = pn.binding.FORMAT_CODES


def _static_call(Ad, Bd, biasd, fin, fout, ta, tb, M, N, K):
    """Raw C-ABI call: no tensor is created between the argument set-up and the launch."""
    L = pn.load()
    out = torch.full((M, N), 0x55, dtype=TORCH[fout], device="cuda")
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    rc = L.posit_gemm_static(stream, CODE[fin], CODE[fout], ta, tb, M, N, K,
                             ctypes.c_void_p(Ad.data_ptr()), Ad.shape[1], ctypes.c_void_p(Bd.data_ptr()), Bd.shape[1],
                             ctypes.c_void_p(biasd.data_ptr()) if biasd is not None else None,
                             ctypes.c_void_p(out.data_ptr()), N)
    assert rc == 0, pn.load().posit_status_string(rc)
    return out


def _case(seed, fin, fout, M, N, K, ta, tb, use_bias, check_oracle):
    rng = np.random.default_rng(seed)
    A = rand_patterns(rng, (K, M) if ta else (M, K), fin, special=0.002)
    B = rand_patterns(rng, (N, K) if tb else (K, N), fin, special=0.002)
    # a few NaR patterns: rows / columns of NaR in the product, carried by the flags in the scratch array
    A[(3 % A.shape[0]), (5 % A.shape[1])] = 1 << (BITS[fin] - 1)
    bias = rand_patterns(rng, (N,), fin, allow_nar=False) if use_bias else None
    Ad, Bd = to_dev(A), to_dev(B)
    biasd = to_dev(bias) if use_bias else None
    need = pn.posit_gemm_workspace(fin, fout, ta, tb, M, N, K)
    assert 0 < need <= 72 << 20, "the case must use the scratch array"
    got = to_np(_static_call(Ad, Bd, biasd, fin, fout, ta, tb, M, N, K), fout)
    ws = torch.full((need,), 0xA5, dtype=torch.uint8, device="cuda")
    ref = to_np(pn.posit_gemm(Ad, Bd, fin, fout, trans_a=ta, trans_b=tb, bias=biasd, workspace=ws), fout)
    assert np.array_equal(got, ref), "%s %dx%dx%d: %d outputs differ from posit_gemm" % (fin, M, N, K, int((got != ref).sum()))
    if check_oracle:
        want, _ = fast.gemm(A, B, fin, fout, trans_a=ta, trans_b=tb, bias=bias)
        assert np.array_equal(got, want), "%s %dx%dx%d differs from the oracle" % (fin, M, N, K)


def test_static_scratch_matches_posit_gemm_on_successive_calls():
    # posit<8,0>, reduction split across workgroups (partial quires + NaR flags in the scratch array: the shapes with at
    # most 64 rows that the gather kernel takes); then a smaller split problem
    _case(1, "p8", "p16", 32, 288, 65536, 1, 0, True, True)
    _case(2, "p8", "p8", 48, 200, 8192, 0, 0, False, True)
    # the packed-operand path (operands, flags and nothing else in the array) followed by a split product
    _case(3, "p8", "p8", 4000, 4096, 1100, 0, 1, True, False)
    _case(4, "p8", "p8", 64, 512, 16384, 0, 0, False, True)
    # multi-limb quires: posit<16,1>, posit<32,2>, posit(8,2) -> posit(12,2); each followed by a smaller one
    _case(5, "p16", "p16", 96, 160, 4096, 1, 0, True, True)
    _case(6, "p16", "p8", 40, 50, 2048, 0, 1, False, True)
    _case(7, "p32", "p32", 24, 40, 2048, 0, 0, True, True)
    _case(8, "p8_2", "p12_2", 300, 200, 4096, 1, 0, True, True)
    _case(9, "p8_2", "p8_2", 100, 90, 8192, 0, 0, False, True)


def test_static_scratch_refuses_what_does_not_fit_and_leaves_the_output_alone():
    L = pn.load()
    M = N = K = 8192
    assert pn.posit_gemm_workspace("p8", "p8", 0, 0, M, N, K) > 72 << 20
    A = torch.zeros((16, 16), dtype=torch.uint8, device="cuda")  # never read: the call is refused before any launch
    out = torch.full((16,), 0x55, dtype=torch.uint8, device="cuda")
    rc = L.posit_gemm_static(None, 0, 0, 0, 0, M, N, K, ctypes.c_void_p(A.data_ptr()), K, ctypes.c_void_p(A.data_ptr()), N, None,
                             ctypes.c_void_p(out.data_ptr()), N)
    assert rc == 3
    torch.cuda.synchronize()
    assert (out.cpu().numpy() == 0x55).all()
    # a problem that needs no workspace at all works too
    rng = np.random.default_rng(11)
    a, b = rand_patterns(rng, (20, 30), "p8"), rand_patterns(rng, (30, 10), "p8")
    got = to_np(pn.posit_gemm_static(to_dev(a), to_dev(b), "p8", "p8"), "p8")
    want, _ = fast.gemm(a, b, "p8", "p8")
    assert np.array_equal(got, want)
