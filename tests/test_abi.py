"""The C-ABI library loads and exports every function include/positnn.h declares;
argument validation returns the documented status codes (no kernel is launched)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "positnn.h")
LIB = os.path.join(ROOT, "paper_2105_00053_amd", "libpositnn_hip.so")


def _declared():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(posit_[a-z0-9_]+)\s*\(", src)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2105_00053_amd import build
        build.build()
    return ctypes.CDLL(LIB)


def test_header_declares_the_expected_entry_points():
    assert _declared() == sorted([
        "posit_gemm", "posit_gemm_static", "posit_gemm_workspace", "posit_conv2d_fwd", "posit_conv2d_bwd_data", "posit_conv2d_bwd_weight",
        "posit_conv2d_workspace", "posit_round", "posit_convert", "posit_axpy", "posit_status_string",
        "posit_relu", "posit_relu_bwd", "posit_maxpool2d_fwd", "posit_maxpool2d_bwd", "posit_avgpool2d_fwd", "posit_avgpool2d_bwd",
        "posit_gemm_noquire", "posit_conv2d_fwd_noquire", "posit_conv2d_bwd_data_noquire", "posit_conv2d_bwd_weight_noquire",
        "posit_unary", "posit_unary_bwd", "posit_cross_entropy", "posit_mse", "posit_axpy_multi"])


def test_every_declared_symbol_is_exported(lib):
    for name in _declared():
        assert hasattr(lib, name), name


def test_status_strings(lib):
    lib.posit_status_string.restype = ctypes.c_char_p
    seen = {lib.posit_status_string(i) for i in range(5)}
    assert len(seen) == 5 and all(seen)
    assert lib.posit_status_string(99)


def test_argument_validation_without_launch():
    from paper_2105_00053_amd import binding as b
    L = b.load()
    null = ctypes.c_void_p(0)
    fake = ctypes.c_void_p(0x1000)  # never dereferenced: the calls below are rejected before any launch
    EINVAL = 1
    assert L.posit_gemm(null, 57, 0, 0, 0, 4, 4, 4, fake, 4, fake, 4, null, fake, 4, null, 0) == EINVAL      # unknown format
    assert L.posit_gemm(null, 0, 0, 0, 0, -1, 4, 4, fake, 4, fake, 4, null, fake, 4, null, 0) == EINVAL     # negative size
    assert L.posit_gemm(null, 0, 0, 0, 0, 4, 4, 4, null, 4, fake, 4, null, fake, 4, null, 0) == EINVAL      # null A
    assert L.posit_gemm(null, 0, 0, 0, 0, 4, 4, 8, fake, 4, fake, 4, null, fake, 4, null, 0) == EINVAL      # lda < K
    assert L.posit_gemm(null, 0, 0, 0, 0, 4, 4, 4, fake, 4, fake, 4, null, fake, 2, null, 0) == EINVAL      # ldc < N
    assert L.posit_gemm(null, 0, 0, 0, 0, 0, 4, 4, null, 4, null, 4, null, null, 4, null, 0) == 0           # empty: ok, nothing touched
    assert L.posit_gemm_noquire(null, 57, 0, 0, 0, 4, 4, 4, fake, 4, fake, 4, null, fake, 4) == EINVAL
    assert L.posit_gemm_noquire(null, 0, 0, 0, 0, 4, 4, 8, fake, 4, fake, 4, null, fake, 4) == EINVAL  # lda < K
    assert L.posit_gemm_noquire(null, 0, 0, 0, 0, 0, 4, 4, null, 4, null, 4, null, null, 4) == 0
    assert L.posit_conv2d_fwd_noquire(null, 0, 0, None, fake, fake, null, fake) == EINVAL
    assert L.posit_unary(null, 7, 0, 4, fake, fake) == EINVAL           # unknown function
    assert L.posit_unary(null, 0, 2, 4, fake, fake) == 2                # posit<32,2>: unsupported
    assert L.posit_unary(null, 0, 0, 0, null, null) == 0
    assert L.posit_unary_bwd(null, 2, 0, 0, 4, fake, fake, fake) == EINVAL  # no gradient entry for exp
    assert L.posit_cross_entropy(null, 0, 1, 1, 4, 10, fake, fake, null, null) == EINVAL  # nothing asked for
    assert L.posit_cross_entropy(null, 0, 2, 1, 4, 10, fake, fake, fake, fake) == 2
    assert L.posit_cross_entropy(null, 0, 1, 1, 0, 10, null, null, fake, null) == EINVAL  # mean over an empty batch
    assert L.posit_mse(null, 0, 1, 1, 4, fake, null, fake, fake) == EINVAL
    assert L.posit_round(null, 0, 0, 4, fake, fake) == EINVAL      # source must be a float type
    assert L.posit_round(null, 100, 100, 4, fake, fake) == EINVAL  # destination must be a posit
    assert L.posit_round(null, 100, 0, 0, null, null) == 0
    assert L.posit_convert(null, 100, 0, 4, fake, fake) == EINVAL
    assert L.posit_axpy(null, 0, 1, 0, 4, null, fake, -1, null) == EINVAL
    assert L.posit_axpy(null, 0, 1, 0, 4, fake, fake, 9, fake) == EINVAL  # bad copy format
    items = (b.AxpyItem * 2)()
    items[0].x, items[0].y, items[0].y_copy, items[0].n = 0x1000, 0x2000, None, 4
    items[1].x, items[1].y, items[1].y_copy, items[1].n = None, 0x2000, None, 4
    assert L.posit_axpy_multi(null, 0, 1, 0, 2, items, 0) == EINVAL   # item 1 has no x
    assert L.posit_axpy_multi(null, 0, 1, 0, 0, None, 0) == 0
    items[1].x, items[1].y_copy = 0x1000, 0x3000
    assert L.posit_axpy_multi(null, 0, 1, 0, 2, items, 77) == EINVAL  # a copy is asked for in an unknown format
    d = b.ConvDesc(1, 1, 4, 4, 1, 5, 5, 0, 0, 1, 1)  # kernel larger than the padded image
    assert L.posit_conv2d_fwd(null, 0, 0, ctypes.byref(d), fake, fake, null, fake, null, 0) == EINVAL
    d = b.ConvDesc(1, 1, 4, 4, 1, 3, 3, 0, 0, 0, 1)  # zero stride
    assert L.posit_conv2d_bwd_data(null, 0, 0, ctypes.byref(d), fake, fake, fake, null, 0) == EINVAL
    assert L.posit_conv2d_bwd_weight(null, 0, 0, None, fake, fake, fake, null, null, 0) == EINVAL
    d = b.ConvDesc(1, 1, 4, 4, 1, 3, 3, 0, 0, 1, 1)
    assert L.posit_conv2d_fwd(null, 0, 0, ctypes.byref(d), fake, fake, null, fake, null, 0) == 3  # needs its workspace
    assert L.posit_conv2d_fwd(null, 0, 0, ctypes.byref(d), fake, fake, null, fake, ctypes.c_void_p(0x1004), 1 << 30) == EINVAL  # workspace alignment
    # workspace of the posit<8,0> convolutions that run on the matrix cores (32 -> 32 channels, 32 x 32, batch 128, 3 x 3, pad 1):
    # forward / backward-data: weight planes (9 k blocks x 1 row block x 2 KB) + input planes (131072 pixels x 2 groups of 16
    # channels x 32 bytes) + 256 bytes of zeros; backward-weight: planes of dy (2 row blocks, 103 slices of 40 k blocks of two
    # pixels x 8 groups of 16 images), planes of x image-minor (32 x 32 x 32 pixels x 8 groups x 32 bytes), a block of ones per
    # group, 256 bytes of zeros, then the slices' partial sums and flags (289 columns: the weights and the bias gradient)
    d = b.ConvDesc(128, 32, 32, 32, 32, 3, 3, 1, 1, 1, 1)
    assert L.posit_conv2d_workspace(0, 0, 0, ctypes.byref(d)) == 9 * 2048 + 131072 * 2 * 32 + 256
    assert L.posit_conv2d_workspace(1, 0, 0, ctypes.byref(d)) == 9 * 2048 + 131072 * 2 * 32 + 256
    assert L.posit_conv2d_workspace(2, 0, 1, ctypes.byref(d)) == 4120 * 2 * 2048 + 32 * 32 * 32 * 8 * 32 + 8 * 32 + 256 + (103 * 32 * 289 + 103 * (32 + 289)) * 4
    d = b.ConvDesc(128, 32, 32, 32, 32, 3, 3, 1, 1, 2, 2)  # strided: forward keeps the dot-product kernel (no digit planes)
    assert L.posit_conv2d_workspace(0, 0, 0, ctypes.byref(d)) < 131072 * 2 * 32
    # average pooling: the weight 1/(kh*kw) must be a posit of fin.  posit<8,0> stops at minpos = 1/64
    assert L.posit_avgpool2d_fwd(null, 0, 0, 1, 16, 16, 16, 8, fake, fake) == 2   # 1/128 < minpos
    assert L.posit_avgpool2d_bwd(null, 0, 0, 1, 16, 16, 16, 8, fake, fake) == 2
    assert L.posit_avgpool2d_fwd(null, 0, 0, 0, 16, 16, 8, 8, null, null) == 0    # 1/64 = minpos: accepted (no planes: nothing launched)
    assert L.posit_avgpool2d_fwd(null, 4, 4, 0, 16, 16, 16, 8, null, null) == 0   # posit(8,2) reaches 2^-24
    assert L.posit_avgpool2d_fwd(null, 0, 0, 1, 6, 6, 3, 2, fake, fake) == 2      # window of 6: no power of two
    # a split reduction without the workspace it asks for
    need = L.posit_gemm_workspace(0, 1, 0, 0, 32, 288, 131072)
    assert need > 0
    assert L.posit_gemm(null, 0, 1, 0, 0, 32, 288, 131072, fake, 131072, fake, 288, null, fake, 288, null, 0) == 3
    assert L.posit_gemm(null, 0, 1, 0, 0, 32, 288, 131072, fake, 131072, fake, 288, null, fake, 288, ctypes.c_void_p(0x1008), need) == EINVAL  # alignment
    # posit<8,0> from 2^28 products up: no split, but both operands are rewritten into the workspace as two int8 digit
    # planes (2 bytes per element, padded to whole tiles and k steps); NaR travels as a marker digit, no flag arrays
    assert L.posit_gemm_workspace(0, 0, 0, 0, 4096, 4096, 4096) == 2 * 4096 * (4096 + 4096)
    assert L.posit_gemm_workspace(0, 0, 0, 0, 2048, 2048, 2048) == 2 * 2048 * (2048 + 2048)
    assert L.posit_gemm_workspace(0, 0, 0, 0, 600, 540, 1700) == 2 * 1728 * (640 + 576)  # 64 x 64 tiles, k in steps of 64
    assert L.posit_gemm_workspace(0, 0, 0, 0, 512, 512, 512) == 0   # below: the reduction cut inside the workgroup
    assert L.posit_gemm(null, 0, 0, 0, 0, 4096, 4096, 4096, fake, 4096, fake, 4096, null, fake, 4096, null, 0) == 3
    # posit(8,1) / posit(8,2) from 2^25 products up (128 outputs each way, K 256 .. 8192): four / eight digit planes per
    # operand in blocks of 32 x 32, a mask byte per block, and the two words of the unions of the masks
    planes = lambda nd, M, N, K: nd * 1024 * ((K + 31) // 32) * (2 * ((M + 63) // 64) + 2 * ((N + 63) // 64))
    masks = lambda M, N, K: sum((((K + 31) // 32) * 2 * ((R + 63) // 64) + 255) // 256 * 256 for R in (M, N))
    assert L.posit_gemm_workspace(4, 4, 0, 0, 1024, 1024, 1024) == planes(8, 1024, 1024, 1024) + masks(1024, 1024, 1024) + 256
    assert L.posit_gemm_workspace(3, 3, 0, 0, 1024, 1024, 1024) == planes(4, 1024, 1024, 1024) + masks(1024, 1024, 1024) + 256
    assert L.posit_gemm_workspace(4, 4, 0, 0, 600, 540, 1700) == planes(8, 600, 540, 1700) + masks(600, 540, 1700) + 256
    assert L.posit_gemm_workspace(4, 4, 0, 0, 1024, 1024, 8224) < planes(8, 1024, 1024, 8224)   # beyond 8192: the fp64 buckets
    # the variant with the library's own scratch array: same checks, and a problem beyond the array is refused before any launch
    assert L.posit_gemm_static(null, 57, 0, 0, 0, 4, 4, 4, fake, 4, fake, 4, null, fake, 4) == EINVAL
    assert L.posit_gemm_static(null, 0, 0, 0, 0, 4, 4, 8, fake, 4, fake, 4, null, fake, 4) == EINVAL
    assert L.posit_gemm_static(null, 0, 0, 0, 0, 0, 4, 4, null, 4, null, 4, null, null, 4) == 0
    assert L.posit_gemm_workspace(0, 0, 0, 0, 8192, 8192, 8192) > (72 << 20)
    assert L.posit_gemm_static(null, 0, 0, 0, 0, 8192, 8192, 8192, fake, 8192, fake, 8192, null, fake, 8192) == 3
