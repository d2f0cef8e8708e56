"""Helpers for the GPU parity tests: numpy <-> device tensors of posit patterns."""
import numpy as np
import torch

import paper_2105_00053_amd as pn

NP_DTYPE = {"p8": np.uint8, "p16": np.uint16, "p32": np.uint32, "p8_1": np.uint8, "p8_2": np.uint8,
            "p10_1": np.uint16, "p10_2": np.uint16, "p12_1": np.uint16, "p12_2": np.uint16}
BITS = {"p8": 8, "p16": 16, "p32": 32, "p8_1": 8, "p8_2": 8, "p10_1": 10, "p10_2": 10, "p12_1": 12, "p12_2": 12}
GENERAL = ["p8_1", "p8_2", "p10_1", "p10_2", "p12_1", "p12_2"]  # formats of the paper's experiments outside Table 1
_VIEW = {np.dtype(np.uint8): torch.uint8, np.dtype(np.uint16): torch.int16, np.dtype(np.uint32): torch.int32}
_NP_SIGNED = {np.dtype(np.uint8): np.uint8, np.dtype(np.uint16): np.int16, np.dtype(np.uint32): np.int32}


def to_dev(a):
    """numpy array of patterns (uint8/16/32) or floats -> device tensor with the same bits."""
    a = np.ascontiguousarray(a)
    if a.dtype in _NP_SIGNED:
        return torch.from_numpy(a.view(_NP_SIGNED[a.dtype])).cuda()
    return torch.from_numpy(a).cuda()


def to_np(t, fmt):
    """device tensor of patterns -> numpy unsigned array."""
    c = t.cpu()
    if c.dtype == torch.uint16:
        c = c.view(torch.int16)
    elif c.dtype == torch.uint32:
        c = c.view(torch.int32)
    return c.numpy().view(NP_DTYPE[fmt])


def rand_patterns(rng, shape, fmt, special=0.02, allow_nar=True):
    b = BITS[fmt]
    a = rng.integers(0, 1 << b, size=shape, dtype=np.uint64)
    sp = [0, 1, (1 << (b - 1)) - 1, (1 << b) - 1, (1 << (b - 1)) + 1, 1 << (b - 2)]
    if allow_nar:
        sp.append(1 << (b - 1))
    s = rng.choice(np.array(sp, dtype=np.uint64), size=shape)
    a = np.where(rng.random(size=shape) < special, s, a)
    if not allow_nar:
        a = np.where(a == (1 << (b - 1)), 1, a)
    return a.astype(NP_DTYPE[fmt])


def mismatches(got, want):
    got = np.asarray(got).astype(np.int64)
    want = np.asarray(want).astype(np.int64)
    assert got.shape == want.shape, (got.shape, want.shape)
    bad = np.argwhere(got != want)
    return bad


def oracle_axpy_chunked(alpha, x, y, fx, fy, fc=None, workers=16):
    """fast.axpy (single-threaded C++ oracle) over slices of a long tensor in parallel threads: elementwise, so the
    slices are independent; ctypes releases the interpreter lock during the call."""
    from concurrent.futures import ThreadPoolExecutor

    from oracle import fast
    n = len(x)
    bounds = [n * i // workers for i in range(workers + 1)]
    with ThreadPoolExecutor(workers) as ex:
        parts = list(ex.map(lambda i: fast.axpy(alpha, x[bounds[i]:bounds[i + 1]], y[bounds[i]:bounds[i + 1]], fx, fy, fc), range(workers)))
    if fc:
        return np.concatenate([p[0] for p in parts]), np.concatenate([p[1] for p in parts])
    return np.concatenate(parts)
