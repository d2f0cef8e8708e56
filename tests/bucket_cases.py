"""Input vectors that fill the guard bits of the fp64 buckets the kernels accumulate in.

For formats of at most 16 bits (other than posit<8,0>) the kernels gather the exact products of up
to 2^G reduction steps in B doubles per output before they enter the integer quire: bucket j holds
multiples of 2^T_j, T_j = (B-j)(54-G), in units of the quire's last bit.  The vectors here are built
from the format alone (through the oracle's decode): for every bucket, runs of the largest product
that lands wholly in it, one product worth a single unit of that bucket, and the runs again with
the opposite sign, so that the exact sum is that single product and any lost bit changes the result.
No arithmetic of the method lives here beyond that selection."""
import numpy as np

from oracle import posit_oracle as po


def bucket_layout(fmt):
    """(B, G, [T_1..T_B]) as the kernels derive them: the fewest buckets that leave G >= 5, G capped at 16."""
    f = po.FORMATS[fmt]
    R = 4 * (f.n - 2) * (1 << f.es)
    for B in range(1, 5):
        if 53 + 54 * (B - 1) - R >= 5 * B:
            G = min((53 + 54 * (B - 1) - R) // B, 16)
            return B, G, [(B - j) * (54 - G) for j in range(1, B + 1)], R
    raise ValueError(fmt)


def _candidates(fmt):
    f = po.FORMATS[fmt]
    maxs = (f.n - 2) * (1 << f.es)
    pats = range(1, 1 << (f.n - 1)) if f.n <= 10 else [p for p in range(1, 1 << (f.n - 1)) if p % 17 == 0 or (p & (p + 1)) == 0 or (p & (p - 1)) == 0]
    vals = [(p, int(po.decode(p, f) * (1 << maxs))) for p in pats]
    step = max(1, len(vals) // 400)
    return vals[::step] + vals[-40:] + vals[:40]


def _best_pair(cands, key):
    best = None
    for p, v in cands:
        for q, w in cands:
            k = key(v * w)
            if k is not None and (best is None or k > best[0]):
                best = (k, p, q)
    return best


def guard_cases(fmt, mults=(1, 2, 4, 8), leads=(0, 5, 16), max_len=300000):
    """Yields (a, b, (sa, sb)): pattern vectors whose exact dot product equals the single product sa * sb."""
    n = po.FORMATS[fmt].n
    full = (1 << n) - 1
    B, G, cuts, R = bucket_layout(fmt)
    cands = _candidates(fmt)
    flush = 1 << G
    for j, T in enumerate(cuts, start=1):
        upper = R if j == 1 else cuts[j - 2] - 1  # products of at most 2^upper land wholly in bucket j or below
        big = _best_pair(cands, lambda P: P if (P <= (1 << upper) and P % (1 << T) == 0) else None)
        small = _best_pair(cands, lambda P: -P if (P % (1 << (T + 1)) == (1 << T)) else None)  # lowest set bit is bit T
        assert big is not None and small is not None, (fmt, j)
        _, ba, bb = big
        _, sa, sb = small
        for mult in mults:
            nb = mult * flush - 1
            if 2 * nb + 17 > max_len:
                continue
            for lead in leads:
                a = np.concatenate([np.zeros(lead), np.full(nb, ba), [sa], np.full(nb, ba)]).astype(np.uint32)
                b = np.concatenate([np.zeros(lead), np.full(nb, bb), [sb], np.full(nb, (-bb) & full)]).astype(np.uint32)
                yield a, b, (sa, sb)
