// Per-element operations of the bandwidth-bound entry points, written as
// functors over raw bit patterns: float -> posit (posit_round), posit -> posit
// and posit -> float (posit_convert; the paper's "convert PyTorch tensors" and
// "mixed precision tensor" utilities, Fig. 2), and the SGD update
// y <- round(y + alpha * x) (posit_axpy; Fig. 2 optimizer).  Every result is
// computed exactly and rounded once.
#pragma once

#include "posit_core.h"

namespace pnn {

template <class FD>
struct RoundF32 {
    PNN_HD uint64_t operator()(uint64_t bits) const {
        Real32 r;
        const int c = real32_from_f32((uint32_t)bits, r);
        if (c == 0) return 0;
        if (c == 2) return FD::NAR;
        return encode_any<FD>(r);
    }
};

template <class FD>
struct RoundF64 {
    PNN_HD uint64_t operator()(uint64_t bits) const {
        Real r;
        const int c = real_from_f64(bits, r);
        if (c == 0) return 0;
        if (c == 2) return FD::NAR;
        if (FD::N <= 16) return encode_any<FD>(narrow(r));
        return encode<FD>(r);
    }
};

template <class FS, class FD>
struct PositToPosit {
    PNN_HD uint64_t operator()(uint64_t p) const {
        const uint32_t q = (uint32_t)p & FS::MASK;
        if (q == 0) return 0;
        if (q == FS::NAR) return FD::NAR;
        return encode_any<FD>(decode_fields32<FS>(q));
    }
};

template <class FS>
struct PositToF32 {
    PNN_HD uint64_t operator()(uint64_t p) const {
        const uint32_t q = (uint32_t)p & FS::MASK;
        if (q == 0) return 0;
        if (q == FS::NAR) return 0x7FC00000u;  // quiet NaN
        return real_to_f32_bits(decode_fields<FS>(q));
    }
};

template <class FS>
struct PositToF64 {
    PNN_HD uint64_t operator()(uint64_t p) const {
        const uint32_t q = (uint32_t)p & FS::MASK;
        if (q == 0) return 0;
        if (q == FS::NAR) return 0x7FF8000000000000ull;
        return real_to_f64_bits(decode_fields<FS>(q));
    }
};

// Exact y + a*x for formats of at most 16 bits, then one rounding to FY.  All
// three patterns are neither zero nor NaR.  Significands are taken with 14
// fraction bits (no such format has more), the product a*x is a 30-bit integer,
// and the sum is formed in a 64-bit window anchored at the larger term: the
// smaller term keeps all its bits unless it lies more than 33 places below, in
// which case what falls off only decides "sticky" (borrowing one window unit when
// it is subtracted).
template <class FX, class FY>
PNN_HD uint32_t axpy_small(uint32_t a, uint32_t x, uint32_t y, bool y_zero) {
    const Real32 ra = decode_fields32<FY>(a), rx = decode_fields32<FX>(x), ry = decode_fields32<FY>(y);
    const uint32_t ma = (1u << 14) | (ra.frac >> 18), mx = (1u << 14) | (rx.frac >> 18);
#if defined(__HIP_DEVICE_COMPILE__)
    const uint32_t mt = (uint32_t)__umul24(ma, mx);  // 2^28 <= mt < 2^30
#else
    const uint32_t mt = ma * mx;
#endif
    const int top = 28 + (int)(mt >> 29);
    const uint64_t bt = (uint64_t)mt << (61 - top);  // leading one at bit 61
    const int st = ra.scale + rx.scale + (top - 28);   // |a*x| = bt * 2^(st - 61)
    // a zero y takes part as magnitude 0 far below everything
    const uint64_t by = y_zero ? 0ull : ((uint64_t)((1u << 14) | (ry.frac >> 18)) << 47);
    const int sy = y_zero ? -100000 : ry.scale;        // |y| = by * 2^(sy - 61)
    const bool nt = ra.neg != rx.neg, ny = ry.neg;
    const bool t_big = (st > sy) || (st == sy && bt >= by);
    const uint64_t big = t_big ? bt : by, small = t_big ? by : bt;
    const int sbig = t_big ? st : sy;
    int d = t_big ? st - sy : sy - st;
    const bool nbig = t_big ? nt : ny;
    const bool far = d >= 64;
    d = far ? 63 : d;
    const uint64_t sh = far ? 0ull : (small >> d);
    const bool lost = far ? (small != 0) : ((sh << d) != small);
    const uint64_t borrow = lost ? 1u : 0u;
    const uint64_t sum = (nt == ny) ? (big + sh) : (big - sh - borrow);
    const int lz = clz64(sum | 1u);
    Real32 r;
    r.neg = nbig;
    r.scale = sbig + (63 - lz) - 61;
    const uint64_t norm = (sum << lz) << 1;  // leading one shifted out
    r.frac = (uint32_t)(norm >> 32);
    r.sticky = lost || ((uint32_t)norm != 0);
    const uint32_t enc = encode32_flat<Fmt<(FY::N <= 16 ? FY::N : 16), FY::ES>>(r);
    return sum == 0 ? 0u : enc;  // exact cancellation
}

// y_new = round_FY( y + alpha * x ), alpha given as a pattern of FY.
template <class FX, class FY>
struct Axpy {
    uint32_t alpha;
    PNN_HD uint32_t operator()(uint32_t x, uint32_t y) const {
        x &= FX::MASK;
        y &= FY::MASK;
        const uint32_t a = alpha & FY::MASK;
        const bool nar = (a == FY::NAR) || (x == FX::NAR) || (y == FY::NAR);
        const bool t_zero = (a == 0) || (x == 0);
        if (FX::N <= 16 && FY::N <= 16) {
            // straight-line: special patterns are replaced by the value one before decoding
            // and the right answer is selected at the end
            const uint32_t one_x = 1u << (FX::N - 2), one_y = 1u << (FY::N - 2);
            const bool xs = (x == 0) || (x == FX::NAR), as = (a == 0) || (a == FY::NAR), ys = (y == 0) || (y == FY::NAR);
            const uint32_t r = axpy_small<FX, FY>(as ? one_y : a, xs ? one_x : x, ys ? one_y : y, ys);
            return nar ? FY::NAR : (t_zero ? y : r);  // y + 0 is y itself
        }
        if (nar) return FY::NAR;
        if (t_zero) return y;
        const Real t = real_mul(decode_fields<FY>(a), decode_fields<FX>(x));
        if (y == 0) return encode<FY>(t);
        Real s;
        if (!real_add(decode_fields<FY>(y), t, s)) return 0;
        return encode<FY>(s);
    }
};

// ---- formats chosen at run time (the (8,1), (8,2), (10,x), (12,x) family of Sec. 4) ----

// kind: 0 = posit (format in f), 1 = binary32, 2 = binary64
struct MapRT {
    int src_kind, dst_kind;
    FmtRT fs, fd;
    PNN_HD uint64_t operator()(uint64_t bits) const {
        Real r;
        int c;  // 0 zero, 1 finite nonzero, 2 NaR / NaN / Inf
        if (src_kind == 1) c = real_from_f32((uint32_t)bits, r);
        else if (src_kind == 2) c = real_from_f64(bits, r);
        else {
            const uint32_t q = (uint32_t)bits & fs.mask();
            c = q == 0 ? 0 : (q == fs.nar() ? 2 : 1);
            if (c == 1) r = decode_rt(q, fs);
        }
        if (dst_kind == 1) return c == 0 ? 0u : (c == 2 ? 0x7FC00000u : real_to_f32_bits(r));
        if (dst_kind == 2) return c == 0 ? 0ull : (c == 2 ? 0x7FF8000000000000ull : real_to_f64_bits(r));
        return c == 0 ? 0u : (c == 2 ? fd.nar() : encode_rt(r, fd));
    }
};

struct AxpyRT {
    FmtRT fx, fy;
    uint32_t alpha;
    PNN_HD uint32_t operator()(uint32_t x, uint32_t y) const {
        x &= fx.mask();
        y &= fy.mask();
        const uint32_t a = alpha & fy.mask();
        if (a == fy.nar() || x == fx.nar() || y == fy.nar()) return fy.nar();
        if (a == 0 || x == 0) return y;
        const Real t = real_mul(decode_rt(a, fy), decode_rt(x, fx));
        if (y == 0) return encode_rt(t, fy);
        Real s;
        if (!real_add(decode_rt(y, fy), t, s)) return 0;
        return encode_rt(s, fy);
    }
};

}  // namespace pnn
