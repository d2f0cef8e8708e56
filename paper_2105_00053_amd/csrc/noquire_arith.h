// Accumulation without the quire (paper Sec. 3.3: the quire is an option of the
// framework; Table 2 reports training "without quire").  Every product and every
// running sum is then itself a posit<n,es>: the exact product (sum) of two
// patterns rounded once, nearest with ties to the even pattern, as the Posit
// Standard defines multiplication and addition (Sec. 3.2).
#pragma once

#include "posit_core.h"

namespace pnn {

// Formats of at most 16 bits: significands of 15 bits, so the product is a 30-bit
// integer and the sum fits a 64-bit window anchored at the larger term (the
// smaller one keeps every bit unless it lies more than 47 places below; what
// falls off then only decides "sticky", borrowing one window unit when it is
// being subtracted).
template <class F>
PNN_HD uint32_t posit_mul_small(uint32_t a, uint32_t b) {  // a, b neither zero nor NaR
    const Real32 ra = decode_fields32<F>(a), rb = decode_fields32<F>(b);
    const uint32_t ma = (1u << 14) | (ra.frac >> 18), mb = (1u << 14) | (rb.frac >> 18);
#if defined(__HIP_DEVICE_COMPILE__)
    const uint32_t mt = (uint32_t)__umul24(ma, mb);  // 2^28 <= mt < 2^30
#else
    const uint32_t mt = ma * mb;
#endif
    const int top = 28 + (int)(mt >> 29);
    Real32 r;
    r.neg = ra.neg != rb.neg;
    r.scale = ra.scale + rb.scale + (top - 28);
    r.frac = mt << (32 - top);  // the leading one leaves the word
    r.sticky = false;
    return encode32<F>(r);
}

template <class F>
PNN_HD uint32_t posit_add_small(uint32_t x, uint32_t y) {  // x, y neither zero nor NaR
    const Real32 rx = decode_fields32<F>(x), ry = decode_fields32<F>(y);
    const uint64_t bx = (uint64_t)((1u << 14) | (rx.frac >> 18)) << 47;  // leading one at bit 61
    const uint64_t by = (uint64_t)((1u << 14) | (ry.frac >> 18)) << 47;
    const bool x_big = (rx.scale > ry.scale) || (rx.scale == ry.scale && bx >= by);
    const uint64_t big = x_big ? bx : by, small = x_big ? by : bx;
    const int sbig = x_big ? rx.scale : ry.scale;
    int d = x_big ? rx.scale - ry.scale : ry.scale - rx.scale;
    const bool far = d >= 64;
    d = far ? 63 : d;
    const uint64_t sh = far ? 0ull : (small >> d);
    const bool lost = far ? true : ((sh << d) != small);
    const uint64_t sum = (rx.neg == ry.neg) ? (big + sh) : (big - sh - (lost ? 1u : 0u));
    if (sum == 0) return 0u;  // exact cancellation
    const int lz = clz64(sum);
    Real32 r;
    r.neg = x_big ? rx.neg : ry.neg;
    r.scale = sbig + (63 - lz) - 61;
    const uint64_t norm = (sum << lz) << 1;  // leading one shifted out
    r.frac = (uint32_t)(norm >> 32);
    r.sticky = lost || ((uint32_t)norm != 0);
    return encode32<F>(r);
}

// Any two patterns: NaR absorbs (also NaR * 0), zero is exact.
template <class F>
PNN_HD uint32_t posit_mul(uint32_t a, uint32_t b) {
    if (a == F::NAR || b == F::NAR) return F::NAR;
    if (a == 0 || b == 0) return 0u;
    if constexpr (F::N <= 16) {
        return posit_mul_small<F>(a, b);
    } else {
        return encode<F>(real_mul(decode_fields<F>(a), decode_fields<F>(b)));
    }
}

template <class F>
PNN_HD uint32_t posit_add(uint32_t a, uint32_t b) {
    if (a == F::NAR || b == F::NAR) return F::NAR;
    if (a == 0) return b;
    if (b == 0) return a;
    if constexpr (F::N <= 16) {
        return posit_add_small<F>(a, b);
    } else {
        Real s;
        if (!real_add(decode_fields<F>(a), decode_fields<F>(b), s)) return 0u;
        return encode<F>(s);
    }
}

// Accumulator policy of the tiled GEMM kernel for this mode: the "quire" is one
// running posit pattern per output.  Terms arrive in order of the reduction index.
template <class F>
struct NoQuire {
    typedef uint32_t Elem;
    static constexpr int L = 1;
    static constexpr bool SPLITTABLE = false;  // the result depends on the order of the terms
    static constexpr int BUCKETS = 0;
    PNN_HD static Elem stage(uint32_t p) { return p == F::NAR ? 0u : p; }  // NaR is tracked by flags outside
    PNN_HD static void mac(uint32_t (&q)[1], Elem a, Elem b) { q[0] = posit_add<F>(q[0], posit_mul<F>(a, b)); }
    PNN_HD static void add_value(uint32_t (&q)[1], Elem a) { q[0] = posit_add<F>(q[0], a); }
    PNN_HD static void add_bias(uint32_t (&q)[1], uint32_t pattern) { add_value(q, stage(pattern)); }
    // the running posit as a real number (false: zero)
    PNN_HD static bool read(const uint32_t (&q)[1], Real& r) {
        if (q[0] == 0) return false;
        r = decode_fields<F>(q[0]);
        return true;
    }
};

}  // namespace pnn
