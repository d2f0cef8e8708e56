// Elementary functions, division and the pieces of the loss functions on posits
// (paper Fig. 2: Sigmoid and TanH activations, Cross Entropy and MSE losses;
// Sec. 3.3 / Fig. 3: the loss stage has a posit precision of its own; Sec. 4,
// Table 4: posit(10,2) or posit(12,2) for it).  The paper prints no algorithm.
// Here every elementary function returns the correctly rounded posit of the real
// function: the value is evaluated in binary64 (relative error of a few 2^-53) and
// rounded once to the format, which for formats of at most 16 bits gives the
// correctly rounded result unless the real value lies within about 2^-50 of a
// rounding boundary; that no pattern of any supported format does is checked
// exhaustively by the tests.  Formats of at most 16 bits only.
#pragma once

#include <math.h>

#include "noquire_arith.h"
#include "quire_arith.h"

namespace pnn {

enum UnaryFn { UNARY_SIGMOID = 0, UNARY_TANH = 1, UNARY_EXP = 2, UNARY_LOG = 3 };

__device__ __forceinline__ double bits_to_double(uint64_t b) { return __longlong_as_double((long long)b); }
__device__ __forceinline__ uint64_t double_to_bits(double d) { return (uint64_t)__double_as_longlong(d); }

// round a finite or infinite binary64 result to posit<F>: zero stands for "positive, below every
// posit" and infinity for "above every posit" (the callers' functions never return an exact zero
// or a NaN on the paths that reach here), so both clamp
template <class F>
__device__ __forceinline__ uint32_t round_double_clamped(double v) {
    Real r;
    const int kind = real_from_f64(double_to_bits(v), r);
    if (kind == 0) return 1u;                                   // underflow: minpos, never zero
    if (kind == 2) return v > 0 ? F::NAR - 1u : F::NAR + 1u;   // overflow: +-maxpos
    return encode<F>(r);
}

template <class F>
__device__ __forceinline__ uint32_t posit_unary(int fn, uint32_t p) {
    static_assert(F::N <= 16, "elementary functions are provided for formats of at most 16 bits");
    p &= F::MASK;
    if (p == F::NAR) return F::NAR;
    const uint32_t one = 1u << (F::N - 2);
    const double x = p == 0 ? 0.0 : bits_to_double(real_to_f64_bits(decode_fields<F>(p)));  // exact
    switch (fn) {
        case UNARY_EXP:
            return p == 0 ? one : round_double_clamped<F>(exp(x));
        case UNARY_LOG:
            if (p == 0 || (p >> (F::N - 1))) return F::NAR;
            return p == one ? 0u : round_double_clamped<F>(log(x));
        case UNARY_SIGMOID:
            return round_double_clamped<F>(1.0 / (1.0 + exp(-x)));  // exp(-x) = inf gives 0: clamps to minpos
        default:
            return p == 0 ? 0u : round_double_clamped<F>(tanh(x));
    }
}

// posit / posit -> posit, the exact quotient rounded once; a zero divisor gives NaR.
template <class F>
PNN_HD uint32_t posit_div(uint32_t a, uint32_t b) {
    static_assert(F::N <= 16, "division is provided for formats of at most 16 bits");
    if (a == F::NAR || b == F::NAR || b == 0) return F::NAR;
    if (a == 0) return 0u;
    const Real32 ra = decode_fields32<F>(a), rb = decode_fields32<F>(b);
    const uint64_t ma = (1u << 14) | (ra.frac >> 18), mb = (1u << 14) | (rb.frac >> 18);
    const uint64_t num = ma << 40;
    const uint64_t q = num / mb, rem = num - q * mb;  // 2^39 < q < 2^41
    const int top = 63 - clz64(q);                    // 39 or 40
    Real32 r;
    r.neg = ra.neg != rb.neg;
    r.scale = ra.scale - rb.scale + (top - 40);
    const uint64_t norm = q << (64 - top);            // leading one shifted out
    r.frac = (uint32_t)(norm >> 32);
    r.sticky = rem != 0 || (uint32_t)norm != 0;
    return encode32<F>(r);
}

// r / d for an integer d >= 1: the 65-bit significand, extended by 32 zero bits, is divided limb
// by limb; the quotient keeps at least 64 significant bits and everything below (further
// quotient bits, the remainder, the incoming sticky) is folded into sticky.  Exact for the single
// rounding that follows: a rounding boundary of r / d is a whole number of r's last place times
// d, so it cannot fall strictly inside the truncated part.
PNN_HD Real real_div_int(const Real& r, uint32_t d) {
    // dividend limbs, most significant first: 1, frac[63:32], frac[31:0], 0
    const uint32_t limb[4] = {1u, (uint32_t)(r.frac >> 32), (uint32_t)r.frac, 0u};
    uint32_t q[4];
    uint64_t rem = 0;
    for (int i = 0; i < 4; ++i) {
        const uint64_t cur = (rem << 32) | limb[i];
        q[i] = (uint32_t)(cur / d);
        rem = cur - (uint64_t)q[i] * d;
    }
    // quotient = q0 * 2^96 + q1 * 2^64 + q2 * 2^32 + q3 in units of 2^(scale - 96); q0 is 0 or 1
    const uint64_t hi = ((uint64_t)q[0] << 32) | q[1], lo = ((uint64_t)q[2] << 32) | q[3];
    Real o;
    o.neg = r.neg;
    // 2^96 <= dividend < 2^97 and d < 2^32, so 2^64 < quotient < 2^97: hi is never zero
    const int lead = 64 + 63 - clz64(hi);  // position of the leading one in (hi, lo): 64 .. 96
    o.scale = r.scale + (lead - 96);
    const int sh = 128 - lead;             // 32 .. 64: shift that pushes the leading one out of bit 127
    uint64_t fh, fl;
    if (sh == 64) { fh = lo; fl = 0; }
    else { fh = (hi << sh) | (lo >> (64 - sh)); fl = lo << sh; }
    o.frac = fh;
    o.sticky = r.sticky || rem != 0 || fl != 0;
    return o;
}

}  // namespace pnn
