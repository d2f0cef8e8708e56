// Scalar arithmetic of the two-bucket posit<16,1> dot product (see gemm_p16_window.h): which operands the buckets
// take, the error-free split of a product, the flush into quire limbs.  __host__ __device__, so that the CPU tests
// exercise the same source.
#pragma once

#include "quire_arith.h"

namespace pnn {

constexpr int PW_LO = 4, PW_HI = 47;      // main operands: multiples of 2^LO below 2^HI (units of minpos = 2^-28)
constexpr int PW_T1 = 51;                 // the cut between the two buckets
constexpr int PW_MAXK = 1024;             // products per output between two flushes
static_assert(2 * PW_HI + 10 <= 53 + PW_T1, "hi bucket: 1024 products of at most 2^(2 HI), multiples of 2^T1");
static_assert(PW_T1 - 1 + 10 <= 53 + 2 * PW_LO, "lo bucket: 1024 rests of at most 2^(T1-1), multiples of 2^(2 LO)");
static_assert(2 * PW_HI <= PW_T1 + 51 && PW_T1 - 2 * PW_LO <= 53, "the cut itself is exact");

// Scaled value of a pattern as the product kernel wants it: main operands as they are, outliers and zero as 0.0,
// NaR as a NaN.  Returns true for an outlier.
PNN_HD bool pw_classify(uint32_t p, double& v) {
    v = 0.0;
    if (p == 0) return false;
    if (p == P16::NAR) {
        v = __builtin_bit_cast(double, (uint64_t)0x7FF8000000000000ull);
        return false;
    }
    bool neg;
    uint32_t sig;
    int sh;
    decode_fixed<P16>(p, neg, sig, sh);
    // sig < 2^13 holds the significand with all its fraction bits: value = sig * 2^sh, below 2^(sh + bit length of sig)
    const int top = sh + 32 - clz32(sig);
    if (sh < PW_LO || top > PW_HI) return true;
    const double m = __builtin_ldexp((double)(int32_t)sig, sh);
    v = neg ? -m : m;
    return false;
}

PNN_HD void pw_mac(double& hi, double& lo, double a, double b) {
    constexpr double C = 1.5 * pow2d(52 + PW_T1);
    const double h = __builtin_fma(a, b, C) - C;
    hi += h;
    lo += __builtin_fma(a, b, -h);
}

// The two buckets of an output into its (zeroed or partial) quire limbs.
PNN_HD void pw_flush(uint32_t (&q)[4], double hi, double lo) {
    quire_add_double<4, PW_T1>(q, hi);
    quire_add_double<4, 2 * PW_LO>(q, lo);
}

}  // namespace pnn
