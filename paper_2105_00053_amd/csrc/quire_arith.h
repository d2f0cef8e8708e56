// Per-format arithmetic of the quire dot product (paper Sec. 2: the quire holds
// exact sums of products; Table 1: 32 / 128 / 512 bits): how a pattern is
// staged into LDS, how one product enters the accumulator limbs, and how the
// accumulator is read out and rounded once.
#pragma once

#include "posit_core.h"

namespace pnn {

// Add the signed value P * 2^s into an L-limb two's-complement accumulator
// (32-bit limbs in registers, carries propagated through every limb above).
// The addend occupies limbs idx, idx+1 and is sign-extended above them; which
// limb receives which word is decided by selects so that no limb is ever
// indexed dynamically.
template <int L>
PNN_HD void quire_add32(uint32_t (&q)[L], int32_t P, int s) {
    const int idx = s >> 5, off = s & 31;
    const int64_t wide = (int64_t)P << off;
    const uint32_t x0 = (uint32_t)wide;
    const uint32_t x1 = (uint32_t)((uint64_t)wide >> 32);
    const uint32_t ext = (uint32_t)((int32_t)x1 >> 31);
    unsigned carry = 0;
#pragma unroll
    for (int l = 0; l < L; ++l) {
        const uint32_t add = (l < idx) ? 0u : (l == idx) ? x0 : (l == idx + 1) ? x1 : ext;
        q[l] = __builtin_addc(q[l], add, carry, &carry);
    }
}

// Same for a product of up to 63 bits plus sign (posit<32,2>: 28 x 28 bits).  The three words of the
// shifted product (sign extension above them) are moved to limb idx by a barrel shift over whole
// limbs: log2(L) rounds of "take the limb `step` below if that bit of idx is set", of which only
// the limbs that can differ from the sign extension cost a select (4 + 6 + 10 + 16 for L = 16,
// against four compares and four selects per limb when every limb tests idx by itself).
template <int L>
PNN_HD void quire_add64(uint32_t (&q)[L], int64_t P, int s) {
    const int idx = s >> 5, off = s & 31;
    const uint64_t lo = (uint64_t)P << off;
    const uint32_t x2 = (uint32_t)((P >> 32) >> (32 - off));  // bits 64..95 of the sign-extended shift
    const uint32_t ext = (uint32_t)((int32_t)x2 >> 31);
    uint32_t v[L];
#pragma unroll
    for (int l = 0; l < L; ++l) v[l] = l == 0 ? (uint32_t)lo : l == 1 ? (uint32_t)(lo >> 32) : l == 2 ? x2 : ext;
#pragma unroll
    for (int step = 1; step < L; step <<= 1) {
        const bool on = (idx & step) != 0;
#pragma unroll
        for (int l = L - 1; l >= 0; --l) v[l] = on ? (l >= step ? v[l - step] : 0u) : v[l];
    }
    unsigned carry = 0;
#pragma unroll
    for (int l = 0; l < L; ++l) q[l] = __builtin_addc(q[l], v[l], carry, &carry);
}

// Sum of two L-limb accumulators (split-K merge): plain multi-word addition,
// associative and exact modulo 2^(32 L).
template <int L>
PNN_HD void quire_merge(uint32_t (&q)[L], const uint32_t (&o)[L]) {
    unsigned carry = 0;
#pragma unroll
    for (int l = 0; l < L; ++l) q[l] = __builtin_addc(q[l], o[l], carry, &carry);
}

// Narrow an accumulator held in L limbs to its true width QB (sign-extend from bit QB-1).
template <int L, int QB>
PNN_HD void quire_wrap(uint32_t (&q)[L]) {
    if (QB >= 32 * L) return;
    constexpr int top = (QB - 1) / 32, bit = (QB - 1) % 32;
    const uint32_t ext = (q[top] >> bit) & 1u ? 0xFFFFFFFFu : 0u;
    if (bit != 31) {
        const uint32_t keep = (1u << (bit + 1)) - 1u;
        q[top] = (q[top] & keep) | (ext & ~keep);
    }
#pragma unroll
    for (int l = top + 1; l < L; ++l) q[l] = ext;
}

// Read the quire of FIN out as a real number (false when exactly zero).
template <class FIN, int L>
PNN_HD bool quire_read(const uint32_t (&qin)[L], Real& r) {
    uint32_t q[L];
#pragma unroll
    for (int l = 0; l < L; ++l) q[l] = qin[l];
    quire_wrap<L, FIN::QBITS>(q);
    return quire_to_real<L>(q, FIN::QFRAC, r);
}

template <class FIN, class FOUT, int L>
PNN_HD uint32_t quire_round(const uint32_t (&q)[L]) {
    Real r;
    if (!quire_read<FIN, L>(q, r)) return 0u;
    return encode<FOUT>(r);
}

// 128-bit quire (posit<16,1>): the sign-extended product shifted by s & 63 is a
// 128-bit value (x0, x1); products landing in the upper half (s >= 64) only keep x0
// (the rest is beyond bit 127, i.e. gone modulo 2^128).  One 128-bit add follows.
PNN_HD void quire_add128(uint32_t (&q)[4], int32_t P, int s) {
    typedef unsigned __int128 u128;
    const int off = s & 63;
    const int64_t p64 = (int64_t)P;
    const uint64_t x0 = (uint64_t)p64 << off;
    const uint64_t x1 = (uint64_t)((p64 >> 1) >> (63 - off));  // bits 64..127 of the shifted value
    const bool upper = s >= 64;
    const uint64_t a0 = upper ? 0ull : x0;
    const uint64_t a1 = upper ? x0 : x1;
    u128 Q = ((u128)(((uint64_t)q[3] << 32) | q[2]) << 64) | (((uint64_t)q[1] << 32) | q[0]);
    Q += ((u128)a1 << 64) | a0;
    q[0] = (uint32_t)Q;
    q[1] = (uint32_t)(Q >> 32);
    q[2] = (uint32_t)(Q >> 64);
    q[3] = (uint32_t)(Q >> 96);
}

template <class F>
struct Arith;

// posit<8,0>: every value is an integer number of minpos = 2^-6 with magnitude at
// most 2^12, so a staged operand is that integer and the 32-bit quire of Table 1
// is an int32 counting units of 2^-12.
template <>
struct Arith<P8> {
    typedef int32_t Elem;
    static constexpr int L = 1;
    PNN_HD static Elem stage(uint32_t p) {
        if (p == 0 || p == P8::NAR) return 0;
        bool neg;
        uint32_t sig;
        int sh;
        decode_fixed<P8>(p, neg, sig, sh);
        const int32_t v = (int32_t)(sig << sh);
        return neg ? -v : v;
    }
    PNN_HD static void mac(uint32_t (&q)[1], Elem a, Elem b) {
#if defined(__HIP_DEVICE_COMPILE__)
        q[0] += (uint32_t)__mul24(a, b);
#else
        q[0] += (uint32_t)(a * b);
#endif
    }
    // + a * 1, the value one being 2^6 minpos
    PNN_HD static void add_value(uint32_t (&q)[1], Elem a) { q[0] += (uint32_t)a << P8::MAXS; }
};

// Formats of at most 16 bits other than posit<8,0> (posit<16,1> and the (8,1), (8,2),
// (10,x), (12,x) family): staged word = signed significand (at most 14 bits) in the
// low half, shift in units of minpos in the high half.  The quire is kept in two
// limbs when it has at most 64 bits, in four up to 128 bits (a 96-bit quire is
// accumulated modulo 2^128 and narrowed when it is read out, which is the same as
// wrapping modulo 2^96 all along), else in QBITS/32 limbs.
template <int N, int ES>
struct Arith<Fmt<N, ES>> {
    typedef Fmt<N, ES> F;
    static_assert(N <= 16, "small-format arithmetic");
    typedef uint32_t Elem;
    static constexpr int L = F::QBITS <= 64 ? 2 : (F::QBITS <= 128 ? 4 : F::QLIMBS);
    PNN_HD static Elem stage(uint32_t p) {
        if (p == 0 || p == F::NAR) return 0;
        bool neg;
        uint32_t sig;
        int sh;
        decode_fixed<F>(p, neg, sig, sh);
        const int32_t v = neg ? -(int32_t)sig : (int32_t)sig;
        return ((uint32_t)sh << 16) | ((uint32_t)v & 0xFFFFu);
    }
    PNN_HD static void add_product(uint32_t (&q)[L], int32_t P, int s) {
        if constexpr (L == 2) {
            uint64_t acc = ((uint64_t)q[1] << 32) | q[0];
            acc += (uint64_t)((int64_t)P << s);  // s <= 4*MAXS/2 + ... < 64 - product width
            q[0] = (uint32_t)acc;
            q[1] = (uint32_t)(acc >> 32);
        } else if constexpr (L == 4) {
            quire_add128(q, P, s);
        } else {
            quire_add32<L>(q, P, s);  // wider quires ((10,2), (12,2)): select-based limb placement
        }
    }
    PNN_HD static void mac(uint32_t (&q)[L], Elem a, Elem b) {
        const int32_t sa = (int16_t)(a & 0xFFFFu), sb = (int16_t)(b & 0xFFFFu);
#if defined(__HIP_DEVICE_COMPILE__)
        const int32_t P = __mul24(sa, sb);
#else
        const int32_t P = sa * sb;
#endif
        add_product(q, P, (int)(a >> 16) + (int)(b >> 16));
    }
    PNN_HD static void add_value(uint32_t (&q)[L], Elem a) {
        add_product(q, (int16_t)(a & 0xFFFFu), (int)(a >> 16) + F::MAXS);
    }
};

// posit<32,2>: staged pair = signed 28-bit significand, shift (0..240, units of
// minpos = 2^-120).
template <>
struct Arith<P32> {
    typedef uint2 Elem;
    static constexpr int L = 16;
    PNN_HD static Elem stage(uint32_t p) {
        Elem e;
        e.x = 0;
        e.y = 0;
        if (p == 0 || p == P32::NAR) return e;
        bool neg;
        uint32_t sig;
        int sh;
        decode_fixed<P32>(p, neg, sig, sh);
        e.x = (uint32_t)(neg ? -(int32_t)sig : (int32_t)sig);
        e.y = (uint32_t)sh;
        return e;
    }
    PNN_HD static void mac(uint32_t (&q)[16], Elem a, Elem b) {
        const int64_t P = (int64_t)(int32_t)a.x * (int64_t)(int32_t)b.x;
        quire_add64<16>(q, P, (int)(a.y + b.y));
    }
    PNN_HD static void add_value(uint32_t (&q)[16], Elem a) {
        quire_add64<16>(q, (int64_t)(int32_t)a.x, (int)a.y + P32::MAXS);
    }
};

// ---- exact accumulation in fp64 "buckets" (formats of at most 16 bits other than posit<8,0>) ----
//
// The quire (Sec. 2) is an exact fixed-point sum; how the sum is carried between two
// read-outs is free as long as it stays exact.  Scaled by 2^MAXS every finite operand is an
// integer of at most 2^(2 MAXS), so a product is an integer P with |P| <= 2^R, R = 4 MAXS,
// whose significand has at most 28 bits: P itself is always a double, only the *sum* is too
// wide.  The sum is therefore kept in B doubles ("buckets"); bucket j only ever receives
// multiples of 2^T_j that are at most 2^(53+T_j-G) in magnitude, so 2^G additions into it are
// exact.  A product is cut into its bucket parts with exact floating-point steps:
//     t = fma(a, b, C_1),  C_1 = 1.5 * 2^(52+T_1):  t - C_1 = P rounded to a multiple of 2^T_1  (= h_1)
//     r = fma(a, b, -h_1)                         :  the rest, |r| <= 2^(T_1-1), exact
//     (r + C_j) - C_j = h_j, r -= h_j             :  the same cut at T_j for the buckets in between
// and the last bucket takes what is left.  With T_j = (B-j)(54-G): bucket 1 sees
// |h_1| <= 2^R and needs R + G - T_1 <= 53, bucket j > 1 sees |h_j| <= 2^(T_(j-1)-1), i.e. exactly
// 2^(53+T_j-G).  After at most 2^G products per output the buckets are emptied into the integer
// quire limbs (one 64-bit integer per bucket, shifted by T_j), which is where the sum lives
// between slices, across a split reduction and at the rounding.  Cost per product: 1, 5, 9 or 13
// fp64 operations for B = 1..4, against 6 to 60 integer operations of the carry-propagating add.
constexpr double pow2d(int e) {
    double r = 1.0;
    for (; e > 0; --e) r *= 2.0;
    for (; e < 0; ++e) r *= 0.5;
    return r;
}

constexpr int bucket_guard(int R, int B) { return (53 + 54 * (B - 1) - R) / B; }  // largest G the bounds above allow
constexpr int bucket_count(int R) {
    for (int B = 1; B <= 4; ++B)
        if (53 + 54 * (B - 1) - R >= 5 * B) return B;
    return 0;
}

// Add d (an integer multiple of 2^T, |d| <= 2^(53+T)) into the limbs.  The integer d / 2^T is read
// off the mantissas of two sums with "1.5 * 2^e" constants: adding 1.5 * 2^(84+T) leaves
// round(d / 2^(32+T)) in the low mantissa word (two's complement, |.| <= 2^21), and the exact rest
// (|rest| <= 2^(31+T), either sign at a tie) plus 1.5 * 2^(52+T) leaves rest / 2^T there modulo 2^32;
// d / 2^T = high * 2^32 + rest / 2^T, so its low word is that word and its high word is high minus
// one when the rest is negative.
template <int L, int T>
PNN_HD void quire_add_double(uint32_t (&q)[L], double d) {
    constexpr int idx = T / 32, off = T % 32;
    constexpr double CH = 1.5 * pow2d(84 + T), CL = 1.5 * pow2d(52 + T);
    const double th = d + CH;
    const double rest = d - (th - CH);
    const double tl = rest + CL;
    const uint32_t lo = (uint32_t)__builtin_bit_cast(uint64_t, tl);
    const uint32_t hi = (uint32_t)__builtin_bit_cast(uint64_t, th) - (rest < 0.0 ? 1u : 0u);
    const int64_t v = (int64_t)(((uint64_t)hi << 32) | lo);
    const uint64_t sl = (uint64_t)v << off;
    const uint32_t w0 = (uint32_t)sl, w1 = (uint32_t)(sl >> 32);
    const uint32_t w2 = off ? (uint32_t)((v >> 32) >> (32 - off)) : (uint32_t)(v >> 63);  // bits 64..95 of the sign-extended shift
    const uint32_t ext = (uint32_t)(v >> 63);
    unsigned carry = 0;
#pragma unroll
    for (int l = idx; l < L; ++l) {
        const uint32_t add = (l == idx) ? w0 : (l == idx + 1) ? w1 : (l == idx + 2) ? w2 : ext;
        q[l] = __builtin_addc(q[l], add, carry, &carry);  // one add-with-carry per limb
    }
}

template <class F>
struct BucketArith {
    static constexpr int R = 4 * F::MAXS;
    static constexpr bool ELIGIBLE = F::N <= 16 && !(F::N == 8 && F::ES == 0);
    static constexpr int B = ELIGIBLE ? bucket_count(R) : 0;
    static constexpr int NB = B > 0 ? B : 1;
    static constexpr int G = B > 0 ? (bucket_guard(R, NB) < 16 ? bucket_guard(R, NB) : 16) : 0;  // products per output between flushes: 2^G
    static constexpr int T(int j) { return (NB - j) * (54 - G); }                                    // j = 1..B; T(B) = 0
    static_assert(B == 0 || (G >= 5 && R + G - T(1) <= 53 && R <= 51 + T(1)), "bucket bounds");

    typedef double Elem;
    // value * 2^MAXS, an integer; zero and NaR stage as 0 (NaR is carried by the row / column flags)
    PNN_HD static Elem stage(uint32_t p) {
        if (p == 0 || p == F::NAR) return 0.0;
        bool neg;
        uint32_t sig;
        int sh;
        decode_fixed<F>(p, neg, sig, sh);
        const double v = __builtin_ldexp((double)(int32_t)sig, sh);
        return neg ? -v : v;
    }
    PNN_HD static void clear(double (&bk)[NB]) {
#pragma unroll
        for (int j = 0; j < NB; ++j) bk[j] = 0.0;
    }
    PNN_HD static void mac(double (&bk)[NB], Elem a, Elem b) {
        if constexpr (NB == 1) {
            bk[0] = __builtin_fma(a, b, bk[0]);
        } else {
            constexpr double C1 = 1.5 * pow2d(52 + T(1));
            const double h1 = __builtin_fma(a, b, C1) - C1;
            bk[0] += h1;
            double r = __builtin_fma(a, b, -h1);
            cut<2>(bk, r);
            bk[NB - 1] += r;
        }
    }
    template <int J>
    PNN_HD static void cut(double (&bk)[NB], double& r) {
        if constexpr (J < NB) {
            constexpr double Cj = 1.5 * pow2d(52 + T(J));
            const double h = (r + Cj) - Cj;
            bk[J - 1] += h;
            r -= h;
            cut<J + 1>(bk, r);
        }
    }
    // Empty the buckets into the limbs (L limbs, accumulated modulo 2^(32 L)).
    template <int L>
    PNN_HD static void flush(uint32_t (&q)[L], double (&bk)[NB]) {
        flush_from<L, 1>(q, bk);
        clear(bk);
    }
    template <int L, int J>
    PNN_HD static void flush_from(uint32_t (&q)[L], const double (&bk)[NB]) {
        quire_add_double<L, T(J)>(q, bk[J - 1]);
        if constexpr (J < NB) flush_from<L, J + 1>(q, bk);
    }
};

// ---- the whole sum in doubles (posit(8,1), posit(8,2)) ----
//
// BucketArith empties its buckets into integer limbs before their guard bits run out.  For the two
// 8-bit formats the kernel can instead carry between doubles and form the limbs once at the end:
// one more double on top (level 0, multiples of 2^TOPG) and, from the bottom up, "carry" steps
//     c = (x_j + 1.5 * 2^(52+g)) - 1.5 * 2^(52+g)   (x_j rounded to a multiple of g = the grain of level j-1)
//     x_j -= c;  x_(j-1) += c                          (both exact: |x_j - c| <= g/2, and see the bounds)
// Schedule and bounds, with R = 4 MAXS the bit length of the largest product:
//   every LOW_EVERY = 16 products all levels below the top bucket carry upwards; the lowest level then holds
//       at most half a grain of the level above plus 16 products' worth: 2^(T-1) + 16 * 2^(T-1) < 2^53 for the
//       split remainders of posit(8,2) (T = T_1 = 49), 2^(TOPG-1) + 16 * 2^R < 2^53 for posit(8,1) (one bucket)
//   every TOP_EVERY = 32 products the top bucket carries into level 0; before that it holds at most
//       2^(TOPG-1) + 32 * 2^R + two carries from below <= 2^(53+T_1)
//   level 0 holds the whole sum above 2^TOPG: K * 2^R / 2^TOPG <= 2^53 for K < 2^31.
// Each level is a multiple of its grain of at most 2^53 grains, so quire_add_double converts it exactly.
template <class F>
struct CascadeArith : BucketArith<F> {
    typedef BucketArith<F> BA;
    static constexpr int NB = BA::NB;
    static constexpr int NL = NB + 1;  // level 0 on top, levels 1..NB are the buckets of BucketArith (NB the lowest)
    static constexpr int LOW_EVERY = 16, TOP_EVERY = 32;
    static constexpr int TOPG = NB == 1 ? 40 : BA::T(1) + 51;
    static constexpr int grain(int level) { return level == 0 ? TOPG : BA::T(level); }
    static constexpr bool ELIGIBLE = BA::B > 0 && F::N == 8 && NB <= 2;
    static_assert(!ELIGIBLE || BA::R + 31 - TOPG <= 53, "level 0 holds the sum of 2^31 products");
    static_assert(!ELIGIBLE || NB != 1 || (TOPG - 1 <= 52 && BA::R + 4 <= 52), "one bucket: half a top grain + 16 products < 2^53");
    static_assert(!ELIGIBLE || NB != 2 || (BA::T(1) + 4 <= 53 && TOPG - 1 <= 51 + BA::T(1) && BA::R + 5 <= 52 + BA::T(1)),
                  "two buckets: 17 half grains in the low one; half a top grain + 32 products + carries in the high one");

    PNN_HD static void clear(double (&c)[NL]) {
#pragma unroll
        for (int j = 0; j < NL; ++j) c[j] = 0.0;
    }
    PNN_HD static void mac(double (&c)[NL], double a, double b) {
        if constexpr (NB == 1) {
            c[1] = __builtin_fma(a, b, c[1]);
        } else {
            constexpr double C1 = 1.5 * pow2d(52 + BA::T(1));
            const double h1 = __builtin_fma(a, b, C1) - C1;
            c[1] += h1;
            c[2] += __builtin_fma(a, b, -h1);
        }
    }
    // carry level J into level J - 1
    template <int J>
    PNN_HD static void carry(double (&c)[NL]) {
        constexpr double C = 1.5 * pow2d(52 + grain(J - 1));
        const double up = (c[J] + C) - C;
        c[J] -= up;
        c[J - 1] += up;
    }
    // after every LOW_EVERY products: everything below the top bucket moves up (one bucket: straight into level 0)
    PNN_HD static void carry_low(double (&c)[NL]) {
        if constexpr (NB == 1) carry<1>(c);
        else carry<2>(c);
    }
    // after every TOP_EVERY products (two buckets only): the top bucket moves into level 0
    PNN_HD static void carry_top(double (&c)[NL]) {
        if constexpr (NB == 2) carry<1>(c);
    }
    template <int L>
    PNN_HD static void to_limbs(uint32_t (&q)[L], const double (&c)[NL]) {
        quire_add_double<L, grain(0)>(q, c[0]);
        quire_add_double<L, grain(1)>(q, c[1]);
        if constexpr (NB == 2) quire_add_double<L, grain(2)>(q, c[2]);
    }
};

}  // namespace pnn
