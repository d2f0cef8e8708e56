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
    uint32_t carry = 0;
#pragma unroll
    for (int l = 0; l < L; ++l) {
        const uint32_t add = (l < idx) ? 0u : (l == idx) ? x0 : (l == idx + 1) ? x1 : ext;
        const uint64_t t = (uint64_t)q[l] + add + carry;
        q[l] = (uint32_t)t;
        carry = (uint32_t)(t >> 32);
    }
}

// Same for a product of up to 63 bits plus sign (posit<32,2>: 28 x 28 bits).
template <int L>
PNN_HD void quire_add64(uint32_t (&q)[L], int64_t P, int s) {
    const int idx = s >> 5, off = s & 31;
    const uint64_t lo = (uint64_t)P << off;
    const uint32_t x0 = (uint32_t)lo;
    const uint32_t x1 = (uint32_t)(lo >> 32);
    const uint32_t x2 = (uint32_t)((P >> 32) >> (32 - off));  // bits 64..95 of the sign-extended shift
    const uint32_t ext = (uint32_t)((int32_t)x2 >> 31);
    uint32_t carry = 0;
#pragma unroll
    for (int l = 0; l < L; ++l) {
        const uint32_t add = (l < idx) ? 0u : (l == idx) ? x0 : (l == idx + 1) ? x1 : (l == idx + 2) ? x2 : ext;
        const uint64_t t = (uint64_t)q[l] + add + carry;
        q[l] = (uint32_t)t;
        carry = (uint32_t)(t >> 32);
    }
}

// Sum of two L-limb accumulators (split-K merge): plain multi-word addition,
// associative and exact modulo 2^(32 L).
template <int L>
PNN_HD void quire_merge(uint32_t (&q)[L], const uint32_t (&o)[L]) {
    uint32_t carry = 0;
#pragma unroll
    for (int l = 0; l < L; ++l) {
        const uint64_t t = (uint64_t)q[l] + o[l] + carry;
        q[l] = (uint32_t)t;
        carry = (uint32_t)(t >> 32);
    }
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

}  // namespace pnn
