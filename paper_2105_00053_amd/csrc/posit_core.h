// Scalar posit<n,es> building blocks used by every kernel of the library:
// field decode (paper Sec. 2, Eq. 2), the single round-to-nearest-even encode
// that ends every quire accumulation (Sec. 3.2 defers it to the Posit Standard),
// and the read-out of a multi-limb quire (Sec. 2; widths from Table 1).
//
// The functions are __host__ __device__ so that the same source can be
// exercised on the CPU by the host-side unit tests; the library itself only
// ever calls them from kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#define PNN_HD __host__ __device__ __forceinline__

namespace pnn {

// posit<N,ES> and its quire, held as 32-bit limbs.  The standard formats take
// the widths of Table 1 (N^2/2 = 32 / 128 / 512 bits).  Other (N,ES) pairs, which
// the paper's experiments use (Sec. 4: posit(8,1), (8,2), (10,x), (12,x)), get
// 4(N-2)2^ES bits for the largest product over the smallest one, one sign bit and
// N-1 carry-guard bits, rounded up to whole limbs.
constexpr int quire_bits_for(int n, int es) {
    return (n == 8 && es == 0) ? 32 : (n == 16 && es == 1) ? 128 : (n == 32 && es == 2) ? 512
           : ((4 * (n - 2) * (1 << es) + 1 + (n - 1) + 31) / 32) * 32;
}

template <int N_, int ES_>
struct Fmt {
    static constexpr int N = N_;
    static constexpr int ES = ES_;
    static constexpr int MAXS = (N_ - 2) << ES_;  // log2(maxpos) = -log2(minpos)
    static constexpr uint32_t MASK = N_ == 32 ? 0xFFFFFFFFu : ((1u << (N_ & 31)) - 1u);
    static constexpr uint32_t NAR = 1u << (N_ - 1);
    static constexpr int FB = N_ - 3 - ES_;          // most fraction bits a pattern can hold
    static constexpr int QBITS = quire_bits_for(N_, ES_);
    static constexpr int QLIMBS = QBITS / 32;
    static constexpr int QFRAC = 2 * MAXS;           // quire LSB = 2^-QFRAC = minpos^2
};
// Unsigned integer type that stores one pattern of an N-bit posit.
template <int NBITS> struct Storage;
template <> struct Storage<8> { typedef uint8_t T; };
template <> struct Storage<10> { typedef uint16_t T; };  // low N bits of the container
template <> struct Storage<12> { typedef uint16_t T; };
template <> struct Storage<16> { typedef uint16_t T; };
template <> struct Storage<32> { typedef uint32_t T; };

using P8 = Fmt<8, 0>;
using P16 = Fmt<16, 1>;
using P32 = Fmt<32, 2>;
using P8_1 = Fmt<8, 1>;
using P8_2 = Fmt<8, 2>;
using P10_1 = Fmt<10, 1>;
using P10_2 = Fmt<10, 2>;
using P12_1 = Fmt<12, 1>;
using P12_2 = Fmt<12, 2>;

// Format codes of the C ABI (pnn_dtype): 0..2 the standard formats of Table 1, 3..8 the
// other (N,ES) pairs of the paper's experiments.
PNN_HD void fmt_params(int code, int& n, int& es) {
    switch (code) {
        case 0: n = 8; es = 0; break;
        case 1: n = 16; es = 1; break;
        case 2: n = 32; es = 2; break;
        case 3: n = 8; es = 1; break;
        case 4: n = 8; es = 2; break;
        case 5: n = 10; es = 1; break;
        case 6: n = 10; es = 2; break;
        case 7: n = 12; es = 1; break;
        default: n = 12; es = 2; break;
    }
}

// A format known only at run time (elementwise kernels on the non-standard formats,
// output format of the GEMM epilogues).
struct FmtRT {
    int n, es;
    PNN_HD int maxs() const { return (n - 2) << es; }
    PNN_HD uint32_t mask() const { return n == 32 ? 0xFFFFFFFFu : ((1u << (n & 31)) - 1u); }
    PNN_HD uint32_t nar() const { return 1u << (n - 1); }
    PNN_HD int bytes() const { return n <= 8 ? 1 : (n <= 16 ? 2 : 4); }
};

PNN_HD FmtRT fmt_of_code(int code) {
    FmtRT f;
    fmt_params(code, f.n, f.es);
    return f;
}

PNN_HD int clz32(uint32_t x) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __clz((int)x);
#else
    return x ? __builtin_clz(x) : 32;
#endif
}

PNN_HD int clz64(uint64_t x) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __clzll((long long)x);
#else
    return x ? __builtin_clzll(x) : 64;
#endif
}

// A nonzero real number: (-1)^neg * 2^scale * (1 + frac / 2^64), plus "something
// nonzero lies below frac" (sticky).
struct Real {
    bool neg;
    int scale;
    uint64_t frac;
    bool sticky;
};

// Field decode of a pattern that is neither 0 nor NaR (Eq. 2), for any n <= 32.
// Negative patterns are two's-complemented first.  The fraction comes back at
// the top of a 32-bit word (a posit carries at most 27 fraction bits); `nf`
// receives how many genuine fraction bits the pattern holds.
PNN_HD void decode_core(uint32_t p, int n, int es, bool& neg, int& scale, uint32_t& frac, int& nf) {
    const uint32_t mask = n == 32 ? 0xFFFFFFFFu : ((1u << (n & 31)) - 1u);
    neg = (p >> (n - 1)) & 1u;
    const uint32_t x = neg ? ((0u - p) & mask) : p;
    const uint32_t y = x << (33 - n);          // first regime bit in bit 31, zeros shifted in below
    const uint32_t lead = y >> 31;
    const int run = clz32(lead ? ~y : y);      // regime run length, 1 .. n-1
    const int k = lead ? run - 1 : -run;
    const uint32_t rest = (y << run) << 1;     // drop the run and the bit that ended it
    const int e = es ? (int)(rest >> ((32 - es) & 31)) : 0;  // cut-off exponent bits arrive as zeros
    frac = rest << es;
    scale = k * (1 << es) + e;
    nf = n - 2 - run - es;
    if (nf < 0) nf = 0;
}

template <class F>
PNN_HD Real decode_fields(uint32_t p, int& nf) {
    Real r;
    uint32_t fr;
    decode_core(p, F::N, F::ES, r.neg, r.scale, fr, nf);
    r.frac = (uint64_t)fr << 32;
    r.sticky = false;
    return r;
}

template <class F>
PNN_HD Real decode_fields(uint32_t p) {
    int nf;
    return decode_fields<F>(p, nf);
}

PNN_HD Real decode_rt(uint32_t p, const FmtRT& f) {
    Real r;
    uint32_t fr;
    int nf;
    decode_core(p, f.n, f.es, r.neg, r.scale, fr, nf);
    r.frac = (uint64_t)fr << 32;
    r.sticky = false;
    return r;
}

// Fixed-point view used by the quire: value = sig * 2^sh * minpos with sig odd or
// carrying exactly the pattern's fraction bits, sh >= 0 (every posit is a whole
// multiple of minpos).  The sign is returned separately.
template <class F>
PNN_HD void decode_fixed(uint32_t p, bool& neg, uint32_t& sig, int& sh) {
    int nf;
    const Real r = decode_fields<F>(p, nf);
    neg = r.neg;
    const uint32_t top = (uint32_t)(r.frac >> 32);
    sig = (1u << nf) | (nf ? (top >> (32 - nf)) : 0u);
    sh = r.scale - nf + F::MAXS;
}

// The one rounding: nearest posit<n,es>, ties to the even pattern, never to 0 or
// NaR.  The unbounded string regime | exponent | fraction is assembled at the
// top of a 64-bit word and cut after n-1 bits.  Any n <= 32.
PNN_HD uint32_t encode_core(const Real& r, int n, int es) {
    const int maxs = (n - 2) << es;
    const uint32_t mask = n == 32 ? 0xFFFFFFFFu : ((1u << (n & 31)) - 1u);
    uint32_t body;
    if (r.scale >= maxs) {
        body = (1u << (n - 1)) - 1u;  // maxpos and beyond
    } else if (r.scale < -maxs) {
        body = 1u;                    // below minpos
    } else {
        const int k = r.scale >> es;  // floor
        const uint32_t e = (uint32_t)(r.scale & ((1 << es) - 1));
        int rl;
        uint64_t regime;
        if (k >= 0) {
            rl = k + 2;
            regime = ((uint64_t)1 << (k + 2)) - 2u;  // k+1 ones, one zero
        } else {
            rl = 1 - k;
            regime = 1u;  // -k zeros, one one
        }
        const int hl = rl + es;  // 2 .. n-1+es
        const uint64_t head = (regime << es) | e;
        const uint64_t w = (head << (64 - hl)) | (r.frac >> hl);
        bool sticky = r.sticky || ((r.frac << (64 - hl)) != 0);
        body = (uint32_t)(w >> (65 - n));
        const uint32_t guard = (uint32_t)(w >> (64 - n)) & 1u;
        sticky = sticky || ((w << n) != 0);
        body += guard & ((sticky ? 1u : 0u) | (body & 1u));
    }
    return r.neg ? ((0u - body) & mask) : body;
}

template <class F>
PNN_HD uint32_t encode(const Real& r) {
    return encode_core(r, F::N, F::ES);
}

PNN_HD uint32_t encode_rt(const Real& r, const FmtRT& f) { return encode_core(r, f.n, f.es); }

// 32-bit variants for the bandwidth-bound kernels: a posit carries at most 27
// fraction bits, so a decoded value fits a 32-bit fraction, and for formats of at
// most 16 bits the cut string regime | exponent | fraction fits one 32-bit word.
struct Real32 {
    bool neg;
    int scale;
    uint32_t frac;  // fraction bits at the top
    bool sticky;
};

PNN_HD Real32 narrow(const Real& r) {
    Real32 o;
    o.neg = r.neg;
    o.scale = r.scale;
    o.frac = (uint32_t)(r.frac >> 32);
    o.sticky = r.sticky || ((uint32_t)r.frac != 0);
    return o;
}

PNN_HD Real widen(const Real32& r) {
    Real o;
    o.neg = r.neg;
    o.scale = r.scale;
    o.frac = (uint64_t)r.frac << 32;
    o.sticky = r.sticky;
    return o;
}

template <class F>
PNN_HD Real32 decode_fields32(uint32_t p) {
    Real32 r;
    int nf;
    decode_core(p, F::N, F::ES, r.neg, r.scale, r.frac, nf);
    r.sticky = false;
    return r;
}

// Same rounding as encode<F>, in one 32-bit word; F::N <= 16.
template <class F>
PNN_HD uint32_t encode32(const Real32& r) {
    static_assert(F::N <= 16, "32-bit encoder is for formats of at most 16 bits");
    uint32_t body;
    if (r.scale >= F::MAXS) {
        body = F::NAR - 1u;
    } else if (r.scale < -F::MAXS) {
        body = 1u;
    } else {
        const int k = r.scale >> F::ES;
        const uint32_t e = (uint32_t)(r.scale & ((1 << F::ES) - 1));
        const int rl = k >= 0 ? k + 2 : 1 - k;
        const uint32_t regime = k >= 0 ? ((1u << (k + 2)) - 2u) : 1u;
        const int hl = rl + F::ES;  // 2 .. N-1+ES <= 17
        const uint32_t head = (regime << F::ES) | e;
        const uint32_t w = (head << (32 - hl)) | (r.frac >> hl);
        bool sticky = r.sticky || ((r.frac << (32 - hl)) != 0);
        body = w >> (33 - F::N);
        const uint32_t guard = (w >> (32 - F::N)) & 1u;
        sticky = sticky || ((w << F::N) != 0);
        body += guard & ((sticky ? 1u : 0u) | (body & 1u));
    }
    return r.neg ? ((0u - body) & F::MASK) : body;
}

// Straight-line form of encode32 for code that is already branch-free: a scale
// beyond the format is replaced by the largest (smallest) regular scale with an
// all-ones (zero) fraction, which rounds to maxpos (minpos).
template <class F>
PNN_HD uint32_t encode32_flat(const Real32& r) {
    static_assert(F::N <= 16, "32-bit encoder is for formats of at most 16 bits");
    const bool over = r.scale >= F::MAXS, under = r.scale < -F::MAXS;
    const int scale = over ? F::MAXS - 1 : (under ? -F::MAXS : r.scale);
    const uint32_t frac = over ? 0xFFFFFFFFu : (under ? 0u : r.frac);
    const bool sticky_in = over ? true : (under ? false : r.sticky);
    const int k = scale >> F::ES;
    const uint32_t e = (uint32_t)(scale & ((1 << F::ES) - 1));
    const bool pos = k >= 0;
    const int rl = pos ? k + 2 : 1 - k;
    const uint32_t regime = pos ? ((1u << ((k + 2) & 31)) - 2u) : 1u;
    const int hl = rl + F::ES;
    const uint32_t head = (regime << F::ES) | e;
    const uint32_t w = (head << (32 - hl)) | (frac >> hl);
    const bool sticky = sticky_in || ((frac << (32 - hl)) != 0) || ((w << F::N) != 0);
    uint32_t body = w >> (33 - F::N);
    const uint32_t guard = (w >> (32 - F::N)) & 1u;
    body += guard & ((sticky ? 1u : 0u) | (body & 1u));
    return r.neg ? ((0u - body) & F::MASK) : body;
}

// Encoder chosen by destination width.
template <class F>
PNN_HD uint32_t encode_any(const Real32& r) {
    if (F::N <= 16) {
        return encode32<Fmt<(F::N <= 16 ? F::N : 16), F::ES>>(r);
    }
    return encode<F>(widen(r));
}

// Read a quire of L 32-bit limbs (two's complement, LSB weight 2^-qfrac) out as a
// Real.  Returns false when the quire is exactly zero.  All limb indices are
// compile-time so the limbs stay in registers.
template <int L>
PNN_HD bool quire_to_real(const uint32_t (&qin)[L], int qfrac, Real& r) {
    uint32_t q[L];
    const bool neg = (qin[L - 1] >> 31) != 0;
    uint32_t carry = neg ? 1u : 0u;
#pragma unroll
    for (int i = 0; i < L; ++i) {
        const uint32_t v = neg ? ~qin[i] : qin[i];
        const uint32_t s = v + carry;
        carry = (s < v) ? 1u : 0u;
        q[i] = s;
    }
    // top nonzero limb and the two below it
    uint32_t hi = 0, mid = 0, lo = 0, below = 0;
    int t = -1;
#pragma unroll
    for (int i = L - 1; i >= 0; --i) {
        if (t < 0 && q[i] != 0) {
            t = i;
            hi = q[i];
            mid = (i > 0) ? q[i > 0 ? i - 1 : 0] : 0u;
            lo = (i > 1) ? q[i > 1 ? i - 2 : 0] : 0u;
        } else if (t >= 0 && i < t - 2) {
            below |= q[i];
        }
    }
    if (t < 0) return false;
    const int lz = clz32(hi);
    r.neg = neg;
    r.scale = 32 * t + 31 - lz - qfrac;
    // 96-bit window (hi, mid, lo) shifted left by lz+1 so that the leading one falls off
    const uint64_t top = ((uint64_t)hi << 32) | mid;
    const uint64_t a = (top << lz) << 1;
    const uint64_t lo_sh = ((uint64_t)lo << lz) << 1;  // lo moved up by lz+1, bits 32.. spill into the window
    r.frac = a | (lo_sh >> 32);
    r.sticky = (below != 0) || ((uint32_t)lo_sh != 0);
    return true;
}

// IEEE binary32 / binary64 -> Real.  Returns 0 for zero, 1 for a finite nonzero
// value, 2 for NaN or infinity.  Subnormals lie far below minpos of every format
// here, so only their being nonzero matters: they get a scale that clamps.
PNN_HD int real_from_f32(uint32_t bits, Real& r) {
    const uint32_t ex = (bits >> 23) & 0xFFu;
    const uint32_t man = bits & 0x7FFFFFu;
    if (ex == 0xFFu) return 2;
    if (ex == 0 && man == 0) return 0;
    r.neg = bits >> 31;
    r.sticky = false;
    if (ex == 0) {
        r.scale = -1000;
        r.frac = 0;
        r.sticky = true;
    } else {
        r.scale = (int)ex - 127;
        r.frac = (uint64_t)man << 41;
    }
    return 1;
}

PNN_HD int real32_from_f32(uint32_t bits, Real32& r) {
    const uint32_t ex = (bits >> 23) & 0xFFu;
    const uint32_t man = bits & 0x7FFFFFu;
    if (ex == 0xFFu) return 2;
    if (ex == 0 && man == 0) return 0;
    r.neg = bits >> 31;
    r.sticky = ex == 0;                       // subnormal: only "nonzero and tiny" matters
    r.scale = ex == 0 ? -1000 : (int)ex - 127;
    r.frac = ex == 0 ? 0u : man << 9;
    return 1;
}

PNN_HD int real_from_f64(uint64_t bits, Real& r) {
    const uint32_t ex = (uint32_t)(bits >> 52) & 0x7FFu;
    const uint64_t man = bits & 0xFFFFFFFFFFFFFull;
    if (ex == 0x7FFu) return 2;
    if (ex == 0 && man == 0) return 0;
    r.neg = bits >> 63;
    r.sticky = false;
    if (ex == 0) {
        r.scale = -2000;
        r.frac = 0;
        r.sticky = true;
    } else {
        r.scale = (int)ex - 1023;
        r.frac = man << 12;
    }
    return 1;
}

// Real (from a posit: at most 27 fraction bits, |scale| <= 120) -> IEEE bits.
// binary64 holds every posit here exactly; binary32 rounds posit<32,2> fractions
// to 23 bits, nearest even, with the carry allowed to run into the exponent.
PNN_HD uint64_t real_to_f64_bits(const Real& r) {
    return ((uint64_t)r.neg << 63) | ((uint64_t)(r.scale + 1023) << 52) | (r.frac >> 12);
}

PNN_HD uint32_t real_to_f32_bits(const Real& r) {
    uint32_t mag = ((uint32_t)(r.scale + 127) << 23) | (uint32_t)(r.frac >> 41);
    const uint64_t rem = r.frac << 23;  // what binary32 cannot hold
    const uint64_t half = (uint64_t)1 << 63;
    if (rem > half || (rem == half && (mag & 1u))) mag += 1;
    return ((uint32_t)r.neg << 31) | mag;
}

// Exact a + b for two nonzero Reals whose fractions fit 60 bits (true for
// posits and products of two posits), returned as a Real with sticky; false when
// the sum is exactly zero.  A 128-bit window is anchored at the larger operand;
// what the smaller one loses off the bottom is folded into sticky, borrowing
// one window unit when it is being subtracted.
PNN_HD bool real_add(const Real& a_in, const Real& b_in, Real& out) {
    Real a = a_in, b = b_in;
    if (b.scale > a.scale || (b.scale == a.scale && b.frac > a.frac)) {
        Real t = a; a = b; b = t;
    }
    typedef unsigned __int128 u128;
    // significand 1.frac with the leading one at bit 124 of the window
    const u128 sa = (((u128)1 << 64) | a.frac) << 60;
    const u128 sb_full = (((u128)1 << 64) | b.frac) << 60;
    const int d = a.scale - b.scale;  // >= 0
    u128 sb;
    bool lost;
    if (d >= 126) {
        sb = 0;
        lost = true;
    } else {
        sb = sb_full >> d;
        lost = (sb << d) != sb_full;
    }
    u128 s;
    if (a.neg == b.neg) {
        s = sa + sb;
    } else {
        s = sa - sb;
        if (lost) s -= 1;  // true value lies strictly between s-1 and s
    }
    if (s == 0 && !lost) return false;
    const uint64_t hi = (uint64_t)(s >> 64), lo = (uint64_t)s;
    const int lz = hi ? clz64(hi) : 64 + clz64(lo);
    const int msb = 127 - lz;
    out.neg = a.neg;
    out.scale = a.scale + (msb - 124);
    const u128 norm = (s << lz) << 1;  // leading one shifted out
    out.frac = (uint64_t)(norm >> 64);
    out.sticky = lost || ((uint64_t)norm != 0) || a.sticky || b.sticky;
    return true;
}

// Exact product of two nonzero Reals holding posits (fractions of at most 27 bits).
PNN_HD Real real_mul(const Real& a, const Real& b) {
    const uint64_t ma = ((uint64_t)1 << 31) | (a.frac >> 33);  // 1.f with 31 fraction bits
    const uint64_t mb = ((uint64_t)1 << 31) | (b.frac >> 33);
    const uint64_t p = ma * mb;  // in [2^62, 2^64)
    Real r;
    r.neg = a.neg != b.neg;
    r.sticky = false;
    if (p >> 63) {
        r.scale = a.scale + b.scale + 1;
        r.frac = p << 1;
    } else {
        r.scale = a.scale + b.scale;
        r.frac = p << 2;
    }
    return r;
}

}  // namespace pnn
