// Large-tensor versions of the two bandwidth-bound operations whose generic kernels are bound by
// instruction count instead: the SGD update y <- round(y + alpha * x) with its narrowed copy (paper
// Fig. 2, optimizer; Sec. 3.3: copies of a tensor in several posit formats; Sec. 4: 16-bit / 12-bit
// optimizer formats) and the narrowing conversion posit<16,1> -> posit<8,0>.
//
// The update.  For formats of at most 16 bits every value is a binary64 number whose low word is
// zero, the product alpha * x has at most 26 significant bits (exact in binary64), and the sum
// t + y is taken with the error-free transformation s = fl(t + y), err = (t + y) - s, so the pair
// (s, err) IS the exact result.  The one rounding to posit<N,ES> needs the leading ~N bits of s and
// "is anything nonzero below them", which err supplies when s itself was rounded.  Decoding is a
// look-up: a table in LDS maps the magnitude pattern to the high word of its binary64 (built once
// per workgroup with the field decoder of Eq. 2; 128 KB for posit<16,1>, so one 1024-thread
// workgroup per compute unit walks the tensor in a grid-stride loop).
//
// The narrowing conversion.  posit<16,1> -> posit<8,0> is a monotone step function of the pattern
// (as a signed integer).  Inside an aligned block of 64 source patterns it takes at most two values,
// so a 1024-entry LDS table of (value at the start of the block, position of the step) replaces the
// decode and re-encode: one look-up, one compare, one add.  The step between neighbouring values
// u, u+1 of the narrow format sits at the 9-bit posit 2u+1 (the rounding rule: ties to the even
// pattern), which posit<16,1> holds exactly.
#pragma once

#include "elementwise_ops.h"

namespace pnn {

PNN_HD double f64_from_words(uint32_t hi, uint32_t lo) { return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo); }
PNN_HD uint32_t f64_hi(double v) { return (uint32_t)(__builtin_bit_cast(uint64_t, v) >> 32); }
PNN_HD uint32_t f64_lo(double v) { return (uint32_t)__builtin_bit_cast(uint64_t, v); }

// bits [sh+31 : sh] of the 64-bit value hi:lo, 0 < sh < 32
PNN_HD uint32_t funnel_shr(uint32_t hi, uint32_t lo, int sh) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_alignbit(hi, lo, (uint32_t)sh);
#else
    return (uint32_t)((((uint64_t)hi << 32) | lo) >> sh);
#endif
}

// High word of the binary64 that equals the posit with magnitude pattern `a` (0 .. 2^(N-1)); the low
// word is zero because no format here has more than 20 fraction bits.  Zero gives 0.0, the NaR
// pattern a quiet NaN: both then pass through the arithmetic as IEEE special values.
template <class F>
PNN_HD uint32_t f64_hi_of_magnitude(uint32_t a) {
    static_assert(F::N <= 16 && F::FB <= 20, "the value must fit the high word of a binary64");
    if (a == 0) return 0u;
    if (a == F::NAR) return 0x7FF80000u;
    const Real32 r = decode_fields32<F>(a);
    return ((uint32_t)(r.scale + 1023) << 20) | (r.frac >> 12);
}

// The same for a signed pattern.
template <class F>
PNN_HD double f64_of_pattern(uint32_t p) {
    p &= F::MASK;
    const bool neg = (p >> (F::N - 1)) & 1u;
    const uint32_t a = neg ? ((0u - p) & F::MASK) : p;
    return f64_from_words(f64_hi_of_magnitude<F>(a) | (neg && a != F::NAR ? 0x80000000u : 0u), 0u);
}

// One rounding of an exact real number to posit<N,ES>, N <= 16.  The number is s + err with s a binary64
// given by its two words and err (|err| at most half a unit of s's last place) by its high word `ehi`
// (0: the number is s itself).  Rounds to nearest with ties to the even pattern and clamps to
// [minpos, maxpos].  Zero and NaN are not handled here: the caller tests for them (f64_is_special) and
// substitutes special_pattern().  Returns the pattern of the magnitude (round_sum_to_body) or the signed
// pattern (round_sum_to_posit).
//
// The string  regime | exponent | fraction  is produced without a table of regimes: with
// k = floor(scale / 2^ES), kk = k for k >= 0 and -k-1 otherwise, an arithmetic right shift by kk of
// "10" followed by the exponent and fraction bits yields kk+1 ones, a zero and the rest; for negative
// k the tail is complemented before and the whole word after the shift, which turns that head into
// kk+1 zeros and a one.  Bits that the cut cannot reach are folded into one bit that no shift here
// pushes out (bit N of the tail), so the sticky information survives in a single word.
template <class F>
PNN_HD uint32_t round_sum_to_body(uint32_t hi, uint32_t lo, uint32_t ehi) {
    static_assert(F::N <= 16, "formats of at most 16 bits");
    constexpr int N = F::N, ES = F::ES;
    constexpr uint32_t MAXHI = (uint32_t)(1023 + F::MAXS) << 20, MINHI = (uint32_t)(1023 - F::MAXS) << 20;
    // err nonzero with the sign opposite to s: the exact magnitude lies just below |s|, which borrows from the high
    // word when s's low word is zero (the low word itself then only has to stay "nonzero": ehi supplies that below)
    const bool toward_zero = (ehi ^ (hi & 0x80000000u)) > 0x80000000u;
    hi -= (toward_zero && lo == 0u) ? 1u : 0u;
    const uint32_t ah0 = hi & 0x7FFFFFFFu;
    // beyond the format's range only the clamped scale matters: the guard bit of a clamped value is zero
    const uint32_t ah = ah0 < MINHI ? MINHI : (ah0 > MAXHI ? MAXHI : ah0);
    const uint32_t h1 = ah - (1023u << 20);  // scale (two's complement) above bit 20, 20 fraction bits below
    const int k = (int32_t)h1 >> (20 + ES);
    const uint32_t sg = (uint32_t)(k >> 31);
    const uint32_t kk = (uint32_t)k ^ sg;
    const uint32_t tail = funnel_shr(h1, lo, 20 + ES);  // the ES exponent bits, then the significand's fraction
    // everything below bit N of the tail: the last HB fraction bits of the high word (when HB > 0) and the low word,
    // or the low 32 + HB bits of the low word; and the error term (shifted so that its sign bit does not count)
    constexpr int HB = N - 12 + ES;
    const uint32_t below = (HB > 0 ? ((h1 & ((1u << (HB > 0 ? HB : 0)) - 1u)) | lo) : (lo & (0xFFFFFFFFu >> (HB < 0 ? -HB : 0)))) | (ehi << 1);
    const uint32_t jam = below != 0u ? (1u << N) : 0u;
    const uint32_t w = funnel_shr(2u, (tail | jam) ^ sg, 2);
    const uint32_t x = (uint32_t)((int32_t)w >> kk) ^ sg;
    const uint32_t lsb = (x >> (33 - N)) & 1u;
    return (x + ((1u << (32 - N)) - 1u) + lsb) >> (33 - N);  // the pattern of the magnitude; the caller applies the sign
}

// The rounded pattern with its sign: two's complement of the magnitude pattern for a negative value.
template <class F>
PNN_HD uint32_t round_sum_to_posit(uint32_t hi, uint32_t lo, uint32_t ehi) {
    const uint32_t body = round_sum_to_body<F>(hi, lo, ehi);
    const uint32_t sm = (uint32_t)((int32_t)hi >> 31);  // all ones for a negative value
    return ((body ^ sm) - sm) & F::MASK;
}

// zero, infinity or NaN
PNN_HD bool f64_is_special(double s) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_class(s, 0x267);  // signalling / quiet NaN, -inf, -0, +0, +inf: one compare-class instruction
#else
    return ((f64_hi(s) & 0x7FFFFFFFu) - 1u) >= 0x7FEFFFFFu;
#endif
}

// What round_sum_to_posit leaves to its caller: hi = high word of s.
template <class F>
PNN_HD uint32_t special_pattern(uint32_t hi) {
    return (hi & 0x7FFFFFFFu) == 0u ? 0u : F::NAR;
}

// The same with the missing part described by two flags: `inexact` (the exact value differs from s, by less than
// one unit of s's last place) and `toward_zero` (the exact magnitude is the smaller one).  NaN gives NaR, zero zero.
template <class F>
PNN_HD uint32_t round_f64_to_posit(double s, bool inexact, bool toward_zero) {
    const uint32_t hi = f64_hi(s);
    const uint32_t ehi = inexact ? (0x3FF00000u | ((hi & 0x80000000u) ^ (toward_zero ? 0x80000000u : 0u))) : 0u;
    const uint32_t pat = round_sum_to_posit<F>(hi, f64_lo(s), ehi);
    return f64_is_special(s) ? special_pattern<F>(hi) : pat;
}

// y + alpha * x, exactly, rounded once to FY (zero and NaN left to the caller, see round_sum_to_posit).
// xd, yd, ad: the operands as binary64 (NaN for NaR); shi receives the high word of the rounded sum.
template <class FY, bool SIGNED_RESULT = true>
PNN_HD uint32_t axpy_f64_core(double ad, double xd, double yd, uint32_t& shi, bool& special) {
    const double t = ad * xd;      // at most 26 significant bits: exact
    const double s = t + yd;
    const double bb = s - t;       // error-free transformation of the sum: s + err == t + yd exactly
    const double err = (t - (s - bb)) + (yd - bb);
    shi = f64_hi(s);
    special = f64_is_special(s);
    if constexpr (SIGNED_RESULT) return round_sum_to_posit<FY>(shi, f64_lo(s), f64_hi(err));
    else return round_sum_to_body<FY>(shi, f64_lo(s), f64_hi(err));
}

template <class FY>
PNN_HD uint32_t axpy_f64(double ad, double xd, double yd) {
    uint32_t shi;
    bool special;
    const uint32_t pat = axpy_f64_core<FY>(ad, xd, yd, shi, special);
    return special ? special_pattern<FY>(shi) : pat;
}

// Entry of the step table of the narrowing conversion FS -> FD for the block of 64 source patterns
// that starts at b * 64: low byte = the result for the first pattern of the block, high byte = thr,
// where pattern p of the block converts to that result plus one exactly when (p & 63) > thr (63: never).
template <class FS, class FD>
PNN_HD uint32_t narrow_step_entry(uint32_t b) {
    static_assert(FS::N == 16 && FD::N == 8, "posit<16,es> to posit<8,es>");
    typedef Fmt<FD::N + 1, FD::ES> Mid;  // its odd patterns are the ties between neighbours of FD
    const uint32_t p0 = b << 6;
    const uint32_t base = (uint32_t)PositToPosit<FS, FD>()(p0) & 0xFFu;
    const int sbase = (int)(int8_t)base;
    int t;  // first source pattern, as a signed integer, that converts to base + 1
    if (base == 0x7Fu) {
        t = 1 << 20;  // nothing above maxpos
    } else if (base == 0x80u) {
        t = -32767;   // NaR is alone; the next pattern is -maxpos already
    } else if (sbase >= 0) {
        if (base == 0u) {
            t = 1;  // every positive value converts to at least minpos
        } else {
            const int m = (int)PositToPosit<Mid, FS>()(2u * base + 1u);
            t = (base & 1u) ? m : m + 1;  // the tie itself goes to the even one of base, base + 1
        }
    } else {
        const int v = -sbase;  // magnitude pattern of base; base + 1 has magnitude v - 1
        if (v == 1) {
            t = 0;  // only zero converts to zero
        } else {
            const int m = (int)PositToPosit<Mid, FS>()(2u * (uint32_t)(v - 1) + 1u);
            t = ((v - 1) & 1) == 0 ? -m : -m + 1;
        }
    }
    const int d = t - (int)(int16_t)p0;
    const uint32_t thr = (d >= 1 && d <= 63) ? (uint32_t)(d - 1) : 63u;
    return base | (thr << 8);
}

PNN_HD uint32_t narrow_step_apply(uint32_t entry, uint32_t p) {
    return (entry + (((p & 63u) > (entry >> 8)) ? 1u : 0u)) & 0xFFu;
}

#if defined(__HIPCC__)

// ---- kernels ----

template <class T, int V>
struct alignas(sizeof(T) * V) Pack {
    T v[V];
};

// dst[i] = round_FD(src[i]) for posit<16,1> -> posit<8,0>; 8 elements per thread and step.
template <class FS, class FD>
__global__ __launch_bounds__(256) void narrow_step_kernel(const uint16_t* __restrict__ src, uint8_t* __restrict__ dst, int64_t nvec) {
    __shared__ uint16_t tab[1024];
    for (int b = threadIdx.x; b < 1024; b += 256) tab[b] = (uint16_t)narrow_step_entry<FS, FD>((uint32_t)b);
    __syncthreads();
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += stride) {
        const uint4 v = reinterpret_cast<const uint4*>(src)[i];
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
        uint32_t o[2] = {0u, 0u};
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t p = (w[j >> 1] >> (16 * (j & 1))) & 0xFFFFu;
            o[j >> 2] |= narrow_step_apply(tab[p >> 6], p) << (8 * (j & 3));
        }
        reinterpret_cast<uint2*>(dst)[i] = make_uint2(o[0], o[1]);
    }
}

typedef short pnn_short2 __attribute__((ext_vector_type(2)));
typedef unsigned short pnn_ushort2 __attribute__((ext_vector_type(2)));

// |a|, |b| of the two 16-bit integers packed in w (the most negative one stays as it is)
__device__ __forceinline__ uint32_t pk_abs16(uint32_t w) {
    const pnn_short2 v = __builtin_bit_cast(pnn_short2, w);
    const pnn_short2 n = -v;
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(v, n));
}

// Decode table in LDS: pattern -> high word of its binary64 (the low word is zero).  Formats of at most 12 bits
// are indexed by the pattern itself; posit<16,1> by the magnitude pattern 0 .. 2^15 (the sign is put back with one
// more operation), which keeps the table at 128 KB.
template <class F>
struct ValueTable {
    static constexpr bool SIGNED = F::N <= 12;
    static constexpr int ENTRIES = SIGNED ? (1 << F::N) : (1 << (F::N - 1)) + 1;
    __device__ __forceinline__ static void fill(uint32_t* tab, int t, int threads) {
        for (int a = t; a < ENTRIES; a += threads) {
            if constexpr (SIGNED) tab[a] = f64_hi(f64_of_pattern<F>((uint32_t)a));
            else tab[a] = f64_hi_of_magnitude<F>((uint32_t)a);
        }
    }
    __device__ __forceinline__ static uint32_t one(const uint32_t* tab, uint32_t p) {
        p &= F::MASK;
        if constexpr (SIGNED) return tab[p];
        const uint32_t neg = (p >> (F::N - 1)) & 1u;
        return tab[neg ? ((0u - p) & F::MASK) : p] | (neg << 31);
    }
    // the two patterns held in the 16-bit halves of w
    __device__ __forceinline__ static void pair(const uint32_t* tab, uint32_t w, uint32_t& h0, uint32_t& h1) {
        if constexpr (SIGNED) {
            const uint32_t m = w & (F::MASK * 0x10001u);
            h0 = tab[m & 0xFFFFu];
            h1 = tab[m >> 16];
        } else {
            const uint32_t a = pk_abs16(w);
            h0 = tab[a & 0xFFFFu] | ((w << 16) & 0x80000000u);
            h1 = tab[a >> 16] | (w & 0x80000000u);
        }
    }
};

// Narrowed copy of the new y: a direct table for sources of at most 12 bits, the step table for posit<16,1> -> posit<8,0>.
template <class FS, class FD>
struct CopyTable {
    static constexpr bool DIRECT = FS::N <= 12;
    static constexpr int ENTRIES = DIRECT ? (1 << FS::N) : 1024;
    typedef uint16_t Entry;
    __device__ __forceinline__ static void fill(Entry* tab, int t, int threads) {
        for (int i = t; i < ENTRIES; i += threads) {
            if constexpr (DIRECT) tab[i] = (Entry)PositToPosit<FS, FD>()((uint64_t)i);
            else tab[i] = (Entry)narrow_step_entry<FS, FD>((uint32_t)i);
        }
    }
    __device__ __forceinline__ static uint32_t apply(const Entry* tab, uint32_t p) {
        if constexpr (DIRECT) return tab[p];
        else return narrow_step_apply(tab[p >> 6], p);
    }
    // the two patterns in the 16-bit halves of pw at once: their copies come back in the low byte of each half
    // (packed 16-bit arithmetic: thr - (p & 63) is negative exactly when the pattern lies past the step)
    __device__ __forceinline__ static uint32_t apply_pair(const Entry* tab, uint32_t pw) {
        const pnn_ushort2 p = __builtin_bit_cast(pnn_ushort2, pw);
        if constexpr (DIRECT) {
            const pnn_ushort2 r = {tab[p.x], tab[p.y]};
            return __builtin_bit_cast(uint32_t, r);
        } else {
            const pnn_ushort2 idx = p >> 6;
            const pnn_ushort2 ent = {tab[idx.x], tab[idx.y]};
            const pnn_ushort2 past = ((ent >> 8) - (p & 63)) >> 15;
            return __builtin_bit_cast(uint32_t, ent + past);
        }
    }
};

// y[i] = round_FY(y[i] + alpha * x[i]); yc[i] = round_FC(new y[i]) when COPY.  Eight elements per thread and step
// (y in 16-bit containers, x in 16- or 8-bit ones); the tensor is walked in a grid-stride loop, the loads of the
// next step issued before the current one is computed.  Zero and NaN results (rare) are patched in after the
// straight-line part, under one wave-wide test per step.
template <class FX, class FY, class FC, bool COPY, int THREADS>
__global__ __launch_bounds__(THREADS) void axpy_f64_kernel(const typename Storage<FX::N>::T* __restrict__ x,
                                                           typename Storage<FY::N>::T* __restrict__ y,
                                                           typename Storage<FC::N>::T* __restrict__ yc, int64_t nvec, uint32_t alpha) {
    typedef typename Storage<FX::N>::T TX;
    typedef typename Storage<FY::N>::T TY;
    typedef typename Storage<FC::N>::T TC;
    static_assert(sizeof(TY) == 2 && sizeof(TC) <= 2 && (sizeof(TX) == 2 || FX::N == 8), "container sizes");
    constexpr bool SAME = FX::N == FY::N && FX::ES == FY::ES;
    constexpr int XW = sizeof(TX) == 2 ? 4 : 2;  // 32-bit words of x per step
    __shared__ uint32_t tabY[ValueTable<FY>::ENTRIES];
    __shared__ uint32_t tabX[SAME ? 1 : ValueTable<FX>::ENTRIES];
    __shared__ typename CopyTable<FY, FC>::Entry tabC[COPY ? CopyTable<FY, FC>::ENTRIES : 1];
    const int t = threadIdx.x;
    ValueTable<FY>::fill(tabY, t, THREADS);
    if constexpr (!SAME) ValueTable<FX>::fill(tabX, t, THREADS);
    if constexpr (COPY) CopyTable<FY, FC>::fill(tabC, t, THREADS);
    __syncthreads();
    const uint32_t* tx = SAME ? tabY : tabX;
    const double ad = f64_from_words(ValueTable<FY>::one(tabY, alpha), 0u);
    const int64_t stride = (int64_t)gridDim.x * THREADS;
    typedef Pack<uint32_t, XW> XV;
    typedef Pack<uint32_t, 4> YV;
    // one step: the update of vector i from its already loaded operands
    auto step = [&](int64_t i, const XV& xv, const YV& yv) {
        uint32_t shi[8], pw[4];  // pw: the new patterns, two per word
        bool any_special = false;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            uint32_t xh[2], yh[2], body[2];
            if constexpr (sizeof(TX) == 2) {
                ValueTable<FX>::pair(tx, xv.v[q], xh[0], xh[1]);
            } else {  // bytes 2q, 2q+1 of the eight; an 8-bit format's table is indexed by the pattern itself
                xh[0] = tx[(xv.v[q >> 1] >> (16 * (q & 1))) & 0xFFu];
                xh[1] = tx[(xv.v[q >> 1] >> (16 * (q & 1) + 8)) & 0xFFu];
            }
            ValueTable<FY>::pair(tabY, yv.v[q], yh[0], yh[1]);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                bool special;
                body[h] = axpy_f64_core<FY, false>(ad, f64_from_words(xh[h], 0u), f64_from_words(yh[h], 0u), shi[2 * q + h], special);
                any_special = any_special || special;
            }
            // the signs of both at once: negative values take the two's complement of the magnitude pattern
            const pnn_short2 sm = __builtin_bit_cast(pnn_short2, __builtin_amdgcn_perm(shi[2 * q + 1], shi[2 * q], 0x07060302u)) >> 15;
            const pnn_short2 mag = __builtin_bit_cast(pnn_short2, body[0] | (body[1] << 16));
            pw[q] = __builtin_bit_cast(uint32_t, (mag ^ sm) - sm) & (FY::MASK * 0x10001u);
        }
        if (__builtin_amdgcn_ballot_w64(any_special) != 0) {  // some lane of the wave met a zero or a NaN: patch those results
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint32_t ah = shi[j] & 0x7FFFFFFFu;
                const uint32_t keep = 0xFFFF0000u >> (16 * (j & 1));
                if (ah == 0u) pw[j >> 1] &= keep;
                else if (ah >= 0x7FF00000u) pw[j >> 1] = (pw[j >> 1] & keep) | (FY::NAR << (16 * (j & 1)));
            }
        }
        reinterpret_cast<Pack<uint32_t, 4>*>(y)[i] = Pack<uint32_t, 4>{{pw[0], pw[1], pw[2], pw[3]}};
        if constexpr (COPY) {
            uint32_t c[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) c[q] = CopyTable<FY, FC>::apply_pair(tabC, pw[q]);
            if constexpr (sizeof(TC) == 1) {  // bytes 0 and 2 of each pair word
                reinterpret_cast<Pack<uint32_t, 2>*>(yc)[i] =
                    Pack<uint32_t, 2>{{__builtin_amdgcn_perm(c[1], c[0], 0x06040200u), __builtin_amdgcn_perm(c[3], c[2], 0x06040200u)}};
            } else {
                constexpr uint32_t m = FC::MASK * 0x10001u;
                reinterpret_cast<Pack<uint32_t, 4>*>(yc)[i] = Pack<uint32_t, 4>{{c[0] & m, c[1] & m, c[2] & m, c[3] & m}};
            }
        }
    };
    // Two vectors in flight per thread: the loads of one are issued before the other is computed (a thread's
    // vectors i, i + stride, ... never overlap another thread's, so loading ahead of the stores is safe).
    int64_t i = (int64_t)blockIdx.x * THREADS + t;
    if (i >= nvec) return;
    XV xa = reinterpret_cast<const XV*>(x)[i];
    YV ya = reinterpret_cast<const YV*>(y)[i];
    for (;;) {
        const int64_t ib = i + stride;
        const bool more_b = ib < nvec;
        XV xb;
        YV yb;
        if (more_b) {
            xb = reinterpret_cast<const XV*>(x)[ib];
            yb = reinterpret_cast<const YV*>(y)[ib];
        }
        step(i, xa, ya);
        if (!more_b) break;
        i = ib + stride;
        const bool more_a = i < nvec;
        if (more_a) {
            xa = reinterpret_cast<const XV*>(x)[i];
            ya = reinterpret_cast<const YV*>(y)[i];
        }
        step(ib, xb, yb);
        if (!more_a) break;
    }
}

#endif  // __HIPCC__

}  // namespace pnn
