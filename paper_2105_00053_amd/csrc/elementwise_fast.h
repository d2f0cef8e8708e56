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

// One rounding of an exact real number to posit<N,ES>, N <= 16.  The number is given as the
// binary64 s plus a flag pair describing what s misses: `inexact` (the exact value differs from s,
// by less than one unit of s's last place) and `toward_zero` (the exact magnitude is the smaller one).
// NaN gives NaR, zero gives zero, everything else is rounded to nearest with ties to the even
// pattern and clamped to [minpos, maxpos].
//
// The string  regime | exponent | fraction  is produced without a table of regimes: with
// k = floor(scale / 2^ES), kk = k for k >= 0 and -k-1 otherwise, an arithmetic right shift by kk of
// "10" followed by the exponent and fraction bits yields kk+1 ones, a zero and the rest; for negative
// k the tail is complemented before and the whole word after the shift, which turns that head into
// kk+1 zeros and a one.  Bits that the cut cannot reach are folded into one bit that no shift here
// pushes out (bit N of the tail), so the sticky information survives in a single word.
template <class F>
PNN_HD uint32_t round_f64_to_posit(double s, bool inexact, bool toward_zero) {
    static_assert(F::N <= 16, "formats of at most 16 bits");
    constexpr int N = F::N, ES = F::ES;
    constexpr uint32_t MAXHI = (uint32_t)(1023 + F::MAXS) << 20, MINHI = (uint32_t)(1023 - F::MAXS) << 20;
    uint32_t hi = f64_hi(s);
    const uint32_t lo = f64_lo(s);
    const uint32_t sm = (uint32_t)((int32_t)hi >> 31);  // all ones for a negative value
    // the exact magnitude lies just below |s|: when s's low word is zero that borrows from the high word
    hi -= (toward_zero && lo == 0u) ? 1u : 0u;
    const uint32_t ah0 = hi & 0x7FFFFFFFu;
    // beyond the format's range only the clamped scale matters: the guard bit of a clamped value is zero
    const uint32_t ah = ah0 < MINHI ? MINHI : (ah0 > MAXHI ? MAXHI : ah0);
    const uint32_t h1 = ah + (1u << 20);  // exponent field + 1 = scale + 1024: its low ES bits are the exponent bits
    const int k = (int)(h1 >> (20 + ES)) - (1024 >> ES);
    const uint32_t sg = (uint32_t)(k >> 31);
    const uint32_t kk = (uint32_t)k ^ sg;
    const uint32_t tail = funnel_shr(h1, lo, 20 + ES);  // exponent bits, then the significand's fraction
    const uint32_t below = (tail & ((1u << N) - 1u)) | (lo << (12 - ES));
    const uint32_t jam = (below != 0u || inexact) ? (1u << N) : 0u;
    const uint32_t w = funnel_shr(2u, (tail | jam) ^ sg, 2);
    const uint32_t x = (uint32_t)((int32_t)w >> kk) ^ sg;
    const uint32_t lsb = (x >> (33 - N)) & 1u;
    const uint32_t body = (x + ((1u << (32 - N)) - 1u) + lsb) >> (33 - N);
    const uint32_t pat = ((body ^ sm) - sm) & F::MASK;
    return ah0 > 0x7FF00000u ? F::NAR : (ah0 == 0u ? 0u : pat);
}

// y + alpha * x, exactly, rounded once to FY.  xd, yd, ad: the operands as binary64 (NaN for NaR).
template <class FY>
PNN_HD uint32_t axpy_f64(double ad, double xd, double yd) {
    const double t = ad * xd;      // at most 26 significant bits: exact
    const double s = t + yd;
    const double bb = s - t;       // error-free transformation of the sum: s + err == t + yd exactly
    const double err = (t - (s - bb)) + (yd - bb);
    const bool inexact = err != 0.0;
    const bool toward_zero = inexact && (((f64_hi(s) ^ f64_hi(err)) >> 31) != 0u);
    return round_f64_to_posit<FY>(s, inexact, toward_zero);
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

// Decode table in LDS: magnitude pattern -> high word of its binary64.
template <class F>
struct MagnitudeTable {
    static constexpr int ENTRIES = (1 << (F::N - 1)) + 1;
    __device__ __forceinline__ static void fill(uint32_t* tab, int t, int threads) {
        for (int a = t; a < ENTRIES; a += threads) tab[a] = f64_hi_of_magnitude<F>((uint32_t)a);
    }
    // value of a signed pattern held in the low N bits of p
    __device__ __forceinline__ static double value(const uint32_t* tab, uint32_t p) {
        const uint32_t neg = (p >> (F::N - 1)) & 1u;
        const uint32_t a = neg ? ((0u - p) & F::MASK) : p;
        return f64_from_words(tab[a] | (neg << 31), 0u);
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
};

// y[i] = round_FY(y[i] + alpha * x[i]); yc[i] = round_FC(new y[i]) when COPY.  V elements of 16 bits (x may be 8-bit)
// per thread and step; the tensor is walked in a grid-stride loop by one workgroup per compute unit.
template <class FX, class FY, class FC, bool COPY, int THREADS>
__global__ __launch_bounds__(THREADS) void axpy_f64_kernel(const typename Storage<FX::N>::T* __restrict__ x,
                                                           typename Storage<FY::N>::T* __restrict__ y,
                                                           typename Storage<FC::N>::T* __restrict__ yc, int64_t nvec, uint32_t alpha) {
    typedef typename Storage<FX::N>::T TX;
    typedef typename Storage<FY::N>::T TY;
    typedef typename Storage<FC::N>::T TC;
    static_assert(sizeof(TY) == 2 && sizeof(TC) <= 2, "the updated tensor is held in 16-bit containers");
    constexpr int V = 8;
    constexpr bool SAME = FX::N == FY::N && FX::ES == FY::ES;
    __shared__ uint32_t tabY[MagnitudeTable<FY>::ENTRIES];
    __shared__ uint32_t tabX[SAME ? 1 : MagnitudeTable<FX>::ENTRIES];
    __shared__ typename CopyTable<FY, FC>::Entry tabC[COPY ? CopyTable<FY, FC>::ENTRIES : 1];
    const int t = threadIdx.x;
    MagnitudeTable<FY>::fill(tabY, t, THREADS);
    if constexpr (!SAME) MagnitudeTable<FX>::fill(tabX, t, THREADS);
    if constexpr (COPY) CopyTable<FY, FC>::fill(tabC, t, THREADS);
    __syncthreads();
    const uint32_t* tx = SAME ? tabY : tabX;
    const double ad = MagnitudeTable<FY>::value(tabY, alpha & FY::MASK);
    const int64_t stride = (int64_t)gridDim.x * THREADS;
    for (int64_t i = (int64_t)blockIdx.x * THREADS + t; i < nvec; i += stride) {
        const Pack<TX, V> xv = reinterpret_cast<const Pack<TX, V>*>(x)[i];
        Pack<TY, V> yv = reinterpret_cast<Pack<TY, V>*>(y)[i];
        Pack<TC, V> cv;
#pragma unroll
        for (int j = 0; j < V; ++j) {
            const double xd = MagnitudeTable<FX>::value(tx, (uint32_t)xv.v[j] & FX::MASK);
            const double yd = MagnitudeTable<FY>::value(tabY, (uint32_t)yv.v[j] & FY::MASK);
            const uint32_t r = axpy_f64<FY>(ad, xd, yd);
            yv.v[j] = (TY)r;
            if constexpr (COPY) cv.v[j] = (TC)CopyTable<FY, FC>::apply(tabC, r);
        }
        reinterpret_cast<Pack<TY, V>*>(y)[i] = yv;
        if constexpr (COPY) reinterpret_cast<Pack<TC, V>*>(yc)[i] = cv;
    }
}

#endif  // __HIPCC__

}  // namespace pnn
