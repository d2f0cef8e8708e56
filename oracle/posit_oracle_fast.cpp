// Plain C++17 CPU oracle for quire-exact posit arithmetic (PositNN, arXiv 2105.00053).
//
// TEST INFRASTRUCTURE ONLY.  Second, faster statement of what the Python oracle
// defines, so that matrices of 1024^3 and more can be checked in full and timed.
// It is validated against the Python oracle and shares no code with the HIP
// library: different decode (bit-by-bit scan), different accumulator (one
// 1024-bit two's-complement integer for every format, narrowed to the quire
// width only at the end), different rounding (emits the unbounded
// regime|exponent|fraction string one bit at a time).
//
// Passages followed: decode = Sec. 2, Eq. 2; formats and quire widths = Table 1;
// quire accumulation in matrix products and convolutions, one rounding =
// Sec. 3.3; hand-written backward passes = Sec. 3.1; tensor conversion, SGD =
// Fig. 2; worker threads split the rows of the left operand = Sec. 3.3.
// Readings where the paper is silent are those of the Python oracle (modular
// quire, NaR absorbing, bias inside the quire, truncated exponent bits are 0,
// padded positions are zero operands of the forward and weight-gradient passes,
// filter taps that reach no output position are no terms of the input gradient; with the quire
// switched off, Sec. 3.3 / Table 2, every product and running sum is rounded,
// terms in order of the reduction index, bias last).
//
// Pins: agreement with the Python oracle on every entry point (tests), which is
// itself pinned to the definition.  Not tuned: no blocking, no SIMD, no tables.

#include <cmath>
#include <cstdint>
#include <cstring>
#include <functional>
#include <thread>
#include <vector>

namespace {

struct Format {
    int n, es, qbits;
    int max_scale() const { return (n - 2) << es; }  // log2(maxpos) = -log2(minpos)
};

bool format_of(int code, Format* f) {
    switch (code) {
        case 0: *f = {8, 0, 32}; return true;
        case 1: *f = {16, 1, 128}; return true;
        case 2: *f = {32, 2, 512}; return true;
        // pairs outside Table 1: 4(n-2)2^es + 1 + (n-1) bits rounded up to 32-bit limbs
        case 3: *f = {8, 1, 64}; return true;
        case 4: *f = {8, 2, 128}; return true;
        case 5: *f = {10, 1, 96}; return true;
        case 6: *f = {10, 2, 160}; return true;
        case 7: *f = {12, 1, 96}; return true;
        case 8: *f = {12, 2, 192}; return true;
    }
    return false;
}

// value = (neg ? -1 : 1) * sig * 2^sh * minpos, sh >= 0
struct Decoded {
    bool nar = false, zero = false, neg = false;
    uint64_t sig = 0;
    int sh = 0;
};

Decoded decode(uint32_t p, const Format& f) {
    Decoded d;
    const uint32_t mask = f.n == 32 ? 0xFFFFFFFFu : ((1u << f.n) - 1u);
    p &= mask;
    if (p == 0) { d.zero = true; return d; }
    if (p == (1u << (f.n - 1))) { d.nar = true; return d; }
    d.neg = (p >> (f.n - 1)) & 1u;
    if (d.neg) p = (0u - p) & mask;  // two's complement before the fields are read
    int pos = f.n - 2;               // walk down from the bit below the sign
    const int r = (p >> pos) & 1;
    int run = 0;
    while (pos >= 0 && (int)((p >> pos) & 1) == r) { ++run; --pos; }
    --pos;  // the bit that ended the run (absent when the run reached bit 0)
    const int k = r ? run - 1 : -run;
    int e = 0;
    for (int i = 0; i < f.es; ++i) {  // exponent bits that were cut off read as 0
        e <<= 1;
        if (pos >= 0) { e |= (p >> pos) & 1; --pos; }
    }
    int nf = 0;
    uint64_t frac = 0;
    while (pos >= 0) { frac = (frac << 1) | ((p >> pos) & 1); ++nf; --pos; }
    const int scale = k * (1 << f.es) + e;
    d.sig = (uint64_t(1) << nf) | frac;  // 1.fraction as an integer
    d.sh = scale - nf + f.max_scale();   // every posit is a whole number of minpos, so sh >= 0
    return d;
}

// 1024-bit two's-complement integer, little-endian 64-bit words.
struct Big {
    static const int W = 16;
    uint64_t w[W];
    Big() { std::memset(w, 0, sizeof w); }
    bool negative() const { return w[W - 1] >> 63; }
    bool is_zero() const {
        for (int i = 0; i < W; ++i) if (w[i]) return false;
        return true;
    }
    int bit(int i) const { return (i < 0 || i >= 64 * W) ? 0 : int((w[i >> 6] >> (i & 63)) & 1); }
    void add(const Big& o) {
        unsigned carry = 0;
        for (int i = 0; i < W; ++i) {
            unsigned __int128 s = (unsigned __int128)w[i] + o.w[i] + carry;
            w[i] = (uint64_t)s;
            carry = (unsigned)(s >> 64);
        }
    }
    void negate() {
        for (int i = 0; i < W; ++i) w[i] = ~w[i];
        Big one; one.w[0] = 1; add(one);
    }
    // this += (neg ? -1 : 1) * v * 2^shift : add or subtract the two words the
    // shifted value occupies, then let the carry / borrow run upwards
    void add_shifted(uint64_t v, int shift, bool neg) {
        const int wi = shift >> 6, bi = shift & 63;
        const uint64_t part[2] = {v << bi, bi ? v >> (64 - bi) : 0};
        unsigned carry = 0;
        for (int i = wi; i < W; ++i) {
            const uint64_t t = (i - wi) < 2 ? part[i - wi] : 0;
            if (i - wi >= 2 && !carry) break;
            if (!neg) {
                unsigned __int128 s = (unsigned __int128)w[i] + t + carry;
                w[i] = (uint64_t)s;
                carry = (unsigned)(s >> 64);
            } else {
                unsigned __int128 s = (unsigned __int128)w[i] - t - carry;
                w[i] = (uint64_t)s;
                carry = (unsigned)((s >> 64) & 1);
            }
        }
    }
    // keep the low `bits` bits and sign-extend from the top one of them
    void wrap(int bits) {
        const int top = bits - 1;
        const int s = bit(top);
        for (int i = bits; i < 64 * W; ++i) {
            uint64_t m = uint64_t(1) << (i & 63);
            if (s) w[i >> 6] |= m; else w[i >> 6] &= ~m;
        }
    }
    bool fits(int bits) const {  // value representable in `bits`-bit two's complement
        const int s = bit(bits - 1);
        for (int i = bits; i < 64 * W; ++i) if (bit(i) != s) return false;
        return true;
    }
};

// Round  (neg ? -1 : 1) * mag * 2^lsb_log2  (mag >= 0 as a Big) to posit `f`.
uint32_t round_big(bool neg, const Big& mag, int lsb_log2, const Format& f) {
    const uint32_t mask = f.n == 32 ? 0xFFFFFFFFu : ((1u << f.n) - 1u);
    int top = -1;
    for (int i = 64 * Big::W - 1; i >= 0; --i) if (mag.bit(i)) { top = i; break; }
    if (top < 0) return 0;
    const int scale = top + lsb_log2;  // |x| = 2^scale * 1.fraction, fraction = bits top-1 .. 0
    bool frac_nonzero = false;
    for (int i = top - 1; i >= 0; --i) if (mag.bit(i)) { frac_nonzero = true; break; }
    const int ms = f.max_scale();
    uint32_t body;
    if (scale >= ms) {
        body = (1u << (f.n - 1)) - 1u;  // >= maxpos
    } else if (scale < -ms || (scale == -ms && !frac_nonzero)) {
        body = 1u;  // <= minpos, never to zero
    } else {
        const int k = (int)std::floor((double)scale / (1 << f.es));
        const int e = scale - k * (1 << f.es);
        const int rlen = k >= 0 ? k + 2 : -k + 1;
        // i-th bit (0 = first) of regime | exponent | fraction | 000...
        auto sbit = [&](int i) -> int {
            if (i < rlen) return k >= 0 ? (i < k + 1 ? 1 : 0) : (i < -k ? 0 : 1);
            i -= rlen;
            if (i < f.es) return (e >> (f.es - 1 - i)) & 1;
            i -= f.es;
            return mag.bit(top - 1 - i);
        };
        const int keep = f.n - 1;
        body = 0;
        for (int i = 0; i < keep; ++i) body = (body << 1) | (uint32_t)sbit(i);
        const int guard = sbit(keep);
        bool sticky = false;
        const int total = rlen + f.es + top;  // bits that can be nonzero
        for (int i = keep + 1; i < total; ++i) if (sbit(i)) { sticky = true; break; }
        if (guard && (sticky || (body & 1u))) body += 1;
    }
    return neg ? ((0u - body) & mask) : body;
}

// quire content (already a Big in units of minpos_in^2) -> posit in fout
uint32_t round_quire(Big q, const Format& fin, const Format& fout) {
    q.wrap(fin.qbits);
    const bool neg = q.negative();
    if (neg) q.negate();
    return round_big(neg, q, -2 * fin.max_scale(), fout);
}

// containers: 8 bits -> uint8, 10 / 12 / 16 bits -> uint16 (pattern in the low bits), 32 -> uint32
uint32_t load(const void* p, int64_t i, const Format& f) {
    if (f.n <= 8) return ((const uint8_t*)p)[i];
    if (f.n <= 16) return ((const uint16_t*)p)[i];
    return ((const uint32_t*)p)[i];
}
void store(void* p, int64_t i, uint32_t v, const Format& f) {
    if (f.n <= 8) ((uint8_t*)p)[i] = (uint8_t)v;
    else if (f.n <= 16) ((uint16_t*)p)[i] = (uint16_t)v;
    else ((uint32_t*)p)[i] = v;
}
uint32_t nar_of(const Format& f) { return 1u << (f.n - 1); }

// Posit Standard arithmetic on patterns, used when the quire is switched off (Sec. 3.3 makes it an
// option; Table 2 trains without it): the exact product / sum rounded once.
uint32_t mul_posit(const Decoded& a, const Decoded& b, const Format& f) {
    if (a.nar || b.nar) return nar_of(f);
    if (a.zero || b.zero) return 0;
    Big prod;  // a.sig * b.sig by shift-and-add over the bits of b.sig
    for (int i = 0; i < 64; ++i)
        if ((b.sig >> i) & 1) prod.add_shifted(a.sig, i, false);
    return round_big(a.neg != b.neg, prod, a.sh + b.sh - 2 * f.max_scale(), f);
}

uint32_t add_posit(uint32_t x, uint32_t y, const Format& f) {
    const Decoded a = decode(x, f), b = decode(y, f);
    if (a.nar || b.nar) return nar_of(f);
    Big t;  // in units of minpos
    if (!a.zero) t.add_shifted(a.sig, a.sh, a.neg);
    if (!b.zero) t.add_shifted(b.sig, b.sh, b.neg);
    const bool neg = t.negative();
    if (neg) t.negate();
    return round_big(neg, t, -f.max_scale(), f);
}

uint32_t convert_posit(uint32_t x, const Format& fs, const Format& fd) {
    const Decoded d = decode(x, fs);
    if (d.nar) return nar_of(fd);
    if (d.zero) return 0;
    Big m;
    m.w[0] = d.sig;
    return round_big(d.neg, m, d.sh - fs.max_scale(), fd);
}

// One output's accumulation.  With the quire: an exact sum in units of minpos^2, rounded once by
// result().  Without it: a running posit of format fin, every product and every sum rounded as it
// is formed, terms in the order they are offered.
struct Accum {
    const Format& f;
    const bool noquire;
    Big q;
    bool nar = false;
    uint32_t run = 0;
    Accum(const Format& fin, int noquire_) : f(fin), noquire(noquire_ != 0) {}
    void mac(const Decoded& a, const Decoded& b) {
        if (noquire) { run = add_posit(run, mul_posit(a, b, f), f); return; }
        if (a.nar || b.nar) { nar = true; return; }
        if (a.zero || b.zero) return;
        q.add_shifted(a.sig * b.sig, a.sh + b.sh, a.neg != b.neg);
    }
    void add_one_times(const Decoded& a) {  // + a * 1
        Decoded one;
        one.sig = 1;
        one.sh = f.max_scale();  // the value one is 2^max_scale minpos
        if (noquire) { run = add_posit(run, mul_posit(a, one, f), f); return; }
        if (a.nar) { nar = true; return; }
        if (a.zero) return;
        q.add_shifted(a.sig, a.sh + f.max_scale(), a.neg);
    }
    bool overflowed() const { return !noquire && !nar && !q.fits(f.qbits); }
    uint32_t result(const Format& fout) const {
        if (noquire) return convert_posit(run, f, fout);
        return nar ? nar_of(fout) : round_quire(q, f, fout);
    }
};

// Worker threads split [0, rows) into contiguous chunks.
void parallel_rows(int64_t rows, int nthreads, const std::function<void(int64_t, int64_t)>& fn) {
    if (nthreads < 1) nthreads = 1;
    if (rows < nthreads) nthreads = rows > 0 ? (int)rows : 1;
    std::vector<std::thread> th;
    const int64_t chunk = (rows + nthreads - 1) / nthreads;
    for (int t = 0; t < nthreads; ++t) {
        const int64_t lo = t * chunk, hi = std::min<int64_t>(rows, lo + chunk);
        if (lo >= hi) break;
        th.emplace_back(fn, lo, hi);
    }
    for (auto& x : th) x.join();
}

std::vector<Decoded> decode_all(const void* p, int64_t count, const Format& f) {
    std::vector<Decoded> v((size_t)count);
    for (int64_t i = 0; i < count; ++i) v[(size_t)i] = decode(load(p, i, f), f);
    return v;
}

struct Conv {
    int64_t N, C, H, W, K, R, S, ph, pw, sh, sw, OH, OW;
};

Decoded make_zero() { Decoded d; d.zero = true; return d; }
const Decoded zero = make_zero();

}  // namespace

extern "C" {

int oracle_hw_threads() {
    unsigned n = std::thread::hardware_concurrency();
    return n ? (int)n : 1;
}

// C[M,N] = round_fout( op(A)[M,K] * op(B)[K,N] (+ bias[N]) ); row-major, ld in elements.
// Only rows [row_lo, row_hi) of C are computed (for sampled checks and timing).
// overflowed (nullable) receives the number of outputs whose exact sum left the quire range.
// noquire != 0 (here and in the convolutions): no quire, every product and partial sum is rounded
// to fin as it is formed, k ascending, bias last; the final posit is converted to fout.
int oracle_gemm(int fin_c, int fout_c, int transA, int transB, int64_t M, int64_t N, int64_t K,
                const void* A, int64_t lda, const void* B, int64_t ldb, const void* bias,
                void* C, int64_t ldc, int64_t row_lo, int64_t row_hi, int nthreads, int64_t* overflowed, int noquire) {
    Format fin, fout;
    if (!format_of(fin_c, &fin) || !format_of(fout_c, &fout)) return 1;
    if (row_lo < 0) row_lo = 0;
    if (row_hi > M) row_hi = M;
    // decode op(B) once, column-major so that the k loop walks memory
    std::vector<Decoded> Bd((size_t)(K * N));
    for (int64_t k = 0; k < K; ++k)
        for (int64_t j = 0; j < N; ++j)
            Bd[(size_t)(j * K + k)] = decode(load(B, transB ? j * ldb + k : k * ldb + j, fin), fin);
    std::vector<Decoded> biasd;
    if (bias) biasd = decode_all(bias, N, fin);
    int64_t total_ovf = 0;
    parallel_rows(row_hi - row_lo, nthreads, [&](int64_t lo, int64_t hi) {
        int64_t local = 0;
        std::vector<Decoded> arow((size_t)K);
        for (int64_t i = row_lo + lo; i < row_lo + hi; ++i) {
            for (int64_t k = 0; k < K; ++k) arow[(size_t)k] = decode(load(A, transA ? k * lda + i : i * lda + k, fin), fin);
            for (int64_t j = 0; j < N; ++j) {
                Accum acc(fin, noquire);
                for (int64_t k = 0; k < K; ++k) acc.mac(arow[(size_t)k], Bd[(size_t)(j * K + k)]);
                if (bias) acc.add_one_times(biasd[(size_t)j]);
                if (acc.overflowed()) ++local;
                store(C, i * ldc + j, acc.result(fout), fout);
            }
        }
        __atomic_fetch_add(&total_ovf, local, __ATOMIC_RELAXED);
    });
    if (overflowed) *overflowed = total_ovf;
    return 0;
}

// y[n,k,oh,ow] = round( sum_{c,r,s} x[n,c,oh*sh+r-ph,ow*sw+s-pw] * w[k,c,r,s] (+ bias[k]) ), NCHW / OIHW
int oracle_conv2d_fwd(int fin_c, int fout_c, const int64_t* d, const void* x, const void* w, const void* bias,
                      void* y, int nthreads, int noquire) {
    Format fin, fout;
    if (!format_of(fin_c, &fin) || !format_of(fout_c, &fout)) return 1;
    Conv c{d[0], d[1], d[2], d[3], d[4], d[5], d[6], d[7], d[8], d[9], d[10], 0, 0};
    c.OH = (c.H + 2 * c.ph - c.R) / c.sh + 1;
    c.OW = (c.W + 2 * c.pw - c.S) / c.sw + 1;
    auto xd = decode_all(x, c.N * c.C * c.H * c.W, fin);
    auto wd = decode_all(w, c.K * c.C * c.R * c.S, fin);
    std::vector<Decoded> bd;
    if (bias) bd = decode_all(bias, c.K, fin);
    parallel_rows(c.N * c.K, nthreads, [&](int64_t lo, int64_t hi) {
        for (int64_t nk = lo; nk < hi; ++nk) {
            const int64_t n = nk / c.K, k = nk % c.K;
            for (int64_t oh = 0; oh < c.OH; ++oh)
                for (int64_t ow = 0; ow < c.OW; ++ow) {
                    Accum acc(fin, noquire);
                    for (int64_t ci = 0; ci < c.C; ++ci)
                        for (int64_t r = 0; r < c.R; ++r) {
                            const int64_t ih = oh * c.sh + r - c.ph;
                            for (int64_t s = 0; s < c.S; ++s) {
                                const int64_t iw = ow * c.sw + s - c.pw;
                                const bool inside = ih >= 0 && ih < c.H && iw >= 0 && iw < c.W;
                                // a padded position holds zero and is an operand like any other
                                acc.mac(inside ? xd[(size_t)(((n * c.C + ci) * c.H + ih) * c.W + iw)] : zero,
                                    wd[(size_t)(((k * c.C + ci) * c.R + r) * c.S + s)]);
                            }
                        }
                    if (bias) acc.add_one_times(bd[(size_t)k]);
                    store(y, ((n * c.K + k) * c.OH + oh) * c.OW + ow, acc.result(fout), fout);
                }
        }
    });
    return 0;
}

// dx[n,c,h,w] = round( sum over (k,r,s) and the (oh,ow) that read x[n,c,h,w] of dy[n,k,oh,ow] * w[k,c,r,s] )
int oracle_conv2d_bwd_data(int fin_c, int fout_c, const int64_t* d, const void* dy, const void* w, void* dx, int nthreads, int noquire) {
    Format fin, fout;
    if (!format_of(fin_c, &fin) || !format_of(fout_c, &fout)) return 1;
    Conv c{d[0], d[1], d[2], d[3], d[4], d[5], d[6], d[7], d[8], d[9], d[10], 0, 0};
    c.OH = (c.H + 2 * c.ph - c.R) / c.sh + 1;
    c.OW = (c.W + 2 * c.pw - c.S) / c.sw + 1;
    auto dyd = decode_all(dy, c.N * c.K * c.OH * c.OW, fin);
    auto wd = decode_all(w, c.K * c.C * c.R * c.S, fin);
    parallel_rows(c.N * c.C, nthreads, [&](int64_t lo, int64_t hi) {
        for (int64_t nc = lo; nc < hi; ++nc) {
            const int64_t n = nc / c.C, ci = nc % c.C;
            for (int64_t h = 0; h < c.H; ++h)
                for (int64_t ww = 0; ww < c.W; ++ww) {
                    Accum acc(fin, noquire);
                    for (int64_t k = 0; k < c.K; ++k)
                        for (int64_t r = 0; r < c.R; ++r) {
                            const int64_t t = h + c.ph - r;
                            const bool row_ok = t >= 0 && t % c.sh == 0 && t / c.sh < c.OH;
                            for (int64_t s = 0; s < c.S; ++s) {
                                const int64_t u = ww + c.pw - s;
                                const bool ok = row_ok && u >= 0 && u % c.sw == 0 && u / c.sw < c.OW;
                                if (!ok) continue;  // no output position reads x[n,c,h,w] through this tap: not a term of the sum
                                acc.mac(dyd[(size_t)(((n * c.K + k) * c.OH + t / c.sh) * c.OW + u / c.sw)],
                                    wd[(size_t)(((k * c.C + ci) * c.R + r) * c.S + s)]);
                            }
                        }
                    store(dx, ((n * c.C + ci) * c.H + h) * c.W + ww, acc.result(fout), fout);
                }
        }
    });
    return 0;
}

// dw[k,c,r,s] = round( sum_{n,oh,ow} dy[n,k,oh,ow] * x[n,c,oh*sh+r-ph,ow*sw+s-pw] ); dbias[k] = round( sum dy[n,k,:,:] )
int oracle_conv2d_bwd_weight(int fin_c, int fout_c, const int64_t* d, const void* dy, const void* x, void* dw,
                             void* dbias, int nthreads, int noquire) {
    Format fin, fout;
    if (!format_of(fin_c, &fin) || !format_of(fout_c, &fout)) return 1;
    Conv c{d[0], d[1], d[2], d[3], d[4], d[5], d[6], d[7], d[8], d[9], d[10], 0, 0};
    c.OH = (c.H + 2 * c.ph - c.R) / c.sh + 1;
    c.OW = (c.W + 2 * c.pw - c.S) / c.sw + 1;
    auto dyd = decode_all(dy, c.N * c.K * c.OH * c.OW, fin);
    auto xd = decode_all(x, c.N * c.C * c.H * c.W, fin);
    parallel_rows(c.K * c.C, nthreads, [&](int64_t lo, int64_t hi) {
        for (int64_t kc = lo; kc < hi; ++kc) {
            const int64_t k = kc / c.C, ci = kc % c.C;
            for (int64_t r = 0; r < c.R; ++r)
                for (int64_t s = 0; s < c.S; ++s) {
                    Accum acc(fin, noquire);
                    for (int64_t n = 0; n < c.N; ++n)
                        for (int64_t oh = 0; oh < c.OH; ++oh) {
                            const int64_t ih = oh * c.sh + r - c.ph;
                            for (int64_t ow = 0; ow < c.OW; ++ow) {
                                const int64_t iw = ow * c.sw + s - c.pw;
                                const bool inside = ih >= 0 && ih < c.H && iw >= 0 && iw < c.W;
                                acc.mac(dyd[(size_t)(((n * c.K + k) * c.OH + oh) * c.OW + ow)],
                                    inside ? xd[(size_t)(((n * c.C + ci) * c.H + ih) * c.W + iw)] : zero);
                            }
                        }
                    store(dw, ((k * c.C + ci) * c.R + r) * c.S + s, acc.result(fout), fout);
                }
        }
    });
    if (dbias) {
        for (int64_t k = 0; k < c.K; ++k) {
            Accum acc(fin, noquire);
            for (int64_t n = 0; n < c.N; ++n)
                for (int64_t i = 0; i < c.OH * c.OW; ++i)
                    acc.add_one_times(dyd[(size_t)((n * c.K + k) * c.OH * c.OW + i)]);
            store(dbias, k, acc.result(fout), fout);
        }
    }
    return 0;
}

// IEEE binary64 -> posit (binary32 inputs are widened exactly by the caller side of this file)
static uint32_t round_double(double v, const Format& f) {
    if (std::isnan(v) || std::isinf(v)) return nar_of(f);
    if (v == 0.0) return 0;
    uint64_t bits;
    std::memcpy(&bits, &v, 8);
    const bool neg = bits >> 63;
    const int ex = int((bits >> 52) & 0x7FF);
    uint64_t man = bits & ((uint64_t(1) << 52) - 1);
    int lsb;
    if (ex == 0) lsb = -1074; else { man |= uint64_t(1) << 52; lsb = ex - 1075; }
    Big m;
    m.w[0] = man;
    return round_big(neg, m, lsb, f);
}

int oracle_round_f32(int fdst_c, int64_t n, const float* src, void* dst) {
    Format f;
    if (!format_of(fdst_c, &f)) return 1;
    for (int64_t i = 0; i < n; ++i) store(dst, i, round_double((double)src[i], f), f);
    return 0;
}

int oracle_round_f64(int fdst_c, int64_t n, const double* src, void* dst) {
    Format f;
    if (!format_of(fdst_c, &f)) return 1;
    for (int64_t i = 0; i < n; ++i) store(dst, i, round_double(src[i], f), f);
    return 0;
}

int oracle_convert(int fsrc_c, int fdst_c, int64_t n, const void* src, void* dst) {
    Format fs, fd;
    if (!format_of(fsrc_c, &fs) || !format_of(fdst_c, &fd)) return 1;
    for (int64_t i = 0; i < n; ++i) {
        Decoded d = decode(load(src, i, fs), fs);
        uint32_t out;
        if (d.nar) out = nar_of(fd);
        else if (d.zero) out = 0;
        else { Big m; m.w[0] = d.sig; out = round_big(d.neg, m, d.sh - fs.max_scale(), fd); }
        store(dst, i, out, fd);
    }
    return 0;
}

// posit -> binary64 is exact for all three formats; binary32 is the hardware's
// nearest-even narrowing of that exact double (one rounding).
int oracle_to_f64(int fsrc_c, int64_t n, const void* src, double* dst) {
    Format fs;
    if (!format_of(fsrc_c, &fs)) return 1;
    for (int64_t i = 0; i < n; ++i) {
        Decoded d = decode(load(src, i, fs), fs);
        double v;
        if (d.nar) v = std::nan("");
        else if (d.zero) v = 0.0;
        else { v = std::ldexp((double)d.sig, d.sh - fs.max_scale()); if (d.neg) v = -v; }
        dst[i] = v;
    }
    return 0;
}

int oracle_to_f32(int fsrc_c, int64_t n, const void* src, float* dst) {
    std::vector<double> t((size_t)n);
    int rc = oracle_to_f64(fsrc_c, n, src, t.data());
    if (rc) return rc;
    for (int64_t i = 0; i < n; ++i) dst[i] = (float)t[(size_t)i];
    return 0;
}

// y <- round_fy( y + alpha * x ), alpha a pattern in fy, x in fx; optional narrowed copy of the new y
int oracle_axpy(int fx_c, int fy_c, uint32_t alpha, int64_t n, const void* x, void* y, int fcopy_c, void* ycopy) {
    Format fx, fy, fc;
    if (!format_of(fx_c, &fx) || !format_of(fy_c, &fy)) return 1;
    const bool copy = ycopy != nullptr;
    if (copy && !format_of(fcopy_c, &fc)) return 1;
    const Decoded a = decode(alpha, fy);
    for (int64_t i = 0; i < n; ++i) {
        const Decoded dx = decode(load(x, i, fx), fx);
        const Decoded dy = decode(load(y, i, fy), fy);
        uint32_t out;
        if (a.nar || dx.nar || dy.nar) out = nar_of(fy);
        else {
            // common unit: minpos_y * minpos_x
            Big s;
            if (!dy.zero) s.add_shifted(dy.sig, dy.sh + fx.max_scale(), dy.neg);
            if (!a.zero && !dx.zero) s.add_shifted(a.sig * dx.sig, a.sh + dx.sh, a.neg != dx.neg);
            const bool neg = s.negative();
            if (neg) s.negate();
            out = round_big(neg, s, -(fy.max_scale() + fx.max_scale()), fy);
        }
        store(y, i, out, fy);
        if (copy) {
            Decoded d = decode(out, fy);
            uint32_t c;
            if (d.nar) c = nar_of(fc);
            else if (d.zero) c = 0;
            else { Big m; m.w[0] = d.sig; c = round_big(d.neg, m, d.sh - fy.max_scale(), fc); }
            store(ycopy, i, c, fc);
        }
    }
    return 0;
}

}  // extern "C"
