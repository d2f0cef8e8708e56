// Host build of the scalar device functions (decode, encode, quire read-out,
// exact add) so that unit tests can drive them on a machine without a GPU.
// Test scaffolding: nothing in the library links or calls this file.
#include "elementwise_fast.h"
#include "quire_arith.h"
#include "conv_p8.h"
#include "p16_window_arith.h"
#include "noquire_arith.h"
#include "loss_ops.h"

using namespace pnn;

namespace {
template <class Op>
void run_map(Op op, int64_t n, const uint64_t* in, uint64_t* out) {
    for (int64_t i = 0; i < n; ++i) out[i] = op(in[i]);
}

template <class FS>
int convert_host(int dst, int64_t n, const uint64_t* in, uint64_t* out) {
    switch (dst) {
        case 0: run_map(PositToPosit<FS, P8>(), n, in, out); return 0;
        case 1: run_map(PositToPosit<FS, P16>(), n, in, out); return 0;
        case 2: run_map(PositToPosit<FS, P32>(), n, in, out); return 0;
        case 100: run_map(PositToF32<FS>(), n, in, out); return 0;
        case 101: run_map(PositToF64<FS>(), n, in, out); return 0;
    }
    return 1;
}

template <class FX, class FY>
void axpy_host(uint32_t alpha, int64_t n, const uint64_t* x, const uint64_t* y, uint64_t* out) {
    Axpy<FX, FY> op;
    op.alpha = alpha;
    for (int64_t i = 0; i < n; ++i) out[i] = op((uint32_t)x[i], (uint32_t)y[i]);
}

// dot product of n staged operands through Arith<F>, rounded to fout
template <class F>
uint32_t dot_host(int fout, int64_t n, const uint32_t* a, const uint32_t* b, int has_bias, uint32_t bias) {
    typedef Arith<F> AR;
    uint32_t q[AR::L];
    for (int l = 0; l < AR::L; ++l) q[l] = 0;
    bool nar = false;
    for (int64_t i = 0; i < n; ++i) {
        if (a[i] == F::NAR || b[i] == F::NAR) nar = true;
        AR::mac(q, AR::stage(a[i]), AR::stage(b[i]));
    }
    if (has_bias) {
        if (bias == F::NAR) nar = true;
        else AR::add_value(q, AR::stage(bias));
    }
    const FmtRT fo = fmt_of_code(fout);
    Real r;
    if (nar) return fo.nar();
    return quire_read<F, AR::L>(q, r) ? encode_rt(r, fo) : 0u;
}

// the same dot product with the quire switched off, through the kernel's accumulator policy
template <class F>
uint32_t dot_noquire_host(int fout, int64_t n, const uint32_t* a, const uint32_t* b, int has_bias, uint32_t bias) {
    typedef NoQuire<F> AR;
    uint32_t q[1] = {0};
    bool nar = false;
    for (int64_t i = 0; i < n; ++i) {
        if (a[i] == F::NAR || b[i] == F::NAR) nar = true;
        AR::mac(q, AR::stage(a[i]), AR::stage(b[i]));
    }
    if (has_bias) {
        if (bias == F::NAR) nar = true;
        else AR::add_value(q, AR::stage(bias));
    }
    const FmtRT fo = fmt_of_code(fout);
    Real r;
    if (nar) return fo.nar();
    return AR::read(q, r) ? encode_rt(r, fo) : 0u;
}

// the same dot product through the fp64 buckets, emptied into the limbs on the kernel's schedule
// (every FLUSH_SLICES slices of GEMM_KT products and at the end); 0xFFFFFFFF: format has no buckets
template <class F>
uint32_t dot_bucket_host(int fout, int64_t n, const uint32_t* a, const uint32_t* b, int has_bias, uint32_t bias) {
    typedef BucketAccum<F> AR;
    if constexpr (AR::BUCKETS == 0) {
        return 0xFFFFFFFFu;
    } else {
        uint32_t q[AR::L];
        for (int l = 0; l < AR::L; ++l) q[l] = 0;
        double bk[AR::NB];
        AR::clear(bk);
        bool nar = false;
        int since = 0;
        for (int64_t k0 = 0; k0 < n; k0 += GEMM_KT) {
            for (int64_t i = k0; i < n && i < k0 + GEMM_KT; ++i) {
                if (a[i] == F::NAR || b[i] == F::NAR) nar = true;
                AR::mac(bk, AR::stage(a[i]), AR::stage(b[i]));
            }
            if (++since == AR::FLUSH_SLICES) {
                since = 0;
                AR::template flush<AR::L>(q, bk);
            }
        }
        AR::template flush<AR::L>(q, bk);
        if (has_bias) {
            if (bias == F::NAR) nar = true;
            else AR::add_bias(q, bias);
        }
        const FmtRT fo = fmt_of_code(fout);
        Real r;
        if (nar) return fo.nar();
        return AR::read(q, r) ? encode_rt(r, fo) : 0u;
    }
}
// the same dot product with the whole sum kept in doubles (CascadeArith), carries on the kernel's schedule:
// after every LOW_EVERY products out of the low levels, after every TOP_EVERY out of the top bucket; limbs at the end
template <class F>
uint32_t dot_cascade_host(int fout, int64_t n, const uint32_t* a, const uint32_t* b, int has_bias, uint32_t bias) {
    typedef CascadeArith<F> CA;
    typedef BucketAccum<F> AR;
    if constexpr (!CA::ELIGIBLE) {
        return 0xFFFFFFFFu;
    } else {
        double c[CA::NL];
        CA::clear(c);
        bool nar = false;
        for (int64_t k0 = 0; k0 < n; k0 += CA::TOP_EVERY) {
            for (int half = 0; half < CA::TOP_EVERY / CA::LOW_EVERY; ++half) {
                for (int64_t i = k0 + half * CA::LOW_EVERY; i < n && i < k0 + (half + 1) * CA::LOW_EVERY; ++i) {
                    if (a[i] == F::NAR || b[i] == F::NAR) nar = true;
                    CA::mac(c, AR::stage(a[i]), AR::stage(b[i]));
                }
                CA::carry_low(c);
            }
            CA::carry_top(c);
        }
        uint32_t q[AR::L];
        for (int l = 0; l < AR::L; ++l) q[l] = 0;
        CA::template to_limbs<AR::L>(q, c);
        if (has_bias) {
            if (bias == F::NAR) nar = true;
            else AR::add_bias(q, bias);
        }
        const FmtRT fo = fmt_of_code(fout);
        Real r;
        if (nar) return fo.nar();
        return AR::read(q, r) ? encode_rt(r, fo) : 0u;
    }
}

// the limbs after adding m * 2^T(j) (bucket j = 1..B of the format, |m| <= 2^53) to zeroed limbs; returns the limb count
template <class F, int J>
int flush_one(int j, double m, uint32_t* out) {
    typedef BucketAccum<F> AR;
    if constexpr (J > AR::NB) {
        return 0;
    } else {
        if (j != J) return flush_one<F, J + 1>(j, m, out);
        uint32_t q[AR::L];
        for (int l = 0; l < AR::L; ++l) q[l] = 0;
        quire_add_double<AR::L, AR::T(J)>(q, m * pow2d(AR::T(J)));
        for (int l = 0; l < AR::L; ++l) out[l] = q[l];
        return AR::L;
    }
}

// the buckets after one product of staged operands a * b entered cleared buckets; cuts[j] = T(j + 1); returns the bucket count
template <class F>
int split_one(uint32_t a, uint32_t b, double* parts, int* cuts) {
    typedef BucketArith<F> BA;
    double bk[BA::NB];
    BA::clear(bk);
    BA::mac(bk, BA::stage(a), BA::stage(b));
    for (int j = 0; j < BA::NB; ++j) {
        parts[j] = bk[j];
        cuts[j] = BA::T(j + 1);
    }
    return BA::NB;
}

}  // namespace

extern "C" {

// One product cut into its bucket parts (the error-free split of BucketArith::mac): parts[j] must be a multiple of
// 2^cuts[j], and the parts must add up to the product.
int hostcheck_bucket_split(int fin, uint32_t a, uint32_t b, double* parts, int* cuts) {
    switch (fin) {
        case 1: return split_one<P16>(a, b, parts, cuts);
        case 3: return split_one<P8_1>(a, b, parts, cuts);
        case 4: return split_one<P8_2>(a, b, parts, cuts);
        case 5: return split_one<P10_1>(a, b, parts, cuts);
        case 6: return split_one<P10_2>(a, b, parts, cuts);
        case 7: return split_one<P12_1>(a, b, parts, cuts);
        case 8: return split_one<P12_2>(a, b, parts, cuts);
        default: return 0;
    }
}

uint32_t hostcheck_dot_cascade(int fin, int fout, int64_t n, const uint32_t* a, const uint32_t* b, int has_bias, uint32_t bias) {
    switch (fin) {
        case 3: return dot_cascade_host<P8_1>(fout, n, a, b, has_bias, bias);
        case 4: return dot_cascade_host<P8_2>(fout, n, a, b, has_bias, bias);
        default: return 0xFFFFFFFFu;
    }
}

uint32_t hostcheck_dot_bucket(int fin, int fout, int64_t n, const uint32_t* a, const uint32_t* b, int has_bias, uint32_t bias) {
    switch (fin) {
        case 1: return dot_bucket_host<P16>(fout, n, a, b, has_bias, bias);
        case 3: return dot_bucket_host<P8_1>(fout, n, a, b, has_bias, bias);
        case 4: return dot_bucket_host<P8_2>(fout, n, a, b, has_bias, bias);
        case 5: return dot_bucket_host<P10_1>(fout, n, a, b, has_bias, bias);
        case 6: return dot_bucket_host<P10_2>(fout, n, a, b, has_bias, bias);
        case 7: return dot_bucket_host<P12_1>(fout, n, a, b, has_bias, bias);
        case 8: return dot_bucket_host<P12_2>(fout, n, a, b, has_bias, bias);
        default: return 0xFFFFFFFFu;
    }
}

int hostcheck_bucket_flush(int fin, int j, double m, uint32_t* out) {
    switch (fin) {
        case 1: return flush_one<P16, 1>(j, m, out);
        case 3: return flush_one<P8_1, 1>(j, m, out);
        case 4: return flush_one<P8_2, 1>(j, m, out);
        case 5: return flush_one<P10_1, 1>(j, m, out);
        case 6: return flush_one<P10_2, 1>(j, m, out);
        case 7: return flush_one<P12_1, 1>(j, m, out);
        case 8: return flush_one<P12_2, 1>(j, m, out);
        default: return 0;
    }
}

// buckets, guard bits G (2^G products between flushes) and cut position T(1) of the format; 0 buckets: not bucketed
void hostcheck_bucket_config(int fin, int* buckets, int* guard, int* top_cut) {
    *buckets = 0; *guard = 0; *top_cut = 0;
    switch (fin) {
        case 1: *buckets = BucketArith<P16>::B; *guard = BucketArith<P16>::G; *top_cut = BucketArith<P16>::T(1); break;
        case 3: *buckets = BucketArith<P8_1>::B; *guard = BucketArith<P8_1>::G; *top_cut = BucketArith<P8_1>::T(1); break;
        case 4: *buckets = BucketArith<P8_2>::B; *guard = BucketArith<P8_2>::G; *top_cut = BucketArith<P8_2>::T(1); break;
        case 5: *buckets = BucketArith<P10_1>::B; *guard = BucketArith<P10_1>::G; *top_cut = BucketArith<P10_1>::T(1); break;
        case 6: *buckets = BucketArith<P10_2>::B; *guard = BucketArith<P10_2>::G; *top_cut = BucketArith<P10_2>::T(1); break;
        case 7: *buckets = BucketArith<P12_1>::B; *guard = BucketArith<P12_1>::G; *top_cut = BucketArith<P12_1>::T(1); break;
        case 8: *buckets = BucketArith<P12_2>::B; *guard = BucketArith<P12_2>::G; *top_cut = BucketArith<P12_2>::T(1); break;
        default: break;
    }
}

uint32_t hostcheck_dot_noquire(int fin, int fout, int64_t n, const uint32_t* a, const uint32_t* b, int has_bias, uint32_t bias) {
    switch (fin) {
        case 0: return dot_noquire_host<P8>(fout, n, a, b, has_bias, bias);
        case 1: return dot_noquire_host<P16>(fout, n, a, b, has_bias, bias);
        case 2: return dot_noquire_host<P32>(fout, n, a, b, has_bias, bias);
        case 3: return dot_noquire_host<P8_1>(fout, n, a, b, has_bias, bias);
        case 4: return dot_noquire_host<P8_2>(fout, n, a, b, has_bias, bias);
        case 5: return dot_noquire_host<P10_1>(fout, n, a, b, has_bias, bias);
        case 6: return dot_noquire_host<P10_2>(fout, n, a, b, has_bias, bias);
        case 7: return dot_noquire_host<P12_1>(fout, n, a, b, has_bias, bias);
        default: return dot_noquire_host<P12_2>(fout, n, a, b, has_bias, bias);
    }
}

// posit<fmt> value times 2^pow2 divided by an integer, rounded once to format fout (the scaling step of the losses)
uint32_t hostcheck_div_int(int fmt, int fout, uint32_t p, int pow2, uint32_t divisor) {
    const FmtRT fi = fmt_of_code(fmt), fo = fmt_of_code(fout);
    if (p == fi.nar()) return fo.nar();
    if (p == 0) return 0;
    Real r = decode_rt(p, fi);
    r.scale += pow2;
    return encode_rt(real_div_int(r, divisor), fo);
}

// posit (x) posit -> posit, rounded once: op 0 = multiply, 1 = add, 2 = divide (formats of at most 16 bits); any patterns
uint32_t hostcheck_posit_op(int fmt, int op, uint32_t a, uint32_t b) {
    if (op == 2) {
        switch (fmt) {
            case 0: return posit_div<P8>(a, b);
            case 1: return posit_div<P16>(a, b);
            case 3: return posit_div<P8_1>(a, b);
            case 4: return posit_div<P8_2>(a, b);
            case 5: return posit_div<P10_1>(a, b);
            case 6: return posit_div<P10_2>(a, b);
            case 7: return posit_div<P12_1>(a, b);
            case 8: return posit_div<P12_2>(a, b);
            default: return 0xFFFFFFFFu;
        }
    }
    switch (fmt) {
        case 0: return op ? posit_add<P8>(a, b) : posit_mul<P8>(a, b);
        case 1: return op ? posit_add<P16>(a, b) : posit_mul<P16>(a, b);
        case 2: return op ? posit_add<P32>(a, b) : posit_mul<P32>(a, b);
        case 3: return op ? posit_add<P8_1>(a, b) : posit_mul<P8_1>(a, b);
        case 4: return op ? posit_add<P8_2>(a, b) : posit_mul<P8_2>(a, b);
        case 5: return op ? posit_add<P10_1>(a, b) : posit_mul<P10_1>(a, b);
        case 6: return op ? posit_add<P10_2>(a, b) : posit_mul<P10_2>(a, b);
        case 7: return op ? posit_add<P12_1>(a, b) : posit_mul<P12_1>(a, b);
        default: return op ? posit_add<P12_2>(a, b) : posit_mul<P12_2>(a, b);
    }
}

int hostcheck_round(int src_float, int dst, int64_t n, const uint64_t* in, uint64_t* out) {
    if (src_float == 100) {
        if (dst == 0) run_map(RoundF32<P8>(), n, in, out);
        else if (dst == 1) run_map(RoundF32<P16>(), n, in, out);
        else run_map(RoundF32<P32>(), n, in, out);
    } else {
        if (dst == 0) run_map(RoundF64<P8>(), n, in, out);
        else if (dst == 1) run_map(RoundF64<P16>(), n, in, out);
        else run_map(RoundF64<P32>(), n, in, out);
    }
    return 0;
}

// run-time-format paths (any posit code 0..8, 100 = binary32, 101 = binary64)
int hostcheck_map_rt(int src, int dst, int64_t n, const uint64_t* in, uint64_t* out) {
    MapRT m;
    m.src_kind = src == 100 ? 1 : (src == 101 ? 2 : 0);
    m.dst_kind = dst == 100 ? 1 : (dst == 101 ? 2 : 0);
    m.fs = fmt_of_code(m.src_kind ? 0 : src);
    m.fd = fmt_of_code(m.dst_kind ? 0 : dst);
    for (int64_t i = 0; i < n; ++i) out[i] = m(in[i]);
    return 0;
}

int hostcheck_axpy_rt(int fx, int fy, uint32_t alpha, int64_t n, const uint64_t* x, const uint64_t* y, uint64_t* out) {
    AxpyRT op;
    op.fx = fmt_of_code(fx);
    op.fy = fmt_of_code(fy);
    op.alpha = alpha;
    for (int64_t i = 0; i < n; ++i) out[i] = op((uint32_t)x[i], (uint32_t)y[i]);
    return 0;
}

// the arithmetic of the large-tensor update kernel (binary64 product, error-free sum, one rounding), element by element
int hostcheck_axpy_f64(int fx, int fy, uint32_t alpha, int64_t n, const uint64_t* x, const uint64_t* y, uint64_t* out) {
#define CASE(FX, FY, a, b)                                                                                                  \
    if (fx == a && fy == b) {                                                                                               \
        const double ad = f64_of_pattern<FY>(alpha);                                                                        \
        for (int64_t i = 0; i < n; ++i) out[i] = axpy_f64<FY>(ad, f64_of_pattern<FX>((uint32_t)x[i]), f64_of_pattern<FY>((uint32_t)y[i])); \
        return 0;                                                                                                           \
    }
    CASE(P16, P16, 1, 1) CASE(P8, P16, 0, 1) CASE(P12_2, P12_2, 8, 8) CASE(P8_2, P12_2, 4, 8) CASE(P8, P8, 0, 0) CASE(P10_1, P12_1, 5, 7)
#undef CASE
    return 1;
}

// The two-bucket dot product of the posit<16,1> GEMM on the host: main operands through pw_mac (at most PW_MAXK products
// between two flushes), products with an outlier operand through the integer multiply-accumulate, as the kernel's
// correction phase takes them; q receives the four quire limbs.  outliers[0..1] count the outliers of a and b.
int hostcheck_pw_dot(int64_t n, const uint32_t* a, const uint32_t* b, uint32_t* q, int* outliers) {
    typedef Arith<P16> AI;
    uint32_t acc[4] = {0, 0, 0, 0};
    double hi = 0.0, lo = 0.0;
    int64_t since = 0;
    outliers[0] = outliers[1] = 0;
    for (int64_t i = 0; i < n; ++i) {
        double va, vb;
        const bool oa = pw_classify(a[i], va), ob = pw_classify(b[i], vb);
        outliers[0] += oa;
        outliers[1] += ob;
        if (oa || ob) {
            if (a[i] != P16::NAR && b[i] != P16::NAR) AI::mac(acc, AI::stage(a[i]), AI::stage(b[i]));
            continue;
        }
        if (va != va || vb != vb) continue;  // NaR: the kernel decides those outputs by flags
        pw_mac(hi, lo, va, vb);
        if (++since == PW_MAXK) {
            pw_flush(acc, hi, lo);
            hi = lo = 0.0;
            since = 0;
        }
    }
    pw_flush(acc, hi, lo);
    for (int l = 0; l < 4; ++l) q[l] = acc[l];
    return 0;
}

// the epilogue rounding of the posit<8,0> kernels: 32-bit quire (units of minpos^2 = 2^-12) -> pattern
int hostcheck_p8_round_quire(int64_t n, const int32_t* in, uint32_t* out) {
    for (int64_t i = 0; i < n; ++i) out[i] = p8_round_quire(in[i]);
    return 0;
}

// posit<16,1> -> posit<8,0> through the step table of the narrowing kernel
int hostcheck_narrow_step(int64_t n, const uint64_t* in, uint64_t* out) {
    for (int64_t i = 0; i < n; ++i) {
        const uint32_t p = (uint32_t)in[i] & 0xFFFFu;
        out[i] = narrow_step_apply(narrow_step_entry<P16, P8>(p >> 6), p);
    }
    return 0;
}

// one rounding of the binary64 s (exact value: s, or just off s as the two flags say) to posit code fmt
uint32_t hostcheck_round_f64(int fmt, double s, int inexact, int toward_zero) {
    switch (fmt) {
        case 0: return round_f64_to_posit<P8>(s, inexact, toward_zero);
        case 1: return round_f64_to_posit<P16>(s, inexact, toward_zero);
        case 3: return round_f64_to_posit<P8_1>(s, inexact, toward_zero);
        case 4: return round_f64_to_posit<P8_2>(s, inexact, toward_zero);
        case 5: return round_f64_to_posit<P10_1>(s, inexact, toward_zero);
        case 6: return round_f64_to_posit<P10_2>(s, inexact, toward_zero);
        case 7: return round_f64_to_posit<P12_1>(s, inexact, toward_zero);
        case 8: return round_f64_to_posit<P12_2>(s, inexact, toward_zero);
        default: return 0xFFFFFFFFu;
    }
}

int hostcheck_convert(int src, int dst, int64_t n, const uint64_t* in, uint64_t* out) {
    if (src == 0) return convert_host<P8>(dst, n, in, out);
    if (src == 1) return convert_host<P16>(dst, n, in, out);
    return convert_host<P32>(dst, n, in, out);
}

int hostcheck_axpy(int fx, int fy, uint32_t alpha, int64_t n, const uint64_t* x, const uint64_t* y, uint64_t* out) {
#define CASE(FX, FY, a, b) if (fx == a && fy == b) { axpy_host<FX, FY>(alpha, n, x, y, out); return 0; }
    CASE(P8, P8, 0, 0) CASE(P8, P16, 0, 1) CASE(P8, P32, 0, 2)
    CASE(P16, P8, 1, 0) CASE(P16, P16, 1, 1) CASE(P16, P32, 1, 2)
    CASE(P32, P8, 2, 0) CASE(P32, P16, 2, 1) CASE(P32, P32, 2, 2)
#undef CASE
    return 1;
}

uint32_t hostcheck_dot(int fin, int fout, int64_t n, const uint32_t* a, const uint32_t* b, int has_bias, uint32_t bias) {
    switch (fin) {
        case 0: return dot_host<P8>(fout, n, a, b, has_bias, bias);
        case 1: return dot_host<P16>(fout, n, a, b, has_bias, bias);
        case 2: return dot_host<P32>(fout, n, a, b, has_bias, bias);
        case 3: return dot_host<P8_1>(fout, n, a, b, has_bias, bias);
        case 4: return dot_host<P8_2>(fout, n, a, b, has_bias, bias);
        case 5: return dot_host<P10_1>(fout, n, a, b, has_bias, bias);
        case 6: return dot_host<P10_2>(fout, n, a, b, has_bias, bias);
        case 7: return dot_host<P12_1>(fout, n, a, b, has_bias, bias);
        default: return dot_host<P12_2>(fout, n, a, b, has_bias, bias);
    }
}

// Implicit-GEMM gather descriptors of the posit<8,0> convolution path, evaluated on the host:
// for virtual element (row, k) of operand A or B of pass `which` (0 fwd, 1 bwd-data, 2 bwd-weight),
// returns 1 and the tensor offset when the element is inside its bounds, 0 when it is a zero operand.
// geom = N, C, H, W, K, R, S, pad_h, pad_w, stride_h, stride_w.  dims receives M, N, K of the kernel view.
int hostcheck_conv_gather(int which, const int64_t* geom, int operand_b, int64_t row, int64_t k, int64_t* offset, int64_t* dims,
                          int64_t* out_index) {
    ConvGeom g;
    g.N = (int)geom[0]; g.C = (int)geom[1]; g.H = (int)geom[2]; g.W = (int)geom[3]; g.K = (int)geom[4]; g.R = (int)geom[5]; g.S = (int)geom[6];
    g.ph = (int)geom[7]; g.pw = (int)geom[8]; g.sh = (int)geom[9]; g.sw = (int)geom[10];
    g.OH = (g.H + 2 * g.ph - g.R) / g.sh + 1;
    g.OW = (g.W + 2 * g.pw - g.S) / g.sw + 1;
    const P8ConvProblem p = p8_problem(which, g, nullptr, nullptr);
    dims[0] = p.M; dims[1] = p.N; dims[2] = p.K;
    const P8Gather& op = operand_b ? p.B : p.A;
    int rp, ry, rx, kp, ky, kx;
    op.row.eval((uint32_t)row, rp, ry, rx);
    op.k.eval((uint32_t)k, kp, ky, kx);
    *offset = (int64_t)rp + kp;
    if (out_index) *out_index = p.out.at((int)row, (int)k);  // (row, k) reused as output (m, n)
    return ((uint32_t)(ry + ky) < (uint32_t)op.LY) && ((uint32_t)(rx + kx) < (uint32_t)op.LX);
}

}  // extern "C"
