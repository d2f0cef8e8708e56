// posit_gemm_noquire / posit_conv2d_*_noquire: the same matrix product and
// convolutions with the quire switched off (paper Sec. 3.3: the quire is an
// option; Table 2 reports training "without quire").  Every product and every
// running sum is rounded to posit<fin>; the terms are taken in order of the
// reduction index of the (implicit) matrix product, so the reduction is never
// split: each output is one sequential chain, outputs run in parallel.
// The tiled kernel and the operand gathers are those of the quire path; only
// the accumulator policy differs (NoQuire<F>: one running pattern per output).
#include "api_common.h"
#include "conv_desc.h"
#include "noquire_arith.h"

namespace pnn {

// 32x32 output tiles: the arithmetic per term is two posit roundings, so operand reuse
// in registers matters little and smaller tiles spread short problems over more CUs.
constexpr int NQ_TM = 2, NQ_TN = 2;

inline GemmPlan noquire_plan(int64_t K) {
    GemmPlan p;
    p.splits = 1;
    p.k_per_split = ((K > 0 ? K : 1) + GEMM_KT - 1) / GEMM_KT * GEMM_KT;
    p.ws_bytes = 0;
    return p;
}

template <class F, class OpA, class OpB, class Out>
hipError_t launch_noquire(hipStream_t st, const OpA& a, const OpB& b, const Out& out, int64_t M, int64_t N, int64_t K,
                          const void* bias, void* C, int fout) {
    return launch_quire_gemm<F, OpA, OpB, Out, NQ_TM, NQ_TN, NoQuire<F>>(st, a, b, out, M, N, K, bias, C, fout, nullptr, noquire_plan(K));
}

template <class F>
int gemm_noquire(hipStream_t st, int fout, int transA, int transB, int64_t M, int64_t N, int64_t K,
                 const void* A, int64_t lda, const void* B, int64_t ldb, const void* bias, void* C, int64_t ldc) {
    typedef typename Storage<F::N>::T T;
    RowMajorOut out{ldc};
    hipError_t e;
    if (!transA && !transB) {
        MatrixOperand<T, true> a{(const T*)A, lda, M, K};
        MatrixOperand<T, false> b{(const T*)B, ldb, N, K};
        e = launch_noquire<F>(st, a, b, out, M, N, K, bias, C, fout);
    } else if (!transA && transB) {
        MatrixOperand<T, true> a{(const T*)A, lda, M, K};
        MatrixOperand<T, true> b{(const T*)B, ldb, N, K};
        e = launch_noquire<F>(st, a, b, out, M, N, K, bias, C, fout);
    } else if (transA && !transB) {
        MatrixOperand<T, false> a{(const T*)A, lda, M, K};
        MatrixOperand<T, false> b{(const T*)B, ldb, N, K};
        e = launch_noquire<F>(st, a, b, out, M, N, K, bias, C, fout);
    } else {
        MatrixOperand<T, false> a{(const T*)A, lda, M, K};
        MatrixOperand<T, true> b{(const T*)B, ldb, N, K};
        e = launch_noquire<F>(st, a, b, out, M, N, K, bias, C, fout);
    }
    return hip_status(e);
}

template <class F>
int conv_fwd_noquire(hipStream_t st, int fout, const ConvGeom& g, const void* x, const void* w, const void* bias, void* y) {
    typedef typename Storage<F::N>::T T;
    const ConvDims d = conv_dims(0, g);
    ConvFwdX<T> a{(const T*)x, g, d.M, d.K};
    MatrixOperand<T, true> b{(const T*)w, d.K, d.N, d.K};
    NchwOut out{(int64_t)g.OH * g.OW, (int64_t)g.K};
    return hip_status(launch_noquire<F>(st, a, b, out, d.M, d.N, d.K, bias, y, fout));
}

template <class F>
int conv_bwd_data_noquire(hipStream_t st, int fout, const ConvGeom& g, const void* dy, const void* w, void* dx) {
    typedef typename Storage<F::N>::T T;
    const ConvDims d = conv_dims(1, g);
    ConvBwdDataDy<T> a{(const T*)dy, g, d.M, d.K};
    ConvBwdDataW<T> b{(const T*)w, g, d.N, d.K};
    NchwOut out{(int64_t)g.H * g.W, (int64_t)g.C};
    const hipError_t e = launch_noquire<F>(st, a, b, out, d.M, d.N, d.K, nullptr, dx, fout);
    if (e != hipSuccess) return PNN_EHIP;
    launch_bwd_data_nar_weights<F>(st, w, g, dx, fout);  // NaR weights were zeros above: mark the positions their taps reach
    return hip_status(hipGetLastError());
}

template <class F>
int conv_bwd_weight_noquire(hipStream_t st, int fout, const ConvGeom& g, const void* dy, const void* x, void* dw, void* dbias) {
    typedef typename Storage<F::N>::T T;
    const ConvDims d = conv_dims(2, g);
    ConvBwdWeightDy<T> a{(const T*)dy, g, d.M, d.K};
    ConvBwdWeightX<T> b{(const T*)x, g, d.N, d.K};
    RowMajorOut out{d.N};
    hipError_t e = launch_noquire<F>(st, a, b, out, d.M, d.N, d.K, nullptr, dw, fout);
    if (e == hipSuccess && dbias) {
        // dbias[k]: the running sum of dy[n,k,:,:] * 1 in the same order (a product with one is exact)
        OnesOperand ones{1u << (F::N - 2), 1, d.K};
        RowMajorOut bout{1};
        e = launch_noquire<F>(st, a, ones, bout, d.M, 1, d.K, nullptr, dbias, fout);
    }
    return hip_status(e);
}

}  // namespace pnn

using namespace pnn;

extern "C" int posit_gemm_noquire(void* stream, int fin, int fout, int transA, int transB, int64_t M, int64_t N, int64_t K,
                                  const void* A, int64_t lda, const void* B, int64_t ldb, const void* bias, void* C, int64_t ldc) {
    if (!is_posit(fin) || !is_posit(fout) || M < 0 || N < 0 || K < 0) return PNN_EINVAL;
    if (M == 0 || N == 0) return PNN_OK;
    if (!C || ldc < N) return PNN_EINVAL;
    if (K > 0) {
        if (!A || !B) return PNN_EINVAL;
        if (lda < (transA ? M : K) || ldb < (transB ? K : N)) return PNN_EINVAL;
    }
    if (M >= ((int64_t)1 << 31) || N >= ((int64_t)1 << 31) || K >= ((int64_t)1 << 31) || M * N >= ((int64_t)1 << 40)) return PNN_EUNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    discard_stale_hip_error();
    PNN_DISPATCH_POSIT(fin, return gemm_noquire<F>(st, fout, transA, transB, M, N, K, A, lda, B, ldb, bias, C, ldc))
    return PNN_EINVAL;
}

extern "C" int posit_conv2d_fwd_noquire(void* stream, int fin, int fout, const pnn_conv2d_desc* desc, const void* x, const void* w,
                                        const void* bias, void* y) {
    ConvGeom g;
    if (!is_posit(fin) || !is_posit(fout) || !conv_geom(desc, &g)) return PNN_EINVAL;
    if (g.N == 0 || g.K == 0) return PNN_OK;
    if (!y || (g.C > 0 && (!x || !w))) return PNN_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    discard_stale_hip_error();
    PNN_DISPATCH_POSIT(fin, return conv_fwd_noquire<F>(st, fout, g, x, w, bias, y))
    return PNN_EINVAL;
}

extern "C" int posit_conv2d_bwd_data_noquire(void* stream, int fin, int fout, const pnn_conv2d_desc* desc, const void* dy,
                                             const void* w, void* dx) {
    ConvGeom g;
    if (!is_posit(fin) || !is_posit(fout) || !conv_geom(desc, &g)) return PNN_EINVAL;
    if (g.N == 0 || g.C == 0) return PNN_OK;
    if (!dx || (g.K > 0 && (!dy || !w))) return PNN_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    discard_stale_hip_error();
    PNN_DISPATCH_POSIT(fin, return conv_bwd_data_noquire<F>(st, fout, g, dy, w, dx))
    return PNN_EINVAL;
}

extern "C" int posit_conv2d_bwd_weight_noquire(void* stream, int fin, int fout, const pnn_conv2d_desc* desc, const void* dy,
                                               const void* x, void* dw, void* dbias) {
    ConvGeom g;
    if (!is_posit(fin) || !is_posit(fout) || !conv_geom(desc, &g)) return PNN_EINVAL;
    if (g.K == 0 || g.C == 0) return PNN_OK;
    if (!dw || (g.N > 0 && (!dy || !x))) return PNN_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    discard_stale_hip_error();
    PNN_DISPATCH_POSIT(fin, return conv_bwd_weight_noquire<F>(st, fout, g, dy, x, dw, dbias))
    return PNN_EINVAL;
}
