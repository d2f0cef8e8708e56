// posit_conv2d_fwd / bwd_data / bwd_weight: quire-exact convolution and its two
// adjoints (paper Sec. 3.1: layers follow LibTorch semantics and the backward
// passes are written by hand; Sec. 3.3: quire accumulation in convolutions).
// Each is an implicit GEMM over the tiled quire kernel:
//   fwd        rows (n,oh,ow)  x cols k          reduce over (c,r,s)
//   bwd_data   rows (n,h,w)    x cols c          reduce over (k,r,s)
//   bwd_weight rows k          x cols (c,r,s)    reduce over (n,oh,ow)
#include "api_common.h"
#include "conv_desc.h"
#include "conv_p8_pre.h"
#include "conv_p8_mfma.h"
#include "conv_b8.h"

namespace pnn {

template <class F> struct ConvTile { static constexpr int TM = 4, TN = 4; };
template <> struct ConvTile<P32> { static constexpr int TM = 2, TN = 2; };

template <class Out>
hipError_t p8_conv_launch(hipStream_t st, const P8ConvProblem& p, const uint8_t* bias, void* C, int fout, void* wsp,
                          const GemmPlan& plan, const Out& merge_out) {
    const P8ConvTile tl = p8_conv_tile(p.M, p.N, p.K);
    const int tiles_m = (p.M + tl.bm - 1) / tl.bm, tiles_n = (p.N + tl.bn - 1) / tl.bn;
    SplitWs ws;
    ws.limbs = nullptr; ws.rowflag = nullptr; ws.colflag = nullptr;
    if (plan.splits > 1) {
        ws.limbs = (uint32_t*)wsp;
        ws.rowflag = ws.limbs + (size_t)plan.splits * p.M * p.N;
        ws.colflag = ws.rowflag + (size_t)plan.splits * p.Mw;
    }
    dim3 grid((unsigned)(tiles_m * tiles_n), 1, (unsigned)plan.splits);
    const uint8_t* kbias = plan.splits > 1 ? nullptr : bias;
    P8ConvOut kout = p.out;
    kout.vec4 = p.out.vec4 && ((uintptr_t)C & 3u) == 0;  // packed stores need an aligned output tensor
#define PNN_LAUNCH_CONV(TY, TX, TM, TN)                                                                                   \
    hipLaunchKernelGGL((p8_conv_kernel<TY, TX, TM, TN>), grid, dim3(256), 0, st, p.A, p.B, kout, kbias, C, fout, p.M, p.N, \
                       p.K, (int)plan.k_per_split, tiles_n, ws, p.transposed)
    if (tl.bm == 128 && tl.bn == 128) PNN_LAUNCH_CONV(16, 16, 8, 8);
    else if (tl.bm == 256 && tl.bn == 64) PNN_LAUNCH_CONV(32, 8, 8, 8);
    else if (tl.bm == 256 && tl.bn == 32) PNN_LAUNCH_CONV(32, 8, 8, 4);
    else if (tl.bm == 128 && tl.bn == 64) PNN_LAUNCH_CONV(16, 16, 8, 4);
    else if (tl.bm == 128 && tl.bn == 32) PNN_LAUNCH_CONV(32, 8, 4, 4);
    else PNN_LAUNCH_CONV(16, 16, 4, 4);
#undef PNN_LAUNCH_CONV
    PNN_CHECK_LAUNCH();
    if (plan.splits > 1) return launch_split_merge<P8, Out>(st, ws, plan.splits, p.Mw, p.Nw, bias, C, fout, merge_out);
    return hipSuccess;
}

// Pre-decoded path: rewrite both operands into the workspace, then run the kernel that reads them.
// Workspace layout: [operand A as int16][operand B as int16][partial quires and flags of a split reduction].
template <class Out>
hipError_t p8_pre_launch(hipStream_t st, P8PrePlan pp, const void* srcA, const void* srcB, const uint8_t* bias, void* C, int fout,
                         void* wsp, const GemmPlan& plan, const Out& merge_out) {
    uint8_t* wbytes = (uint8_t*)wsp;
    pp.job[0].src = (const uint8_t*)srcA; pp.job[0].dst = (uint16_t*)wbytes;
    pp.job[1].src = (const uint8_t*)srcB; pp.job[1].dst = (uint16_t*)(wbytes + pp.bytes[0]);
    pp.job[0].aligned = ((uintptr_t)srcA & 3u) == 0;
    pp.job[1].aligned = ((uintptr_t)srcB & 3u) == 0;
    pp.A.base = pp.job[0].dst;
    pp.B.base = pp.job[1].dst;
    const int64_t work0 = (int64_t)pp.job[0].rows * (pp.job[0].pitch / 8), work1 = (int64_t)pp.job[1].rows * (pp.job[1].pitch / 8);
    int64_t blocks = ((work0 > work1 ? work0 : work1) + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(p8_predecode_kernel, dim3((unsigned)blocks, 2), dim3(256), 0, st, pp.job[0], pp.job[1]);
    PNN_CHECK_LAUNCH();

    const P8ConvTile tl = p8_conv_tile(pp.M, pp.N, pp.K);
    const int tiles_m = (pp.M + tl.bm - 1) / tl.bm, tiles_n = (pp.N + tl.bn - 1) / tl.bn;
    SplitWs ws;
    ws.limbs = nullptr; ws.rowflag = nullptr; ws.colflag = nullptr;
    if (plan.splits > 1) {
        ws.limbs = (uint32_t*)(wbytes + pp.bytes[0] + pp.bytes[1]);
        ws.rowflag = ws.limbs + (size_t)plan.splits * pp.M * pp.N;
        ws.colflag = ws.rowflag + (size_t)plan.splits * pp.Mw;
    }
    dim3 grid((unsigned)(tiles_m * tiles_n), 1, (unsigned)plan.splits);
    const uint8_t* kbias = plan.splits > 1 ? nullptr : bias;
    P8ConvOut kout = pp.out;
    kout.vec4 = pp.out.vec4 && ((uintptr_t)C & 3u) == 0;
#define PNN_LAUNCH_PRE(TY, TX, TM, TN)                                                                                       \
    hipLaunchKernelGGL((p8_conv_pre_kernel<TY, TX, TM, TN>), grid, dim3(256), 0, st, pp.A, pp.B, kout, kbias, C, fout, pp.M, \
                       pp.N, pp.K, (int)plan.k_per_split, tiles_n, ws, pp.transposed)
    if (tl.bm == 128 && tl.bn == 128) PNN_LAUNCH_PRE(16, 16, 8, 8);
    else if (tl.bm == 256 && tl.bn == 64) PNN_LAUNCH_PRE(32, 8, 8, 8);
    else if (tl.bm == 256 && tl.bn == 32) PNN_LAUNCH_PRE(32, 8, 8, 4);
    else if (tl.bm == 128 && tl.bn == 64) PNN_LAUNCH_PRE(16, 16, 8, 4);
    else if (tl.bm == 128 && tl.bn == 32) PNN_LAUNCH_PRE(32, 8, 4, 4);
    else PNN_LAUNCH_PRE(16, 16, 4, 4);
#undef PNN_LAUNCH_PRE
    PNN_CHECK_LAUNCH();
    if (plan.splits > 1) return launch_split_merge<P8, Out>(st, ws, plan.splits, pp.Mw, pp.Nw, bias, C, fout, merge_out);
    return hipSuccess;
}

// The pre-decoded path serves this pass: geometry fits, and no split reduction over padded rows.
inline bool p8_pre_usable(int which, const ConvGeom& g, P8PrePlan* pp, GemmPlan* plan) {
    *pp = p8_pre_plan(which, g);
    if (!pp->ok) return false;
    *plan = p8_conv_plan(pp->M, pp->N, pp->K);
    return !(pp->padded_rows && plan->splits > 1);
}

// workspace of the pre-decoded path: the two rewritten operands, then the split partials
inline size_t p8_pre_ws_bytes(const P8PrePlan& pp, const GemmPlan& plan) { return pp.bytes[0] + pp.bytes[1] + plan.ws_bytes; }

hipError_t p8_conv_launch_rowmajor(hipStream_t st, const P8ConvProblem& p, const uint8_t* bias, void* C, int fout, void* wsp,
                                   const GemmPlan& plan, int64_t ld) {
    RowMajorOut o{ld};
    return p8_conv_launch(st, p, bias, C, fout, wsp, plan, o);
}

hipError_t p8_conv_launch_nchw(hipStream_t st, const P8ConvProblem& p, const uint8_t* bias, void* C, int fout, void* wsp,
                               const GemmPlan& plan, int64_t spatial, int64_t channels) {
    NchwOut o{spatial, channels};
    return p8_conv_launch(st, p, bias, C, fout, wsp, plan, o);
}

// posit(8,1) / posit(8,2): the byte-gather kernel with fp64 buckets
template <class F>
constexpr bool is_b8() { return F::N == 8 && F::ES != 0; }

template <class F>
GemmPlan conv_plan(const ConvDims& d) {
    return plan_split(d.M, d.N, d.K, 16 * ConvTile<F>::TM, 16 * ConvTile<F>::TN, Arith<F>::L);
}

template <class F>
size_t conv_ws(int which, const ConvGeom& g) {
    const ConvDims d = conv_dims(which, g);
    if (d.M <= 0 || d.N <= 0) return 0;
    size_t b = conv_plan<F>(d).ws_bytes;
    if ((F::N == 8 && F::ES == 0) && p8_conv_eligible(which, g)) {
        const P8ConvProblem p = p8_problem(which, g, nullptr, nullptr);
        b = p8_conv_plan(p.M, p.N, p.K).ws_bytes;
        P8PrePlan pp;
        GemmPlan pplan;
        if (p8_pre_usable(which, g, &pp, &pplan)) b = p8_pre_ws_bytes(pp, pplan);
        const P8ConvMfmaPlan mp = p8_conv_mfma_plan(which, g);
        if (mp.ok) b = mp.total();
        if (which == 2) {
            const P8ConvBwPlan bp = p8_conv_bw_plan(g, true);
            if (bp.ok) b = bp.total();
        }
    }
    if constexpr (is_b8<F>()) {
        if (p8_conv_eligible(which, g)) {
            const P8ConvProblem p = p8_problem(which, g, nullptr, nullptr);
            b = b8_conv_plan<F>(p.M, p.N, p.K).ws_bytes;
        }
    }
    if (which == 2) {  // the bias gradient runs after the weight gradient and reuses the start of the workspace
        const size_t b2 = bias_grad_ws_bytes<F>(g.N, g.K, g.OH * g.OW);
        if (b2 > b) b = b2;
    }
    return b;
}

template <class F>
int conv_fwd(hipStream_t st, int fout, const ConvGeom& g, const void* x, const void* w, const void* bias, void* y,
             void* ws, size_t ws_bytes) {
    typedef typename Storage<F::N>::T T;
    const ConvDims d = conv_dims(0, g);
    if ((F::N == 8 && F::ES == 0) && p8_conv_eligible(0, g)) {
        const P8ConvMfmaPlan mp = p8_conv_mfma_plan(0, g);
        if (mp.ok) {  // integer matrix cores
            if (!ws || ws_bytes < mp.total()) return PNN_EWORKSPACE;
            return hip_status(launch_p8_conv_mfma(st, mp, x, w, (const uint8_t*)bias, y, fout, ws));
        }
        P8PrePlan pp;
        GemmPlan pplan;
        if (p8_pre_usable(0, g, &pp, &pplan)) {
            if (!ws || ws_bytes < p8_pre_ws_bytes(pp, pplan)) return PNN_EWORKSPACE;
            NchwOut mout{(int64_t)g.OH * g.OW, (int64_t)g.K};
            return hip_status(p8_pre_launch(st, pp, x, w, (const uint8_t*)bias, y, fout, ws, pplan, mout));
        }
        const P8ConvProblem p = p8_problem(0, g, x, w);
        const GemmPlan plan = p8_conv_plan(p.M, p.N, p.K);
        if (plan.ws_bytes > 0 && (!ws || ws_bytes < plan.ws_bytes)) return PNN_EWORKSPACE;
        NchwOut mout{(int64_t)g.OH * g.OW, (int64_t)g.K};
        return hip_status(p8_conv_launch(st, p, (const uint8_t*)bias, y, fout, ws, plan, mout));
    }
    if constexpr (is_b8<F>()) {
        if (p8_conv_eligible(0, g)) {
            const P8ConvProblem p = p8_problem(0, g, x, w);
            const GemmPlan plan = b8_conv_plan<F>(p.M, p.N, p.K);
            if (plan.ws_bytes > 0 && (!ws || ws_bytes < plan.ws_bytes)) return PNN_EWORKSPACE;
            NchwOut mout{(int64_t)g.OH * g.OW, (int64_t)g.K};
            return hip_status(b8_conv_launch<F>(st, p, (const uint8_t*)bias, y, fout, ws, plan, mout));
        }
    }
    const GemmPlan plan = conv_plan<F>(d);
    if (plan.ws_bytes > 0 && (!ws || ws_bytes < plan.ws_bytes)) return PNN_EWORKSPACE;
    ConvFwdX<T> a{(const T*)x, g, d.M, d.K};
    MatrixOperand<T, true> b{(const T*)w, d.K, d.N, d.K};
    NchwOut out{(int64_t)g.OH * g.OW, (int64_t)g.K};
    return hip_status(launch_quire_gemm<F, decltype(a), decltype(b), NchwOut, ConvTile<F>::TM, ConvTile<F>::TN>(
        st, a, b, out, d.M, d.N, d.K, bias, y, fout, ws, plan));
}

// The product kernels of this pass treat NaR weights as zeros; the outputs such a weight reaches are marked last.
template <class F>
int conv_bwd_data_product(hipStream_t st, int fout, const ConvGeom& g, const void* dy, const void* w, void* dx, void* ws, size_t ws_bytes) {
    typedef typename Storage<F::N>::T T;
    const ConvDims d = conv_dims(1, g);
    if ((F::N == 8 && F::ES == 0) && p8_conv_eligible(1, g)) {
        const P8ConvMfmaPlan mp = p8_conv_mfma_plan(1, g);
        if (mp.ok) {  // integer matrix cores
            if (!ws || ws_bytes < mp.total()) return PNN_EWORKSPACE;
            return hip_status(launch_p8_conv_mfma(st, mp, dy, w, nullptr, dx, fout, ws));
        }
        P8PrePlan pp;
        GemmPlan pplan;
        if (p8_pre_usable(1, g, &pp, &pplan)) {
            if (!ws || ws_bytes < p8_pre_ws_bytes(pp, pplan)) return PNN_EWORKSPACE;
            NchwOut mout{(int64_t)g.H * g.W, (int64_t)g.C};
            return hip_status(p8_pre_launch(st, pp, dy, w, nullptr, dx, fout, ws, pplan, mout));
        }
        const P8ConvProblem p = p8_problem(1, g, dy, w);
        const GemmPlan plan = p8_conv_plan(p.M, p.N, p.K);
        if (plan.ws_bytes > 0 && (!ws || ws_bytes < plan.ws_bytes)) return PNN_EWORKSPACE;
        NchwOut mout{(int64_t)g.H * g.W, (int64_t)g.C};
        return hip_status(p8_conv_launch(st, p, nullptr, dx, fout, ws, plan, mout));
    }
    if constexpr (is_b8<F>()) {
        if (p8_conv_eligible(1, g)) {
            const P8ConvProblem p = p8_problem(1, g, dy, w);
            const GemmPlan plan = b8_conv_plan<F>(p.M, p.N, p.K);
            if (plan.ws_bytes > 0 && (!ws || ws_bytes < plan.ws_bytes)) return PNN_EWORKSPACE;
            NchwOut mout{(int64_t)g.H * g.W, (int64_t)g.C};
            return hip_status(b8_conv_launch<F>(st, p, nullptr, dx, fout, ws, plan, mout));
        }
    }
    const GemmPlan plan = conv_plan<F>(d);
    if (plan.ws_bytes > 0 && (!ws || ws_bytes < plan.ws_bytes)) return PNN_EWORKSPACE;
    ConvBwdDataDy<T> a{(const T*)dy, g, d.M, d.K};
    ConvBwdDataW<T> b{(const T*)w, g, d.N, d.K};
    NchwOut out{(int64_t)g.H * g.W, (int64_t)g.C};
    return hip_status(launch_quire_gemm<F, decltype(a), decltype(b), NchwOut, ConvTile<F>::TM, ConvTile<F>::TN>(
        st, a, b, out, d.M, d.N, d.K, nullptr, dx, fout, ws, plan));
}

template <class F>
int conv_bwd_data(hipStream_t st, int fout, const ConvGeom& g, const void* dy, const void* w, void* dx, void* ws, size_t ws_bytes) {
    const int rc = conv_bwd_data_product<F>(st, fout, g, dy, w, dx, ws, ws_bytes);
    if (rc != PNN_OK) return rc;
    launch_bwd_data_nar_weights<F>(st, w, g, dx, fout);
    return hip_status(hipGetLastError());
}

template <class F>
int conv_bwd_weight(hipStream_t st, int fout, const ConvGeom& g, const void* dy, const void* x, void* dw, void* dbias,
                    void* ws, size_t ws_bytes) {
    typedef typename Storage<F::N>::T T;
    const ConvDims d = conv_dims(2, g);
    const bool fastp8 = (F::N == 8 && F::ES == 0) && p8_conv_eligible(2, g);
    const size_t bias_ws = bias_grad_ws_bytes<F>(g.N, g.K, g.OH * g.OW);
    GemmPlan plan = conv_plan<F>(d);
    P8ConvProblem p8p;
    if (fastp8) {
        const P8ConvBwPlan bp = p8_conv_bw_plan(g, dbias != nullptr);
        if (bp.ok) {  // integer matrix cores, split reduction; the bias gradient rides along as a column of ones
            if (!ws || ws_bytes < bp.total()) return PNN_EWORKSPACE;
            return hip_status(launch_p8_conv_bw_mfma(st, bp, dy, x, dw, dbias, fout, ws));
        }
        P8PrePlan pp;
        GemmPlan pplan;
        if (p8_pre_usable(2, g, &pp, &pplan)) {
            if (!ws || ws_bytes < p8_pre_ws_bytes(pp, pplan) || (dbias && ws_bytes < bias_ws)) return PNN_EWORKSPACE;
            RowMajorOut pout{d.N};
            hipError_t pe = p8_pre_launch(st, pp, x, dy, nullptr, dw, fout, ws, pplan, pout);  // operand A is x, B is dy
            if (pe == hipSuccess && dbias) pe = launch_bias_grad<F>(st, dy, dbias, fout, g.N, g.K, g.OH * g.OW, ws);
            return hip_status(pe);
        }
    }
    if (fastp8) {
        p8p = p8_problem(2, g, dy, x);
        plan = p8_conv_plan(p8p.M, p8p.N, p8p.K);
    }
    bool fastb8 = false;
    if constexpr (is_b8<F>()) {
        if (p8_conv_eligible(2, g)) {
            fastb8 = true;
            p8p = p8_problem(2, g, dy, x);
            plan = b8_conv_plan<F>(p8p.M, p8p.N, p8p.K);
        }
    }
    if (plan.ws_bytes > 0 && (!ws || ws_bytes < plan.ws_bytes)) return PNN_EWORKSPACE;
    if (dbias && bias_ws > 0 && (!ws || ws_bytes < bias_ws)) return PNN_EWORKSPACE;
    ConvBwdWeightDy<T> a{(const T*)dy, g, d.M, d.K};
    ConvBwdWeightX<T> b{(const T*)x, g, d.N, d.K};
    RowMajorOut out{d.N};
    hipError_t e;
    if (fastp8) {
        e = p8_conv_launch(st, p8p, nullptr, dw, fout, ws, plan, out);
    } else if (fastb8) {
        if constexpr (is_b8<F>()) e = b8_conv_launch<F>(st, p8p, nullptr, dw, fout, ws, plan, out);
        else e = hipErrorInvalidValue;
    } else
        e = launch_quire_gemm<F, decltype(a), decltype(b), RowMajorOut, ConvTile<F>::TM, ConvTile<F>::TN>(
            st, a, b, out, d.M, d.N, d.K, nullptr, dw, fout, ws, plan);
    // dbias[k] = sum dy[n,k,:,:] * 1 : one quire per channel; its slice partials reuse the workspace (stream order)
    if (e == hipSuccess && dbias) e = launch_bias_grad<F>(st, dy, dbias, fout, g.N, g.K, g.OH * g.OW, ws);
    return hip_status(e);
}

}  // namespace pnn

using namespace pnn;

extern "C" size_t posit_conv2d_workspace(int which, int fin, int fout, const pnn_conv2d_desc* desc) {
    (void)fout;
    ConvGeom g;
    if (which < 0 || which > 2 || !is_posit(fin) || !conv_geom(desc, &g)) return 0;
    PNN_DISPATCH_POSIT(fin, return conv_ws<F>(which, g))
    return 0;
}

extern "C" int posit_conv2d_fwd(void* stream, int fin, int fout, const pnn_conv2d_desc* desc, const void* x, const void* w,
                                const void* bias, void* y, void* workspace, size_t workspace_bytes) {
    ConvGeom g;
    if (!is_posit(fin) || !is_posit(fout) || !conv_geom(desc, &g)) return PNN_EINVAL;
    if (g.N == 0 || g.K == 0) return PNN_OK;
    if (!y || (g.C > 0 && (!x || !w))) return PNN_EINVAL;
    if (workspace && !aligned(workspace, 16)) return PNN_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    discard_stale_hip_error();
    PNN_DISPATCH_POSIT(fin, return conv_fwd<F>(st, fout, g, x, w, bias, y, workspace, workspace_bytes))
    return PNN_EINVAL;
}

extern "C" int posit_conv2d_bwd_data(void* stream, int fin, int fout, const pnn_conv2d_desc* desc, const void* dy,
                                     const void* w, void* dx, void* workspace, size_t workspace_bytes) {
    ConvGeom g;
    if (!is_posit(fin) || !is_posit(fout) || !conv_geom(desc, &g)) return PNN_EINVAL;
    if (g.N == 0 || g.C == 0) return PNN_OK;
    if (!dx || (g.K > 0 && (!dy || !w))) return PNN_EINVAL;
    if (workspace && !aligned(workspace, 16)) return PNN_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    discard_stale_hip_error();
    PNN_DISPATCH_POSIT(fin, return conv_bwd_data<F>(st, fout, g, dy, w, dx, workspace, workspace_bytes))
    return PNN_EINVAL;
}

extern "C" int posit_conv2d_bwd_weight(void* stream, int fin, int fout, const pnn_conv2d_desc* desc, const void* dy,
                                       const void* x, void* dw, void* dbias, void* workspace, size_t workspace_bytes) {
    ConvGeom g;
    if (!is_posit(fin) || !is_posit(fout) || !conv_geom(desc, &g)) return PNN_EINVAL;
    if (g.K == 0 || g.C == 0) return PNN_OK;
    if (!dw || (g.N > 0 && (!dy || !x))) return PNN_EINVAL;
    if (workspace && !aligned(workspace, 16)) return PNN_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    discard_stale_hip_error();
    PNN_DISPATCH_POSIT(fin, return conv_bwd_weight<F>(st, fout, g, dy, x, dw, dbias, workspace, workspace_bytes))
    return PNN_EINVAL;
}
