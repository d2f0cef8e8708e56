// posit_gemm: quire-exact matrix product (paper Sec. 3.3; the Linear layer's
// forward, backward-data and backward-weight passes of Sec. 3.1 are its
// transposition cases).
#include <mutex>

#include "api_common.h"
#include "conv_p8.h"
#include "gemm_p8_w4.h"
#include "gemm_p8_mfma.h"
#include "gemm_b8_mfma.h"
#include "conv_b8.h"
#include "gemm_bucket_pre.h"
#include "gemm_p16_window.h"
#include "gemm_p32_lds.h"

namespace pnn {

template <class F> struct GemmTile { static constexpr int TM = 4, TN = 4; };
template <> struct GemmTile<P32> { static constexpr int TM = 2, TN = 2; };

// posit<8,0> problems with both output dimensions beyond one small tile take the dot2 kernel
inline bool use_p8_kernel(int64_t M, int64_t N) { return M > 64 && N > 64; }

// ... and of those, the ones with too few 128 x 128 tiles to fill the chip go to the 64 x 64 kernel whose four waves
// split the reduction (larger products decode and pack their operands once instead)
inline bool use_p8_w4(int64_t M, int64_t N, int64_t K) { return use_p8_kernel(M, N) && p8_w4_fits(M, N, K) && !p8_packed_gemm_fits(M, N, K); }

// posit(8,1) / posit(8,2): the byte-gather kernel with fp64 buckets
template <class F>
constexpr bool is_b8() { return F::N == 8 && F::ES != 0; }

template <class F>
GemmPlan gemm_plan(int64_t M, int64_t N, int64_t K) {
    if constexpr (is_b8<F>()) {
        if (p8_small_gemm_fits(M, N, K)) {  // one thread group per output: no workspace
            GemmPlan p;
            p.splits = 1; p.k_per_split = K; p.ws_bytes = 0;
            return p;
        }
        if (b8_mfma_fits<F>(M, N, K)) {  // digit planes of both operands for the integer matrix cores
            GemmPlan p;
            p.splits = 1; p.k_per_split = K; p.ws_bytes = b8_mfma_layout<F>(M, N, K).total();
            return p;
        }
        if (M < ((int64_t)1 << 31) && N < ((int64_t)1 << 31) && K < ((int64_t)1 << 31)) return b8_conv_plan<F>((int)M, (int)N, (int)K);
    }
    if ((F::N == 8 && F::ES == 0) && p8_small_gemm_fits(M, N, K)) {  // one thread group per output: no workspace
        GemmPlan p;
        p.splits = 1; p.k_per_split = K; p.ws_bytes = 0;
        return p;
    }
    if ((F::N == 8 && F::ES == 0) && p8_mfma_fits(M, N, K)) {  // digit planes of both operands for the integer matrix cores
        GemmPlan p;
        p.splits = 1; p.k_per_split = K; p.ws_bytes = p8_mfma_layout(M, N, K).total();
        return p;
    }
    if ((F::N == 8 && F::ES == 0) && use_p8_w4(M, N, K)) return p8_w4_plan(M, N, K).gemm;  // the reduction is cut inside the workgroup first
    if ((F::N == 8 && F::ES == 0) && use_p8_kernel(M, N)) {
        GemmPlan p = plan_split(M, N, K, P8_BM, P8_BN, 1, P8_KT);
        if (p8_packed_gemm_fits(M, N, K)) p.ws_bytes += p8_packed_layout(M, N, K).total();  // operands packed once, ahead of the split partials
        return p;
    }
    // other posit<8,0> shapes go to the gather kernel (tile chosen per shape); the plan does not depend on pitches
    if ((F::N == 8 && F::ES == 0) && M < ((int64_t)1 << 31) && N < ((int64_t)1 << 31) && K < ((int64_t)1 << 31)) return p8_conv_plan((int)M, (int)N, (int)K);
    if (F::N == 32 && p32_lds_fits(M, N, K)) {  // the quire of every output lives in LDS for the whole reduction: no workspace
        GemmPlan p;
        p.splits = 1; p.k_per_split = K; p.ws_bytes = 0;
        return p;
    }
    if (F::N == 16 && pw_fits(M, N, K)) return pw_plan(M, N, K).gemm;          // posit<16,1>: operands decoded once, two buckets + outlier bitmaps
    if (bucket_pre_fits<F>(M, N, K)) return bucket_pre_plan<F>(M, N, K).gemm;  // operands decoded once into the workspace
    return plan_split(M, N, K, 16 * GemmTile<F>::TM, 16 * GemmTile<F>::TN, Arith<F>::L);
}

template <class F>
int gemm_dispatch(hipStream_t st, int fout, int transA, int transB, int64_t M, int64_t N, int64_t K,
                  const void* A, int64_t lda, const void* B, int64_t ldb, const void* bias, void* C, int64_t ldc,
                  void* ws, size_t ws_bytes) {
    typedef typename Storage<F::N>::T T;
    constexpr int TM = GemmTile<F>::TM, TN = GemmTile<F>::TN;
    const GemmPlan plan = gemm_plan<F>(M, N, K);
    if (plan.ws_bytes > 0 && (!ws || ws_bytes < plan.ws_bytes)) return PNN_EWORKSPACE;
    RowMajorOut out;
    out.ld = ldc;
    hipError_t e;
    if ((F::N == 8 && F::ES == 0) && p8_small_gemm_fits(M, N, K))
        return hip_status(launch_p8_small_gemm(st, transA, transB, (const uint8_t*)A, lda, (const uint8_t*)B, ldb, (const uint8_t*)bias, C, ldc,
                                               fout, M, N, K));
    if ((F::N == 8 && F::ES == 0) && p8_mfma_fits(M, N, K))
        return hip_status(launch_p8_mfma_gemm(st, transA, transB, (const uint8_t*)A, lda, (const uint8_t*)B, ldb, (const uint8_t*)bias, C, ldc, fout,
                                              M, N, K, ws));
    if ((F::N == 8 && F::ES == 0) && use_p8_w4(M, N, K)) {
        const uint8_t* a8 = (const uint8_t*)A;
        const uint8_t* b8 = (const uint8_t*)B;
        const uint8_t* bias8 = (const uint8_t*)bias;
        if (!transA && !transB) e = launch_p8_gemm_w4<true, false>(st, a8, lda, b8, ldb, bias8, C, ldc, fout, M, N, K, ws);
        else if (!transA && transB) e = launch_p8_gemm_w4<true, true>(st, a8, lda, b8, ldb, bias8, C, ldc, fout, M, N, K, ws);
        else if (transA && !transB) e = launch_p8_gemm_w4<false, false>(st, a8, lda, b8, ldb, bias8, C, ldc, fout, M, N, K, ws);
        else e = launch_p8_gemm_w4<false, true>(st, a8, lda, b8, ldb, bias8, C, ldc, fout, M, N, K, ws);
        return hip_status(e);
    }
    if ((F::N == 8 && F::ES == 0) && use_p8_kernel(M, N) && p8_packed_gemm_fits(M, N, K)) {
        return hip_status(launch_p8_gemm_packed(st, transA, transB, (const uint8_t*)A, lda, (const uint8_t*)B, ldb, (const uint8_t*)bias, C, ldc,
                                                fout, M, N, K, ws, plan));
    }
    if ((F::N == 8 && F::ES == 0) && use_p8_kernel(M, N)) {
        const uint8_t* a8 = (const uint8_t*)A;
        const uint8_t* b8 = (const uint8_t*)B;
        const uint8_t* bias8 = (const uint8_t*)bias;
        // operand tiles are (rows x k): A's rows are m, B's rows are n; B is k-contiguous only when transposed
        if (!transA && !transB) e = launch_p8_gemm<true, false>(st, a8, lda, b8, ldb, bias8, C, ldc, fout, M, N, K, ws, plan);
        else if (!transA && transB) e = launch_p8_gemm<true, true>(st, a8, lda, b8, ldb, bias8, C, ldc, fout, M, N, K, ws, plan);
        else if (transA && !transB) e = launch_p8_gemm<false, false>(st, a8, lda, b8, ldb, bias8, C, ldc, fout, M, N, K, ws, plan);
        else e = launch_p8_gemm<false, true>(st, a8, lda, b8, ldb, bias8, C, ldc, fout, M, N, K, ws, plan);
        return hip_status(e);
    }
    if ((F::N == 8 && F::ES == 0) && p8_gemm_as_gather_fits(transA, transB, M, N, K, lda, ldb)) {
        const P8ConvProblem p = p8_gemm_problem(transA, transB, (int)M, (int)N, (int)K, A, (int)lda, B, (int)ldb, ldc);
        return hip_status(p8_conv_launch_rowmajor(st, p, (const uint8_t*)bias, C, fout, ws, plan, ldc));
    }
    if constexpr (is_b8<F>()) {
        if (p8_small_gemm_fits(M, N, K))
            return hip_status(launch_b8_small_gemm<F>(st, transA, transB, (const uint8_t*)A, lda, (const uint8_t*)B, ldb, (const uint8_t*)bias, C,
                                                      ldc, fout, M, N, K));
        if (b8_mfma_fits<F>(M, N, K))
            return hip_status(launch_b8_mfma_gemm<F>(st, transA, transB, (const uint8_t*)A, lda, (const uint8_t*)B, ldb, (const uint8_t*)bias, C, ldc,
                                                     fout, M, N, K, ws));
        if (p8_gemm_as_gather_fits(transA, transB, M, N, K, lda, ldb)) {
            const P8ConvProblem p = p8_gemm_problem(transA, transB, (int)M, (int)N, (int)K, A, (int)lda, B, (int)ldb, ldc);
            RowMajorOut mo{ldc};
            return hip_status(b8_conv_launch<F>(st, p, (const uint8_t*)bias, C, fout, ws, plan, mo));
        }
    }
    if constexpr (F::N == 32) {
        if (p32_lds_fits(M, N, K)) {
            if (!transA && !transB) {
                MatrixOperand<T, true> a{(const T*)A, lda, M, K};
                MatrixOperand<T, false> b{(const T*)B, ldb, N, K};
                return hip_status(launch_p32_lds_gemm(st, a, b, M, N, K, bias, C, ldc, fout));
            } else if (!transA && transB) {
                MatrixOperand<T, true> a{(const T*)A, lda, M, K};
                MatrixOperand<T, true> b{(const T*)B, ldb, N, K};
                return hip_status(launch_p32_lds_gemm(st, a, b, M, N, K, bias, C, ldc, fout));
            } else if (transA && !transB) {
                MatrixOperand<T, false> a{(const T*)A, lda, M, K};
                MatrixOperand<T, false> b{(const T*)B, ldb, N, K};
                return hip_status(launch_p32_lds_gemm(st, a, b, M, N, K, bias, C, ldc, fout));
            } else {
                MatrixOperand<T, false> a{(const T*)A, lda, M, K};
                MatrixOperand<T, true> b{(const T*)B, ldb, N, K};
                return hip_status(launch_p32_lds_gemm(st, a, b, M, N, K, bias, C, ldc, fout));
            }
        }
    }
    if constexpr (F::N == 16) {
        if (pw_fits(M, N, K)) return hip_status(launch_pw_gemm(st, transA, transB, A, lda, B, ldb, bias, C, ldc, fout, M, N, K, ws));
    }
    if constexpr (bucket_pre_format<F>()) {
        if (bucket_pre_fits<F>(M, N, K))
            return hip_status(launch_bucket_pre_gemm<F>(st, transA, transB, A, lda, B, ldb, bias, C, ldc, fout, M, N, K, ws));
    }
    // op(A)[i,k]: k contiguous unless transA.  op(B)[k,j] seen as rows j: k contiguous only when transB.
    if (!transA && !transB) {
        MatrixOperand<T, true> a{(const T*)A, lda, M, K};
        MatrixOperand<T, false> b{(const T*)B, ldb, N, K};
        e = launch_quire_gemm<F, decltype(a), decltype(b), RowMajorOut, TM, TN>(st, a, b, out, M, N, K, bias, C, fout, ws, plan);
    } else if (!transA && transB) {
        MatrixOperand<T, true> a{(const T*)A, lda, M, K};
        MatrixOperand<T, true> b{(const T*)B, ldb, N, K};
        e = launch_quire_gemm<F, decltype(a), decltype(b), RowMajorOut, TM, TN>(st, a, b, out, M, N, K, bias, C, fout, ws, plan);
    } else if (transA && !transB) {
        MatrixOperand<T, false> a{(const T*)A, lda, M, K};
        MatrixOperand<T, false> b{(const T*)B, ldb, N, K};
        e = launch_quire_gemm<F, decltype(a), decltype(b), RowMajorOut, TM, TN>(st, a, b, out, M, N, K, bias, C, fout, ws, plan);
    } else {
        MatrixOperand<T, false> a{(const T*)A, lda, M, K};
        MatrixOperand<T, true> b{(const T*)B, ldb, N, K};
        e = launch_quire_gemm<F, decltype(a), decltype(b), RowMajorOut, TM, TN>(st, a, b, out, M, N, K, bias, C, fout, ws, plan);
    }
    return hip_status(e);
}

}  // namespace pnn

using namespace pnn;

extern "C" size_t posit_gemm_workspace(int fin, int fout, int transA, int transB, int64_t M, int64_t N, int64_t K) {
    (void)fout; (void)transA; (void)transB;
    if (!is_posit(fin) || M <= 0 || N <= 0 || K < 0) return 0;
    PNN_DISPATCH_POSIT(fin, return gemm_plan<F>(M, N, K).ws_bytes)
    return 0;
}

// Argument checks shared by the entry points below.  *launch is set when there is work to do.
static int gemm_check_args(int fin, int fout, int transA, int transB, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
                           const void* B, int64_t ldb, const void* C, int64_t ldc, bool* launch) {
    *launch = false;
    if (!is_posit(fin) || !is_posit(fout) || M < 0 || N < 0 || K < 0) return PNN_EINVAL;
    if (M == 0 || N == 0) return PNN_OK;
    if (!C || ldc < N) return PNN_EINVAL;
    if (K > 0) {
        if (!A || !B) return PNN_EINVAL;
        if (lda < (transA ? M : K) || ldb < (transB ? K : N)) return PNN_EINVAL;
    }
    if (M >= ((int64_t)1 << 31) || N >= ((int64_t)1 << 31) || K >= ((int64_t)1 << 31) || M * N >= ((int64_t)1 << 40)) return PNN_EUNSUPPORTED;
    *launch = true;
    return PNN_OK;
}

extern "C" int posit_gemm(void* stream, int fin, int fout, int transA, int transB, int64_t M, int64_t N, int64_t K,
                          const void* A, int64_t lda, const void* B, int64_t ldb, const void* bias, void* C, int64_t ldc,
                          void* workspace, size_t workspace_bytes) {
    bool launch;
    const int rc = gemm_check_args(fin, fout, transA, transB, M, N, K, A, lda, B, ldb, C, ldc, &launch);
    if (!launch) return rc;
    if (workspace && ((uintptr_t)workspace & 15u) != 0) return PNN_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    discard_stale_hip_error();
    PNN_DISPATCH_POSIT(fin, return gemm_dispatch<F>(st, fout, transA, transB, M, N, K, A, lda, B, ldb, bias, C, ldc, workspace, workspace_bytes))
    return PNN_EINVAL;
}

// ---- posit_gemm for callers that cannot allocate device memory ----
//
// The workspace of posit_gemm (partial quires of a split reduction, packed operands) lives in a
// fixed array inside the library's code object instead of a caller's buffer.  Each GPU the library
// runs on holds its own copy of the array at its own address; in host code the array's name is
// only a handle for hipGetSymbolAddress, never a device address, so the address is looked up once
// per device (first call with that device current) and that pointer is what the kernels receive.

static __device__ __align__(256) unsigned char scratch[PNN_GEMM_STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
void* g_scratch_ptr[MAX_DEVICES];  // per device: device address of `scratch`, null until looked up
std::mutex g_scratch_mutex;

// Device address of the current device's copy of `scratch`.
int scratch_address(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return PNN_EHIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return PNN_EHIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return PNN_OK;
}
}  // namespace

extern "C" int posit_gemm_static(void* stream, int fin, int fout, int transA, int transB, int64_t M, int64_t N, int64_t K,
                                 const void* A, int64_t lda, const void* B, int64_t ldb, const void* bias, void* C, int64_t ldc) {
    bool launch;
    const int rc = gemm_check_args(fin, fout, transA, transB, M, N, K, A, lda, B, ldb, C, ldc, &launch);
    if (!launch) return rc;
    const size_t need = posit_gemm_workspace(fin, fout, transA, transB, M, N, K);
    if (need > PNN_GEMM_STATIC_SCRATCH_BYTES) return PNN_EWORKSPACE;  // beyond the fixed array: posit_gemm with a caller's workspace
    void* ws = nullptr;
    if (need > 0) {
        const int rs = scratch_address(&ws);
        if (rs != PNN_OK) return rs;
    }
    hipStream_t st = (hipStream_t)stream;
    discard_stale_hip_error();
    const size_t ws_bytes = need > 0 ? (size_t)PNN_GEMM_STATIC_SCRATCH_BYTES : 0;
    PNN_DISPATCH_POSIT(fin, return gemm_dispatch<F>(st, fout, transA, transB, M, N, K, A, lda, B, ldb, bias, C, ldc, ws, ws_bytes))
    return PNN_EINVAL;
}
