// Exact layer glue between the dot-product layers (paper Fig. 2: ReLU, maximum and
// average pooling): bandwidth-bound kernels on posit patterns.  ReLU and max
// pooling only compare patterns as signed integers; average pooling is the quire
// dot product of the window with the weight 2^-log2(window), rounded once.
#include "api_common.h"
#include "quire_gemm.h"

namespace pnn {

// sign-extend an nbits-wide pattern held in a wider container: posit order == signed integer order
__device__ __forceinline__ int32_t as_signed(uint32_t p, int nbits) {
    return (int32_t)(p << (32 - nbits)) >> (32 - nbits);
}

template <class T>
__global__ __launch_bounds__(256) void relu_kernel(const T* __restrict__ x, T* __restrict__ y, int64_t n, int nbits) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const uint32_t mask = nbits == 32 ? 0xFFFFFFFFu : ((1u << nbits) - 1u);
    const uint32_t p = (uint32_t)x[i] & mask;
    y[i] = (T)((as_signed(p, nbits) > 0 || p == (1u << (nbits - 1))) ? p : 0u);
}

// 16 bytes per thread; n16 = number of whole 16-byte groups (pointers 16-byte aligned)
template <class T>
__global__ __launch_bounds__(256) void relu_vec_kernel(const uint4* __restrict__ x, uint4* __restrict__ y, int64_t n16, int nbits) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n16) return;
    constexpr int PER = 4 / (int)sizeof(T);  // elements per 32-bit word
    constexpr int EB = 8 * (int)sizeof(T);
    const uint32_t mask = nbits == 32 ? 0xFFFFFFFFu : ((1u << nbits) - 1u);
    const uint4 v = x[i];
    uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        uint32_t o = 0;
#pragma unroll
        for (int e = 0; e < PER; ++e) {
            const uint32_t p = (PER == 1 ? w[q] : (w[q] >> (EB * e))) & mask;
            const uint32_t r = (as_signed(p, nbits) > 0 || p == (1u << (nbits - 1))) ? p : 0u;
            o |= PER == 1 ? r : (r << (EB * e));
        }
        w[q] = o;
    }
    y[i] = make_uint4(w[0], w[1], w[2], w[3]);
}

// same-width forward output and gradient (the common case): 16 bytes of each per thread
template <class T>
__global__ __launch_bounds__(256) void relu_bwd_vec_kernel(const uint4* __restrict__ yf, const uint4* __restrict__ dy, uint4* __restrict__ dx,
                                                           int64_t n16, int ybits, int dbits) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n16) return;
    constexpr int PER = 4 / (int)sizeof(T);
    constexpr int EB = 8 * (int)sizeof(T);
    const uint32_t ymask = ybits == 32 ? 0xFFFFFFFFu : ((1u << ybits) - 1u);
    const uint32_t emask = EB == 32 ? 0xFFFFFFFFu : ((1u << EB) - 1u);
    const uint4 a = yf[i], b = dy[i];
    const uint32_t ya[4] = {a.x, a.y, a.z, a.w}, da[4] = {b.x, b.y, b.z, b.w};
    uint32_t w[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        uint32_t o = 0;
#pragma unroll
        for (int e = 0; e < PER; ++e) {
            const uint32_t yv = (PER == 1 ? ya[q] : (ya[q] >> (EB * e))) & ymask;
            const uint32_t dv = (PER == 1 ? da[q] : (da[q] >> (EB * e))) & emask;
            const uint32_t r = yv == (1u << (ybits - 1)) ? (1u << (dbits - 1)) : (as_signed(yv, ybits) > 0 ? dv : 0u);
            o |= PER == 1 ? r : (r << (EB * e));
        }
        w[q] = o;
    }
    dx[i] = make_uint4(w[0], w[1], w[2], w[3]);
}

template <class TY, class TD>
__global__ __launch_bounds__(256) void relu_bwd_kernel(const TY* __restrict__ yf, const TD* __restrict__ dy, TD* __restrict__ dx, int64_t n,
                                                       int ybits, int dbits) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const uint32_t ymask = ybits == 32 ? 0xFFFFFFFFu : ((1u << ybits) - 1u);
    const uint32_t yv = (uint32_t)yf[i] & ymask;
    dx[i] = yv == (1u << (ybits - 1)) ? (TD)(1u << (dbits - 1)) : (as_signed(yv, ybits) > 0 ? dy[i] : (TD)0);
}

template <class T>
__global__ __launch_bounds__(256) void maxpool_fwd_kernel(const T* __restrict__ x, T* __restrict__ y, uint8_t* __restrict__ idx,
                                                          int64_t total, int H, int W, int kh, int kw, int nbits) {
    const int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (o >= total) return;
    const int OW = W / kw, OH = H / kh;
    const int ow = (int)(o % OW);
    const int64_t t = o / OW;
    const int oh = (int)(t % OH);
    const int64_t p = t / OH;
    const T* base = x + (p * H + (int64_t)oh * kh) * W + (int64_t)ow * kw;
    T best = base[0];
    int bi = 0;
    for (int r = 0; r < kh; ++r)
        for (int c = 0; c < kw; ++c) {
            const T v = base[(int64_t)r * W + c];
            if (as_signed((uint32_t)v, nbits) > as_signed((uint32_t)best, nbits)) { best = v; bi = r * kw + c; }
        }
    y[o] = best;
    idx[o] = (uint8_t)bi;
}

template <class T>
__global__ __launch_bounds__(256) void maxpool_bwd_kernel(const T* __restrict__ dy, const uint8_t* __restrict__ idx, T* __restrict__ dx,
                                                          int64_t total_in, int H, int W, int kh, int kw) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total_in) return;
    const int w = (int)(i % W);
    const int64_t t = i / W;
    const int h = (int)(t % H);
    const int64_t p = t / H;
    const int OW = W / kw, OH = H / kh;
    const int64_t o = (p * OH + h / kh) * OW + w / kw;
    const int pos = (h % kh) * kw + (w % kw);
    dx[i] = (idx[o] == pos) ? dy[o] : (T)0;
}

// The same, four consecutive elements of a row per thread (W a multiple of 4, fewer than 2^32 elements): 32-bit index
// arithmetic, the window coordinates of the four stepped instead of divided, one store.
template <class T>
__global__ __launch_bounds__(256) void maxpool_bwd_vec4_kernel(const T* __restrict__ dy, const uint8_t* __restrict__ idx, T* __restrict__ dx,
                                                               uint32_t quads, uint32_t H, uint32_t W, uint32_t kh, uint32_t kw) {
    struct alignas(4 * sizeof(T)) Vec4 { T v[4]; };
    const uint32_t q = blockIdx.x * 256u + threadIdx.x;
    if (q >= quads) return;
    const uint32_t wq = W / 4;
    const uint32_t t = q / wq, w0 = (q - t * wq) * 4;
    const uint32_t p = t / H, h = t - p * H;
    const uint32_t OW = W / kw, OH = H / kh;
    const uint32_t hq = h / kh;
    uint32_t o = (p * OH + hq) * OW + w0 / kw, wm = w0 % kw;
    const uint32_t hk = (h - hq * kh) * kw;
    Vec4 out;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        out.v[u] = (idx[o] == hk + wm) ? dy[o] : (T)0;
        if (++wm == kw) { wm = 0; ++o; }
    }
    reinterpret_cast<Vec4*>(dx)[q] = out;
}

// average pooling: quire dot of the window with the weight 2^-shift (a posit of FIN), one rounding
template <class FIN>
__global__ __launch_bounds__(256) void avgpool_fwd_kernel(const typename Storage<FIN::N>::T* __restrict__ x, void* __restrict__ y, int fout,
                                                          int64_t total, int H, int W, int kh, int kw, uint32_t weight) {
    typedef Arith<FIN> AR;
    const int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (o >= total) return;
    const int OW = W / kw, OH = H / kh;
    const int ow = (int)(o % OW);
    const int64_t t = o / OW;
    const int oh = (int)(t % OH);
    const int64_t p = t / OH;
    const typename Storage<FIN::N>::T* base = x + (p * H + (int64_t)oh * kh) * W + (int64_t)ow * kw;
    uint32_t q[AR::L];
#pragma unroll
    for (int l = 0; l < AR::L; ++l) q[l] = 0;
    bool nar = false;
    const typename AR::Elem wq = AR::stage(weight);
    for (int r = 0; r < kh; ++r)
        for (int c = 0; c < kw; ++c) {
            const uint32_t v = base[(int64_t)r * W + c];
            if (v == FIN::NAR) nar = true;
            AR::mac(q, AR::stage(v), wq);
        }
    round_store<QuireAccum<FIN>, AR::L>(q, nar, fout, y, o);
}

template <class FIN>
__global__ __launch_bounds__(256) void avgpool_bwd_kernel(const typename Storage<FIN::N>::T* __restrict__ dy, void* __restrict__ dx, int fout,
                                                          int64_t total_in, int H, int W, int kh, int kw, uint32_t weight) {
    typedef Arith<FIN> AR;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total_in) return;
    const int w = (int)(i % W);
    const int64_t t = i / W;
    const int h = (int)(t % H);
    const int64_t p = t / H;
    const int OW = W / kw, OH = H / kh;
    const uint32_t v = dy[(p * OH + h / kh) * OW + w / kw];
    uint32_t q[AR::L];
#pragma unroll
    for (int l = 0; l < AR::L; ++l) q[l] = 0;
    AR::mac(q, AR::stage(v), AR::stage(weight));
    round_store<QuireAccum<FIN>, AR::L>(q, v == FIN::NAR, fout, dx, i);
}

inline unsigned blocks_for(int64_t n) { return (unsigned)((n + 255) / 256); }

// pattern of 2^-shift in posit<N,ES>: one / useed^k ... found by construction: value 2^-s has
// regime k = floor(-s / 2^ES), exponent e = -s - k*2^ES, no fraction.
inline uint32_t pow2_pattern(int nbits, int es, int s) {
    const int scale = -s;
    int k = scale >> es;  // floor
    const int e = scale - k * (1 << es);
    // k < 0 here (s > 0): -k zeros, a one, then the exponent bits
    const int rl = 1 - k;
    const int used = rl + es;                 // bits after the sign
    uint32_t body = ((1u << es) | (uint32_t)e);  // "1" then e
    body = body << ((nbits - 1) - used);
    return s == 0 ? (1u << (nbits - 2)) : body;
}

// The pooling weight 2^-s is a posit of format `code` only down to minpos = 2^-((n-2) 2^es).
inline bool pool_weight_fits(int code, int s) {
    int n, es;
    fmt_params(code, n, es);
    return s <= ((n - 2) << es);
}

inline int window_shift(int64_t kh, int64_t kw) {
    const int64_t a = kh * kw;
    if (a <= 0 || (a & (a - 1))) return -1;
    int s = 0;
    while (((int64_t)1 << s) < a) ++s;
    return s;
}

inline bool pool_args_ok(int64_t planes, int64_t H, int64_t W, int64_t kh, int64_t kw) {
    if (planes < 0 || H <= 0 || W <= 0 || kh <= 0 || kw <= 0) return false;
    if (H % kh || W % kw || kh * kw > 255) return false;
    if (H >= ((int64_t)1 << 30) || W >= ((int64_t)1 << 30)) return false;
    return true;
}

}  // namespace pnn

using namespace pnn;

namespace pnn {
inline int bits_of(int code) { int n, es; fmt_params(code, n, es); return n; }

// CALL sees `T`, the container type of format code `code`
#define PNN_BY_STORAGE(code, CALL)                                     \
    switch (elem_size(code)) {                                          \
        case 1: { typedef uint8_t T; CALL; } break;                     \
        case 2: { typedef uint16_t T; CALL; } break;                    \
        default: { typedef uint32_t T; CALL; } break;                   \
    }

template <class TY>
void relu_bwd_pick(hipStream_t st, int fmt_y, int fmt_d, int64_t n, const void* yf, const void* dy, void* dx) {
    PNN_BY_STORAGE(fmt_d, hipLaunchKernelGGL((relu_bwd_kernel<TY, T>), dim3(blocks_for(n)), dim3(256), 0, st, (const TY*)yf,
                                             (const T*)dy, (T*)dx, n, bits_of(fmt_y), bits_of(fmt_d)))
}
}  // namespace pnn

extern "C" int posit_relu(void* stream, int fmt, int64_t n, const void* x, void* y) {
    if (!is_posit(fmt) || n < 0) return PNN_EINVAL;
    if (n == 0) return PNN_OK;
    if (!x || !y) return PNN_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    discard_stale_hip_error();
    int64_t done = 0;  // elements covered by the 16-byte kernel
    if (aligned(x, 16) && aligned(y, 16)) {
        const int64_t per16 = 16 / (int64_t)elem_size(fmt), n16 = n / per16;
        if (n16 > 0)
            PNN_BY_STORAGE(fmt, hipLaunchKernelGGL(relu_vec_kernel<T>, dim3(blocks_for(n16)), dim3(256), 0, st, (const uint4*)x, (uint4*)y,
                                                   n16, bits_of(fmt)))
        done = n16 * per16;
    }
    if (done < n)
        PNN_BY_STORAGE(fmt, hipLaunchKernelGGL(relu_kernel<T>, dim3(blocks_for(n - done)), dim3(256), 0, st, (const T*)x + done,
                                               (T*)y + done, n - done, bits_of(fmt)))
    return hip_status(hipGetLastError());
}

extern "C" int posit_relu_bwd(void* stream, int fmt_y, int fmt_d, int64_t n, const void* y_fwd, const void* dy, void* dx) {
    if (!is_posit(fmt_y) || !is_posit(fmt_d) || n < 0) return PNN_EINVAL;
    if (n == 0) return PNN_OK;
    if (!y_fwd || !dy || !dx) return PNN_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    discard_stale_hip_error();
    int64_t done = 0;
    if (elem_size(fmt_y) == elem_size(fmt_d) && aligned(y_fwd, 16) && aligned(dy, 16) && aligned(dx, 16)) {
        const int64_t per16 = 16 / (int64_t)elem_size(fmt_d), n16 = n / per16;
        if (n16 > 0)
            PNN_BY_STORAGE(fmt_d, hipLaunchKernelGGL(relu_bwd_vec_kernel<T>, dim3(blocks_for(n16)), dim3(256), 0, st, (const uint4*)y_fwd,
                                                     (const uint4*)dy, (uint4*)dx, n16, bits_of(fmt_y), bits_of(fmt_d)))
        done = n16 * per16;
    }
    if (done < n) {
        const char* yb = (const char*)y_fwd + done * (int64_t)elem_size(fmt_y);
        const char* db = (const char*)dy + done * (int64_t)elem_size(fmt_d);
        char* xb = (char*)dx + done * (int64_t)elem_size(fmt_d);
        PNN_BY_STORAGE(fmt_y, relu_bwd_pick<T>(st, fmt_y, fmt_d, n - done, yb, db, xb))
    }
    return hip_status(hipGetLastError());
}

extern "C" int posit_maxpool2d_fwd(void* stream, int fmt, int64_t planes, int64_t H, int64_t W, int64_t kh, int64_t kw,
                                   const void* x, void* y, void* idx) {
    if (!is_posit(fmt) || !pool_args_ok(planes, H, W, kh, kw)) return PNN_EINVAL;
    if (planes == 0) return PNN_OK;
    if (!x || !y || !idx) return PNN_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    discard_stale_hip_error();
    const int64_t total = planes * (H / kh) * (W / kw);
    PNN_BY_STORAGE(fmt, hipLaunchKernelGGL(maxpool_fwd_kernel<T>, dim3(blocks_for(total)), dim3(256), 0, st, (const T*)x, (T*)y,
                                           (uint8_t*)idx, total, (int)H, (int)W, (int)kh, (int)kw, bits_of(fmt)))
    return hip_status(hipGetLastError());
}

extern "C" int posit_maxpool2d_bwd(void* stream, int fmt, int64_t planes, int64_t H, int64_t W, int64_t kh, int64_t kw,
                                   const void* dy, const void* idx, void* dx) {
    if (!is_posit(fmt) || !pool_args_ok(planes, H, W, kh, kw)) return PNN_EINVAL;
    if (planes == 0) return PNN_OK;
    if (!dy || !dx || !idx) return PNN_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    discard_stale_hip_error();
    const int64_t total = planes * H * W;
    if (W % 4 == 0 && total < ((int64_t)1 << 32) && ((uintptr_t)dx & 15u) == 0) {
        const uint32_t quads = (uint32_t)(total / 4);
        PNN_BY_STORAGE(fmt, hipLaunchKernelGGL(maxpool_bwd_vec4_kernel<T>, dim3((quads + 255u) / 256u), dim3(256), 0, st, (const T*)dy,
                                               (const uint8_t*)idx, (T*)dx, quads, (uint32_t)H, (uint32_t)W, (uint32_t)kh, (uint32_t)kw))
        return hip_status(hipGetLastError());
    }
    PNN_BY_STORAGE(fmt, hipLaunchKernelGGL(maxpool_bwd_kernel<T>, dim3(blocks_for(total)), dim3(256), 0, st, (const T*)dy,
                                           (const uint8_t*)idx, (T*)dx, total, (int)H, (int)W, (int)kh, (int)kw))
    return hip_status(hipGetLastError());
}

extern "C" int posit_avgpool2d_fwd(void* stream, int fin, int fout, int64_t planes, int64_t H, int64_t W, int64_t kh, int64_t kw,
                                   const void* x, void* y) {
    if (!is_posit(fin) || !is_posit(fout) || !pool_args_ok(planes, H, W, kh, kw)) return PNN_EINVAL;
    const int s = window_shift(kh, kw);
    if (s < 0 || !pool_weight_fits(fin, s)) return PNN_EUNSUPPORTED;  // window not a power of two, or 1/window below minpos of fin
    if (planes == 0) return PNN_OK;
    if (!x || !y) return PNN_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    discard_stale_hip_error();
    const int64_t total = planes * (H / kh) * (W / kw);
    PNN_DISPATCH_POSIT(fin, hipLaunchKernelGGL(avgpool_fwd_kernel<F>, dim3(blocks_for(total)), dim3(256), 0, st,
                                               (const typename Storage<F::N>::T*)x, y, fout, total, (int)H, (int)W, (int)kh, (int)kw,
                                               pow2_pattern(F::N, F::ES, s)))
    return hip_status(hipGetLastError());
}

extern "C" int posit_avgpool2d_bwd(void* stream, int fin, int fout, int64_t planes, int64_t H, int64_t W, int64_t kh, int64_t kw,
                                   const void* dy, void* dx) {
    if (!is_posit(fin) || !is_posit(fout) || !pool_args_ok(planes, H, W, kh, kw)) return PNN_EINVAL;
    const int s = window_shift(kh, kw);
    if (s < 0 || !pool_weight_fits(fin, s)) return PNN_EUNSUPPORTED;
    if (planes == 0) return PNN_OK;
    if (!dy || !dx) return PNN_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    discard_stale_hip_error();
    const int64_t total = planes * H * W;
    PNN_DISPATCH_POSIT(fin, hipLaunchKernelGGL(avgpool_bwd_kernel<F>, dim3(blocks_for(total)), dim3(256), 0, st,
                                               (const typename Storage<F::N>::T*)dy, dx, fout, total, (int)H, (int)W, (int)kh, (int)kw,
                                               pow2_pattern(F::N, F::ES, s)))
    return hip_status(hipGetLastError());
}
