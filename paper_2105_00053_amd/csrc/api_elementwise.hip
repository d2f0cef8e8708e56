// posit_round, posit_convert, posit_axpy: the bandwidth-bound entry points
// (paper Fig. 2: tensor conversion, mixed-precision copies, SGD).  One thread
// handles a short vector of consecutive elements so that the widest type moves
// 16 bytes per access; a scalar kernel covers unaligned pointers and the tail.
#include "api_common.h"
#include "elementwise_fast.h"

namespace pnn {

template <class TS, class TD, int V, class Op>
__global__ __launch_bounds__(256) void map_vec_kernel(const TS* __restrict__ src, TD* __restrict__ dst, int64_t nvec, Op op) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= nvec) return;
    const Pack<TS, V> in = reinterpret_cast<const Pack<TS, V>*>(src)[i];
    Pack<TD, V> o;
#pragma unroll
    for (int j = 0; j < V; ++j) o.v[j] = (TD)op((uint64_t)in.v[j]);
    reinterpret_cast<Pack<TD, V>*>(dst)[i] = o;
}

template <class TS, class TD, class Op>
__global__ __launch_bounds__(256) void map_scalar_kernel(const TS* __restrict__ src, TD* __restrict__ dst, int64_t begin, int64_t n, Op op) {
    const int64_t i = begin + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    dst[i] = (TD)op((uint64_t)src[i]);
}

// 8-bit sources: the conversion is a function of 256 patterns, so each workgroup
// evaluates it once into an LDS table and then only looks bytes up.  One thread
// produces one 16-byte store (V = 16 / sizeof(TD) elements), so that both the
// loads and the stores of a wavefront are contiguous.
template <class TD, class Op>
__global__ __launch_bounds__(256) void map_p8_table_kernel(const uint8_t* __restrict__ src, TD* __restrict__ dst, int64_t nvec, Op op) {
    constexpr int V = 16 / sizeof(TD);
    __shared__ TD table[256];
    table[threadIdx.x] = (TD)op((uint64_t)threadIdx.x);
    __syncthreads();
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= nvec) return;
    const Pack<uint8_t, V> in = reinterpret_cast<const Pack<uint8_t, V>*>(src)[i];
    Pack<TD, V> o;
#pragma unroll
    for (int j = 0; j < V; ++j) o.v[j] = table[in.v[j]];
    reinterpret_cast<Pack<TD, V>*>(dst)[i] = o;
}

template <class TS, class TD, class Op>
int launch_map(hipStream_t st, const void* src, void* dst, int64_t n, Op op);

template <class TD, class Op>
int launch_map_p8(hipStream_t st, const void* src, void* dst, int64_t n, Op op) {
    int64_t done = 0;
    constexpr int V = 16 / sizeof(TD);
    if (aligned(src, V) && aligned(dst, 16)) {
        const int64_t nvec = n / V;
        if (nvec > 0) {
            hipLaunchKernelGGL((map_p8_table_kernel<TD, Op>), dim3((unsigned)((nvec + 255) / 256)), dim3(256), 0, st,
                               (const uint8_t*)src, (TD*)dst, nvec, op);
            done = nvec * V;
            if (hipGetLastError() != hipSuccess) return PNN_EHIP;  // stop at the first failed launch
        }
    }
    if (done < n) {
        const int64_t rest = n - done;
        hipLaunchKernelGGL((map_scalar_kernel<uint8_t, TD, Op>), dim3((unsigned)((rest + 255) / 256)), dim3(256), 0, st,
                           (const uint8_t*)src, (TD*)dst, done, n, op);
    }
    return hip_status(hipGetLastError());
}

template <class TS, class TD, class Op>
int launch_map(hipStream_t st, const void* src, void* dst, int64_t n, Op op) {
    constexpr int WIDE = sizeof(TS) > sizeof(TD) ? sizeof(TS) : sizeof(TD);
    constexpr int V = 16 / WIDE;
    int64_t done = 0;
    if (aligned(src, sizeof(TS) * V) && aligned(dst, sizeof(TD) * V)) {
        const int64_t nvec = n / V;
        if (nvec > 0) {
            hipLaunchKernelGGL((map_vec_kernel<TS, TD, V, Op>), dim3((unsigned)((nvec + 255) / 256)), dim3(256), 0, st,
                               (const TS*)src, (TD*)dst, nvec, op);
            done = nvec * V;
            if (hipGetLastError() != hipSuccess) return PNN_EHIP;  // stop at the first failed launch
        }
    }
    if (done < n) {
        const int64_t rest = n - done;
        hipLaunchKernelGGL((map_scalar_kernel<TS, TD, Op>), dim3((unsigned)((rest + 255) / 256)), dim3(256), 0, st,
                           (const TS*)src, (TD*)dst, done, n, op);
    }
    return hip_status(hipGetLastError());
}

template <class TX, class TY, class TC, int V, class Op, class Cp>
__global__ __launch_bounds__(256) void axpy_vec_kernel(const TX* __restrict__ x, TY* __restrict__ y, TC* __restrict__ yc,
                                                       int64_t nvec, Op op, Cp cp) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= nvec) return;
    const Pack<TX, V> xv = reinterpret_cast<const Pack<TX, V>*>(x)[i];
    Pack<TY, V> yv = reinterpret_cast<Pack<TY, V>*>(y)[i];
#pragma unroll
    for (int j = 0; j < V; ++j) yv.v[j] = (TY)op((uint32_t)xv.v[j], (uint32_t)yv.v[j]);
    reinterpret_cast<Pack<TY, V>*>(y)[i] = yv;
    if (yc) {  // narrowed copy of the new y (uniform branch)
        Pack<TC, V> cv;
#pragma unroll
        for (int j = 0; j < V; ++j) cv.v[j] = (TC)cp((uint64_t)yv.v[j]);
        reinterpret_cast<Pack<TC, V>*>(yc)[i] = cv;
    }
}

template <class TX, class TY, class TC, class Op, class Cp>
__global__ __launch_bounds__(256) void axpy_scalar_kernel(const TX* __restrict__ x, TY* __restrict__ y, TC* __restrict__ yc,
                                                          int64_t begin, int64_t n, Op op, Cp cp) {
    const int64_t i = begin + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const uint32_t r = op((uint32_t)x[i], (uint32_t)y[i]);
    y[i] = (TY)r;
    if (yc) yc[i] = (TC)cp((uint64_t)r);
}

template <class FX, class FY, class FC>
int launch_axpy(hipStream_t st, uint32_t alpha, int64_t n, const void* x, void* y, void* yc) {
    typedef typename Storage<FX::N>::T TX;
    typedef typename Storage<FY::N>::T TY;
    typedef typename Storage<FC::N>::T TC;
    constexpr int W0 = sizeof(TX) > sizeof(TY) ? sizeof(TX) : sizeof(TY);
    constexpr int WIDE = W0 > (int)sizeof(TC) ? W0 : (int)sizeof(TC);
    constexpr int V = 16 / WIDE;
    Axpy<FX, FY> op;
    op.alpha = alpha;
    PositToPosit<FY, FC> cp;
    int64_t done = 0;
    if (aligned(x, sizeof(TX) * V) && aligned(y, sizeof(TY) * V) && (!yc || aligned(yc, sizeof(TC) * V))) {
        const int64_t nvec = n / V;
        if (nvec > 0) {
            hipLaunchKernelGGL((axpy_vec_kernel<TX, TY, TC, V, Axpy<FX, FY>, PositToPosit<FY, FC>>),
                               dim3((unsigned)((nvec + 255) / 256)), dim3(256), 0, st, (const TX*)x, (TY*)y, (TC*)yc, nvec, op, cp);
            done = nvec * V;
            if (hipGetLastError() != hipSuccess) return PNN_EHIP;  // stop at the first failed launch
        }
    }
    if (done < n) {
        const int64_t rest = n - done;
        hipLaunchKernelGGL((axpy_scalar_kernel<TX, TY, TC, Axpy<FX, FY>, PositToPosit<FY, FC>>),
                           dim3((unsigned)((rest + 255) / 256)), dim3(256), 0, st, (const TX*)x, (TY*)y, (TC*)yc, done, n, op, cp);
    }
    return hip_status(hipGetLastError());
}

// ---- large tensors, formats of at most 16 bits: binary64 arithmetic with LDS decode tables ----

// Below this many elements the per-workgroup table set-up outweighs what the cheaper per-element work saves.
constexpr int64_t AXPY_F64_MIN_16 = (int64_t)1 << 22;  // posit<16,1> tables: 128 KB per workgroup
constexpr int64_t AXPY_F64_MIN_12 = (int64_t)1 << 19;  // 12-bit formats: a few KB
constexpr int64_t NARROW_STEP_MIN = (int64_t)1 << 20;

inline int compute_units() {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) {
        (void)hipGetLastError();
        return 256;
    }
    return cus;
}

// Launches the binary64 kernel on the first n - n % 8 elements; returns false (nothing launched) when it does not apply.
template <class FX, class FY, class FC, bool COPY>
bool launch_axpy_f64(hipStream_t st, uint32_t alpha, int64_t n, const void* x, void* y, void* yc, int64_t* done) {
    typedef typename Storage<FX::N>::T TX;
    typedef typename Storage<FY::N>::T TY;
    typedef typename Storage<FC::N>::T TC;
    constexpr int V = 8;
    constexpr bool BIG = FY::N > 12;  // the decode table fills most of a compute unit's LDS: one workgroup each
    const int64_t nvec = n / V;
    if (n < (BIG ? AXPY_F64_MIN_16 : AXPY_F64_MIN_12) || nvec == 0) return false;
    if (!aligned(x, sizeof(TX) * V) || !aligned(y, sizeof(TY) * V) || (COPY && !aligned(yc, sizeof(TC) * V))) return false;
    constexpr int THREADS = 1024;
    int64_t blocks = (int64_t)compute_units() * (BIG ? 1 : 2);
    const int64_t need = (nvec + THREADS - 1) / THREADS;
    if (blocks > need) blocks = need;
    hipLaunchKernelGGL((axpy_f64_kernel<FX, FY, FC, COPY, THREADS>), dim3((unsigned)blocks), dim3(THREADS), 0, st, (const TX*)x, (TY*)y,
                       (TC*)yc, nvec, alpha);
    *done = nvec * V;
    return true;
}

// Format triples the binary64 kernel is built for: the default mixed-precision set-up (16-bit optimizer, 8-bit
// compute copy) and the paper's final one (posit(12,2) optimizer, posit(8,2) layers: Sec. 4, Table 4).
inline bool axpy_f64_dispatch(hipStream_t st, int fx, int fy, int fcopy, bool copy, uint32_t alpha, int64_t n, const void* x, void* y,
                              void* yc, int64_t* done) {
#define PNN_AXPY_F64(FX, FY, FC, CX, CY, CC)                                                                  \
    if (fx == CX && fy == CY) {                                                                               \
        if (!copy) return launch_axpy_f64<FX, FY, FC, false>(st, alpha, n, x, y, nullptr, done);              \
        if (fcopy == CC) return launch_axpy_f64<FX, FY, FC, true>(st, alpha, n, x, y, yc, done);              \
        return false;                                                                                         \
    }
    PNN_AXPY_F64(P16, P16, P8, PNN_POSIT16_1, PNN_POSIT16_1, PNN_POSIT8_0)
    PNN_AXPY_F64(P8, P16, P8, PNN_POSIT8_0, PNN_POSIT16_1, PNN_POSIT8_0)
    PNN_AXPY_F64(P12_2, P12_2, P8_2, PNN_POSIT12_2, PNN_POSIT12_2, PNN_POSIT8_2)
    PNN_AXPY_F64(P8_2, P12_2, P8_2, PNN_POSIT8_2, PNN_POSIT12_2, PNN_POSIT8_2)
#undef PNN_AXPY_F64
    return false;
}

template <class FX, class FY>
int axpy_pick_copy(hipStream_t st, uint32_t alpha, int64_t n, const void* x, void* y, int fcopy, void* yc) {
    if (!yc) return launch_axpy<FX, FY, FY>(st, alpha, n, x, y, nullptr);
    switch (fcopy) {
        case PNN_POSIT8_0: return launch_axpy<FX, FY, P8>(st, alpha, n, x, y, yc);
        case PNN_POSIT16_1: return launch_axpy<FX, FY, P16>(st, alpha, n, x, y, yc);
        case PNN_POSIT32_2: return launch_axpy<FX, FY, P32>(st, alpha, n, x, y, yc);
    }
    return PNN_EINVAL;
}

template <class FX>
int axpy_pick_y(hipStream_t st, int fy, uint32_t alpha, int64_t n, const void* x, void* y, int fcopy, void* yc) {
    switch (fy) {
        case PNN_POSIT8_0: return axpy_pick_copy<FX, P8>(st, alpha, n, x, y, fcopy, yc);
        case PNN_POSIT16_1: return axpy_pick_copy<FX, P16>(st, alpha, n, x, y, fcopy, yc);
        case PNN_POSIT32_2: return axpy_pick_copy<FX, P32>(st, alpha, n, x, y, fcopy, yc);
    }
    return PNN_EINVAL;
}

template <class FS>
int convert_from(hipStream_t st, int dst, int64_t n, const void* s, void* d) {
    typedef typename Storage<FS::N>::T TS;
    if (FS::N == 8) {
        switch (dst) {
            case PNN_POSIT8_0: return launch_map_p8<uint8_t>(st, s, d, n, PositToPosit<FS, P8>());
            case PNN_POSIT16_1: return launch_map_p8<uint16_t>(st, s, d, n, PositToPosit<FS, P16>());
            case PNN_POSIT32_2: return launch_map_p8<uint32_t>(st, s, d, n, PositToPosit<FS, P32>());
            case PNN_F32: return launch_map_p8<uint32_t>(st, s, d, n, PositToF32<FS>());
            case PNN_F64: return launch_map_p8<uint64_t>(st, s, d, n, PositToF64<FS>());
        }
        return PNN_EINVAL;
    }
    if (FS::N == 16 && dst == PNN_POSIT8_0 && n >= NARROW_STEP_MIN && aligned(s, 16) && aligned(d, 8)) {
        // step-table kernel on whole vectors of 8, the generic kernel on what is left
        const int64_t nvec = n / 8;
        int64_t blocks = (nvec + 255) / 256;
        const int64_t cap = (int64_t)compute_units() * 8;
        if (blocks > cap) blocks = cap;
        hipLaunchKernelGGL((narrow_step_kernel<P16, P8>), dim3((unsigned)blocks), dim3(256), 0, st, (const uint16_t*)s, (uint8_t*)d, nvec);
        if (hipGetLastError() != hipSuccess) return PNN_EHIP;
        const int64_t done = nvec * 8;
        if (done == n) return PNN_OK;
        return launch_map<TS, uint8_t>(st, (const TS*)s + done, (uint8_t*)d + done, n - done, PositToPosit<FS, P8>());
    }
    switch (dst) {
        case PNN_POSIT8_0: return launch_map<TS, uint8_t>(st, s, d, n, PositToPosit<FS, P8>());
        case PNN_POSIT16_1: return launch_map<TS, uint16_t>(st, s, d, n, PositToPosit<FS, P16>());
        case PNN_POSIT32_2: return launch_map<TS, uint32_t>(st, s, d, n, PositToPosit<FS, P32>());
        case PNN_F32: return launch_map<TS, uint32_t>(st, s, d, n, PositToF32<FS>());
        case PNN_F64: return launch_map<TS, uint64_t>(st, s, d, n, PositToF64<FS>());
    }
    return PNN_EINVAL;
}

// Any-format kernels: element sizes and formats are run-time values (uniform branches).
__device__ __forceinline__ uint64_t load_elem(const void* p, int64_t i, int bytes) {
    if (bytes == 1) return ((const uint8_t*)p)[i];
    if (bytes == 2) return ((const uint16_t*)p)[i];
    if (bytes == 4) return ((const uint32_t*)p)[i];
    return ((const uint64_t*)p)[i];
}

__device__ __forceinline__ void store_elem(void* p, int64_t i, int bytes, uint64_t v) {
    if (bytes == 1) ((uint8_t*)p)[i] = (uint8_t)v;
    else if (bytes == 2) ((uint16_t*)p)[i] = (uint16_t)v;
    else if (bytes == 4) ((uint32_t*)p)[i] = (uint32_t)v;
    else ((uint64_t*)p)[i] = v;
}

__global__ __launch_bounds__(256) void map_rt_kernel(const void* __restrict__ src, void* __restrict__ dst, int sbytes, int dbytes,
                                                     int64_t n, MapRT op) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    store_elem(dst, i, dbytes, op(load_elem(src, i, sbytes)));
}

__global__ __launch_bounds__(256) void axpy_rt_kernel(const void* __restrict__ x, void* __restrict__ y, void* __restrict__ yc, int xbytes,
                                                      int ybytes, int cbytes, int64_t n, AxpyRT op, MapRT cp) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const uint32_t r = op((uint32_t)load_elem(x, i, xbytes), (uint32_t)load_elem(y, i, ybytes));
    store_elem(y, i, ybytes, r);
    if (yc) store_elem(yc, i, cbytes, cp((uint64_t)r));
}

// Several tensors in one launch (the SGD update of a whole model: many small tensors, each a launch
// of its own otherwise).  blockIdx.y picks the tensor; the descriptors travel as kernel arguments.
constexpr int AXPY_MULTI_MAX = 16;
struct AxpyItems {
    const void* x[AXPY_MULTI_MAX];
    void* y[AXPY_MULTI_MAX];
    void* yc[AXPY_MULTI_MAX];
    int64_t n[AXPY_MULTI_MAX];
};

__global__ __launch_bounds__(256) void axpy_multi_kernel(AxpyItems items, int xbytes, int ybytes, int cbytes, AxpyRT op, MapRT cp) {
    const int it = blockIdx.y;
    const void* x = items.x[it];
    void* y = items.y[it];
    void* yc = items.yc[it];
    const int64_t n = items.n[it];
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
        const uint32_t r = op((uint32_t)load_elem(x, i, xbytes), (uint32_t)load_elem(y, i, ybytes));
        store_elem(y, i, ybytes, r);
        if (yc) store_elem(yc, i, cbytes, cp((uint64_t)r));
    }
}

inline MapRT make_map(int src, int dst) {
    MapRT m;
    m.src_kind = src == PNN_F32 ? 1 : (src == PNN_F64 ? 2 : 0);
    m.dst_kind = dst == PNN_F32 ? 1 : (dst == PNN_F64 ? 2 : 0);
    m.fs = fmt_of_code(m.src_kind ? 0 : src);
    m.fd = fmt_of_code(m.dst_kind ? 0 : dst);
    return m;
}

inline int launch_map_rt(hipStream_t st, int src, int dst, int64_t n, const void* s, void* d) {
    hipLaunchKernelGGL(map_rt_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, s, d, (int)elem_size(src), (int)elem_size(dst), n,
                       make_map(src, dst));
    return hip_status(hipGetLastError());
}

}  // namespace pnn

using namespace pnn;

extern "C" int posit_round(void* stream, int src_float, int dst_posit, int64_t n, const void* src, void* dst) {
    if (!is_float(src_float) || !is_posit(dst_posit) || n < 0) return PNN_EINVAL;
    if (n == 0) return PNN_OK;
    if (!src || !dst) return PNN_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    discard_stale_hip_error();
    if (!is_standard(dst_posit)) return launch_map_rt(st, src_float, dst_posit, n, src, dst);
    if (src_float == PNN_F32) {
        switch (dst_posit) {
            case PNN_POSIT8_0: return launch_map<uint32_t, uint8_t>(st, src, dst, n, RoundF32<P8>());
            case PNN_POSIT16_1: return launch_map<uint32_t, uint16_t>(st, src, dst, n, RoundF32<P16>());
            default: return launch_map<uint32_t, uint32_t>(st, src, dst, n, RoundF32<P32>());
        }
    }
    switch (dst_posit) {
        case PNN_POSIT8_0: return launch_map<uint64_t, uint8_t>(st, src, dst, n, RoundF64<P8>());
        case PNN_POSIT16_1: return launch_map<uint64_t, uint16_t>(st, src, dst, n, RoundF64<P16>());
        default: return launch_map<uint64_t, uint32_t>(st, src, dst, n, RoundF64<P32>());
    }
}

extern "C" int posit_convert(void* stream, int src, int dst, int64_t n, const void* src_ptr, void* dst_ptr) {
    if (!is_posit(src) || !(is_posit(dst) || is_float(dst)) || n < 0) return PNN_EINVAL;
    if (n == 0) return PNN_OK;
    if (!src_ptr || !dst_ptr) return PNN_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    discard_stale_hip_error();
    if (!is_standard(src) || !is_standard(dst)) return launch_map_rt(st, src, dst, n, src_ptr, dst_ptr);
    switch (src) {
        case PNN_POSIT8_0: return convert_from<P8>(st, dst, n, src_ptr, dst_ptr);
        case PNN_POSIT16_1: return convert_from<P16>(st, dst, n, src_ptr, dst_ptr);
        default: return convert_from<P32>(st, dst, n, src_ptr, dst_ptr);
    }
}

extern "C" int posit_axpy(void* stream, int fx, int fy, uint32_t alpha_bits, int64_t n, const void* x, void* y,
                          int fcopy, void* y_copy) {
    if (!is_posit(fx) || !is_posit(fy) || n < 0) return PNN_EINVAL;
    if (y_copy && !is_posit(fcopy)) return PNN_EINVAL;
    if (n == 0) return PNN_OK;
    if (!x || !y) return PNN_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    discard_stale_hip_error();
    {
        int64_t done = 0;
        if (axpy_f64_dispatch(st, fx, fy, fcopy, y_copy != nullptr, alpha_bits, n, x, y, y_copy, &done)) {
            if (hipGetLastError() != hipSuccess) return PNN_EHIP;
            if (done == n) return PNN_OK;
            // the last n % 8 elements go through the generic path below
            x = (const uint8_t*)x + done * elem_size(fx);
            y = (uint8_t*)y + done * elem_size(fy);
            if (y_copy) y_copy = (uint8_t*)y_copy + done * elem_size(fcopy);
            n -= done;
        }
    }
    if (!is_standard(fx) || !is_standard(fy) || (y_copy && !is_standard(fcopy))) {
        AxpyRT op;
        op.fx = fmt_of_code(fx);
        op.fy = fmt_of_code(fy);
        op.alpha = alpha_bits;
        const int fc = y_copy ? fcopy : fy;
        hipLaunchKernelGGL(axpy_rt_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, x, y, y_copy, (int)elem_size(fx),
                           (int)elem_size(fy), (int)elem_size(fc), n, op, make_map(fy, fc));
        return hip_status(hipGetLastError());
    }
    switch (fx) {
        case PNN_POSIT8_0: return axpy_pick_y<P8>(st, fy, alpha_bits, n, x, y, fcopy, y_copy);
        case PNN_POSIT16_1: return axpy_pick_y<P16>(st, fy, alpha_bits, n, x, y, fcopy, y_copy);
        default: return axpy_pick_y<P32>(st, fy, alpha_bits, n, x, y, fcopy, y_copy);
    }
}

extern "C" int posit_axpy_multi(void* stream, int fx, int fy, uint32_t alpha_bits, int count, const pnn_axpy_item* items, int fcopy) {
    if (!is_posit(fx) || !is_posit(fy) || count < 0 || (count > 0 && !items)) return PNN_EINVAL;
    bool any_copy = false;
    for (int i = 0; i < count; ++i) {
        if (items[i].n < 0) return PNN_EINVAL;
        if (items[i].n > 0 && (!items[i].x || !items[i].y)) return PNN_EINVAL;
        any_copy = any_copy || items[i].y_copy != nullptr;
    }
    if (any_copy && !is_posit(fcopy)) return PNN_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    discard_stale_hip_error();
    AxpyRT op;
    op.fx = fmt_of_code(fx);
    op.fy = fmt_of_code(fy);
    op.alpha = alpha_bits;
    const int fc = any_copy ? fcopy : fy;
    bool launched = false;
    for (int base = 0; base < count; base += AXPY_MULTI_MAX) {
        AxpyItems pack;
        int used = 0;
        int64_t longest = 0;
        for (int i = base; i < count && i < base + AXPY_MULTI_MAX; ++i) {
            if (items[i].n == 0) continue;
            pack.x[used] = items[i].x; pack.y[used] = items[i].y; pack.yc[used] = items[i].y_copy; pack.n[used] = items[i].n;
            if (items[i].n > longest) longest = items[i].n;
            ++used;
        }
        if (used == 0) continue;
        int64_t blocks = (longest + 255) / 256;
        if (blocks > 1024) blocks = 1024;
        hipLaunchKernelGGL(axpy_multi_kernel, dim3((unsigned)blocks, (unsigned)used), dim3(256), 0, st, pack, (int)elem_size(fx),
                           (int)elem_size(fy), (int)elem_size(fc), op, make_map(fy, fc));
        launched = true;
    }
    return launched ? hip_status(hipGetLastError()) : PNN_OK;
}

extern "C" const char* posit_status_string(int status) {
    switch (status) {
        case PNN_OK: return "ok";
        case PNN_EINVAL: return "invalid argument";
        case PNN_EUNSUPPORTED: return "unsupported format combination";
        case PNN_EWORKSPACE: return "workspace too small";
        case PNN_EHIP: return "HIP runtime error";
    }
    return "unknown status";
}
