// posit_unary / posit_unary_bwd / posit_cross_entropy / posit_mse: activations and
// losses on posits (paper Fig. 2: Sigmoid, TanH, Cross Entropy, MSE; Fig. 3 and
// Sec. 4, Table 4: the loss stage runs in a posit format of its own).  Small,
// latency-bound kernels: the losses see batch x classes values, so one workgroup
// handles the whole batch and reduces the per-row losses exactly in the loss
// format's quire.
#include "api_common.h"
#include "loss_ops.h"

namespace pnn {

__device__ __forceinline__ uint32_t load_pattern(const void* p, int64_t i, int bytes) {
    return bytes == 1 ? (uint32_t)((const uint8_t*)p)[i] : (uint32_t)((const uint16_t*)p)[i];
}
__device__ __forceinline__ void store_pattern(void* p, int64_t i, int bytes, uint32_t v) {
    if (bytes == 1) ((uint8_t*)p)[i] = (uint8_t)v;
    else ((uint16_t*)p)[i] = (uint16_t)v;
}

// pattern of run-time format fs -> posit<F>, one rounding
template <class F>
__device__ __forceinline__ uint32_t convert_in(uint32_t p, const FmtRT& fs) {
    p &= fs.mask();
    if (p == 0) return 0u;
    if (p == fs.nar()) return F::NAR;
    return encode<F>(decode_rt(p, fs));
}

// posit<F> value times 2^pow2 divided by an integer and rounded once to run-time format fd.  F has at
// most 16 bits: the significand has at most 14 bits, so one 64-bit division gives a quotient of at
// least 18 + 31 significant bits and a remainder that decides "sticky".
template <class F>
__device__ __forceinline__ uint32_t scaled_out(uint32_t g, int pow2, uint32_t divisor, const FmtRT& fd) {
    if (g == F::NAR) return fd.nar();
    if (g == 0) return 0u;
    const Real32 r = decode_fields32<F>(g);
    const uint64_t sig = (1u << 14) | (r.frac >> 18);       // 1.fraction with 14 fraction bits
    const uint64_t num = sig << 49;                           // < 2^64
    const uint64_t q = num / divisor, rem = num - q * divisor;  // divisor < 2^32: q >= 2^31
    const int top = 63 - clz64(q);
    Real o;
    o.neg = r.neg;
    o.scale = r.scale + pow2 + (top - 63);  // num = sig * 2^49 = value * 2^(63 - scale)
    o.frac = top == 0 ? 0 : (q << (64 - top));
    o.sticky = rem != 0;
    return encode_rt(o, fd);
}

template <class F>
__device__ __forceinline__ int32_t ordered(uint32_t p) { return (int32_t)(p << (32 - F::N)) >> (32 - F::N); }

template <class F>
__device__ __forceinline__ uint32_t negate(uint32_t p) { return (0u - p) & F::MASK; }

template <class F>
__global__ __launch_bounds__(256) void unary_kernel(int fn, const void* __restrict__ x, void* __restrict__ y, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    constexpr int bytes = F::N <= 8 ? 1 : 2;
    store_pattern(y, i, bytes, posit_unary<F>(fn, load_pattern(x, i, bytes)));
}

// gradient through an activation from its forward output, in rounded operations of posit<FD>
template <class FD>
__global__ __launch_bounds__(256) void unary_bwd_kernel(int fn, FmtRT fy, const void* __restrict__ yf, const void* __restrict__ dy,
                                                        void* __restrict__ dx, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    constexpr int bytes = FD::N <= 8 ? 1 : 2;
    const uint32_t one = 1u << (FD::N - 2);
    const uint32_t yc = convert_in<FD>(load_pattern(yf, i, fy.bytes()), fy);
    const uint32_t d = load_pattern(dy, i, bytes) & FD::MASK;
    uint32_t t;
    if (fn == UNARY_SIGMOID) t = posit_mul<FD>(yc, posit_add<FD>(one, yc == FD::NAR ? FD::NAR : negate<FD>(yc)));
    else {
        const uint32_t sq = posit_mul<FD>(yc, yc);
        t = posit_add<FD>(one, sq == FD::NAR ? FD::NAR : negate<FD>(sq));
    }
    store_pattern(dx, i, bytes, posit_mul<FD>(d, t));
}

// merge the 256 private quires of a workgroup (exact), result in thread 0's q
template <int L>
__device__ __forceinline__ void block_merge(uint32_t (&q)[L], uint32_t (*part)[L], int t) {
    for (int half = 128; half >= 1; half >>= 1) {
        if (t >= half && t < 2 * half) {
#pragma unroll
            for (int l = 0; l < L; ++l) part[t - half][l] = q[l];
        }
        __syncthreads();
        if (t < half) {
            uint32_t o[L];
#pragma unroll
            for (int l = 0; l < L; ++l) o[l] = part[t][l];
            quire_merge<L>(q, o);
        }
        __syncthreads();
    }
}

template <class FL>
__global__ __launch_bounds__(256) void cross_entropy_kernel(FmtRT fz, FmtRT fg, int B, int C, const void* __restrict__ logits,
                                                            const int32_t* __restrict__ labels, void* __restrict__ loss,
                                                            void* __restrict__ dlogits) {
    typedef Arith<FL> AR;
    constexpr int L = AR::L;
    __shared__ uint32_t part[128][L];
    __shared__ uint32_t bad_s;
    const int t = threadIdx.x;
    if (t == 0) bad_s = 0;
    uint32_t ql[L];
#pragma unroll
    for (int l = 0; l < L; ++l) ql[l] = 0;
    bool bad = false;
    const uint32_t one = 1u << (FL::N - 2);
    const int zb = fz.bytes(), gb = fg.bytes();
    for (int b = t; b < B; b += 256) {
        const int64_t base = (int64_t)b * C;
        const int label = labels[b];
        bool rownar = label < 0 || label >= C;
        uint32_t m = 0;
        for (int j = 0; j < C; ++j) {  // the largest logit
            const uint32_t z = convert_in<FL>(load_pattern(logits, base + j, zb), fz);
            if (z == FL::NAR) rownar = true;
            else if (j == 0 || ordered<FL>(z) > ordered<FL>(m)) m = z;
        }
        if (rownar) {
            bad = true;
            if (dlogits)
                for (int j = 0; j < C; ++j) store_pattern(dlogits, base + j, gb, fg.nar());
            continue;
        }
        const uint32_t negm = negate<FL>(m);
        uint32_t qs[L];
#pragma unroll
        for (int l = 0; l < L; ++l) qs[l] = 0;
        for (int j = 0; j < C; ++j) {  // S = round(sum_j exp(z_j - m)), the sum exact
            const uint32_t z = convert_in<FL>(load_pattern(logits, base + j, zb), fz);
            const uint32_t e = posit_unary<FL>(UNARY_EXP, posit_add<FL>(z, negm));
            AR::add_value(qs, AR::stage(e));
        }
        const uint32_t S = quire_round<FL, FL, L>(qs);
        uint32_t tl = 0;
        for (int j = 0; j < C; ++j) {  // p_j = e_j / S, g_j = p_j - [j == label]
            const uint32_t z = convert_in<FL>(load_pattern(logits, base + j, zb), fz);
            const uint32_t tj = posit_add<FL>(z, negm);
            if (j == label) tl = tj;
            if (dlogits) {
                const uint32_t p = posit_div<FL>(posit_unary<FL>(UNARY_EXP, tj), S);
                const uint32_t g = posit_add<FL>(p, j == label ? negate<FL>(one) : 0u);
                store_pattern(dlogits, base + j, gb, scaled_out<FL>(g, 0, (uint32_t)B, fg));
            }
        }
        const uint32_t row_loss = posit_add<FL>(posit_unary<FL>(UNARY_LOG, S), negate<FL>(tl));
        AR::add_value(ql, AR::stage(row_loss));
    }
    __syncthreads();
    if (bad) bad_s = 1;  // every writer stores the same value
    block_merge<L>(ql, part, t);
    if (t == 0 && loss) {
        uint32_t res = FL::NAR;
        if (!bad_s) {
            Real r;
            res = quire_read<FL, L>(ql, r) ? encode<FL>(real_div_int(r, (uint32_t)B)) : 0u;
        }
        store_pattern(loss, 0, FL::N <= 8 ? 1 : 2, res);
    }
}

// The same computation with one lane per (row, class): CP = the power of two >= classes lanes serve a
// row, 256 / CP rows are in flight per pass, the first lane of a row does the row's serial parts
// (maximum, exact sum of the exponentials, row loss).  For classes <= 256; same results as
// cross_entropy_kernel, which serves wider rows.
template <class FL>
__global__ __launch_bounds__(256) void cross_entropy_lanes_kernel(FmtRT fz, FmtRT fg, int B, int C, int CP, const void* __restrict__ logits,
                                                                  const int32_t* __restrict__ labels, void* __restrict__ loss,
                                                                  void* __restrict__ dlogits) {
    typedef Arith<FL> AR;
    constexpr int L = AR::L;
    __shared__ uint32_t part[128][L];
    __shared__ uint32_t bad_s;
    __shared__ uint32_t zs[256], ts[256], es[256];  // per lane: converted logit, logit - max, its exponential
    __shared__ uint32_t Ms[256], Ss[256], rowbad[256];  // per row in flight: maximum, rounded sum, NaR / bad label
    const int t = threadIdx.x;
    if (t == 0) bad_s = 0;
    uint32_t ql[L];
#pragma unroll
    for (int l = 0; l < L; ++l) ql[l] = 0;
    bool bad = false;
    const uint32_t one = 1u << (FL::N - 2);
    const int zb = fz.bytes(), gb = fg.bytes();
    const int R = 256 / CP, rl = t / CP, j = t - rl * CP;
    const int first = rl * CP;
    // several workgroups share the rows when only the gradient is wanted (the host passes loss == null then)
    for (int b0 = blockIdx.x * R; b0 < B; b0 += gridDim.x * R) {
        const int b = b0 + rl;
        const bool row_live = b < B, active = row_live && j < C;
        const int64_t at = (int64_t)b * C + j;
        const uint32_t z = active ? convert_in<FL>(load_pattern(logits, at, zb), fz) : 0u;
        const int label = row_live ? labels[b] : 0;
        zs[t] = z;
        __syncthreads();
        if (j == 0 && row_live) {
            bool rn = label < 0 || label >= C;
            uint32_t m = 0;
            for (int jj = 0; jj < C; ++jj) {
                const uint32_t zz = zs[first + jj];
                if (zz == FL::NAR) rn = true;
                else if (jj == 0 || ordered<FL>(zz) > ordered<FL>(m)) m = zz;
            }
            rowbad[rl] = rn;
            Ms[rl] = m;
        }
        __syncthreads();
        const bool rn = row_live && rowbad[rl] != 0;
        uint32_t e = 0;
        if (active && !rn) {
            const uint32_t tj = posit_add<FL>(z, negate<FL>(Ms[rl]));
            e = posit_unary<FL>(UNARY_EXP, tj);
            ts[t] = tj;
            es[t] = e;
        }
        __syncthreads();
        if (j == 0 && row_live) {
            if (rn) {
                bad = true;
            } else {
                uint32_t qs[L];
#pragma unroll
                for (int l = 0; l < L; ++l) qs[l] = 0;
                for (int jj = 0; jj < C; ++jj) AR::add_value(qs, AR::stage(es[first + jj]));
                const uint32_t S = quire_round<FL, FL, L>(qs);
                Ss[rl] = S;
                const uint32_t row_loss = posit_add<FL>(posit_unary<FL>(UNARY_LOG, S), negate<FL>(ts[first + label]));
                AR::add_value(ql, AR::stage(row_loss));
            }
        }
        __syncthreads();
        if (active && dlogits) {
            uint32_t out = fg.nar();
            if (!rn) {
                const uint32_t p = posit_div<FL>(e, Ss[rl]);
                const uint32_t g = posit_add<FL>(p, j == label ? negate<FL>(one) : 0u);
                out = scaled_out<FL>(g, 0, (uint32_t)B, fg);
            }
            store_pattern(dlogits, at, gb, out);
        }
    }
    __syncthreads();
    if (bad) bad_s = 1;  // every writer stores the same value
    block_merge<L>(ql, part, t);
    if (t == 0 && loss) {
        uint32_t res = FL::NAR;
        if (!bad_s) {
            Real r;
            res = quire_read<FL, L>(ql, r) ? encode<FL>(real_div_int(r, (uint32_t)B)) : 0u;
        }
        store_pattern(loss, 0, FL::N <= 8 ? 1 : 2, res);
    }
}

template <class FL>
__global__ __launch_bounds__(256) void mse_kernel(FmtRT fp, FmtRT fg, int64_t n, const void* __restrict__ pred,
                                                  const void* __restrict__ target, void* __restrict__ loss, void* __restrict__ dpred) {
    typedef Arith<FL> AR;
    constexpr int L = AR::L;
    __shared__ uint32_t part[128][L];
    __shared__ uint32_t bad_s;
    const int t = threadIdx.x;
    if (t == 0) bad_s = 0;
    uint32_t q[L];
#pragma unroll
    for (int l = 0; l < L; ++l) q[l] = 0;
    bool bad = false;
    const int pb = fp.bytes(), gb = fg.bytes();
    for (int64_t i = t; i < n; i += 256) {
        const uint32_t a = convert_in<FL>(load_pattern(pred, i, pb), fp), b = convert_in<FL>(load_pattern(target, i, pb), fp);
        const uint32_t d = (a == FL::NAR || b == FL::NAR) ? FL::NAR : posit_add<FL>(a, negate<FL>(b));
        if (dpred) store_pattern(dpred, i, gb, scaled_out<FL>(d, 1, (uint32_t)n, fg));  // 2 d / n
        if (d == FL::NAR) bad = true;
        else AR::mac(q, AR::stage(d), AR::stage(d));
    }
    __syncthreads();
    if (bad) bad_s = 1;
    block_merge<L>(q, part, t);
    if (t == 0 && loss) {
        uint32_t res = FL::NAR;
        if (!bad_s) {
            Real r;
            res = quire_read<FL, L>(q, r) ? encode<FL>(real_div_int(r, (uint32_t)n)) : 0u;
        }
        store_pattern(loss, 0, FL::N <= 8 ? 1 : 2, res);
    }
}

inline bool is_small_posit(int f) { return is_posit(f) && f != PNN_POSIT32_2; }

// CALL sees `F`, a format of at most 16 bits
#define PNN_DISPATCH_SMALL(code, CALL)                      \
    switch (code) {                                          \
        case PNN_POSIT8_0: { typedef P8 F; CALL; } break;     \
        case PNN_POSIT16_1: { typedef P16 F; CALL; } break;   \
        case PNN_POSIT8_1: { typedef P8_1 F; CALL; } break;   \
        case PNN_POSIT8_2: { typedef P8_2 F; CALL; } break;   \
        case PNN_POSIT10_1: { typedef P10_1 F; CALL; } break; \
        case PNN_POSIT10_2: { typedef P10_2 F; CALL; } break; \
        case PNN_POSIT12_1: { typedef P12_1 F; CALL; } break; \
        default: { typedef P12_2 F; CALL; } break;            \
    }

}  // namespace pnn

using namespace pnn;

extern "C" int posit_unary(void* stream, int fn, int fmt, int64_t n, const void* x, void* y) {
    if (fn < UNARY_SIGMOID || fn > UNARY_LOG || !is_posit(fmt) || n < 0) return PNN_EINVAL;
    if (!is_small_posit(fmt)) return PNN_EUNSUPPORTED;
    if (n == 0) return PNN_OK;
    if (!x || !y) return PNN_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    discard_stale_hip_error();
    PNN_DISPATCH_SMALL(fmt, hipLaunchKernelGGL(unary_kernel<F>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, fn, x, y, n))
    return hip_status(hipGetLastError());
}

extern "C" int posit_unary_bwd(void* stream, int fn, int fmt_y, int fmt_d, int64_t n, const void* y_fwd, const void* dy, void* dx) {
    if ((fn != UNARY_SIGMOID && fn != UNARY_TANH) || !is_posit(fmt_y) || !is_posit(fmt_d) || n < 0) return PNN_EINVAL;
    if (!is_small_posit(fmt_y) || !is_small_posit(fmt_d)) return PNN_EUNSUPPORTED;
    if (n == 0) return PNN_OK;
    if (!y_fwd || !dy || !dx) return PNN_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    discard_stale_hip_error();
    const FmtRT fy = fmt_of_code(fmt_y);
    PNN_DISPATCH_SMALL(fmt_d, hipLaunchKernelGGL(unary_bwd_kernel<F>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, fn, fy, y_fwd,
                                                 dy, dx, n))
    return hip_status(hipGetLastError());
}

extern "C" int posit_cross_entropy(void* stream, int f_logits, int f_loss, int f_grad, int64_t batch, int64_t classes,
                                   const void* logits, const int32_t* labels, void* loss, void* dlogits) {
    if (!is_posit(f_logits) || !is_posit(f_loss) || !is_posit(f_grad) || batch < 0 || classes < 0) return PNN_EINVAL;
    if (!is_small_posit(f_logits) || !is_small_posit(f_loss) || !is_small_posit(f_grad)) return PNN_EUNSUPPORTED;
    if (batch >= ((int64_t)1 << 31) || classes >= ((int64_t)1 << 31)) return PNN_EUNSUPPORTED;
    if (batch == 0 || classes == 0) return loss ? PNN_EINVAL : PNN_OK;  // a mean over nothing has no value
    if (!logits || !labels || (!loss && !dlogits)) return PNN_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    discard_stale_hip_error();
    const FmtRT fz = fmt_of_code(f_logits), fg = fmt_of_code(f_grad);
    if (classes <= 256) {
        int cp = 1;
        while (cp < classes) cp *= 2;
        // the mean over the batch is reduced inside one workgroup; without it the rows are independent
        int64_t blocks = 1;
        if (!loss) {
            blocks = (batch * cp + 255) / 256;
            if (blocks > 256) blocks = 256;
        }
        PNN_DISPATCH_SMALL(f_loss, hipLaunchKernelGGL(cross_entropy_lanes_kernel<F>, dim3((unsigned)blocks), dim3(256), 0, st, fz, fg, (int)batch,
                                                      (int)classes, cp, logits, labels, loss, dlogits))
    } else {
        PNN_DISPATCH_SMALL(f_loss, hipLaunchKernelGGL(cross_entropy_kernel<F>, dim3(1), dim3(256), 0, st, fz, fg, (int)batch, (int)classes,
                                                      logits, labels, loss, dlogits))
    }
    return hip_status(hipGetLastError());
}

extern "C" int posit_mse(void* stream, int f_pred, int f_loss, int f_grad, int64_t n, const void* pred, const void* target, void* loss,
                         void* dpred) {
    if (!is_posit(f_pred) || !is_posit(f_loss) || !is_posit(f_grad) || n < 0) return PNN_EINVAL;
    if (!is_small_posit(f_pred) || !is_small_posit(f_loss) || !is_small_posit(f_grad)) return PNN_EUNSUPPORTED;
    if (n >= ((int64_t)1 << 31)) return PNN_EUNSUPPORTED;
    if (n == 0) return !loss ? PNN_OK : PNN_EINVAL;
    if (!pred || !target || (!loss && !dpred)) return PNN_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    discard_stale_hip_error();
    const FmtRT fp = fmt_of_code(f_pred), fg = fmt_of_code(f_grad);
    PNN_DISPATCH_SMALL(f_loss, hipLaunchKernelGGL(mse_kernel<F>, dim3(1), dim3(256), 0, st, fp, fg, n, pred, target, loss, dpred))
    return hip_status(hipGetLastError());
}
