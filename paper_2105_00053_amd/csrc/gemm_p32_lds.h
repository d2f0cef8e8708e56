// posit<32,2> matrix product with the 512-bit quire of Table 1 (paper Sec. 2, Sec. 3.3) kept in LDS as lazily
// carried 64-bit limbs.
//
// In registers the 512-bit accumulate costs 72 vector instructions per product: the limb a product lands on depends
// on the data, registers cannot be indexed, so the three words of the shifted product reach their limbs through
// rounds of selects, and a 16-limb carry chain follows.  LDS can be indexed.  Here every thread owns ONE output and
// keeps its quire in LDS as 18 signed 64-bit words q[l], l = 0 .. 17, the sum being  sum_l q[l] * 2^(32 l)  (limbs 16
// and 17 only catch what lies beyond bit 511 and is dropped: the quire wraps modulo 2^512).  A product P * 2^s, P a
// signed integer of at most 57 bits, s = 32 idx + off, is the signed integer V = P << off of at most 89 bits:
//     V = w0 + w1 * 2^32 + w2 * 2^64,  w0, w1 its low words taken as unsigned, w2 the rest taken as signed,
// and three LDS additions without return value, q[idx] += w0, q[idx + 1] += w1, q[idx + 2] += w2 (sign-extended to 64
// bits), add it exactly: no carry moves between limbs until the end, and no limb overflows (|q[l]| < K * 2^32 with
// K < 2^31).  The carries are propagated once, when the thread reads its limbs back after the loop.  About 14 vector
// instructions and 3 LDS additions per product; the LDS additions (7 cycles each per wave on a compute unit) set the
// rate.  16 x 16 outputs per workgroup of 256 threads, 36 KB of quires + 4 KB of staged operands.
#pragma once

#include "quire_gemm.h"

namespace pnn {

constexpr int P32L_T = 16;        // outputs per tile edge
constexpr int P32L_KT = 16;       // reduction steps per staged slice
constexpr int P32L_LIMBS = 18;    // 16 limbs of the quire + 2 that catch the words beyond bit 511

template <class OpA, class OpB>
__global__ __launch_bounds__(256) void p32_lds_gemm_kernel(OpA opa, OpB opb, int64_t M, int64_t N, int64_t K, const uint32_t* __restrict__ bias,
                                                           void* __restrict__ C, int64_t ldc, int fout, int tiles_n) {
    typedef Arith<P32> AR;
    typedef AR::Elem Elem;
    constexpr int T = P32L_T, KT = P32L_KT;
    __shared__ unsigned long long q[P32L_LIMBS][256];  // [limb][thread]: a wave's addresses fall on distinct banks whatever idx is
    __shared__ Elem As[2][KT][T];
    __shared__ Elem Bs[2][KT][T];
    __shared__ uint32_t rowNaR[T];
    __shared__ uint32_t colNaR[T];

    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int64_t tile = blockIdx.x;
    const int64_t m0 = (tile / tiles_n) * T, n0 = (tile % tiles_n) * T;

#pragma unroll
    for (int l = 0; l < P32L_LIMBS; ++l) q[l][tid] = 0;
    if (tid < T) rowNaR[tid] = 0;
    else if (tid < 2 * T) colNaR[tid - T] = 0;

    // one element of each operand per thread and slice; consecutive threads walk the dimension that is contiguous in memory
    const int ka = OpA::KFAST ? (tid % KT) : (tid / T), ra = OpA::KFAST ? (tid / KT) : (tid % T);
    const int kb = OpB::KFAST ? (tid % KT) : (tid / T), rb = OpB::KFAST ? (tid / KT) : (tid % T);
    uint32_t pa = 0, pb = 0;
    auto fetch = [&](int64_t k0) {
        pa = (k0 + ka < K) ? opa(m0 + ra, k0 + ka) : 0u;
        pb = (k0 + kb < K) ? opb(n0 + rb, k0 + kb) : 0u;
    };
    auto stage = [&](int buf) {
        if (pa == P32::NAR) rowNaR[ra] = 1;
        if (pb == P32::NAR) colNaR[rb] = 1;
        As[buf][ka][ra] = AR::stage(pa);
        Bs[buf][kb][rb] = AR::stage(pb);
    };

    __syncthreads();  // flags and quires initialised
    if (K > 0) {
        fetch(0);
        stage(0);
    }
    __syncthreads();
    int cur = 0;
    for (int64_t k0 = 0; k0 < K; k0 += KT, cur ^= 1) {
        const bool more = k0 + KT < K;
        if (more) fetch(k0 + KT);
#pragma unroll 4
        for (int kk = 0; kk < KT; ++kk) {
            const Elem a = As[cur][kk][ty], b = Bs[cur][kk][tx];
            const int64_t P = (int64_t)(int32_t)a.x * (int64_t)(int32_t)b.x;  // zero when either operand is zero (or NaR)
            const int s = (int)(a.y + b.y);
            const int idx = s >> 5, off = s & 31;
            const uint64_t lo = (uint64_t)P << off;
            const int64_t w2 = (P >> 32) >> (32 - off);  // bits 64 and up of the signed shift, sign included
            unsigned long long* at = &q[idx][tid];
            __hip_atomic_fetch_add(at, (unsigned long long)(uint32_t)lo, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            __hip_atomic_fetch_add(at + 256, (unsigned long long)(uint32_t)(lo >> 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            __hip_atomic_fetch_add(at + 512, (unsigned long long)w2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
        if (more) stage(cur ^ 1);  // the other buffer was last read one barrier ago
        __syncthreads();
    }

    const int64_t m = m0 + ty, n = n0 + tx;
    if (m >= M || n >= N) return;
    // carries, once: limb l of the two's complement quire is the low word of q[l] + carry, the carry its (signed) rest
    uint32_t limbs[16];
    int64_t carry = 0;
#pragma unroll
    for (int l = 0; l < 16; ++l) {
        const int64_t v = (int64_t)q[l][tid] + carry;  // |q[l]| < 2^63 / 2 and |carry| < 2^32: no overflow
        limbs[l] = (uint32_t)v;
        carry = v >> 32;
    }
    bool nar = (rowNaR[ty] | colNaR[tx]) != 0;
    if (bias) {
        const uint32_t bp = bias[n];
        if (bp == P32::NAR) nar = true;
        else AR::add_value(limbs, AR::stage(bp));
    }
    round_store<QuireAccum<P32>, 16>(limbs, nar, fout, C, m * ldc + n);
}

// Shapes this kernel takes: enough 16 x 16 tiles to fill the chip (otherwise the reduction would have to be cut
// across workgroups, which the register kernel does through the workspace).
inline bool p32_lds_fits(int64_t M, int64_t N, int64_t K) {
    const int64_t tiles = ((M + P32L_T - 1) / P32L_T) * ((N + P32L_T - 1) / P32L_T);
    return tiles >= 768 && K >= 1 && M < ((int64_t)1 << 31) && N < ((int64_t)1 << 31) && K < ((int64_t)1 << 31);
}

template <class OpA, class OpB>
hipError_t launch_p32_lds_gemm(hipStream_t st, const OpA& a, const OpB& b, int64_t M, int64_t N, int64_t K, const void* bias, void* C, int64_t ldc,
                               int fout) {
    const int64_t tiles_m = (M + P32L_T - 1) / P32L_T, tiles_n = (N + P32L_T - 1) / P32L_T;
    hipLaunchKernelGGL((p32_lds_gemm_kernel<OpA, OpB>), dim3((unsigned)(tiles_m * tiles_n)), dim3(256), 0, st, a, b, M, N, K,
                       (const uint32_t*)bias, C, ldc, fout, (int)tiles_n);
    return hipGetLastError();
}

}  // namespace pnn
