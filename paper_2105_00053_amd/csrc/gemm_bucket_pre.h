// posit_gemm for the formats whose exact sum is carried in fp64 buckets (posit<16,1> and the 10- / 12-bit
// formats; paper Sec. 2 quire, Sec. 3.3 matrix product): operands decoded once, ahead of the product.
//
// The tile kernel of quire_gemm.h decodes every operand pattern each time a workgroup stages it: about 35
// lane-operations per element, i.e. 35 (1/BM + 1/BN) per multiply-accumulate on top of the 9 the three-bucket
// accumulate of posit<16,1> costs.  Here a first pass writes both operands as doubles (value * 2^MAXS, an
// integer; NaR as a NaN) in the layout the product wants -- reduction index major, output index contiguous,
// padded to whole tiles with zeros -- and the product kernel only copies 16-byte runs of doubles into LDS and
// multiplies: no decode, no bounds tests, no index arithmetic per element in the main loop.  The doubles are
// read from the workspace (8 bytes per operand element); with 64 x 64 or 32 x 32 tiles of outputs and the
// reduction cut over gridDim.z when the tiles alone would not fill the chip (partial quires through the
// workspace, merged and rounded once by split_merge_kernel).
//
// The buckets of an output are emptied into quire limbs after the loop; where a workgroup's part of the reduction
// exceeds 2^G products (G = the guard bits of BucketArith<F>) the 32 x 32 kernel is instantiated with the limbs
// held in registers all along and empties the buckets into them every 2^G products (FLUSH).
#pragma once

#include "quire_gemm.h"

namespace pnn {

constexpr int BP_KT = 16;        // reduction steps per staged slice
constexpr int BP_THREADS = 256;  // 16 x 16 threads, TM x TN outputs each
constexpr int BP_PRE_TILE = 64;  // the decode pass works on 64 x 64 element tiles

template <class F>
constexpr bool bucket_pre_format() {
    return BucketArith<F>::B > 0 && F::N != 8 && F::N != 16;  // the 8-bit formats and posit<16,1> have kernels of their own
}

// value * 2^MAXS of a pattern as a double; zero for the zero pattern, a NaN for NaR
template <class F>
PNN_HD double bucket_operand(uint32_t p) {
    if (p == F::NAR) return __builtin_bit_cast(double, (uint64_t)0x7FF8000000000000ull);
    return BucketArith<F>::stage(p);
}

// dst[k][r] (pitch Rp, k < Kp) = operand element (r, k), zero outside rows x K.  KFAST: src[r * ld + k], the tile is
// transposed through LDS so that both the reads (along k) and the writes (along r) are contiguous; otherwise
// src[k * ld + r] and the copy is direct.
template <class F, bool KFAST>
__global__ __launch_bounds__(256) void bucket_predecode_kernel(const typename Storage<F::N>::T* __restrict__ src, int64_t ld, int64_t rows,
                                                               int64_t K, double* __restrict__ dst, int64_t Rp, int64_t Kp) {
    constexpr int PT = BP_PRE_TILE;
    __shared__ double tile[KFAST ? PT : 1][KFAST ? PT + 1 : 1];
    const int64_t r0 = (int64_t)blockIdx.x * PT, k0 = (int64_t)blockIdx.y * PT;
    const int t = threadIdx.x;
    if constexpr (KFAST) {
#pragma unroll 4
        for (int i = 0; i < PT * PT / 256; ++i) {
            const int e = t + 256 * i;
            const int kk = e % PT, rr = e / PT;
            const int64_t r = r0 + rr, k = k0 + kk;
            tile[kk][rr] = (r < rows && k < K) ? bucket_operand<F>(src[r * ld + k]) : 0.0;
        }
        __syncthreads();
#pragma unroll 4
        for (int i = 0; i < PT * PT / 256; ++i) {
            const int e = t + 256 * i;
            const int rr = e % PT, kk = e / PT;
            if (k0 + kk < Kp) dst[(k0 + kk) * Rp + r0 + rr] = tile[kk][rr];
        }
    } else {
#pragma unroll 4
        for (int i = 0; i < PT * PT / 256; ++i) {
            const int e = t + 256 * i;
            const int rr = e % PT, kk = e / PT;
            const int64_t r = r0 + rr, k = k0 + kk;
            if (k < Kp) dst[k * Rp + r] = (r < rows && k < K) ? bucket_operand<F>(src[k * ld + r]) : 0.0;
        }
    }
}

// C tile (16 TM x 16 TN) = sum over k in [z kq, (z + 1) kq) of Ap[k][m] * Bp[k][n], exactly, in the buckets of
// BucketArith<F>.  Ap / Bp: decoded operands, pitches Mp / Np (multiples of the tile), kq a multiple of BP_KT,
// every (k, m) and (k, n) the grid touches is inside the padded arrays.
template <class F, int TM, int TN, bool FLUSH>
__global__ __launch_bounds__(BP_THREADS) void bucket_pre_gemm_kernel(const double* __restrict__ Ap, const double* __restrict__ Bp, int64_t Mp,
                                                                     int64_t Np, int64_t kq,
                                                                     const typename Storage<F::N>::T* __restrict__ bias,
                                                                     void* __restrict__ C, int64_t ldc, int fout, int64_t M, int64_t N,
                                                                     SplitWs ws, int tiles_n) {
    typedef BucketAccum<F> AR;
    typedef BucketArith<F> BA;
    constexpr int L = AR::L, NB = BA::NB, KT = BP_KT;
    constexpr int BM = 16 * TM, BN = 16 * TN;
    constexpr int CA = KT * BM / 2 / BP_THREADS, CB = KT * BN / 2 / BP_THREADS;  // 16-byte runs per thread and slice
    static_assert(TM % 2 == 0 && TN % 2 == 0 && CA >= 1 && CB >= 1, "whole 16-byte runs per thread");

    __shared__ __align__(16) double As[2][KT][BM];
    __shared__ __align__(16) double Bs[2][KT][BN];
    __shared__ uint32_t rowNaR[BM];
    __shared__ uint32_t colNaR[BN];

    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int64_t tile = blockIdx.x;
    const int64_t m0 = (tile / tiles_n) * BM, n0 = (tile % tiles_n) * BN;
    const int64_t kbeg = (int64_t)blockIdx.z * kq, kend = kbeg + kq;

    for (int i = tid; i < BM; i += BP_THREADS) rowNaR[i] = 0;
    for (int i = tid; i < BN; i += BP_THREADS) colNaR[i] = 0;

    double bk[TM][TN][NB];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) BA::clear(bk[i][j]);

    uint32_t acc[FLUSH ? TM : 1][FLUSH ? TN : 1][L];  // FLUSH: the limbs the buckets are emptied into along the way
    if constexpr (FLUSH) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int l = 0; l < L; ++l) acc[i][j][l] = 0;
    }
    int since_flush = 0;  // products in the buckets

    double2 ra[CA], rb[CB];
    auto fetch = [&](int64_t k0) {
#pragma unroll
        for (int i = 0; i < CA; ++i) {
            const int c = tid + BP_THREADS * i;
            const int kk = c / (BM / 2), r2 = c % (BM / 2);
            ra[i] = *reinterpret_cast<const double2*>(Ap + (k0 + kk) * Mp + m0 + 2 * r2);
        }
#pragma unroll
        for (int i = 0; i < CB; ++i) {
            const int c = tid + BP_THREADS * i;
            const int kk = c / (BN / 2), r2 = c % (BN / 2);
            rb[i] = *reinterpret_cast<const double2*>(Bp + (k0 + kk) * Np + n0 + 2 * r2);
        }
    };
    // copy the fetched runs into LDS; a NaN is a NaR operand: it raises the flag of its row (column) of outputs
    auto stage = [&](int buf) {
#pragma unroll
        for (int i = 0; i < CA; ++i) {
            const int c = tid + BP_THREADS * i;
            const int kk = c / (BM / 2), r2 = c % (BM / 2);
            if (ra[i].x != ra[i].x) rowNaR[2 * r2] = 1;
            if (ra[i].y != ra[i].y) rowNaR[2 * r2 + 1] = 1;
            *reinterpret_cast<double2*>(&As[buf][kk][2 * r2]) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < CB; ++i) {
            const int c = tid + BP_THREADS * i;
            const int kk = c / (BN / 2), r2 = c % (BN / 2);
            if (rb[i].x != rb[i].x) colNaR[2 * r2] = 1;
            if (rb[i].y != rb[i].y) colNaR[2 * r2 + 1] = 1;
            *reinterpret_cast<double2*>(&Bs[buf][kk][2 * r2]) = rb[i];
        }
    };

    __syncthreads();  // flags initialised before any stage() raises one
    fetch(kbeg);
    stage(0);
    __syncthreads();
    int cur = 0;
    for (int64_t k0 = kbeg; k0 < kend; k0 += KT, cur ^= 1) {
        const bool more = k0 + KT < kend;
        if (more) fetch(k0 + KT);
#pragma unroll 4
        for (int kk = 0; kk < KT; ++kk) {
            double a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; i += 2) {
                const double2 v = *reinterpret_cast<const double2*>(&As[cur][kk][ty * TM + i]);
                a[i] = v.x;
                a[i + 1] = v.y;
            }
#pragma unroll
            for (int j = 0; j < TN; j += 2) {
                const double2 v = *reinterpret_cast<const double2*>(&Bs[cur][kk][tx * TN + j]);
                b[j] = v.x;
                b[j + 1] = v.y;
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) BA::mac(bk[i][j], a[i], b[j]);
        }
        if constexpr (FLUSH) {
            since_flush += KT;
            if (since_flush + KT > (1 << BA::G)) {  // the next slice would exceed the guard bits
                since_flush = 0;
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) BA::template flush<L>(acc[i][j], bk[i][j]);
            }
        }
        if (more) stage(cur ^ 1);  // the other buffer was last read one barrier ago
        __syncthreads();
    }

    const int64_t z = blockIdx.z;
    uint32_t* lim = gridDim.z > 1 ? ws.limbs + z * M * N * L : nullptr;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int64_t m = m0 + ty * TM + i;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int64_t n = n0 + tx * TN + j;
            if (n >= N) continue;
            bool nar = (rowNaR[ty * TM + i] | colNaR[tx * TN + j]) != 0;
            uint32_t q[L];
#pragma unroll
            for (int l = 0; l < L; ++l) q[l] = FLUSH ? acc[FLUSH ? i : 0][FLUSH ? j : 0][l] : 0u;
            if (!nar) BA::template flush<L>(q, bk[i][j]);  // a NaR output's buckets hold NaNs: nothing to read off
            if (lim) {
#pragma unroll
                for (int l = 0; l < L; ++l) lim[(m * N + n) * L + l] = q[l];
            } else {
                if (bias) {
                    const uint32_t bp = bias[n];
                    if (bp == F::NAR) nar = true;
                    else AR::add_bias(q, bp);
                }
                round_store<AR, L>(q, nar, fout, C, m * ldc + n);
            }
        }
    }
    if (lim) {  // flags of this slice of the reduction, as quire_gemm_kernel stores them
        if (n0 == 0)
            for (int i = tid; i < BM; i += BP_THREADS)
                if (m0 + i < M) ws.rowflag[z * M + m0 + i] = rowNaR[i];
        if (m0 == 0)
            for (int i = tid; i < BN; i += BP_THREADS)
                if (n0 + i < N) ws.colflag[z * N + n0 + i] = colNaR[i];
    }
}

// ---- host side ----

struct BucketPrePlan {
    GemmPlan gemm;       // splits, k per split (multiple of BP_KT), workspace bytes in all
    int tile;            // 32 or 64: outputs per tile edge
    bool flush;          // a workgroup adds more products per output than the buckets' guard bits allow at once
    int64_t Mp, Np, Kp;  // padded extents of the decoded operands
    size_t b_off, split_off;  // byte offsets inside the workspace (decoded A at 0)
};

template <class F>
bool bucket_pre_fits(int64_t M, int64_t N, int64_t K) {
    if constexpr (!bucket_pre_format<F>()) return false;
    return M >= 96 && N >= 96 && K >= 64 && M < ((int64_t)1 << 31) && N < ((int64_t)1 << 31) && K < ((int64_t)1 << 31);
}

template <class F>
BucketPrePlan bucket_pre_plan(int64_t M, int64_t N, int64_t K) {
    BucketPrePlan p;
    const int64_t tiles64 = ((M + 63) / 64) * ((N + 63) / 64);
    p.tile = (tiles64 >= 640 && BucketArith<F>::NB <= 3) ? 64 : 32;  // four buckets per output: 16 outputs per thread do not fit the registers
    const int64_t tiles = ((M + p.tile - 1) / p.tile) * ((N + p.tile - 1) / p.tile);
    int64_t splits = 1;
    if (tiles < 768 && K >= 512) {
        splits = (1024 + tiles - 1) / tiles;
        if (splits > K / 256) splits = K / 256;
        if (splits > 64) splits = 64;
    }
    if (splits < 1) splits = 1;
    int64_t kq = (K + splits - 1) / splits;
    kq = (kq + BP_KT - 1) / BP_KT * BP_KT;
    splits = (K + kq - 1) / kq;
    p.flush = kq > ((int64_t)1 << BucketArith<F>::G);
    if (p.flush) p.tile = 32;  // 4 outputs per thread leave room for their limbs
    p.gemm.splits = (int)splits;
    p.gemm.k_per_split = kq;
    p.Kp = splits * kq;
    p.Mp = (M + 63) / 64 * 64;
    p.Np = (N + 63) / 64 * 64;
    p.b_off = (size_t)p.Kp * p.Mp * sizeof(double);
    p.split_off = p.b_off + (size_t)p.Kp * p.Np * sizeof(double);
    p.gemm.ws_bytes = p.split_off + (splits > 1 ? (size_t)splits * ((size_t)M * N * Arith<F>::L + M + N) * sizeof(uint32_t) : 0);
    return p;
}

template <class F>
hipError_t launch_bucket_pre_gemm(hipStream_t st, int transA, int transB, const void* A, int64_t lda, const void* B, int64_t ldb,
                                  const void* bias, void* C, int64_t ldc, int fout, int64_t M, int64_t N, int64_t K, void* workspace) {
    typedef typename Storage<F::N>::T T;
    constexpr int L = Arith<F>::L;
    const BucketPrePlan p = bucket_pre_plan<F>(M, N, K);
    double* Ap = (double*)workspace;
    double* Bp = (double*)((char*)workspace + p.b_off);
    const dim3 ga((unsigned)(p.Mp / BP_PRE_TILE), (unsigned)((p.Kp + BP_PRE_TILE - 1) / BP_PRE_TILE));
    const dim3 gb((unsigned)(p.Np / BP_PRE_TILE), (unsigned)((p.Kp + BP_PRE_TILE - 1) / BP_PRE_TILE));
    // op(A)[m,k] is A[m * lda + k] unless transA; op(B)[k,n] is B[k * ldb + n] unless transB
    if (!transA) hipLaunchKernelGGL((bucket_predecode_kernel<F, true>), ga, dim3(256), 0, st, (const T*)A, lda, M, K, Ap, p.Mp, p.Kp);
    else hipLaunchKernelGGL((bucket_predecode_kernel<F, false>), ga, dim3(256), 0, st, (const T*)A, lda, M, K, Ap, p.Mp, p.Kp);
    PNN_CHECK_LAUNCH();
    if (transB) hipLaunchKernelGGL((bucket_predecode_kernel<F, true>), gb, dim3(256), 0, st, (const T*)B, ldb, N, K, Bp, p.Np, p.Kp);
    else hipLaunchKernelGGL((bucket_predecode_kernel<F, false>), gb, dim3(256), 0, st, (const T*)B, ldb, N, K, Bp, p.Np, p.Kp);
    PNN_CHECK_LAUNCH();
    SplitWs ws;
    ws.limbs = nullptr;
    ws.rowflag = nullptr;
    ws.colflag = nullptr;
    if (p.gemm.splits > 1) {
        ws.limbs = (uint32_t*)((char*)workspace + p.split_off);
        ws.rowflag = ws.limbs + (size_t)p.gemm.splits * M * N * L;
        ws.colflag = ws.rowflag + (size_t)p.gemm.splits * M;
    }
    const int64_t tiles_m = (M + p.tile - 1) / p.tile, tiles_n = (N + p.tile - 1) / p.tile;
    const dim3 grid((unsigned)(tiles_m * tiles_n), 1, (unsigned)p.gemm.splits);
    if (p.flush)
        hipLaunchKernelGGL((bucket_pre_gemm_kernel<F, 2, 2, true>), grid, dim3(BP_THREADS), 0, st, Ap, Bp, p.Mp, p.Np, p.gemm.k_per_split,
                           (const T*)bias, C, ldc, fout, M, N, ws, (int)tiles_n);
    else if (p.tile == 64)
        hipLaunchKernelGGL((bucket_pre_gemm_kernel<F, 4, 4, false>), grid, dim3(BP_THREADS), 0, st, Ap, Bp, p.Mp, p.Np, p.gemm.k_per_split,
                           (const T*)bias, C, ldc, fout, M, N, ws, (int)tiles_n);
    else
        hipLaunchKernelGGL((bucket_pre_gemm_kernel<F, 2, 2, false>), grid, dim3(BP_THREADS), 0, st, Ap, Bp, p.Mp, p.Np, p.gemm.k_per_split,
                           (const T*)bias, C, ldc, fout, M, N, ws, (int)tiles_n);
    PNN_CHECK_LAUNCH();
    if (p.gemm.splits > 1) {
        RowMajorOut out{ldc};
        return launch_split_merge<F, RowMajorOut>(st, ws, p.gemm.splits, M, N, bias, C, fout, out);
    }
    return hipSuccess;
}

}  // namespace pnn
