// Implicit-GEMM kernel for the 8-bit posit formats other than posit<8,0> (posit(8,1) and
// posit(8,2) of the paper's experiments, Sec. 4; (8,2) is the format its final configuration
// runs every layer in): convolution forward, backward-data, backward-weight (Sec. 3.1) and
// plain matrix products, all quire-exact (Sec. 3.3).
//
// Operands are fetched with the byte-gather descriptors of the posit<8,0> kernel (affine row /
// reduction index maps, 8-byte runs read as aligned words where the layout allows), decoded
// through a 256-entry LDS table into LDS tiles of doubles, and multiplied into the doubles of
// CascadeArith<F>: the exact sum of an output stays in two or three doubles for the whole
// reduction (carries between them every 16 and 32 products) and becomes the integer quire
// limbs once, in the epilogue, which rounds them once.  256 threads as 16 x 16, TM x TN outputs
// per thread: workgroup tiles of 64 x 64, 64 x 32, 32 x 32 or 16 x 16, chosen per problem (small
// layers need many small tiles to occupy the chip, a 32-channel layer wastes half of a 64-wide
// tile; a 128 x 32 tile would need 80 KB of LDS and leave each CU a single workgroup).
#pragma once

#include "conv_p8.h"

namespace pnn {

template <int BR>
struct B8Stage {
    typedef P8GatherStage<BR> G;
    // decode the 16 bytes of every work item and store them as doubles into dst[k][row]; flags may be null
    // (NaR patterns of that operand are then zeros and nothing more)
    __device__ __forceinline__ static void stage(const P8Frag (&f)[G::PER_THREAD], double (*dst)[BR], const double* tab, uint32_t* flags,
                                                 int t, int mode) {
#pragma unroll
        for (int i = 0; i < G::PER_THREAD; ++i) {
            const int w = t + 256 * i;
            if (G::ITEMS % 256 != 0 && w >= G::ITEMS) continue;
            const uint32_t nar = nar_bytes(f[i].w[0]) | nar_bytes(f[i].w[1]) | nar_bytes(f[i].w[2]) | nar_bytes(f[i].w[3]);
            if (mode == P8_K_RUN) {  // one row, 16 consecutive k
                const int row = w % BR, kq = w / BR;
#pragma unroll
                for (int b = 0; b < 16; ++b) dst[16 * kq + b][row] = tab[(f[i].w[b >> 2] >> (8 * (b & 3))) & 0xFFu];
                if (nar && flags) flags[row] = 1;
                continue;
            }
            const int kp = w / G::GROUPS, c = (w % G::GROUPS) * 8;  // 8 rows at k = 2 kp and 2 kp + 1
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                double d[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) d[j] = tab[(f[i].w[2 * h + (j >> 2)] >> (8 * (j & 3))) & 0xFFu];
#pragma unroll
                for (int j = 0; j < 8; j += 2) *reinterpret_cast<double2*>(&dst[2 * kp + h][c + j]) = make_double2(d[j], d[j + 1]);
            }
            if (nar && flags) {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const uint32_t lo = (f[i].w[j >> 2] >> (8 * (j & 3))) & 0xFFu;
                    const uint32_t hi = (f[i].w[2 + (j >> 2)] >> (8 * (j & 3))) & 0xFFu;
                    if (lo == 0x80u || hi == 0x80u) flags[c + j] = 1;
                }
            }
        }
    }
};

// `bias` (nullable) is indexed by output column n.  With gridDim.z > 1 the partial quires of this
// slice of the reduction go to the workspace (L limbs per output) and a merge kernel finishes.
template <class F, int TM, int TN>
__global__ __launch_bounds__(256) void b8_conv_kernel(P8Gather A, P8Gather B, P8ConvOut out, const uint8_t* __restrict__ bias,
                                                      void* __restrict__ C, int fout, int M, int N, int K, int k_per_split,
                                                      int tiles_n, SplitWs ws, int ws_transposed) {
    typedef BucketAccum<F> AR;
    typedef CascadeArith<F> CA;
    static_assert(F::N == 8 && CA::ELIGIBLE && P8_KT == CA::TOP_EVERY && P8_KT == 2 * CA::LOW_EVERY, "carry schedule of a 32-wide slice");
    constexpr int BM = 16 * TM, BN = 16 * TN, L = AR::L, NL = CA::NL;
    static_assert(BM % 8 == 0 && BN % 8 == 0 && BM + BN <= 256, "tile shape");
    typedef P8GatherStage<BM> GA;
    typedef P8GatherStage<BN> GB;
    __shared__ __attribute__((aligned(16))) double As[2][P8_KT][BM];
    __shared__ __attribute__((aligned(16))) double Bs[2][P8_KT][BN];
    __shared__ int4 rinfoA[BM];
    __shared__ int4 rinfoB[BN];
    __shared__ int4 kinfoA[2][P8_KT];  // slice kt uses kinfo[kt & 1], filled two iterations ahead
    __shared__ int4 kinfoB[2][P8_KT];
    __shared__ double tab[256];
    __shared__ uint32_t rowNaR[BM];
    __shared__ uint32_t colNaR[BN];

    const int t = threadIdx.x;
    const int tx = t & 15, ty = t >> 4;
    const int tile = blockIdx.x;
    const int m0 = (tile / tiles_n) * BM, n0 = (tile % tiles_n) * BN;
    const int kbeg = blockIdx.z * k_per_split;
    const int kend = (kbeg + k_per_split < K) ? kbeg + k_per_split : K;

    tab[t] = AR::stage((uint32_t)t);
    if (t < BM) {
        int4 ri = make_int4(0, OUT_OF_RANGE, 0, 0);
        if (m0 + t < M) A.row.eval((uint32_t)(m0 + t), ri.x, ri.y, ri.z);
        rinfoA[t] = ri;
        rowNaR[t] = 0;
    } else if (t < BM + BN) {
        const int r = t - BM;
        int4 ri = make_int4(0, OUT_OF_RANGE, 0, 0);
        if (n0 + r < N) B.row.eval((uint32_t)(n0 + r), ri.x, ri.y, ri.z);
        rinfoB[r] = ri;
        colNaR[r] = 0;
    }

    double sum[TM][TN][NL];  // the exact sum of each output, spread over NL doubles
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) CA::clear(sum[i][j]);

    const int nkt = (kend - kbeg + P8_KT - 1) / P8_KT;
    uint32_t* const aflags = A.quiet_nar ? nullptr : rowNaR;
    uint32_t* const bflags = B.quiet_nar ? nullptr : colNaR;
    // B's work items go to the threads A's leave idle when both fit the workgroup
    const int tb = (GA::ITEMS + GB::ITEMS <= 256) ? ((t + 256 - GA::ITEMS) & 255) : t;
    if (t < P8_KT) p8_fill_kinfo(A, kinfoA[0], kbeg, kend, t);
    else if (t < 2 * P8_KT) p8_fill_kinfo(B, kinfoB[0], kbeg, kend, t - P8_KT);
    __syncthreads();
    {
        P8Frag fa[GA::PER_THREAD], fb[GB::PER_THREAD];
        if (nkt > 0) {
            GA::fetch(A, rinfoA, kinfoA[0], kbeg, kend, M - m0, t, fa);
            GB::fetch(B, rinfoB, kinfoB[0], kbeg, kend, N - n0, tb, fb);
            if (nkt > 1) {
                if (t < P8_KT) p8_fill_kinfo(A, kinfoA[1], kbeg + P8_KT, kend, t);
                else if (t < 2 * P8_KT) p8_fill_kinfo(B, kinfoB[1], kbeg + P8_KT, kend, t - P8_KT);
            }
            B8Stage<BM>::stage(fa, As[0], tab, aflags, t, A.mode);
            B8Stage<BN>::stage(fb, Bs[0], tab, bflags, tb, B.mode);
        }
    }
    __syncthreads();

    for (int kt = 0; kt < nkt; ++kt) {
        const int cur = kt & 1;
        const bool more = kt + 1 < nkt;
        P8Frag fa[GA::PER_THREAD], fb[GB::PER_THREAD];
        if (more) {
            const int k0 = kbeg + (kt + 1) * P8_KT;
            GA::fetch(A, rinfoA, kinfoA[cur ^ 1], k0, kend, M - m0, t, fa);
            GB::fetch(B, rinfoB, kinfoB[cur ^ 1], k0, kend, N - n0, tb, fb);
        }
        if (kt + 2 < nkt) {  // kinfo[cur] was last read when slice kt was fetched, one barrier ago
            const int k2 = kbeg + (kt + 2) * P8_KT;
            if (t < P8_KT) p8_fill_kinfo(A, kinfoA[cur], k2, kend, t);
            else if (t < 2 * P8_KT) p8_fill_kinfo(B, kinfoB[cur], k2, kend, t - P8_KT);
        }
#pragma unroll
        for (int half = 0; half < 2; ++half) {
#pragma unroll 4
            for (int kq = 0; kq < CA::LOW_EVERY; ++kq) {
                const int kk = half * CA::LOW_EVERY + kq;
                double a[TM], b[TN];
                if constexpr (TM % 2 == 0) {
#pragma unroll
                    for (int q = 0; q < TM; q += 2) {
                        const double2 v = *reinterpret_cast<const double2*>(&As[cur][kk][ty * TM + q]);
                        a[q] = v.x; a[q + 1] = v.y;
                    }
                } else {
#pragma unroll
                    for (int q = 0; q < TM; ++q) a[q] = As[cur][kk][ty * TM + q];
                }
                if constexpr (TN % 2 == 0) {
#pragma unroll
                    for (int q = 0; q < TN; q += 2) {
                        const double2 v = *reinterpret_cast<const double2*>(&Bs[cur][kk][tx * TN + q]);
                        b[q] = v.x; b[q + 1] = v.y;
                    }
                } else {
#pragma unroll
                    for (int q = 0; q < TN; ++q) b[q] = Bs[cur][kk][tx * TN + q];
                }
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) CA::mac(sum[i][j], a[i], b[j]);
            }
            // 16 products per output since the last carry out of the low levels
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) CA::carry_low(sum[i][j]);
        }
        // 32 products since the top bucket last carried into level 0
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) CA::carry_top(sum[i][j]);
        if (more) {
            B8Stage<BM>::stage(fa, As[cur ^ 1], tab, aflags, t, A.mode);
            B8Stage<BN>::stage(fb, Bs[cur ^ 1], tab, bflags, tb, B.mode);
        }
        __syncthreads();
    }

#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int lr = ty * TM + i;
        const int m = m0 + lr;
        if (m >= M) continue;
        const bool rnar = rowNaR[lr] != 0;
        const int64_t rp = gridDim.z == 1 ? out.row_part(m) : 0;
        if (rp < 0) continue;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int lc = tx * TN + j;
            const int n = n0 + lc;
            if (n >= N) continue;
            uint32_t q[L];  // the sum as integer quire limbs, modulo 2^(32 L)
#pragma unroll
            for (int l = 0; l < L; ++l) q[l] = 0;
            CA::template to_limbs<L>(q, sum[i][j]);
            if (gridDim.z == 1) {
                bool nar = rnar || colNaR[lc] != 0;
                if (bias) {
                    const uint32_t bp = bias[n];
                    if (bp == F::NAR) nar = true;
                    else AR::add_bias(q, bp);
                }
                round_store<AR, L>(q, nar, fout, C, rp + (int64_t)n * out.nstride);
            } else {
                // partial quire; the merge kernel sees an (Mw x Nw) row-major problem
                const int64_t z = blockIdx.z;
                const int64_t idx = ws_transposed ? ((int64_t)n * M + m) : ((int64_t)m * N + n);
#pragma unroll
                for (int l = 0; l < L; ++l) ws.limbs[(z * (int64_t)M * N + idx) * L + l] = q[l];
            }
        }
    }
    if (gridDim.z > 1) {
        const int64_t z = blockIdx.z;
        uint32_t* rflag = ws_transposed ? ws.colflag : ws.rowflag;  // flags in the orientation of the merge kernel
        uint32_t* cflag = ws_transposed ? ws.rowflag : ws.colflag;
        // the first tile column stores the row flags of its tile row (identical in every column), the
        // first tile row the column flags: every entry is written, so the workspace needs no clearing
        if (n0 == 0)
            for (int r = t; r < BM; r += 256)
                if (m0 + r < M) rflag[z * M + m0 + r] = rowNaR[r];
        if (m0 == 0)
            for (int r = t; r < BN; r += 256)
                if (n0 + r < N) cflag[z * N + n0 + r] = colNaR[r];
    }
}

// Workgroup tile.  Larger tiles reuse staged operands more; smaller ones waste less of a ragged
// edge and give the 256 CUs enough workgroups on small layers.  Score = useful fraction of the
// tiles x how far the grid fills the chip (a long reduction can be split instead) x operand reuse.
struct B8Tile { int bm, bn; };
static const B8Tile B8_TILES[] = {{64, 64}, {64, 32}, {32, 32}, {16, 16}};

inline B8Tile b8_tile(int M, int N, int K) {
    const bool can_split = K >= 1024;
    B8Tile best = B8_TILES[0];
    double best_score = -1.0;
    for (const B8Tile& t : B8_TILES) {
        const int64_t blocks = (int64_t)((M + t.bm - 1) / t.bm) * ((N + t.bn - 1) / t.bn);
        const double util = ((double)M * N) / ((double)blocks * t.bm * t.bn);
        const double fill = (can_split || blocks >= 512) ? 1.0 : (double)blocks / 512.0;
        const double reuse = (double)(t.bm * t.bn) / (t.bm + t.bn) / 32.0;  // MACs per staged element, relative to 64 x 64
        const double score = util * fill * (0.5 + 0.5 * reuse);
        if (score > best_score) { best_score = score; best = t; }
    }
    return best;
}

template <class F>
inline GemmPlan b8_conv_plan(int M, int N, int K) {
    const B8Tile tl = b8_tile(M, N, K);
    return plan_split(M, N, K, tl.bm, tl.bn, Arith<F>::L, P8_KT);
}

// Launch on a problem built by p8_problem / p8_gemm_problem; merge_out maps the merged (Mw x Nw)
// result to the output tensor.
template <class F, class Out>
hipError_t b8_conv_launch(hipStream_t st, const P8ConvProblem& p, const uint8_t* bias, void* C, int fout, void* wsp,
                          const GemmPlan& plan, const Out& merge_out) {
    constexpr int L = Arith<F>::L;
    const B8Tile tl = b8_tile(p.M, p.N, p.K);
    const int tiles_m = (p.M + tl.bm - 1) / tl.bm, tiles_n = (p.N + tl.bn - 1) / tl.bn;
    SplitWs ws;
    ws.limbs = nullptr; ws.rowflag = nullptr; ws.colflag = nullptr;
    if (plan.splits > 1) {
        ws.limbs = (uint32_t*)wsp;
        ws.rowflag = ws.limbs + (size_t)plan.splits * p.M * p.N * L;
        ws.colflag = ws.rowflag + (size_t)plan.splits * p.Mw;
    }
    dim3 grid((unsigned)(tiles_m * tiles_n), 1, (unsigned)plan.splits);
    const uint8_t* kbias = plan.splits > 1 ? nullptr : bias;
#define PNN_LAUNCH_B8(TM, TN)                                                                                                  \
    hipLaunchKernelGGL((b8_conv_kernel<F, TM, TN>), grid, dim3(256), 0, st, p.A, p.B, p.out, kbias, C, fout, p.M, p.N, p.K, \
                       (int)plan.k_per_split, tiles_n, ws, p.transposed)
    if (tl.bm == 64 && tl.bn == 64) PNN_LAUNCH_B8(4, 4);
    else if (tl.bm == 64) PNN_LAUNCH_B8(4, 2);
    else if (tl.bm == 32) PNN_LAUNCH_B8(2, 2);
    else PNN_LAUNCH_B8(1, 1);
#undef PNN_LAUNCH_B8
    PNN_CHECK_LAUNCH();
    if (plan.splits > 1) return launch_split_merge<F, Out>(st, ws, plan.splits, p.Mw, p.Nw, bias, C, fout, merge_out);
    return hipSuccess;
}

// Small matrix products (the fully connected layers of the small networks: a few thousand outputs,
// a reduction of a few hundred): one output per group of S threads that split the reduction, so that
// the outputs spread over many workgroups instead of one or two tiles walking the reduction slice
// by slice.  Each thread gathers its products in the fp64 buckets (emptied into its private limbs
// every 32 products), the S partial quires of an output are summed through LDS (exact) and rounded once.
//   element strides: A(m,k) = A[m*a_m + k*a_k], B(k,n) = B[k*b_k + n*b_n]
template <class F>
__global__ __launch_bounds__(256) void b8_small_gemm_kernel(const uint8_t* __restrict__ A, int64_t a_m, int64_t a_k,
                                                            const uint8_t* __restrict__ B, int64_t b_k, int64_t b_n,
                                                            const uint8_t* __restrict__ bias, void* __restrict__ C, int64_t ldc, int fout,
                                                            int M, int N, int K, int S, int k_per_split) {
    typedef BucketAccum<F> AR;
    static_assert(F::N == 8 && AR::BUCKETS > 0 && (1 << AR::G) >= 32, "8-bit bucketed format");
    constexpr int L = AR::L, NB = AR::NB;
    __shared__ double tab[256];
    __shared__ uint32_t part[256][L];
    __shared__ uint32_t nars[256];
    const int t = threadIdx.x;
    tab[t] = AR::stage((uint32_t)t);
    __syncthreads();
    const int OB = 256 / S;  // outputs per workgroup
    const int ol = t % OB, s = t / OB;
    const int64_t o = (int64_t)blockIdx.x * OB + ol;
    const bool live = o < (int64_t)M * N;
    const int m = live ? (int)(o / N) : 0, n = live ? (int)(o - (int64_t)m * N) : 0;
    const int k_lo = s * k_per_split, k_hi = k_lo + k_per_split < K ? k_lo + k_per_split : K;
    uint32_t q[L];
#pragma unroll
    for (int l = 0; l < L; ++l) q[l] = 0;
    double bk[NB];
    AR::clear(bk);
    uint32_t nar = 0;
    if (live) {
        const uint8_t* ap = A + (int64_t)m * a_m + (int64_t)k_lo * a_k;
        const uint8_t* bp = B + (int64_t)n * b_n + (int64_t)k_lo * b_k;
        for (int kb = k_lo; kb < k_hi; kb += 32) {  // at most 32 products between two flushes
            const int ke = kb + 32 < k_hi ? kb + 32 : k_hi;
            int k = kb;
            for (; k + 4 <= ke; k += 4) {
                uint32_t a[4], b[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    a[u] = ap[u * a_k];
                    b[u] = bp[u * b_k];
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    nar |= (a[u] == 0x80u) | (b[u] == 0x80u);
                    AR::mac(bk, tab[a[u]], tab[b[u]]);
                }
                ap += 4 * a_k;
                bp += 4 * b_k;
            }
            for (; k < ke; ++k) {
                const uint32_t a = *ap, b = *bp;
                nar |= (a == 0x80u) | (b == 0x80u);
                AR::mac(bk, tab[a], tab[b]);
                ap += a_k;
                bp += b_k;
            }
            AR::template flush<L>(q, bk);
        }
    }
#pragma unroll
    for (int l = 0; l < L; ++l) part[t][l] = q[l];
    nars[t] = nar;
    __syncthreads();
    if (s != 0 || !live) return;
    for (int z = 1; z < S; ++z) {
        uint32_t o2[L];
#pragma unroll
        for (int l = 0; l < L; ++l) o2[l] = part[z * OB + ol][l];
        quire_merge<L>(q, o2);
        nar |= nars[z * OB + ol];
    }
    bool isnar = nar != 0;
    if (bias) {
        const uint32_t bpat = bias[n];
        if (bpat == F::NAR) isnar = true;
        else AR::add_bias(q, bpat);
    }
    round_store<AR, L>(q, isnar, fout, C, (int64_t)m * ldc + n);
}

template <class F>
inline hipError_t launch_b8_small_gemm(hipStream_t stream, int transA, int transB, const uint8_t* A, int64_t lda, const uint8_t* B,
                                       int64_t ldb, const uint8_t* bias, void* C, int64_t ldc, int fout, int64_t M, int64_t N, int64_t K) {
    // threads per output: keep at least 32 reduction steps per thread, and stop once about 1024 workgroups exist
    int S = 1;
    while (S < 64 && K / (2 * S) >= 32 && (M * N * S) / 256 < 1024) S *= 2;
    const int kps = (int)((K + S - 1) / S);
    const int OB = 256 / S;
    const int64_t blocks = (M * N + OB - 1) / OB;
    hipLaunchKernelGGL(b8_small_gemm_kernel<F>, dim3((unsigned)blocks), dim3(256), 0, stream, A, transA ? (int64_t)1 : lda,
                       transA ? lda : (int64_t)1, B, transB ? (int64_t)1 : ldb, transB ? ldb : (int64_t)1, bias, C, ldc, fout, (int)M, (int)N,
                       (int)K, S, kps);
    return hipGetLastError();
}

}  // namespace pnn
