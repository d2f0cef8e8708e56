// posit<8,0> implicit-GEMM convolution on the packed dot-product kernel (paper
// Sec. 3.1: convolution layers and their hand-written backward passes; Sec. 3.3:
// quire accumulation in convolutions; Table 1: 32-bit quire).
//
// All three passes are C[m,n] = sum_k A(m,k) * B(n,k) over virtual operand
// matrices whose elements live at   base + rowpart(row) + kpart(k)   in a tensor
// and are zero unless  0 <= rowy(row)+ky(k) < LY  and  0 <= rowx(row)+kx(k) < LX
// (the image bounds; padding and partner-less taps are zero operands).  rowpart,
// rowy, rowx are affine in the (up to three) coordinates a row index splits into,
// likewise for k, so one run-time description covers
//   forward        A: rows (n,oh,ow), k (c,r,s) on x      B: rows ko,      k (c,r,s) on w
//   backward-data  A: rows (n,h,w),   k (ko,r,s) on dy    B: rows c,       k (ko,r,s) on w   (stride 1)
//   backward-weight (computed transposed)
//                  A: rows (c,r,s),   k (n,oh,ow) on x    B: rows ko,      k (n,oh,ow) on dy
// The kernel body is the one of the GEMM kernel: decode through the LDS table at
// staging, (k,k+1) pairs packed per 32-bit LDS word, v_dot2_i32_i16 on an 8 x TN
// register tile, NaR as row/column flags, int32 quire rounded once.
#pragma once

#include "gemm_p8.h"

namespace pnn {

// n / d for 0 <= n < 2^31 by multiply-high (d >= 1)
struct FastDiv {
    uint32_t d, mul, shift;
    PNN_HD uint32_t div(uint32_t n) const {
#if defined(__HIP_DEVICE_COMPILE__)
        return (uint32_t)((__umulhi(n, mul) + n) >> shift);
#else
        return (uint32_t)(((uint32_t)(((uint64_t)n * mul) >> 32) + n) >> shift);
#endif
    }
};

inline FastDiv make_fastdiv(uint32_t d) {
    FastDiv f;
    f.d = d;
    uint32_t s = 0;
    while (((uint64_t)1 << s) < d) ++s;
    // floor(2^32 * (2^s - d) / d) + 1 ; with n < 2^31 the sum mulhi + n cannot overflow 32 bits
    f.mul = (uint32_t)(((((uint64_t)1 << s) - d) << 32) / d + 1);
    f.shift = s;
    return f;
}

// index -> (c2, c1, c0) with index = (c2 * d1 + c1) * d0 + c0, then three affine forms
struct AffineIndex {
    FastDiv d1d0, d0;  // divide by d1*d0, then the remainder by d0
    int part2, part1, part0, partc;
    int y1, y0, yc;    // y depends on c1 (and c0 for flattened cases), x on c0
    int x1, x0, xc;
    PNN_HD void eval(uint32_t idx, int& part, int& y, int& x) const {
        const uint32_t c2 = d1d0.div(idx);
        const uint32_t rem = idx - c2 * d1d0.d;
        const uint32_t c1 = d0.div(rem);
        const uint32_t c0 = rem - c1 * d0.d;
        part = (int)c2 * part2 + (int)c1 * part1 + (int)c0 * part0 + partc;
        y = (int)c1 * y1 + (int)c0 * y0 + yc;
        x = (int)c1 * x1 + (int)c0 * x0 + xc;
    }
};

struct P8Gather {
    const uint8_t* base;
    int rows, K;     // extents of the virtual matrix
    int LY, LX;      // bounds for y and x
    AffineIndex row, k;
};

constexpr int OUT_OF_RANGE = -(1 << 28);  // a y that can never pass the bounds test

struct P8ConvOut {
    // element index of output (m, n) = mpart(m) + n * nstride, mpart affine in m's coordinates
    FastDiv md;          // m = c1 * md.d + c0
    int64_t m1, m0;      // mpart = c1 * m1 + c0 * m0
    int64_t nstride;
    PNN_HD int64_t at(int m, int n) const {
        const uint32_t c1 = md.div((uint32_t)m);
        const uint32_t c0 = (uint32_t)m - c1 * md.d;
        return (int64_t)c1 * m1 + (int64_t)c0 * m0 + (int64_t)n * nstride;
    }
};

// One operand slice: BR rows x 32 k.  Work item w handles k-pair w / (BR/8) and rows 8*(w % (BR/8)) .. +7.
template <int BR>
struct P8GatherStage {
    static constexpr int GROUPS = BR / 8;
    static constexpr int ITEMS = GROUPS * P8_KP;
    static constexpr int PER_THREAD = (ITEMS + 255) / 256;

    // fetch the 16 bytes of every work item of this thread
    __device__ __forceinline__ static void fetch(const P8Gather& op, const int4* __restrict__ rinfo, int k0, int kend, int t,
                                                 P8Frag (&f)[PER_THREAD]) {
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            const int w = t + 256 * i;
            f[i].w[0] = f[i].w[1] = f[i].w[2] = f[i].w[3] = 0;
            if (ITEMS % 256 != 0 && w >= ITEMS) continue;
            const int kp = w / GROUPS, g = w % GROUPS;
            int kpart[2], ky[2], kx[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int k = k0 + 2 * kp + h;
                op.k.eval((uint32_t)(k < kend ? k : 0), kpart[h], ky[h], kx[h]);
                if (k >= kend) ky[h] = OUT_OF_RANGE;
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int4 ri = rinfo[g * 8 + j];  // part, y, x
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const bool ok = ((uint32_t)(ri.y + ky[h]) < (uint32_t)op.LY) && ((uint32_t)(ri.z + kx[h]) < (uint32_t)op.LX);
                    const uint32_t byte = ok ? (uint32_t)op.base[ri.x + kpart[h]] : 0u;
                    f[i].w[2 * h + (j >> 2)] |= byte << (8 * (j & 3));
                }
            }
        }
    }

    // decode + pack + store into dst[k-pair][row]; flags[row] for NaR
    template <int LD>
    __device__ __forceinline__ static void stage(const P8Frag (&f)[PER_THREAD], uint32_t (*dst)[LD], const uint16_t* tab,
                                                 uint32_t* flags, int t) {
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            const int w = t + 256 * i;
            if (ITEMS % 256 != 0 && w >= ITEMS) continue;
            const int kp = w / GROUPS, c = (w % GROUPS) * 8;
            uint32_t d[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint32_t lo = (f[i].w[j >> 2] >> (8 * (j & 3))) & 0xFFu;
                const uint32_t hi = (f[i].w[2 + (j >> 2)] >> (8 * (j & 3))) & 0xFFu;
                d[j] = (uint32_t)tab[lo] | ((uint32_t)tab[hi] << 16);
            }
            *reinterpret_cast<uint4*>(&dst[kp][c]) = make_uint4(d[0], d[1], d[2], d[3]);
            *reinterpret_cast<uint4*>(&dst[kp][c + 4]) = make_uint4(d[4], d[5], d[6], d[7]);
            const uint32_t nar = nar_bytes(f[i].w[0]) | nar_bytes(f[i].w[1]) | nar_bytes(f[i].w[2]) | nar_bytes(f[i].w[3]);
            if (nar) {
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

// TY x TX threads (= 256), register tile TM x TN, workgroup tile BM = TY*TM by BN = TX*TN.
// `bias` (nullable) is indexed by output column n.  With gridDim.z > 1 partial quires go to the workspace.
template <int TY, int TX, int TM, int TN>
__global__ __launch_bounds__(256, 3) void p8_conv_kernel(P8Gather A, P8Gather B, P8ConvOut out, const uint8_t* __restrict__ bias,
                                                         void* __restrict__ C, int fout, int M, int N, int K, int k_per_split,
                                                         int tiles_n, SplitWs ws, int ws_transposed) {
    static_assert(TY * TX == 256 && (TM == 4 || TM == 8) && (TN == 4 || TN == 8), "tile shape");
    constexpr int BM = TY * TM, BN = TX * TN;
    typedef P8GatherStage<BM> SA;
    typedef P8GatherStage<BN> SB;
    __shared__ __attribute__((aligned(16))) uint32_t As[2][P8_KP][BM];
    __shared__ __attribute__((aligned(16))) uint32_t Bs[2][P8_KP][BN];
    __shared__ int4 rinfoA[BM];
    __shared__ int4 rinfoB[BN];
    __shared__ uint16_t tab[256];
    __shared__ uint32_t rowNaR[BM];
    __shared__ uint32_t colNaR[BN];

    const int t = threadIdx.x;
    const int tx = t % TX, ty = t / TX;
    const int tile = blockIdx.x;
    const int m0 = (tile / tiles_n) * BM, n0 = (tile % tiles_n) * BN;
    const int kbeg = blockIdx.z * k_per_split;
    const int kend = (kbeg + k_per_split < K) ? kbeg + k_per_split : K;

    tab[t] = (uint16_t)Arith<P8>::stage((uint32_t)t);
    for (int r = t; r < BM; r += 256) {
        int4 ri = make_int4(0, OUT_OF_RANGE, 0, 0);
        if (m0 + r < M) A.row.eval((uint32_t)(m0 + r), ri.x, ri.y, ri.z);
        rinfoA[r] = ri;
        rowNaR[r] = 0;
    }
    for (int r = t; r < BN; r += 256) {
        int4 ri = make_int4(0, OUT_OF_RANGE, 0, 0);
        if (n0 + r < N) B.row.eval((uint32_t)(n0 + r), ri.x, ri.y, ri.z);
        rinfoB[r] = ri;
        colNaR[r] = 0;
    }

    int32_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = 0;

    const int nkt = (kend - kbeg + P8_KT - 1) / P8_KT;
    __syncthreads();
    {
        P8Frag fa[SA::PER_THREAD], fb[SB::PER_THREAD];
        if (nkt > 0) {
            SA::fetch(A, rinfoA, kbeg, kend, t, fa);
            SB::fetch(B, rinfoB, kbeg, kend, t, fb);
            SA::template stage<BM>(fa, As[0], tab, rowNaR, t);
            SB::template stage<BN>(fb, Bs[0], tab, colNaR, t);
        }
    }
    __syncthreads();

    for (int kt = 0; kt < nkt; ++kt) {
        const int cur = kt & 1;
        const bool more = kt + 1 < nkt;
        P8Frag fa[SA::PER_THREAD], fb[SB::PER_THREAD];
        if (more) {
            const int k0 = kbeg + (kt + 1) * P8_KT;
            SA::fetch(A, rinfoA, k0, kend, t, fa);
            SB::fetch(B, rinfoB, k0, kend, t, fb);
        }
#pragma unroll 2
        for (int kp = 0; kp < P8_KP; ++kp) {
            uint32_t a[TM], b[TN];
#pragma unroll
            for (int q = 0; q < TM / 4; ++q) {
                const uint4 v = *reinterpret_cast<const uint4*>(&As[cur][kp][q * (TY * 4) + ty * 4]);
                a[4 * q] = v.x; a[4 * q + 1] = v.y; a[4 * q + 2] = v.z; a[4 * q + 3] = v.w;
            }
#pragma unroll
            for (int q = 0; q < TN / 4; ++q) {
                const uint4 v = *reinterpret_cast<const uint4*>(&Bs[cur][kp][q * (TX * 4) + tx * 4]);
                b[4 * q] = v.x; b[4 * q + 1] = v.y; b[4 * q + 2] = v.z; b[4 * q + 3] = v.w;
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] = dot2_acc(a[i], b[j], acc[i][j]);
        }
        if (more) {
            SA::template stage<BM>(fa, As[cur ^ 1], tab, rowNaR, t);
            SB::template stage<BN>(fb, Bs[cur ^ 1], tab, colNaR, t);
        }
        __syncthreads();
    }

#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int lr = (i >> 2) * (TY * 4) + ty * 4 + (i & 3);
        const int m = m0 + lr;
        if (m >= M) continue;
        const bool rnar = rowNaR[lr] != 0;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int lc = (j >> 2) * (TX * 4) + tx * 4 + (j & 3);
            const int n = n0 + lc;
            if (n >= N) continue;
            if (gridDim.z == 1) {
                int32_t q = acc[i][j];
                bool nar = rnar || colNaR[lc] != 0;
                if (bias) {
                    const uint32_t bp = bias[n];
                    if (bp == 0x80u) nar = true;
                    else q += (int32_t)(int16_t)tab[bp] << P8::MAXS;
                }
                const int64_t at = out.at(m, n);
                if (fout == 0) {
                    ((uint8_t*)C)[at] = (uint8_t)(nar ? 0x80u : p8_round_quire(q));
                } else {
                    const uint32_t q1[1] = {(uint32_t)q};
                    round_store<QuireAccum<P8>, 1>(q1, nar, fout, C, at);
                }
            } else {
                // partial quire; the merge kernel sees an (Mw x Nw) row-major problem
                const int64_t z = blockIdx.z;
                const int64_t idx = ws_transposed ? ((int64_t)n * M + m) : ((int64_t)m * N + n);
                ws.limbs[z * (int64_t)M * N + idx] = (uint32_t)acc[i][j];
            }
        }
    }
    if (gridDim.z > 1) {
        const int64_t z = blockIdx.z;
        // flags in the orientation of the merge kernel: its rows are our columns when transposed
        uint32_t* rflag = ws_transposed ? ws.colflag : ws.rowflag;
        uint32_t* cflag = ws_transposed ? ws.rowflag : ws.colflag;
        for (int r = t; r < BM; r += 256)
            if (m0 + r < M && rowNaR[r]) atomicOr(&rflag[z * M + m0 + r], 1u);
        for (int r = t; r < BN; r += 256)
            if (n0 + r < N && colNaR[r]) atomicOr(&cflag[z * N + n0 + r], 1u);
    }
}

// ---- posit<8,0> path: implicit GEMM on the packed dot-product kernel ----

inline AffineIndex affine(uint32_t d1, uint32_t d0, int p2, int p1, int p0, int pc, int y1, int y0, int yc, int x1, int x0, int xc) {
    AffineIndex a;
    a.d1d0 = make_fastdiv(d1 * d0);
    a.d0 = make_fastdiv(d0);
    a.part2 = p2; a.part1 = p1; a.part0 = p0; a.partc = pc;
    a.y1 = y1; a.y0 = y0; a.yc = yc;
    a.x1 = x1; a.x0 = x0; a.xc = xc;
    return a;
}

struct P8ConvProblem {
    P8Gather A, B;
    P8ConvOut out;
    int M, N, K;          // kernel view: rows of A, rows of B, reduction
    int64_t Mw, Nw;       // row-major view of the merged result (differs when computed transposed)
    int transposed;
};

// every tensor offset must fit a signed 32-bit integer
inline bool p8_conv_fits(const ConvGeom& g) {
    const int64_t lim = ((int64_t)1 << 31) - 1;
    return (int64_t)g.N * g.C * g.H * g.W < lim && (int64_t)g.N * g.K * g.OH * g.OW < lim && (int64_t)g.K * g.C * g.R * g.S < lim;
}

inline P8ConvProblem p8_problem(int which, const ConvGeom& g, const void* t0, const void* t1) {
    P8ConvProblem p;
    const int HW = g.H * g.W, OHW = g.OH * g.OW, RS = g.R * g.S, CRS = g.C * RS;
    if (which == 0) {  // t0 = x, t1 = w
        p.M = g.N * OHW; p.N = g.K; p.K = CRS; p.transposed = 0;
        p.A.base = (const uint8_t*)t0; p.A.rows = p.M; p.A.K = p.K; p.A.LY = g.H; p.A.LX = g.W;
        p.A.row = affine(g.OH, g.OW, g.C * HW, g.sh * g.W, g.sw, -g.ph * g.W - g.pw, g.sh, 0, -g.ph, 0, g.sw, -g.pw);
        p.A.k = affine(g.R, g.S, HW, g.W, 1, 0, 1, 0, 0, 0, 1, 0);
        p.B.base = (const uint8_t*)t1; p.B.rows = p.N; p.B.K = p.K; p.B.LY = 1; p.B.LX = 1;
        p.B.row = affine(1, 1, CRS, 0, 0, 0, 0, 0, 0, 0, 0, 0);
        p.B.k = affine(1, 1, 1, 0, 0, 0, 0, 0, 0, 0, 0, 0);
        p.out.md = make_fastdiv(OHW); p.out.m1 = (int64_t)g.K * OHW; p.out.m0 = 1; p.out.nstride = OHW;
    } else if (which == 1) {  // t0 = dy, t1 = w ; stride 1 only
        p.M = g.N * HW; p.N = g.C; p.K = g.K * RS; p.transposed = 0;
        p.A.base = (const uint8_t*)t0; p.A.rows = p.M; p.A.K = p.K; p.A.LY = g.OH; p.A.LX = g.OW;
        p.A.row = affine(g.H, g.W, g.K * OHW, g.OW, 1, g.ph * g.OW + g.pw, 1, 0, g.ph, 0, 1, g.pw);
        p.A.k = affine(g.R, g.S, OHW, -g.OW, -1, 0, -1, 0, 0, 0, -1, 0);
        p.B.base = (const uint8_t*)t1; p.B.rows = p.N; p.B.K = p.K; p.B.LY = 1; p.B.LX = 1;
        p.B.row = affine(1, 1, RS, 0, 0, 0, 0, 0, 0, 0, 0, 0);
        p.B.k = affine(RS, 1, CRS, 1, 0, 0, 0, 0, 0, 0, 0, 0);
        p.out.md = make_fastdiv(HW); p.out.m1 = (int64_t)g.C * HW; p.out.m0 = 1; p.out.nstride = HW;
    } else {  // t0 = dy, t1 = x ; computed transposed: rows (c,r,s), columns ko
        p.M = CRS; p.N = g.K; p.K = g.N * OHW; p.transposed = 1;
        p.A.base = (const uint8_t*)t1; p.A.rows = p.M; p.A.K = p.K; p.A.LY = g.H; p.A.LX = g.W;
        p.A.row = affine(g.R, g.S, HW, g.W, 1, -g.ph * g.W - g.pw, 1, 0, -g.ph, 0, 1, -g.pw);
        p.A.k = affine(g.OH, g.OW, g.C * HW, g.sh * g.W, g.sw, 0, g.sh, 0, 0, 0, g.sw, 0);
        p.B.base = (const uint8_t*)t0; p.B.rows = p.N; p.B.K = p.K; p.B.LY = 1; p.B.LX = 1;
        p.B.row = affine(1, 1, OHW, 0, 0, 0, 0, 0, 0, 0, 0, 0);
        p.B.k = affine(OHW, 1, g.K * OHW, 1, 0, 0, 0, 0, 0, 0, 0, 0);
        p.out.md = make_fastdiv(1); p.out.m1 = 1; p.out.m0 = 0; p.out.nstride = CRS;
    }
    p.Mw = p.transposed ? p.N : p.M;
    p.Nw = p.transposed ? p.M : p.N;
    return p;
}

// Workgroup tile (rows x columns of the virtual GEMM).  Larger tiles reuse staged
// operands more; smaller ones give the 256 CUs enough workgroups on the small
// layers.  Pick the largest tile that still yields >= 512 workgroups (counting the
// reduction split), else the one with the most workgroups.
struct P8ConvTile { int bm, bn; };
static const P8ConvTile P8_CONV_TILES[] = {{128, 128}, {256, 64}, {256, 32}, {128, 64}, {64, 64}};

inline int64_t p8_conv_blocks(const P8ConvTile& t, int M, int N) {
    return (int64_t)((M + t.bm - 1) / t.bm) * ((N + t.bn - 1) / t.bn);
}

inline P8ConvTile p8_conv_tile(int M, int N, int K) {
    const bool can_split = K >= 1024;  // a long reduction supplies the parallelism by itself
    P8ConvTile best = P8_CONV_TILES[4];
    double best_score = -1.0;
    for (const P8ConvTile& t : P8_CONV_TILES) {
        const int64_t blocks = p8_conv_blocks(t, M, N);
        const double util = ((double)M * N) / ((double)blocks * t.bm * t.bn);  // useful fraction of the tiles
        const double fill = (can_split || blocks >= 512) ? 1.0 : (double)blocks / 512.0;
        // operand reuse: MACs per staged element, relative to the 128 x 128 tile
        const double reuse = (double)(t.bm * t.bn) / (t.bm + t.bn) / 64.0;
        const double score = util * fill * (0.5 + 0.5 * reuse);
        if (score > best_score) { best_score = score; best = t; }
    }
    return best;
}

inline GemmPlan p8_conv_plan(int M, int N, int K) {
    const P8ConvTile tl = p8_conv_tile(M, N, K);
    return plan_split(M, N, K, tl.bm, tl.bn, 1, P8_KT);
}

inline bool p8_conv_eligible(int which, const ConvGeom& g) {
    if (!p8_conv_fits(g)) return false;
    if (which == 1 && (g.sh != 1 || g.sw != 1)) return false;
    return true;
}


// Plain (possibly transposed, pitched) matrices as gather operands: small or oddly
// shaped posit<8,0> products use the same kernel as the convolutions.
inline bool p8_gemm_as_gather_fits(int transA, int transB, int64_t M, int64_t N, int64_t K, int64_t lda, int64_t ldb) {
    const int64_t lim = ((int64_t)1 << 31) - 1;
    const int64_t a_ext = transA ? K * lda : M * lda, b_ext = transB ? N * ldb : K * ldb;
    return a_ext < lim && b_ext < lim && M < lim && N < lim && K < lim;
}

inline P8ConvProblem p8_gemm_problem(int transA, int transB, int M, int N, int K, const void* A, int lda, const void* B, int ldb, int64_t ldc) {
    P8ConvProblem p;
    p.M = M; p.N = N; p.K = K; p.transposed = 0;
    p.A.base = (const uint8_t*)A; p.A.rows = M; p.A.K = K; p.A.LY = 1; p.A.LX = 1;
    p.A.row = affine(1, 1, transA ? 1 : lda, 0, 0, 0, 0, 0, 0, 0, 0, 0);
    p.A.k = affine(1, 1, transA ? lda : 1, 0, 0, 0, 0, 0, 0, 0, 0, 0);
    p.B.base = (const uint8_t*)B; p.B.rows = N; p.B.K = K; p.B.LY = 1; p.B.LX = 1;
    p.B.row = affine(1, 1, transB ? ldb : 1, 0, 0, 0, 0, 0, 0, 0, 0, 0);
    p.B.k = affine(1, 1, transB ? 1 : ldb, 0, 0, 0, 0, 0, 0, 0, 0, 0);
    p.out.md = make_fastdiv(1); p.out.m1 = ldc; p.out.m0 = 0; p.out.nstride = 1;
    p.Mw = M; p.Nw = N;
    return p;
}

// defined in api_conv.hip (the only translation unit that instantiates p8_conv_kernel)
hipError_t p8_conv_launch_rowmajor(hipStream_t st, const P8ConvProblem& p, const uint8_t* bias, void* C, int fout, void* wsp,
                                   const GemmPlan& plan, int64_t ld);
hipError_t p8_conv_launch_nchw(hipStream_t st, const P8ConvProblem& p, const uint8_t* bias, void* C, int fout, void* wsp,
                               const GemmPlan& plan, int64_t spatial, int64_t channels);

}  // namespace pnn
