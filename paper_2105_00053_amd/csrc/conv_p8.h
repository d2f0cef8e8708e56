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

// How the staging code may fetch an operand.  GENERIC: one byte at a time, each with its own
// address and bounds test.  ROW_RUN: the 8 rows of an aligned group sit at 8 consecutive bytes
// (same y, x advancing by xstep = 0 or 1), as for the image operand of the forward and
// backward-data passes at unit stride.  K_RUN: the same along the reduction index, as for
// weights, k-contiguous matrices and both operands of the backward-weight pass at unit stride.
// A run is fetched as aligned 32-bit words and trimmed to the positions inside the bounds.
enum P8GatherMode { P8_GENERIC = 0, P8_ROW_RUN = 1, P8_K_RUN = 2 };

struct P8Gather {
    const uint8_t* base;
    int rows, K;     // extents of the virtual matrix
    int LY, LX;      // bounds for y and x
    int mode, xstep; // P8GatherMode; x advance along a run
    int quiet_nar;   // NaR patterns of this operand count as zero and raise no row / column flag (the weights of
                     // the backward-data pass, whose NaR entries reach only part of a channel: marked by a kernel of their own)
    AffineIndex row, k;
};

constexpr int OUT_OF_RANGE = -(1 << 28);  // a y that can never pass the bounds test

struct P8ConvOut {
    // element index of output (m, n) = mpart(m) + n * nstride, mpart affine in m's coordinates
    FastDiv md;          // m = c1 * md.d + c0
    int64_t m1, m0;      // mpart = c1 * m1 + c0 * m0
    int64_t nstride;
    int vec4;            // rows 4q .. 4q+3 of one column are four consecutive bytes at a multiple of four
    // rows laid out over a padded width: c0 = r * wd.d + col, only col < wvalid exists and then
    // c0 stands for r * wvalid + col (wpad = 0: c0 is used as it is)
    int wpad, wvalid;
    FastDiv wd;
    // the part of the index that depends on the row; -1: the row is padding and has no output element
    PNN_HD int64_t row_part(int m) const {
        const uint32_t c1 = md.div((uint32_t)m);
        uint32_t c0 = (uint32_t)m - c1 * md.d;
        if (wpad) {
            const uint32_t r = wd.div(c0), col = c0 - r * wd.d;
            if (col >= (uint32_t)wvalid) return -1;
            c0 = r * (uint32_t)wvalid + col;
        }
        return (int64_t)c1 * m1 + (int64_t)c0 * m0;
    }
    PNN_HD int64_t at(int m, int n) const {
        const int64_t rp = row_part(m);
        return rp < 0 ? -1 : rp + (int64_t)n * nstride;
    }
};

// Positions [jlo, jhi) of an 8-long run that lie inside the bounds: the run's first element has
// coordinates (y, xs), x advances by xstep, at most jmax positions exist.
__device__ __forceinline__ void p8_run_window(int y, int xs, int xstep, int jmax, int LY, int LX, int& jlo, int& jhi) {
    const bool yok = (uint32_t)y < (uint32_t)LY;
    if (xstep) {
        jlo = xs < 0 ? -xs : 0;
        jhi = LX - xs < jmax ? LX - xs : jmax;
    } else {
        jlo = 0;
        jhi = ((uint32_t)xs < (uint32_t)LX) ? jmax : 0;
    }
    if (!yok) jhi = 0;
    if (jhi <= jlo) { jlo = 0; jhi = 0; }
}

// The 8 bytes at byte offset `off` of `base` (4-byte aligned), positions outside [jlo, jhi) zeroed.
// Only aligned 32-bit words that hold a wanted byte are read (the others are re-pointed at the
// first wanted word, or at the start of the tensor when nothing is wanted), so no access leaves
// the words the tensor itself occupies.
__device__ __forceinline__ void p8_load_run8(const uint8_t* __restrict__ base, int off, int jlo, int jhi, uint32_t& lo, uint32_t& hi) {
    const bool any = jlo < jhi;
    const int wfirst = any ? ((off + jlo) & ~3) : 0, wlast = any ? ((off + jhi - 1) & ~3) : -4;
    const int a4 = off & ~3;
    uint32_t d[3];
#pragma unroll
    for (int i = 0; i < 3; ++i) {
        const int wa = a4 + 4 * i;
        const bool need = wa >= wfirst && wa <= wlast;
        const uint32_t v = *reinterpret_cast<const uint32_t*>(base + (need ? wa : wfirst));
        d[i] = need ? v : 0u;
    }
    const uint32_t sh = (uint32_t)off & 3u;
    const uint32_t l = __builtin_amdgcn_alignbyte(d[1], d[0], sh);  // bytes off .. off+3
    const uint32_t h = __builtin_amdgcn_alignbyte(d[2], d[1], sh);  // bytes off+4 .. off+7
    const uint64_t keep = any ? ((~0ull >> (8 * (8 - jhi))) & (~0ull << (8 * jlo))) : 0ull;
    lo = l & (uint32_t)keep;
    hi = h & (uint32_t)(keep >> 32);
}

// One operand slice: BR rows x 32 k, 16 bytes per work item.  GENERIC and ROW_RUN: item w handles
// k-pair w / (BR/8) and rows 8*(w % (BR/8)) .. +7 (frag words 2h, 2h+1 = the 8 rows at k-half h).
// K_RUN: item w handles row w % BR and the 16 k starting at 16*(w / BR) (frag words in k order).
// `tshift` rotates the thread-to-item map so that a short operand does not share threads with
// the other operand's items.
template <int BR>
struct P8GatherStage {
    static constexpr int GROUPS = BR / 8;
    static constexpr int ITEMS = GROUPS * P8_KP;  // = 2 * BR
    static constexpr int PER_THREAD = (ITEMS + 255) / 256;

    // fetch the 16 bytes of every work item of this thread; kinfo = (part, y, x) of the slice's 32 k
    __device__ __forceinline__ static void fetch(const P8Gather& op, const int4* __restrict__ rinfo, const int4* __restrict__ kinfo,
                                                 int k0, int kend, int rows_in_tile, int t, P8Frag (&f)[PER_THREAD]) {
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            const int w = t + 256 * i;
            f[i].w[0] = f[i].w[1] = f[i].w[2] = f[i].w[3] = 0;
            if (ITEMS % 256 != 0 && w >= ITEMS) continue;
            if (op.mode == P8_K_RUN) {
                const int row = w % BR, kq = w / BR;
                const int4 ri = rinfo[row];
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int kl = 16 * kq + 8 * h;
                    const int4 ki = kinfo[kl];
                    const int left = kend - (k0 + kl);
                    int jlo, jhi;
                    p8_run_window(ri.y + ki.y, ri.z + ki.z, op.xstep, left < 8 ? left : 8, op.LY, op.LX, jlo, jhi);
                    p8_load_run8(op.base, ri.x + ki.x, jlo, jhi, f[i].w[2 * h], f[i].w[2 * h + 1]);
                }
                continue;
            }
            const int kp = w / GROUPS, g = w % GROUPS;
            if (op.mode == P8_ROW_RUN) {
                const int4 ri = rinfo[g * 8];
                const int left = rows_in_tile - g * 8;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int4 ki = kinfo[2 * kp + h];
                    int jlo, jhi;
                    p8_run_window(ri.y + ki.y, ri.z + ki.z, op.xstep, left < 8 ? left : 8, op.LY, op.LX, jlo, jhi);
                    p8_load_run8(op.base, ri.x + ki.x, jlo, jhi, f[i].w[2 * h], f[i].w[2 * h + 1]);
                }
                continue;
            }
            const int4 k0i = kinfo[2 * kp], k1i = kinfo[2 * kp + 1];
            const int kpart[2] = {k0i.x, k1i.x}, ky[2] = {k0i.y, k1i.y}, kx[2] = {k0i.z, k1i.z};
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

    // decode + pack + store into dst[k-pair][row]; flags[row] for NaR (flags may be null: NaR is then just a zero)
    template <int LD>
    __device__ __forceinline__ static void stage(const P8Frag (&f)[PER_THREAD], uint32_t (*dst)[LD], const uint16_t* tab,
                                                 uint32_t* flags, int t, int mode) {
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            const int w = t + 256 * i;
            if (ITEMS % 256 != 0 && w >= ITEMS) continue;
            const uint32_t nar = nar_bytes(f[i].w[0]) | nar_bytes(f[i].w[1]) | nar_bytes(f[i].w[2]) | nar_bytes(f[i].w[3]);
            if (mode == P8_K_RUN) {
                const int row = w % BR, kq = w / BR;
#pragma unroll
                for (int j = 0; j < 8; ++j) {  // bytes 2j, 2j+1 of the 16 are k-pair 8*kq + j
                    const uint32_t word = f[i].w[j >> 1] >> (16 * (j & 1));
                    dst[8 * kq + j][row] = (uint32_t)tab[word & 0xFFu] | ((uint32_t)tab[(word >> 8) & 0xFFu] << 16);
                }
                if (nar && flags) flags[row] = 1;
                continue;
            }
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

// (part, y, x) of the 32 reduction indices of the slice starting at k0; beyond kend: never in bounds
__device__ __forceinline__ void p8_fill_kinfo(const P8Gather& op, int4* kinfo, int k0, int kend, int lane) {
    const int k = k0 + lane;
    int4 ki = make_int4(0, OUT_OF_RANGE, 0, 0);
    if (k < kend) op.k.eval((uint32_t)k, ki.x, ki.y, ki.z);
    kinfo[lane] = ki;
}

// Epilogue shared by the convolution kernels: add the bias, round each 32-bit quire once and
// store it (or park the partial quire and the NaR flags of a split reduction in the workspace).
// Thread (ty, tx) owns rows (i>>2)*(TY*4) + ty*4 + (i&3) and columns (j>>2)*(TX*4) + tx*4 + (j&3).
// With out.vec4 set, the four rows i&3 = 0..3 of one column land on four consecutive bytes that
// start at a multiple of four, and posit<8,0> results are stored as one 32-bit word.
template <int TY, int TX, int TM, int TN>
__device__ __forceinline__ void p8_conv_epilogue(const int32_t (&acc)[TM][TN], const P8ConvOut& out, const uint8_t* __restrict__ bias,
                                                 void* __restrict__ C, int fout, int M, int N, int m0, int n0, const SplitWs& ws,
                                                 int ws_transposed, const uint16_t* tab, const uint32_t* rowNaR, const uint32_t* colNaR) {
    const int t = threadIdx.x;
    const int tx = t % TX, ty = t / TX;
    constexpr int BM = TY * TM, BN = TX * TN;
    if (gridDim.z == 1 && fout == 0 && out.vec4) {
#pragma unroll
        for (int ig = 0; ig < TM / 4; ++ig) {
            const int lr = ig * (TY * 4) + ty * 4;
            const int m = m0 + lr;
            if (m >= M) continue;  // M is a multiple of four here: the four rows are all inside or all outside
            const int64_t rp = out.row_part(m);
            if (rp < 0) continue;  // so are the four columns of a padded width (a multiple of four too)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int lc = (j >> 2) * (TX * 4) + tx * 4 + (j & 3);
                const int n = n0 + lc;
                if (n >= N) continue;
                int32_t badd = 0;
                bool cnar = colNaR[lc] != 0;
                if (bias) {
                    const uint32_t bp = bias[n];
                    if (bp == 0x80u) cnar = true;
                    else badd = (int32_t)(int16_t)tab[bp] << P8::MAXS;
                }
                uint32_t word = 0;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const bool nar = cnar || rowNaR[lr + r] != 0;
                    word |= (nar ? 0x80u : p8_round_quire(acc[ig * 4 + r][j] + badd)) << (8 * r);
                }
                *reinterpret_cast<uint32_t*>((uint8_t*)C + rp + (int64_t)n * out.nstride) = word;
            }
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int lr = (i >> 2) * (TY * 4) + ty * 4 + (i & 3);
        const int m = m0 + lr;
        if (m >= M) continue;
        const bool rnar = rowNaR[lr] != 0;
        const int64_t rp = gridDim.z == 1 ? out.row_part(m) : 0;
        if (rp < 0) continue;
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
                const int64_t at = rp + (int64_t)n * out.nstride;
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
    __shared__ int4 kinfoA[2][P8_KT];  // slice kt uses kinfo[kt & 1], filled two iterations ahead
    __shared__ int4 kinfoB[2][P8_KT];
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
    uint32_t* const aflags = A.quiet_nar ? nullptr : rowNaR;
    uint32_t* const bflags = B.quiet_nar ? nullptr : colNaR;
    // B's work items start on the threads that A's leave idle when A has fewer items than threads
    const int tb = (SA::ITEMS < 256) ? ((t + 128) & 255) : t;
    if (t < P8_KT) p8_fill_kinfo(A, kinfoA[0], kbeg, kend, t);
    else if (t < 2 * P8_KT) p8_fill_kinfo(B, kinfoB[0], kbeg, kend, t - P8_KT);
    __syncthreads();
    {
        P8Frag fa[SA::PER_THREAD], fb[SB::PER_THREAD];
        if (nkt > 0) {
            SA::fetch(A, rinfoA, kinfoA[0], kbeg, kend, M - m0, t, fa);
            SB::fetch(B, rinfoB, kinfoB[0], kbeg, kend, N - n0, tb, fb);
            if (nkt > 1) {
                if (t < P8_KT) p8_fill_kinfo(A, kinfoA[1], kbeg + P8_KT, kend, t);
                else if (t < 2 * P8_KT) p8_fill_kinfo(B, kinfoB[1], kbeg + P8_KT, kend, t - P8_KT);
            }
            SA::template stage<BM>(fa, As[0], tab, aflags, t, A.mode);
            SB::template stage<BN>(fb, Bs[0], tab, bflags, tb, B.mode);
        }
    }
    __syncthreads();

    for (int kt = 0; kt < nkt; ++kt) {
        const int cur = kt & 1;
        const bool more = kt + 1 < nkt;
        P8Frag fa[SA::PER_THREAD], fb[SB::PER_THREAD];
        if (more) {
            const int k0 = kbeg + (kt + 1) * P8_KT;
            SA::fetch(A, rinfoA, kinfoA[cur ^ 1], k0, kend, M - m0, t, fa);
            SB::fetch(B, rinfoB, kinfoB[cur ^ 1], k0, kend, N - n0, tb, fb);
        }
        if (kt + 2 < nkt) {  // kinfo[cur] was last read when slice kt was fetched, one barrier ago
            const int k2 = kbeg + (kt + 2) * P8_KT;
            if (t < P8_KT) p8_fill_kinfo(A, kinfoA[cur], k2, kend, t);
            else if (t < 2 * P8_KT) p8_fill_kinfo(B, kinfoB[cur], k2, kend, t - P8_KT);
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
            SA::template stage<BM>(fa, As[cur ^ 1], tab, aflags, t, A.mode);
            SB::template stage<BN>(fb, Bs[cur ^ 1], tab, bflags, tb, B.mode);
        }
        __syncthreads();
    }

    p8_conv_epilogue<TY, TX, TM, TN>(acc, out, bias, C, fout, M, N, m0, n0, ws, ws_transposed, tab, rowNaR, colNaR);
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

// x advance (0 or 1) when every aligned group of 8 consecutive indices maps to 8 consecutive bytes
// at one y; -1 when the index does not run through memory that way.
inline int affine_run_step(const AffineIndex& a) {
    if (a.d0.d % 8 == 0) return (a.part0 == 1 && a.y0 == 0 && (a.x0 == 0 || a.x0 == 1)) ? a.x0 : -1;
    if (a.d0.d != 1) return -1;
    if (a.d1d0.d % 8 == 0) return (a.part1 == 1 && a.y1 == 0 && (a.x1 == 0 || a.x1 == 1)) ? a.x1 : -1;
    if (a.d1d0.d == 1) return a.part2 == 1 ? 0 : -1;  // single index: y and x do not depend on it
    return -1;
}

// Choose the cheapest fetch the operand's layout allows (word loads need a 4-byte aligned tensor).
inline void p8_pick_mode(P8Gather& op) {
    op.mode = P8_GENERIC;
    op.xstep = 0;
    if (((uintptr_t)op.base & 3u) != 0) return;
    const int ks = affine_run_step(op.k), rs = affine_run_step(op.row);
    if (ks >= 0) { op.mode = P8_K_RUN; op.xstep = ks; }
    else if (rs >= 0) { op.mode = P8_ROW_RUN; op.xstep = rs; }
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
        p.out.md = make_fastdiv(OHW); p.out.m1 = (int64_t)g.K * OHW; p.out.m0 = 1; p.out.nstride = OHW; p.out.vec4 = OHW % 4 == 0; p.out.wpad = 0; p.out.wvalid = 0; p.out.wd = make_fastdiv(1);
    } else if (which == 1) {  // t0 = dy, t1 = w ; stride 1 only
        p.M = g.N * HW; p.N = g.C; p.K = g.K * RS; p.transposed = 0;
        p.A.base = (const uint8_t*)t0; p.A.rows = p.M; p.A.K = p.K; p.A.LY = g.OH; p.A.LX = g.OW;
        p.A.row = affine(g.H, g.W, g.K * OHW, g.OW, 1, g.ph * g.OW + g.pw, 1, 0, g.ph, 0, 1, g.pw);
        p.A.k = affine(g.R, g.S, OHW, -g.OW, -1, 0, -1, 0, 0, 0, -1, 0);
        p.B.base = (const uint8_t*)t1; p.B.rows = p.N; p.B.K = p.K; p.B.LY = 1; p.B.LX = 1;
        p.B.row = affine(1, 1, RS, 0, 0, 0, 0, 0, 0, 0, 0, 0);
        p.B.k = affine(RS, 1, CRS, 1, 0, 0, 0, 0, 0, 0, 0, 0);
        p.out.md = make_fastdiv(HW); p.out.m1 = (int64_t)g.C * HW; p.out.m0 = 1; p.out.nstride = HW; p.out.vec4 = HW % 4 == 0; p.out.wpad = 0; p.out.wvalid = 0; p.out.wd = make_fastdiv(1);
    } else {  // t0 = dy, t1 = x ; computed transposed: rows (c,r,s), columns ko
        p.M = CRS; p.N = g.K; p.K = g.N * OHW; p.transposed = 1;
        p.A.base = (const uint8_t*)t1; p.A.rows = p.M; p.A.K = p.K; p.A.LY = g.H; p.A.LX = g.W;
        p.A.row = affine(g.R, g.S, HW, g.W, 1, -g.ph * g.W - g.pw, 1, 0, -g.ph, 0, 1, -g.pw);
        p.A.k = affine(g.OH, g.OW, g.C * HW, g.sh * g.W, g.sw, 0, g.sh, 0, 0, 0, g.sw, 0);
        p.B.base = (const uint8_t*)t0; p.B.rows = p.N; p.B.K = p.K; p.B.LY = 1; p.B.LX = 1;
        p.B.row = affine(1, 1, OHW, 0, 0, 0, 0, 0, 0, 0, 0, 0);
        p.B.k = affine(OHW, 1, g.K * OHW, 1, 0, 0, 0, 0, 0, 0, 0, 0);
        p.out.md = make_fastdiv(1); p.out.m1 = 1; p.out.m0 = 0; p.out.nstride = CRS; p.out.vec4 = 0; p.out.wpad = 0; p.out.wvalid = 0; p.out.wd = make_fastdiv(1);
    }
    p.Mw = p.transposed ? p.N : p.M;
    p.Nw = p.transposed ? p.M : p.N;
    p.A.quiet_nar = 0;
    p.B.quiet_nar = which == 1;  // backward-data: a NaR weight reaches only the positions its tap reaches
    p8_pick_mode(p.A);
    p8_pick_mode(p.B);
    return p;
}

// Workgroup tile (rows x columns of the virtual GEMM).  Larger tiles reuse staged
// operands more; smaller ones give the 256 CUs enough workgroups on the small
// layers.  Pick the largest tile that still yields >= 512 workgroups (counting the
// reduction split), else the one with the most workgroups.
struct P8ConvTile { int bm, bn; };
static const P8ConvTile P8_CONV_TILES[] = {{128, 128}, {256, 64}, {256, 32}, {128, 64}, {64, 64}, {128, 32}};

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
        // workgroups once the reduction is split the way plan_split() will (at least 256 steps per slice, at most 256 slices)
        int64_t slices = 1;
        if (can_split && blocks < 1024) {
            slices = (1024 + blocks - 1) / blocks;
            if (slices > K / 256) slices = K / 256;
            if (slices > 256) slices = 256;
        }
        const int64_t workgroups = blocks * slices;
        const double fill = workgroups >= 1024 ? 1.0 : (double)workgroups / 1024.0;  // four waves per SIMD
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
    p.out.md = make_fastdiv(1); p.out.m1 = ldc; p.out.m0 = 0; p.out.nstride = 1; p.out.vec4 = 0; p.out.wpad = 0; p.out.wvalid = 0; p.out.wd = make_fastdiv(1);
    p.Mw = M; p.Nw = N;
    p.A.quiet_nar = 0; p.B.quiet_nar = 0;
    p8_pick_mode(p.A);
    p8_pick_mode(p.B);
    return p;
}

// defined in api_conv.hip (the only translation unit that instantiates p8_conv_kernel)
hipError_t p8_conv_launch_rowmajor(hipStream_t st, const P8ConvProblem& p, const uint8_t* bias, void* C, int fout, void* wsp,
                                   const GemmPlan& plan, int64_t ld);
hipError_t p8_conv_launch_nchw(hipStream_t st, const P8ConvProblem& p, const uint8_t* bias, void* C, int fout, void* wsp,
                               const GemmPlan& plan, int64_t spatial, int64_t channels);

}  // namespace pnn
