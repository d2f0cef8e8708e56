// posit<8,0> convolution from pre-decoded operands (paper Sec. 3.1 / 3.3: convolution
// layers, forward and both backward passes, accumulated in the 32-bit quire of Table 1).
//
// In the implicit GEMM every element of the image operand is staged once per filter tap
// and per column tile, and each staging repeats the same work: bounds tests for the zero
// padding and the table decode of the pattern.  Here a cheap first kernel rewrites both
// operands ONCE into the workspace as decoded 16-bit integers (value / minpos, |v| <= 4096;
// NaR becomes the marker -32768) in a layout where nothing is left to test:
//   image operands get their zero border written out, with a row pitch that is a multiple of 8;
//   matrix operands get a row pitch padded with zeros to a multiple of 32;
//   the backward-data weights are transposed to [c][(ko,r,s)] on the way (their NaR entries become
//   zeros: which outputs such a weight makes NaR depends on the tap, see bwd_data_nar_weights_kernel).
// The main kernel then fetches 16-byte runs (8 consecutive rows at one k, or 8 consecutive k
// of one row) with no predicate other than "row / k inside the problem", and stages them with
// at most one permute per 32-bit LDS word.  A marker never needs removing: it raises the NaR
// flag of its row (column), and every output of that row (column) is NaR whatever its
// accumulator holds.
#pragma once

#include "conv_p8.h"

namespace pnn {

constexpr uint32_t P8_NAR_MARK = 0x8000u;  // int16 -32768: no posit<8,0> decodes to it

// ---- first kernel: decode (and pad / transpose) an operand into int16 ----

// dst is [rows][pitch] int16; element (row, col) comes from src[offset(row, col)] or is zero.
//  IMAGE: row = (plane, yp), col = xp:  y = yp - pad_t, x = xp - pad_l inside [0,H) x [0,W) -> plane*H*W + y*W + x
//  ROWS:  col < K -> row*K + col
//  WT:    backward-data weights, row = c, col = ko*RS + rs < K -> (ko*C + row)*RS + rs
enum P8PreKind { P8_PRE_NONE = 0, P8_PRE_IMAGE = 1, P8_PRE_ROWS = 2, P8_PRE_WT = 3 };

struct P8PreJob {
    int kind;
    const uint8_t* src;
    uint16_t* dst;
    int rows, pitch;           // dst shape
    int H, W, Hp, pad_t, pad_l;  // IMAGE (rows = planes * Hp)
    int K, C, RS;              // ROWS / WT
    int aligned;               // src is 4-byte aligned: runs of 8 source bytes are fetched as aligned words
    FastDiv by_groups, by_hp;  // divisions by pitch / 8 and by Hp
};

__global__ __launch_bounds__(256) void p8_predecode_kernel(P8PreJob j0, P8PreJob j1) {
    __shared__ uint16_t tab[256];
    const P8PreJob& job = blockIdx.y == 0 ? j0 : j1;
    const int t = threadIdx.x;
    tab[t] = t == 0x80 ? (uint16_t)P8_NAR_MARK : (uint16_t)Arith<P8>::stage((uint32_t)t);
    __syncthreads();
    if (job.kind == P8_PRE_NONE) return;
    const int groups = job.pitch / 8;
    const uint32_t total = (uint32_t)job.rows * (uint32_t)groups;  // rows * pitch < 2^30 is checked on the host
    for (uint32_t w = blockIdx.x * 256u + t; w < total; w += gridDim.x * 256u) {
        const int row = (int)job.by_groups.div(w), c0 = (int)(w - (uint32_t)row * (uint32_t)groups) * 8;
        uint32_t d[4] = {0, 0, 0, 0};
        if (job.kind == P8_PRE_IMAGE || job.kind == P8_PRE_ROWS) {
            // the 8 source bytes are consecutive: positions [jlo, jhi) of them exist
            int64_t line;
            int x0, width;
            bool live = true;
            if (job.kind == P8_PRE_IMAGE) {
                const int plane = (int)job.by_hp.div((uint32_t)row), y = row - plane * job.Hp - job.pad_t;
                live = (uint32_t)y < (uint32_t)job.H;
                line = ((int64_t)plane * job.H + y) * job.W;
                x0 = c0 - job.pad_l;
                width = job.W;
            } else {
                line = (int64_t)row * job.K;
                x0 = c0;
                width = job.K;
            }
            int jlo = x0 < 0 ? -x0 : 0, jhi = width - x0 < 8 ? width - x0 : 8;
            if (!live || jhi <= jlo) { jlo = 0; jhi = 0; }
            uint32_t lo = 0, hi = 0;
            if (job.aligned && line + x0 + 8 < ((int64_t)1 << 31) && line + x0 > -((int64_t)1 << 31)) {
                p8_load_run8(job.src, (int)(line + x0), jlo, jhi, lo, hi);
            } else {
                for (int e = jlo; e < jhi; ++e) {
                    const uint32_t b = job.src[line + x0 + e];
                    if (e < 4) lo |= b << (8 * e); else hi |= b << (8 * (e - 4));
                }
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t b = ((e < 4 ? lo : hi) >> (8 * (e & 3))) & 0xFFu;
                const uint32_t v = (e >= jlo && e < jhi) ? tab[b] : 0u;
                d[e >> 1] |= v << (16 * (e & 1));
            }
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int col = c0 + e;
                uint32_t v = 0;
                if (col < job.K) {
                    const int ko = col / job.RS, rs = col - ko * job.RS;
                    const uint32_t b = job.src[((int64_t)ko * job.C + row) * job.RS + rs];
                    v = b == 0x80u ? 0u : tab[b];  // a NaR weight of this pass is a zero here: the outputs it reaches are marked afterwards
                }
                d[e >> 1] |= v << (16 * (e & 1));
            }
        }
        *reinterpret_cast<uint4*>(job.dst + (int64_t)row * job.pitch + c0) = make_uint4(d[0], d[1], d[2], d[3]);
    }
}

// ---- main kernel ----

// An operand of the main kernel: element (row, k) is the int16 at base[rowpart(row) + kpart(k)].
// rows_run: the 8 rows of an aligned group are 8 consecutive elements (else the 8 k of an aligned group are).
struct P16Operand {
    const uint16_t* base;
    AffineIndex row, k;
    int rows_run;
    // k runs over a padded width (backward-weight, image operand): only columns < kvalid of it are terms of the
    // reduction, and what the buffer holds beyond them (neighbouring data) is cleared when fetched; 0: no such columns
    int kvalid;
};

struct __attribute__((packed, aligned(2))) P16Run {  // 8 consecutive int16, two-byte aligned
    uint32_t w[4];
};

struct P16Frag {
    uint32_t w[8];
};

// true when one of the two 16-bit halves of some word is the NaR marker: valid values keep bits 15
// and 14 equal (|v| <= 4096), the marker alone has bit 15 set and bit 14 clear
__device__ __forceinline__ uint32_t p16_marks(uint32_t w) { return w & ~(w << 1) & 0x80008000u; }

// BR rows x 32 k of one operand, 32 bytes per work item.
//  rows_run: item w handles k-pair w / (BR/8) and rows 8*(w % (BR/8)) .. +7 (words 0..3: the 8 rows at the
//            even k, words 4..7: at the odd k);
//  else:     item w handles row w % BR and the 16 k starting at 16*(w / BR) (words in k order).
template <int BR>
struct P16Stage {
    static constexpr int GROUPS = BR / 8;
    static constexpr int ITEMS = 2 * BR;
    static constexpr int PER_THREAD = (ITEMS + 255) / 256;

    // rpart[r] / kpart[k]: element offset of row r of the tile / of reduction index k of the slice, or -1 outside the problem
    __device__ __forceinline__ static void fetch(const P16Operand& op, const int* __restrict__ rpart, const int* __restrict__ kpart,
                                                 int t, P16Frag (&f)[PER_THREAD]) {
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            const int w = t + 256 * i;
#pragma unroll
            for (int q = 0; q < 8; ++q) f[i].w[q] = 0;
            if (ITEMS % 256 != 0 && w >= ITEMS) continue;
            int r, k[2];
            if (op.rows_run) {
                r = rpart[(w % GROUPS) * 8];
                k[0] = kpart[2 * (w / GROUPS)];
                k[1] = kpart[2 * (w / GROUPS) + 1];
            } else {
                r = rpart[w % BR];
                k[0] = kpart[16 * (w / BR)];
                k[1] = kpart[16 * (w / BR) + 8];
            }
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                if (r < 0 || k[h] < 0) continue;
                const P16Run v = *reinterpret_cast<const P16Run*>(op.base + r + k[h]);
#pragma unroll
                for (int q = 0; q < 4; ++q) f[i].w[4 * h + q] = v.w[q];
            }
        }
    }

    // kvalid / kcol: see P16Operand::kvalid; the clearing is done here, where the fetched words are first
    // used, so that the loads of fetch() stay in flight during the multiply-accumulate loop
    template <int LD>
    __device__ __forceinline__ static void stage(P16Frag (&f)[PER_THREAD], uint32_t (*dst)[LD], uint32_t* flags, int t, int rows_run,
                                                 int kvalid, const int* __restrict__ kcol) {
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            const int w = t + 256 * i;
            if (ITEMS % 256 != 0 && w >= ITEMS) continue;
            if (kvalid && !rows_run) {
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int live = kvalid - kcol[16 * (w / BR) + 8 * h];  // leading elements of the run that are terms
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int left = live - 2 * q;  // elements 2q, 2q+1 of the run
                        if (left < 2) f[i].w[4 * h + q] = left == 1 ? (f[i].w[4 * h + q] & 0xFFFFu) : 0u;
                    }
                }
            }
            uint32_t marks = 0;
#pragma unroll
            for (int q = 0; q < 8; ++q) marks |= p16_marks(f[i].w[q]);
            if (!rows_run) {
                const int row = w % BR, kq = w / BR;
#pragma unroll
                for (int q = 0; q < 8; ++q) dst[8 * kq + q][row] = f[i].w[q];  // word q = (k, k+1) pair 8*kq + q
                if (marks) flags[row] = 1;
                continue;
            }
            const int kp = w / GROUPS, c = (w % GROUPS) * 8;
            uint32_t d[8];
#pragma unroll
            for (int q = 0; q < 4; ++q) {  // rows 2q, 2q+1: low halves from the even k, high halves from the odd k
                const uint32_t e = f[i].w[q], o = f[i].w[4 + q];
                d[2 * q] = (e & 0xFFFFu) | (o << 16);
                d[2 * q + 1] = (e >> 16) | (o & 0xFFFF0000u);
            }
            *reinterpret_cast<uint4*>(&dst[kp][c]) = make_uint4(d[0], d[1], d[2], d[3]);
            *reinterpret_cast<uint4*>(&dst[kp][c + 4]) = make_uint4(d[4], d[5], d[6], d[7]);
            if (marks) {
#pragma unroll
                for (int q = 0; q < 8; ++q)
                    if (p16_marks(d[q])) flags[c + q] = 1;
            }
        }
    }
};

__device__ __forceinline__ void p16_fill_kpart(const P16Operand& op, int* kpart, int* kcol, int k0, int kend, int lane) {
    const int k = k0 + lane;
    int part = -1, y, x = 0;
    if (k < kend) op.k.eval((uint32_t)k, part, y, x);
    kpart[lane] = part;
    kcol[lane] = x;  // column within the padded width (meaningful when op.kvalid is set)
}

template <int TY, int TX, int TM, int TN>
__global__ __launch_bounds__(256, 3) void p8_conv_pre_kernel(P16Operand A, P16Operand B, P8ConvOut out, const uint8_t* __restrict__ bias,
                                                             void* __restrict__ C, int fout, int M, int N, int K, int k_per_split,
                                                             int tiles_n, SplitWs ws, int ws_transposed) {
    static_assert(TY * TX == 256 && (TM == 4 || TM == 8) && (TN == 4 || TN == 8), "tile shape");
    constexpr int BM = TY * TM, BN = TX * TN;
    typedef P16Stage<BM> SA;
    typedef P16Stage<BN> SB;
    __shared__ __attribute__((aligned(16))) uint32_t As[2][P8_KP][BM];
    __shared__ __attribute__((aligned(16))) uint32_t Bs[2][P8_KP][BN];
    __shared__ int rpartA[BM];
    __shared__ int rpartB[BN];
    __shared__ int kpartA[2][P8_KT];  // slice kt uses kpart[kt & 1], filled two iterations ahead
    __shared__ int kpartB[2][P8_KT];
    __shared__ int kcolA[2][P8_KT];
    __shared__ int kcolB[2][P8_KT];
    __shared__ uint16_t tab[256];     // for the bias only
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
        int part = -1, y, x;
        if (m0 + r < M) A.row.eval((uint32_t)(m0 + r), part, y, x);
        rpartA[r] = part;
        rowNaR[r] = 0;
    }
    for (int r = t; r < BN; r += 256) {
        int part = -1, y, x;
        if (n0 + r < N) B.row.eval((uint32_t)(n0 + r), part, y, x);
        rpartB[r] = part;
        colNaR[r] = 0;
    }

    int32_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = 0;

    const int nkt = (kend - kbeg + P8_KT - 1) / P8_KT;
    const int tb = (SA::ITEMS < 256) ? ((t + 128) & 255) : t;  // B's items start on the threads A leaves idle
    if (t < P8_KT) p16_fill_kpart(A, kpartA[0], kcolA[0], kbeg, kend, t);
    else if (t < 2 * P8_KT) p16_fill_kpart(B, kpartB[0], kcolB[0], kbeg, kend, t - P8_KT);
    __syncthreads();
    {
        P16Frag fa[SA::PER_THREAD], fb[SB::PER_THREAD];
        if (nkt > 0) {
            SA::fetch(A, rpartA, kpartA[0], t, fa);
            SB::fetch(B, rpartB, kpartB[0], tb, fb);
            if (nkt > 1) {
                if (t < P8_KT) p16_fill_kpart(A, kpartA[1], kcolA[1], kbeg + P8_KT, kend, t);
                else if (t < 2 * P8_KT) p16_fill_kpart(B, kpartB[1], kcolB[1], kbeg + P8_KT, kend, t - P8_KT);
            }
            SA::template stage<BM>(fa, As[0], rowNaR, t, A.rows_run, A.kvalid, kcolA[0]);
            SB::template stage<BN>(fb, Bs[0], colNaR, tb, B.rows_run, B.kvalid, kcolB[0]);
        }
    }
    __syncthreads();

    for (int kt = 0; kt < nkt; ++kt) {
        const int cur = kt & 1;
        const bool more = kt + 1 < nkt;
        P16Frag fa[SA::PER_THREAD], fb[SB::PER_THREAD];
        if (more) {
            SA::fetch(A, rpartA, kpartA[cur ^ 1], t, fa);
            SB::fetch(B, rpartB, kpartB[cur ^ 1], tb, fb);
        }
        if (kt + 2 < nkt) {  // kpart[cur] was last read when slice kt was fetched, one barrier ago
            const int k2 = kbeg + (kt + 2) * P8_KT;
            if (t < P8_KT) p16_fill_kpart(A, kpartA[cur], kcolA[cur], k2, kend, t);
            else if (t < 2 * P8_KT) p16_fill_kpart(B, kpartB[cur], kcolB[cur], k2, kend, t - P8_KT);
        }
        // register fragments of k-pair kp + 1 are read from LDS while the dot products of k-pair kp issue
        uint32_t a[2][TM], b[2][TN];
        auto load_frag = [&](int kp, int buf) {
#pragma unroll
            for (int q = 0; q < TM / 4; ++q) {
                const uint4 v = *reinterpret_cast<const uint4*>(&As[cur][kp][q * (TY * 4) + ty * 4]);
                a[buf][4 * q] = v.x; a[buf][4 * q + 1] = v.y; a[buf][4 * q + 2] = v.z; a[buf][4 * q + 3] = v.w;
            }
#pragma unroll
            for (int q = 0; q < TN / 4; ++q) {
                const uint4 v = *reinterpret_cast<const uint4*>(&Bs[cur][kp][q * (TX * 4) + tx * 4]);
                b[buf][4 * q] = v.x; b[buf][4 * q + 1] = v.y; b[buf][4 * q + 2] = v.z; b[buf][4 * q + 3] = v.w;
            }
        };
        auto multiply = [&](int buf) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] = dot2_acc(a[buf][i], b[buf][j], acc[i][j]);
        };
        load_frag(0, 0);
#pragma unroll 1
        for (int kp = 0; kp < P8_KP - 2; kp += 2) {
            load_frag(kp + 1, 1);
            multiply(0);
            load_frag(kp + 2, 0);
            multiply(1);
        }
        load_frag(P8_KP - 1, 1);
        multiply(0);
        multiply(1);
        if (more) {
            SA::template stage<BM>(fa, As[cur ^ 1], rowNaR, t, A.rows_run, A.kvalid, kcolA[cur ^ 1]);
            SB::template stage<BN>(fb, Bs[cur ^ 1], colNaR, tb, B.rows_run, B.kvalid, kcolB[cur ^ 1]);
        }
        __syncthreads();
    }
    p8_conv_epilogue<TY, TX, TM, TN>(acc, out, bias, C, fout, M, N, m0, n0, ws, ws_transposed, tab, rowNaR, colNaR);
}

// ---- host side ----

struct P8PrePlan {
    bool ok;               // this pass and geometry can use the pre-decoded path
    bool padded_rows;      // some rows of the kernel's problem are padding (no split reduction then)
    P8PreJob job[2];       // operand A, operand B (src / dst filled at launch)
    P16Operand A, B;       // bases filled at launch
    size_t bytes[2];       // workspace bytes of the two rewritten operands (each a multiple of 256)
    P8ConvOut out;
    int M, N, K, transposed;
    int64_t Mw, Nw;
};

inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// which: 0 forward, 1 backward-data, 2 backward-weight (computed transposed), as in p8_problem.
// Needs unit stride.  So that aligned groups of 8 rows (or of 8 reduction indices) are runs in
// memory whatever the image width, the index that runs over output columns (forward,
// backward-weight) or input columns (backward-data) runs over a width rounded up to a multiple
// of 8: the extra columns read zeros or neighbouring data from the padded buffers, add nothing
// to a reduction (the other operand is zero there) and are skipped when outputs are stored
// (padded_rows: such rows exist, and a split reduction, whose partials are laid out by row, is
// not offered).
inline P8PrePlan p8_pre_plan(int which, const ConvGeom& g) {
    P8PrePlan p;
    p.ok = false;
    p.padded_rows = false;
    if (g.sh != 1 || g.sw != 1 || !p8_conv_fits(g)) return p;
    if (g.N <= 0 || g.C <= 0 || g.K <= 0) return p;  // an empty operand: nothing to rewrite, the gathered kernel copes
    const int OHW = g.OH * g.OW, HW = g.H * g.W, RS = g.R * g.S, CRS = g.C * RS;
    const int64_t lim = ((int64_t)1 << 30);
    P8PreJob& ja = p.job[0];
    P8PreJob& jb = p.job[1];
    ja = P8PreJob{};
    jb = P8PreJob{};
    p.out.wpad = 0; p.out.wvalid = 0; p.out.wd = make_fastdiv(1);
    p.A.kvalid = 0;
    p.B.kvalid = 0;
    if (which == 0) {
        // x with its zero border: Hp = H + 2 ph rows; columns up to OWq - 1 + S - 1 are read
        const int OWq = (int)round_up((size_t)g.OW, 8);
        const int Hp = g.H + 2 * g.ph;
        const int need = g.W + 2 * g.pw > OWq + g.S - 1 ? g.W + 2 * g.pw : OWq + g.S - 1;
        const int Wp = (int)round_up((size_t)need, 8);
        if ((int64_t)g.N * g.C * Hp * Wp >= lim || (int64_t)g.N * g.OH * OWq >= lim) return p;
        ja.kind = P8_PRE_IMAGE; ja.rows = g.N * g.C * Hp; ja.pitch = Wp; ja.H = g.H; ja.W = g.W; ja.Hp = Hp; ja.pad_t = g.ph; ja.pad_l = g.pw;
        const int Kp = (int)round_up((size_t)CRS, 32);
        jb.kind = P8_PRE_ROWS; jb.rows = g.K; jb.pitch = Kp; jb.K = CRS;
        p.M = g.N * g.OH * OWq; p.N = g.K; p.K = CRS; p.transposed = 0;
        p.padded_rows = OWq != g.OW;
        // rows (n, oh, owq) -> n*C*Hp*Wp + oh*Wp + owq ; k (c, r, s) -> c*Hp*Wp + r*Wp + s
        p.A.row = affine(g.OH, OWq, g.C * Hp * Wp, Wp, 1, 0, 0, 0, 0, 0, 0, 0);
        p.A.k = affine(g.R, g.S, Hp * Wp, Wp, 1, 0, 0, 0, 0, 0, 0, 0);
        p.A.rows_run = 1;
        p.B.row = affine(1, 1, Kp, 0, 0, 0, 0, 0, 0, 0, 0, 0);
        p.B.k = affine(1, 1, 1, 0, 0, 0, 0, 0, 0, 0, 0, 0);
        p.B.rows_run = 0;
        p.out.md = make_fastdiv(g.OH * OWq); p.out.m1 = (int64_t)g.K * OHW; p.out.m0 = 1; p.out.nstride = OHW;
        p.out.vec4 = g.OW % 4 == 0;
        if (p.padded_rows) { p.out.wpad = 1; p.out.wvalid = g.OW; p.out.wd = make_fastdiv(OWq); }
    } else if (which == 1) {
        // dx[h,w] reads dy[h + ph - r, w + pw - s]: border of R-1-ph rows and S-1-pw columns (a negative one is a crop: not handled here)
        const int bt = g.R - 1 - g.ph, bl = g.S - 1 - g.pw;
        if (bt < 0 || bl < 0) return p;
        const int Wq = (int)round_up((size_t)g.W, 8);
        const int Hp = g.OH + 2 * bt;
        const int need = g.OW + 2 * bl > Wq + g.S - 1 ? g.OW + 2 * bl : Wq + g.S - 1;
        const int Wp = (int)round_up((size_t)need, 8);
        if (Hp < g.H + g.R - 1) return p;  // every tap of every row must land inside
        if ((int64_t)g.N * g.K * Hp * Wp >= lim || (int64_t)g.N * g.H * Wq >= lim) return p;
        ja.kind = P8_PRE_IMAGE; ja.rows = g.N * g.K * Hp; ja.pitch = Wp; ja.H = g.OH; ja.W = g.OW; ja.Hp = Hp; ja.pad_t = bt; ja.pad_l = bl;
        const int Kd = g.K * RS, Kp = (int)round_up((size_t)Kd, 32);
        jb.kind = P8_PRE_WT; jb.rows = g.C; jb.pitch = Kp; jb.K = Kd; jb.C = g.C; jb.RS = RS;
        p.M = g.N * g.H * Wq; p.N = g.C; p.K = Kd; p.transposed = 0;
        p.padded_rows = Wq != g.W;
        // rows (n, h, wq) -> n*K*Hp*Wp + h*Wp + wq ; k (ko, r, s) -> ko*Hp*Wp + (R-1-r)*Wp + (S-1-s)
        p.A.row = affine(g.H, Wq, g.K * Hp * Wp, Wp, 1, 0, 0, 0, 0, 0, 0, 0);
        p.A.k = affine(g.R, g.S, Hp * Wp, -Wp, -1, (g.R - 1) * Wp + (g.S - 1), 0, 0, 0, 0, 0, 0);
        p.A.rows_run = 1;
        p.B.row = affine(1, 1, Kp, 0, 0, 0, 0, 0, 0, 0, 0, 0);
        p.B.k = affine(1, 1, 1, 0, 0, 0, 0, 0, 0, 0, 0, 0);
        p.B.rows_run = 0;
        p.out.md = make_fastdiv(g.H * Wq); p.out.m1 = (int64_t)g.C * HW; p.out.m0 = 1; p.out.nstride = HW;
        p.out.vec4 = g.W % 4 == 0;
        if (p.padded_rows) { p.out.wpad = 1; p.out.wvalid = g.W; p.out.wd = make_fastdiv(Wq); }
    } else {
        const int OWq = (int)round_up((size_t)g.OW, 8);
        const int Hp = g.H + 2 * g.ph;
        const int need = g.W + 2 * g.pw > OWq + g.S - 1 ? g.W + 2 * g.pw : OWq + g.S - 1;
        const int Wp = (int)round_up((size_t)need, 8);
        if ((int64_t)g.N * g.C * Hp * Wp >= lim) return p;
        ja.kind = P8_PRE_IMAGE; ja.rows = g.N * g.C * Hp; ja.pitch = Wp; ja.H = g.H; ja.W = g.W; ja.Hp = Hp; ja.pad_t = g.ph; ja.pad_l = g.pw;
        // dy as [n][ko][oh][owq], zero beyond the real width: the reduction index (n, oh, owq) runs over the padded width
        if ((int64_t)g.N * g.K * g.OH * OWq >= lim) return p;
        jb.kind = P8_PRE_IMAGE; jb.rows = g.N * g.K * g.OH; jb.pitch = OWq; jb.H = g.OH; jb.W = g.OW; jb.Hp = g.OH; jb.pad_t = 0; jb.pad_l = 0;
        p.M = CRS; p.N = g.K; p.K = g.N * g.OH * OWq; p.transposed = 1;
        // rows (c, r, s) -> c*Hp*Wp + r*Wp + s ; k (n, oh, owq) -> n*C*Hp*Wp + oh*Wp + owq
        p.A.row = affine(g.R, g.S, Hp * Wp, Wp, 1, 0, 0, 0, 0, 0, 0, 0);
        p.A.k = affine(g.OH, OWq, g.C * Hp * Wp, Wp, 1, 0, 0, 0, 0, 0, 1, 0);  // x = owq, the column within the padded width
        p.A.rows_run = 0;
        p.A.kvalid = OWq != g.OW ? g.OW : 0;
        const int OHWq = g.OH * OWq;
        p.B.row = affine(1, 1, OHWq, 0, 0, 0, 0, 0, 0, 0, 0, 0);
        p.B.k = affine(OHWq, 1, g.K * OHWq, 1, 0, 0, 0, 0, 0, 0, 0, 0);
        p.B.rows_run = 0;
        p.out.md = make_fastdiv(1); p.out.m1 = 1; p.out.m0 = 0; p.out.nstride = CRS; p.out.vec4 = 0;
    }
    // a run may start up to 31 elements before the end of the last row and always reads 8: keep 64 bytes of slack
    if ((int64_t)ja.rows * ja.pitch >= lim || (int64_t)jb.rows * jb.pitch >= lim) return p;
    for (P8PreJob* j : {&ja, &jb}) {
        j->by_groups = make_fastdiv((uint32_t)(j->pitch / 8));
        j->by_hp = make_fastdiv((uint32_t)(j->kind == P8_PRE_IMAGE && j->Hp > 0 ? j->Hp : 1));
    }
    p.bytes[0] = round_up((size_t)ja.rows * ja.pitch * 2 + 64, 256);
    p.bytes[1] = round_up((size_t)jb.rows * jb.pitch * 2 + 64, 256);
    p.Mw = p.transposed ? p.N : p.M;
    p.Nw = p.transposed ? p.M : p.N;
    p.ok = true;
    return p;
}

}  // namespace pnn
