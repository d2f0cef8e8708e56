// posit<16,1> matrix product with a 128-bit quire (paper Sec. 2, Table 1; Sec. 3.3): two fp64 buckets for the
// operands of ordinary magnitude, an exact integer correction for the rest.
//
// Scaled by 2^28 every posit<16,1> is an integer of at most 2^56, so products span 112 bits and the general
// bucket accumulate (BucketArith) needs three doubles per output and nine fp64 operations per product.  Almost all
// operands of real tensors sit in a much narrower band.  An operand is called *main* when its scaled value is a
// multiple of 2^LO below 2^HI (LO = 4, HI = 47: magnitudes from about 2^-23 to 2^18); products of two main operands
// are multiples of 2^(2 LO) below 2^(2 HI), an 86-bit span that two doubles cover with ten guard bits each:
//     h = fma(a, b, C) - C, C = 1.5 * 2^(52+T1), T1 = 51:  the product rounded to a multiple of 2^T1, |h| <= 2^94
//     r = fma(a, b, -h):  the rest, a multiple of 2^8 with |r| <= 2^50, exact
//     hi += h (multiples of 2^51, exact up to 2^104: 1024 products);  lo += r (multiples of 2^8, exact up to 2^61: 2048)
// -- five fp64 operations per product and 4 registers per output instead of nine and 6.  A workgroup therefore
// adds at most 1024 products into the buckets of one output (the planner cuts longer reductions over gridDim.z).
//
// Every other finite operand (an *outlier*: long-regime values near minpos or maxpos) is staged as zero in the
// decoded arrays and marked in a bitmap per row of A and per column of B (one bit per reduction index).  With
// A = Am + Ao and B = Bm + Bo:  A B = Am Bm + Ao B + Am Bo.  The first term is the bucket product; the owner of an
// output adds the other two after the loop, straight into the quire limbs with the integer multiply-accumulate of
// Arith<posit<16,1>>, reading the raw patterns: for every marked k of its row of A the product with B[k][n] (main or
// not), and for every marked k of its column of B the product with A[m][k] unless that is marked too (already
// taken).  NaR is a NaN in the decoded arrays and raises the row / column flag when staged, as in gemm_bucket_pre.h.
// The result is the exact quire sum for any input; only the time depends on the share of outliers (about 80
// lane-operations per outlier product against 5 per main product).
//
// Work distribution: 32 x 32 output tiles; the four waves of a workgroup all work on the same tile, each lane on a
// 4 x 4 block of it, each wave on a quarter of every staged slice of the reduction; the partial buckets meet in LDS
// (exact: the sum of the four partial bucket sums is the bucket sum of the whole slice) in such a way that every
// wave ends up owning one row of each lane's block, so the flush, the corrections and the rounding are spread
// over all four waves.  1024 x 1024 outputs are 1024 workgroups = four waves per SIMD with no second launch.
#pragma once

#include "gemm_bucket_pre.h"

namespace pnn {

constexpr int PW_LO = 4, PW_HI = 47;      // main operands: multiples of 2^LO below 2^HI (units of minpos = 2^-28)
constexpr int PW_T1 = 51;                 // the cut between the two buckets
constexpr int PW_MAXK = 1024;             // products per output between two flushes
constexpr int PW_TILE = 32;               // outputs per tile edge
constexpr int PW_KT = 32;                 // reduction steps per staged slice
static_assert(2 * PW_HI + 10 <= 53 + PW_T1, "hi bucket: 1024 products of at most 2^(2 HI), multiples of 2^T1");
static_assert(PW_T1 - 1 + 10 <= 53 + 2 * PW_LO, "lo bucket: 1024 rests of at most 2^(T1-1), multiples of 2^(2 LO)");
static_assert(2 * PW_HI <= PW_T1 + 51 && PW_T1 - 2 * PW_LO <= 53, "the cut itself is exact");

// Scaled value of a pattern as the product kernel wants it: main operands as they are, outliers and zero as 0.0,
// NaR as a NaN.  Returns true for an outlier.
PNN_HD bool pw_classify(uint32_t p, double& v) {
    v = 0.0;
    if (p == 0) return false;
    if (p == P16::NAR) {
        v = __builtin_bit_cast(double, (uint64_t)0x7FF8000000000000ull);
        return false;
    }
    bool neg;
    uint32_t sig;
    int sh;
    decode_fixed<P16>(p, neg, sig, sh);
    // sig < 2^13 holds the significand with all its fraction bits: value = sig * 2^sh, below 2^(sh + bit length of sig)
    const int top = sh + 32 - clz32(sig);
    if (sh < PW_LO || top > PW_HI) return true;
    const double m = __builtin_ldexp((double)(int32_t)sig, sh);
    v = neg ? -m : m;
    return false;
}

PNN_HD void pw_mac(double& hi, double& lo, double a, double b) {
    constexpr double C = 1.5 * pow2d(52 + PW_T1);
    const double h = __builtin_fma(a, b, C) - C;
    hi += h;
    lo += __builtin_fma(a, b, -h);
}

// The two buckets of an output into its (zeroed or partial) quire limbs.
PNN_HD void pw_flush(uint32_t (&q)[4], double hi, double lo) {
    quire_add_double<4, PW_T1>(q, hi);
    quire_add_double<4, 2 * PW_LO>(q, lo);
}

struct PwOperand {
    const uint16_t* src;  // patterns: element (r, k) at src[r * ld + k] (kfast) or src[k * ld + r]
    int64_t ld, rows;
    double* dst;          // [Kp][Rp] decoded, outliers as zeros
    int64_t Rp;
    uint32_t* bits;       // [Rp][Kp / 32] outlier bitmap, bit k % 32 of word k / 32
    int kfast;
};

// Decode pass over both operands (blockIdx.z picks one): 64 x 64 element tiles.
__global__ __launch_bounds__(256) void pw_predecode_kernel(PwOperand opa, PwOperand opb, int64_t K, int64_t Kp) {
    constexpr int PT = 64;
    __shared__ double tile[PT][PT + 1];
    __shared__ uint32_t obits[PT][2];
    const PwOperand o = blockIdx.z == 0 ? opa : opb;
    const int64_t r0 = (int64_t)blockIdx.x * PT, k0 = (int64_t)blockIdx.y * PT;
    if (r0 >= o.Rp) return;
    const int64_t words = Kp / 32;
    const int t = threadIdx.x;
    if (o.kfast) {  // a wave reads 64 consecutive k of one row: the outlier bits of that row come from one ballot
#pragma unroll 4
        for (int i = 0; i < PT * PT / 256; ++i) {
            const int e = t + 256 * i;
            const int kk = e % PT, rr = e / PT;
            const int64_t r = r0 + rr, k = k0 + kk;
            double v = 0.0;
            bool out = false;
            if (r < o.rows && k < K) out = pw_classify(o.src[r * o.ld + k], v);
            tile[kk][rr] = v;
            const uint64_t mask = __ballot(out);
            if (kk == 0 && k0 < Kp) o.bits[r * words + k0 / 32] = (uint32_t)mask;
            if (kk == 32 && k0 + 32 < Kp) o.bits[r * words + k0 / 32 + 1] = (uint32_t)(mask >> 32);
        }
        __syncthreads();
#pragma unroll 4
        for (int i = 0; i < PT * PT / 256; ++i) {
            const int e = t + 256 * i;
            const int rr = e % PT, kk = e / PT;
            if (k0 + kk < Kp) o.dst[(k0 + kk) * o.Rp + r0 + rr] = tile[kk][rr];
        }
    } else {  // a wave reads 64 consecutive rows at one k: outlier bits are collected per row in LDS
        if (t < 2 * PT) obits[t >> 1][t & 1] = 0;
        __syncthreads();
#pragma unroll 4
        for (int i = 0; i < PT * PT / 256; ++i) {
            const int e = t + 256 * i;
            const int rr = e % PT, kk = e / PT;
            const int64_t r = r0 + rr, k = k0 + kk;
            double v = 0.0;
            bool out = false;
            if (r < o.rows && k < K) out = pw_classify(o.src[k * o.ld + r], v);
            if (k < Kp) o.dst[k * o.Rp + r] = v;
            if (out) atomicOr(&obits[rr][kk >> 5], 1u << (kk & 31));
        }
        __syncthreads();
        if (t < 2 * PT) {
            const int rr = t >> 1, half = t & 1;
            if (k0 + 32 * half < Kp) o.bits[(r0 + rr) * words + k0 / 32 + half] = obits[rr][half];
        }
    }
}

struct PwGemm {
    const double* Ap;  // [Kp][Mp]
    const double* Bp;  // [Kp][Np]
    int64_t Mp, Np, kq;
    const uint32_t* bitsA;  // [Mp][words]
    const uint32_t* bitsB;  // [Np][words]
    int64_t words;
    const uint16_t* A;  // raw patterns, for the corrections
    const uint16_t* B;
    int64_t lda, ldb;
    int transA, transB;
    const uint16_t* bias;
    void* C;
    int64_t ldc;
    int fout;
    int64_t M, N;
    SplitWs ws;
    int tiles_n;
};

// Finish the four outputs (m, n .. n + 3) of one lane: buckets into limbs, outlier products of the reduction
// slice [kbeg, kend), then either the partial quire (lim) or bias, the one rounding and the store.
__device__ __forceinline__ void pw_finish(const PwGemm& g, const double (&acc)[4][2], int64_t m, int64_t n, bool rownar, const uint32_t* colnar,
                                          int64_t kbeg, int64_t kend, uint32_t* lim) {
    typedef Arith<P16> AI;
    typedef BucketAccum<P16> AR;
    if (m >= g.M) return;
    uint32_t q[4][4];
    bool nar[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        nar[j] = rownar || colnar[j] != 0;
#pragma unroll
        for (int l = 0; l < 4; ++l) q[j][l] = 0;
        if (!nar[j]) pw_flush(q[j], acc[j][0], acc[j][1]);  // a NaR output's buckets hold NaNs
    }
    auto rawA = [&](int64_t k) -> uint32_t { return g.transA ? g.A[k * g.lda + m] : g.A[m * g.lda + k]; };
    auto rawB = [&](int64_t k, int64_t nn) -> uint32_t { return g.transB ? g.B[nn * g.ldb + k] : g.B[k * g.ldb + nn]; };
    const uint32_t* ba = g.bitsA + m * g.words;
    const int64_t w0 = kbeg / 32, w1 = kend / 32;
    for (int64_t wd = w0; wd < w1; ++wd) {  // outliers of row m of A, against B whatever it holds
        uint32_t bits = ba[wd];
        while (bits) {
            const int64_t k = wd * 32 + (__ffs((int)bits) - 1);
            bits &= bits - 1;
            const uint32_t a = AI::stage(rawA(k));
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (n + j < g.N) AI::mac(q[j], a, AI::stage(rawB(k, n + j)));
        }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {  // outliers of column n + j of B, against the main operands of A
        if (n + j >= g.N) continue;
        const uint32_t* bb = g.bitsB + (n + j) * g.words;
        for (int64_t wd = w0; wd < w1; ++wd) {
            uint32_t bits = bb[wd];
            if (bits == 0) continue;
            bits &= ~ba[wd];
            while (bits) {
                const int64_t k = wd * 32 + (__ffs((int)bits) - 1);
                bits &= bits - 1;
                AI::mac(q[j], AI::stage(rawA(k)), AI::stage(rawB(k, n + j)));
            }
        }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if (n + j >= g.N) continue;
        if (lim) {
#pragma unroll
            for (int l = 0; l < 4; ++l) lim[(m * g.N + n + j) * 4 + l] = q[j][l];
        } else {
            bool isnar = nar[j];
            if (g.bias) {
                const uint32_t bp = g.bias[n + j];
                if (bp == P16::NAR) isnar = true;
                else AR::add_bias(q[j], bp);
            }
            round_store<AR, 4>(q[j], isnar, g.fout, g.C, m * g.ldc + n + j);
        }
    }
}

__global__ __launch_bounds__(256, 4) void pw_gemm_kernel(PwGemm g) {
    constexpr int T = PW_TILE, KT = PW_KT, KPER = KT / 4;
    constexpr int CH = KT * T / 2 / 256;  // 16-byte runs per thread, operand and slice
    static_assert(CH == 2, "two runs per thread");
    __shared__ __align__(16) double As[2][KT][T];
    __shared__ __align__(16) double Bs[2][KT][T];
    __shared__ uint32_t rowNaR[T];
    __shared__ uint32_t colNaR[T];
    static_assert(sizeof(As) >= 4 * 64 * 8 * sizeof(double), "the partial buckets of a quarter of the tile fit the staging buffer");

    const int tid = threadIdx.x;
    const int lane = tid & 63, w = tid >> 6;
    const int lx = lane & 7, ly = lane >> 3;
    const int64_t tile = blockIdx.x;
    const int64_t m0 = (tile / g.tiles_n) * T, n0 = (tile % g.tiles_n) * T;
    const int64_t kbeg = (int64_t)blockIdx.z * g.kq, kend = kbeg + g.kq;

    if (tid < T) rowNaR[tid] = 0;
    else if (tid < 2 * T) colNaR[tid - T] = 0;

    double bk[4][4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) bk[i][j][0] = bk[i][j][1] = 0.0;

    double2 ra[CH], rb[CH];
    auto fetch = [&](int64_t k0) {
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int c = tid + 256 * i;
            const int kk = c / (T / 2), r2 = c % (T / 2);
            ra[i] = *reinterpret_cast<const double2*>(g.Ap + (k0 + kk) * g.Mp + m0 + 2 * r2);
            rb[i] = *reinterpret_cast<const double2*>(g.Bp + (k0 + kk) * g.Np + n0 + 2 * r2);
        }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int c = tid + 256 * i;
            const int kk = c / (T / 2), r2 = c % (T / 2);
            if (ra[i].x != ra[i].x) rowNaR[2 * r2] = 1;
            if (ra[i].y != ra[i].y) rowNaR[2 * r2 + 1] = 1;
            if (rb[i].x != rb[i].x) colNaR[2 * r2] = 1;
            if (rb[i].y != rb[i].y) colNaR[2 * r2 + 1] = 1;
            *reinterpret_cast<double2*>(&As[buf][kk][2 * r2]) = ra[i];
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
        for (int s = 0; s < KPER; ++s) {
            const int kk = w * KPER + s;  // this wave's quarter of the slice
            double a[4], b[4];
            {
                const double2 v0 = *reinterpret_cast<const double2*>(&As[cur][kk][ly * 4]);
                const double2 v1 = *reinterpret_cast<const double2*>(&As[cur][kk][ly * 4 + 2]);
                a[0] = v0.x; a[1] = v0.y; a[2] = v1.x; a[3] = v1.y;
                const double2 u0 = *reinterpret_cast<const double2*>(&Bs[cur][kk][lx * 4]);
                const double2 u1 = *reinterpret_cast<const double2*>(&Bs[cur][kk][lx * 4 + 2]);
                b[0] = u0.x; b[1] = u0.y; b[2] = u1.x; b[3] = u1.y;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) pw_mac(bk[i][j][0], bk[i][j][1], a[i], b[j]);
        }
        if (more) stage(cur ^ 1);  // the other buffer was last read one barrier ago
        __syncthreads();
    }

    // The four partial tiles meet in LDS: in round p wave w hands the row (w + p) % 4 of every lane's block to the
    // wave that owns it, which adds it to its own partial sums of that row.
    double* red = &As[0][0][0];
#pragma unroll
    for (int p = 1; p < 4; ++p) {
        const int dest = (w + p) & 3;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (i != dest) continue;  // uniform over the wave
            double2* slot = reinterpret_cast<double2*>(red + ((size_t)dest * 64 + lane) * 8);
#pragma unroll
            for (int j = 0; j < 4; ++j) slot[j] = make_double2(bk[i][j][0], bk[i][j][1]);
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (i != w) continue;
            const double2* slot = reinterpret_cast<const double2*>(red + ((size_t)w * 64 + lane) * 8);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const double2 v = slot[j];
                bk[i][j][0] += v.x;
                bk[i][j][1] += v.y;
            }
        }
        __syncthreads();
    }
    double own[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (i != w) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            own[j][0] = bk[i][j][0];
            own[j][1] = bk[i][j][1];
        }
    }

    const int64_t z = blockIdx.z;
    uint32_t* lim = gridDim.z > 1 ? g.ws.limbs + z * g.M * g.N * 4 : nullptr;
    const int row = ly * 4 + w, col = lx * 4;
    pw_finish(g, own, m0 + row, n0 + col, rowNaR[row] != 0, &colNaR[col], kbeg, kend, lim);
    if (lim) {  // flags of this slice of the reduction, as quire_gemm_kernel stores them
        if (n0 == 0 && tid < T && m0 + tid < g.M) g.ws.rowflag[z * g.M + m0 + tid] = rowNaR[tid];
        if (m0 == 0 && tid < T && n0 + tid < g.N) g.ws.colflag[z * g.N + n0 + tid] = colNaR[tid];
    }
}

// ---- host side ----

struct PwPlan {
    GemmPlan gemm;  // splits, k per split (a multiple of PW_KT, at most PW_MAXK), workspace bytes in all
    int64_t Mp, Np, Kp;
    size_t b_off, bits_a_off, bits_b_off, split_off;  // byte offsets inside the workspace (decoded A at 0)
};

inline bool pw_fits(int64_t M, int64_t N, int64_t K) {
    return M >= 96 && N >= 96 && K >= 64 && M < ((int64_t)1 << 31) && N < ((int64_t)1 << 31) && K < ((int64_t)1 << 31);
}

inline PwPlan pw_plan(int64_t M, int64_t N, int64_t K) {
    PwPlan p;
    const int64_t tiles = ((M + PW_TILE - 1) / PW_TILE) * ((N + PW_TILE - 1) / PW_TILE);
    int64_t splits = (K + PW_MAXK - 1) / PW_MAXK;
    if (tiles * splits < 768) {  // fewer workgroups than the chip holds at once: cut the reduction further, down to 128 steps
        int64_t more = (1024 + tiles * splits - 1) / (tiles * splits);
        const int64_t by_k = K / splits / 128;
        if (more > by_k) more = by_k;
        if (more > 8) more = 8;
        if (more > 1) splits *= more;
    }
    int64_t kq = (K + splits - 1) / splits;
    kq = (kq + PW_KT - 1) / PW_KT * PW_KT;
    if (kq > PW_MAXK) kq = PW_MAXK;
    splits = (K + kq - 1) / kq;
    p.gemm.splits = (int)splits;
    p.gemm.k_per_split = kq;
    p.Kp = splits * kq;
    p.Mp = (M + 63) / 64 * 64;
    p.Np = (N + 63) / 64 * 64;
    p.b_off = (size_t)p.Kp * p.Mp * sizeof(double);
    p.bits_a_off = p.b_off + (size_t)p.Kp * p.Np * sizeof(double);
    p.bits_b_off = p.bits_a_off + (size_t)p.Mp * (p.Kp / 32) * sizeof(uint32_t);
    p.split_off = p.bits_b_off + (size_t)p.Np * (p.Kp / 32) * sizeof(uint32_t);
    p.split_off = (p.split_off + 15) / 16 * 16;
    p.gemm.ws_bytes = p.split_off + (splits > 1 ? (size_t)splits * ((size_t)M * N * 4 + M + N) * sizeof(uint32_t) : 0);
    return p;
}

inline hipError_t launch_pw_gemm(hipStream_t st, int transA, int transB, const void* A, int64_t lda, const void* B, int64_t ldb, const void* bias,
                                 void* C, int64_t ldc, int fout, int64_t M, int64_t N, int64_t K, void* workspace) {
    const PwPlan p = pw_plan(M, N, K);
    char* base = (char*)workspace;
    PwOperand oa{(const uint16_t*)A, lda, M, (double*)base, p.Mp, (uint32_t*)(base + p.bits_a_off), transA ? 0 : 1};
    PwOperand ob{(const uint16_t*)B, ldb, N, (double*)(base + p.b_off), p.Np, (uint32_t*)(base + p.bits_b_off), transB ? 1 : 0};
    const int64_t rmax = p.Mp > p.Np ? p.Mp : p.Np;
    hipLaunchKernelGGL(pw_predecode_kernel, dim3((unsigned)(rmax / 64), (unsigned)((p.Kp + 63) / 64), 2), dim3(256), 0, st, oa, ob, K, p.Kp);
    PNN_CHECK_LAUNCH();
    PwGemm g;
    g.Ap = oa.dst;
    g.Bp = ob.dst;
    g.Mp = p.Mp;
    g.Np = p.Np;
    g.kq = p.gemm.k_per_split;
    g.bitsA = oa.bits;
    g.bitsB = ob.bits;
    g.words = p.Kp / 32;
    g.A = (const uint16_t*)A;
    g.B = (const uint16_t*)B;
    g.lda = lda;
    g.ldb = ldb;
    g.transA = transA;
    g.transB = transB;
    g.bias = (const uint16_t*)bias;
    g.C = C;
    g.ldc = ldc;
    g.fout = fout;
    g.M = M;
    g.N = N;
    g.ws.limbs = nullptr;
    g.ws.rowflag = nullptr;
    g.ws.colflag = nullptr;
    if (p.gemm.splits > 1) {
        g.ws.limbs = (uint32_t*)(base + p.split_off);
        g.ws.rowflag = g.ws.limbs + (size_t)p.gemm.splits * M * N * 4;
        g.ws.colflag = g.ws.rowflag + (size_t)p.gemm.splits * M;
    }
    const int64_t tiles_m = (M + PW_TILE - 1) / PW_TILE, tiles_n = (N + PW_TILE - 1) / PW_TILE;
    g.tiles_n = (int)tiles_n;
    hipLaunchKernelGGL(pw_gemm_kernel, dim3((unsigned)(tiles_m * tiles_n), 1, (unsigned)p.gemm.splits), dim3(256), 0, st, g);
    PNN_CHECK_LAUNCH();
    if (p.gemm.splits > 1) {
        RowMajorOut out{ldc};
        return launch_split_merge<P16, RowMajorOut>(st, g.ws, p.gemm.splits, M, N, bias, C, fout, out);
    }
    return hipSuccess;
}

}  // namespace pnn
