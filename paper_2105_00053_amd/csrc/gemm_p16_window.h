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
// works through its part of the reduction in chunks of 1024 steps and empties the buckets into the quire limbs of
// the outputs after each.
//
// Every other finite operand (an *outlier*: long-regime values near minpos or maxpos) is staged as zero in the
// decoded arrays and marked in a bitmap per row of A and per column of B (one bit per reduction index).  With
// A = Am + Ao and B = Bm + Bo:  A B = Am Bm + Ao B + Am Bo.  The first term is the bucket product; the owner of an
// output adds the other two after the loop, straight into the quire limbs with the integer multiply-accumulate of
// Arith<posit<16,1>>, from the raw patterns: for every marked k of its row of A the product with B[k][n] (main or
// not), and for every marked k of its column of B the product with A[m][k] unless that is an outlier too (already
// taken).  The workgroup gathers the outliers of its tile and their partners into LDS together (bitmaps, patterns
// and partners are three sweeps of independent loads, not one dependent chain per output).  NaR is a NaN in the decoded arrays and raises the row / column flag when staged, as in gemm_bucket_pre.h.
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
#include "p16_window_arith.h"

namespace pnn {

constexpr int PW_TILE = 32;  // outputs per tile edge
constexpr int PW_KT = 32;    // reduction steps per staged slice

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

// Integer-staged operand of the correction products; `main_only` turns an outlier into a zero (its products are
// taken from its own bitmap entry instead).
__device__ __forceinline__ uint32_t pw_stage_int(uint32_t p, bool main_only) {
    if (p == 0 || p == P16::NAR) return 0u;
    bool neg;
    uint32_t sig;
    int sh;
    decode_fixed<P16>(p, neg, sig, sh);
    if (main_only && (sh < PW_LO || sh + 32 - clz32(sig) > PW_HI)) return 0u;
    const int32_t v = neg ? -(int32_t)sig : (int32_t)sig;
    return ((uint32_t)sh << 16) | ((uint32_t)v & 0xFFFFu);  // the layout of Arith<P16>::Elem
}

constexpr int PW_CAP = 224;  // outliers of one tile handled per pass of the correction

// LDS of the correction phase, laid over the staging buffers once the main loop is done.
struct PwFix {
    uint32_t part[PW_CAP][PW_TILE];  // partner operands of entry e: the 32 columns of B (row outlier) or rows of A (column outlier)
    uint32_t own[PW_CAP];            // the outlier itself
    uint32_t ent[PW_CAP];            // line << 16 | k - kbeg; lines 0..31 are rows of the tile, 32..63 its columns
    int next[PW_CAP];                // entries of one line are chained: head[line] -> next[] -> ... -> -1
    int head[2 * PW_TILE];
    int count;
    int remaining;
};

// CHUNKED: the workgroup's part of the reduction may exceed PW_MAXK steps (otherwise the planner guarantees one chunk).
template <bool CHUNKED>
__global__ __launch_bounds__(256, 4) void pw_gemm_kernel(PwGemm g) {
    typedef Arith<P16> AI;
    typedef BucketAccum<P16> AR;
    constexpr int T = PW_TILE, KT = PW_KT, KPER = KT / 4;
    constexpr int CH = KT * T / 2 / 256;  // 16-byte runs per thread, operand and slice
    static_assert(CH == 2, "two runs per thread");
    __shared__ __align__(16) double staging[2][2][KT][T];  // [operand][buffer][k][row or column]
    __shared__ uint32_t rowNaR[T];
    __shared__ uint32_t colNaR[T];
    static_assert(sizeof(staging) >= 4 * 64 * 8 * sizeof(double), "the partial buckets of a quarter of the tile fit the staging buffer");
    static_assert(sizeof(staging) >= sizeof(PwFix), "so do the lists of the correction phase");
    double (*As)[KT][T] = staging[0];
    double (*Bs)[KT][T] = staging[1];

    const int tid = threadIdx.x;
    const int lane = tid & 63, w = tid >> 6;
    const int lx = lane & 7, ly = lane >> 3;
    const int64_t tile = blockIdx.x;
    const int64_t m0 = (tile / g.tiles_n) * T, n0 = (tile % g.tiles_n) * T;
    const int64_t kbeg = (int64_t)blockIdx.z * g.kq, kend = kbeg + g.kq;

    if (tid < T) rowNaR[tid] = 0;
    else if (tid < 2 * T) colNaR[tid - T] = 0;

    double bk[4][4][2];
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

    // The lane's four final outputs are (row, col .. col + 3) of the tile.  Their quire limbs exist in registers only
    // between the end of a chunk's main loop and the end of its corrections; from one chunk to the next they rest in
    // the workspace (the slot of this slice of the reduction, which also is where a split reduction leaves them).
    const int row = ly * 4 + w, col = lx * 4;
    const int64_t m = m0 + row, n = n0 + col;
    const int64_t z = blockIdx.z;
    uint32_t* lim = g.ws.limbs ? g.ws.limbs + z * g.M * g.N * 4 : nullptr;
    PwFix& fx = *reinterpret_cast<PwFix*>(&staging[0][0][0][0]);
    auto rawA = [&](int64_t r, int64_t k) -> uint32_t { return g.transA ? g.A[k * g.lda + r] : g.A[r * g.lda + k]; };
    auto rawB = [&](int64_t k, int64_t c) -> uint32_t { return g.transB ? g.B[c * g.ldb + k] : g.B[k * g.ldb + c]; };

    __syncthreads();  // flags initialised before any stage() raises one
    // The reduction in chunks of at most PW_MAXK products: buckets, meeting in LDS, flush into the limbs, corrections.
    for (int64_t c0 = kbeg; c0 < kend; c0 += CHUNKED ? (int64_t)PW_MAXK : g.kq) {
        const int64_t c1 = (CHUNKED && c0 + PW_MAXK < kend) ? c0 + PW_MAXK : kend;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) bk[i][j][0] = bk[i][j][1] = 0.0;
        fetch(c0);
        stage(0);
        __syncthreads();
        int cur = 0;
        for (int64_t k0 = c0; k0 < c1; k0 += KT, cur ^= 1) {
            const bool more = k0 + KT < c1;
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
        double* red = &staging[0][0][0][0];
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

        // This lane now owns the outputs (row, col .. col + 3) of the tile: buckets into limbs.  (The buckets of a NaR
        // output hold NaNs and leave garbage in its limbs; the flags decide that output.)
        uint32_t q[4][4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const bool resume = CHUNKED && c0 != kbeg && m < g.M && n + j < g.N;  // limbs of the chunks before this one
#pragma unroll
            for (int l = 0; l < 4; ++l) q[j][l] = resume ? lim[(m * g.N + n + j) * 4 + l] : 0u;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (i != w) continue;
#pragma unroll
            for (int j = 0; j < 4; ++j) pw_flush(q[j], bk[i][j][0], bk[i][j][1]);
        }

        // Outlier products of this tile over [c0, c1).  All 256 threads read the bitmaps of the 32 rows and 32
        // columns (four threads per line, up to eight words each), list the marked (line, k) in LDS, fetch and decode
        // every outlier and its 32 partners in one sweep of independent loads, and then each lane walks the chain of
        // its row and of its four columns.  More outliers than the list holds take further passes.
        const int line = tid >> 2, sub = tid & 3;
        const int nwords = (int)((c1 - c0) / 32);
        uint32_t wb[8];
        {
            const uint32_t* bits = line < T ? g.bitsA + (m0 + line) * g.words : g.bitsB + (n0 + line - T) * g.words;
            bits += c0 / 32;
#pragma unroll
            for (int i = 0; i < 8; ++i) wb[i] = (sub + 4 * i < nwords) ? bits[sub + 4 * i] : 0u;
        }
        for (;;) {
            if (tid < 2 * T) fx.head[tid] = -1;
            if (tid == 0) {
                fx.count = 0;
                fx.remaining = 0;
            }
            __syncthreads();
            bool full = false;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                while (wb[i] != 0 && !full) {
                    const int slot = atomicAdd(&fx.count, 1);
                    if (slot >= PW_CAP) {
                        full = true;
                        break;
                    }
                    const int b = __ffs((int)wb[i]) - 1;
                    wb[i] &= wb[i] - 1;
                    fx.ent[slot] = ((uint32_t)line << 16) | (uint32_t)((sub + 4 * i) * 32 + b);
                    fx.next[slot] = atomicExch(&fx.head[line], slot);
                }
            }
            if (full) fx.remaining = 1;  // every writer stores the same value
            __syncthreads();
            const int listed = fx.count < PW_CAP ? fx.count : PW_CAP;
            for (int item = tid; item < listed * (T + 1); item += 256) {
                const int e = item / (T + 1), c = item % (T + 1);
                const uint32_t en = fx.ent[e];
                const int ln = (int)(en >> 16);
                const int64_t k = c0 + (int64_t)(en & 0xFFFFu);
                uint32_t v;
                if (ln < T) {  // outlier of A at (m0 + ln, k): partners are B[k][n0 ..], whatever they hold
                    if (c == T) v = pw_stage_int(rawA(m0 + ln, k), false);
                    else v = (n0 + c < g.N) ? pw_stage_int(rawB(k, n0 + c), false) : 0u;
                } else {       // outlier of B at (k, n0 + ln - T): partners are the main operands A[m0 ..][k]
                    if (c == T) v = pw_stage_int(rawB(k, n0 + ln - T), false);
                    else v = (m0 + c < g.M) ? pw_stage_int(rawA(m0 + c, k), true) : 0u;
                }
                if (c == T) fx.own[e] = v;
                else fx.part[e][c] = v;
            }
            __syncthreads();
            for (int e = fx.head[row]; e >= 0; e = fx.next[e]) {
                const uint32_t a = fx.own[e];
#pragma unroll
                for (int j = 0; j < 4; ++j) AI::mac(q[j], a, fx.part[e][col + j]);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j)
                for (int e = fx.head[T + col + j]; e >= 0; e = fx.next[e]) AI::mac(q[j], fx.part[e][row], fx.own[e]);
            const int again = fx.remaining;
            __syncthreads();
            if (!again) break;
        }

        bool nar[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) nar[j] = (rowNaR[row] | colNaR[col + j]) != 0;
        const bool last = !CHUNKED || c1 == kend;
        if (m < g.M) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (n + j >= g.N) continue;
                if (!last || gridDim.z > 1) {
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
    }

    if (gridDim.z > 1) {  // flags of this slice of the reduction, as quire_gemm_kernel stores them
        if (n0 == 0 && tid < T && m0 + tid < g.M) g.ws.rowflag[z * g.M + m0 + tid] = rowNaR[tid];
        if (m0 == 0 && tid < T && n0 + tid < g.N) g.ws.colflag[z * g.N + n0 + tid] = colNaR[tid];
    }
}

// ---- host side ----

struct PwPlan {
    GemmPlan gemm;  // splits, k per split (a multiple of PW_KT), workspace bytes in all
    int64_t Mp, Np, Kp;
    size_t b_off, bits_a_off, bits_b_off, split_off;  // byte offsets inside the workspace (decoded A at 0)
};

inline bool pw_fits(int64_t M, int64_t N, int64_t K) {
    return M >= 96 && N >= 96 && K >= 64 && M < ((int64_t)1 << 31) && N < ((int64_t)1 << 31) && K < ((int64_t)1 << 31);
}

inline PwPlan pw_plan(int64_t M, int64_t N, int64_t K) {
    PwPlan p;
    const int64_t tiles = ((M + PW_TILE - 1) / PW_TILE) * ((N + PW_TILE - 1) / PW_TILE);
    // One chunk of PW_MAXK steps per workgroup where that takes at most 8 slices of the reduction (partial quires
    // through the workspace, one merge launch); longer reductions are cut 8 ways and each workgroup works through
    // its slice chunk by chunk.
    int64_t splits = (K + PW_MAXK - 1) / PW_MAXK;
    if (splits > 8) splits = 8;
    if (tiles * splits < 768) {  // fewer workgroups than the chip holds at once: cut the reduction further, down to 128 steps
        int64_t more = (1024 + tiles * splits - 1) / (tiles * splits);
        const int64_t by_k = K / splits / 128;
        if (more > by_k) more = by_k;
        if (more > 8) more = 8;
        if (more > 1) splits *= more;
    }
    int64_t kq = (K + splits - 1) / splits;
    kq = (kq + PW_KT - 1) / PW_KT * PW_KT;
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
    // partial quires: one set per slice of a split reduction; a workgroup that works through several chunks parks its limbs there too
    const bool parks = splits > 1 || kq > PW_MAXK;
    p.gemm.ws_bytes = p.split_off + (parks ? (size_t)splits * ((size_t)M * N * 4 + M + N) * sizeof(uint32_t) : 0);
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
    if (p.gemm.splits > 1 || p.gemm.k_per_split > PW_MAXK) {
        g.ws.limbs = (uint32_t*)(base + p.split_off);
        g.ws.rowflag = g.ws.limbs + (size_t)p.gemm.splits * M * N * 4;
        g.ws.colflag = g.ws.rowflag + (size_t)p.gemm.splits * M;
    }
    const int64_t tiles_m = (M + PW_TILE - 1) / PW_TILE, tiles_n = (N + PW_TILE - 1) / PW_TILE;
    g.tiles_n = (int)tiles_n;
    const dim3 grid((unsigned)(tiles_m * tiles_n), 1, (unsigned)p.gemm.splits);
    if (p.gemm.k_per_split > PW_MAXK) hipLaunchKernelGGL(pw_gemm_kernel<true>, grid, dim3(256), 0, st, g);
    else hipLaunchKernelGGL(pw_gemm_kernel<false>, grid, dim3(256), 0, st, g);
    PNN_CHECK_LAUNCH();
    if (p.gemm.splits > 1) {
        RowMajorOut out{ldc};
        return launch_split_merge<P16, RowMajorOut>(st, g.ws, p.gemm.splits, M, N, bias, C, fout, out);
    }
    return hipSuccess;
}

}  // namespace pnn
