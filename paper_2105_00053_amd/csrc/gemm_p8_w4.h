// posit<8,0> quire GEMM for products too small to fill the chip with 128 x 128 tiles (paper
// Sec. 3.3: quire-accumulated matrix product; Table 1: 32-bit quire).
//
// A 1024^3 product has 64 tiles of 128 x 128: a quarter of the compute units would work.  Cutting
// the reduction over workgroups fills the chip but sends every partial tile through memory and needs
// a second launch to merge them.  Here the cut is made INSIDE the workgroup instead: a workgroup
// owns a 64 x 64 tile of C, and each of its four waves computes that whole tile over its own quarter
// of the reduction, with the 8 x 8 register tile per lane and the LDS traffic per dot product of the
// large kernel (four 128-bit LDS reads feed 64 v_dot2_i32_i16).  The four partial tiles meet in LDS
// at the end (int32 addition modulo 2^32 is the quire's own arithmetic, so the order does not
// matter), every wave rounds a quarter of the outputs, and the call is one launch with no workspace.
//
// A wave stages its own 64-row x 32-k operand slices into its own LDS tiles, so the main loop has no
// workgroup barrier at all: LDS operations of one wave execute in program order, which makes the
// write of the next slice after the reads of the current one safe with a single buffer.  Global
// loads of the next slice are in flight while the current one is multiplied.
#pragma once

#include "gemm_p8.h"

namespace pnn {

constexpr int W4_T = 64;  // tile edge

struct W4Frag {
    uint32_t w[8];
};

// The 32 bytes of this lane for a 64-row x 32-k operand slice starting at (r0, k0).
//  KFAST (k contiguous):  lane = row; the 32 bytes are k0 .. k0+31 of that row.
//  else (rows contiguous): lane = (k-pair lane/4, 16 rows starting at 16*(lane%4)): w[0..3] = the rows at the even k, w[4..7] at the odd k.
// `fast`: the slice is interior and every address is 16-byte aligned; otherwise bytes are fetched one by one and read as
// zero outside [0,R) x [0,kend).
template <bool KFAST>
__device__ __forceinline__ W4Frag w4_fetch(const uint8_t* __restrict__ p, int64_t ld, int R, int r0, int k0, int kend, int lane, bool fast) {
    W4Frag f;
    if (KFAST) {
        const int row = r0 + lane;
        if (fast) {
            const uint4* q = reinterpret_cast<const uint4*>(p + (int64_t)row * ld + k0);
            const uint4 v0 = q[0], v1 = q[1];
            f.w[0] = v0.x; f.w[1] = v0.y; f.w[2] = v0.z; f.w[3] = v0.w;
            f.w[4] = v1.x; f.w[5] = v1.y; f.w[6] = v1.z; f.w[7] = v1.w;
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                uint32_t w = 0;
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const int k = k0 + 4 * i + b;
                    const uint32_t byte = (row < R && k < kend) ? p[(int64_t)row * ld + k] : 0u;
                    w |= byte << (8 * b);
                }
                f.w[i] = w;
            }
        }
    } else {
        const int k = k0 + 2 * (lane >> 2), row = r0 + (lane & 3) * 16;
        if (fast) {
            const uint4 v0 = *reinterpret_cast<const uint4*>(p + (int64_t)k * ld + row);
            const uint4 v1 = *reinterpret_cast<const uint4*>(p + (int64_t)(k + 1) * ld + row);
            f.w[0] = v0.x; f.w[1] = v0.y; f.w[2] = v0.z; f.w[3] = v0.w;
            f.w[4] = v1.x; f.w[5] = v1.y; f.w[6] = v1.z; f.w[7] = v1.w;
        } else {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    uint32_t w = 0;
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        const int r = row + 4 * i + b;
                        const uint32_t byte = (r < R && k + h < kend) ? p[(int64_t)(k + h) * ld + r] : 0u;
                        w |= byte << (8 * b);
                    }
                    f.w[4 * h + i] = w;
                }
            }
        }
    }
    return f;
}

// Decode through the LDS table and store as packed (k, k+1) pairs into dst[k-pair][row]; flags[row] for NaR.
template <bool KFAST>
__device__ __forceinline__ void w4_stage(const W4Frag& f, uint32_t (*dst)[W4_T], const uint16_t* tab, uint32_t* flags, int lane) {
    uint32_t nar = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) nar |= nar_bytes(f.w[i]);
    if (KFAST) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t w = f.w[i];
            dst[2 * i][lane] = (uint32_t)tab[w & 0xFFu] | ((uint32_t)tab[(w >> 8) & 0xFFu] << 16);
            dst[2 * i + 1][lane] = (uint32_t)tab[(w >> 16) & 0xFFu] | ((uint32_t)tab[w >> 24] << 16);
        }
        if (nar) flags[lane] = 1;
    } else {
        const int kp = lane >> 2, c = (lane & 3) * 16;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            uint32_t d[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t lo = (f.w[q] >> (8 * j)) & 0xFFu, hi = (f.w[4 + q] >> (8 * j)) & 0xFFu;
                d[j] = (uint32_t)tab[lo] | ((uint32_t)tab[hi] << 16);
            }
            *reinterpret_cast<uint4*>(&dst[kp][c + 4 * q]) = make_uint4(d[0], d[1], d[2], d[3]);
        }
        if (nar) {
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const uint32_t lo = (f.w[j >> 2] >> (8 * (j & 3))) & 0xFFu, hi = (f.w[4 + (j >> 2)] >> (8 * (j & 3))) & 0xFFu;
                if (lo == 0x80u || hi == 0x80u) flags[c + j] = 1;
            }
        }
    }
}

// kq: reduction indices per wave (a multiple of 32); wave w of workgroup z takes [(WAVES z + w) * kq, min(K, (WAVES z + w + 1) * kq)).
// With gridDim.z > 1 the workgroup's merged tile is a partial quire that goes to the workspace (layout of SplitWs) and
// split_merge_kernel finishes.  WAVES = 4 or 8: a grid that gives a compute unit a single workgroup wants the eight-wave
// form, since one wave alone on a SIMD issues at about half the rate that two or more reach together.
template <bool A_KFAST, bool B_KFAST, int WAVES>
__global__ __launch_bounds__(64 * WAVES, WAVES == 8 ? 2 : 4) void p8_gemm_w4_kernel(
    const uint8_t* __restrict__ A, int64_t lda, const uint8_t* __restrict__ B, int64_t ldb, const uint8_t* __restrict__ bias,
    void* __restrict__ C, int64_t ldc, int fout, int M, int N, int K, int kq, int tiles_m, int tiles_n, int a_aligned, int b_aligned,
    SplitWs ws) {
    static_assert(WAVES == 4 || WAVES == 8, "four or eight waves");
    // [wave][operand][k-pair][row]: 8 KB per wave, reused for the reduction of the partial tiles
    __shared__ __attribute__((aligned(16))) uint32_t tiles[WAVES][2][P8_KP][W4_T];
    __shared__ uint16_t tab[256];
    __shared__ uint32_t rowNaR[WAVES][W4_T];
    __shared__ __attribute__((aligned(16))) uint32_t colNaR[WAVES][W4_T];

    const int t = threadIdx.x;
    const int w = t >> 6, lane = t & 63;
    const int tx = lane & 7, ty = lane >> 3;
    // a row (column) is NaR when any wave met a NaR in its part of the reduction
    auto any_flag = [](const uint32_t (*flags)[W4_T], int at) {
        uint32_t f = 0;
#pragma unroll
        for (int v = 0; v < WAVES; ++v) f |= flags[v][at];
        return f;
    };

    // XCD-aware order: consecutive workgroup ids go round-robin to the 8 XCDs, so give each XCD a contiguous run of
    // tiles, walked in bands of 8 tile-rows, column by column inside a band (neighbours share operand panels in L2)
    const int nblk = tiles_m * tiles_n;
    int lid = blockIdx.x;
    if ((nblk & 7) == 0) lid = (blockIdx.x & 7) * (nblk >> 3) + (blockIdx.x >> 3);
    const int band = lid / (8 * tiles_n);
    const int band_rows = (tiles_m - band * 8) < 8 ? (tiles_m - band * 8) : 8;
    const int in_band = lid - band * 8 * tiles_n;
    const int m0 = (band * 8 + in_band % band_rows) * W4_T;
    const int n0 = (in_band / band_rows) * W4_T;

    const int kbeg = ((int)blockIdx.z * WAVES + w) * kq;
    const int kend = (kbeg + kq < K) ? kbeg + kq : K;
    const int nkt = kbeg < kend ? (kend - kbeg + P8_KT - 1) / P8_KT : 0;

    // eight waves (registers to spare): the first slice's loads are in flight while the decode table is built
    constexpr bool EARLY_FETCH = WAVES == 8;
    W4Frag fa0, fb0;
    auto fetch_first = [&]() {
        const bool kin = kbeg + P8_KT <= kend;
        fa0 = w4_fetch<A_KFAST>(A, lda, M, m0, kbeg, kend, lane, (m0 + W4_T <= M) && a_aligned && kin);
        fb0 = w4_fetch<B_KFAST>(B, ldb, N, n0, kbeg, kend, lane, (n0 + W4_T <= N) && b_aligned && kin);
    };
    if (EARLY_FETCH && nkt > 0) fetch_first();
    if (t < 256) tab[t] = (uint16_t)Arith<P8>::stage((uint32_t)t);
    rowNaR[w][lane] = 0;
    colNaR[w][lane] = 0;

    int32_t acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = 0;

    uint32_t (*As)[W4_T] = tiles[w][0];
    uint32_t (*Bs)[W4_T] = tiles[w][1];
    const bool a_rows_in = (m0 + W4_T <= M) && a_aligned;
    const bool b_rows_in = (n0 + W4_T <= N) && b_aligned;

    __syncthreads();  // table and flags ready
    if (nkt > 0) {
        if (!EARLY_FETCH) fetch_first();
        w4_stage<A_KFAST>(fa0, As, tab, rowNaR[w], lane);
        w4_stage<B_KFAST>(fb0, Bs, tab, colNaR[w], lane);
    }
    __builtin_amdgcn_wave_barrier();
    for (int kt = 0; kt < nkt; ++kt) {
        const bool more = kt + 1 < nkt;
        W4Frag fa, fb;
        if (more) {
            const int k0 = kbeg + (kt + 1) * P8_KT;
            const bool kin = k0 + P8_KT <= kend;
            fa = w4_fetch<A_KFAST>(A, lda, M, m0, k0, kend, lane, a_rows_in && kin);
            fb = w4_fetch<B_KFAST>(B, ldb, N, n0, k0, kend, lane, b_rows_in && kin);
        }
#pragma unroll 2
        for (int kp = 0; kp < P8_KP; ++kp) {
            const uint4 a0 = *reinterpret_cast<const uint4*>(&As[kp][ty * 4]);
            const uint4 a1 = *reinterpret_cast<const uint4*>(&As[kp][32 + ty * 4]);
            const uint4 b0 = *reinterpret_cast<const uint4*>(&Bs[kp][tx * 4]);
            const uint4 b1 = *reinterpret_cast<const uint4*>(&Bs[kp][32 + tx * 4]);
            const uint32_t a[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
            const uint32_t b[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[i][j] = dot2_acc(a[i], b[j], acc[i][j]);
        }
        // the wave's LDS operations execute in program order: the writes below follow the reads above
        __builtin_amdgcn_wave_barrier();
        if (more) {
            w4_stage<A_KFAST>(fa, As, tab, rowNaR[w], lane);
            w4_stage<B_KFAST>(fb, Bs, tab, colNaR[w], lane);
        }
        __builtin_amdgcn_wave_barrier();
    }

    // ---- the four partial tiles -> one: register i of a lane belongs to the wave i / 2 in the end ----
    uint32_t* red = &tiles[0][0][0][0];  // 2048 dwords per wave
    __syncthreads();                     // every wave is done with its operand tiles
    // a row (column) is NaR when any wave met a NaR in its part of the reduction: gathered into entry 0 (read again only
    // after the barriers of the reduction below)
    if (t < W4_T) rowNaR[0][t] = any_flag(rowNaR, t);
    else if (t < 2 * W4_T) colNaR[0][t - W4_T] = any_flag(colNaR, t - W4_T);
    // In the end wave w owns the registers i = w * RPW .. w * RPW + RPW - 1 of every lane's 8 x 8 block, i.e. the rows
    // (i / 4) * 32 + ty * 4 + i % 4 of the tile: one row per wave with eight waves, two with four.
    constexpr int RPW = 8 / WAVES;
    int32_t fin[RPW][8];
    auto row_of = [&](int ii) { const int i = w * RPW + ii; return (i >> 2) * 32 + ty * 4 + (i & 3); };
    if constexpr (WAVES == 8) {
        // Eight partial tiles, eight owners: in round r the waves hand their registers of rows 4r .. 4r + 3 to the
        // owners of those rows (slot (owner, writer): 8 registers x 64 lanes as two 16-byte words per lane; 28 slots of
        // 2 KB), and each owner adds the seven slots meant for it to its own registers.
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            if (r) __syncthreads();  // the owners of round 0 have read their slots
#pragma unroll
            for (int o = 0; o < 4; ++o) {
                const int i = 4 * r + o;
                if (w == i) continue;  // uniform over the wave
                const int wr = w < i ? w : w - 1;
                uint4* dst = reinterpret_cast<uint4*>(red + (o * 7 + wr) * 512) + lane;
                dst[0] = make_uint4((uint32_t)acc[i][0], (uint32_t)acc[i][1], (uint32_t)acc[i][2], (uint32_t)acc[i][3]);
                dst[64] = make_uint4((uint32_t)acc[i][4], (uint32_t)acc[i][5], (uint32_t)acc[i][6], (uint32_t)acc[i][7]);
            }
            __syncthreads();
            if ((w >> 2) != r) continue;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if (i != w) continue;
#pragma unroll
                for (int j = 0; j < 8; ++j) fin[0][j] = acc[i][j];
            }
#pragma unroll
            for (int wr = 0; wr < 7; ++wr) {
                const uint4* src = reinterpret_cast<const uint4*>(red + ((w & 3) * 7 + wr) * 512) + lane;
                const uint4 v0 = src[0], v1 = src[64];
                fin[0][0] += (int32_t)v0.x; fin[0][1] += (int32_t)v0.y; fin[0][2] += (int32_t)v0.z; fin[0][3] += (int32_t)v0.w;
                fin[0][4] += (int32_t)v1.x; fin[0][5] += (int32_t)v1.y; fin[0][6] += (int32_t)v1.z; fin[0][7] += (int32_t)v1.w;
            }
        }
    } else {
        // four partial tiles -> one: waves 2, 3 hand theirs to waves 0, 1, which then spread the quarters
        if (w >= 2 && w < 4) {
            uint32_t* dst = red + (w - 2) * 4096 + lane;
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int j = 0; j < 8; ++j) dst[(i * 8 + j) * 64] = (uint32_t)acc[i][j];
        }
        __syncthreads();
        if (w < 2) {
            const uint32_t* src = red + w * 4096 + lane;
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[i][j] += (int32_t)src[(i * 8 + j) * 64];
        }
        __syncthreads();
        // wave 0 parks the quarters 1, 2, 3 of its sum in slots 0, 1, 2 of region X; wave 1 the quarters 0, 2, 3 of its sum
        // in slots 0, 1, 2 of region Y (a slot: 16 registers x 64 lanes)
        uint32_t* X = red;
        uint32_t* Y = red + 3 * 1024;
        if (w < 2) {
#pragma unroll
            for (int qq = 0; qq < 4; ++qq) {
                if (qq == w) continue;  // own quarter stays in registers
                const int slot = (w == 0) ? qq - 1 : (qq == 0 ? 0 : qq - 1);
                uint32_t* dst = (w == 0 ? X : Y) + slot * 1024 + lane;
#pragma unroll
                for (int ii = 0; ii < 2; ++ii)
#pragma unroll
                    for (int j = 0; j < 8; ++j) dst[(ii * 8 + j) * 64] = (uint32_t)acc[2 * qq + ii][j];
            }
        }
        __syncthreads();
        {
            const int xs = w - 1;                  // slot of quarter w in X (w >= 1)
            const int ys = w == 0 ? 0 : w - 1;     // slot of quarter w in Y (w != 1)
#pragma unroll
            for (int ii = 0; ii < 2; ++ii)
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int at = (ii * 8 + j) * 64 + lane;
                    int32_t v;
                    if (w == 0) v = acc[ii][j] + (int32_t)Y[ys * 1024 + at];
                    else if (w == 1) v = acc[2 + ii][j] + (int32_t)X[xs * 1024 + at];
                    else v = (int32_t)X[xs * 1024 + at] + (int32_t)Y[ys * 1024 + at];
                    fin[ii][j] = v;
                }
        }
    }

    if (gridDim.z > 1) {  // a slice of the reduction: park the partial quires and the NaR flags of this slice
        const int64_t z = blockIdx.z;
        uint32_t* lim = ws.limbs + z * (int64_t)M * N;
#pragma unroll
        for (int ii = 0; ii < RPW; ++ii) {
            const int m = m0 + row_of(ii);
            if (m >= M) continue;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int n = n0 + (j >> 2) * 32 + tx * 4 + (j & 3);
                if (n < N) lim[(int64_t)m * N + n] = (uint32_t)fin[ii][j];
            }
        }
        // the first tile column stores the row flags of its tile row (identical in every column), the first tile row the
        // column flags: every entry is written, so the workspace needs no clearing
        if (t < W4_T) {
            if (n0 == 0 && m0 + t < M) ws.rowflag[z * M + m0 + t] = rowNaR[0][t];
        } else if (t < 2 * W4_T) {
            const int c = t - W4_T;
            if (m0 == 0 && n0 + c < N) ws.colflag[z * N + n0 + c] = colNaR[0][c];
        }
        return;
    }
    // ---- round once and store ----
    // The quires with the bias and the NaR flags first, then ONE test of the output format around the whole tile: the
    // posit<8,0> path is a compact run of code (a format test inside the loops would scatter it between sixteen copies of
    // the general encoder, and a wave pays an instruction-cache miss for every jump over one of them).
    uint32_t qv[RPW][8];
    bool narv[RPW][8];
    const uint4 c0 = *reinterpret_cast<const uint4*>(&colNaR[0][tx * 4]);
    const uint4 c1 = *reinterpret_cast<const uint4*>(&colNaR[0][32 + tx * 4]);
    const uint32_t cflag[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
#pragma unroll
    for (int ii = 0; ii < RPW; ++ii) {
        const int lr = row_of(ii);
        const bool rnar = rowNaR[0][lr] != 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int n = n0 + (j >> 2) * 32 + tx * 4 + (j & 3);
            int32_t q = fin[ii][j];
            bool nar = rnar || cflag[j] != 0;
            if (bias && n < N) {
                const uint32_t bp = bias[n];
                if (bp == 0x80u) nar = true;
                else q += (int32_t)(int16_t)tab[bp] << P8::MAXS;  // + bias * 1
            }
            narv[ii][j] = nar;
            qv[ii][j] = (uint32_t)q;
        }
    }
    if (fout == 0) {
#pragma unroll
        for (int ii = 0; ii < RPW; ++ii) {
            const int m = m0 + row_of(ii);
            if (m >= M) continue;
#pragma unroll
            for (int jh = 0; jh < 2; ++jh) {
                const int n = n0 + jh * 32 + tx * 4;
                uint32_t out[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) out[j] = narv[ii][jh * 4 + j] ? 0x80u : p8_round_quire((int32_t)qv[ii][jh * 4 + j]);
                uint8_t* crow = (uint8_t*)C + (int64_t)m * ldc + n;
                if (n + 4 <= N && (((uintptr_t)crow) & 3) == 0) {
                    *reinterpret_cast<uint32_t*>(crow) = out[0] | (out[1] << 8) | (out[2] << 16) | (out[3] << 24);
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (n + j < N) crow[j] = (uint8_t)out[j];
                }
            }
        }
    } else {
#pragma unroll
        for (int ii = 0; ii < RPW; ++ii) {
            const int m = m0 + row_of(ii);
            if (m >= M) continue;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int n = n0 + (j >> 2) * 32 + tx * 4 + (j & 3);
                if (n >= N) continue;
                const uint32_t q1[1] = {qv[ii][j]};
                round_store<QuireAccum<P8>, 1>(q1, narv[ii][j], fout, C, (int64_t)m * ldc + n);
            }
        }
    }
}

// Shapes this kernel takes: both output dimensions beyond one tile, at least one 32-wide slice for every wave, and too
// few 128 x 128 tiles for the large kernel to fill the chip without cutting the reduction across workgroups.
inline bool p8_w4_fits(int64_t M, int64_t N, int64_t K) {
    if (M <= W4_T || N <= W4_T || K < 128) return false;
    const int64_t tiles128 = ((M + P8_BM - 1) / P8_BM) * ((N + P8_BN - 1) / P8_BN);
    return tiles128 < 1024;
}

// Eight waves per workgroup when the tiles alone leave a compute unit at most one workgroup (then every SIMD still runs
// two waves), four otherwise.  With few tiles and a long reduction the reduction is also cut across workgroups
// (gridDim.z slices, merged by split_merge_kernel): aim at about 384 workgroups, keep at least 128 reduction steps per wave.
struct P8W4Plan {
    GemmPlan gemm;  // splits = gridDim.z, k_per_split = reduction indices per workgroup
    int waves;
};

inline P8W4Plan p8_w4_plan(int64_t M, int64_t N, int64_t K) {
    P8W4Plan p;
    const int64_t tiles = ((M + W4_T - 1) / W4_T) * ((N + W4_T - 1) / W4_T);
    p.waves = (tiles <= 320 && K >= 256) ? 8 : 4;
    int64_t z = 1;
    if (tiles < 256) {
        z = (384 + tiles - 1) / tiles;
        const int64_t by_k = K / (128 * p.waves);
        if (z > by_k) z = by_k;
        if (z > 64) z = 64;
        if (z < 1) z = 1;
    }
    const int64_t wz = p.waves * z;
    const int64_t kq = ((K + wz - 1) / wz + P8_KT - 1) / P8_KT * P8_KT;  // per wave
    z = (K + p.waves * kq - 1) / (p.waves * kq);                         // slices that actually hold work
    p.gemm.splits = (int)z;
    p.gemm.k_per_split = p.waves * kq;
    p.gemm.ws_bytes = z > 1 ? (size_t)z * ((size_t)M * N + M + N) * sizeof(uint32_t) : 0;
    return p;
}

template <bool A_KFAST, bool B_KFAST>
hipError_t launch_p8_gemm_w4(hipStream_t stream, const uint8_t* A, int64_t lda, const uint8_t* B, int64_t ldb, const uint8_t* bias, void* C,
                             int64_t ldc, int fout, int64_t M, int64_t N, int64_t K, void* workspace) {
    const P8W4Plan wp = p8_w4_plan(M, N, K);
    const GemmPlan& plan = wp.gemm;
    const int tiles_m = (int)((M + W4_T - 1) / W4_T), tiles_n = (int)((N + W4_T - 1) / W4_T);
    // 16-byte vector loads: along k for a k-contiguous operand, along the rows otherwise
    const int a_al = ((uintptr_t)A % 16 == 0) && (lda % 16 == 0);
    const int b_al = ((uintptr_t)B % 16 == 0) && (ldb % 16 == 0);
    const int kq = (int)(plan.k_per_split / wp.waves);
    SplitWs ws;
    ws.limbs = nullptr; ws.rowflag = nullptr; ws.colflag = nullptr;
    if (plan.splits > 1) {
        ws.limbs = (uint32_t*)workspace;
        ws.rowflag = ws.limbs + (size_t)plan.splits * M * N;
        ws.colflag = ws.rowflag + (size_t)plan.splits * M;
    }
    const dim3 grid((unsigned)(tiles_m * tiles_n), 1, (unsigned)plan.splits);
    const uint8_t* kbias = plan.splits > 1 ? nullptr : bias;  // the merge adds it
    if (wp.waves == 8)
        hipLaunchKernelGGL((p8_gemm_w4_kernel<A_KFAST, B_KFAST, 8>), grid, dim3(512), 0, stream, A, lda, B, ldb, kbias, C, ldc, fout, (int)M,
                           (int)N, (int)K, kq, tiles_m, tiles_n, a_al, b_al, ws);
    else
        hipLaunchKernelGGL((p8_gemm_w4_kernel<A_KFAST, B_KFAST, 4>), grid, dim3(256), 0, stream, A, lda, B, ldb, kbias, C, ldc, fout, (int)M,
                           (int)N, (int)K, kq, tiles_m, tiles_n, a_al, b_al, ws);
    PNN_CHECK_LAUNCH();
    if (plan.splits > 1) {
        RowMajorOut out{ldc};
        return launch_split_merge<P8, RowMajorOut>(stream, ws, plan.splits, M, N, bias, C, fout, out);
    }
    return hipSuccess;
}

}  // namespace pnn
