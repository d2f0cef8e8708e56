// posit<8,0> quire GEMM, the throughput kernel (paper Sec. 3.3: quire-accumulated
// matrix product; Table 1: 32-bit quire for 8-bit posits).
//
// Every posit<8,0> value is a whole number of minpos = 2^-6 no larger than 2^12
// in magnitude, so a decoded operand is a 14-bit signed integer and the 32-bit
// quire is an int32 counting units of minpos^2 = 2^-12.  One v_dot2_i32_i16
// performs two exact multiply-adds into that quire, which makes the packed
// 16-bit dot product the fastest exact integer-VALU primitive for this format.
//
// Layout of the work: a 256-thread workgroup owns a 128 x 128 tile of C and
// walks the reduction 32 elements at a time.  Patterns are fetched with 16-byte
// (k-contiguous operand) or 8-byte (row-contiguous operand) coalesced loads,
// decoded through a 256-entry table in LDS (Eq. 2 evaluated once per pattern
// when the workgroup starts) and stored to LDS as pairs (k, k+1) packed in one
// 32-bit word, [k-pair][row].  Each thread then reads 4+4 A words and 4+4 B
// words per k-pair with four 128-bit LDS loads and issues 64 dot2 instructions
// on its 8 x 8 register tile.  Global loads for the next slice are in flight
// while the current one is consumed; LDS is double-buffered so one barrier per
// slice suffices.  NaR patterns decode to zero and raise a per-row / per-column
// flag that is applied when the tile is rounded.
#pragma once

#include "quire_gemm.h"

namespace pnn {

constexpr int P8_BM = 128, P8_BN = 128, P8_KT = 32, P8_KP = P8_KT / 2;

typedef short p8_short2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ int32_t dot2_acc(uint32_t a, uint32_t b, int32_t c) {
    return __builtin_amdgcn_sdot2(__builtin_bit_cast(p8_short2, a), __builtin_bit_cast(p8_short2, b), c, false);
}

// nonzero iff one of the four bytes of w is 0x80 (NaR)
__device__ __forceinline__ uint32_t nar_bytes(uint32_t w) {
    const uint32_t t = w ^ 0x80808080u;
    return (t - 0x01010101u) & ~t & 0x80808080u;
}

struct P8Frag {
    uint32_t w[4];
};

// Fetch this thread's 16 bytes of a 128-row x 32-k operand tile.
//  KFAST (k contiguous in memory): thread t holds row t/2, k offsets (t%2)*16 .. +15.
//  otherwise (rows contiguous):    thread t holds k-pair t/16, rows (t%16)*8 .. +7:
//                                  w[0..1] = the 8 bytes at k even, w[2..3] = at k odd.
// `fast` says the tile is interior and the addresses are aligned; otherwise bytes
// are fetched one by one and read as zero outside [0,R) x [0,kend).
template <bool KFAST>
__device__ __forceinline__ P8Frag p8_fetch(const uint8_t* __restrict__ p, int64_t ld, int R, int r0, int k0, int kend,
                                           int t, bool fast) {
    P8Frag f;
    if (KFAST) {
        const int row = r0 + (t >> 1), kk = k0 + (t & 1) * 16;
        if (fast) {
            const uint4 v = *reinterpret_cast<const uint4*>(p + (int64_t)row * ld + kk);
            f.w[0] = v.x; f.w[1] = v.y; f.w[2] = v.z; f.w[3] = v.w;
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                uint32_t w = 0;
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const int k = kk + 4 * i + b;
                    const uint32_t byte = (row < R && k < kend) ? p[(int64_t)row * ld + k] : 0u;
                    w |= byte << (8 * b);
                }
                f.w[i] = w;
            }
        }
    } else {
        const int k = k0 + 2 * (t >> 4), row = r0 + (t & 15) * 8;
        if (fast) {
            const uint2 lo = *reinterpret_cast<const uint2*>(p + (int64_t)k * ld + row);
            const uint2 hi = *reinterpret_cast<const uint2*>(p + (int64_t)(k + 1) * ld + row);
            f.w[0] = lo.x; f.w[1] = lo.y; f.w[2] = hi.x; f.w[3] = hi.y;
        } else {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    uint32_t w = 0;
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        const int r = row + 4 * i + b;
                        const uint32_t byte = (r < R && k + h < kend) ? p[(int64_t)(k + h) * ld + r] : 0u;
                        w |= byte << (8 * b);
                    }
                    f.w[2 * h + i] = w;
                }
            }
        }
    }
    return f;
}

// Decode the fetched patterns through the LDS table and store them as packed
// (k, k+1) pairs into dst[k-pair][row]; raise flags[row] for NaR patterns.
template <bool KFAST>
__device__ __forceinline__ void p8_stage(const P8Frag& f, uint32_t (*dst)[P8_BM], const uint16_t* tab, uint32_t* flags, int t) {
    const uint32_t nar = nar_bytes(f.w[0]) | nar_bytes(f.w[1]) | nar_bytes(f.w[2]) | nar_bytes(f.w[3]);
    if (KFAST) {
        const int row = t >> 1, kp0 = (t & 1) * 8;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t w = f.w[i];
            const uint32_t d0 = (uint32_t)tab[w & 0xFFu] | ((uint32_t)tab[(w >> 8) & 0xFFu] << 16);
            const uint32_t d1 = (uint32_t)tab[(w >> 16) & 0xFFu] | ((uint32_t)tab[w >> 24] << 16);
            dst[kp0 + 2 * i][row] = d0;
            dst[kp0 + 2 * i + 1][row] = d1;
        }
        if (nar) flags[row] = 1;
    } else {
        const int kp = t >> 4, c = (t & 15) * 8;
        uint32_t d[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t lo = (f.w[j >> 2] >> (8 * (j & 3))) & 0xFFu;
            const uint32_t hi = (f.w[2 + (j >> 2)] >> (8 * (j & 3))) & 0xFFu;
            d[j] = (uint32_t)tab[lo] | ((uint32_t)tab[hi] << 16);
        }
        *reinterpret_cast<uint4*>(&dst[kp][c]) = make_uint4(d[0], d[1], d[2], d[3]);
        *reinterpret_cast<uint4*>(&dst[kp][c + 4]) = make_uint4(d[4], d[5], d[6], d[7]);
        if (nar) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint32_t lo = (f.w[j >> 2] >> (8 * (j & 3))) & 0xFFu;
                const uint32_t hi = (f.w[2 + (j >> 2)] >> (8 * (j & 3))) & 0xFFu;
                if (lo == 0x80u || hi == 0x80u) flags[c + j] = 1;
            }
        }
    }
}

// ---- operands decoded and packed once (large products) ----
//
// For a product of some 10^10 MACs the per-slice decode of the kernel below (table look-ups and
// packing: a sixth of its vector instructions) is worth doing once instead: p8_pack_kernel rewrites
// an operand into the workspace as X2[k-pair][row] = (decoded X(row, 2kp), decoded X(row, 2kp+1)),
// two int16 in a dword, exactly the word the LDS tiles hold, rows padded to a multiple of 128 and the
// reduction to a multiple of 32 with zeros.  The main kernel then copies 16-byte runs of X2 straight
// into LDS.  NaR patterns are stored as zero and raise flags[row] (cleared beforehand).
//   element strides: X(row, k) = src[row * s_r + k * s_k], one of the strides is 1
//   s_k == 1: a thread takes one row and 8 k-pairs (16 consecutive bytes); the 32 rows of a half wave
//             make every store 128 contiguous bytes
//   s_r == 1: a thread takes one k-pair and 4 consecutive rows (one 16-byte store)
struct P8PackJob {
    const uint8_t* src;
    int64_t s_r, s_k;
    int rows, K;
    uint32_t* dst;
    int Rp, Kp2;
    uint32_t* flags;
};

// Both operands are packed by one launch: the first blocks0 workgroups take job0, the rest job1;
// a job's workgroups are numbered along its rows first (bx), then along the reduction (by).
template <int UNUSED = 0>
__global__ __launch_bounds__(256) void p8_pack_kernel(P8PackJob job0, P8PackJob job1, unsigned blocks0) {
    __shared__ uint16_t tab[256];
    const int t = threadIdx.x;
    tab[t] = (uint16_t)Arith<P8>::stage((uint32_t)t);
    __syncthreads();
    const bool first = blockIdx.x < blocks0;
    const P8PackJob& job = first ? job0 : job1;
    const unsigned lin = first ? blockIdx.x : blockIdx.x - blocks0;
    const unsigned gx = job.s_k == 1 ? (unsigned)((job.Rp + 31) / 32) : (unsigned)((job.Rp / 4 + 63) / 64);
    const unsigned bx = lin % gx, by = lin / gx;
    const uint8_t* __restrict__ src = job.src;
    const int64_t s_r = job.s_r, s_k = job.s_k;
    const int rows = job.rows, K = job.K, Rp = job.Rp, Kp2 = job.Kp2;
    uint32_t* __restrict__ dst = job.dst;
    uint32_t* __restrict__ flags = job.flags;
    if (s_k == 1) {
        // block: 32 rows x 64 k-pairs (8 groups of 8); bx over row blocks, by over groups of 64 k-pairs
        const int row = (int)bx * 32 + (t & 31);
        const int kp0 = (int)by * 64 + (t >> 5) * 8;
        if (row >= Rp || kp0 >= Kp2) return;
        uint32_t out[8];
        bool nar = false;
        const uint8_t* p = src + (int64_t)row * s_r + 2 * (int64_t)kp0;
        const bool inside = row < rows && 2 * kp0 + 16 <= K;
        uint32_t w[4] = {0, 0, 0, 0};
        if (inside && (((uintptr_t)p) & 3u) == 0) {
#pragma unroll
            for (int i = 0; i < 4; ++i) w[i] = reinterpret_cast<const uint32_t*>(p)[i];
        } else if (row < rows) {
#pragma unroll
            for (int b = 0; b < 16; ++b)
                if (2 * kp0 + b < K) w[b >> 2] |= (uint32_t)p[b] << (8 * (b & 3));
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t lo = (w[j >> 1] >> (16 * (j & 1))) & 0xFFu, hi = (w[j >> 1] >> (16 * (j & 1) + 8)) & 0xFFu;
            nar |= (lo == 0x80u) | (hi == 0x80u);
            out[j] = (uint32_t)tab[lo] | ((uint32_t)tab[hi] << 16);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (kp0 + j < Kp2) dst[(int64_t)(kp0 + j) * Rp + row] = out[j];
        if (nar) atomicOr(&flags[row], 1u);
    } else {
        // block: 4 k-pairs x 256 rows; thread = (k-pair, 4 consecutive rows)
        const int r4 = ((int)bx * 64 + (t & 63)) * 4;
        const int kp = (int)by * 4 + (t >> 6);
        if (r4 >= Rp || kp >= Kp2) return;
        uint32_t out[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = r4 + i;
            uint32_t lo = 0, hi = 0;
            if (r < rows) {
                if (2 * kp < K) lo = src[(int64_t)r * s_r + (int64_t)(2 * kp) * s_k];
                if (2 * kp + 1 < K) hi = src[(int64_t)r * s_r + (int64_t)(2 * kp + 1) * s_k];
            }
            if (lo == 0x80u || hi == 0x80u) atomicOr(&flags[r], 1u);
            out[i] = (uint32_t)tab[lo] | ((uint32_t)tab[hi] << 16);
        }
        *reinterpret_cast<uint4*>(dst + (int64_t)kp * Rp + r4) = make_uint4(out[0], out[1], out[2], out[3]);
    }
}

template <int UNUSED = 0>
__global__ void p8_fill_zero_kernel(uint32_t* p, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

// int32 quire (units of 2^-12) -> posit<8,0>, nearest, ties to even pattern, clamped to +-minpos / +-maxpos.
// Straight-line code (an epilogue calls it for every output of a tile; branches per call cost more than they save):
// with k = floor(log2 |value|), kk = k for k >= 0 and -k-1 otherwise, an arithmetic right shift by kk of "10" followed by
// the fraction gives kk+1 ones, a zero and the fraction; for negative k the fraction is complemented before and the whole
// word after the shift, which turns that head into kk+1 zeros and a one.  The eight fraction bits that the shifts can
// push out are folded into bit 8 first, which always lies below the guard bit and is never pushed out itself.
PNN_HD uint32_t p8_round_quire(int32_t q) {
    const uint32_t sm = (uint32_t)(q >> 31);  // all ones for a negative sum
    const uint32_t mag = ((uint32_t)q ^ sm) - sm;
    const int lz = clz32(mag);
    const int k0 = 19 - lz;                              // floor(log2(mag)) - 12
    const bool beyond = k0 >= 6 || k0 < -6;              // at or past maxpos / below minpos: the end pattern, no fraction
    const int k = k0 > 6 ? 6 : (k0 < -6 ? -6 : k0);
    const uint32_t frac = beyond ? 0u : ((mag << (lz & 31)) << 1);  // fraction bits at the top, leading one gone
    const uint32_t sg = (uint32_t)(k >> 31);
    const uint32_t kk = (uint32_t)k ^ sg;
    const uint32_t jam = (frac & 0xFFu) ? 0x100u : 0u;
    const uint32_t w = 0x80000000u | (((frac | jam) ^ sg) >> 2);
    const uint32_t x = (uint32_t)((int32_t)w >> kk) ^ sg;  // 7 kept bits, the guard bit, sticky bits
    const uint32_t body = (x + 0x00FFFFFFu + ((x >> 25) & 1u)) >> 25;
    const uint32_t pat = ((body ^ sm) - sm) & 0xFFu;
    return q == 0 ? 0u : pat;
}

// PACKED: A and B point at operands rewritten by p8_pack_kernel (lda, ldb: their padded row counts),
// rowflag_g / colflag_g at the NaR flags that kernel raised.
template <bool A_KFAST, bool B_KFAST, bool PACKED = false>
__global__ __launch_bounds__(256, 4) void p8_gemm_kernel(
    const uint8_t* __restrict__ A, int64_t lda, const uint8_t* __restrict__ B, int64_t ldb,
    const uint8_t* __restrict__ bias, void* __restrict__ C, int64_t ldc, int fout,
    int M, int N, int K, int k_per_split, int tiles_m, int tiles_n, int a_aligned, int b_aligned, SplitWs ws,
    const uint32_t* __restrict__ rowflag_g = nullptr, const uint32_t* __restrict__ colflag_g = nullptr) {
    __shared__ __attribute__((aligned(16))) uint32_t As[2][P8_KP][P8_BM];
    __shared__ __attribute__((aligned(16))) uint32_t Bs[2][P8_KP][P8_BN];
    __shared__ uint16_t tab[256];
    __shared__ uint32_t rowNaR[P8_BM];
    __shared__ uint32_t colNaR[P8_BN];

    const int t = threadIdx.x;
    const int tx = t & 15, ty = t >> 4;

    // XCD-aware order: consecutive workgroup ids go round-robin to the 8 XCDs, so give each XCD
    // a contiguous run of tiles (neighbouring tiles share operand panels in that XCD's L2).
    const int nblk = tiles_m * tiles_n;
    int lid = blockIdx.x;
    if ((nblk & 7) == 0) lid = (blockIdx.x & 7) * (nblk >> 3) + (blockIdx.x >> 3);
    // tiles are walked in bands of 8 tile-rows, column by column inside a band
    const int band = lid / (8 * tiles_n);
    const int band_rows = (tiles_m - band * 8) < 8 ? (tiles_m - band * 8) : 8;
    const int in_band = lid - band * 8 * tiles_n;
    const int m0 = (band * 8 + in_band % band_rows) * P8_BM;
    const int n0 = (in_band / band_rows) * P8_BN;

    const int kbeg = blockIdx.z * k_per_split;
    const int kend = (kbeg + k_per_split < K) ? kbeg + k_per_split : K;

    tab[t] = (uint16_t)Arith<P8>::stage((uint32_t)t);
    if constexpr (PACKED) {  // the flags are known beforehand (padded to whole tiles)
        if (t < P8_BM) rowNaR[t] = rowflag_g[m0 + t]; else colNaR[t - P8_BM] = colflag_g[n0 + t - P8_BM];
    } else {
        if (t < P8_BM) rowNaR[t] = 0; else colNaR[t - P8_BM] = 0;
    }

    int32_t acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = 0;

    const bool a_rows_in = (m0 + P8_BM <= M) && a_aligned;
    const bool b_rows_in = (n0 + P8_BN <= N) && b_aligned;
    const int nkt = (kend - kbeg + P8_KT - 1) / P8_KT;

    __syncthreads();  // table and flags ready
    if constexpr (PACKED) {
        // this thread's two 16-byte runs of a slice: k-pairs t/32 and t/32 + 8, rows (t%32)*4 .. +3; running pointers, one slice = 16 k-pairs
        const uint32_t* pa = reinterpret_cast<const uint32_t*>(A) + (int64_t)(kbeg / 2 + (t >> 5)) * lda + m0 + (t & 31) * 4;
        const uint32_t* pb = reinterpret_cast<const uint32_t*>(B) + (int64_t)(kbeg / 2 + (t >> 5)) * ldb + n0 + (t & 31) * 4;
        const int64_t a_half = 8 * lda, b_half = 8 * ldb;
        uint32_t* const sa = &As[0][t >> 5][(t & 31) * 4];
        uint32_t* const sb = &Bs[0][t >> 5][(t & 31) * 4];
        constexpr int HALF = 8 * P8_BM, BUF = P8_KP * P8_BM;  // dwords between the two runs / the two buffers
        if (nkt > 0) {
            const uint4 a0 = *reinterpret_cast<const uint4*>(pa), a1 = *reinterpret_cast<const uint4*>(pa + a_half);
            const uint4 b0 = *reinterpret_cast<const uint4*>(pb), b1 = *reinterpret_cast<const uint4*>(pb + b_half);
            *reinterpret_cast<uint4*>(sa) = a0; *reinterpret_cast<uint4*>(sa + HALF) = a1;
            *reinterpret_cast<uint4*>(sb) = b0; *reinterpret_cast<uint4*>(sb + HALF) = b1;
        }
        __syncthreads();
        for (int kt = 0; kt < nkt; ++kt) {
            const int cur = kt & 1;
            const bool more = kt + 1 < nkt;
            uint4 fa0, fa1, fb0, fb1;
            if (more) {
                pa += 2 * a_half;
                pb += 2 * b_half;
                fa0 = *reinterpret_cast<const uint4*>(pa); fa1 = *reinterpret_cast<const uint4*>(pa + a_half);
                fb0 = *reinterpret_cast<const uint4*>(pb); fb1 = *reinterpret_cast<const uint4*>(pb + b_half);
            }
#pragma unroll 2
            for (int kp = 0; kp < P8_KP; ++kp) {
                const uint4 a0 = *reinterpret_cast<const uint4*>(&As[cur][kp][ty * 4]);
                const uint4 a1 = *reinterpret_cast<const uint4*>(&As[cur][kp][64 + ty * 4]);
                const uint4 b0 = *reinterpret_cast<const uint4*>(&Bs[cur][kp][tx * 4]);
                const uint4 b1 = *reinterpret_cast<const uint4*>(&Bs[cur][kp][64 + tx * 4]);
                const uint32_t a[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
                const uint32_t b[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
#pragma unroll
                for (int i = 0; i < 8; ++i)
#pragma unroll
                    for (int j = 0; j < 8; ++j) acc[i][j] = dot2_acc(a[i], b[j], acc[i][j]);
            }
            if (more) {
                const int nxt = (cur ^ 1) * BUF;
                *reinterpret_cast<uint4*>(sa + nxt) = fa0; *reinterpret_cast<uint4*>(sa + nxt + HALF) = fa1;
                *reinterpret_cast<uint4*>(sb + nxt) = fb0; *reinterpret_cast<uint4*>(sb + nxt + HALF) = fb1;
            }
            __syncthreads();
        }
    } else {
    if (nkt > 0) {
        const bool kin = kbeg + P8_KT <= kend;
        const P8Frag fa = p8_fetch<A_KFAST>(A, lda, M, m0, kbeg, kend, t, a_rows_in && kin);
        const P8Frag fb = p8_fetch<B_KFAST>(B, ldb, N, n0, kbeg, kend, t, b_rows_in && kin);
        p8_stage<A_KFAST>(fa, As[0], tab, rowNaR, t);
        p8_stage<B_KFAST>(fb, Bs[0], tab, colNaR, t);
    }
    __syncthreads();

    for (int kt = 0; kt < nkt; ++kt) {
        const int cur = kt & 1;
        const bool more = kt + 1 < nkt;
        P8Frag fa, fb;
        if (more) {
            const int k0 = kbeg + (kt + 1) * P8_KT;
            const bool kin = k0 + P8_KT <= kend;
            fa = p8_fetch<A_KFAST>(A, lda, M, m0, k0, kend, t, a_rows_in && kin);
            fb = p8_fetch<B_KFAST>(B, ldb, N, n0, k0, kend, t, b_rows_in && kin);
        }
#pragma unroll 2
        for (int kp = 0; kp < P8_KP; ++kp) {
            const uint4 a0 = *reinterpret_cast<const uint4*>(&As[cur][kp][ty * 4]);
            const uint4 a1 = *reinterpret_cast<const uint4*>(&As[cur][kp][64 + ty * 4]);
            const uint4 b0 = *reinterpret_cast<const uint4*>(&Bs[cur][kp][tx * 4]);
            const uint4 b1 = *reinterpret_cast<const uint4*>(&Bs[cur][kp][64 + tx * 4]);
            const uint32_t a[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
            const uint32_t b[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[i][j] = dot2_acc(a[i], b[j], acc[i][j]);
        }
        if (more) {
            p8_stage<A_KFAST>(fa, As[cur ^ 1], tab, rowNaR, t);
            p8_stage<B_KFAST>(fb, Bs[cur ^ 1], tab, colNaR, t);
        }
        __syncthreads();
    }

    }

    // rows / columns of this thread's register tile
    if (gridDim.z == 1) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int lr = (i < 4) ? ty * 4 + i : 64 + ty * 4 + (i - 4);
            const int m = m0 + lr;
            if (m >= M) continue;
            const bool rnar = rowNaR[lr] != 0;
#pragma unroll
            for (int jh = 0; jh < 2; ++jh) {
                const int lc = jh * 64 + tx * 4;
                const int n = n0 + lc;
                uint32_t res[4];
                bool narv[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    int32_t q = acc[i][jh * 4 + j];
                    bool nar = rnar || colNaR[lc + j] != 0;
                    if (bias && n + j < N) {
                        const uint32_t bp = bias[n + j];
                        if (bp == 0x80u) nar = true;
                        else q += (int32_t)(int16_t)tab[bp] << P8::MAXS;  // + bias * 1
                    }
                    narv[j] = nar;
                    res[j] = (uint32_t)q;
                }
                if (fout == 0) {
                    uint32_t out[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) out[j] = narv[j] ? 0x80u : p8_round_quire((int32_t)res[j]);
                    uint8_t* crow = (uint8_t*)C + (int64_t)m * ldc + n;
                    if (n + 4 <= N && (((uintptr_t)crow) & 3) == 0) {
                        *reinterpret_cast<uint32_t*>(crow) = out[0] | (out[1] << 8) | (out[2] << 16) | (out[3] << 24);
                    } else {
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            if (n + j < N) crow[j] = (uint8_t)out[j];
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        if (n + j >= N) continue;
                        const uint32_t q1[1] = {res[j]};
                        round_store<QuireAccum<P8>, 1>(q1, narv[j], fout, C, (int64_t)m * ldc + n + j);
                    }
                }
            }
        }
    } else {
        const int64_t z = blockIdx.z;
        uint32_t* lim = ws.limbs + z * (int64_t)M * N;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int lr = (i < 4) ? ty * 4 + i : 64 + ty * 4 + (i - 4);
            const int m = m0 + lr;
            if (m >= M) continue;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int n = n0 + ((j < 4) ? tx * 4 + j : 64 + tx * 4 + (j - 4));
                if (n < N) lim[(int64_t)m * N + n] = (uint32_t)acc[i][j];
            }
        }
        // the first tile column stores the row flags of its tile row (identical in every column), the
        // first tile row the column flags: every entry is written, so the workspace needs no clearing
        if (t < P8_BM) {
            if (n0 == 0 && m0 + t < M) ws.rowflag[z * M + m0 + t] = rowNaR[t];
        } else {
            const int c = t - P8_BM;
            if (m0 == 0 && n0 + c < N) ws.colflag[z * N + n0 + c] = colNaR[c];
        }
    }
}

// Host launcher.  Returns hipSuccess or the launch error.
template <bool A_KFAST, bool B_KFAST>
hipError_t launch_p8_gemm(hipStream_t stream, const uint8_t* A, int64_t lda, const uint8_t* B, int64_t ldb,
                          const uint8_t* bias, void* C, int64_t ldc, int fout, int64_t M, int64_t N, int64_t K,
                          void* workspace, const GemmPlan& plan) {
    const int tiles_m = (int)((M + P8_BM - 1) / P8_BM), tiles_n = (int)((N + P8_BN - 1) / P8_BN);
    // vector loads need aligned addresses: 16 bytes along k, 8 bytes along rows
    const int a_al = A_KFAST ? (((uintptr_t)A % 16 == 0) && (lda % 16 == 0)) : (((uintptr_t)A % 8 == 0) && (lda % 8 == 0));
    const int b_al = B_KFAST ? (((uintptr_t)B % 16 == 0) && (ldb % 16 == 0)) : (((uintptr_t)B % 8 == 0) && (ldb % 8 == 0));
    SplitWs ws;
    ws.limbs = nullptr; ws.rowflag = nullptr; ws.colflag = nullptr;
    if (plan.splits > 1) {
        ws.limbs = (uint32_t*)workspace;
        ws.rowflag = ws.limbs + (size_t)plan.splits * M * N;
        ws.colflag = ws.rowflag + (size_t)plan.splits * M;
    }
    dim3 grid((unsigned)(tiles_m * tiles_n), 1, (unsigned)plan.splits);
    hipLaunchKernelGGL((p8_gemm_kernel<A_KFAST, B_KFAST>), grid, dim3(256), 0, stream, A, lda, B, ldb, bias, C, ldc, fout,
                       (int)M, (int)N, (int)K, (int)plan.k_per_split, tiles_m, tiles_n, a_al, b_al, ws);
    PNN_CHECK_LAUNCH();
    if (plan.splits > 1) {
        RowMajorOut out{ldc};
        return launch_split_merge<P8, RowMajorOut>(stream, ws, plan.splits, M, N, bias, C, fout, out);
    }
    return hipSuccess;
}

// ---- large problems: operands packed once ----

// Worth it when the saved per-slice decode outweighs one more pass over the operands.
inline bool p8_packed_gemm_fits(int64_t M, int64_t N, int64_t K) {
    return M >= 1024 && N >= 1024 && K >= 1024 && M * N * K >= ((int64_t)1 << 34) && M < ((int64_t)1 << 30) && N < ((int64_t)1 << 30);
}

struct P8PackedLayout {
    int64_t Mp, Np, Kp2;          // rows padded to 128, k-pairs padded to 16
    size_t a_bytes, b_bytes, flag_bytes;
    size_t total() const { return a_bytes + b_bytes + flag_bytes; }
};

inline P8PackedLayout p8_packed_layout(int64_t M, int64_t N, int64_t K) {
    P8PackedLayout l;
    l.Mp = (M + P8_BM - 1) / P8_BM * P8_BM;
    l.Np = (N + P8_BN - 1) / P8_BN * P8_BN;
    l.Kp2 = (K + P8_KT - 1) / P8_KT * P8_KP;
    l.a_bytes = (size_t)l.Kp2 * l.Mp * sizeof(uint32_t);
    l.b_bytes = (size_t)l.Kp2 * l.Np * sizeof(uint32_t);
    l.flag_bytes = (size_t)(l.Mp + l.Np) * sizeof(uint32_t);
    return l;
}

inline dim3 p8_pack_grid(const P8PackJob& j) {
    if (j.s_k == 1) return dim3((unsigned)((j.Rp + 31) / 32), (unsigned)((j.Kp2 + 63) / 64));
    return dim3((unsigned)((j.Rp / 4 + 63) / 64), (unsigned)((j.Kp2 + 3) / 4));
}

inline void launch_p8_pack(hipStream_t stream, const P8PackJob& a, const P8PackJob& b) {
    const dim3 ga = p8_pack_grid(a), gb = p8_pack_grid(b);
    const unsigned na = ga.x * ga.y, nb = gb.x * gb.y;
    hipLaunchKernelGGL(p8_pack_kernel<0>, dim3(na + nb), dim3(256), 0, stream, a, b, na);
}

// Workspace: [A2][B2][row flags (Mp)][column flags (Np)][partial quires and flags of a split reduction].
inline hipError_t launch_p8_gemm_packed(hipStream_t stream, int transA, int transB, const uint8_t* A, int64_t lda, const uint8_t* B,
                                        int64_t ldb, const uint8_t* bias, void* C, int64_t ldc, int fout, int64_t M, int64_t N,
                                        int64_t K, void* workspace, const GemmPlan& plan) {
    // the packed kernel walks whole 32-wide slices from kbeg with no masking at kend (the padding holds zeros), so
    // the slices of a split reduction must begin on slice boundaries or neighbours would both count the overlap
    if (plan.splits > 1 && plan.k_per_split % P8_KT != 0) return hipErrorInvalidValue;
    const P8PackedLayout l = p8_packed_layout(M, N, K);
    uint8_t* wb = (uint8_t*)workspace;
    uint32_t* A2 = (uint32_t*)wb;
    uint32_t* B2 = (uint32_t*)(wb + l.a_bytes);
    uint32_t* rowflag = (uint32_t*)(wb + l.a_bytes + l.b_bytes);
    uint32_t* colflag = rowflag + l.Mp;
    const int64_t nflags = l.Mp + l.Np;
    hipLaunchKernelGGL(p8_fill_zero_kernel<0>, dim3((unsigned)((nflags + 255) / 256)), dim3(256), 0, stream, rowflag, nflags);
    PNN_CHECK_LAUNCH();
    // op(A)(m, k): stride (lda, 1), transposed (1, lda); op(B)(k, n) seen as rows n: stride (1, ldb), transposed (ldb, 1)
    const P8PackJob ja{A, transA ? (int64_t)1 : lda, transA ? lda : (int64_t)1, (int)M, (int)K, A2, (int)l.Mp, (int)l.Kp2, rowflag};
    const P8PackJob jb{B, transB ? ldb : (int64_t)1, transB ? (int64_t)1 : ldb, (int)N, (int)K, B2, (int)l.Np, (int)l.Kp2, colflag};
    launch_p8_pack(stream, ja, jb);
    PNN_CHECK_LAUNCH();
    const int tiles_m = (int)(l.Mp / P8_BM), tiles_n = (int)(l.Np / P8_BN);
    SplitWs ws;
    ws.limbs = nullptr; ws.rowflag = nullptr; ws.colflag = nullptr;
    if (plan.splits > 1) {
        ws.limbs = (uint32_t*)(wb + l.total());
        ws.rowflag = ws.limbs + (size_t)plan.splits * M * N;
        ws.colflag = ws.rowflag + (size_t)plan.splits * M;
    }
    dim3 grid((unsigned)(tiles_m * tiles_n), 1, (unsigned)plan.splits);
    hipLaunchKernelGGL((p8_gemm_kernel<true, true, true>), grid, dim3(256), 0, stream, (const uint8_t*)A2, l.Mp, (const uint8_t*)B2, l.Np,
                       bias, C, ldc, fout, (int)M, (int)N, (int)K, (int)plan.k_per_split, tiles_m, tiles_n, 1, 1, ws,
                       (const uint32_t*)rowflag, (const uint32_t*)colflag);
    PNN_CHECK_LAUNCH();
    if (plan.splits > 1) {
        RowMajorOut out{ldc};
        return launch_split_merge<P8, RowMajorOut>(stream, ws, plan.splits, M, N, bias, C, fout, out);
    }
    return hipSuccess;
}

// ---- small problems ----
//
// A product with few outputs (the fully connected layers of a small network at batch 64: 64 x 120 x 400,
// 120 x 400 x 64, ...) gives the tiled kernel one or two workgroups, which then walk the reduction
// slice by slice, each slice a chain of global load -> LDS -> barrier -> multiply: tens of
// microseconds of latency for a few MMAC.  Here every output gets S threads of its own (S a power
// of two, splitting the reduction), outputs spread over as many workgroups as there are, operands
// come straight from global memory (lanes of a wave share the A element and read consecutive B
// elements) and decode through the LDS table; the S partial sums of an output meet in LDS (int32
// addition modulo 2^32: exact in the 32-bit quire) and are rounded once.
//   element strides: A(m,k) = A[m*a_m + k*a_k], B(k,n) = B[k*b_k + n*b_n]
template <int UNUSED = 0>  // a template so that every translation unit may include this header
__global__ __launch_bounds__(256) void p8_small_gemm_kernel(const uint8_t* __restrict__ A, int64_t a_m, int64_t a_k,
                                                            const uint8_t* __restrict__ B, int64_t b_k, int64_t b_n,
                                                            const uint8_t* __restrict__ bias, void* __restrict__ C, int64_t ldc, int fout,
                                                            int M, int N, int K, int S, int k_per_split) {
    __shared__ int32_t tab[256];
    __shared__ uint32_t part[256];
    __shared__ uint32_t nars[256];
    const int t = threadIdx.x;
    tab[t] = Arith<P8>::stage((uint32_t)t);
    __syncthreads();
    const int OB = 256 / S;  // outputs per workgroup
    const int ol = t % OB, s = t / OB;
    const int64_t o = (int64_t)blockIdx.x * OB + ol;
    const bool live = o < (int64_t)M * N;
    const int m = live ? (int)(o / N) : 0, n = live ? (int)(o - (int64_t)m * N) : 0;
    const int k_lo = s * k_per_split, k_hi = k_lo + k_per_split < K ? k_lo + k_per_split : K;
    uint32_t acc = 0, nar = 0;
    if (live) {
        const uint8_t* ap = A + (int64_t)m * a_m + (int64_t)k_lo * a_k;
        const uint8_t* bp = B + (int64_t)n * b_n + (int64_t)k_lo * b_k;
        int k = k_lo;
        for (; k + 4 <= k_hi; k += 4) {
            uint32_t a[4], b[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                a[u] = ap[u * a_k];
                b[u] = bp[u * b_k];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                nar |= (a[u] == 0x80u) | (b[u] == 0x80u);
                acc += (uint32_t)__mul24(tab[a[u]], tab[b[u]]);
            }
            ap += 4 * a_k;
            bp += 4 * b_k;
        }
        for (; k < k_hi; ++k) {
            const uint32_t a = *ap, b = *bp;
            nar |= (a == 0x80u) | (b == 0x80u);
            acc += (uint32_t)__mul24(tab[a], tab[b]);
            ap += a_k;
            bp += b_k;
        }
    }
    part[t] = acc;
    nars[t] = nar;
    __syncthreads();
    if (s != 0 || !live) return;
    for (int z = 1; z < S; ++z) {
        acc += part[z * OB + ol];
        nar |= nars[z * OB + ol];
    }
    bool isnar = nar != 0;
    if (bias) {
        const uint32_t bpat = bias[n];
        if (bpat == 0x80u) isnar = true;
        else acc += (uint32_t)tab[bpat] << P8::MAXS;
    }
    const int64_t at = (int64_t)m * ldc + n;
    if (fout == 0) {
        ((uint8_t*)C)[at] = (uint8_t)(isnar ? 0x80u : p8_round_quire((int32_t)acc));
    } else {
        const uint32_t q1[1] = {acc};
        round_store<QuireAccum<P8>, 1>(q1, isnar, fout, C, at);
    }
}

// Problems the small kernel takes: little work, and either few outputs or a reduction of at most two slices (the
// tiled kernels execute their long instruction stream once per workgroup there: instruction fetch, not arithmetic,
// sets their time -- 19 us for 128 x 2048 x 10 against 4).
inline bool p8_small_gemm_fits(int64_t M, int64_t N, int64_t K) {
    return M * N * K <= ((int64_t)1 << 26) && K >= 1 && (M * N <= 65536 || (K <= 64 && M * N <= ((int64_t)1 << 21)));
}

inline hipError_t launch_p8_small_gemm(hipStream_t stream, int transA, int transB, const uint8_t* A, int64_t lda, const uint8_t* B,
                                       int64_t ldb, const uint8_t* bias, void* C, int64_t ldc, int fout, int64_t M, int64_t N, int64_t K) {
    // threads per output: keep at least 32 reduction steps per thread, and stop once about 1024 workgroups exist
    int S = 1;
    while (S < 64 && K / (2 * S) >= 32 && (M * N * S) / 256 < 1024) S *= 2;
    const int kps = (int)((K + S - 1) / S);
    const int OB = 256 / S;
    const int64_t blocks = (M * N + OB - 1) / OB;
    hipLaunchKernelGGL(p8_small_gemm_kernel<0>, dim3((unsigned)blocks), dim3(256), 0, stream, A, transA ? (int64_t)1 : lda, transA ? lda : (int64_t)1,
                       B, transB ? (int64_t)1 : ldb, transB ? ldb : (int64_t)1, bias, C, ldc, fout, (int)M, (int)N, (int)K, S, kps);
    return hipGetLastError();
}

}  // namespace pnn
