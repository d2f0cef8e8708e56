// posit<8,0> matrix product with the 32-bit quire of Table 1 (paper Sec. 2, Sec. 3.3) on the integer matrix cores.
//
// A decoded posit<8,0> is an integer v of at most 13 bits plus sign (units of minpos = 2^-6), and the quire is the
// int32 sum of the products modulo 2^32.  Integer matrix instructions multiply int8 by int8 into int32 exactly, so v is
// written in two base-128 digits, v = 128 hi + lo with hi = v >> 7 in [-32, 32] and lo = v & 127 in [0, 127], and
//     a b = 2^14 (ah bh) + 2^7 (ah bl + al bh) + (al bl):
// three int32 sums per output -- HH, X (both cross terms share it) and LL -- fed by four int8 products per posit
// product, combined once after the reduction as (HH << 14) + (X << 7) + LL in 32-bit arithmetic.  Every step is exact
// modulo 2^32 (a sum that wraps in one of the three accumulators wraps the same way in the combination, since the
// shifts only discard high bits), so the result is the quire's bit for bit, wrap-around included.  The int8 matrix
// rate of the chip is 64 times the rate of the packed 16-bit dot product per instruction slot, which leaves a factor
// of 8 after the four products: v_mfma_i32_32x32x32_i8 does 32768 int8 products in 32 cycles on one SIMD.
//
// Lane layout of that instruction (checked on the hardware): lane l holds, for A, row l % 32 and the 16 consecutive
// reduction indices starting at 16 (l / 32); for B column l % 32 and the same indices; register r of the result is
// row (r % 4) + 8 (r / 4) + 4 (l / 32), column l % 32.  The order of the reduction indices inside a block does not
// matter as long as both operands use the same one.
//
// A first launch (p8_digits_kernel) decodes both operands through the LDS table and writes their digit planes into the
// workspace in exactly the order the instruction wants them: [k block of 32][row block of 32][digit][lane][16 bytes],
// zero-padded to whole tiles; NaR is the high digit -128, which no value has (|hi| <= 32).  The product kernel then never rearranges
// anything: 16-byte copies from there into LDS, 16-byte LDS reads into the operand registers.  128 x 128 outputs per
// workgroup of four waves, 64 x 64 per wave as 2 x 2 blocks x 3 sums = 192 accumulator registers.  Every wave sees
// the whole reduction of its rows and columns, so the waves find the NaR markers themselves (three vector operations
// per high-digit register, the two waves that share a block splitting it): no flag arrays, no atomics, no clearing
// launch.
#pragma once

#include "gemm_p8.h"

namespace pnn {

typedef int pm_v4i __attribute__((ext_vector_type(4)));
typedef int pm_v16i __attribute__((ext_vector_type(16)));

constexpr int PM_MIN_MN = 128;                   // smallest output extent each way
constexpr int64_t PM_MIN_MNK = (int64_t)1 << 28;  // smallest product count
constexpr int PM_MIN_TILES = 81;                 // fewest 64 x 64 tiles: below, kernels that cut the reduction across workgroups win
constexpr int PM_MIN_WGS = 512;                  // workgroups wanted before a larger tile is chosen
constexpr int PM_MIN_KB_SPLIT = 16;              // fewest k blocks of 32 per slice
constexpr int PM_KSTEP = 2;    // k blocks (of 32) per staged step
constexpr int PM_NAR_HI = -128;  // high digit that marks NaR

// Bits 7 of the bytes of the result mark the bytes of w whose top two bits are "10": among high digits (values in
// [-32, 32]: top bits 00 or 11) only the NaR marker.  The other bits of the result are noise, masked when read.
__device__ __forceinline__ uint32_t pm_marker_bits(uint32_t w) { return w & ~(w << 1); }

struct P8DigitJob {
    const uint8_t* src;
    int64_t s_r, s_k;   // element (row, k) at src[row * s_r + k * s_k]; one of the two is 1
    int rows, K;
    uint8_t* dst;       // [KB][RB][2][64][16]
    int RB, KB;         // padded extents in blocks of 32
};

// Both operands in one launch: the first blocks0 workgroups take job0, the rest job1.  A workgroup handles one k block
// and eight row blocks: 512 lane slots of 16 bytes per digit, two per thread.
template <int UNUSED = 0>
__global__ __launch_bounds__(256) void p8_digits_kernel(P8DigitJob job0, P8DigitJob job1, unsigned blocks0) {
    __shared__ int16_t tab[256];
    const int t = threadIdx.x;
    tab[t] = t == 0x80 ? (int16_t)(PM_NAR_HI * 128) : (int16_t)Arith<P8>::stage((uint32_t)t);
    __syncthreads();
    const bool first = blockIdx.x < blocks0;
    const P8DigitJob& job = first ? job0 : job1;
    const unsigned lin = first ? blockIdx.x : blockIdx.x - blocks0;
    const unsigned gx = (unsigned)((job.RB + 7) / 8);
    const int bx = (int)(lin % gx), kb = (int)(lin / gx);
    // Rows contiguous in memory (s_r == 1: an operand stored reduction index major): the 32 x 256 patterns of the
    // workgroup's block go through LDS, read as 16-byte runs along the rows and picked up along k.
    __shared__ __attribute__((aligned(16))) uint8_t tile[32][256];
    const bool via_lds = job.s_k != 1;
    if (via_lds) {
        const int kk = t >> 3, seg = (t & 7) * 32;  // thread: 32 consecutive rows at one k
        const int k = kb * 32 + kk;
        const int row0 = bx * 256 + seg;
        uint32_t w[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        if (k < job.K && row0 < job.rows) {
            const uint8_t* p = job.src + (int64_t)k * job.s_k + row0;
            if (row0 + 32 <= job.rows && (((uintptr_t)p) & 15u) == 0) {
                const uint4 v0 = reinterpret_cast<const uint4*>(p)[0], v1 = reinterpret_cast<const uint4*>(p)[1];
                w[0] = v0.x; w[1] = v0.y; w[2] = v0.z; w[3] = v0.w; w[4] = v1.x; w[5] = v1.y; w[6] = v1.z; w[7] = v1.w;
            } else {
                for (int b = 0; b < 32; ++b)
                    if (row0 + b < job.rows) w[b >> 2] |= (uint32_t)p[b] << (8 * (b & 3));
            }
        }
        uint4* d = reinterpret_cast<uint4*>(&tile[kk][seg]);
        d[0] = make_uint4(w[0], w[1], w[2], w[3]);
        d[1] = make_uint4(w[4], w[5], w[6], w[7]);
        __syncthreads();
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int slot = t + 256 * h;
        const int rb = bx * 8 + (slot >> 6), lane = slot & 63;
        if (rb >= job.RB) continue;
        const int row = rb * 32 + (lane & 31), k0 = kb * 32 + 16 * (lane >> 5);
        uint32_t w[4] = {0, 0, 0, 0};
        if (via_lds) {
#pragma unroll
            for (int b = 0; b < 16; ++b) w[b >> 2] |= (uint32_t)tile[16 * (lane >> 5) + b][(slot >> 6) * 32 + (lane & 31)] << (8 * (b & 3));
        } else if (row < job.rows) {
            const uint8_t* p = job.src + (int64_t)row * job.s_r + (int64_t)k0 * job.s_k;
            if (k0 + 16 <= job.K && (((uintptr_t)p) & 15u) == 0) {
                const uint4 v = *reinterpret_cast<const uint4*>(p);
                w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
            } else {
#pragma unroll
                for (int b = 0; b < 16; ++b)
                    if (k0 + b < job.K) w[b >> 2] |= (uint32_t)p[b] << (8 * (b & 3));
            }
        }
        uint32_t hi[4] = {0, 0, 0, 0}, lo[4] = {0, 0, 0, 0};
#pragma unroll
        for (int b = 0; b < 16; ++b) {
            const uint32_t pat = (w[b >> 2] >> (8 * (b & 3))) & 0xFFu;
            const int v = tab[pat];  // -16384 for NaR: high digit -128, low digit 0
            hi[b >> 2] |= ((uint32_t)(v >> 7) & 0xFFu) << (8 * (b & 3));
            lo[b >> 2] |= ((uint32_t)v & 0x7Fu) << (8 * (b & 3));
        }
        uint4* out = reinterpret_cast<uint4*>(job.dst) + ((int64_t)(kb * job.RB + rb) * 2) * 64 + lane;
        out[0] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
        out[64] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
    }
}

// Ad / Bd: digit planes of p8_digits_kernel with RBA / RBB row blocks (multiples of 2 BI / 2 BJ) and KB k blocks (a
// multiple of PM_KSTEP).  Four waves as 2 x 2; a wave owns BI x BJ blocks of 32 x 32 outputs, the workgroup 64 BI x 64 BJ.
//
// SPLIT: workgroup (tile, z) reduces the kb_per_split k blocks from z kb_per_split on and leaves its 32-bit sums and
// its NaR flags in the workspace of a split reduction (ws: partial quires [z][M N], row flags [z][M], column flags
// [z][N]); the merging launch adds, rounds and stores.  For products with few output tiles and a long reduction.
template <int BI, int BJ, bool SPLIT = false>
__global__ __launch_bounds__(256, (BI * BJ == 4 ? 2 : BI * BJ == 2 ? 3 : 4)) void p8_mfma_gemm_kernel(
    const uint8_t* __restrict__ Ad, const uint8_t* __restrict__ Bd, int RBA, int RBB, int KB, const uint8_t* __restrict__ bias, void* __restrict__ C,
    int64_t ldc, int fout, int M, int N, int tiles_m, int tiles_n, int kb_per_split = 0, SplitWs ws = SplitWs{nullptr, nullptr, nullptr}) {
    constexpr int NA = 2 * BI * 2, NB = 2 * BJ * 2;  // runs of 1 KB (row block, digit) per k block and operand
    constexpr int TR = 64 * BI, TC = 64 * BJ;        // tile extents
    // [buffer][k block of the step][A runs, then B runs][lane]: 64 KB for 128 x 128 outputs
    __shared__ uint4 stage[2][PM_KSTEP][(NA + NB) * 64];

    const int t = threadIdx.x;
    const int lane = t & 63, w = __builtin_amdgcn_readfirstlane(t >> 6);  // the wave number, known to be uniform
    const int wy = w >> 1, wx = w & 1;

    // XCD-aware order: consecutive workgroup ids go round-robin to the 8 XCDs, so give each XCD a contiguous run of
    // tiles, walked in bands of 8 tile-rows, column by column inside a band (neighbours share operand panels in L2)
    const int nblk = tiles_m * tiles_n;
    int lid = blockIdx.x;
    if ((nblk & 7) == 0) lid = (blockIdx.x & 7) * (nblk >> 3) + (blockIdx.x >> 3);
    const int band = lid / (8 * tiles_n);
    const int band_rows = (tiles_m - band * 8) < 8 ? (tiles_m - band * 8) : 8;
    const int in_band = lid - band * 8 * tiles_n;
    const int tm = band * 8 + in_band % band_rows, tn = in_band / band_rows;

    // markers met in this lane's row of the row block / column of the column block this wave searches (its half of every k block)
    uint32_t row_nar = 0, col_nar = 0;
    pm_v16i hh[BI][BJ], xx[BI][BJ], ll[BI][BJ];
#pragma unroll
    for (int i = 0; i < BI; ++i)
#pragma unroll
        for (int j = 0; j < BJ; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) hh[i][j][r] = xx[i][j][r] = ll[i][j][r] = 0;

    // One step is PM_KSTEP (NA + NB) runs of 1 KB, each a run in the workspace too.  Every wave copies a quarter of them
    // straight into LDS: the load writes 16 bytes per lane at consecutive LDS addresses from a wave-uniform base, which
    // is exactly a run, and passes through no register.
    const uint4* ga = reinterpret_cast<const uint4*>(Ad) + (int64_t)tm * NA * 64;
    const uint4* gb = reinterpret_cast<const uint4*>(Bd) + (int64_t)tn * NB * 64;
    const int64_t a_kb = (int64_t)RBA * 2 * 64, b_kb = (int64_t)RBB * 2 * 64;  // words per k block
    constexpr int RUNS = PM_KSTEP * (NA + NB) / 4;  // per wave and step
    static_assert(PM_KSTEP * (NA + NB) % 4 == 0, "runs split evenly over the four waves");
    // Where this wave's runs come from and how far they move per step: wave-uniform, worked out once, so that the
    // loop issues its copies without a branch.  Run number kk (NA + NB) + sub is also its place in the buffer.
    const uint4* src[RUNS];
    int64_t adv[RUNS];
#pragma unroll
    for (int c = 0; c < RUNS; ++c) {
        const int run = w * RUNS + c;
        const int kk = run / (NA + NB), sub = run % (NA + NB);
        const bool isb = sub >= NA;
        src[c] = isb ? gb + kk * b_kb + (sub - NA) * 64 : ga + kk * a_kb + sub * 64;
        adv[c] = PM_KSTEP * (isb ? b_kb : a_kb);
        if (SPLIT) src[c] += (int64_t)blockIdx.y * kb_per_split * (isb ? b_kb : a_kb);
    }
    auto issue = [&](int buf) {
#pragma unroll
        for (int c = 0; c < RUNS; ++c) {
            uint4* dst = &stage[buf][0][0] + (w * RUNS + c) * 64;  // the same for every lane
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src[c] + lane),
                                             (__attribute__((address_space(3))) void*)dst, 16, 0, 0);
            src[c] += adv[c];
        }
    };

    // the two waves that share a row block (column block) split the search for NaR markers when a wave has two blocks
    // each way: wave (wy, wx) looks at its row block wx and its column block wy; with one block both waves look at it
    const int ia = BI == 2 ? wx : 0, jb = BJ == 2 ? wy : 0;

    issue(0);
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's runs are in LDS
    __syncthreads();
    int cur = 0;
    const int nkb = SPLIT ? kb_per_split : KB;
    for (int kb0 = 0; kb0 < nkb; kb0 += PM_KSTEP, cur ^= 1) {
        if (kb0 + PM_KSTEP < nkb) issue(cur ^ 1);  // the other buffer was last read one barrier ago
#pragma unroll
        for (int kk = 0; kk < PM_KSTEP; ++kk) {
            pm_v4i ah[BI], al[BI], bh[BJ], bl[BJ];
#pragma unroll
            for (int i = 0; i < BI; ++i) {
                ah[i] = __builtin_bit_cast(pm_v4i, stage[cur][kk][((BI * wy + i) * 2 + 0) * 64 + lane]);
                al[i] = __builtin_bit_cast(pm_v4i, stage[cur][kk][((BI * wy + i) * 2 + 1) * 64 + lane]);
            }
#pragma unroll
            for (int j = 0; j < BJ; ++j) {
                bh[j] = __builtin_bit_cast(pm_v4i, stage[cur][kk][(NA + (BJ * wx + j) * 2 + 0) * 64 + lane]);
                bl[j] = __builtin_bit_cast(pm_v4i, stage[cur][kk][(NA + (BJ * wx + j) * 2 + 1) * 64 + lane]);
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                row_nar |= pm_marker_bits((uint32_t)(ia ? ah[BI - 1][q] : ah[0][q]));
                col_nar |= pm_marker_bits((uint32_t)(jb ? bh[BJ - 1][q] : bh[0][q]));
            }
#pragma unroll
            for (int i = 0; i < BI; ++i)
#pragma unroll
                for (int j = 0; j < BJ; ++j) {
                    hh[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ah[i], bh[j], hh[i][j], 0, 0, 0);
                    xx[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ah[i], bl[j], xx[i][j], 0, 0, 0);
                    xx[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(al[i], bh[j], xx[i][j], 0, 0, 0);
                    ll[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(al[i], bl[j], ll[i][j], 0, 0, 0);
                }
        }
        // keep the wait behind the step's matrix instructions: they need no memory, and hoisting the barrier over them
        // would shorten the time the copies have to arrive
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the next step's runs of this wave are in LDS
        __syncthreads();
    }

    // ---- the three sums into the quire, round once, store ----
    // NaR: lanes l and l + 32 hold the two halves of the reduction of row (column) l % 32 of the block their wave
    // searched; the NaR flags of the tile's rows and columns meet in LDS (the staging buffers are free now).
    uint32_t* rowv = reinterpret_cast<uint32_t*>(&stage[0][0][0]);
    uint32_t* colv = rowv + TR;
    row_nar = (row_nar | (uint32_t)__shfl_xor((int)row_nar, 32)) & 0x80808080u;
    col_nar = (col_nar | (uint32_t)__shfl_xor((int)col_nar, 32)) & 0x80808080u;
    if (lane < 32) {
        rowv[(wy * BI + ia) * 32 + lane] = row_nar;  // with one block per wave both waves of the pair write the same flag
        colv[(wx * BJ + jb) * 32 + lane] = col_nar;
    }
    __syncthreads();
    if (SPLIT) {
        const int64_t z = blockIdx.y;
        // the first tile column stores the row flags of its tile row (the same in every column), the first tile row the
        // column flags: every entry is written, so the workspace needs no clearing
        if (tn == 0 && t < TR && tm * TR + t < M) ws.rowflag[z * M + tm * TR + t] = rowv[t];
        if (tm == 0 && t < TC && tn * TC + t < N) ws.colflag[z * N + tn * TC + t] = colv[t];
        uint32_t* lim = ws.limbs + z * (int64_t)M * N;
#pragma unroll
        for (int j = 0; j < BJ; ++j) {
            const int n = tn * TC + (wx * BJ + j) * 32 + (lane & 31);
            if (n >= N) continue;
#pragma unroll
            for (int i = 0; i < BI; ++i) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int m = tm * TR + (wy * BI + i) * 32 + (r & 3) + 8 * (r >> 2) + 4 * (lane >> 5);
                    if (m < M) lim[(int64_t)m * N + n] = ((uint32_t)hh[i][j][r] << 14) + ((uint32_t)xx[i][j][r] << 7) + (uint32_t)ll[i][j][r];
                }
            }
        }
        return;
    }
    rowv += wy * 32 * BI;
    colv += wx * 32 * BJ;
    const int m_base = tm * TR + wy * 32 * BI, n_base = tn * TC + wx * 32 * BJ;
#pragma unroll
    for (int j = 0; j < BJ; ++j) {
        const int n = n_base + j * 32 + (lane & 31);
        if (n >= N) continue;
        bool cnar = colv[j * 32 + (lane & 31)] != 0;
        int32_t badd = 0;
        if (bias) {
            const uint32_t bp = bias[n];
            if (bp == 0x80u) cnar = true;
            else badd = (int32_t)Arith<P8>::stage(bp) << P8::MAXS;  // + bias * 1
        }
#pragma unroll
        for (int i = 0; i < BI; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int lr = i * 32 + (r & 3) + 8 * (r >> 2) + 4 * (lane >> 5);
                const int m = m_base + lr;
                if (m >= M) continue;
                const uint32_t q = ((uint32_t)hh[i][j][r] << 14) + ((uint32_t)xx[i][j][r] << 7) + (uint32_t)ll[i][j][r] + (uint32_t)badd;
                const bool nar = cnar || rowv[lr] != 0;
                const int64_t at = (int64_t)m * ldc + n;
                if (fout == 0) {
                    ((uint8_t*)C)[at] = (uint8_t)(nar ? 0x80u : p8_round_quire((int32_t)q));
                } else {
                    const uint32_t q1[1] = {q};
                    round_store<QuireAccum<P8>, 1>(q1, nar, fout, C, at);
                }
            }
        }
    }
}

// ---- host side ----

struct P8MfmaLayout {
    int BI, BJ;        // blocks of 32 per wave each way: the workgroup tile is 64 BI x 64 BJ
    int RBA, RBB, KB;  // padded extents in blocks of 32
    int splits, kb_per_split;  // slices of the reduction (1: none) and their length in k blocks; KB = splits * kb_per_split
    size_t a_bytes, b_bytes, part_bytes;
    size_t total() const { return a_bytes + b_bytes + part_bytes; }
};

// Slices for a product with fewer than PM_MIN_TILES tiles of 64 x 64: about two workgroups per compute unit, each
// slice at least PM_MIN_KB_SPLIT k blocks long; fewer than 2 means the split form does not serve the shape.
inline int64_t p8_mfma_slices(int64_t M, int64_t N, int64_t K) {
    const int64_t tiles = ((M + 63) / 64) * ((N + 63) / 64), kb_total = (K + 31) / 32;
    int64_t s = (PM_MIN_WGS + tiles - 1) / tiles;
    if (s > kb_total / PM_MIN_KB_SPLIT) s = kb_total / PM_MIN_KB_SPLIT;
    return s;
}

inline bool p8_mfma_fits(int64_t M, int64_t N, int64_t K) {
    if (K < 256 || M * N * K < PM_MIN_MNK || M > ((int64_t)1 << 20) || N > ((int64_t)1 << 20) || K > ((int64_t)1 << 20)) return false;
    const int64_t tiles = ((M + 63) / 64) * ((N + 63) / 64);
    if (tiles >= PM_MIN_TILES) return M >= PM_MIN_MN && N >= PM_MIN_MN;
    return M >= PM_MIN_MN && N >= PM_MIN_MN && M * N < ((int64_t)1 << 24) && p8_mfma_slices(M, N, K) >= 2;
}

// The largest tile that still gives every compute unit two workgroups; 64 x 64 otherwise.
inline P8MfmaLayout p8_mfma_layout(int64_t M, int64_t N, int64_t K) {
    auto cdiv = [](int64_t a, int64_t b) { return (a + b - 1) / b; };
    P8MfmaLayout l;
    l.BI = l.BJ = 1;
    if (cdiv(M, 128) * cdiv(N, 128) >= PM_MIN_WGS) l.BI = l.BJ = 2;
    else if (M >= N && cdiv(M, 128) * cdiv(N, 64) >= PM_MIN_WGS) l.BI = 2;
    else if (cdiv(M, 64) * cdiv(N, 128) >= PM_MIN_WGS) l.BJ = 2;
    else if (cdiv(M, 128) * cdiv(N, 64) >= PM_MIN_WGS) l.BI = 2;
    l.RBA = (int)cdiv(M, 64 * l.BI) * 2 * l.BI;
    l.RBB = (int)cdiv(N, 64 * l.BJ) * 2 * l.BJ;
    l.KB = (int)cdiv(K, 32 * PM_KSTEP) * PM_KSTEP;
    l.splits = 1;
    l.kb_per_split = l.KB;
    l.part_bytes = 0;
    if (cdiv(M, 64) * cdiv(N, 64) < PM_MIN_TILES) {  // few outputs, long reduction: 64 x 64 tiles (chosen above), slices of k blocks
        const int64_t kb_total = cdiv(K, 32);
        int64_t splits = p8_mfma_slices(M, N, K);
        if (splits < 1) splits = 1;
        int64_t kbps = cdiv(cdiv(kb_total, splits), PM_KSTEP) * PM_KSTEP;
        splits = cdiv(kb_total, kbps);
        l.splits = (int)splits;
        l.kb_per_split = (int)kbps;
        l.KB = (int)(splits * kbps);
        l.part_bytes = splits > 1 ? ((size_t)splits * M * N + (size_t)splits * (M + N)) * 4 : 0;
    }
    l.a_bytes = (size_t)l.KB * l.RBA * 2048;
    l.b_bytes = (size_t)l.KB * l.RBB * 2048;
    return l;
}

inline hipError_t launch_p8_mfma_gemm(hipStream_t stream, int transA, int transB, const uint8_t* A, int64_t lda, const uint8_t* B, int64_t ldb,
                                      const uint8_t* bias, void* C, int64_t ldc, int fout, int64_t M, int64_t N, int64_t K, void* workspace) {
    const P8MfmaLayout l = p8_mfma_layout(M, N, K);
    uint8_t* base = (uint8_t*)workspace;
    uint8_t* Ad = base;
    uint8_t* Bd = base + l.a_bytes;
    // op(A)[m,k] is A[m * lda + k] unless transA; op(B)[k,n] is B[k * ldb + n] unless transB
    P8DigitJob ja{A, transA ? (int64_t)1 : lda, transA ? lda : (int64_t)1, (int)M, (int)K, Ad, l.RBA, l.KB};
    P8DigitJob jb{B, transB ? ldb : (int64_t)1, transB ? (int64_t)1 : ldb, (int)N, (int)K, Bd, l.RBB, l.KB};
    const unsigned blocks0 = (unsigned)((l.RBA + 7) / 8) * (unsigned)l.KB, blocks1 = (unsigned)((l.RBB + 7) / 8) * (unsigned)l.KB;
    hipLaunchKernelGGL(p8_digits_kernel<0>, dim3(blocks0 + blocks1), dim3(256), 0, stream, ja, jb, blocks0);
    PNN_CHECK_LAUNCH();
    const int tiles_m = l.RBA / (2 * l.BI), tiles_n = l.RBB / (2 * l.BJ);
    if (l.splits > 1) {
        SplitWs ws;
        ws.limbs = reinterpret_cast<uint32_t*>(base + l.a_bytes + l.b_bytes);
        ws.rowflag = ws.limbs + (size_t)l.splits * M * N;
        ws.colflag = ws.rowflag + (size_t)l.splits * M;
        hipLaunchKernelGGL((p8_mfma_gemm_kernel<1, 1, true>), dim3((unsigned)(tiles_m * tiles_n), (unsigned)l.splits), dim3(256), 0, stream, Ad, Bd, l.RBA,
                           l.RBB, l.KB, (const uint8_t*)nullptr, (void*)nullptr, (int64_t)0, fout, (int)M, (int)N, tiles_m, tiles_n, l.kb_per_split, ws);
        PNN_CHECK_LAUNCH();
        RowMajorOut out{ldc};
        return launch_split_merge<P8, RowMajorOut>(stream, ws, l.splits, M, N, bias, C, fout, out);
    }
    const dim3 grid((unsigned)(tiles_m * tiles_n));
#define PNN_PM_LAUNCH(bi, bj)                                                                                                                    \
    hipLaunchKernelGGL((p8_mfma_gemm_kernel<bi, bj>), grid, dim3(256), 0, stream, Ad, Bd, l.RBA, l.RBB, l.KB, bias, C, ldc, fout, (int)M, (int)N, \
                       tiles_m, tiles_n, 0, SplitWs{nullptr, nullptr, nullptr})
    if (l.BI == 2 && l.BJ == 2) PNN_PM_LAUNCH(2, 2);
    else if (l.BI == 2) PNN_PM_LAUNCH(2, 1);
    else if (l.BJ == 2) PNN_PM_LAUNCH(1, 2);
    else PNN_PM_LAUNCH(1, 1);
#undef PNN_PM_LAUNCH
    return hipGetLastError();
}

}  // namespace pnn
