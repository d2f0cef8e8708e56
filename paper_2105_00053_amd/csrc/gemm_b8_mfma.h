// posit(8,1) / posit(8,2) matrix product with the exact quire (paper Sec. 2, Sec. 3.3; the formats of Sec. 4) on the
// integer matrix cores: the digit decomposition of gemm_p8_mfma.h carried over the whole range of the format.
//
// These formats have few significand bits and a wide range.  In units of minpos a decoded posit(8,2) is an integer v of
// at most 49 bits plus sign (a 4-bit significand over 49 binades), a posit(8,1) one of 25 bits; written in ND = 8
// (resp. 4) base-128 digits that all carry the sign of v, v = sum_i d_i 128^i with d_i in [-127, 127], at most two
// adjacent digits are non-zero.  A product is then
//     a b = sum_s 128^s  sum_{i + j = s} a_i b_j ,
// 2 ND - 1 int32 sums per output fed by ND^2 int8 products per posit product, combined once after the reduction into
// the quire (exact: every partial sum stays below 2^31 for reductions of up to 8192, which is what this kernel takes).
// No window and no outliers: the whole range is covered.
//
// Most of the ND^2 digit products multiply zeros.  The digit kernel therefore writes, per (k block of 32, row block of
// 32) one byte whose bit i says whether digit plane i holds anything, and the product kernel skips every digit pair one
// of whose planes is empty: data spread over a few binades (activations, weights, gradients of one layer) fills two to
// four adjacent planes, 4 to 16 of the 64 products.  The skipping is by whole planes of a block, uniform for a wave,
// and changes nothing in the result.
//
// Layout of the rewritten operands: [k block][row block][digit][lane][16 bytes] in the lane order of
// v_mfma_i32_32x32x32_i8 (see gemm_p8_mfma.h), NaR as the top digit -128, which no value has (|d_i| <= 127, and the
// top digit of a value is at most 8 in magnitude).
#pragma once

#include "gemm_p8_mfma.h"

namespace pnn {

template <class F>
struct B8Mfma {
    static constexpr int BITS = 2 * F::MAXS + 2;         // magnitude up to 2^(2 MAXS) and the sign
    static constexpr int ND = (BITS + 6) / 7;            // base-128 digits
    static constexpr int NC = 2 * ND - 1;                // digit positions of a product
    static constexpr int MAXK = 8192;                    // ND * 2^14 * K < 2^31
    // When all that an operand holds lies in a few adjacent digit planes (the usual case for the tensors of one layer: a
    // few binades around one scale), a product kernel over WINA or WINB planes serves: posit(8,2) 4 or 5 planes, 7 or 9
    // sums instead of 15 (112 / 144 registers, three / two waves per SIMD instead of one); posit(8,1) 3 planes, 5 sums
    // instead of 7.  0: no such variant.
    static constexpr int WINA = ND > 5 ? 4 : (ND == 4 ? 3 : 0), WINB = ND > 5 ? 5 : 0;
    // below these sizes the launches of the union and of one more product kernel cost more than the variant saves
    static constexpr int64_t WINA_MIN_MNK = ND > 5 ? 0 : (int64_t)1 << 32, WINB_MIN_MNK = (int64_t)1 << 31;
    static_assert(ND <= 8, "one mask byte per block");
    static_assert((int64_t)ND * 16384 * MAXK <= ((int64_t)1 << 31), "int32 sums");
};

constexpr int64_t B8_NAR_VALUE = (int64_t)1 << 62;  // stands for NaR in the table of values (no value is that large)

// The value of a pattern in units of minpos.
template <class F>
__device__ __forceinline__ int64_t b8_fixed(uint32_t p) {
    if (p == 0) return 0;
    if (p == F::NAR) return B8_NAR_VALUE;
    bool neg;
    uint32_t sig;
    int sh;
    decode_fixed<F>(p, neg, sig, sh);
    const int64_t v = (int64_t)sig << sh;
    return neg ? -v : v;
}

struct B8DigitJob {
    const uint8_t* src;
    int64_t s_r, s_k;   // element (row, k) at src[row * s_r + k * s_k]; one of the two is 1
    int rows, K;
    uint8_t* dst;       // [KB][RB][ND][64][16]
    uint8_t* mask;      // [KB][RB]: bit i set when digit plane i of the block holds a non-zero byte
    int RB, KB;
};

// Both operands in one launch: the first blocks0 workgroups take job0, the rest job1.  A workgroup handles one k block
// and eight row blocks (one wave per row block and pass), an operand stored reduction-index-major goes through an LDS tile.
template <class F>
__global__ __launch_bounds__(256) void b8_digits_kernel(B8DigitJob job0, B8DigitJob job1, unsigned blocks0) {
    constexpr int ND = B8Mfma<F>::ND;
    __shared__ int64_t tab[256];
    __shared__ __attribute__((aligned(16))) uint8_t tile[32][256];
    const int t = threadIdx.x;
    tab[t] = b8_fixed<F>((uint32_t)t);
    const bool first = blockIdx.x < blocks0;
    const B8DigitJob& job = first ? job0 : job1;
    const unsigned lin = first ? blockIdx.x : blockIdx.x - blocks0;
    const unsigned gx = (unsigned)((job.RB + 7) / 8);
    const int bx = (int)(lin % gx), kb = (int)(lin / gx);
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
    }
    __syncthreads();  // the table, and the tile if there is one
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int slot = t + 256 * h;
        const int rb = bx * 8 + (slot >> 6), lane = slot & 63;  // a wave: one row block
        if (rb >= job.RB) continue;
        const int row = rb * 32 + (lane & 31), k0 = kb * 32 + 16 * (lane >> 5);
        uint32_t pat[16];
#pragma unroll
        for (int b = 0; b < 16; ++b) pat[b] = 0;
        if (via_lds) {
#pragma unroll
            for (int b = 0; b < 16; ++b) pat[b] = tile[16 * (lane >> 5) + b][(slot >> 6) * 32 + (lane & 31)];
        } else if (row < job.rows) {
            const uint8_t* p = job.src + (int64_t)row * job.s_r + (int64_t)k0 * job.s_k;
            if (k0 + 16 <= job.K && (((uintptr_t)p) & 15u) == 0) {
                const uint4 v = *reinterpret_cast<const uint4*>(p);
                const uint32_t wv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int b = 0; b < 16; ++b) pat[b] = (wv[b >> 2] >> (8 * (b & 3))) & 0xFFu;
            } else {
#pragma unroll
                for (int b = 0; b < 16; ++b)
                    if (k0 + b < job.K) pat[b] = p[b];
            }
        }
        uint32_t dig[ND][4];
#pragma unroll
        for (int i = 0; i < ND; ++i)
#pragma unroll
            for (int q = 0; q < 4; ++q) dig[i][q] = 0;
#pragma unroll
        for (int b = 0; b < 16; ++b) {
            const int64_t v = tab[pat[b]];
            if (v == B8_NAR_VALUE) {
                dig[ND - 1][b >> 2] |= 0x80u << (8 * (b & 3));  // the marker: top digit -128 above zeros
                continue;
            }
            const bool neg = v < 0;
            const uint64_t mag = (uint64_t)(neg ? -v : v);
#pragma unroll
            for (int i = 0; i < ND; ++i) {
                const int d = (int)((mag >> (7 * i)) & 0x7Fu);
                dig[i][b >> 2] |= ((uint32_t)(neg ? -d : d) & 0xFFu) << (8 * (b & 3));
            }
        }
        uint4* out = reinterpret_cast<uint4*>(job.dst) + ((int64_t)(kb * job.RB + rb) * ND) * 64 + lane;
        uint32_t m = 0;
#pragma unroll
        for (int i = 0; i < ND; ++i) {
            // an empty plane is not written: the mask keeps the product kernel from copying or reading it
            if (__ballot((dig[i][0] | dig[i][1] | dig[i][2] | dig[i][3]) != 0) != 0) {
                m |= 1u << i;
                out[i * 64] = make_uint4(dig[i][0], dig[i][1], dig[i][2], dig[i][3]);
            }
        }
        if (lane == 0) job.mask[(int64_t)kb * job.RB + rb] = (uint8_t)m;
    }
}

// all[o] = the OR of the n[o] mask bytes of operand o (o = blockIdx.x: 0, 1): which digit planes the operand uses at all.
// m0 / m1 are 16-byte aligned.
template <int UNUSED = 0>
__global__ __launch_bounds__(1024) void b8_mask_union_kernel(const uint8_t* __restrict__ m0, int64_t n0, const uint8_t* __restrict__ m1, int64_t n1,
                                                             uint32_t* __restrict__ all) {
    __shared__ uint32_t part[16];
    const uint8_t* m = blockIdx.x == 0 ? m0 : m1;
    const int64_t n = blockIdx.x == 0 ? n0 : n1;
    const int t = threadIdx.x;
    uint32_t u = 0;
    const int64_t n16 = n >> 4;
    for (int64_t i = t; i < n16; i += 1024) {
        const uint4 v = reinterpret_cast<const uint4*>(m)[i];
        u |= v.x | v.y | v.z | v.w;
    }
    u |= u >> 16;
    u |= u >> 8;
    for (int64_t i = (n16 << 4) + t; i < n; i += 1024) u |= m[i];
    u &= 0xFFu;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) u |= (uint32_t)__shfl_xor((int)u, d);
    if ((t & 63) == 0) part[t >> 6] = u;
    __syncthreads();
    if (t == 0) {
        uint32_t r = 0;
        for (int i = 0; i < 16; ++i) r |= part[i];
        all[blockIdx.x] = r;
    }
}

// Ad / Bd: digit planes with RBA / RBB row blocks (multiples of 2) and KB k blocks; ma / mb their masks.
// 64 x 64 outputs per workgroup of four waves (2 x 2), one block of 32 x 32 and its sums per wave.
//
// NP = ND: every digit plane takes part, 2 ND - 1 sums.  NP < ND: the planes oa .. oa + NP - 1 of A and
// ob .. ob + NP - 1 of B, where oa / ob is the lowest plane that the operand uses anywhere; sum s then stands at digit
// position s + oa + ob.  all[0] / all[1] (the OR of the operand's masks) gives the span of planes the operands use; the
// kernels of several NP are launched one after the other, each told the next smaller NP launched (below, 0 if none),
// and only the smallest one that covers the span does the work: the others return at once.
template <class F, int NP>
__global__ __launch_bounds__(256, ((2 * NP - 1) * 16 > 160 ? 1 : 2)) void b8_mfma_gemm_kernel(
    const uint8_t* __restrict__ Ad, const uint8_t* __restrict__ Bd, const uint8_t* __restrict__ ma, const uint8_t* __restrict__ mb,
    const uint32_t* __restrict__ all, int RBA, int RBB, int KB, const uint8_t* __restrict__ bias, void* __restrict__ C, int64_t ldc, int fout, int M, int N,
    int tiles_m, int tiles_n, int below) {
    constexpr int ND = B8Mfma<F>::ND, NC = 2 * NP - 1;
    int oa = 0, ob = 0;
    if constexpr (B8Mfma<F>::WINA != 0) {
        const uint32_t ga = __builtin_amdgcn_readfirstlane(all[0]), gb = __builtin_amdgcn_readfirstlane(all[1]);
        const int la = ga ? __builtin_ctz(ga) : 0, lb = gb ? __builtin_ctz(gb) : 0;
        const uint32_t u = (ga >> la) | (gb >> lb);
        const int span = u ? 32 - __builtin_clz(u) : 0;  // planes from the lowest to the highest one in use
        if (below > 0 && span <= below) return;          // a smaller kernel serves
        if constexpr (NP < ND) {
            if (span > NP) return;                       // a larger one
            oa = la;
            ob = lb;
        }
    }
    constexpr int RPB = 4 * NP;  // runs of 1 KB per k block: two row blocks and two column blocks of NP planes
    typedef QuireAccum<F> AR;
    constexpr int L = AR::L;
    __shared__ uint4 stage[2][RPB * 64];

    const int t = threadIdx.x;
    const int lane = t & 63, w = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wy = w >> 1, wx = w & 1;
    const int tm = blockIdx.x % tiles_m, tn = blockIdx.x / tiles_m;

    pm_v16i acc[NC];
#pragma unroll
    for (int s = 0; s < NC; ++s)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[s][r] = 0;

    // copies: wave w takes ND of the k block's 4 ND runs (A: row block 0, 1; B: column block 0, 1), wave-uniform addresses
    const int64_t a_kb = (int64_t)RBA * ND * 64, b_kb = (int64_t)RBB * ND * 64;  // words per k block
    const uint4* src = (w < 2) ? reinterpret_cast<const uint4*>(Ad) + ((int64_t)tm * 2 + w) * ND * 64
                               : reinterpret_cast<const uint4*>(Bd) + ((int64_t)tn * 2 + (w - 2)) * ND * 64;
    const int64_t adv = (w < 2) ? a_kb : b_kb;
    const int oc = (w < 2) ? oa : ob;  // the first plane that takes part, of the operand this wave copies
    src += oc * 64;
    // the empty planes of the block are not copied either (nobody reads them): mk is the mask of the block being copied
    auto issue = [&](int buf, uint32_t mk) {
        mk >>= oc;
#pragma unroll
        for (int c = 0; c < NP; ++c)
            if (mk & (1u << c))
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + c * 64 + lane),
                                                 (__attribute__((address_space(3))) void*)(&stage[buf][0] + (w * NP + c) * 64), 16, 0, 0);
        src += adv;
    };
    // masks, one k block ahead (every lane loads the same byte): of the row block and the column block this wave
    // multiplies, and of the block it copies (waves 0, 1: row blocks 0, 1 of A; waves 2, 3: column blocks 0, 1 of B)
    const uint8_t* pma = ma + (tm * 2 + wy);
    const uint8_t* pmb = mb + (tn * 2 + wx);
    const uint8_t* pmc = (w < 2) ? ma + (tm * 2 + w) : mb + (tn * 2 + (w - 2));
    const int64_t mc_kb = (w < 2) ? RBA : RBB;
    uint32_t mka_next = pma[0], mkb_next = pmb[0];
    uint32_t mkc_next = KB > 1 ? pmc[mc_kb] : 0u;  // of k block 1

    uint32_t row_nar = 0, col_nar = 0;
    issue(0, __builtin_amdgcn_readfirstlane((uint32_t)pmc[0]));
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    __syncthreads();
    int cur = 0;
    for (int kb = 0; kb < KB; ++kb, cur ^= 1) {
        const uint32_t mka = __builtin_amdgcn_readfirstlane(mka_next) >> oa, mkb = __builtin_amdgcn_readfirstlane(mkb_next) >> ob;
        if (kb + 1 < KB) {
            issue(cur ^ 1, __builtin_amdgcn_readfirstlane(mkc_next));  // the other buffer was last read one barrier ago
            mka_next = pma[(int64_t)(kb + 1) * RBA];
            mkb_next = pmb[(int64_t)(kb + 1) * RBB];
            if (kb + 2 < KB) mkc_next = pmc[(int64_t)(kb + 2) * mc_kb];
        }
        const uint4* sa = &stage[cur][0] + (wy * NP) * 64 + lane;
        const uint4* sb = &stage[cur][0] + ((2 + wx) * NP) * 64 + lane;
        if constexpr (ND == 8 && NP != 5) {
            // the planes of B in registers, every plane of A read once
            pm_v4i b[NP];
#pragma unroll
            for (int j = 0; j < NP; ++j) {
                if (!(mkb & (1u << j))) continue;
                b[j] = __builtin_bit_cast(pm_v4i, sb[j * 64]);
                if (ob + j == ND - 1) {  // the plane of the NaR marker
#pragma unroll
                    for (int q = 0; q < 4; ++q) col_nar |= pm_marker_bits((uint32_t)b[j][q]);
                }
            }
#pragma unroll
            for (int i = 0; i < NP; ++i) {
                if (!(mka & (1u << i))) continue;
                const pm_v4i a = __builtin_bit_cast(pm_v4i, sa[i * 64]);
                if (oa + i == ND - 1) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) row_nar |= pm_marker_bits((uint32_t)a[q]);
                }
#pragma unroll
                for (int j = 0; j < NP; ++j)
                    if (mkb & (1u << j)) acc[i + j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b[j], acc[i + j], 0, 0, 0);
            }
        } else {
            // one plane of B and one of A in registers at a time; the planes of A are read again for every plane of B
            // (LDS has the time).  The registers saved are a third wave per SIMD for the kernel of nine sums, and the
            // posit(8,1) kernels run 5 % faster this way (the posit(8,2) kernel of seven sums 2 % slower, and the one
            // over all planes has a single wave per SIMD to wait for its reads: above).
#pragma unroll
            for (int j = 0; j < NP; ++j) {
                if (!(mkb & (1u << j))) continue;
                const pm_v4i b = __builtin_bit_cast(pm_v4i, sb[j * 64]);
                if (ob + j == ND - 1) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) col_nar |= pm_marker_bits((uint32_t)b[q]);
                }
#pragma unroll
                for (int i = 0; i < NP; ++i) {
                    if (!(mka & (1u << i))) continue;
                    const pm_v4i a = __builtin_bit_cast(pm_v4i, sa[i * 64]);
                    if (oa + i == ND - 1) {
#pragma unroll
                        for (int q = 0; q < 4; ++q) row_nar |= pm_marker_bits((uint32_t)a[q]);
                    }
                    acc[i + j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[i + j], 0, 0, 0);
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the next k block's runs of this wave are in LDS
        __syncthreads();
    }

    // ---- the sums into the quire, round once, store ----
    uint32_t* rowv = reinterpret_cast<uint32_t*>(&stage[0][0]);
    uint32_t* colv = rowv + 64;
    row_nar = (row_nar | (uint32_t)__shfl_xor((int)row_nar, 32)) & 0x80808080u;
    col_nar = (col_nar | (uint32_t)__shfl_xor((int)col_nar, 32)) & 0x80808080u;
    if (lane < 32) {
        if (wx == 0) rowv[wy * 32 + lane] = row_nar;  // the two waves of a row block saw the same rows
        if (wy == 0) colv[wx * 32 + lane] = col_nar;
    }
    __syncthreads();
    const int n = tn * 64 + wx * 32 + (lane & 31);
    if (n >= N) return;
    bool cnar = colv[wx * 32 + (lane & 31)] != 0;
    uint32_t bp = 0;
    if (bias) {
        bp = bias[n];
        if (bp == F::NAR) cnar = true;
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int lr = (r & 3) + 8 * (r >> 2) + 4 * (lane >> 5);
        const int m = tm * 64 + wy * 32 + lr;
        if (m >= M) continue;
        // the sums at their digit positions (shifts known at compile time), then the offset of the window: the quire,
        // modulo 2^(32 L) like every addition into it
        uint32_t q[L];
        if constexpr (L == 4) {
            __int128 v = 0;
#pragma unroll
            for (int s = 0; s < NC; ++s) v += (__int128)acc[s][r] << (7 * s);
            const unsigned __int128 x = (unsigned __int128)v << (7 * (oa + ob));
            q[0] = (uint32_t)x;
            q[1] = (uint32_t)(x >> 32);
            q[2] = (uint32_t)(x >> 64);
            q[3] = (uint32_t)(x >> 96);
        } else {
            static_assert(L == 2, "64-bit or 128-bit quire");
            uint64_t v = 0;
#pragma unroll
            for (int s = 0; s < NC; ++s) v += (uint64_t)(int64_t)acc[s][r] << (7 * s);
            const uint64_t x = v << (7 * (oa + ob));
            q[0] = (uint32_t)x;
            q[1] = (uint32_t)(x >> 32);
        }
        if (bias && bp != F::NAR) AR::add_bias(q, bp);
        const bool nar = cnar || rowv[wy * 32 + lr] != 0;
        round_store<AR, L>(q, nar, fout, C, (int64_t)m * ldc + n);
    }
}

// ---- host side ----

template <class F>
struct B8MfmaLayout {
    int RBA, RBB, KB;
    size_t a_bytes, b_bytes, ma_bytes, mb_bytes;
    size_t total() const { return a_bytes + b_bytes + ma_bytes + mb_bytes + 256; }  // and the two words of all masks
};

template <class F>
inline bool b8_mfma_fits(int64_t M, int64_t N, int64_t K) {
    return M >= 128 && N >= 128 && K >= 256 && K <= B8Mfma<F>::MAXK && M * N * K >= ((int64_t)1 << 25) && ((M + 63) / 64) * ((N + 63) / 64) >= 32 &&
           M <= ((int64_t)1 << 20) && N <= ((int64_t)1 << 20);
}

template <class F>
inline B8MfmaLayout<F> b8_mfma_layout(int64_t M, int64_t N, int64_t K) {
    constexpr int ND = B8Mfma<F>::ND;
    B8MfmaLayout<F> l;
    l.RBA = (int)((M + 63) / 64) * 2;
    l.RBB = (int)((N + 63) / 64) * 2;
    l.KB = (int)((K + 31) / 32);
    l.a_bytes = (size_t)l.KB * l.RBA * ND * 1024;
    l.b_bytes = (size_t)l.KB * l.RBB * ND * 1024;
    l.ma_bytes = ((size_t)l.KB * l.RBA + 255) / 256 * 256;
    l.mb_bytes = ((size_t)l.KB * l.RBB + 255) / 256 * 256;
    return l;
}

template <class F>
inline hipError_t launch_b8_mfma_gemm(hipStream_t stream, int transA, int transB, const uint8_t* A, int64_t lda, const uint8_t* B, int64_t ldb,
                                      const uint8_t* bias, void* C, int64_t ldc, int fout, int64_t M, int64_t N, int64_t K, void* workspace) {
    const B8MfmaLayout<F> l = b8_mfma_layout<F>(M, N, K);
    uint8_t* base = (uint8_t*)workspace;
    uint8_t* Ad = base;
    uint8_t* Bd = Ad + l.a_bytes;
    uint8_t* ma = Bd + l.b_bytes;
    uint8_t* mb = ma + l.ma_bytes;
    uint32_t* all = (uint32_t*)(mb + l.mb_bytes);
    // op(A)[m,k] is A[m * lda + k] unless transA; op(B)[k,n] is B[k * ldb + n] unless transB
    B8DigitJob ja{A, transA ? (int64_t)1 : lda, transA ? lda : (int64_t)1, (int)M, (int)K, Ad, ma, l.RBA, l.KB};
    B8DigitJob jb{B, transB ? ldb : (int64_t)1, transB ? (int64_t)1 : ldb, (int)N, (int)K, Bd, mb, l.RBB, l.KB};
    const unsigned blocks0 = (unsigned)((l.RBA + 7) / 8) * (unsigned)l.KB, blocks1 = (unsigned)((l.RBB + 7) / 8) * (unsigned)l.KB;
    hipLaunchKernelGGL(b8_digits_kernel<F>, dim3(blocks0 + blocks1), dim3(256), 0, stream, ja, jb, blocks0);
    PNN_CHECK_LAUNCH();
    const int tiles_m = l.RBA / 2, tiles_n = l.RBB / 2;
    constexpr int ND = B8Mfma<F>::ND, WINA = B8Mfma<F>::WINA, WINB = B8Mfma<F>::WINB;
    const dim3 grid((unsigned)(tiles_m * tiles_n));
    int below = 0;
    if constexpr (WINA != 0) if (M * N * K >= B8Mfma<F>::WINA_MIN_MNK) {
        hipLaunchKernelGGL(b8_mask_union_kernel<0>, dim3(2), dim3(1024), 0, stream, ma, (int64_t)l.KB * l.RBA, mb, (int64_t)l.KB * l.RBB, all);
        PNN_CHECK_LAUNCH();
        hipLaunchKernelGGL((b8_mfma_gemm_kernel<F, WINA>), grid, dim3(256), 0, stream, Ad, Bd, ma, mb, all, l.RBA, l.RBB, l.KB, bias, C, ldc, fout, (int)M,
                           (int)N, tiles_m, tiles_n, 0);
        PNN_CHECK_LAUNCH();
        below = WINA;
        if constexpr (WINB != 0) {
            if (M * N * K >= B8Mfma<F>::WINB_MIN_MNK) {
                hipLaunchKernelGGL((b8_mfma_gemm_kernel<F, WINB>), grid, dim3(256), 0, stream, Ad, Bd, ma, mb, all, l.RBA, l.RBB, l.KB, bias, C, ldc, fout,
                                   (int)M, (int)N, tiles_m, tiles_n, WINA);
                PNN_CHECK_LAUNCH();
                below = WINB;
            }
        }
    }
    hipLaunchKernelGGL((b8_mfma_gemm_kernel<F, ND>), grid, dim3(256), 0, stream, Ad, Bd, ma, mb, all, l.RBA, l.RBB, l.KB, bias, C, ldc, fout, (int)M, (int)N,
                       tiles_m, tiles_n, below);
    return hipGetLastError();
}

}  // namespace pnn
