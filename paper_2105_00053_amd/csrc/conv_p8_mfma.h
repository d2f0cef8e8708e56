// posit<8,0> convolution, forward and backward-data, with the 32-bit quire of Table 1 (paper Sec. 2, Sec. 3.1,
// Sec. 3.3) on the integer matrix cores: the implicit-GEMM form of gemm_p8_mfma.h.
//
// Rows of the product are output channels, columns are output positions (n, oh, ow), the reduction runs over
// (tap, input channel).  The arithmetic is that of the matrix product: two base-128 digits per decoded operand, four
// int8 products and three int32 sums per posit product, exact modulo 2^32, combined and rounded once.
//
// The matrix instruction takes, per lane, 16 consecutive reduction indices of one column.  With the reduction ordered
// tap-major, channel-minor these are 16 consecutive channels of ONE input pixel, so a first launch rewrites the input
// tensor as digit planes in pixel-major order, [pixel (n, h, w)][group of 16 channels][digit][16 bytes], and the
// product kernel gathers: every lane of a copy names its own 16 bytes (the pixel its column reads for that tap, or a
// block of zeros where the tap falls into the padding or beyond the tensor) and the copy lands in LDS in lane order,
// which is the operand layout.  Nothing is unfolded in memory: the input is read where it lies, once per tap, mostly
// from L2.  The weights are rewritten (in the same launch) into the row-block layout of the matrix kernel with the same
// reduction order; for backward-data they are taken transposed and flipped, NaR as zero (the outputs a NaR weight
// reaches are marked by the pass that follows, as for the other backward-data kernels).
//
// These two passes: stride 1 only.  Backward-weight, whose reduction runs over images and positions, is the second half
// of this file.
#pragma once

#include "gemm_p8_mfma.h"

namespace pnn {

constexpr int PCM_MAXK16 = 512;  // most (tap, channel group) pairs, padding included (4 KB of LDS)
constexpr int PCM_STAGES = 4;    // k blocks in flight per workgroup

// s_waitcnt immediate: at most n vector-memory operations outstanding, the other counters unconstrained
constexpr int pcm_vmcnt(int n) { return (n & 0xF) | ((n >> 4) << 14) | 0x0F70; }

// The barrier of the ring: the bare instruction.  __syncthreads() puts a fence in front of it that waits for EVERY
// outstanding copy of the wave, the ones running ahead included, which would shorten the ring to one block.  What the
// ring needs holds without a fence: a wave's copies of the block it is about to read have landed (the counted wait in
// front of the barrier), and every wave's LDS reads of the block about to be overwritten have returned (their data was
// consumed by matrix instructions earlier in program order; nothing may be scheduled across the barrier).
__device__ __forceinline__ void pcm_ring_barrier() {
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

struct P8ConvMfmaPlan {
    bool ok;
    int which;                 // 0 forward, 1 backward-data
    int NI, CI, HI, WI;        // the gathered tensor: x (forward) or dy (backward-data)
    int HO, WO, MO;            // output extents per image and output channels
    int R, S, offh, offw;      // tap (r, s) of output (oh, ow) reads input (oh + r - offh, ow + s - offw)
    int WK, WC;                // the weight tensor is [WK][WC][R][S]
    int Cg, K16, KB;           // channel groups of 16, reduction length in 16s, k blocks of 32
    int BI, BJ, WY, RBA;       // blocks of 32 per wave each way, waves along the rows, padded row blocks of the weights
    int64_t P;                 // output positions NI * HO * WO
    size_t w_bytes, act_bytes;
    size_t total() const { return w_bytes + act_bytes + 256; }
};

inline P8ConvMfmaPlan p8_conv_mfma_plan(int which, const ConvGeom& g) {
    P8ConvMfmaPlan p;
    p.ok = false;
    p.which = which;
    if (which > 1 || g.sh != 1 || g.sw != 1) return p;
    p.NI = g.N; p.R = g.R; p.S = g.S; p.WK = g.K; p.WC = g.C;
    if (which == 0) {
        p.CI = g.C; p.HI = g.H; p.WI = g.W; p.HO = g.OH; p.WO = g.OW; p.MO = g.K; p.offh = g.ph; p.offw = g.pw;
    } else {
        p.CI = g.K; p.HI = g.OH; p.WI = g.OW; p.HO = g.H; p.WO = g.W; p.MO = g.C; p.offh = g.R - 1 - g.ph; p.offw = g.S - 1 - g.pw;
    }
    if (p.NI <= 0 || p.CI <= 0 || p.HI <= 0 || p.WI <= 0 || p.HO <= 0 || p.WO <= 0 || p.MO <= 0) return p;
    p.Cg = (p.CI + 15) / 16;
    p.K16 = g.R * g.S * p.Cg;
    p.KB = (p.K16 + 1) / 2;
    p.P = (int64_t)p.NI * p.HO * p.WO;
    const int64_t pin = (int64_t)p.NI * p.HI * p.WI;
    if (2 * p.KB > PCM_MAXK16 || p.HI > 16384 || p.WI > 16384 || g.R > 4096 || g.S > 4096) return p;
    if (pin * p.Cg * 2 >= ((int64_t)1 << 30) || p.P >= ((int64_t)1 << 30) || p.P * p.MO >= ((int64_t)1 << 40)) return p;
    // worth the two rewriting launches: enough products, enough positions to fill the chip, enough rows to use a block
    const int64_t macs = p.P * p.MO * p.CI * g.R * g.S;
    if (macs < ((int64_t)1 << 24) || p.P < 8192 || p.MO < 4 || p.CI < 8) return p;
    p.WY = p.MO > 32 ? 2 : 1;
    p.BI = (p.MO > 64 && ((p.MO + 127) / 128) * ((p.P + 63) / 64) >= 256) ? 2 : 1;  // 128-row tiles only if every compute unit still gets one
    const int64_t tiles_m = (p.MO + 32 * p.WY * p.BI - 1) / (32 * p.WY * p.BI);
    p.BJ = (p.WY == 2 && p.BI == 1 && tiles_m * ((p.P + 127) / 128) >= PM_MIN_WGS) ? 2 : 1;
    p.RBA = (int)tiles_m * p.WY * p.BI;
    p.w_bytes = (size_t)p.KB * p.RBA * 2048;
    p.act_bytes = (size_t)pin * p.Cg * 32;
    p.ok = true;
    return p;
}

// One launch rewrites both operands; the first wblocks workgroups take the weights (few threads, long chains of loads:
// started first), the rest the input tensor.
//
// Input tensor [NI][CI][HW] -> digit planes [NI * HW][Cg][2][16]; channels beyond CI are zeros.  One thread per channel
// group and PX consecutive pixels (PX = 4 when HW is a multiple of 4 and the tensor is 4-byte aligned: one 32-bit load
// per channel); consecutive threads take consecutive pixels, so every load is coalesced.
//
// Weights [WK][WC][R][S] -> [KB][RBA][2][64][16] (and the 32 zero bytes behind the input planes) in the lane order of
// the matrix instruction, reduction index 16 ((r S + s) Cg + cg) + channel.  Forward: row = output channel k,
// channel = c.  Backward-data: row = c, channel = k, the tap taken at (R-1-r, S-1-s), NaR written as zero.  One
// thread per (k block, row block, lane).
template <int PX>
__global__ __launch_bounds__(256) void p8_conv_digits_kernel(const uint8_t* __restrict__ src, int HW, int64_t pixels, uint8_t* __restrict__ act,
                                                             const uint8_t* __restrict__ w, P8ConvMfmaPlan p, uint8_t* __restrict__ wdst,
                                                             uint4* __restrict__ zero, unsigned wblocks) {
    __shared__ int16_t tab[256];
    const int t = threadIdx.x;
    tab[t] = t == 0x80 ? (int16_t)(PM_NAR_HI * 128) : (int16_t)Arith<P8>::stage((uint32_t)t);
    __syncthreads();
    if (blockIdx.x < wblocks) {
        const int64_t idx = (int64_t)blockIdx.x * 256 + t;
        if (idx < 2) zero[idx] = make_uint4(0, 0, 0, 0);  // what the product kernel reads for padding (no memset: graph capture)
        if (idx >= (int64_t)p.KB * p.RBA * 64) return;
        const int lane = (int)(idx & 63);
        const int rb = (int)((idx >> 6) % p.RBA), kb = (int)((idx >> 6) / p.RBA);
        const int row = rb * 32 + (lane & 31), k16 = kb * 2 + (lane >> 5);
        uint32_t hi[4] = {0, 0, 0, 0}, lo[4] = {0, 0, 0, 0};
        if (row < p.MO && k16 < p.K16) {
            const int tap = k16 / p.Cg, cg = k16 - tap * p.Cg;
            const int r = tap / p.S, s = tap - r * p.S;
            const int nch = p.CI - cg * 16 < 16 ? p.CI - cg * 16 : 16;
            // forward: w[row][ch][r][s]; backward-data: w[ch][row][R-1-r][S-1-s]
            const int64_t rs = (int64_t)p.R * p.S;
            const uint8_t* q = p.which == 0 ? w + ((int64_t)row * p.WC + cg * 16) * rs + r * p.S + s
                                            : w + ((int64_t)cg * 16 * p.WC + row) * rs + (p.R - 1 - r) * p.S + (p.S - 1 - s);
            const int64_t step = p.which == 0 ? rs : rs * p.WC;
            uint32_t pat[16];
#pragma unroll
            for (int b = 0; b < 16; ++b) pat[b] = b < nch ? q[b * step] : 0u;  // all loads in flight together
#pragma unroll
            for (int b = 0; b < 16; ++b) {
                int v = tab[pat[b]];
                if (pat[b] == 0x80u && p.which != 0) v = 0;
                hi[b >> 2] |= ((uint32_t)(v >> 7) & 0xFFu) << (8 * (b & 3));
                lo[b >> 2] |= ((uint32_t)v & 0x7Fu) << (8 * (b & 3));
            }
        }
        uint4* out = reinterpret_cast<uint4*>(wdst) + ((int64_t)(kb * p.RBA + rb) * 2) * 64 + lane;
        out[0] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
        out[64] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
        return;
    }
    const int64_t groups = pixels / PX;  // PX divides HW, hence pixels
    const int64_t idx = (int64_t)(blockIdx.x - wblocks) * 256 + t;
    if (idx >= groups * p.Cg) return;
    const int cg = (int)(idx / groups);
    const int64_t pix = (idx - (int64_t)cg * groups) * PX;
    const int64_t img = pix / HW, hw = pix - img * HW;
    const uint8_t* q = src + (img * p.CI + cg * 16) * (int64_t)HW + hw;
    const int nch = p.CI - cg * 16 < 16 ? p.CI - cg * 16 : 16;
    uint32_t word[16];
#pragma unroll
    for (int b = 0; b < 16; ++b) {
        if (b >= nch) word[b] = 0;
        else if (PX == 4) word[b] = *reinterpret_cast<const uint32_t*>(q + (int64_t)b * HW);
        else word[b] = q[(int64_t)b * HW];
    }
#pragma unroll
    for (int px = 0; px < PX; ++px) {
        uint32_t hi[4] = {0, 0, 0, 0}, lo[4] = {0, 0, 0, 0};
#pragma unroll
        for (int b = 0; b < 16; ++b) {
            const int v = tab[(word[b] >> (8 * px)) & 0xFFu];  // pattern 0 decodes to 0: channels beyond CI stay zero
            hi[b >> 2] |= ((uint32_t)(v >> 7) & 0xFFu) << (8 * (b & 3));
            lo[b >> 2] |= ((uint32_t)v & 0x7Fu) << (8 * (b & 3));
        }
        uint4* out = reinterpret_cast<uint4*>(act) + ((pix + px) * p.Cg + cg) * 2;
        out[0] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
        out[1] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
    }
}

struct P8ConvMfmaArgs {
    const uint8_t* Ad;    // weight digit planes
    const uint8_t* act;   // input digit planes
    const uint8_t* zero;  // 32 bytes of zeros
    int RBA, KB, K16, Cg;
    int HI, WI, HO, WO, S, offh, offw, MO;
    int P;
    const uint8_t* bias;
    void* out;
    int fout, tiles_m, tiles_n;
};

// Four waves as WY x (4 / WY), a wave owns BI x BJ blocks of 32 x 32 outputs (rows: output channels, columns:
// positions).  WY = 1 (all four waves side by side along the positions, 32 x 128 outputs) serves layers of at most 32
// output channels, where a second row of waves would multiply and round nothing but padding.
template <int BI, int BJ, int WY>
__global__ __launch_bounds__(256, (BI * BJ == 2 ? 3 : 4)) void p8_conv_mfma_kernel(P8ConvMfmaArgs a) {
    constexpr int WX = 4 / WY;
    static_assert(WY == 2 || (WY == 1 && BI == 1 && BJ == 1), "wave layouts");
    constexpr int NA = WY * BI * 2, NB = WX * BJ * 2;  // runs of 1 KB (block, digit) per k block and operand
    constexpr int TR = 32 * BI * WY, TC = 32 * BJ * WX;
    // A ring of PCM_STAGES k blocks, copies running PCM_STAGES - 1 blocks ahead: a convolution's reduction is short
    // (tens of k blocks) and a block's matrix instructions take a fraction of a copy's latency, so depth hides it.
    __shared__ uint4 stage[PCM_STAGES][(NA + NB) * 64];
    __shared__ int2 ktab[PCM_MAXK16];  // per 16 reduction indices: offset of the tap and channel group in the planes, (dh, dw) packed

    const int t = threadIdx.x;
    const int lane = t & 63, w = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wy = WY == 2 ? w >> 1 : 0, wx = WY == 2 ? (w & 1) : w;
    const int tm = blockIdx.x % a.tiles_m, tn = blockIdx.x / a.tiles_m;

    for (int k = t; k < 2 * a.KB; k += 256) {
        int2 e = make_int2(0, 0x7FFF);  // beyond the reduction: a row offset no pixel has
        if (k < a.K16) {
            const int tap = k / a.Cg, cg = k - tap * a.Cg;
            const int r = tap / a.S, s = tap - r * a.S;
            const int dh = r - a.offh, dw = s - a.offw;
            e.x = ((dh * a.WI + dw) * a.Cg + cg) * 2;
            e.y = (int)(((uint32_t)dh & 0xFFFFu) | ((uint32_t)dw << 16));
        }
        ktab[k] = e;
    }

    uint32_t row_nar = 0, col_nar = 0;
    pm_v16i hh[BI][BJ], xx[BI][BJ], ll[BI][BJ];
#pragma unroll
    for (int i = 0; i < BI; ++i)
#pragma unroll
        for (int j = 0; j < BJ; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) hh[i][j][r] = xx[i][j][r] = ll[i][j][r] = 0;

    // Weights: wave w copies ARUNS of the k block's NA runs from wave-uniform addresses, as in the matrix product (with
    // only two runs the waves pair up and copy the same run twice: every wave then has the same number of copies in
    // flight, which the wait below counts).
    constexpr int ARUNS = NA >= 4 ? NA / 4 : 1;
    const int arun0 = (w * ARUNS) % NA;
    const int64_t a_kb = (int64_t)a.RBA * 2 * 64;
    const uint4* asrc = reinterpret_cast<const uint4*>(a.Ad) + (int64_t)tm * NA * 64 + arun0 * 64;
    // Input: the k block's NB runs are (column block, digit) pairs.  With four column blocks in the tile wave w gathers
    // both digits of column block w; with two, digit w % 2 of column block w / 2.  Lane l of a copy serves column
    // l % 32 of the block and the 16 reduction indices of half l / 32.
    constexpr bool HALF = WX * BJ == 2;
    const int cb = HALF ? (w >> 1) : w;
    const int hw_o = a.HO * a.WO;
    int oh, ow, base;
    {
        const int pos = tn * TC + cb * 32 + (lane & 31);
        if (pos < a.P) {
            const int img = pos / hw_o, rem = pos - img * hw_o;
            oh = rem / a.WO;
            ow = rem - oh * a.WO;
            base = ((img * a.HI + oh) * a.WI + ow) * a.Cg * 2;
        } else {
            oh = -40000;  // no tap brings this into the tensor
            ow = 0;
            base = 0;
        }
    }
    const uint4* actq = reinterpret_cast<const uint4*>(a.act) + (HALF ? (w & 1) : 0);
    const uint4* zeroq = reinterpret_cast<const uint4*>(a.zero);

    auto issue = [&](int kb) {
        uint4* sbuf = &stage[kb % PCM_STAGES][0];
#pragma unroll
        for (int c = 0; c < ARUNS; ++c)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(asrc + c * 64 + lane),
                                             (__attribute__((address_space(3))) void*)(sbuf + (arun0 + c) * 64), 16, 0, 0);
        asrc += a_kb;
        const int2 e = ktab[kb * 2 + (lane >> 5)];
        const int dh = (int)(short)(e.y & 0xFFFF), dw = e.y >> 16;
        const int ih = oh + dh, iw = ow + dw;
        const bool inside = (unsigned)ih < (unsigned)a.HI && (unsigned)iw < (unsigned)a.WI;
        const uint4* s = inside ? actq + (base + e.x) : zeroq;
        if (!HALF) {
            uint4* d = sbuf + (NA + cb * 2) * 64;  // the same for every lane
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)s, (__attribute__((address_space(3))) void*)d, 16, 0, 0);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(s + 1), (__attribute__((address_space(3))) void*)(d + 64),
                                             16, 0, 0);
        } else {
            uint4* d = sbuf + (NA + cb * 2 + (w & 1)) * 64;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)s, (__attribute__((address_space(3))) void*)d, 16, 0, 0);
        }
    };
    constexpr int LOADS = ARUNS + (HALF ? 1 : 2);  // copies per wave and k block

    // the blocks this wave searches for NaR markers: two waves that share blocks split them
    const int ia = BI == 2 ? wx : 0, jb = (BJ == 2 && WY == 2) ? wy : 0;

    __syncthreads();  // ktab
#pragma unroll
    for (int k = 0; k < PCM_STAGES - 1; ++k)
        if (k < a.KB) issue(k);
    for (int kb = 0; kb < a.KB; ++kb) {
        // k block kb has arrived once at most the copies of the PCM_STAGES - 2 blocks issued after it are outstanding
        // (copies complete in order); near the end fewer were issued, so wait for all
        if (kb + PCM_STAGES - 2 < a.KB) __builtin_amdgcn_s_waitcnt(pcm_vmcnt((PCM_STAGES - 2) * LOADS));
        else __builtin_amdgcn_s_waitcnt(pcm_vmcnt(0));
        pcm_ring_barrier();  // everyone's copies of block kb are in LDS, and everyone has finished reading block kb - 1
        if (kb + PCM_STAGES - 1 < a.KB) issue(kb + PCM_STAGES - 1);  // into the buffer of block kb - 1
        const uint4* sb = &stage[kb % PCM_STAGES][0];
        pm_v4i ah[BI], al[BI], bh[BJ], bl[BJ];
#pragma unroll
        for (int i = 0; i < BI; ++i) {
            ah[i] = __builtin_bit_cast(pm_v4i, sb[((BI * wy + i) * 2 + 0) * 64 + lane]);
            al[i] = __builtin_bit_cast(pm_v4i, sb[((BI * wy + i) * 2 + 1) * 64 + lane]);
        }
#pragma unroll
        for (int j = 0; j < BJ; ++j) {
            bh[j] = __builtin_bit_cast(pm_v4i, sb[(NA + (BJ * wx + j) * 2 + 0) * 64 + lane]);
            bl[j] = __builtin_bit_cast(pm_v4i, sb[(NA + (BJ * wx + j) * 2 + 1) * 64 + lane]);
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
        __builtin_amdgcn_sched_barrier(0);  // a block's reads and matrix instructions stay inside its own iteration
    }
    __syncthreads();  // the last block is read: the buffers are free for the NaR flags

    // ---- the three sums into the quire, round once, store ----
    // Row flags (NaR weight or NaR bias in the channel) and the bias addends meet in LDS; column flags too.
    uint32_t* rowv = reinterpret_cast<uint32_t*>(&stage[0][0]);
    uint32_t* colv = rowv + TR;
    int32_t* rowb = reinterpret_cast<int32_t*>(colv + TC);
    row_nar = (row_nar | (uint32_t)__shfl_xor((int)row_nar, 32)) & 0x80808080u;
    col_nar = (col_nar | (uint32_t)__shfl_xor((int)col_nar, 32)) & 0x80808080u;
    if (lane < 32) {
        const int lr = (wy * BI + ia) * 32 + lane;
        if ((BI == 2 && WY == 2) || wx == 0) {  // one writer per row
            int32_t badd = 0;
            const int m = tm * TR + lr;
            if (a.bias && m < a.MO) {
                const uint32_t bp = a.bias[m];
                if (bp == 0x80u) row_nar = 1;
                else badd = (int32_t)Arith<P8>::stage(bp) << P8::MAXS;  // + bias * 1
            }
            rowv[lr] = row_nar;
            rowb[lr] = badd;
        }
        colv[(wx * BJ + jb) * 32 + lane] = col_nar;  // with one block per wave both waves of the pair write the same flag
    }
    __syncthreads();
    rowv += wy * 32 * BI;
    rowb += wy * 32 * BI;
    colv += wx * 32 * BJ;
    // The matrix instruction leaves a lane with one position and 16 BI channels: stored from there, every store
    // instruction would write 1 byte per lane, 32 bytes per channel row.  The rounded tile goes through LDS instead
    // (buffers 1 .. of the ring; buffer 0 holds the NaR flags) and leaves in 16-byte runs along the positions.
    const FmtRT fo = fmt_of_code(a.fout);
    const int esz = fo.n <= 8 ? 1 : (fo.n <= 16 ? 2 : 4);
    uint8_t* tileb = reinterpret_cast<uint8_t*>(&stage[1][0]);
    static_assert((PCM_STAGES - 1) * (NA + NB) * 1024 >= TR * TC * 4, "the rounded tile fits behind the NaR flags");
#pragma unroll
    for (int j = 0; j < BJ; ++j) {
        const int lc = (wx * BJ + j) * 32 + (lane & 31);
        const bool cnar = colv[j * 32 + (lane & 31)] != 0;
#pragma unroll
        for (int i = 0; i < BI; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int lr = i * 32 + (r & 3) + 8 * (r >> 2) + 4 * (lane >> 5);
                const uint32_t q = ((uint32_t)hh[i][j][r] << 14) + ((uint32_t)xx[i][j][r] << 7) + (uint32_t)ll[i][j][r] + (uint32_t)rowb[lr];
                const bool nar = cnar || rowv[lr] != 0;
                const int at = (wy * 32 * BI + lr) * TC + lc;
                if (a.fout == 0) {
                    tileb[at] = (uint8_t)(nar ? 0x80u : p8_round_quire((int32_t)q));
                } else {
                    const uint32_t q1[1] = {q};
                    round_store<QuireAccum<P8>, 1>(q1, nar, a.fout, tileb, at);
                }
            }
        }
    }
    __syncthreads();
    const int per_run = 16 / esz;            // outputs per 16-byte run
    const int runs_per_row = TC / per_run;
    for (int run = t; run < TR * runs_per_row; run += 256) {
        const int lr = run / runs_per_row, c0 = (run - lr * runs_per_row) * per_run;
        const int m = tm * TR + lr, n0 = tn * TC + c0;
        if (m >= a.MO || n0 >= a.P) continue;
        const uint8_t* src = tileb + (lr * TC + c0) * esz;
        const int img = n0 / hw_o, rem = n0 - img * hw_o;
        uint8_t* dst = (uint8_t*)a.out + (((int64_t)img * a.MO + m) * hw_o + rem) * esz;
        if (rem + per_run <= hw_o && n0 + per_run <= a.P && (((uintptr_t)dst) & 15u) == 0) {
            *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(src);  // one image, whole run, aligned
        } else {
            for (int c = 0; c < per_run && n0 + c < a.P; ++c) {
                const int n = n0 + c;
                const int im = n / hw_o, re = n - im * hw_o;
                uint8_t* d = (uint8_t*)a.out + (((int64_t)im * a.MO + m) * hw_o + re) * esz;
                for (int bb = 0; bb < esz; ++bb) d[bb] = src[c * esz + bb];
            }
        }
    }
}

// in: x (forward) or dy (backward-data); workspace: [weight planes][input planes][256 bytes of zeros]
inline hipError_t launch_p8_conv_mfma(hipStream_t stream, const P8ConvMfmaPlan& p, const void* in, const void* w, const uint8_t* bias, void* out,
                                      int fout, void* workspace) {
    uint8_t* base = (uint8_t*)workspace;
    uint8_t* Ad = base;
    uint8_t* act = base + p.w_bytes;
    uint8_t* zero = act + p.act_bytes;
    const int64_t pixels = (int64_t)p.NI * p.HI * p.WI;
    const int HW = p.HI * p.WI;
    const unsigned wblocks = (unsigned)(((int64_t)p.KB * p.RBA * 64 + 255) / 256);
    if (HW % 4 == 0 && ((uintptr_t)in & 3u) == 0) {
        const unsigned ablocks = (unsigned)((pixels / 4 * p.Cg + 255) / 256);
        hipLaunchKernelGGL(p8_conv_digits_kernel<4>, dim3(wblocks + ablocks), dim3(256), 0, stream, (const uint8_t*)in, HW, pixels, act,
                           (const uint8_t*)w, p, Ad, reinterpret_cast<uint4*>(zero), wblocks);
    } else {
        const unsigned ablocks = (unsigned)((pixels * p.Cg + 255) / 256);
        hipLaunchKernelGGL(p8_conv_digits_kernel<1>, dim3(wblocks + ablocks), dim3(256), 0, stream, (const uint8_t*)in, HW, pixels, act,
                           (const uint8_t*)w, p, Ad, reinterpret_cast<uint4*>(zero), wblocks);
    }
    PNN_CHECK_LAUNCH();
    P8ConvMfmaArgs a;
    a.Ad = Ad; a.act = act; a.zero = zero;
    a.RBA = p.RBA; a.KB = p.KB; a.K16 = p.K16; a.Cg = p.Cg;
    a.HI = p.HI; a.WI = p.WI; a.HO = p.HO; a.WO = p.WO; a.S = p.S; a.offh = p.offh; a.offw = p.offw; a.MO = p.MO;
    a.P = (int)p.P;
    a.bias = bias; a.out = out; a.fout = fout;
    a.tiles_m = p.RBA / (p.WY * p.BI);
    const int tc = 32 * p.BJ * (4 / p.WY);
    a.tiles_n = (int)((p.P + tc - 1) / tc);
    const dim3 grid((unsigned)(a.tiles_m * a.tiles_n));
    if (p.WY == 1) hipLaunchKernelGGL((p8_conv_mfma_kernel<1, 1, 1>), grid, dim3(256), 0, stream, a);
    else if (p.BI == 2) hipLaunchKernelGGL((p8_conv_mfma_kernel<2, 1, 2>), grid, dim3(256), 0, stream, a);
    else if (p.BJ == 2) hipLaunchKernelGGL((p8_conv_mfma_kernel<1, 2, 2>), grid, dim3(256), 0, stream, a);
    else hipLaunchKernelGGL((p8_conv_mfma_kernel<1, 1, 2>), grid, dim3(256), 0, stream, a);
    return hipGetLastError();
}


// ---- backward-weight: dw[k][c][r][s] = sum over (n, oh, ow) of dy[n][k][oh][ow] x[n][c][oh sh + r - ph][ow sw + s - pw] ----
//
// A matrix product with few outputs (K x CRS) and a long reduction (image, position).  The matrix instruction wants 16
// consecutive reduction indices per lane.  Ordered position-major, IMAGE-minor these are 16 images at one pixel, so the
// pass is the forward kernel's gather with batch and channels trading places: one launch rewrites x as digit planes
// [c][h][w][group of 16 images][digit][16 bytes] and dy in the row-block layout of the matrix kernel (rows k, reduction
// index 16 ((oh OW + ow) NG + g) + image, through an LDS tile so that reads and writes are both contiguous); the product
// kernel copies dy's runs from wave-uniform addresses and gathers x: lane (column (c, r, s), 16 reduction indices)
// names the 16 bytes of pixel (oh sh + r - ph, ow sw + s - pw) of channel c and image group g, or a block of zeros in the
// padding.  Nothing is unfolded; any stride.  The reduction is cut into slices ((tile, z) reduces kb_per_split k blocks,
// about 512 workgroups in all) whose 32-bit sums and NaR flags the merging launch adds, rounds and stores.  The bias
// gradient, db[k] = sum of dy[.][k][.][.] * 1, is one more column: its lanes gather a block that holds 1 for every image
// of the group, and the merge routes the column to its own tensor.

struct P8ConvBwPlan {
    bool ok;
    ConvGeom g;
    int M, N, crs;             // outputs: K x CRS, or K x (CRS + 1) with the bias gradient as the last column
    int NG;                    // groups of 16 images
    int K16;                   // reduction length in 16s: OH OW NG
    int RBA, RBB, KB;          // row blocks of dy's planes, column blocks, k blocks (= splits * kb_per_split)
    int splits, kb_per_split;
    size_t a_bytes, x_bytes, ones_bytes, part_bytes;
    size_t total() const { return a_bytes + x_bytes + ones_bytes + 256 + part_bytes; }
};

inline P8ConvBwPlan p8_conv_bw_plan(const ConvGeom& g, bool with_bias) {
    P8ConvBwPlan p;
    p.ok = false;
    p.g = g;
    const int64_t crs = (int64_t)g.C * g.R * g.S;
    const int64_t P = (int64_t)g.N * g.OH * g.OW;
    if (g.K < 4 || crs < 16 || crs > 65536 || g.K > 65536 || P < 4096 || P >= ((int64_t)1 << 30)) return p;
    if ((int64_t)g.K * crs * P < ((int64_t)1 << 22)) return p;  // below, the three launches cost more than the dot-product kernel
    p.NG = (g.N + 15) / 16;
    const int64_t k16 = (int64_t)g.OH * g.OW * p.NG;
    if ((int64_t)g.C * g.H * g.W * p.NG * 2 >= ((int64_t)1 << 30) || k16 >= ((int64_t)1 << 28) || g.H > 16384 || g.W > 16384) return p;
    p.K16 = (int)k16;
    p.M = g.K;
    p.crs = (int)crs;
    p.N = (int)crs + (with_bias ? 1 : 0);
    const int tiles_m = (p.M + 63) / 64, tiles_n = (p.N + 63) / 64;
    p.RBA = tiles_m * 2;
    p.RBB = tiles_n * 2;
    const int64_t kb_total = (k16 + 1) / 2;
    int64_t splits = (512 + tiles_m * tiles_n - 1) / (tiles_m * tiles_n);  // about two workgroups per compute unit (measured against one and four)
    if (splits > kb_total / 8) splits = kb_total / 8;                        // at least 8 k blocks per slice
    if (splits < 1) splits = 1;
    const int64_t kbps = (kb_total + splits - 1) / splits;
    splits = (kb_total + kbps - 1) / kbps;
    p.splits = (int)splits;
    p.kb_per_split = (int)kbps;
    p.KB = (int)(splits * kbps);
    p.a_bytes = (size_t)p.KB * p.RBA * 2048;
    p.x_bytes = (size_t)g.C * g.H * g.W * p.NG * 32;
    p.ones_bytes = (size_t)p.NG * 32;
    if (p.a_bytes >= ((size_t)1 << 32)) return p;
    p.part_bytes = ((size_t)p.splits * p.M * p.N + (size_t)p.splits * (p.M + p.N)) * 4;
    p.ok = true;
    return p;
}

constexpr int PCB_PITCH = 68;  // bytes per row of the transposition tile: 64 positions + 4, so that rows fall on different banks

// ablocks workgroups rewrite dy, the rest x (and the blocks of ones and zeros).
//   dy: workgroup (row block rb, image group g, chunk of 64 positions) loads the 16 x 32 x 64 patterns with the positions
//       along the lanes, keeps them in LDS, and writes, per position and row, the 16 images' digits: 512 contiguous bytes
//       per position and digit in [k block][row block][digit][lane][16 bytes].  Positions beyond OH OW (up to the padded
//       reduction length 2 KB) are written as zeros.
//   x:  one thread per (channel, PX consecutive pixels, image group); 16 loads a pixel-plane apart, coalesced along the pixels.
template <int PX>
__global__ __launch_bounds__(256) void p8_conv_bw_digits_kernel(const uint8_t* __restrict__ dy, const uint8_t* __restrict__ x, P8ConvBwPlan p,
                                                                uint8_t* __restrict__ Ad, uint8_t* __restrict__ xb, uint4* __restrict__ ones,
                                                                uint4* __restrict__ zero, unsigned ablocks, int chunks) {
    __shared__ int16_t tab[256];
    __shared__ __attribute__((aligned(16))) uint8_t tile[16][32][PCB_PITCH];
    const int t = threadIdx.x;
    tab[t] = t == 0x80 ? (int16_t)(PM_NAR_HI * 128) : (int16_t)Arith<P8>::stage((uint32_t)t);
    const ConvGeom& g = p.g;
    const int ohw = g.OH * g.OW;
    if (blockIdx.x < ablocks) {
        const int chunk = (int)(blockIdx.x % (unsigned)chunks);
        const int gi = (int)((blockIdx.x / (unsigned)chunks) % (unsigned)p.NG);
        const int rb = (int)(blockIdx.x / (unsigned)(chunks * p.NG));
        // loads in batches of eight before their LDS stores, so that eight are in flight per thread
        if (ohw % 4 == 0 && ((uintptr_t)dy & 3u) == 0) {  // four positions per load
#pragma unroll 1
            for (int base = 0; base < 32; base += 8) {
                uint32_t v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int item = (base + u) * 256 + t;
                    const int pair = item >> 4, q4 = item & 15;
                    const int img = gi * 16 + (pair >> 5), row = rb * 32 + (pair & 31), pos = chunk * 64 + q4 * 4;
                    v[u] = (img < g.N && row < g.K && pos < ohw) ? *reinterpret_cast<const uint32_t*>(dy + ((int64_t)img * g.K + row) * ohw + pos) : 0u;
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int item = (base + u) * 256 + t;
                    const int pair = item >> 4, q4 = item & 15;
                    *reinterpret_cast<uint32_t*>(&tile[pair >> 5][pair & 31][q4 * 4]) = v[u];
                }
            }
        } else {
#pragma unroll 1
            for (int base = 0; base < 128; base += 8) {
                uint8_t v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int pair = (base + u) * 4 + (t >> 6), pos = chunk * 64 + (t & 63);
                    const int img = gi * 16 + (pair >> 5), row = rb * 32 + (pair & 31);
                    v[u] = (img < g.N && row < g.K && pos < ohw) ? dy[((int64_t)img * g.K + row) * ohw + pos] : (uint8_t)0;
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int pair = (base + u) * 4 + (t >> 6);
                    tile[pair >> 5][pair & 31][t & 63] = v[u];
                }
            }
        }
        __syncthreads();
        for (int item = t; item < 64 * 32; item += 256) {
            const int pl = item >> 5, rr = item & 31;
            const int64_t k16 = (int64_t)(chunk * 64 + pl) * p.NG + gi;
            if (k16 >= 2 * (int64_t)p.KB) continue;
            uint32_t hi[4] = {0, 0, 0, 0}, lo[4] = {0, 0, 0, 0};
#pragma unroll
            for (int b = 0; b < 16; ++b) {
                const int v = tab[tile[b][rr][pl]];
                hi[b >> 2] |= ((uint32_t)(v >> 7) & 0xFFu) << (8 * (b & 3));
                lo[b >> 2] |= ((uint32_t)v & 0x7Fu) << (8 * (b & 3));
            }
            const int kb = (int)(k16 >> 1), lane = (int)(k16 & 1) * 32 + rr;
            uint4* out = reinterpret_cast<uint4*>(Ad) + ((int64_t)(kb * p.RBA + rb) * 2) * 64 + lane;
            out[0] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
            out[64] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
        }
        return;
    }
    __syncthreads();
    const int64_t idx = (int64_t)(blockIdx.x - ablocks) * 256 + t;
    if (idx < 2) zero[idx] = make_uint4(0, 0, 0, 0);  // what the product kernel reads for padding (no memset: graph capture)
    if (idx < p.NG) {  // the column of ones: 1 = 64 units of 2^-6 = low digit 64, for the images the group really has
        uint32_t lo[4] = {0, 0, 0, 0};
        for (int b = 0; b < 16; ++b)
            if ((int)idx * 16 + b < g.N) lo[b >> 2] |= 64u << (8 * (b & 3));
        ones[idx * 2] = make_uint4(0, 0, 0, 0);
        ones[idx * 2 + 1] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
    }
    const int HW = g.H * g.W;
    const int64_t planes = (int64_t)g.C * HW;  // pixels of all channels of one image
    const int64_t groups = planes / PX;
    if (idx >= groups * p.NG) return;
    const int gi = (int)(idx / groups);
    const int64_t pix = (idx - (int64_t)gi * groups) * PX;  // (c, h, w) as one index
    const int nimg = g.N - gi * 16 < 16 ? g.N - gi * 16 : 16;
    const uint8_t* q = x + (int64_t)gi * 16 * planes + pix;
    uint32_t word[16];
#pragma unroll
    for (int b = 0; b < 16; ++b) {
        if (b >= nimg) word[b] = 0;
        else if (PX == 4) word[b] = *reinterpret_cast<const uint32_t*>(q + (int64_t)b * planes);
        else word[b] = q[(int64_t)b * planes];
    }
#pragma unroll
    for (int px = 0; px < PX; ++px) {
        uint32_t hi[4] = {0, 0, 0, 0}, lo[4] = {0, 0, 0, 0};
#pragma unroll
        for (int b = 0; b < 16; ++b) {
            const int v = tab[(word[b] >> (8 * px)) & 0xFFu];
            hi[b >> 2] |= ((uint32_t)(v >> 7) & 0xFFu) << (8 * (b & 3));
            lo[b >> 2] |= ((uint32_t)v & 0x7Fu) << (8 * (b & 3));
        }
        uint4* out = reinterpret_cast<uint4*>(xb) + ((pix + px) * p.NG + gi) * 2;
        out[0] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
        out[1] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
    }
}

struct P8ConvBwArgs {
    const uint8_t* Ad;    // dy's digit planes
    const uint8_t* xb;    // x's digit planes, image-minor
    const uint8_t* ones;  // per image group: the digits of 1 for the images it has
    const uint8_t* zero;  // 32 bytes of zeros
    int RBA, kb_per_split;
    int NG, OH, OW, H, W, R, S, ph, pw, sh, sw;
    int crs, M, N;
    SplitWs ws;
    int tiles_m, tiles_n;
};

// 64 x 64 outputs per workgroup of four waves (2 x 2, one block of 32 x 32 each); workgroup (tile, z) reduces slice z.
template <int UNUSED = 0>
__global__ __launch_bounds__(256, 4) void p8_conv_bw_mfma_kernel(P8ConvBwArgs a) {
    constexpr int NA = 4, NB = 4;  // runs of 1 KB (block, digit) per k block and operand
    constexpr int TR = 64, TC = 64;
    __shared__ uint4 stage[PCM_STAGES][(NA + NB) * 64];

    const int t = threadIdx.x;
    const int lane = t & 63, w = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wy = w >> 1, wx = w & 1;
    const int tm = blockIdx.x % a.tiles_m, tn = blockIdx.x / a.tiles_m;
    const int z = blockIdx.y;
    const int kb0 = z * a.kb_per_split;

    uint32_t row_nar = 0, col_nar = 0;
    pm_v16i hh, xx, ll;
#pragma unroll
    for (int r = 0; r < 16; ++r) hh[r] = xx[r] = ll[r] = 0;

    // dy: wave w copies run w of the k block's four (row block w / 2, digit w % 2) from a wave-uniform address
    const int64_t a_kb = (int64_t)a.RBA * 2 * 64;
    const uint4* asrc = reinterpret_cast<const uint4*>(a.Ad) + kb0 * a_kb + (int64_t)tm * NA * 64 + w * 64;
    // x: wave w gathers digit w % 2 of column block w / 2; lane l serves column l % 32 of the block and the 16 reduction
    // indices (one pixel, one image group) of half l / 32
    const int cb = w >> 1, digit = w & 1;
    const int n = tn * TC + cb * 32 + (lane & 31);
    int kind = 2, cbase = 0, dr = 0, ds = 0;  // kind 0: a column (c, r, s); 1: the column of ones; 2: beyond the columns
    if (n < a.crs) {
        const int rs = a.R * a.S;
        const int c = n / rs, tp = n - c * rs;
        const int r = tp / a.S, s = tp - r * a.S;
        kind = 0;
        cbase = c * a.H * a.W * a.NG * 2 + digit;
        dr = r - a.ph;
        ds = s - a.pw;
    } else if (n < a.N) {
        kind = 1;
    }
    // the reduction index of this lane's half, as (oh, ow, image group), stepped from k block to k block
    int oh, ow, gi;
    {
        const int k16 = kb0 * 2 + (lane >> 5);
        const int pos = k16 / a.NG;
        gi = k16 - pos * a.NG;
        oh = pos / a.OW;
        ow = pos - oh * a.OW;
    }
    const uint4* xq = reinterpret_cast<const uint4*>(a.xb);
    const uint4* onesq = reinterpret_cast<const uint4*>(a.ones) + digit;
    const uint4* zeroq = reinterpret_cast<const uint4*>(a.zero);

    int issued = 0;
    auto issue = [&]() {
        uint4* sbuf = &stage[issued % PCM_STAGES][0];
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(asrc + lane),
                                         (__attribute__((address_space(3))) void*)(sbuf + w * 64), 16, 0, 0);
        asrc += a_kb;
        const uint4* s = zeroq;
        if (oh < a.OH) {  // inside the reduction (its padded end reads zeros)
            if (kind == 0) {
                const int ih = oh * a.sh + dr, iw = ow * a.sw + ds;
                if ((unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W) s = xq + (cbase + ((ih * a.W + iw) * a.NG + gi) * 2);
            } else if (kind == 1) {
                s = onesq + gi * 2;
            }
        }
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)s,
                                         (__attribute__((address_space(3))) void*)(sbuf + (NA + cb * 2 + digit) * 64), 16, 0, 0);
        gi += 2;  // the next k block: two reduction indices of 16 further
        while (gi >= a.NG) {
            gi -= a.NG;
            if (++ow == a.OW) {
                ow = 0;
                ++oh;
            }
        }
        ++issued;
    };
    constexpr int LOADS = 2;  // copies per wave and k block

    const int nkb = a.kb_per_split;
#pragma unroll
    for (int k = 0; k < PCM_STAGES - 1; ++k)
        if (k < nkb) issue();
    for (int kb = 0; kb < nkb; ++kb) {
        // k block kb has arrived once at most the copies of the PCM_STAGES - 2 blocks issued after it are outstanding
        // (copies complete in order); near the end fewer were issued, so wait for all
        if (kb + PCM_STAGES - 2 < nkb) __builtin_amdgcn_s_waitcnt(pcm_vmcnt((PCM_STAGES - 2) * LOADS));
        else __builtin_amdgcn_s_waitcnt(pcm_vmcnt(0));
        pcm_ring_barrier();  // everyone's copies of block kb are in LDS, and everyone has finished reading block kb - 1
        if (kb + PCM_STAGES - 1 < nkb) issue();  // into the buffer of block kb - 1
        const uint4* sb = &stage[kb % PCM_STAGES][0];
        const pm_v4i ah = __builtin_bit_cast(pm_v4i, sb[(wy * 2 + 0) * 64 + lane]);
        const pm_v4i al = __builtin_bit_cast(pm_v4i, sb[(wy * 2 + 1) * 64 + lane]);
        const pm_v4i bh = __builtin_bit_cast(pm_v4i, sb[(NA + wx * 2 + 0) * 64 + lane]);
        const pm_v4i bl = __builtin_bit_cast(pm_v4i, sb[(NA + wx * 2 + 1) * 64 + lane]);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            row_nar |= pm_marker_bits((uint32_t)ah[q]);
            col_nar |= pm_marker_bits((uint32_t)bh[q]);
        }
        hh = __builtin_amdgcn_mfma_i32_32x32x32_i8(ah, bh, hh, 0, 0, 0);
        xx = __builtin_amdgcn_mfma_i32_32x32x32_i8(ah, bl, xx, 0, 0, 0);
        xx = __builtin_amdgcn_mfma_i32_32x32x32_i8(al, bh, xx, 0, 0, 0);
        ll = __builtin_amdgcn_mfma_i32_32x32x32_i8(al, bl, ll, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);  // a block's reads and matrix instructions stay inside its own iteration
    }
    __syncthreads();  // the last block is read: the buffers are free for the NaR flags

    // ---- this slice's sums and NaR flags into the split workspace ----
    uint32_t* rowv = reinterpret_cast<uint32_t*>(&stage[0][0]);
    uint32_t* colv = rowv + TR;
    row_nar = (row_nar | (uint32_t)__shfl_xor((int)row_nar, 32)) & 0x80808080u;
    col_nar = (col_nar | (uint32_t)__shfl_xor((int)col_nar, 32)) & 0x80808080u;
    if (lane < 32) {
        if (wx == 0) rowv[wy * 32 + lane] = row_nar;  // the two waves of a row block saw the same rows
        if (wy == 0) colv[wx * 32 + lane] = col_nar;
    }
    __syncthreads();
    const int64_t M = a.M, N = a.N;
    // the first tile column stores the row flags of its tile row (the same in every column), the first tile row the
    // column flags: every entry is written, so the workspace needs no clearing
    if (tn == 0 && t < TR && tm * TR + t < M) a.ws.rowflag[z * M + tm * TR + t] = rowv[t];
    if (tm == 0 && t < TC && tn * TC + t < N) a.ws.colflag[z * N + tn * TC + t] = colv[t];
    uint32_t* lim = a.ws.limbs + z * M * N;
    const int nn = tn * TC + wx * 32 + (lane & 31);
    if (nn < N) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = tm * TR + wy * 32 + (r & 3) + 8 * (r >> 2) + 4 * (lane >> 5);
            if (m < M) lim[(int64_t)m * N + nn] = ((uint32_t)hh[r] << 14) + ((uint32_t)xx[r] << 7) + (uint32_t)ll[r];
        }
    }
}

// workspace: [planes of dy][planes of x][blocks of ones][256 bytes of zeros][partial sums and flags of the slices]
inline hipError_t launch_p8_conv_bw_mfma(hipStream_t stream, const P8ConvBwPlan& p, const void* dy, const void* x, void* dw, void* dbias,
                                         int fout, void* workspace) {
    uint8_t* base = (uint8_t*)workspace;
    uint8_t* Ad = base;
    uint8_t* xb = base + p.a_bytes;
    uint8_t* ones = xb + p.x_bytes;
    uint8_t* zero = ones + p.ones_bytes;
    SplitWs ws;
    ws.limbs = reinterpret_cast<uint32_t*>(zero + 256);
    ws.rowflag = ws.limbs + (size_t)p.splits * p.M * p.N;
    ws.colflag = ws.rowflag + (size_t)p.splits * p.M;
    const ConvGeom& g = p.g;
    const int posmax = (2 * p.KB + p.NG - 1) / p.NG;  // positions up to the padded end of the reduction
    const int chunks = (posmax + 63) / 64;
    const unsigned ablocks = (unsigned)p.RBA * (unsigned)p.NG * (unsigned)chunks;
    const int64_t planes = (int64_t)g.C * g.H * g.W;
    if (planes % 4 == 0 && ((uintptr_t)x & 3u) == 0) {
        const unsigned xblocks = (unsigned)((planes / 4 * p.NG + 255) / 256);
        hipLaunchKernelGGL(p8_conv_bw_digits_kernel<4>, dim3(ablocks + xblocks), dim3(256), 0, stream, (const uint8_t*)dy, (const uint8_t*)x, p, Ad, xb,
                           reinterpret_cast<uint4*>(ones), reinterpret_cast<uint4*>(zero), ablocks, chunks);
    } else {
        const unsigned xblocks = (unsigned)((planes * p.NG + 255) / 256);
        hipLaunchKernelGGL(p8_conv_bw_digits_kernel<1>, dim3(ablocks + xblocks), dim3(256), 0, stream, (const uint8_t*)dy, (const uint8_t*)x, p, Ad, xb,
                           reinterpret_cast<uint4*>(ones), reinterpret_cast<uint4*>(zero), ablocks, chunks);
    }
    PNN_CHECK_LAUNCH();
    P8ConvBwArgs a;
    a.Ad = Ad; a.xb = xb; a.ones = ones; a.zero = zero;
    a.RBA = p.RBA; a.kb_per_split = p.kb_per_split;
    a.NG = p.NG; a.OH = g.OH; a.OW = g.OW; a.H = g.H; a.W = g.W; a.R = g.R; a.S = g.S; a.ph = g.ph; a.pw = g.pw; a.sh = g.sh; a.sw = g.sw;
    a.crs = p.crs; a.M = p.M; a.N = p.N;
    a.ws = ws;
    a.tiles_m = p.RBA / 2;
    a.tiles_n = p.RBB / 2;
    hipLaunchKernelGGL(p8_conv_bw_mfma_kernel<0>, dim3((unsigned)(a.tiles_m * a.tiles_n), (unsigned)p.splits), dim3(256), 0, stream, a);
    PNN_CHECK_LAUNCH();
    if (p.N > p.crs) {
        WeightAndBiasOut out{(int64_t)p.crs, dbias};
        return launch_split_merge<P8, WeightAndBiasOut>(stream, ws, p.splits, p.M, p.N, nullptr, dw, fout, out);
    }
    RowMajorOut out{(int64_t)p.N};
    return launch_split_merge<P8, RowMajorOut>(stream, ws, p.splits, p.M, p.N, nullptr, dw, fout, out);
}

}  // namespace pnn
