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
// Stride 1 only.  Backward-weight reduces over the positions, where 16 consecutive indices are 16 pixels of a shifted
// row that crosses the padding: it stays on the dot-product kernels.
#pragma once

#include "gemm_p8_mfma.h"

namespace pnn {

constexpr int PCM_MAXK16 = 512;  // most (tap, channel group) pairs, padding included (4 KB of LDS)
constexpr int PCM_STAGES = 4;    // k blocks in flight per workgroup

// s_waitcnt immediate: at most n vector-memory operations outstanding, the other counters unconstrained
constexpr int pcm_vmcnt(int n) { return (n & 0xF) | ((n >> 4) << 14) | 0x0F70; }

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
    if (macs < ((int64_t)1 << 26) || p.P < 8192 || p.MO < 16 || p.CI < 8) return p;
    p.WY = p.MO > 32 ? 2 : 1;
    p.BI = p.MO > 64 ? 2 : 1;
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
        __syncthreads();  // everyone's copies of block kb are in LDS, and everyone has finished reading block kb - 1
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
    __syncthreads();  // the last block is read: the buffers are free for the verdicts

    // ---- the three sums into the quire, round once, store ----
    // Row verdicts (NaR weight or NaR bias in the channel) and the bias addends meet in LDS; column verdicts too.
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
        colv[(wx * BJ + jb) * 32 + lane] = col_nar;  // with one block per wave both waves of the pair write the same verdict
    }
    __syncthreads();
    rowv += wy * 32 * BI;
    rowb += wy * 32 * BI;
    colv += wx * 32 * BJ;
    // The matrix instruction leaves a lane with one position and 16 BI channels: stored from there, every store
    // instruction would write 1 byte per lane, 32 bytes per channel row.  The rounded tile goes through LDS instead
    // (buffers 1 .. of the ring; buffer 0 holds the verdicts) and leaves in 16-byte runs along the positions.
    const FmtRT fo = fmt_of_code(a.fout);
    const int esz = fo.n <= 8 ? 1 : (fo.n <= 16 ? 2 : 4);
    uint8_t* tileb = reinterpret_cast<uint8_t*>(&stage[1][0]);
    static_assert((PCM_STAGES - 1) * (NA + NB) * 1024 >= TR * TC * 4, "the rounded tile fits behind the verdicts");
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
// A matrix product with few outputs (K x CRS) and a long reduction (the positions).  The matrix instruction wants 16
// consecutive reduction indices per lane, here 16 consecutive positions of one channel: runs of dy as it lies in
// memory, but runs of x shifted by the tap and cut by the padding.  So this pass does unfold: one launch writes the digit
// planes of dy (rows k) and of the unfolded input (rows (c, r, s), zeros where the tap leaves the tensor) in the
// layout of the matrix product kernel, [k block][row block][digit][lane][16 bytes], and that kernel runs in its split
// form, a few hundred slices of the positions per output tile, merged by the usual launch.  The unfolded planes are
// 2 R S times the input, written and read once; that traffic, not the matrix cores, sets the time.

struct __attribute__((packed, aligned(1))) P8Run16 { uint32_t w[4]; };  // 16 bytes at any address

struct P8ConvBwPlan {
    bool ok;
    ConvGeom g;
    int M, N;                  // outputs: K x CRS, or K x (CRS + 1) with the bias gradient as the last column
    int crs;
    int64_t P;                 // reduction: N OH OW positions
    int RBA, RBB, KB;          // padded extents in blocks of 32 (KB = splits * kb_per_split)
    int splits, kb_per_split;
    size_t a_bytes, b_bytes, part_bytes;
    size_t total() const { return a_bytes + b_bytes + part_bytes; }
};

inline P8ConvBwPlan p8_conv_bw_plan(const ConvGeom& g, bool with_bias) {
    P8ConvBwPlan p;
    p.ok = false;
    p.g = g;
    const int64_t crs = (int64_t)g.C * g.R * g.S;
    p.P = (int64_t)g.N * g.OH * g.OW;
    if (g.K < 16 || crs < 16 || crs > 65536 || g.K > 65536 || p.P < 4096 || p.P >= ((int64_t)1 << 30)) return p;
    if ((int64_t)g.K * crs * p.P < ((int64_t)1 << 26)) return p;
    if ((int64_t)g.N * g.C * g.H * g.W >= ((int64_t)1 << 31) || (int64_t)g.N * g.K * g.OH * g.OW >= ((int64_t)1 << 31)) return p;
    p.M = g.K;
    p.crs = (int)crs;
    p.N = (int)crs + (with_bias ? 1 : 0);  // db[k] = sum over the positions of dy[k] * 1: a column of ones
    const int tiles_m = (p.M + 63) / 64, tiles_n = (p.N + 63) / 64;
    p.RBA = tiles_m * 2;
    p.RBB = tiles_n * 2;
    const int64_t kb_total = (p.P + 31) / 32;
    int64_t splits = (1024 + tiles_m * tiles_n - 1) / (tiles_m * tiles_n);  // about four workgroups per compute unit
    if (splits > kb_total / 8) splits = kb_total / 8;                        // at least 8 k blocks per slice
    if (splits < 1) splits = 1;
    int64_t kbps = (kb_total + splits - 1) / splits;
    kbps = (kbps + PM_KSTEP - 1) / PM_KSTEP * PM_KSTEP;
    splits = (kb_total + kbps - 1) / kbps;
    p.splits = (int)splits;
    p.kb_per_split = (int)kbps;
    p.KB = (int)(splits * kbps);
    p.a_bytes = (size_t)p.KB * p.RBA * 2048;
    p.b_bytes = (size_t)p.KB * p.RBB * 2048;
    if (p.a_bytes + p.b_bytes >= ((size_t)1 << 32)) return p;
    p.part_bytes = ((size_t)p.splits * p.M * p.N + (size_t)p.splits * (p.M + p.N)) * 4;
    p.ok = true;
    return p;
}

// The first ablocks workgroups write the planes of dy, the rest those of the unfolded input.  One thread per
// (k block, row block, lane): 16 consecutive positions of one row.
template <int UNUSED = 0>
__global__ __launch_bounds__(256) void p8_conv_bw_digits_kernel(const uint8_t* __restrict__ dy, const uint8_t* __restrict__ x, P8ConvBwPlan p,
                                                                uint8_t* __restrict__ Ad, uint8_t* __restrict__ Bd, unsigned ablocks) {
    __shared__ int16_t tab[256];
    const int t = threadIdx.x;
    tab[t] = t == 0x80 ? (int16_t)(PM_NAR_HI * 128) : (int16_t)Arith<P8>::stage((uint32_t)t);
    __syncthreads();
    const ConvGeom& g = p.g;
    const int ohw = g.OH * g.OW;
    const bool first = blockIdx.x < ablocks;
    const int RB = first ? p.RBA : p.RBB;
    const int64_t idx = (int64_t)(first ? blockIdx.x : blockIdx.x - ablocks) * 256 + t;
    if (idx >= (int64_t)p.KB * RB * 64) return;
    const int lane = (int)(idx & 63);
    const int rb = (int)((idx >> 6) % RB), kb = (int)((idx >> 6) / RB);
    const int row = rb * 32 + (lane & 31);
    const int64_t p0 = (int64_t)kb * 32 + 16 * (lane >> 5);
    uint32_t pat[16];
#pragma unroll
    for (int b = 0; b < 16; ++b) pat[b] = 0;
    if (p0 < p.P && row < (first ? p.M : p.N)) {
        int img = (int)(p0 / ohw);
        int rem = (int)(p0 - (int64_t)img * ohw);
        if (first) {
            const uint8_t* q = dy + ((int64_t)img * g.K + row) * ohw + rem;
            if (rem + 16 <= ohw && ((uintptr_t)q & 15u) == 0) {  // within one image (hence within the tensor), aligned
                const uint4 v = *reinterpret_cast<const uint4*>(q);
                const uint32_t wv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int b = 0; b < 16; ++b) pat[b] = (wv[b >> 2] >> (8 * (b & 3))) & 0xFFu;
            } else {
#pragma unroll
                for (int b = 0; b < 16; ++b) {
                    if (p0 + b < p.P) pat[b] = dy[((int64_t)img * g.K + row) * ohw + rem];
                    if (++rem == ohw) { rem = 0; ++img; }
                }
            }
        } else {
            if (row == p.crs) {  // the column of ones behind the unfolded input
#pragma unroll
                for (int b = 0; b < 16; ++b) pat[b] = p0 + b < p.P ? 0x40u : 0u;
            }
            const int rs = g.R * g.S;
            const int c = row / rs, tp = row - c * rs;
            const int r = tp / g.S, s = tp - r * g.S;
            int oh = rem / g.OW, ow = rem - oh * g.OW;
            // Unit stride and the 16 positions in one output row: they read 16 consecutive bytes of one input row, cut
            // by at most a few columns of padding at either end.  One 16-byte load (of any alignment) from the nearest
            // start inside the row, shifted by the bytes that fall into the padding.
            const int iw0 = ow + s - g.pw;
            const int start = iw0 < 0 ? 0 : (iw0 + 16 > g.W ? g.W - 16 : iw0);
            const int d = iw0 - start;  // < 0: the run begins in the left padding; > 0: it ends in the right padding
            if (row == p.crs) {
            } else if (g.sw == 1 && g.W >= 16 && ow + 16 <= g.OW && p0 + 16 <= p.P && d >= -3 && d <= 3) {
                const int ih = oh * g.sh + r - g.ph;
                if ((unsigned)ih < (unsigned)g.H) {
                    const P8Run16 v = *reinterpret_cast<const P8Run16*>(x + (((int64_t)img * g.C + c) * g.H + ih) * g.W + start);
                    uint32_t wv[4] = {v.w[0], v.w[1], v.w[2], v.w[3]};
                    if (d < 0) {
                        const int sh = -8 * d;
#pragma unroll
                        for (int i = 3; i >= 0; --i) wv[i] = (wv[i] << sh) | (i > 0 ? wv[i - 1] >> (32 - sh) : 0u);
                    } else if (d > 0) {
                        const int sh = 8 * d;
#pragma unroll
                        for (int i = 0; i < 4; ++i) wv[i] = (wv[i] >> sh) | (i < 3 ? wv[i + 1] << (32 - sh) : 0u);
                    }
#pragma unroll
                    for (int b = 0; b < 16; ++b) pat[b] = (wv[b >> 2] >> (8 * (b & 3))) & 0xFFu;
                }  // a row of padding: zeros
            } else {
#pragma unroll
                for (int b = 0; b < 16; ++b) {
                    const int ih = oh * g.sh + r - g.ph, iw = ow * g.sw + s - g.pw;
                    if (p0 + b < p.P && (unsigned)ih < (unsigned)g.H && (unsigned)iw < (unsigned)g.W)
                        pat[b] = x[(((int64_t)img * g.C + c) * g.H + ih) * g.W + iw];
                    if (++ow == g.OW) {
                        ow = 0;
                        if (++oh == g.OH) { oh = 0; ++img; }
                    }
                }
            }
        }
    }
    uint32_t hi[4] = {0, 0, 0, 0}, lo[4] = {0, 0, 0, 0};
#pragma unroll
    for (int b = 0; b < 16; ++b) {
        const int v = tab[pat[b]];
        hi[b >> 2] |= ((uint32_t)(v >> 7) & 0xFFu) << (8 * (b & 3));
        lo[b >> 2] |= ((uint32_t)v & 0x7Fu) << (8 * (b & 3));
    }
    uint4* out = reinterpret_cast<uint4*>(first ? Ad : Bd) + ((int64_t)(kb * RB + rb) * 2) * 64 + lane;
    out[0] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
    out[64] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
}

// workspace: [planes of dy][planes of the unfolded input][partial sums and flags of the slices]
inline hipError_t launch_p8_conv_bw_mfma(hipStream_t stream, const P8ConvBwPlan& p, const void* dy, const void* x, void* dw, void* dbias,
                                         int fout, void* workspace) {
    uint8_t* base = (uint8_t*)workspace;
    uint8_t* Ad = base;
    uint8_t* Bd = base + p.a_bytes;
    SplitWs ws;
    ws.limbs = reinterpret_cast<uint32_t*>(base + p.a_bytes + p.b_bytes);
    ws.rowflag = ws.limbs + (size_t)p.splits * p.M * p.N;
    ws.colflag = ws.rowflag + (size_t)p.splits * p.M;
    const unsigned ablocks = (unsigned)(((int64_t)p.KB * p.RBA * 64 + 255) / 256), bblocks = (unsigned)(((int64_t)p.KB * p.RBB * 64 + 255) / 256);
    hipLaunchKernelGGL(p8_conv_bw_digits_kernel<0>, dim3(ablocks + bblocks), dim3(256), 0, stream, (const uint8_t*)dy, (const uint8_t*)x, p, Ad, Bd,
                       ablocks);
    PNN_CHECK_LAUNCH();
    const int tiles_m = p.RBA / 2, tiles_n = p.RBB / 2;
    hipLaunchKernelGGL((p8_mfma_gemm_kernel<1, 1, true>), dim3((unsigned)(tiles_m * tiles_n), (unsigned)p.splits), dim3(256), 0, stream, Ad, Bd, p.RBA,
                       p.RBB, p.KB, (const uint8_t*)nullptr, (void*)nullptr, (int64_t)0, fout, p.M, p.N, tiles_m, tiles_n, p.kb_per_split, ws);
    PNN_CHECK_LAUNCH();
    if (p.N > p.crs) {
        WeightAndBiasOut out{(int64_t)p.crs, dbias};
        return launch_split_merge<P8, WeightAndBiasOut>(stream, ws, p.splits, p.M, p.N, nullptr, dw, fout, out);
    }
    RowMajorOut out{(int64_t)p.N};
    return launch_split_merge<P8, RowMajorOut>(stream, ws, p.splits, p.M, p.N, nullptr, dw, fout, out);
}

}  // namespace pnn
