// Tiled quire-exact GEMM kernel shared by posit_gemm and the three convolution
// entry points (paper Sec. 3.3: matrix products and convolutions accumulate in
// the quire and round once; Sec. 3.1: forward, backward-data and backward-weight
// are written out by hand).  The convolutions are "implicit GEMMs": the kernel
// is the same, only the functors that map (row, k) of the virtual matrices to
// an address in the NCHW / KCRS tensors differ.
//
// Work split: one 256-thread workgroup computes a BM x BN tile of C.  For each
// KT-wide slice of the reduction, the threads fetch patterns from HBM, decode
// them once (Eq. 2) into the staged form of Arith<FIN>, and park them in LDS;
// then each thread multiplies its TM x TN register tile against the slice,
// adding every exact product into per-output quire limbs held in VGPRs
// (directly, or through fp64 buckets that are emptied into the limbs before
// their guard bits run out: accumulator policies below).  NaR
// never enters the arithmetic: a NaR pattern is staged as zero and raises an
// LDS flag for its row (of A) or column (of B), applied when the tile is
// rounded.  With gridDim.z > 1 the reduction is split across workgroups, which
// write their limb partial sums to a workspace; a second kernel merges the
// partial quires with carry and rounds (exact, order-independent).
#pragma once

#include "quire_arith.h"

// After a kernel launch inside a chain of launches: stop at the first failure, so that no later kernel
// reads what a kernel that never ran should have written.
#define PNN_CHECK_LAUNCH()                                 \
    do {                                                   \
        const hipError_t pnn_e_ = hipGetLastError();       \
        if (pnn_e_ != hipSuccess) return pnn_e_;           \
    } while (0)

namespace pnn {

// ---- operand functors: pattern of virtual element (row, k); zero outside ----

// Row-major matrix; KFAST: element (row,k) at p[row*ld + k], else at p[k*ld + row].
template <class T, bool KFAST_>
struct MatrixOperand {
    static constexpr bool KFAST = KFAST_;
    static constexpr bool RAISES_NAR = true;  // a NaR pattern of this operand makes its whole row (column) of outputs NaR
    const T* p;
    int64_t ld, rows, K;
    __device__ __forceinline__ uint32_t operator()(int64_t row, int64_t k) const {
        if (row >= rows || k >= K) return 0u;
        return KFAST_ ? p[row * ld + k] : p[k * ld + row];
    }
};

// A column of ones (pattern `one`): turns the kernel into a row sum (bias gradient).
struct OnesOperand {
    static constexpr bool KFAST = true;
    static constexpr bool RAISES_NAR = true;
    uint32_t one;
    int64_t rows, K;
    __device__ __forceinline__ uint32_t operator()(int64_t row, int64_t k) const {
        return (row < rows && k < K) ? one : 0u;
    }
};

struct ConvGeom {
    int N, C, H, W, K, R, S, ph, pw, sh, sw, OH, OW;
};

// Forward, left operand: row = (n, oh, ow), k = (c, r, s) -> x[n, c, oh*sh+r-ph, ow*sw+s-pw]
template <class T>
struct ConvFwdX {
    static constexpr bool KFAST = false;
    static constexpr bool RAISES_NAR = true;
    const T* x;
    ConvGeom g;
    int64_t rows, K;
    __device__ __forceinline__ uint32_t operator()(int64_t row, int64_t k) const {
        if (row >= rows || k >= K) return 0u;
        const int ohw = g.OH * g.OW;
        const int n = (int)(row / ohw), rem = (int)(row % ohw);
        const int oh = rem / g.OW, ow = rem % g.OW;
        const int rs = g.R * g.S;
        const int c = (int)k / rs, t = (int)k % rs;
        const int r = t / g.S, s = t % g.S;
        const int ih = oh * g.sh + r - g.ph, iw = ow * g.sw + s - g.pw;
        if (ih < 0 || ih >= g.H || iw < 0 || iw >= g.W) return 0u;
        return x[(((int64_t)n * g.C + c) * g.H + ih) * g.W + iw];
    }
};

// Backward-data, left operand: row = (n, h, w), k = (ko, r, s) -> dy[n, ko, (h+ph-r)/sh, (w+pw-s)/sw]
template <class T>
struct ConvBwdDataDy {
    static constexpr bool KFAST = false;
    static constexpr bool RAISES_NAR = true;
    const T* dy;
    ConvGeom g;
    int64_t rows, K;
    __device__ __forceinline__ uint32_t operator()(int64_t row, int64_t k) const {
        if (row >= rows || k >= K) return 0u;
        const int hw = g.H * g.W;
        const int n = (int)(row / hw), rem = (int)(row % hw);
        const int h = rem / g.W, w = rem % g.W;
        const int rs = g.R * g.S;
        const int ko = (int)k / rs, t = (int)k % rs;
        const int r = t / g.S, s = t % g.S;
        const int th = h + g.ph - r, tw = w + g.pw - s;
        if (th < 0 || tw < 0) return 0u;
        const int oh = th / g.sh, ow = tw / g.sw;
        if (oh * g.sh != th || ow * g.sw != tw || oh >= g.OH || ow >= g.OW) return 0u;
        return dy[(((int64_t)n * g.K + ko) * g.OH + oh) * g.OW + ow];
    }
};

// Backward-data, right operand: row = c, k = (ko, r, s) -> w[ko, c, r, s].  A NaR weight is staged as zero and
// raises no flag: it makes NaR only the input positions its tap reaches (bwd_data_nar_weights_kernel).
template <class T>
struct ConvBwdDataW {
    static constexpr bool KFAST = true;
    static constexpr bool RAISES_NAR = false;
    const T* w;
    ConvGeom g;
    int64_t rows, K;
    __device__ __forceinline__ uint32_t operator()(int64_t row, int64_t k) const {
        if (row >= rows || k >= K) return 0u;
        const int rs = g.R * g.S;
        const int ko = (int)k / rs, t = (int)k % rs;
        return w[((int64_t)ko * g.C + row) * rs + t];
    }
};

// Backward-weight, left operand: row = ko, k = (n, oh, ow) -> dy[n, ko, oh, ow]
template <class T>
struct ConvBwdWeightDy {
    static constexpr bool KFAST = true;
    static constexpr bool RAISES_NAR = true;
    const T* dy;
    ConvGeom g;
    int64_t rows, K;
    __device__ __forceinline__ uint32_t operator()(int64_t row, int64_t k) const {
        if (row >= rows || k >= K) return 0u;
        const int ohw = g.OH * g.OW;
        const int n = (int)(k / ohw), rem = (int)(k % ohw);
        return dy[((int64_t)n * g.K + row) * ohw + rem];
    }
};

// Backward-weight, right operand: row = (c, r, s), k = (n, oh, ow) -> x[n, c, oh*sh+r-ph, ow*sw+s-pw]
template <class T>
struct ConvBwdWeightX {
    static constexpr bool KFAST = true;
    static constexpr bool RAISES_NAR = true;
    const T* x;
    ConvGeom g;
    int64_t rows, K;
    __device__ __forceinline__ uint32_t operator()(int64_t row, int64_t k) const {
        if (row >= rows || k >= K) return 0u;
        const int ohw = g.OH * g.OW;
        const int n = (int)(k / ohw), rem = (int)(k % ohw);
        const int oh = rem / g.OW, ow = rem % g.OW;
        const int rs = g.R * g.S;
        const int c = (int)row / rs, t = (int)row % rs;
        const int r = t / g.S, s = t % g.S;
        const int ih = oh * g.sh + r - g.ph, iw = ow * g.sw + s - g.pw;
        if (ih < 0 || ih >= g.H || iw < 0 || iw >= g.W) return 0u;
        return x[(((int64_t)n * g.C + c) * g.H + ih) * g.W + iw];
    }
};

// ---- where output (row, col) lives ----

struct RowMajorOut {
    int64_t ld;
    __device__ __forceinline__ int64_t operator()(int64_t row, int64_t col) const { return row * ld + col; }
};

// row = (n, spatial), col = channel  ->  [n][channel][spatial]
struct NchwOut {
    int64_t spatial, channels;
    __device__ __forceinline__ int64_t operator()(int64_t row, int64_t col) const {
        const int64_t n = row / spatial, rem = row % spatial;
        return (n * channels + col) * spatial + rem;
    }
};

// Backward-weight of a convolution with the bias gradient as one more column (the product of dy with a column of
// ones): columns below `weights` go to the weight gradient, row-major with that pitch; column `weights` to bias_grad[row].
struct WeightAndBiasOut {
    int64_t weights;
    void* bias_grad;
    __device__ __forceinline__ int64_t operator()(int64_t row, int64_t col) const { return row * weights + col; }
};

// Where a merged output goes: the tensor C at the functor's index, unless the functor names another tensor.
template <class Out>
__device__ __forceinline__ void* merge_dest(const Out& out, void* C, int64_t m, int64_t n, int64_t& at) {
    at = out(m, n);
    return C;
}
__device__ __forceinline__ void* merge_dest(const WeightAndBiasOut& out, void* C, int64_t m, int64_t n, int64_t& at) {
    if (n == out.weights) {
        at = m;
        return out.bias_grad;
    }
    at = out(m, n);
    return C;
}

// Workspace layout for a split reduction, per split z:
//   limbs  [z][M*N][L] uint32   partial quires
//   rowflag[z][M], colflag[z][N] uint32   NaR seen in that row of A / column of B
struct SplitWs {
    uint32_t* limbs;
    uint32_t* rowflag;
    uint32_t* colflag;
};

constexpr int GEMM_THREADS = 256;
constexpr int GEMM_KT = 16;

// Accumulator policy "quire": Arith<F> plus the read-out of the limbs as a real number.
// SPLITTABLE: partial accumulators of slices of the reduction can be merged exactly.
// BUCKETS: fp64 buckets carried per output beside the limbs (0: products go straight into the limbs).
template <class F>
struct QuireAccum : Arith<F> {
    static constexpr bool SPLITTABLE = true;
    static constexpr int BUCKETS = 0;
    PNN_HD static bool read(const uint32_t (&q)[Arith<F>::L], Real& r) { return quire_read<F, Arith<F>::L>(q, r); }
    PNN_HD static void add_bias(uint32_t (&q)[Arith<F>::L], uint32_t pattern) { Arith<F>::add_value(q, Arith<F>::stage(pattern)); }
};

// Accumulator policy "quire through fp64 buckets": the same exact sum, with the products of up to
// 2^G reduction steps gathered in BUCKETS doubles per output before they enter the limbs
// (BucketArith).  Everything outside the inner loop (bias, split merge, read-out) is integer.
template <class F>
struct BucketAccum : BucketArith<F> {
    static constexpr int L = Arith<F>::L;
    static constexpr bool SPLITTABLE = true;
    static constexpr int BUCKETS = BucketArith<F>::B;
    static constexpr int FLUSH_SLICES = (1 << BucketArith<F>::G) / GEMM_KT;  // slices of the reduction between two flushes
    static_assert(BUCKETS == 0 || FLUSH_SLICES >= 1, "a slice must fit the guard bits");
    PNN_HD static bool read(const uint32_t (&q)[L], Real& r) { return quire_read<F, L>(q, r); }
    PNN_HD static void add_bias(uint32_t (&q)[L], uint32_t pattern) { Arith<F>::add_value(q, Arith<F>::stage(pattern)); }
};

template <class F, bool BUCKETED = (BucketArith<F>::B > 0)>
struct DefaultAccumOf { typedef QuireAccum<F> type; };
template <class F>
struct DefaultAccumOf<F, true> { typedef BucketAccum<F> type; };
template <class F>
using DefaultAccum = typename DefaultAccumOf<F>::type;

// Round an accumulator of policy AR to the output format chosen at run time (format
// code of the C ABI) and store it in that format's container.
template <class AR, int L>
__device__ __forceinline__ void round_store(const uint32_t (&q)[L], bool nar, int fout, void* C, int64_t at) {
    const FmtRT fo = fmt_of_code(fout);
    Real r;
    const bool nonzero = AR::read(q, r);
    const uint32_t res = nar ? fo.nar() : (nonzero ? encode_rt(r, fo) : 0u);
    if (fo.n <= 8) ((uint8_t*)C)[at] = (uint8_t)res;
    else if (fo.n <= 16) ((uint16_t*)C)[at] = (uint16_t)res;
    else ((uint32_t*)C)[at] = res;
}

template <class FIN, class OpA, class OpB, class Out, int TM, int TN, class AR>
__global__ __launch_bounds__(GEMM_THREADS) void quire_gemm_kernel(
    OpA opa, OpB opb, Out out, int64_t M, int64_t N, int64_t K, int64_t k_per_split,
    const typename Storage<FIN::N>::T* __restrict__ bias, void* __restrict__ C, int fout,
    SplitWs ws, int tiles_n) {
    typedef typename AR::Elem Elem;
    constexpr int L = AR::L;
    constexpr int BM = 16 * TM, BN = 16 * TN, KT = GEMM_KT;

    __shared__ Elem As[2][KT][BM + 1];  // double-buffered: slice kt + 1 is staged while slice kt is multiplied
    __shared__ Elem Bs[2][KT][BN + 1];
    __shared__ uint32_t rowNaR[BM];
    __shared__ uint32_t colNaR[BN];

    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int64_t tile = blockIdx.x;
    const int64_t m0 = (tile / tiles_n) * BM, n0 = (tile % tiles_n) * BN;
    const int64_t kbeg = (int64_t)blockIdx.z * k_per_split;
    const int64_t kend = (kbeg + k_per_split < K) ? kbeg + k_per_split : K;

    for (int i = tid; i < BM; i += GEMM_THREADS) rowNaR[i] = 0;
    for (int i = tid; i < BN; i += GEMM_THREADS) colNaR[i] = 0;

    uint32_t acc[TM][TN][L];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int l = 0; l < L; ++l) acc[i][j][l] = 0;
    constexpr int NBK = AR::BUCKETS > 0 ? AR::BUCKETS : 1;
    double bk[TM][TN][NBK];  // fp64 buckets of the bucketed policies (unused otherwise)
    int since_flush = 0;
    if constexpr (AR::BUCKETS > 0) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) AR::clear(bk[i][j]);
    }

    // Element e = tid + 256 i of a slice: consecutive threads walk the dimension that is contiguous in memory.
    constexpr int EA = BM * KT / GEMM_THREADS, EB = BN * KT / GEMM_THREADS;
    static_assert(BM * KT % GEMM_THREADS == 0 && BN * KT % GEMM_THREADS == 0, "whole elements per thread");
    uint32_t pa[EA], pb[EB];  // patterns of the next slice, fetched before the current one is multiplied
    auto fetch = [&](int64_t k0) {
#pragma unroll
        for (int i = 0; i < EA; ++i) {
            const int e = tid + GEMM_THREADS * i;
            const int kk = OpA::KFAST ? (e % KT) : (e / BM);
            const int r = OpA::KFAST ? (e / KT) : (e % BM);
            const int64_t k = k0 + kk;
            pa[i] = (k < kend) ? opa(m0 + r, k) : 0u;
        }
#pragma unroll
        for (int i = 0; i < EB; ++i) {
            const int e = tid + GEMM_THREADS * i;
            const int kk = OpB::KFAST ? (e % KT) : (e / BN);
            const int r = OpB::KFAST ? (e / KT) : (e % BN);
            const int64_t k = k0 + kk;
            pb[i] = (k < kend) ? opb(n0 + r, k) : 0u;
        }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int i = 0; i < EA; ++i) {
            const int e = tid + GEMM_THREADS * i;
            const int kk = OpA::KFAST ? (e % KT) : (e / BM);
            const int r = OpA::KFAST ? (e / KT) : (e % BM);
            if (OpA::RAISES_NAR && pa[i] == FIN::NAR) rowNaR[r] = 1;
            As[buf][kk][r] = AR::stage(pa[i]);
        }
#pragma unroll
        for (int i = 0; i < EB; ++i) {
            const int e = tid + GEMM_THREADS * i;
            const int kk = OpB::KFAST ? (e % KT) : (e / BN);
            const int r = OpB::KFAST ? (e / KT) : (e % BN);
            if (OpB::RAISES_NAR && pb[i] == FIN::NAR) colNaR[r] = 1;
            Bs[buf][kk][r] = AR::stage(pb[i]);
        }
    };

    __syncthreads();  // flags initialised before any stage() raises one
    if (kbeg < kend) {
        fetch(kbeg);
        stage(0);
    }
    __syncthreads();
    int cur = 0;
    for (int64_t k0 = kbeg; k0 < kend; k0 += KT, cur ^= 1) {
        const bool more = k0 + KT < kend;
        if (more) fetch(k0 + KT);
#pragma unroll 2
        for (int kk = 0; kk < KT; ++kk) {
            Elem a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) a[i] = As[cur][kk][ty * TM + i];
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = Bs[cur][kk][tx * TN + j];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    if constexpr (AR::BUCKETS > 0) AR::mac(bk[i][j], a[i], b[j]);
                    else AR::mac(acc[i][j], a[i], b[j]);
                }
        }
        if constexpr (AR::BUCKETS > 0) {
            if (++since_flush == AR::FLUSH_SLICES) {  // the buckets' guard bits are used up: empty them into the limbs
                since_flush = 0;
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) AR::template flush<L>(acc[i][j], bk[i][j]);
            }
        }
        if (more) stage(cur ^ 1);  // the other buffer was last read one barrier ago
        __syncthreads();
    }
    if constexpr (AR::BUCKETS > 0) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) AR::template flush<L>(acc[i][j], bk[i][j]);
    }
    __syncthreads();

    if (gridDim.z == 1) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int64_t m = m0 + ty * TM + i;
            if (m >= M) continue;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int64_t n = n0 + tx * TN + j;
                if (n >= N) continue;
                bool nar = (rowNaR[ty * TM + i] | colNaR[tx * TN + j]) != 0;
                if (bias) {
                    const uint32_t bp = bias[n];
                    if (bp == FIN::NAR) nar = true;
                    else AR::add_bias(acc[i][j], bp);
                }
                round_store<AR, L>(acc[i][j], nar, fout, C, out(m, n));
            }
        }
    } else {
        const int64_t z = blockIdx.z;
        uint32_t* lim = ws.limbs + z * M * N * L;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int64_t m = m0 + ty * TM + i;
            if (m >= M) continue;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int64_t n = n0 + tx * TN + j;
                if (n >= N) continue;
#pragma unroll
                for (int l = 0; l < L; ++l) lim[(m * N + n) * L + l] = acc[i][j][l];
            }
        }
        // All tiles of a tile row see the same rows of A over this slice of the reduction, hence the same
        // row flags: the tile in the first column stores them (every entry, set or not, so the workspace
        // needs no clearing); likewise the first tile row stores the column flags.
        if (n0 == 0)
            for (int i = tid; i < BM; i += GEMM_THREADS)
                if (m0 + i < M) ws.rowflag[z * M + m0 + i] = rowNaR[i];
        if (m0 == 0)
            for (int i = tid; i < BN; i += GEMM_THREADS)
                if (n0 + i < N) ws.colflag[z * N + n0 + i] = colNaR[i];
    }
}

// Merge the per-split partial quires, add the bias, round once, store.  A
// 256-thread workgroup handles 32 consecutive outputs; its 8 thread rows each sum
// every 8th split (independent loads in flight, 128-byte coalesced rows), then the
// 8 partial quires of an output are combined through LDS with carry-propagating adds
// (8 outputs and 32 thread rows where there are few outputs and 200 or more splits).
// Integer addition modulo 2^(32 L) is associative, so the order does not matter.
// With few splits one thread per output (ZG = 1) is enough.
template <class FIN, class Out, int MERGE_ZG>
__global__ __launch_bounds__(256) void split_merge_kernel(SplitWs ws, int splits, int64_t M, int64_t N,
                                                          const typename Storage<FIN::N>::T* __restrict__ bias,
                                                          void* __restrict__ C, int fout, Out out) {
    typedef Arith<FIN> AR;
    constexpr int L = AR::L;
    constexpr int MERGE_OUTS = 256 / MERGE_ZG;
    __shared__ uint32_t part_s[MERGE_ZG > 1 ? MERGE_ZG : 1][MERGE_ZG > 1 ? MERGE_OUTS : 1][L];
    __shared__ uint32_t nar_s[MERGE_ZG > 1 ? MERGE_ZG : 1][MERGE_ZG > 1 ? MERGE_OUTS : 1];
    const int o = threadIdx.x % MERGE_OUTS, zg = threadIdx.x / MERGE_OUTS;
    const int64_t total = M * N;
    const int64_t idx = (int64_t)blockIdx.x * MERGE_OUTS + o;
    const bool live = idx < total;
    const int64_t m = live ? idx / N : 0, n = live ? idx % N : 0;
    uint32_t q[L];
#pragma unroll
    for (int l = 0; l < L; ++l) q[l] = 0;
    uint32_t nar = 0;
    if (live) {
#pragma unroll 4
        for (int z = zg; z < splits; z += MERGE_ZG) {
            uint32_t part[L];
#pragma unroll
            for (int l = 0; l < L; ++l) part[l] = ws.limbs[((int64_t)z * total + idx) * L + l];
            quire_merge<L>(q, part);
            nar |= ws.rowflag[(int64_t)z * M + m] | ws.colflag[(int64_t)z * N + n];
        }
    }
    if (MERGE_ZG > 1) {
#pragma unroll
        for (int l = 0; l < L; ++l) part_s[zg][o][l] = q[l];
        nar_s[zg][o] = nar;
        __syncthreads();
        if (zg != 0) return;
#pragma unroll
        for (int g = 1; g < MERGE_ZG; ++g) {
            uint32_t part[L];
#pragma unroll
            for (int l = 0; l < L; ++l) part[l] = part_s[g][o][l];
            quire_merge<L>(q, part);
            nar |= nar_s[g][o];
        }
    }
    if (!live) return;
    bool isnar = nar != 0;
    if (bias) {
        const uint32_t bp = bias[n];
        if (bp == FIN::NAR) isnar = true;
        else AR::add_value(q, AR::stage(bp));
    }
    int64_t at;
    void* dst = merge_dest(out, C, m, n, at);
    round_store<QuireAccum<FIN>, L>(q, isnar, fout, dst, at);
}

// Bias gradient of a convolution (the row sum of the backward-weight pass against a column of
// ones): dbias[k] = round_fout( sum_{n,i} dy[n][k][i] * 1 ), one quire per channel.  Workgroup
// (k, s) sums slice s of the batch for channel k: every thread adds 16-byte runs of the channel's
// planes into a private quire (posit<8,0> decodes through an LDS table), the 256 private quires
// are merged pairwise through LDS (exact: integer addition).  With one slice thread 0 rounds and
// stores; with several, the slice's quire and NaR flag go to the workspace and
// bias_grad_finish_kernel merges the slices of a channel and rounds once.
template <class FIN>
__global__ __launch_bounds__(256) void bias_grad_kernel(const typename Storage<FIN::N>::T* __restrict__ dy, void* __restrict__ dbias,
                                                        int fout, int batch, int channels, int spatial, int vec, int batch_per_slice,
                                                        uint32_t* __restrict__ partial) {
    typedef Arith<FIN> AR;
    typedef typename Storage<FIN::N>::T T;
    constexpr int L = AR::L;
    constexpr int V = 16 / (int)sizeof(T);
    constexpr bool TABLE = FIN::N == 8 && FIN::ES == 0;
    __shared__ uint32_t part[128][L];
    __shared__ uint32_t nar_s;
    __shared__ int32_t tab[TABLE ? 256 : 1];
    const int k = blockIdx.x, t = threadIdx.x;
    const int n_lo = blockIdx.y * batch_per_slice;
    const int n_hi = n_lo + batch_per_slice < batch ? n_lo + batch_per_slice : batch;
    const int nb = n_hi > n_lo ? n_hi - n_lo : 0;
    uint32_t q[L];
#pragma unroll
    for (int l = 0; l < L; ++l) q[l] = 0;
    bool nar = false;
    if (t == 0) nar_s = 0;
    if constexpr (TABLE) {
        tab[t] = (int32_t)AR::stage((uint32_t)t);
        __syncthreads();
    }
    auto add = [&](uint32_t v) {
        if (v == FIN::NAR) nar = true;
        else if constexpr (TABLE) q[0] += (uint32_t)tab[v] << FIN::MAXS;
        else AR::add_value(q, AR::stage(v));
    };
    if (vec) {  // spatial is a multiple of V and the tensor is 16-byte aligned
        const int per_plane = spatial / V;
        const int chunks = nb * per_plane;
#pragma unroll 4
        for (int c = t; c < chunks; c += 256) {
            const int n = c / per_plane, i = (c - n * per_plane) * V;
            const uint4 w = *reinterpret_cast<const uint4*>(dy + ((int64_t)(n_lo + n) * channels + k) * spatial + i);
            const uint32_t words[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
            for (int e = 0; e < V; ++e)
                add((words[e * (int)sizeof(T) / 4] >> (8 * ((e * (int)sizeof(T)) & 3))) & (uint32_t)(T)~(T)0);
        }
    } else {
        const int total = nb * spatial;
        for (int e = t; e < total; e += 256) {
            const int n = e / spatial, i = e - n * spatial;
            add(dy[((int64_t)(n_lo + n) * channels + k) * spatial + i]);
        }
    }
    __syncthreads();
    if (nar) nar_s = 1;  // benign race: every writer stores the same value
    for (int half = 128; half >= 1; half >>= 1) {
        if (t >= half && t < 2 * half) {
#pragma unroll
            for (int l = 0; l < L; ++l) part[t - half][l] = q[l];
        }
        __syncthreads();
        if (t < half) {
            uint32_t o[L];
#pragma unroll
            for (int l = 0; l < L; ++l) o[l] = part[t][l];
            quire_merge<L>(q, o);
        }
        __syncthreads();
    }
    if (t != 0) return;
    if (gridDim.y == 1) {
        round_store<QuireAccum<FIN>, L>(q, nar_s != 0, fout, dbias, k);
    } else {  // [slice][channel][L limbs + flag]
        uint32_t* slot = partial + ((int64_t)blockIdx.y * channels + k) * (L + 1);
#pragma unroll
        for (int l = 0; l < L; ++l) slot[l] = q[l];
        slot[L] = nar_s;
    }
}

template <class FIN>
__global__ __launch_bounds__(256) void bias_grad_finish_kernel(const uint32_t* __restrict__ partial, int slices, int channels,
                                                               void* __restrict__ dbias, int fout) {
    constexpr int L = Arith<FIN>::L;
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (k >= channels) return;
    uint32_t q[L];
#pragma unroll
    for (int l = 0; l < L; ++l) q[l] = 0;
    uint32_t nar = 0;
    for (int s = 0; s < slices; ++s) {
        const uint32_t* slot = partial + ((int64_t)s * channels + k) * (L + 1);
        uint32_t o[L];
#pragma unroll
        for (int l = 0; l < L; ++l) o[l] = slot[l];
        quire_merge<L>(q, o);
        nar |= slot[L];
    }
    round_store<QuireAccum<FIN>, L>(q, nar != 0, fout, dbias, k);
}

// Slices of the batch per channel: enough workgroups to occupy the chip, at least 8192 elements each.
inline int bias_grad_slices(int batch, int channels, int spatial) {
    if (channels <= 0 || batch <= 1) return 1;
    int want = (512 + channels - 1) / channels;
    const int64_t per_channel = (int64_t)batch * spatial;
    const int64_t by_work = per_channel / 8192;
    if (want > by_work) want = (int)by_work;
    if (want > batch) want = batch;
    if (want > 64) want = 64;
    return want < 1 ? 1 : want;
}

template <class FIN>
size_t bias_grad_ws_bytes(int batch, int channels, int spatial) {
    const int s = bias_grad_slices(batch, channels, spatial);
    return s > 1 ? (size_t)s * channels * (Arith<FIN>::L + 1) * sizeof(uint32_t) : 0;
}

// `partial` must hold bias_grad_ws_bytes<FIN>() bytes (may be null when that is 0).
template <class FIN>
hipError_t launch_bias_grad(hipStream_t stream, const void* dy, void* dbias, int fout, int batch, int channels, int spatial,
                            void* partial) {
    typedef typename Storage<FIN::N>::T T;
    constexpr int V = 16 / (int)sizeof(T);
    const int vec = (spatial % V == 0) && (((uintptr_t)dy) % 16 == 0);
    const int slices = bias_grad_slices(batch, channels, spatial);
    const int per = (batch + slices - 1) / slices;
    const int used = per > 0 ? (batch + per - 1) / per : 1;  // slices that actually hold images
    hipLaunchKernelGGL(bias_grad_kernel<FIN>, dim3((unsigned)channels, (unsigned)(slices > 1 ? used : 1)), dim3(256), 0, stream,
                       (const T*)dy, dbias, fout, batch, channels, spatial, vec, slices > 1 ? per : batch, (uint32_t*)partial);
    PNN_CHECK_LAUNCH();
    if (slices > 1)
        hipLaunchKernelGGL(bias_grad_finish_kernel<FIN>, dim3((unsigned)((channels + 255) / 256)), dim3(256), 0, stream,
                           (const uint32_t*)partial, used, channels, dbias, fout);
    return hipGetLastError();
}

// Backward-data pass, NaR weights.  dx[n,c,h,w] sums dy[n,k,oh,ow] * w[k,c,r,s] over the (k,r,s,oh,ow) with
// oh*sh + r - ph == h and ow*sw + s - pw == w, so a NaR weight w[k,c,r,s] makes NaR exactly the positions of
// channel c that its tap (r,s) reaches from some output position -- not the whole channel, as a column flag of
// the implicit matrix product would.  The product kernels therefore stage NaR weights of this pass as zeros, and
// this kernel, launched after them on the same stream, writes NaR to those positions: one thread per weight, which
// returns at once unless its weight is NaR (the common case: one read of the weight tensor).
template <class T>
__global__ __launch_bounds__(256) void bwd_data_nar_weights_kernel(const T* __restrict__ w, uint32_t w_nar, ConvGeom g, void* __restrict__ dx,
                                                                   int fout) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t total = (int64_t)g.K * g.C * g.R * g.S;
    if (i >= total || (uint32_t)w[i] != w_nar) return;
    const int s = (int)(i % g.S), r = (int)((i / g.S) % g.R), c = (int)((i / ((int64_t)g.R * g.S)) % g.C);
    const FmtRT fo = fmt_of_code(fout);
    const uint32_t nar = fo.nar();
    for (int n = 0; n < g.N; ++n)
        for (int oh = 0; oh < g.OH; ++oh) {
            const int h = oh * g.sh + r - g.ph;
            if (h < 0 || h >= g.H) continue;
            for (int ow = 0; ow < g.OW; ++ow) {
                const int x = ow * g.sw + s - g.pw;
                if (x < 0 || x >= g.W) continue;
                const int64_t at = (((int64_t)n * g.C + c) * g.H + h) * g.W + x;
                if (fo.n <= 8) ((uint8_t*)dx)[at] = (uint8_t)nar;
                else if (fo.n <= 16) ((uint16_t*)dx)[at] = (uint16_t)nar;
                else ((uint32_t*)dx)[at] = nar;
            }
        }
}

template <class FIN>
void launch_bwd_data_nar_weights(hipStream_t stream, const void* w, const ConvGeom& g, void* dx, int fout) {
    typedef typename Storage<FIN::N>::T T;
    const int64_t total = (int64_t)g.K * g.C * g.R * g.S;
    if (total <= 0 || g.N <= 0) return;
    hipLaunchKernelGGL(bwd_data_nar_weights_kernel<T>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, (const T*)w,
                       (uint32_t)FIN::NAR, g, dx, fout);
}

// ---- host side ----

template <class FIN, class Out>
hipError_t launch_split_merge(hipStream_t stream, const SplitWs& ws, int splits, int64_t M, int64_t N, const void* bias, void* C, int fout,
                        const Out& out) {
    typedef typename Storage<FIN::N>::T TI;
    const int64_t total = M * N;
    if (splits >= 200 && total <= ((int64_t)1 << 18)) {  // few outputs, very many slices (backward-weight): 32 thread rows share the slices of an output
        hipLaunchKernelGGL((split_merge_kernel<FIN, Out, 32>), dim3((unsigned)((total + 7) / 8)), dim3(256), 0, stream, ws, splits, M, N,
                           (const TI*)bias, C, fout, out);
    } else if (splits >= 16) {
        hipLaunchKernelGGL((split_merge_kernel<FIN, Out, 8>), dim3((unsigned)((total + 31) / 32)), dim3(256), 0, stream, ws, splits, M, N,
                           (const TI*)bias, C, fout, out);
    } else {
        hipLaunchKernelGGL((split_merge_kernel<FIN, Out, 1>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, ws, splits, M, N,
                           (const TI*)bias, C, fout, out);
    }
    return hipGetLastError();
}

struct GemmPlan {
    int splits;
    int64_t k_per_split;
    size_t ws_bytes;
};

// How many ways to split the reduction: when the output tiles alone leave the
// 256 CUs short of about four workgroups each and the reduction is long enough
// to keep at least 256 steps per slice.
inline GemmPlan plan_split(int64_t M, int64_t N, int64_t K, int BM, int BN, int L, int KT = GEMM_KT) {
    GemmPlan p;
    const int64_t tiles = ((M + BM - 1) / BM) * ((N + BN - 1) / BN);
    int splits = 1;
    const int64_t target = 1024;
    if (tiles < target && K >= 1024) {
        int64_t s = (target + tiles - 1) / (tiles > 0 ? tiles : 1);
        const int64_t max_by_k = K / 256;
        if (s > max_by_k) s = max_by_k;
        if (s > 256) s = 256;
        if (s >= 2) splits = (int)s;
    }
    int64_t kps = (K + splits - 1) / splits;
    kps = (kps + KT - 1) / KT * KT;
    if (kps < KT) kps = KT;
    splits = (int)((K + kps - 1) / kps);
    if (splits < 1) splits = 1;
    p.splits = splits;
    p.k_per_split = kps;
    p.ws_bytes = splits > 1 ? (size_t)splits * ((size_t)M * N * L + M + N) * sizeof(uint32_t) : 0;
    return p;
}

template <class FIN, class OpA, class OpB, class Out, int TM, int TN, class AR = DefaultAccum<FIN>>
hipError_t launch_quire_gemm(hipStream_t stream, const OpA& opa, const OpB& opb, const Out& out,
                             int64_t M, int64_t N, int64_t K, const void* bias, void* C, int fout,
                             void* workspace, const GemmPlan& plan) {
    typedef typename Storage<FIN::N>::T TI;
    constexpr int BM = 16 * TM, BN = 16 * TN, L = AR::L;
    if (plan.splits > 1 && !AR::SPLITTABLE) return hipErrorInvalidValue;  // order-dependent accumulation cannot be split
    const int64_t tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    SplitWs ws;
    ws.limbs = nullptr;
    ws.rowflag = nullptr;
    ws.colflag = nullptr;
    if (plan.splits > 1) {
        ws.limbs = (uint32_t*)workspace;
        ws.rowflag = ws.limbs + (size_t)plan.splits * M * N * L;
        ws.colflag = ws.rowflag + (size_t)plan.splits * M;
    }
    dim3 grid((unsigned)(tiles_m * tiles_n), 1, (unsigned)plan.splits);
    hipLaunchKernelGGL((quire_gemm_kernel<FIN, OpA, OpB, Out, TM, TN, AR>), grid, dim3(GEMM_THREADS), 0, stream,
                       opa, opb, out, M, N, K, plan.k_per_split, (const TI*)bias, C, fout, ws, (int)tiles_n);
    PNN_CHECK_LAUNCH();
    if (plan.splits > 1) return launch_split_merge<FIN, Out>(stream, ws, plan.splits, M, N, bias, C, fout, out);
    return hipSuccess;
}

}  // namespace pnn
