/* positnn.h - C ABI of the quire-exact posit library for AMD MI355X (gfx950).
 *
 * The library implements the hot path of posit neural-network training as
 * described in "PositNN: Training Deep Neural Networks with Mixed Low-Precision
 * Posit" (arXiv 2105.00053): every matrix product and convolution (forward,
 * backward-data, backward-weight) is a set of dot products whose operands are
 * posit<n,es> numbers (Sec. 2, Eq. 2), whose products are accumulated without
 * any rounding in a quire (Sec. 2; widths in Table 1) and which are rounded to a
 * posit exactly once at the end (Sec. 3.3, "option to use quires for the
 * accumulations").  Around it sit the bandwidth-bound helpers of Fig. 2:
 * tensor conversion, copies of a tensor in several posit formats, and the SGD
 * weight update.
 *
 * General conventions
 *  - Every data pointer is a DEVICE pointer owned by the caller.  The library
 *    never allocates, frees or keeps device memory and has no mutable global
 *    state; calls are asynchronous on `stream` (a hipStream_t passed as void*,
 *    NULL = the default stream).
 *  - posit<8,0> / <16,1> / <32,2> elements are stored as uint8 / uint16 / uint32
 *    bit patterns (other formats: see pnn_dtype); PNN_F32 / PNN_F64 are IEEE
 *    binary32 / binary64.
 *  - Outputs must not alias inputs, except `y` of posit_axpy (updated in place).
 *  - Every function returns a pnn_status.  Invalid arguments (null pointer,
 *    negative size, leading dimension too small, unknown format) give
 *    PNN_EINVAL and nothing is launched; a format combination that is not
 *    built gives PNN_EUNSUPPORTED; a workspace smaller than the matching
 *    *_workspace() query gives PNN_EWORKSPACE; a HIP launch error gives
 *    PNN_EHIP.  Zero-sized problems return PNN_OK and touch nothing.
 *  - Special values: the pattern 10...0 (NaR) in any operand that takes part in
 *    an output makes that output NaR, also when it is multiplied by zero.
 *  - The quire of format `fin` is a two's-complement integer of 32 / 128 / 512
 *    bits (Table 1) whose unit is minpos^2; it wraps modulo 2^bits if a sum ever
 *    leaves that range (Table 1 guarantees 127 / 32767 / 2^31-1 products).
 */
#ifndef POSITNN_H
#define POSITNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PNN_POSIT8_0 = 0,  /* posit<8,0>,  uint8  storage, 32-bit quire  (Table 1) */
    PNN_POSIT16_1 = 1, /* posit<16,1>, uint16 storage, 128-bit quire (Table 1) */
    PNN_POSIT32_2 = 2, /* posit<32,2>, uint32 storage, 512-bit quire (Table 1) */
    /* formats of the paper's experiments (Sec. 4) that Table 1 does not list; the quire has
     * 4(n-2)2^es + 1 + (n-1) bits rounded up to a multiple of 32; 10- and 12-bit patterns
     * occupy the low bits of a uint16: outputs carry 0 in the upper bits, inputs must too (a
     * set upper bit gives an unspecified value for that element, never an invalid access) */
    PNN_POSIT8_1 = 3,  /* posit<8,1>,  uint8,  64-bit quire  */
    PNN_POSIT8_2 = 4,  /* posit<8,2>,  uint8,  128-bit quire */
    PNN_POSIT10_1 = 5, /* posit<10,1>, uint16, 96-bit quire  */
    PNN_POSIT10_2 = 6, /* posit<10,2>, uint16, 160-bit quire */
    PNN_POSIT12_1 = 7, /* posit<12,1>, uint16, 96-bit quire  */
    PNN_POSIT12_2 = 8, /* posit<12,2>, uint16, 192-bit quire */
    PNN_F32 = 100,     /* IEEE binary32: posit_round / posit_convert only */
    PNN_F64 = 101      /* IEEE binary64: posit_round / posit_convert only */
} pnn_dtype;

typedef enum {
    PNN_OK = 0,
    PNN_EINVAL = 1,
    PNN_EUNSUPPORTED = 2,
    PNN_EWORKSPACE = 3,
    PNN_EHIP = 4
} pnn_status;

/* Quire-exact matrix product (Sec. 3.3; Linear layer forward, backward-data and
 * backward-weight are its three transposition cases, Sec. 3.1):
 *
 *   C[i,j] = round_fout( sum_k op(A)[i,k] * op(B)[k,j]  (+ bias[j]) ),  i < M, j < N
 *
 * op(X) = X or X^T (transX != 0).  All matrices are row-major as stored; lda,
 * ldb, ldc are row pitches in elements (lda >= K, or >= M when transA; ldb >= N,
 * or >= K when transB; ldc >= N).  A, B and bias (length N, may be NULL) are in
 * format `fin`, which also fixes the quire; C is in `fout`.  The sum is exact,
 * the bias enters the quire as bias*1, and one rounding (nearest, ties to the
 * even pattern, never to zero or NaR) produces C.  K == 0 gives the rounded
 * bias (or zero).  `workspace` (device, 16-byte aligned, else PNN_EINVAL) must hold
 * at least posit_gemm_workspace(...) bytes (else PNN_EWORKSPACE); it may be NULL
 * when that query returns 0.  Its contents on entry do not matter and are not
 * preserved (partial quires of a split reduction; both operands rewritten once:
 * for posit<8,0> products of 2^28 multiply-adds and more as two int8 digit planes
 * each, 2 bytes per element; for posit<8,1> / posit<8,2> products of 2^25 and more
 * (128 outputs each way, K from 256 to 8192) as four / eight; for posit<16,1> and the 10- / 12-bit formats from
 * 96 x 96 outputs on as doubles, 8 bytes per element). */
int posit_gemm(void* stream, int fin, int fout, int transA, int transB,
               int64_t M, int64_t N, int64_t K,
               const void* A, int64_t lda, const void* B, int64_t ldb,
               const void* bias, void* C, int64_t ldc,
               void* workspace, size_t workspace_bytes);

/* Bytes of device workspace posit_gemm wants for this problem (0 = none).  The arguments are those of
 * the call it sizes; the answer depends on fin, M, N and K only (fout, transA, transB are accepted so
 * that the query can follow any future kernel choice without a change of this interface). */
size_t posit_gemm_workspace(int fin, int fout, int transA, int transB, int64_t M, int64_t N, int64_t K);

/* posit_gemm for callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc).  Same result, arguments and status
 * codes as posit_gemm, but the workspace is a fixed array of PNN_GEMM_STATIC_SCRATCH_BYTES inside
 * the library's code object (each GPU the library runs on holds one copy until the process ends),
 * so the call neither takes a workspace nor allocates or frees anything.  A problem whose
 * posit_gemm_workspace() exceeds PNN_GEMM_STATIC_SCRATCH_BYTES returns PNN_EWORKSPACE with nothing
 * launched (72 MiB covers the 4096^3 posit<8,0> product and every matrix product of the five
 * benchmark configurations).  The device that owns the pointers and the stream must be the
 * current device.  Every call on a GPU uses that GPU's one array, which keeps the previous call's
 * contents (the kernels overwrite or clear what they read): calls that may overlap in time on one
 * GPU -- from different streams or threads -- race on it and must be serialised by the caller. */
#define PNN_GEMM_STATIC_SCRATCH_BYTES ((size_t)72 << 20)
int posit_gemm_static(void* stream, int fin, int fout, int transA, int transB,
                      int64_t M, int64_t N, int64_t K,
                      const void* A, int64_t lda, const void* B, int64_t ldb,
                      const void* bias, void* C, int64_t ldc);

/* 2-D convolution geometry (Sec. 3.1: layers follow LibTorch semantics):
 * cross-correlation, activations NCHW, weights [K][C][R][S], zero padding,
 * dilation 1, one group.  Output size OH = (H + 2*pad_h - R) / stride_h + 1. */
typedef struct {
    int64_t N, C, H, W; /* input batch, channels, height, width */
    int64_t K, R, S;    /* output channels, kernel height, kernel width */
    int64_t pad_h, pad_w, stride_h, stride_w;
} pnn_conv2d_desc;

/* y[n,k,oh,ow] = round_fout( sum_{c,r,s} x[n,c,oh*stride_h+r-pad_h,ow*stride_w+s-pad_w] * w[k,c,r,s] (+ bias[k]) )
 * taps outside the image contribute exact zeros.  x, w, bias (nullable) in fin; y in fout. */
int posit_conv2d_fwd(void* stream, int fin, int fout, const pnn_conv2d_desc* desc,
                     const void* x, const void* w, const void* bias, void* y,
                     void* workspace, size_t workspace_bytes);

/* Adjoint with respect to x: dx[n,c,h,w] = round_fout( sum of dy[n,k,oh,ow] * w[k,c,r,s]
 * over all (k,r,s,oh,ow) with oh*stride_h+r-pad_h == h and ow*stride_w+s-pad_w == w ): what
 * LibTorch's flow (W^T times dY, columns scattered back, Sec. 3.1) accumulates per position.
 * A tap (k,r,s) that reaches no output position from (h,w) is no term of that sum, so a NaR
 * weight makes NaR only the positions its tap reaches, a NaR dy entry the positions it is
 * scattered to (in the forward and backward-weight passes, by contrast, padded positions are
 * zero operands of a matrix product and NaR * 0 = NaR spreads over the whole channel / filter). */
int posit_conv2d_bwd_data(void* stream, int fin, int fout, const pnn_conv2d_desc* desc,
                          const void* dy, const void* w, void* dx,
                          void* workspace, size_t workspace_bytes);

/* Adjoint with respect to w: dw[k,c,r,s] = round_fout( sum_{n,oh,ow} dy[n,k,oh,ow] *
 * x[n,c,oh*stride_h+r-pad_h,ow*stride_w+s-pad_w] ): ONE quire over the whole
 * batch, one rounding.  dbias (nullable) receives round_fout( sum_{n,oh,ow} dy[n,k,oh,ow] ). */
int posit_conv2d_bwd_weight(void* stream, int fin, int fout, const pnn_conv2d_desc* desc,
                            const void* dy, const void* x, void* dw, void* dbias,
                            void* workspace, size_t workspace_bytes);

/* which: 0 = fwd, 1 = bwd_data, 2 = bwd_weight.  Bytes of workspace (0 = none) that the matching
 * call needs: device memory, 16-byte aligned (PNN_EINVAL otherwise), contents undefined on entry and
 * on return.  It holds the partial quires of a split reduction and, for posit<8,0>, the operands
 * rewritten once: as decoded 16-bit integers with the zero border written out (about twice the size of
 * the tensors), or, from 2^26 multiply-adds on, as int8 digit planes (forward and backward-data: twice
 * the gathered tensor, channels padded to 16; backward-weight: twice x and twice dy, the batch padded
 * to 16).  The calls of one stream may share one workspace.  The answer
 * depends on which, fin and desc (fout is accepted for the same reason as in posit_gemm_workspace). */
size_t posit_conv2d_workspace(int which, int fin, int fout, const pnn_conv2d_desc* desc);

/* The same four operations with the quire switched off (Sec. 3.3: the quire is an
 * option of the framework; Table 2 reports training "without quire").  Each output
 * is the chain  s_0 = 0,  s_t = round_fin( s_{t-1} + round_fin( a_t * b_t ) )  over
 * the terms t of its dot product in ascending order of the reduction index
 * (posit_gemm: k; fwd: (c,r,s); bwd_data: (k,r,s); bwd_weight and dbias: (n,oh,ow);
 * the last index fastest), then  s = round_fin( s + bias )  when a bias is given,
 * and the result stored is round_fout(s).  Padded positions are zero operands as
 * above (adding their zero products changes no chain) and bwd_data has the terms of
 * posit_conv2d_bwd_data; NaR is absorbing.  Arguments, layouts and
 * status codes are those of the quire entry points; no workspace is needed (the
 * order-dependent reduction is never split).  The result in general differs from
 * the quire result; it is deterministic and independent of the launch shape. */
int posit_gemm_noquire(void* stream, int fin, int fout, int transA, int transB,
                       int64_t M, int64_t N, int64_t K,
                       const void* A, int64_t lda, const void* B, int64_t ldb,
                       const void* bias, void* C, int64_t ldc);
int posit_conv2d_fwd_noquire(void* stream, int fin, int fout, const pnn_conv2d_desc* desc,
                             const void* x, const void* w, const void* bias, void* y);
int posit_conv2d_bwd_data_noquire(void* stream, int fin, int fout, const pnn_conv2d_desc* desc,
                                  const void* dy, const void* w, void* dx);
int posit_conv2d_bwd_weight_noquire(void* stream, int fin, int fout, const pnn_conv2d_desc* desc,
                                    const void* dy, const void* x, void* dw, void* dbias);

/* The same update for several tensors in one launch (Fig. 2, optimizer: one SGD step touches every
 * parameter tensor of the model, most of them small).  items is a HOST array of count entries; each
 * is updated exactly as posit_axpy would: y[i] = round_fy(y[i] + alpha * x[i]), y_copy (nullable per
 * item) receiving round_fcopy of the new y.  The tensors must not overlap. */
typedef struct {
    const void* x; /* device, fx */
    void* y;       /* device, fy, in place */
    void* y_copy;  /* device, fcopy, or NULL */
    int64_t n;
} pnn_axpy_item;
int posit_axpy_multi(void* stream, int fx, int fy, uint32_t alpha_bits, int count,
                     const pnn_axpy_item* items, int fcopy);

/* Elementary functions (Fig. 2: Sigmoid and TanH activations; exp and log are the pieces of the
 * Cross Entropy loss).  The paper prints no algorithm: y[i] is the correctly rounded posit<fmt> of
 * the real function at the value of x[i] (nearest, ties to the even pattern, never 0 or NaR for a
 * nonzero finite value: e^x and sigmoid clamp to minpos / maxpos).  NaR gives NaR; log of zero or
 * of a negative value gives NaR; exact cases: exp(0) = 1, log(1) = 0, tanh(0) = 0, sigmoid(0) = 1/2.
 * Formats of at most 16 bits (PNN_EUNSUPPORTED for posit<32,2>). */
typedef enum { PNN_SIGMOID = 0, PNN_TANH = 1, PNN_EXP = 2, PNN_LOG = 3 } pnn_function;
int posit_unary(void* stream, int fn, int fmt, int64_t n, const void* x, void* y);

/* Gradient through PNN_SIGMOID or PNN_TANH from the forward OUTPUT y_fwd (format fmt_y), in posit
 * operations of the gradient's format fmt_d, each rounded: with y' = round_fmt_d(y_fwd),
 * sigmoid: dx = dy * (y' * (1 - y'));  tanh: dx = dy * (1 - y' * y').  dy and dx are in fmt_d. */
int posit_unary_bwd(void* stream, int fn, int fmt_y, int fmt_d, int64_t n,
                    const void* y_fwd, const void* dy, void* dx);

/* Softmax cross entropy with mean reduction (Fig. 2), computed in the loss format f_loss (Fig. 3: the
 * loss stage has its own precision; Sec. 4, Table 4: posit(10,2) / posit(12,2)).  logits is
 * [batch][classes] in f_logits, labels holds one int32 class index per row (device memory).  Per
 * row, every operation rounded to f_loss: z_j = round(logit_j); m = max_j z_j; t_j = z_j - m;
 * e_j = exp(t_j); S = round(sum_j e_j) with the sum exact (quire); p_j = e_j / S;
 * g_j = p_j - [j == label]; row loss = log(S) - t_label.  Outputs (each may be NULL, not both):
 * dlogits[b][j] = round_f_grad(g_j / batch), exact division, one rounding; loss (one pattern of
 * f_loss) = round((sum_b row loss_b) / batch), exact sum (quire) and division, one rounding.  A NaR
 * logit or a label outside 0..classes-1 makes that row's gradient and the loss NaR.  Formats of at
 * most 16 bits.  One workgroup processes the whole batch: meant for batch x classes of a few 10^5. */
int posit_cross_entropy(void* stream, int f_logits, int f_loss, int f_grad, int64_t batch, int64_t classes,
                        const void* logits, const int32_t* labels, void* loss, void* dlogits);

/* Mean squared error (Fig. 2) over n elements in the loss format: d_i = round_f_loss(pred_i) -
 * round_f_loss(target_i) rounded to f_loss; loss = round_f_loss((sum_i d_i^2) / n), squares summed
 * exactly in f_loss's quire; dpred_i = round_f_grad(2 d_i / n), exact inside.  pred and target are
 * in f_pred.  NaR anywhere makes the loss and that element's gradient NaR.  Outputs may be NULL
 * (not both).  Formats of at most 16 bits. */
int posit_mse(void* stream, int f_pred, int f_loss, int f_grad, int64_t n,
              const void* pred, const void* target, void* loss, void* dpred);

/* Float tensor -> posit tensor (Fig. 2, tensor conversion): dst[i] = round_dst(src[i]),
 * src_float in {PNN_F32, PNN_F64}.  NaN and +-Inf give NaR, -0.0 gives 0,
 * nonzero values never round to zero (they clamp to +-minpos / +-maxpos). */
int posit_round(void* stream, int src_float, int dst_posit, int64_t n, const void* src, void* dst);

/* posit -> posit of another format (one rounding; exact when widening
 * <8,0> -> <16,1> -> <32,2>), or posit -> PNN_F32 / PNN_F64 (exact, except
 * posit<32,2> -> binary32 which rounds to nearest even; NaR gives NaN). */
int posit_convert(void* stream, int src, int dst, int64_t n, const void* src_ptr, void* dst_ptr);

/* SGD-style update (Fig. 2, optimizer): y[i] = round_fy( y[i] + alpha * x[i] ),
 * exact inside, one rounding.  alpha_bits is a posit pattern of format fy (for
 * SGD: the rounded value of -learning_rate); x is in fx, y in fy (in place).
 * When y_copy is not NULL it receives round_fcopy(new y[i]): the narrow copy
 * of the weights that the compute kernels read (Sec. 3.3).  fcopy is ignored
 * when y_copy is NULL. */
int posit_axpy(void* stream, int fx, int fy, uint32_t alpha_bits, int64_t n,
               const void* x, void* y, int fcopy, void* y_copy);

/* ---- exact layer glue (Fig. 2: ReLU activation, maximum and average pooling) ----
 * None of these is a dot product, but each has an exact definition on posit patterns, so a
 * whole training step can stay on the device and remain bit-comparable with the oracle.
 * posit ordering is the signed-integer ordering of the patterns (Sec. 2: two's complement). */

/* y[i] = x[i] if x[i] > 0, else 0 (NaR stays NaR).  In place allowed (y == x). */
int posit_relu(void* stream, int fmt, int64_t n, const void* x, void* y);

/* dx[i] = dy[i] where the forward output y_fwd[i] is positive, else 0 (NaR where y_fwd[i] is NaR).
 * y_fwd in fmt_y, dy and dx in fmt_d. */
int posit_relu_bwd(void* stream, int fmt_y, int fmt_d, int64_t n, const void* y_fwd, const void* dy, void* dx);

/* Non-overlapping kh x kw maximum pooling of `planes` images of H x W (planes = batch * channels):
 * y[p,oh,ow] = max over the window, compared as signed integers (NaR is the smallest pattern);
 * idx[p,oh,ow] (uint8) = position of the FIRST maximum in row-major window order.  H, W must be
 * multiples of kh, kw; kh*kw <= 255. */
int posit_maxpool2d_fwd(void* stream, int fmt, int64_t planes, int64_t H, int64_t W, int64_t kh, int64_t kw,
                        const void* x, void* y, void* idx);

/* Routes dy[p,oh,ow] to the recorded window position of dx, zeros elsewhere. */
int posit_maxpool2d_bwd(void* stream, int fmt, int64_t planes, int64_t H, int64_t W, int64_t kh, int64_t kw,
                        const void* dy, const void* idx, void* dx);

/* Non-overlapping kh x kw average pooling with kh*kw a power of two: the exact quire dot product of the
 * window with the weight 1/(kh*kw), one rounding: y = round_fout( sum_window x * 2^-log2(kh*kw) ).
 * The weight must be a posit of fin: a window that is no power of two, or larger than 1/minpos of fin
 * (posit<8,0>: more than 64 elements), gives PNN_EUNSUPPORTED.
 * Identical to posit_conv2d_fwd on a one-channel image with a constant kernel and stride = window. */
int posit_avgpool2d_fwd(void* stream, int fin, int fout, int64_t planes, int64_t H, int64_t W, int64_t kh, int64_t kw,
                        const void* x, void* y);

/* Adjoint of the above: dx[p,h,w] = round_fout( dy[p,h/kh,w/kw] * 2^-log2(kh*kw) ). */
int posit_avgpool2d_bwd(void* stream, int fin, int fout, int64_t planes, int64_t H, int64_t W, int64_t kh, int64_t kw,
                        const void* dy, void* dx);

/* Human-readable name of a status code (static storage, never NULL). */
const char* posit_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* POSITNN_H */
