// Host-side reading of a pnn_conv2d_desc: validation, output size, and the
// dimensions of the implicit GEMM each of the three passes runs as (paper
// Sec. 3.1: convolution forward, backward-data, backward-weight).
#pragma once

#include "api_common.h"
#include "quire_gemm.h"

namespace pnn {

inline bool conv_geom(const pnn_conv2d_desc* d, ConvGeom* g) {
    if (!d) return false;
    if (d->N < 0 || d->C < 0 || d->H <= 0 || d->W <= 0 || d->K < 0 || d->R <= 0 || d->S <= 0) return false;
    if (d->pad_h < 0 || d->pad_w < 0 || d->stride_h <= 0 || d->stride_w <= 0) return false;
    if (d->H + 2 * d->pad_h < d->R || d->W + 2 * d->pad_w < d->S) return false;
    const int64_t lim = (int64_t)1 << 30;
    if (d->N >= lim || d->C >= lim || d->H >= lim || d->W >= lim || d->K >= lim || d->R >= lim || d->S >= lim) return false;
    g->N = (int)d->N; g->C = (int)d->C; g->H = (int)d->H; g->W = (int)d->W;
    g->K = (int)d->K; g->R = (int)d->R; g->S = (int)d->S;
    g->ph = (int)d->pad_h; g->pw = (int)d->pad_w; g->sh = (int)d->stride_h; g->sw = (int)d->stride_w;
    g->OH = (int)((d->H + 2 * d->pad_h - d->R) / d->stride_h + 1);
    g->OW = (int)((d->W + 2 * d->pad_w - d->S) / d->stride_w + 1);
    // every index the kernels form must fit 31 bits
    if ((int64_t)g->C * g->R * g->S >= lim || (int64_t)g->K * g->R * g->S >= lim) return false;
    if ((int64_t)g->N * g->OH * g->OW >= lim || (int64_t)g->N * g->H * g->W >= lim) return false;
    return true;
}

struct ConvDims {
    int64_t M, N, K;
};

inline ConvDims conv_dims(int which, const ConvGeom& g) {
    ConvDims d;
    if (which == 0) { d.M = (int64_t)g.N * g.OH * g.OW; d.N = g.K; d.K = (int64_t)g.C * g.R * g.S; }
    else if (which == 1) { d.M = (int64_t)g.N * g.H * g.W; d.N = g.C; d.K = (int64_t)g.K * g.R * g.S; }
    else { d.M = g.K; d.N = (int64_t)g.C * g.R * g.S; d.K = (int64_t)g.N * g.OH * g.OW; }
    return d;
}

}  // namespace pnn
