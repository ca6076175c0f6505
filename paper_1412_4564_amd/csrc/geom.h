// Host-side geometry of one convolution call: validated sizes, derived counts.
// MatConvNet manual (arXiv 1412.4564) Sec. 4.1: output size, groups, size error.
#pragma once
#include <stdint.h>
#include "../../include/mcnconv.h"

namespace mcn {

// Plain-old-data handed to kernels by value.
struct Geom {
    int H, W, D, N;
    int Hf, Wf, Df, K;
    int Sh, Sw;
    int Pt, Pb, Pl, Pr;
    int Ho, Wo;
    int G;    // groups = D / Df
    int Kg;   // filters per group = K / G
};

inline int64_t numel_x(const Geom &g) { return (int64_t)g.H * g.W * g.D * g.N; }
inline int64_t numel_w(const Geom &g) { return (int64_t)g.Hf * g.Wf * g.Df * g.K; }
inline int64_t numel_y(const Geom &g) { return (int64_t)g.Ho * g.Wo * g.K * g.N; }

// Validate the descriptor (Sec. 4.1: "Output size", "Filter groups") and fill g.
inline int make_geom(const mcn_conv_desc *d, Geom *g) {
    if (!d) return MCN_BAD_ARG;
    if (d->H < 1 || d->W < 1 || d->D < 1 || d->N < 1) return MCN_BAD_ARG;
    if (d->Hf < 1 || d->Wf < 1 || d->Df < 1 || d->K < 1) return MCN_BAD_ARG;
    if (d->stride_h < 1 || d->stride_w < 1) return MCN_BAD_ARG;
    if (d->pad_top < 0 || d->pad_bottom < 0 || d->pad_left < 0 || d->pad_right < 0) return MCN_BAD_ARG;
    if (d->precision < MCN_PREC_FP32 || d->precision > MCN_PREC_FP32_BF16X3) return MCN_BAD_ARG;
    if (d->D % d->Df != 0) return MCN_BAD_GROUPS;
    const int G = d->D / d->Df;
    if (d->K % G != 0) return MCN_BAD_GROUPS;
    const int64_t hp = (int64_t)d->H + d->pad_top + d->pad_bottom;
    const int64_t wp = (int64_t)d->W + d->pad_left + d->pad_right;
    if (hp < d->Hf || wp < d->Wf) return MCN_FILTER_TOO_LARGE;
    const int64_t Ho = (hp - d->Hf) / d->stride_h + 1;   // numerator >= 0: plain division is floor
    const int64_t Wo = (wp - d->Wf) / d->stride_w + 1;
    const int64_t lim = (int64_t)1 << 31;
    if (hp >= lim || wp >= lim) return MCN_UNSUPPORTED;
    g->H = d->H; g->W = d->W; g->D = d->D; g->N = d->N;
    g->Hf = d->Hf; g->Wf = d->Wf; g->Df = d->Df; g->K = d->K;
    g->Sh = d->stride_h; g->Sw = d->stride_w;
    g->Pt = d->pad_top; g->Pb = d->pad_bottom; g->Pl = d->pad_left; g->Pr = d->pad_right;
    g->Ho = (int)Ho; g->Wo = (int)Wo;
    g->G = G; g->Kg = d->K / G;
    // 32-bit element offsets are used on the device.
    if ((double)d->H * d->W * d->D * d->N >= (double)lim) return MCN_UNSUPPORTED;
    if ((double)d->Hf * d->Wf * d->Df * d->K >= (double)lim) return MCN_UNSUPPORTED;
    if ((double)Ho * Wo * d->K * d->N >= (double)lim) return MCN_UNSUPPORTED;
    return MCN_OK;
}

}  // namespace mcn
