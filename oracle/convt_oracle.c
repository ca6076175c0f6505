/*
 * CPU oracle for the convolution transpose block (forward, and the three
 * derivatives).
 *
 * THIS IS TEST INFRASTRUCTURE.  It exists so that the GPU library can be
 * checked against something that a reader can compare with the paper by eye.
 * Only tests, the smoke check and the benchmark's CPU-baseline leg may call
 * it; the product path never does.  It shares no code with the GPU path, and
 * none with the convolution oracle either (tests play the two against each
 * other through the transposition identity, which only means something if
 * they are written separately).
 *
 * What it follows (MatConvNet manual, arXiv 1412.4564):
 *   - Sec. 4.2 "Convolution transpose": the block computes vec y = M^T vec x,
 *     where M is the matrix of the convolution block of Sec. 4.1 that would
 *     take an array of y's shape to an array of x's shape with the same
 *     filter bank, stride = the upsampling factors and padding = the crops;
 *   - Sec. 6.2: in one dimension that convolution is
 *         x_i = sum_{i'} f_{i'} y_{S(i-1) + i' - C^-},
 *     so entry (i, i'') of M is f_{i'' - S(i-1) + C^-} (zero when that index
 *     falls outside 1..H'), and its transpose gives
 *         y_{i''} = sum_i f_{i'' - S(i-1) + C^-} x_i;
 *   - Sec. 4.2 / Sec. 5.3: the output height  H'' = S_h (H-1) + H' - C^- - C^+
 *     (the smallest of the S_h heights whose convolution has height H), and
 *     likewise the width;
 *   - Sec. 4.2: filter k of the bank is the slice f[:,:,k,:], i.e. the THIRD
 *     index of f runs over output channels and the FOURTH over input channels;
 *   - Sec. 2.3.2 eq. (projected): the backward mode returns d<p,y>/dx and
 *     d<p,y>/df for p = dzdy.  y is bilinear in (x, f), so these are the same
 *     products regrouped.
 *
 * Readings taken where the manual is silent:
 *   - a bias b (one value per output channel) is added to every sample of y,
 *     as in the convolution block; its derivative is the sum of dzdy over
 *     i'', j'' and the batch;
 *   - filter groups: with G groups, x has D channels (G divides D), f is
 *     H' x W' x K' x D and y has G*K' channels; input channels
 *     m*D/G .. (m+1)*D/G - 1 feed output channels m*K' .. (m+1)*K' - 1.  This
 *     is the transpose of the grouped convolution of Sec. 4.1 "Filter groups"
 *     run from y's shape to x's shape;
 *   - arrays are stored first index fastest (the vec() order of Sec. 2.3.1);
 *   - crops that leave no output (H'' < 1 or W'' < 1) are an error;
 *   - dzdf and dzdb are summed over the batch.
 *
 * Arithmetic: everything is double.  No blocking, no buffers, no BLAS: the
 * loops are the sum above in two dimensions.
 *
 * All indices below are 0-based: the filter index  i'' - S(i-1) + C^-
 * (1-based i'', i) becomes  io - S*i + Ct.
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t H, W, D, N;        /* x : H x W x D x N                                   */
    int32_t Hf, Wf, Kf, G;     /* f : H' x W' x K' x D ;  G groups, y has G*K' channels */
    int32_t Uh, Uw;            /* upsampling factors, vertical then horizontal        */
    int32_t Ct, Cb, Cl, Cr;    /* crops: top, bottom, left, right                     */
} orct_geom;

enum { ORCT_OK = 0, ORCT_BAD_ARG = 1, ORCT_BAD_GROUPS = 2, ORCT_CROP_TOO_LARGE = 3 };

/* Sec. 4.2:  H'' = S_h (H - 1) + H' - C^- - C^+  and the same for W''. */
int orct_output_size(const orct_geom *g, int32_t *Ho, int32_t *Wo) {
    if (!g) return ORCT_BAD_ARG;
    if (g->H < 1 || g->W < 1 || g->D < 1 || g->N < 1) return ORCT_BAD_ARG;
    if (g->Hf < 1 || g->Wf < 1 || g->Kf < 1 || g->G < 1) return ORCT_BAD_ARG;
    if (g->Uh < 1 || g->Uw < 1) return ORCT_BAD_ARG;
    if (g->Ct < 0 || g->Cb < 0 || g->Cl < 0 || g->Cr < 0) return ORCT_BAD_ARG;
    if (g->D % g->G != 0) return ORCT_BAD_GROUPS;
    const int64_t ho = (int64_t)g->Uh * (g->H - 1) + g->Hf - g->Ct - g->Cb;
    const int64_t wo = (int64_t)g->Uw * (g->W - 1) + g->Wf - g->Cl - g->Cr;
    if (ho < 1 || wo < 1) return ORCT_CROP_TOO_LARGE;
    if (Ho) *Ho = (int32_t)ho;
    if (Wo) *Wo = (int32_t)wo;
    return ORCT_OK;
}

int orct_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* addresses, first index fastest; K = G * Kf output channels */
#define XA(i, j, d, n)    ((int64_t)(i) + (int64_t)g->H  * ((j) + (int64_t)g->W  * ((d) + (int64_t)g->D * (n))))
#define FA(fi, fj, k, d)  ((int64_t)(fi) + (int64_t)g->Hf * ((fj) + (int64_t)g->Wf * ((k) + (int64_t)g->Kf * (d))))
#define YA(io, jo, c, n)  ((int64_t)(io) + (int64_t)Ho * ((jo) + (int64_t)Wo * ((c) + (int64_t)K * (n))))

/* One output sample: the 1-D sum of Sec. 6.2 taken over rows and columns and
 * over the input channels of the group that output channel c belongs to. */
static double forward_one(const orct_geom *g, const double *x, const double *f, const double *b,
                          int io, int jo, int c, int n) {
    const int Dg = g->D / g->G;          /* input channels per group            */
    const int grp = c / g->Kf;           /* group of this output channel        */
    const int k = c % g->Kf;             /* its place on the third axis of f    */
    double acc = b ? b[c] : 0.0;
    for (int d = grp * Dg; d < (grp + 1) * Dg; ++d)
        for (int j = 0; j < g->W; ++j) {
            const int fj = jo - g->Uw * j + g->Cl;
            if (fj < 0 || fj >= g->Wf) continue;         /* f is zero outside its support */
            for (int i = 0; i < g->H; ++i) {
                const int fi = io - g->Uh * i + g->Ct;
                if (fi < 0 || fi >= g->Hf) continue;
                acc += f[FA(fi, fj, k, d)] * x[XA(i, j, d, n)];
            }
        }
    return acc;
}

/* y = M^T x + b.  b may be NULL. */
int orct_forward(const orct_geom *g, const double *x, const double *f, const double *b, double *y) {
    int32_t Ho, Wo;
    int st = orct_output_size(g, &Ho, &Wo);
    if (st) return st;
    if (!x || !f || !y) return ORCT_BAD_ARG;
    const int K = g->G * g->Kf;
    const int64_t planes = (int64_t)g->N * K;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t t = 0; t < planes; ++t) {
        const int n = (int)(t / K), c = (int)(t % K);
        for (int jo = 0; jo < Wo; ++jo)
            for (int io = 0; io < Ho; ++io)
                y[YA(io, jo, c, n)] = forward_one(g, x, f, b, io, jo, c, n);
    }
    return ORCT_OK;
}

/* Forward at chosen places only: idx[] holds linear addresses into y. */
int orct_forward_at(const orct_geom *g, const double *x, const double *f, const double *b,
                    const int64_t *idx, int64_t count, double *out) {
    int32_t Ho, Wo;
    int st = orct_output_size(g, &Ho, &Wo);
    if (st) return st;
    if (!x || !f || !idx || !out) return ORCT_BAD_ARG;
    const int K = g->G * g->Kf;
    const int64_t total = (int64_t)Ho * Wo * K * g->N;
    for (int64_t t = 0; t < count; ++t)
        if (idx[t] < 0 || idx[t] >= total) return ORCT_BAD_ARG;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t t = 0; t < count; ++t) {
        int64_t a = idx[t];
        const int io = (int)(a % Ho); a /= Ho;
        const int jo = (int)(a % Wo); a /= Wo;
        const int c = (int)(a % K);
        const int n = (int)(a / K);
        out[t] = forward_one(g, x, f, b, io, jo, c, n);
    }
    return ORCT_OK;
}

/* dzdx = d<dzdy, y>/dx = M dzdy: x[i,j,d,n] enters y[io,jo,c,n] with the
 * coefficient f[io - Uh*i + Ct, jo - Uw*j + Cl, k, d]; running over the
 * filter index instead of io gives io = Uh*i + fi - Ct. */
static double backward_data_one(const orct_geom *g, int Ho, int Wo, const double *f, const double *dzdy,
                                int i, int j, int d, int n) {
    const int K = g->G * g->Kf;
    const int grp = d / (g->D / g->G);
    double acc = 0.0;
    for (int k = 0; k < g->Kf; ++k)
        for (int fj = 0; fj < g->Wf; ++fj) {
            const int jo = g->Uw * j + fj - g->Cl;
            if (jo < 0 || jo >= Wo) continue;            /* cropped away */
            for (int fi = 0; fi < g->Hf; ++fi) {
                const int io = g->Uh * i + fi - g->Ct;
                if (io < 0 || io >= Ho) continue;
                acc += f[FA(fi, fj, k, d)] * dzdy[YA(io, jo, grp * g->Kf + k, n)];
            }
        }
    return acc;
}

int orct_backward_data(const orct_geom *g, const double *f, const double *dzdy, double *dzdx) {
    int32_t Ho, Wo;
    int st = orct_output_size(g, &Ho, &Wo);
    if (st) return st;
    if (!f || !dzdy || !dzdx) return ORCT_BAD_ARG;
    const int64_t planes = (int64_t)g->N * g->D;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t t = 0; t < planes; ++t) {
        const int n = (int)(t / g->D), d = (int)(t % g->D);
        for (int j = 0; j < g->W; ++j)
            for (int i = 0; i < g->H; ++i)
                dzdx[XA(i, j, d, n)] = backward_data_one(g, Ho, Wo, f, dzdy, i, j, d, n);
    }
    return ORCT_OK;
}

int orct_backward_data_at(const orct_geom *g, const double *f, const double *dzdy,
                          const int64_t *idx, int64_t count, double *out) {
    int32_t Ho, Wo;
    int st = orct_output_size(g, &Ho, &Wo);
    if (st) return st;
    if (!f || !dzdy || !idx || !out) return ORCT_BAD_ARG;
    const int64_t total = (int64_t)g->H * g->W * g->D * g->N;
    for (int64_t t = 0; t < count; ++t)
        if (idx[t] < 0 || idx[t] >= total) return ORCT_BAD_ARG;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t t = 0; t < count; ++t) {
        int64_t a = idx[t];
        const int i = (int)(a % g->H); a /= g->H;
        const int j = (int)(a % g->W); a /= g->W;
        const int d = (int)(a % g->D);
        const int n = (int)(a / g->D);
        out[t] = backward_data_one(g, Ho, Wo, f, dzdy, i, j, d, n);
    }
    return ORCT_OK;
}

/* dzdf[fi,fj,k,d] = d<dzdy, y>/df: the coefficient of f[fi,fj,k,d] in
 * y[Uh*i + fi - Ct, Uw*j + fj - Cl, grp(d)*Kf + k, n] is x[i,j,d,n]. */
static double backward_filter_one(const orct_geom *g, int Ho, int Wo, const double *x, const double *dzdy,
                                  int fi, int fj, int k, int d) {
    const int K = g->G * g->Kf;
    const int c = (d / (g->D / g->G)) * g->Kf + k;
    double acc = 0.0;
    for (int n = 0; n < g->N; ++n)
        for (int j = 0; j < g->W; ++j) {
            const int jo = g->Uw * j + fj - g->Cl;
            if (jo < 0 || jo >= Wo) continue;
            for (int i = 0; i < g->H; ++i) {
                const int io = g->Uh * i + fi - g->Ct;
                if (io < 0 || io >= Ho) continue;
                acc += x[XA(i, j, d, n)] * dzdy[YA(io, jo, c, n)];
            }
        }
    return acc;
}

int orct_backward_filter(const orct_geom *g, const double *x, const double *dzdy, double *dzdf) {
    int32_t Ho, Wo;
    int st = orct_output_size(g, &Ho, &Wo);
    if (st) return st;
    if (!x || !dzdy || !dzdf) return ORCT_BAD_ARG;
    const int64_t slices = (int64_t)g->D * g->Kf;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t t = 0; t < slices; ++t) {
        const int d = (int)(t / g->Kf), k = (int)(t % g->Kf);
        for (int fj = 0; fj < g->Wf; ++fj)
            for (int fi = 0; fi < g->Hf; ++fi)
                dzdf[FA(fi, fj, k, d)] = backward_filter_one(g, Ho, Wo, x, dzdy, fi, fj, k, d);
    }
    return ORCT_OK;
}

int orct_backward_filter_at(const orct_geom *g, const double *x, const double *dzdy,
                            const int64_t *idx, int64_t count, double *out) {
    int32_t Ho, Wo;
    int st = orct_output_size(g, &Ho, &Wo);
    if (st) return st;
    if (!x || !dzdy || !idx || !out) return ORCT_BAD_ARG;
    const int64_t total = (int64_t)g->Hf * g->Wf * g->Kf * g->D;
    for (int64_t t = 0; t < count; ++t)
        if (idx[t] < 0 || idx[t] >= total) return ORCT_BAD_ARG;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t t = 0; t < count; ++t) {
        int64_t a = idx[t];
        const int fi = (int)(a % g->Hf); a /= g->Hf;
        const int fj = (int)(a % g->Wf); a /= g->Wf;
        const int k = (int)(a % g->Kf);
        const int d = (int)(a / g->Kf);
        out[t] = backward_filter_one(g, Ho, Wo, x, dzdy, fi, fj, k, d);
    }
    return ORCT_OK;
}

/* dzdb[c] = sum over i'', j'' and the batch of dzdy[:, :, c, :]. */
int orct_backward_bias(const orct_geom *g, const double *dzdy, double *dzdb) {
    int32_t Ho, Wo;
    int st = orct_output_size(g, &Ho, &Wo);
    if (st) return st;
    if (!dzdy || !dzdb) return ORCT_BAD_ARG;
    const int K = g->G * g->Kf;
    for (int c = 0; c < K; ++c) {
        double acc = 0.0;
        for (int n = 0; n < g->N; ++n)
            for (int jo = 0; jo < Wo; ++jo)
                for (int io = 0; io < Ho; ++io)
                    acc += dzdy[YA(io, jo, c, n)];
        dzdb[c] = acc;
    }
    return ORCT_OK;
}
