/*
 * CPU oracle for the convolution block (forward, and the three derivatives).
 *
 * THIS IS TEST INFRASTRUCTURE.  It exists so that the GPU library can be
 * checked against something that a reader can compare with the paper by eye.
 * Only tests, the smoke check and the benchmark's CPU-baseline leg may call
 * it; the product path never does.  It shares no code with the GPU path.
 *
 * What it follows (MatConvNet manual, arXiv 1412.4564):
 *   - Sec. 4.1 "Convolution", paragraph "Padding and stride": the summation
 *     that defines y from x, the filter bank f and the biases b;
 *   - Sec. 4.1 "Output size" and Sec. 5.2 eq. (filtered-height): H'' and W'';
 *   - Sec. 4.1 "Filter groups": which input channels a filter reads;
 *   - Sec. 2.3.2 eq. (projected): the backward mode returns d<p,y>/dx and
 *     d<p,y>/dw for p = dzdy; because y is bilinear in (x, f) and affine in b
 *     these are the exact adjoints of the forward sum (Sec. 6.1, boxed
 *     formulas, are the same thing in matrix form).
 *
 * Readings taken where the manual is silent or garbled:
 *   - the displayed sums drop the filter index on f and put a stray d'' on x;
 *     read as  f[i',j',d',d''] * x[...,d'];
 *   - no filter flip: indices of f and x increase together (correlation);
 *   - arrays are stored first index fastest (the vec() order of Sec. 2.3.1),
 *     so x[i,j,d,n] sits at i + H*(j + W*(d + D*n)), 0-based;
 *   - with g = D/D' groups the filters are split into g consecutive blocks of
 *     D''/g; block m reads input channels m*D' .. (m+1)*D'-1;
 *   - dzdb[k] = sum of dzdy over i'', j'' and the batch (y is affine in b with
 *     coefficient one); dzdw and dzdb are summed over the batch;
 *   - stride = (S_h, S_w), pad = (top, bottom, left, right); bottom and right
 *     pads only enter through the output size;
 *   - any pad >= 0 is accepted; a window lying wholly in padding gives b[k].
 *
 * Arithmetic: everything is double.  Callers convert their fp32 test data to
 * double exactly, so the result is the exact sum up to fp64 rounding.
 * No blocking, no im2row buffer, no BLAS: the loops are the formula.
 *
 * All indices below are 0-based: the manual's  S_h(i''-1) + i' - P_h^-
 * (1-based i'', i') becomes  S_h*io + fi - Pt.
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t H, W, D, N;        /* x : H x W x D x N                     */
    int32_t Hf, Wf, Df, K;     /* f : H' x W' x D' x D''  (K = D'')     */
    int32_t Sh, Sw;            /* strides, vertical then horizontal     */
    int32_t Pt, Pb, Pl, Pr;    /* pads: top, bottom, left, right        */
} orc_geom;

enum { ORC_OK = 0, ORC_BAD_ARG = 1, ORC_BAD_GROUPS = 2, ORC_FILTER_TOO_LARGE = 3 };

/* floor(a / b) for b > 0 and any sign of a */
static int64_t floordiv(int64_t a, int64_t b) {
    int64_t q = a / b;
    if ((a % b != 0) && ((a < 0) != (b < 0))) --q;
    return q;
}

/* Sec. 4.1 "Output size":  H'' = 1 + floor((H - H' + Pt + Pb) / Sh).
 * The padded input must be at least as large as the filter, else an error. */
int orc_output_size(const orc_geom *g, int32_t *Ho, int32_t *Wo) {
    if (!g) return ORC_BAD_ARG;
    if (g->H < 1 || g->W < 1 || g->D < 1 || g->N < 1) return ORC_BAD_ARG;
    if (g->Hf < 1 || g->Wf < 1 || g->Df < 1 || g->K < 1) return ORC_BAD_ARG;
    if (g->Sh < 1 || g->Sw < 1) return ORC_BAD_ARG;
    if (g->Pt < 0 || g->Pb < 0 || g->Pl < 0 || g->Pr < 0) return ORC_BAD_ARG;
    if (g->D % g->Df != 0) return ORC_BAD_GROUPS;
    if (g->K % (g->D / g->Df) != 0) return ORC_BAD_GROUPS;
    if (g->H + g->Pt + g->Pb < g->Hf) return ORC_FILTER_TOO_LARGE;
    if (g->W + g->Pl + g->Pr < g->Wf) return ORC_FILTER_TOO_LARGE;
    if (Ho) *Ho = 1 + (int32_t)floordiv((int64_t)g->H - g->Hf + g->Pt + g->Pb, g->Sh);
    if (Wo) *Wo = 1 + (int32_t)floordiv((int64_t)g->W - g->Wf + g->Pl + g->Pr, g->Sw);
    return ORC_OK;
}

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* addresses, first index fastest */
#define XADDR(i, j, d, n)   ((int64_t)(i) + (int64_t)g->H  * ((j) + (int64_t)g->W  * ((d) + (int64_t)g->D  * (n))))
#define FADDR(fi, fj, fd, k) ((int64_t)(fi) + (int64_t)g->Hf * ((fj) + (int64_t)g->Wf * ((fd) + (int64_t)g->Df * (k))))
#define YADDR(io, jo, k, n) ((int64_t)(io) + (int64_t)Ho * ((jo) + (int64_t)Wo * ((k) + (int64_t)g->K * (n))))

/* One output sample of the forward sum (Sec. 4.1, "Padding and stride"). */
static double forward_one(const orc_geom *g, const double *x, const double *f,
                          const double *b, int io, int jo, int k, int n) {
    const int Kg = g->K / (g->D / g->Df);   /* filters per group            */
    const int grp = k / Kg;                 /* group this filter belongs to */
    double acc = b ? b[k] : 0.0;
    for (int fd = 0; fd < g->Df; ++fd)
        for (int fj = 0; fj < g->Wf; ++fj)
            for (int fi = 0; fi < g->Hf; ++fi) {
                int i = g->Sh * io + fi - g->Pt;
                int j = g->Sw * jo + fj - g->Pl;
                if (i < 0 || i >= g->H || j < 0 || j >= g->W) continue; /* zero extension */
                acc += f[FADDR(fi, fj, fd, k)] * x[XADDR(i, j, grp * g->Df + fd, n)];
            }
    return acc;
}

/* y = x * f + b.  b may be NULL (no bias). */
int orc_forward(const orc_geom *g, const double *x, const double *f,
                const double *b, double *y) {
    int32_t Ho, Wo;
    int st = orc_output_size(g, &Ho, &Wo);
    if (st) return st;
    if (!x || !f || !y) return ORC_BAD_ARG;
    const int64_t nk = (int64_t)g->N * g->K;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t t = 0; t < nk; ++t) {
        int n = (int)(t / g->K), k = (int)(t % g->K);
        for (int jo = 0; jo < Wo; ++jo)
            for (int io = 0; io < Ho; ++io)
                y[YADDR(io, jo, k, n)] = forward_one(g, x, f, b, io, jo, k, n);
    }
    return ORC_OK;
}

/* Forward at chosen places only: idx[] holds linear addresses into y. */
int orc_forward_at(const orc_geom *g, const double *x, const double *f,
                   const double *b, const int64_t *idx, int64_t count, double *out) {
    int32_t Ho, Wo;
    int st = orc_output_size(g, &Ho, &Wo);
    if (st) return st;
    if (!x || !f || !idx || !out) return ORC_BAD_ARG;
    const int64_t total = (int64_t)Ho * Wo * g->K * g->N;
    for (int64_t t = 0; t < count; ++t)
        if (idx[t] < 0 || idx[t] >= total) return ORC_BAD_ARG;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t t = 0; t < count; ++t) {
        int64_t a = idx[t];
        int io = (int)(a % Ho); a /= Ho;
        int jo = (int)(a % Wo); a /= Wo;
        int k  = (int)(a % g->K);
        int n  = (int)(a / g->K);
        out[t] = forward_one(g, x, f, b, io, jo, k, n);
    }
    return ORC_OK;
}

/* dzdx = d<dzdy, y>/dx.  The same terms as the forward sum: each product
 * f * x inside y[io,jo,k,n] contributes f * dzdy[io,jo,k,n] to the derivative
 * of that x (scatter form).  Samples of x that no window reaches stay exactly
 * zero.  The loops are ordered so that one thread owns one (channel, image)
 * plane of dzdx, so no two threads write one element. */
int orc_backward_data(const orc_geom *g, const double *f, const double *dzdy,
                      double *dzdx) {
    int32_t Ho, Wo;
    int st = orc_output_size(g, &Ho, &Wo);
    if (st) return st;
    if (!f || !dzdy || !dzdx) return ORC_BAD_ARG;
    const int Kg = g->K / (g->D / g->Df);
    memset(dzdx, 0, sizeof(double) * (size_t)g->H * g->W * g->D * g->N);
    const int64_t planes = (int64_t)g->N * g->D;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t t = 0; t < planes; ++t) {
        const int n = (int)(t / g->D), d = (int)(t % g->D);
        const int grp = d / g->Df, fd = d % g->Df;   /* d = grp * Df + fd */
        for (int k = grp * Kg; k < (grp + 1) * Kg; ++k)   /* the filters that read channel d */
            for (int jo = 0; jo < Wo; ++jo)
                for (int io = 0; io < Ho; ++io) {
                    const double p = dzdy[YADDR(io, jo, k, n)];
                    for (int fj = 0; fj < g->Wf; ++fj)
                        for (int fi = 0; fi < g->Hf; ++fi) {
                            int i = g->Sh * io + fi - g->Pt;
                            int j = g->Sw * jo + fj - g->Pl;
                            if (i < 0 || i >= g->H || j < 0 || j >= g->W) continue;
                            dzdx[XADDR(i, j, d, n)] += f[FADDR(fi, fj, fd, k)] * p;
                        }
                }
    }
    return ORC_OK;
}

/* One sample of dzdx written as a gather: all (io, fi) with
 * Sh*io + fi - Pt = i, all (jo, fj) with Sw*jo + fj - Pl = j, and all filters
 * of the group that reads channel d.  (The 1-D form of this is the
 * convolution-transpose sum of Sec. 6.2.) */
static double backward_data_one(const orc_geom *g, int Ho, int Wo, const double *f,
                                const double *dzdy, int i, int j, int d, int n) {
    const int Kg = g->K / (g->D / g->Df);
    const int grp = d / g->Df, fd = d % g->Df;
    double acc = 0.0;
    for (int k = grp * Kg; k < (grp + 1) * Kg; ++k)
        for (int fj = 0; fj < g->Wf; ++fj) {
            int tj = j + g->Pl - fj;
            if (tj < 0 || tj % g->Sw != 0) continue;
            int jo = tj / g->Sw;
            if (jo >= Wo) continue;
            for (int fi = 0; fi < g->Hf; ++fi) {
                int ti = i + g->Pt - fi;
                if (ti < 0 || ti % g->Sh != 0) continue;
                int io = ti / g->Sh;
                if (io >= Ho) continue;
                acc += f[FADDR(fi, fj, fd, k)] * dzdy[YADDR(io, jo, k, n)];
            }
        }
    return acc;
}

int orc_backward_data_at(const orc_geom *g, const double *f, const double *dzdy,
                         const int64_t *idx, int64_t count, double *out) {
    int32_t Ho, Wo;
    int st = orc_output_size(g, &Ho, &Wo);
    if (st) return st;
    if (!f || !dzdy || !idx || !out) return ORC_BAD_ARG;
    const int64_t total = (int64_t)g->H * g->W * g->D * g->N;
    for (int64_t t = 0; t < count; ++t)
        if (idx[t] < 0 || idx[t] >= total) return ORC_BAD_ARG;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t t = 0; t < count; ++t) {
        int64_t a = idx[t];
        int i = (int)(a % g->H); a /= g->H;
        int j = (int)(a % g->W); a /= g->W;
        int d = (int)(a % g->D);
        int n = (int)(a / g->D);
        out[t] = backward_data_one(g, Ho, Wo, f, dzdy, i, j, d, n);
    }
    return ORC_OK;
}

/* One sample of dzdw = d<dzdy, y>/df: every product f * x in the forward sum
 * that carries this filter coefficient contributes x * dzdy; summed over the
 * output positions and over the batch. */
static double backward_filter_one(const orc_geom *g, int Ho, int Wo, const double *x,
                                  const double *dzdy, int fi, int fj, int fd, int k) {
    const int Kg = g->K / (g->D / g->Df);
    const int grp = k / Kg;
    double acc = 0.0;
    for (int n = 0; n < g->N; ++n)
        for (int jo = 0; jo < Wo; ++jo)
            for (int io = 0; io < Ho; ++io) {
                int i = g->Sh * io + fi - g->Pt;
                int j = g->Sw * jo + fj - g->Pl;
                if (i < 0 || i >= g->H || j < 0 || j >= g->W) continue;
                acc += x[XADDR(i, j, grp * g->Df + fd, n)] * dzdy[YADDR(io, jo, k, n)];
            }
    return acc;
}

int orc_backward_filter(const orc_geom *g, const double *x, const double *dzdy,
                        double *dzdw) {
    int32_t Ho, Wo;
    int st = orc_output_size(g, &Ho, &Wo);
    if (st) return st;
    if (!x || !dzdy || !dzdw) return ORC_BAD_ARG;
    const int64_t total = (int64_t)g->Hf * g->Wf * g->Df * g->K;
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t a0 = 0; a0 < total; ++a0) {
        int64_t a = a0;
        int fi = (int)(a % g->Hf); a /= g->Hf;
        int fj = (int)(a % g->Wf); a /= g->Wf;
        int fd = (int)(a % g->Df);
        int k  = (int)(a / g->Df);
        dzdw[a0] = backward_filter_one(g, Ho, Wo, x, dzdy, fi, fj, fd, k);
    }
    return ORC_OK;
}

int orc_backward_filter_at(const orc_geom *g, const double *x, const double *dzdy,
                           const int64_t *idx, int64_t count, double *out) {
    int32_t Ho, Wo;
    int st = orc_output_size(g, &Ho, &Wo);
    if (st) return st;
    if (!x || !dzdy || !idx || !out) return ORC_BAD_ARG;
    const int64_t total = (int64_t)g->Hf * g->Wf * g->Df * g->K;
    for (int64_t t = 0; t < count; ++t)
        if (idx[t] < 0 || idx[t] >= total) return ORC_BAD_ARG;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t t = 0; t < count; ++t) {
        int64_t a = idx[t];
        int fi = (int)(a % g->Hf); a /= g->Hf;
        int fj = (int)(a % g->Wf); a /= g->Wf;
        int fd = (int)(a % g->Df);
        int k  = (int)(a / g->Df);
        out[t] = backward_filter_one(g, Ho, Wo, x, dzdy, fi, fj, fd, k);
    }
    return ORC_OK;
}

/* dzdb[k] = sum over i'', j'' and the batch of dzdy[., ., k, .]. */
int orc_backward_bias(const orc_geom *g, const double *dzdy, double *dzdb) {
    int32_t Ho, Wo;
    int st = orc_output_size(g, &Ho, &Wo);
    if (st) return st;
    if (!dzdy || !dzdb) return ORC_BAD_ARG;
#pragma omp parallel for schedule(static)
    for (int k = 0; k < g->K; ++k) {
        double acc = 0.0;
        for (int n = 0; n < g->N; ++n)
            for (int jo = 0; jo < Wo; ++jo)
                for (int io = 0; io < Ho; ++io)
                    acc += dzdy[YADDR(io, jo, k, n)];
        dzdb[k] = acc;
    }
    return ORC_OK;
}
