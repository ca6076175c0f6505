/*
 * CPU oracle for the spatial pooling block (max and average; forward and backward).
 *
 * THIS IS TEST INFRASTRUCTURE: only tests, the smoke check and the benchmark's
 * CPU-baseline leg may call it; the product path never does, and it shares no
 * code with the GPU path.
 *
 * What it follows (MatConvNet manual, arXiv 1412.4564):
 *   - Sec. 4.3 "Spatial pooling": y[i'',j'',d] is the maximum, or the average, of
 *     x over an H' x W' window of channel d;
 *   - Sec. 4.3 "Padding and stride": windows are placed like the filters of the
 *     convolution block (stride, four pads), but a window that straddles the
 *     boundary is CROPPED: max pooling behaves as if x were extended with
 *     -infinity, average pooling divides by the number of samples actually
 *     inside the array (not by H'W');
 *   - Sec. 5.2: output size floor((H - H' + P^- + P^+)/S) + 1, and the
 *     restriction P <= H' - 1 (Sec. 5.2.1), which guarantees that every window
 *     holds at least one sample;
 *   - Sec. 6.3: y = S(x) x with a selector matrix S (one 1 per row for max,
 *     the normalisation factors for average) and dz/dx = S(x)^T dz/dy.
 *
 * Readings taken where the manual is silent:
 *   - when a window holds its maximum more than once (a null set, Sec. 6.3), S
 *     selects the first one in memory order (rows fastest, then columns);
 *   - arrays are stored first index fastest (Sec. 2.3.1);
 *   - pads larger than H' - 1 / W' - 1 are an error.
 *
 * Arithmetic: double.  The loops are the definition: the backward pass builds
 * S(x)^T dz/dy by visiting every window and adding its share to the samples
 * it selects (one thread owns one (channel, image) plane, so no two threads
 * write one element).
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t H, W, D, N;        /* x : H x W x D x N                 */
    int32_t Hp, Wp;            /* window H' x W'                    */
    int32_t Sh, Sw;            /* strides                           */
    int32_t Pt, Pb, Pl, Pr;    /* pads: top, bottom, left, right    */
    int32_t method;            /* 0 = max, 1 = average              */
} orp_geom;

enum { ORP_OK = 0, ORP_BAD_ARG = 1, ORP_PAD_TOO_LARGE = 2, ORP_WINDOW_TOO_LARGE = 3 };

int orp_output_size(const orp_geom *g, int32_t *Ho, int32_t *Wo) {
    if (!g) return ORP_BAD_ARG;
    if (g->H < 1 || g->W < 1 || g->D < 1 || g->N < 1) return ORP_BAD_ARG;
    if (g->Hp < 1 || g->Wp < 1 || g->Sh < 1 || g->Sw < 1) return ORP_BAD_ARG;
    if (g->Pt < 0 || g->Pb < 0 || g->Pl < 0 || g->Pr < 0) return ORP_BAD_ARG;
    if (g->method != 0 && g->method != 1) return ORP_BAD_ARG;
    if (g->Pt > g->Hp - 1 || g->Pb > g->Hp - 1 || g->Pl > g->Wp - 1 || g->Pr > g->Wp - 1) return ORP_PAD_TOO_LARGE;
    if (g->H + g->Pt + g->Pb < g->Hp || g->W + g->Pl + g->Pr < g->Wp) return ORP_WINDOW_TOO_LARGE;
    if (Ho) *Ho = (g->H - g->Hp + g->Pt + g->Pb) / g->Sh + 1;     /* numerator >= 0 */
    if (Wo) *Wo = (g->W - g->Wp + g->Pl + g->Pr) / g->Sw + 1;
    return ORP_OK;
}

#define XA(i, j) ((int64_t)(i) + (int64_t)g->H * (j))
#define YA(io, jo) ((int64_t)(io) + (int64_t)Ho * (jo))

/* the part of window (io, jo) that lies inside the array: rows [i0, i1), columns [j0, j1) */
static void window(const orp_geom *g, int io, int jo, int *i0, int *i1, int *j0, int *j1) {
    *i0 = g->Sh * io - g->Pt;
    *i1 = *i0 + g->Hp;
    *j0 = g->Sw * jo - g->Pl;
    *j1 = *j0 + g->Wp;
    if (*i0 < 0) *i0 = 0;
    if (*j0 < 0) *j0 = 0;
    if (*i1 > g->H) *i1 = g->H;
    if (*j1 > g->W) *j1 = g->W;
}

int orp_forward(const orp_geom *g, const double *x, double *y) {
    int32_t Ho, Wo;
    int st = orp_output_size(g, &Ho, &Wo);
    if (st) return st;
    if (!x || !y) return ORP_BAD_ARG;
    const int64_t planes = (int64_t)g->D * g->N;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < planes; ++t) {
        const double *xp = x + t * g->H * g->W;
        double *yp = y + t * Ho * Wo;
        for (int jo = 0; jo < Wo; ++jo)
            for (int io = 0; io < Ho; ++io) {
                int i0, i1, j0, j1;
                window(g, io, jo, &i0, &i1, &j0, &j1);
                if (g->method == 0) {
                    double m = xp[XA(i0, j0)];
                    for (int j = j0; j < j1; ++j)
                        for (int i = i0; i < i1; ++i)
                            if (xp[XA(i, j)] > m) m = xp[XA(i, j)];
                    yp[YA(io, jo)] = m;
                } else {
                    double s = 0.0;
                    for (int j = j0; j < j1; ++j)
                        for (int i = i0; i < i1; ++i) s += xp[XA(i, j)];
                    yp[YA(io, jo)] = s / (double)((i1 - i0) * (j1 - j0));
                }
            }
    }
    return ORP_OK;
}

/* dzdx = S(x)^T dzdy.  x is needed for max pooling only (may be NULL for average). */
int orp_backward(const orp_geom *g, const double *x, const double *dzdy, double *dzdx) {
    int32_t Ho, Wo;
    int st = orp_output_size(g, &Ho, &Wo);
    if (st) return st;
    if (!dzdy || !dzdx || (g->method == 0 && !x)) return ORP_BAD_ARG;
    const int64_t planes = (int64_t)g->D * g->N;
    memset(dzdx, 0, sizeof(double) * (size_t)planes * g->H * g->W);
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < planes; ++t) {
        const double *xp = x ? x + t * g->H * g->W : NULL;
        const double *pp = dzdy + t * Ho * Wo;
        double *dp = dzdx + t * g->H * g->W;
        for (int jo = 0; jo < Wo; ++jo)
            for (int io = 0; io < Ho; ++io) {
                int i0, i1, j0, j1;
                window(g, io, jo, &i0, &i1, &j0, &j1);
                if (g->method == 0) {
                    int bi = i0, bj = j0;             /* first maximum in memory order */
                    for (int j = j0; j < j1; ++j)
                        for (int i = i0; i < i1; ++i)
                            if (xp[XA(i, j)] > xp[XA(bi, bj)]) { bi = i; bj = j; }
                    dp[XA(bi, bj)] += pp[YA(io, jo)];
                } else {
                    const double share = pp[YA(io, jo)] / (double)((i1 - i0) * (j1 - j0));
                    for (int j = j0; j < j1; ++j)
                        for (int i = i0; i < i1; ++i) dp[XA(i, j)] += share;
                }
            }
    }
    return ORP_OK;
}
