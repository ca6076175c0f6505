// Spatial pooling (max and average), forward and backward: streaming kernels, one result per
// thread, lanes along the first (fastest) array index.
//
// MatConvNet manual (arXiv 1412.4564) Sec. 4.3: y[io,jo,d,n] is the maximum / the average of x over
// the window rows Sh*io-Pt .. +H'-1, columns Sw*jo-Pl .. +W'-1 of plane (d,n), cropped to the
// array (max: as if padded with -infinity; average: divided by the number of samples inside).
// Sec. 6.3: y = S(x) x, dz/dx = S(x)^T dz/dy; for max pooling S selects one sample per window --
// the first maximum in memory order (rows fastest) -- and the backward pass is written as a
// gather: a sample adds the dzdy of every window that selects it, so no two threads write one
// element and the result does not depend on scheduling.
#pragma once
#include <hip/hip_runtime.h>

namespace mcn {

struct PoolGeom {
    int H, W, D, N;
    int Hp, Wp, Sh, Sw, Pt, Pl;
    int Ho, Wo;
    int method;      // 0 max, 1 average
};

__global__ __launch_bounds__(256) void pool_forward_kernel(PoolGeom g, const float *__restrict__ x,
                                                           float *__restrict__ y, int total) {
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int io = idx % g.Ho;
    int t = idx / g.Ho;
    const int jo = t % g.Wo;
    const int plane = t / g.Wo;
    const float *xp = x + (size_t)plane * g.H * g.W;
    const int i0 = max(g.Sh * io - g.Pt, 0), i1 = min(g.Sh * io - g.Pt + g.Hp, g.H);
    const int j0 = max(g.Sw * jo - g.Pl, 0), j1 = min(g.Sw * jo - g.Pl + g.Wp, g.W);
    if (g.method == 0) {
        float m = xp[i0 + g.H * j0];
        for (int j = j0; j < j1; ++j)
            for (int i = i0; i < i1; ++i) m = fmaxf(m, xp[i + g.H * j]);
        y[idx] = m;
    } else {
        float s = 0.f;
        for (int j = j0; j < j1; ++j)
            for (int i = i0; i < i1; ++i) s += xp[i + g.H * j];
        y[idx] = s / (float)((i1 - i0) * (j1 - j0));
    }
}

__global__ __launch_bounds__(256) void pool_backward_kernel(PoolGeom g, const float *__restrict__ x,
                                                            const float *__restrict__ dzdy,
                                                            float *__restrict__ dzdx, int total) {
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int i = idx % g.H;
    int t = idx / g.H;
    const int j = t % g.W;
    const int plane = t / g.W;
    const float *pp = dzdy + (size_t)plane * g.Ho * g.Wo;
    // windows that hold (i, j): Sh*io - Pt <= i <= Sh*io - Pt + Hp - 1
    const int io_lo = max((i + g.Pt - g.Hp + g.Sh) / g.Sh, 0);       // ceil((i + Pt - Hp + 1) / Sh) where that is >= 0
    const int io_hi = min((i + g.Pt) / g.Sh, g.Ho - 1);
    const int jo_lo = max((j + g.Pl - g.Wp + g.Sw) / g.Sw, 0);
    const int jo_hi = min((j + g.Pl) / g.Sw, g.Wo - 1);
    float acc = 0.f;
    if (g.method == 0) {
        const float *xp = x + (size_t)plane * g.H * g.W;
        const float mine = xp[i + g.H * j];
        for (int jo = jo_lo; jo <= jo_hi; ++jo)
            for (int io = io_lo; io <= io_hi; ++io) {
                const int i0 = max(g.Sh * io - g.Pt, 0), i1 = min(g.Sh * io - g.Pt + g.Hp, g.H);
                const int j0 = max(g.Sw * jo - g.Pl, 0), j1 = min(g.Sw * jo - g.Pl + g.Wp, g.W);
                // selected iff no sample of the window is larger and none before (i, j) is equal
                bool sel = true;
                for (int jj = j0; jj < j1; ++jj)
                    for (int ii = i0; ii < i1; ++ii) {
                        const float v = xp[ii + g.H * jj];
                        const bool before = jj < j || (jj == j && ii < i);
                        if (v > mine || (before && v == mine)) sel = false;
                    }
                if (sel) acc += pp[io + g.Ho * jo];
            }
    } else {
        for (int jo = jo_lo; jo <= jo_hi; ++jo) {
            const int j0 = max(g.Sw * jo - g.Pl, 0), j1 = min(g.Sw * jo - g.Pl + g.Wp, g.W);
            for (int io = io_lo; io <= io_hi; ++io) {
                const int i0 = max(g.Sh * io - g.Pt, 0), i1 = min(g.Sh * io - g.Pt + g.Hp, g.H);
                acc += pp[io + g.Ho * jo] / (float)((i1 - i0) * (j1 - j0));
            }
        }
    }
    dzdx[idx] = acc;
}

}  // namespace mcn
