// Spatial pooling (max and average), forward and backward: streaming kernels, one result per
// thread, lanes along the first (fastest) array index.
//
// MatConvNet manual (arXiv 1412.4564) Sec. 4.3: y[io,jo,d,n] is the maximum / the average of x over
// the window rows Sh*io-Pt .. +H'-1, columns Sw*jo-Pl .. +W'-1 of plane (d,n), cropped to the
// array (max: as if padded with -infinity; average: divided by the number of samples inside).
// Sec. 6.3: y = S(x) x, dz/dx = S(x)^T dz/dy; for max pooling S selects one sample per window --
// the first maximum in memory order (rows fastest) -- and the backward pass is written as a
// gather: a sample adds the dzdy of every window that selects it, so no two threads write one
// element and the result does not depend on scheduling.  Which sample a window selects is found
// once per window by pool_argmax_kernel (one byte per window: the position inside the window);
// windows of more than 256 samples take the one-kernel form that rescans the windows.
//
// These kernels move 4-12 bytes per result, so index arithmetic is what they could lose time on:
// the divisions that split a thread's flat index into plane, column and row, and those by the
// strides, are multiplications by reciprocals prepared on the host (exact for every index below 2^31).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "fastdiv.h"

namespace mcn {

struct PoolGeom {
    int H, W, D, N;
    int Hp, Wp, Sh, Sw, Pt, Pl;
    int Ho, Wo;
    int method;      // 0 max, 1 average
    Div32 dH, dHo, dSh, dSw;  // exact for every index below 2^31 (fastdiv.h)
    FastDiv64 dIn, dOut;     // by the plane sizes H*W and Ho*Wo
};

// HP, WP > 0: window size known at compile time.  The window's samples are then read with clamped
// addresses and no branches, so that all loads are in flight together (a loop with run-time bounds
// issues them one after the other); samples outside the input are left out by selection, in the same
// order as the loop takes them.
template <int HP, int WP>
__global__ __launch_bounds__(256) void pool_forward_kernel(PoolGeom g, const float *__restrict__ x,
                                                           float *__restrict__ y, unsigned total) {
    const unsigned idx = blockIdx.x * 256u + threadIdx.x;
    if (idx >= total) return;
    const unsigned plane = div64(idx, g.dOut);
    const int e = (int)(idx - plane * (unsigned)(g.Ho * g.Wo));
    const int jo = div32(e, g.dHo), io = e - jo * g.Ho;
    const float *xp = x + (size_t)plane * g.H * g.W;
    if constexpr (HP > 0) {
        const int oi = g.Sh * io - g.Pt, oj = g.Sw * jo - g.Pl;
        float v[WP][HP];
        bool ok[WP][HP];
#pragma unroll
        for (int fj = 0; fj < WP; ++fj)
#pragma unroll
            for (int fi = 0; fi < HP; ++fi) {
                const int i = oi + fi, j = oj + fj;
                ok[fj][fi] = (unsigned)i < (unsigned)g.H && (unsigned)j < (unsigned)g.W;
                v[fj][fi] = xp[min(max(i, 0), g.H - 1) + g.H * min(max(j, 0), g.W - 1)];
            }
        float r = 0.f;
        int cnt = 0;
#pragma unroll
        for (int fj = 0; fj < WP; ++fj)
#pragma unroll
            for (int fi = 0; fi < HP; ++fi) {
                if (g.method == 0) r = !ok[fj][fi] ? r : cnt == 0 ? v[fj][fi] : fmaxf(r, v[fj][fi]);
                else r += ok[fj][fi] ? v[fj][fi] : 0.f;
                cnt += ok[fj][fi] ? 1 : 0;
            }
        y[idx] = g.method == 0 ? r : r / (float)cnt;
        return;
    }
    const int i0 = max(g.Sh * io - g.Pt, 0), i1 = min(g.Sh * io - g.Pt + g.Hp, g.H);
    const int j0 = max(g.Sw * jo - g.Pl, 0), j1 = min(g.Sw * jo - g.Pl + g.Wp, g.W);
    float r;
    if (g.method == 0) {
        r = xp[i0 + g.H * j0];
        for (int j = j0; j < j1; ++j)
            for (int i = i0; i < i1; ++i) r = fmaxf(r, xp[i + g.H * j]);
    } else {
        float s = 0.f;
        for (int j = j0; j < j1; ++j)
            for (int i = i0; i < i1; ++i) s += xp[i + g.H * j];
        r = s / (float)((i1 - i0) * (j1 - j0));
    }
    y[idx] = r;
}

// The windows that hold sample (i, j): Sh*io - Pt <= i <= Sh*io - Pt + Hp - 1, clipped to the output.
struct WindowRange {
    int io_lo, io_hi, jo_lo, jo_hi;
};
__device__ inline WindowRange windows_of(const PoolGeom &g, int i, int j) {
    WindowRange r;
    const int a = i + g.Pt - g.Hp + g.Sh, b = j + g.Pl - g.Wp + g.Sw;     // ceil((i + Pt - Hp + 1) / Sh) = floor(a / Sh)
    r.io_lo = a > 0 ? div32(a, g.dSh) : 0;
    r.io_hi = min(div32(i + g.Pt, g.dSh), g.Ho - 1);
    r.jo_lo = b > 0 ? div32(b, g.dSw) : 0;
    r.jo_hi = min(div32(j + g.Pl, g.dSw), g.Wo - 1);
    return r;
}

// code[io,jo,plane] = fi + Hp*fj of the first maximum of window (io, jo), (fi, fj) counted from the
// window's uncropped origin.  Needs Hp*Wp <= 256.
template <int HP, int WP>
__global__ __launch_bounds__(256) void pool_argmax_kernel(PoolGeom g, const float *__restrict__ x,
                                                          unsigned char *__restrict__ code, unsigned total) {
    const unsigned idx = blockIdx.x * 256u + threadIdx.x;
    if (idx >= total) return;
    const unsigned plane = div64(idx, g.dOut);
    const int e = (int)(idx - plane * (unsigned)(g.Ho * g.Wo));
    const int jo = div32(e, g.dHo), io = e - jo * g.Ho;
    const float *xp = x + (size_t)plane * g.H * g.W;
    const int oi = g.Sh * io - g.Pt, oj = g.Sw * jo - g.Pl;
    if constexpr (HP > 0) {
        float v[WP][HP];
#pragma unroll
        for (int fj = 0; fj < WP; ++fj)
#pragma unroll
            for (int fi = 0; fi < HP; ++fi)
                v[fj][fi] = xp[min(max(oi + fi, 0), g.H - 1) + g.H * min(max(oj + fj, 0), g.W - 1)];
        float m = 0.f;
        int best = -1;
#pragma unroll
        for (int fj = 0; fj < WP; ++fj)
#pragma unroll
            for (int fi = 0; fi < HP; ++fi) {
                const bool ok = (unsigned)(oi + fi) < (unsigned)g.H && (unsigned)(oj + fj) < (unsigned)g.W;
                const bool take = ok && (best < 0 || v[fj][fi] > m);
                m = take ? v[fj][fi] : m;
                best = take ? fi + HP * fj : best;
            }
        code[idx] = (unsigned char)best;
        return;
    }
    const int i0 = max(oi, 0), i1 = min(oi + g.Hp, g.H);
    const int j0 = max(oj, 0), j1 = min(oj + g.Wp, g.W);
    float m = xp[i0 + g.H * j0];
    int best = (i0 - oi) + g.Hp * (j0 - oj);
    for (int j = j0; j < j1; ++j)
        for (int i = i0; i < i1; ++i) {
            const float v = xp[i + g.H * j];
            if (v > m) { m = v; best = (i - oi) + g.Hp * (j - oj); }
        }
    code[idx] = (unsigned char)best;
}

// dzdx[i,j] = sum of dzdy over the windows whose code points at (i, j)
// NH, NW > 0: at most NH x NW windows hold one sample (ceil(Hp / Sh) x ceil(Wp / Sw)); their codes and
// derivatives are read with clamped addresses and no branches.
template <int NH, int NW>
__global__ __launch_bounds__(256) void pool_backward_max_coded_kernel(PoolGeom g, const unsigned char *__restrict__ code,
                                                                      const float *__restrict__ dzdy,
                                                                      float *__restrict__ dzdx, unsigned total) {
    const unsigned idx = blockIdx.x * 256u + threadIdx.x;
    if (idx >= total) return;
    const unsigned plane = div64(idx, g.dIn);
    const int e = (int)(idx - plane * (unsigned)(g.H * g.W));
    const int j = div32(e, g.dH), i = e - j * g.H;
    const size_t pbase = (size_t)plane * g.Ho * g.Wo;
    const WindowRange r = windows_of(g, i, j);
    float acc = 0.f;
    if constexpr (NH > 0) {
        unsigned char c[NW][NH];
        float p[NW][NH];
#pragma unroll
        for (int b = 0; b < NW; ++b)
#pragma unroll
            for (int a = 0; a < NH; ++a) {
                const size_t at = pbase + min(r.io_lo + a, g.Ho - 1) + (size_t)g.Ho * min(r.jo_lo + b, g.Wo - 1);
                c[b][a] = code[at];
                p[b][a] = dzdy[at];
            }
#pragma unroll
        for (int b = 0; b < NW; ++b)
#pragma unroll
            for (int a = 0; a < NH; ++a) {
                const int io = r.io_lo + a, jo = r.jo_lo + b;
                const int fi = i - (g.Sh * io - g.Pt), fj = j - (g.Sw * jo - g.Pl);
                if (io <= r.io_hi && jo <= r.jo_hi && c[b][a] == fi + g.Hp * fj) acc += p[b][a];
            }
        dzdx[idx] = acc;
        return;
    }
    for (int jo = r.jo_lo; jo <= r.jo_hi; ++jo) {
        const int fj = j - (g.Sw * jo - g.Pl);
        for (int io = r.io_lo; io <= r.io_hi; ++io) {
            const int fi = i - (g.Sh * io - g.Pt);
            const size_t a = pbase + io + (size_t)g.Ho * jo;
            if (code[a] == fi + g.Hp * fj) acc += dzdy[a];
        }
    }
    dzdx[idx] = acc;
}

// Max pooling whose windows do not overlap (stride = window size): every sample lies in at most one window,
// so one thread per window reads its samples, finds the first maximum and writes the window's share of dzdx
// (the derivative at the maximum, zero elsewhere) in one pass: x, dzdy and dzdx each move once and no code
// array is needed.  Rows and columns past the last window are cleared by the last windows of each column / row.
template <int HP, int WP>
__global__ __launch_bounds__(256) void pool_backward_max_disjoint_kernel(PoolGeom g, const float *__restrict__ x,
                                                                         const float *__restrict__ dzdy,
                                                                         float *__restrict__ dzdx, unsigned total) {
    const unsigned idx = blockIdx.x * 256u + threadIdx.x;
    if (idx >= total) return;
    const unsigned plane = div64(idx, g.dOut);
    const int e = (int)(idx - plane * (unsigned)(g.Ho * g.Wo));
    const int jo = div32(e, g.dHo), io = e - jo * g.Ho;
    const size_t base = (size_t)plane * g.H * g.W;
    const float *xp = x + base;
    float *dp = dzdx + base;
    const int oi = HP * io - g.Pt, oj = WP * jo - g.Pl;
    const float p = dzdy[idx];
    float v[WP][HP];
#pragma unroll
    for (int fj = 0; fj < WP; ++fj)
#pragma unroll
        for (int fi = 0; fi < HP; ++fi)
            v[fj][fi] = xp[min(max(oi + fi, 0), g.H - 1) + g.H * min(max(oj + fj, 0), g.W - 1)];
    float m = 0.f;
    int best = -1;
#pragma unroll
    for (int fj = 0; fj < WP; ++fj)
#pragma unroll
        for (int fi = 0; fi < HP; ++fi) {
            const bool ok = (unsigned)(oi + fi) < (unsigned)g.H && (unsigned)(oj + fj) < (unsigned)g.W;
            const bool take = ok && (best < 0 || v[fj][fi] > m);
            m = take ? v[fj][fi] : m;
            best = take ? fi + HP * fj : best;
        }
#pragma unroll
    for (int fj = 0; fj < WP; ++fj)
#pragma unroll
        for (int fi = 0; fi < HP; ++fi)
            if ((unsigned)(oi + fi) < (unsigned)g.H && (unsigned)(oj + fj) < (unsigned)g.W)
                dp[(oi + fi) + g.H * (oj + fj)] = best == fi + HP * fj ? p : 0.f;
    // samples no window reads
    const int i_end = io == g.Ho - 1 ? g.H : oi + HP;          // rows [oi + HP, i_end) below this window
    const int j_end = jo == g.Wo - 1 ? g.W : oj + WP;          // columns [oj + WP, j_end) right of it
    for (int j = max(oj, 0); j < min(oj + WP, g.W); ++j)
        for (int i = oi + HP; i < i_end; ++i) dp[i + g.H * j] = 0.f;
    for (int j = oj + WP; j < j_end; ++j)
        for (int i = max(oi, 0); i < i_end; ++i) dp[i + g.H * j] = 0.f;
}

// One-kernel backward pass: average pooling, and max pooling with windows too large for a byte code.
__global__ __launch_bounds__(256) void pool_backward_kernel(PoolGeom g, const float *__restrict__ x,
                                                            const float *__restrict__ dzdy,
                                                            float *__restrict__ dzdx, unsigned total) {
    const unsigned idx = blockIdx.x * 256u + threadIdx.x;
    if (idx >= total) return;
    const unsigned plane = div64(idx, g.dIn);
    const int e = (int)(idx - plane * (unsigned)(g.H * g.W));
    const int j = div32(e, g.dH), i = e - j * g.H;
    const float *pp = dzdy + (size_t)plane * g.Ho * g.Wo;
    const WindowRange r = windows_of(g, i, j);
    float acc = 0.f;
    if (g.method == 0) {
        const float *xp = x + (size_t)plane * g.H * g.W;
        const float mine = xp[e];
        for (int jo = r.jo_lo; jo <= r.jo_hi; ++jo)
            for (int io = r.io_lo; io <= r.io_hi; ++io) {
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
        for (int jo = r.jo_lo; jo <= r.jo_hi; ++jo) {
            const int j0 = max(g.Sw * jo - g.Pl, 0), j1 = min(g.Sw * jo - g.Pl + g.Wp, g.W);
            for (int io = r.io_lo; io <= r.io_hi; ++io) {
                const int i0 = max(g.Sh * io - g.Pt, 0), i1 = min(g.Sh * io - g.Pt + g.Hp, g.H);
                acc += pp[io + g.Ho * jo] / (float)((i1 - i0) * (j1 - j0));
            }
        }
    }
    dzdx[idx] = acc;
}

}  // namespace mcn
