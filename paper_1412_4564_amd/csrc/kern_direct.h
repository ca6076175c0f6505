// Direct (one result per thread / per wave) kernels: the general fallback that
// accepts every geometry.  They evaluate the sums of Sec. 4.1 of the MatConvNet
// manual (arXiv 1412.4564) and their adjoints (Sec. 2.3.2, Sec. 6.1) term by
// term in fp32.  Lanes run along the first (fastest) array index so that global
// accesses are coalesced.
#pragma once
#include <hip/hip_runtime.h>
#include "geom.h"

namespace mcn {

// y[io,jo,k,n] = b[k] + sum w[fi,fj,fd,k] * x[Sh*io+fi-Pt, Sw*jo+fj-Pl, grp*Df+fd, n]
__global__ __launch_bounds__(256) void direct_forward_kernel(Geom g, const float *__restrict__ x,
                                                             const float *__restrict__ w,
                                                             const float *__restrict__ b,
                                                             float *__restrict__ y, int total, int relu) {
    int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    int io = idx % g.Ho;
    int t = idx / g.Ho;
    int jo = t % g.Wo;
    t /= g.Wo;
    int k = t % g.K;
    int n = t / g.K;
    const int grp = k / g.Kg;
    const float *wk = w + (size_t)k * g.Hf * g.Wf * g.Df;
    const float *xn = x + ((size_t)n * g.D + (size_t)grp * g.Df) * g.H * g.W;
    const int i0 = g.Sh * io - g.Pt, j0 = g.Sw * jo - g.Pl;
    float acc = b ? b[k] : 0.f;
    for (int fd = 0; fd < g.Df; ++fd) {
        for (int fj = 0; fj < g.Wf; ++fj) {
            int j = j0 + fj;
            if (j < 0 || j >= g.W) continue;
            for (int fi = 0; fi < g.Hf; ++fi) {
                int i = i0 + fi;
                if (i < 0 || i >= g.H) continue;
                acc = fmaf(wk[fi + g.Hf * (fj + g.Wf * fd)], xn[i + g.H * (j + (size_t)g.W * fd)], acc);
            }
        }
    }
    y[idx] = relu ? fmaxf(acc, 0.f) : acc;
}

// dzdx[i,j,d,n] = sum over k in group(d), and all (io,fi), (jo,fj) with
// Sh*io+fi-Pt = i, Sw*jo+fj-Pl = j, of w[fi,fj,fd,k] * dzdy[io,jo,k,n].
__global__ __launch_bounds__(256) void direct_backward_data_kernel(Geom g, const float *__restrict__ w,
                                                                   const float *__restrict__ dzdy,
                                                                   float *__restrict__ dzdx, int total) {
    int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    int i = idx % g.H;
    int t = idx / g.H;
    int j = t % g.W;
    t /= g.W;
    int d = t % g.D;
    int n = t / g.D;
    const int grp = d / g.Df, fd = d % g.Df;
    const size_t ysz = (size_t)g.Ho * g.Wo;
    float acc = 0.f;
    for (int kk = 0; kk < g.Kg; ++kk) {
        const int k = grp * g.Kg + kk;
        const float *wk = w + ((size_t)k * g.Df + fd) * g.Hf * g.Wf;
        const float *pk = dzdy + ((size_t)n * g.K + k) * ysz;
        for (int fj = 0; fj < g.Wf; ++fj) {
            int tj = j + g.Pl - fj;
            if (tj < 0) break;            // tj only decreases with fj
            int jo = tj / g.Sw;
            if (tj - jo * g.Sw != 0 || jo >= g.Wo) continue;
            for (int fi = 0; fi < g.Hf; ++fi) {
                int ti = i + g.Pt - fi;
                if (ti < 0) break;
                int io = ti / g.Sh;
                if (ti - io * g.Sh != 0 || io >= g.Ho) continue;
                acc = fmaf(wk[fi + g.Hf * fj], pk[io + (size_t)g.Ho * jo], acc);
            }
        }
    }
    dzdx[idx] = acc;
}

// out[0..total) = 0  (samples of dzdx that no filter tap reaches when a stride exceeds the filter)
__global__ __launch_bounds__(256) void zero_fill_kernel(float *__restrict__ out, int total) {
    const long long lo = (long long)blockIdx.x * 1024, hi = lo + 1024 < total ? lo + 1024 : total;
    for (long long e = lo + threadIdx.x; e < hi; e += 256) out[e] = 0.f;
}

// out[p + plane*(c + C*n)] = bias[c]  (start value of an output whose contributions are written,
// or left out, per stride phase: the convolution transpose with a bias)
__global__ __launch_bounds__(256) void bias_fill_kernel(float *__restrict__ out, const float *__restrict__ bias,
                                                        int plane, int C, int total) {
    const long long lo = (long long)blockIdx.x * 1024, hi = lo + 1024 < total ? lo + 1024 : total;
    for (long long e = lo + threadIdx.x; e < hi; e += 256) out[e] = bias[(e / plane) % C];
}

// out[p + plane*(c + C*n)] += bias[c]
__global__ __launch_bounds__(256) void bias_add_kernel(float *__restrict__ out, const float *__restrict__ bias,
                                                       int plane, int C, int total) {
    const long long lo = (long long)blockIdx.x * 1024, hi = lo + 1024 < total ? lo + 1024 : total;
    for (long long e = lo + threadIdx.x; e < hi; e += 256) out[e] += bias[(e / plane) % C];
}

__device__ inline float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    return v;
}

// One wavefront per filter coefficient:
// dzdw[fi,fj,fd,k] = sum_{n,jo,io} x[Sh*io+fi-Pt, Sw*jo+fj-Pl, grp*Df+fd, n] * dzdy[io,jo,k,n]
__global__ __launch_bounds__(256) void direct_backward_filter_kernel(Geom g, const float *__restrict__ x,
                                                                     const float *__restrict__ dzdy,
                                                                     float *__restrict__ dzdw, int total) {
    const int lane = threadIdx.x & 63;
    int e = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (e >= total) return;                 // whole wave leaves together
    int fi = e % g.Hf;
    int t = e / g.Hf;
    int fj = t % g.Wf;
    t /= g.Wf;
    int fd = t % g.Df;
    int k = t / g.Df;
    const int grp = k / g.Kg;
    // valid io range: 0 <= Sh*io + fi - Pt < H
    int lo_i = g.Pt - fi;  lo_i = lo_i > 0 ? (lo_i + g.Sh - 1) / g.Sh : 0;
    int hi_i = g.H - 1 + g.Pt - fi;  hi_i = hi_i < 0 ? -1 : hi_i / g.Sh;  if (hi_i > g.Ho - 1) hi_i = g.Ho - 1;
    int lo_j = g.Pl - fj;  lo_j = lo_j > 0 ? (lo_j + g.Sw - 1) / g.Sw : 0;
    int hi_j = g.W - 1 + g.Pl - fj;  hi_j = hi_j < 0 ? -1 : hi_j / g.Sw;  if (hi_j > g.Wo - 1) hi_j = g.Wo - 1;
    float acc = 0.f;
    for (int n = 0; n < g.N; ++n) {
        const float *xc = x + ((size_t)n * g.D + (size_t)grp * g.Df + fd) * g.H * g.W;
        const float *pc = dzdy + ((size_t)n * g.K + k) * g.Ho * g.Wo;
        for (int jo = lo_j; jo <= hi_j; ++jo) {
            const float *xr = xc + (size_t)g.H * (g.Sw * jo + fj - g.Pl) + (fi - g.Pt);
            const float *pr = pc + (size_t)g.Ho * jo;
            for (int io = lo_i + lane; io <= hi_i; io += 64) acc = fmaf(xr[g.Sh * io], pr[io], acc);
        }
    }
    acc = wave_sum(acc);
    if (lane == 0) dzdw[e] = acc;
}

// ---- bias derivative: dzdb[k] = sum_{n,jo,io} dzdy[io,jo,k,n] ------------------
// Stage 1: block (k, s) sums the units u = s, s+S, ... where unit u = (n, chunk c)
// covers dzdy[c*CH .. min((c+1)*CH, HoWo)) of image n, filter k.  Stage 2 adds the S
// partials of each k in a fixed order, so the result does not depend on scheduling.
constexpr int BIAS_CHUNK = 4096;

__global__ __launch_bounds__(256) void bias_partial_kernel(const float *__restrict__ dzdy, float *__restrict__ part,
                                                           int HoWo, int K, int N, int chunks, int S) {
    const int k = blockIdx.x, s = blockIdx.y;
    const int units = N * chunks;
    float acc = 0.f;
    for (int u = s; u < units; u += S) {
        const int n = u / chunks, c = u - n * chunks;
        const float *p = dzdy + ((size_t)n * K + k) * HoWo;
        const int lo = c * BIAS_CHUNK;
        const int hi = min(lo + BIAS_CHUNK, HoWo);
        for (int e = lo + threadIdx.x; e < hi; e += 256) acc += p[e];
    }
    __shared__ float red[4];
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) part[(size_t)k * S + s] = (red[0] + red[1]) + (red[2] + red[3]);
}

// The same with 16-byte loads, four of them in flight per thread before the first addition: for planes of a
// multiple of 4 samples in an array aligned to 16 bytes (then every (n, k) plane and every chunk is aligned).
// The order of the additions differs from the kernel above but is as fixed.
__global__ __launch_bounds__(256) void bias_partial_v4_kernel(const float *__restrict__ dzdy, float *__restrict__ part,
                                                              int HoWo, int K, int N, int chunks, int S) {
    const int k = blockIdx.x, s = blockIdx.y;
    const int units = N * chunks;
    float4 a0 = {0.f, 0.f, 0.f, 0.f}, a1 = a0, a2 = a0, a3 = a0;
    for (int u = s; u < units; u += S) {
        const int n = u / chunks, c = u - n * chunks;
        const float4 *p = reinterpret_cast<const float4 *>(dzdy + ((size_t)n * K + k) * HoWo);
        const int lo = c * (BIAS_CHUNK / 4);
        const int hi = min(lo + BIAS_CHUNK / 4, HoWo / 4);
        const int e = lo + threadIdx.x;
        const float4 z = {0.f, 0.f, 0.f, 0.f};
        static_assert(BIAS_CHUNK == 4 * 4 * 256, "four 16-byte loads per thread and chunk");
        const float4 v0 = e < hi ? p[e] : z, v1 = e + 256 < hi ? p[e + 256] : z;
        const float4 v2 = e + 512 < hi ? p[e + 512] : z, v3 = e + 768 < hi ? p[e + 768] : z;
        a0.x += v0.x; a0.y += v0.y; a0.z += v0.z; a0.w += v0.w;
        a1.x += v1.x; a1.y += v1.y; a1.z += v1.z; a1.w += v1.w;
        a2.x += v2.x; a2.y += v2.y; a2.z += v2.z; a2.w += v2.w;
        a3.x += v3.x; a3.y += v3.y; a3.z += v3.z; a3.w += v3.w;
    }
    float acc = ((a0.x + a0.y) + (a0.z + a0.w)) + ((a1.x + a1.y) + (a1.z + a1.w)) +
                (((a2.x + a2.y) + (a2.z + a2.w)) + ((a3.x + a3.y) + (a3.z + a3.w)));
    __shared__ float red[4];
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) part[(size_t)k * S + s] = (red[0] + red[1]) + (red[2] + red[3]);
}

// ---- ReLU mask fused with the bias derivative ------------------------------------------------------
// Sec. 6.4.1 of the manual: through y = max(0, p) the derivative is dz/dp = [p > 0] dz/dy, and
// y > 0 exactly where p > 0.  One pass reads y and dzdy, writes dzdp = [y > 0] * dzdy (the derivative
// that the convolution's own backward passes take) and sums it per filter (dzdb).  Same two stages,
// same unit order as bias_partial_kernel.  dzdp may be the array dzdy (each element is read, then
// written, by one thread).
__global__ __launch_bounds__(256) void relu_bias_partial_kernel(const float *__restrict__ y, const float *dzdy,
                                                                float *dzdp, float *__restrict__ part, int HoWo,
                                                                int K, int N, int chunks, int S) {
    const int k = blockIdx.x, s = blockIdx.y;
    const int units = N * chunks;
    float acc = 0.f;
    for (int u = s; u < units; u += S) {
        const int n = u / chunks, c = u - n * chunks;
        const size_t base = ((size_t)n * K + k) * HoWo;
        const int lo = c * BIAS_CHUNK;
        const int hi = min(lo + BIAS_CHUNK, HoWo);
        for (int e = lo + threadIdx.x; e < hi; e += 256) {
            const float m = y[base + e] > 0.f ? dzdy[base + e] : 0.f;
            dzdp[base + e] = m;
            acc += m;
        }
    }
    __shared__ float red[4];
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) part[(size_t)k * S + s] = (red[0] + red[1]) + (red[2] + red[3]);
}
// small output planes: as bias_rows_partial_kernel
__global__ __launch_bounds__(256) void relu_bias_rows_partial_kernel(const float *__restrict__ y, const float *dzdy,
                                                                     float *dzdp, float *__restrict__ part,
                                                                     int KHoWo, int N, int S) {
    const int e = blockIdx.x * 256 + threadIdx.x, s = blockIdx.y;
    if (e >= KHoWo) return;
    float acc = 0.f;
    for (int n = s; n < N; n += S) {
        const size_t a = (size_t)n * KHoWo + e;
        const float m = y[a] > 0.f ? dzdy[a] : 0.f;
        dzdp[a] = m;
        acc += m;
    }
    part[(size_t)s * KHoWo + e] = acc;
}

// Small output planes (down to the 1x1 output of a fully-connected layer): one image of dzdy is
// a contiguous row of K*HoWo values, so threads run along that row and step over the images.
// Stage 1: part[s][e] = sum over images n = s, s+S, ... of dzdy[e + K*HoWo*n], e = p + HoWo*k.
__global__ __launch_bounds__(256) void bias_rows_partial_kernel(const float *__restrict__ dzdy, float *__restrict__ part,
                                                                int KHoWo, int N, int S) {
    const int e = blockIdx.x * 256 + threadIdx.x, s = blockIdx.y;
    if (e >= KHoWo) return;
    float acc = 0.f;
    for (int n = s; n < N; n += S) acc += dzdy[(size_t)n * KHoWo + e];
    part[(size_t)s * KHoWo + e] = acc;
}
// Stage 2: one wavefront per filter adds its S*HoWo partials in a fixed order.
__global__ __launch_bounds__(256) void bias_rows_final_kernel(const float *__restrict__ part, float *__restrict__ dzdb,
                                                              int HoWo, int K, int S) {
    const int lane = threadIdx.x & 63;
    const int k = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (k >= K) return;                 // whole wave leaves together
    const int KHoWo = K * HoWo, total = S * HoWo;
    float acc = 0.f;
    for (int u = lane; u < total; u += 64) {
        const int s = u / HoWo, p = u - s * HoWo;
        acc += part[(size_t)s * KHoWo + (size_t)k * HoWo + p];
    }
    acc = wave_sum(acc);
    if (lane == 0) dzdb[k] = acc;
}

__global__ __launch_bounds__(256) void bias_final_kernel(const float *__restrict__ part, float *__restrict__ dzdb,
                                                         int K, int S) {
    int k = blockIdx.x * 256 + threadIdx.x;
    if (k >= K) return;
    float acc = 0.f;
    for (int s = 0; s < S; ++s) acc += part[(size_t)k * S + s];
    dzdb[k] = acc;
}

}  // namespace mcn
