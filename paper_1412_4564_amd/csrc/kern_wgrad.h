// Filter derivative on the fp32 matrix cores, as a split-K implicit GEMM.
//
// MatConvNet manual (arXiv 1412.4564) Sec. 6.1: dz/dF = phi(x)^T dz/dY, summed over
// the batch, i.e.
//   dzdw[fi,fj,c,k] = sum_{n,jo,io} x[Sh*io+fi-Pt, Sw*jo+fj-Pl, g*Cg+c, n] * dzdy[io,jo,k,n].
// GEMM view:  OUT[k][r] = sum_p DY[k][p] * PATCH[r][p],  r = fi + Hf*(fj + Wf*c)  (the memory order
// of one filter), p = output pixel.  The reduction runs over pixels, two per
// v_mfma_f32_32x32x2_f32.  A block owns a tile of TK filters x TR coefficients and one
// slice of the pixels (split-K); it walks its slice in chunks of PCH pixels, staging in LDS
// the dzdy tile [k][pixel] and, per input channel of its r range, the slab of x that those
// pixels read (no im2row buffer).  Lanes run along r, so the final stores are coalesced.
// Partial tiles go to a workspace and are summed in a fixed order by a second kernel, so
// results do not depend on scheduling.
//
// Pixels are numbered as in the forward kernel: rows are cut into row blocks of TI rows,
// and inside a row block q = ii + TI*(jo + Wo*n).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "kern_igemm.h"

namespace mcn {

struct WgradParams {
    int H, W, N, Ctot, Cg;
    int Ho, Wo, Ktot, Kg, G;
    int Hf, Wf, Sh, Sw, Pt, Pl;
    int TI, RB;          // rows per row block, row blocks
    int Wp;              // chained-column pitch of one image
    int SR, SRP, SC;     // slab rows, padded row pitch, columns
    int CP;              // slab channel pitch
    int KT, RT;          // filter tiles per group, r tiles
    int QN;              // TI*Wo*N
    int QS;              // pixels per split (multiple of PCH)
    int SPR;             // splits per row block
    int R;               // Hf*Wf*Cg
    int direct_out;      // 1: single split, write dzdw itself
    int XS;              // floats per slab buffer (max channels of an r tile * CP)
    int EPTU;            // slab elements per thread actually needed: ceil(SC*SR / threads)
};

template <int WK, int WR, int MK, int MR, int PCH, int EPT, int NCHMAX>
__global__ __launch_bounds__(64 * WK * WR) void wgrad_kernel(WgradParams P, const float *__restrict__ x,
                                                             const float *__restrict__ dzdy,
                                                             float *__restrict__ outp) {
    constexpr int NT = 64 * WK * WR;
    constexpr int TK = WK * MK * 32;
    constexpr int TR = WR * MR * 32;
    constexpr int PCHP = PCH + 1;            // odd pitch: conflict-free column reads of the dzdy tile
    constexpr int KSTEP = NT / PCH;          // filters covered by one pass of the block over the tile
    constexpr int KPT = (TK + KSTEP - 1) / KSTEP;   // dzdy elements per thread per chunk
    constexpr int STEPS = PCH / 2;
    static_assert(NT % PCH == 0, "tile/thread mismatch");

    extern __shared__ __align__(16) float lds[];
    // [2][TK*PCHP] dzdy tiles, [2][2*STEPS] pixel->slab offsets, [2][NCHMAX*CP] slabs
    float *ybuf = lds;
    int *tabbuf = reinterpret_cast<int *>(lds + 2 * TK * PCHP);   // [2][PCH]
    float *xbuf = lds + 2 * TK * PCHP + 2 * PCH;
    const int CP = P.CP, SRP = P.SRP;
    const int T = P.Hf * P.Wf;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int wk = wave % WK, wr = wave / WK;

    int b = blockIdx.x;
    const int rt = b % P.RT; b /= P.RT;
    const int kt = b % P.KT; b /= P.KT;
    const int g = b % P.G;   b /= P.G;
    const int sp = b % P.SPR;
    const int rb = b / P.SPR;
    const int split_id = rb * P.SPR + sp;

    const int q_lo = sp * P.QS;
    const int q_hi = min(q_lo + P.QS, P.QN);
    const int HW = P.H * P.W, HoWo = P.Ho * P.Wo;

    // channels of this r tile
    const int r_lo = rt * TR;
    const int r_hi = min(r_lo + TR, P.R);
    const int c_lo = r_lo / T;
    const int nch = (r_hi - 1) / T - c_lo + 1;          // <= NCHMAX (host guarantees)

    __amdgpu_buffer_rsrc_t xrs = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(x + ((size_t)g * P.Cg + c_lo) * HW), 0, 0x7fffffff, 0x00020000);
    __amdgpu_buffer_rsrc_t yrs = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(dzdy + ((size_t)g * P.Kg + (size_t)kt * TK) * HoWo), 0, 0x7fffffff, 0x00020000);

    // slab elements of this thread (compact [col][row] index; padded pitch in LDS)
    int s_col[EPT], s_lds[EPT];
    unsigned s_row[EPT];
    const int row0 = rb * P.TI * P.Sh - P.Pt;
#pragma unroll
    for (int s = 0; s < EPT; ++s) {
        const int e = tid + NT * s;
        const int col = e / P.SR;
        const int r = e - col * P.SR;
        const int i = row0 + r;
        s_col[s] = col;
        s_lds[s] = (col < P.SC) ? col * SRP + r : -1;
        s_row[s] = (col < P.SC && i >= 0 && i < P.H) ? 4u * (unsigned)i : SLAB_INVALID;
    }

    // dzdy tile element of this thread: pixel slot pl, filters kb + KSTEP*s
    const int pl = tid % PCH;
    const int kb = tid / PCH;
    const int klim = min(P.Kg - kt * TK, TK);       // filters of this tile that exist

    // lane's B offsets: r -> (channel, tap) -> slab offset
    int roff[MR];
#pragma unroll
    for (int mr = 0; mr < MR; ++mr) {
        const int r = r_lo + (wr * MR + mr) * 32 + l32;
        int o = 0;
        if (r < P.R) {
            const int c = r / T;
            const int tap = r - c * T;
            const int fj = tap / P.Hf;
            const int fi = tap - fj * P.Hf;
            o = (c - c_lo) * CP + fj * SRP + fi;
        }
        roff[mr] = o;
    }
    const int aoff = (wk * MK * 32 + l32) * PCHP + half;

    floatx16 acc[MK][MR];
#pragma unroll
    for (int mk = 0; mk < MK; ++mk)
#pragma unroll
        for (int mr = 0; mr < MR; ++mr)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mk][mr][v] = 0.f;

    float yreg[KPT];
    float xreg[NCHMAX][EPT];
    int tabreg = 0;

    auto load_chunk = [&](int qa) {
        // chunk geometry (uniform)
        const int c_first = qa / P.TI;
        const int n_first = c_first / P.Wo;
        const int u0 = (c_first - n_first * P.Wo) * P.Sw;
        // this thread's pixel
        const int q = qa + pl;
        const int c = q / P.TI;
        const int ii = q - c * P.TI;
        const int n = c / P.Wo;
        const int jo = c - n * P.Wo;
        const int io = rb * P.TI + ii;
        const bool pok = q < q_hi && io < P.Ho;
        tabreg = pok ? ii * P.Sh + SRP * (jo * P.Sw + (n - n_first) * P.Wp - u0) : 0;
        const unsigned ybase = pok ? 4u * (unsigned)(io + P.Ho * jo + n * (P.Ktot * HoWo) + kb * HoWo) : SLAB_INVALID;
#pragma unroll
        for (int s = 0; s < KPT; ++s) {
            const unsigned vo = (kb + KSTEP * s < klim) ? ybase : SLAB_INVALID;
            yreg[s] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(yrs, vo, (unsigned)(KSTEP * s) * (unsigned)HoWo * 4u, 0));
        }
        unsigned goff[EPT];
#pragma unroll
        for (int s = 0; s < EPT; ++s) {
            const int U = u0 + s_col[s];
            const int ni = (U >= P.Wp ? 1 : 0) + (U >= 2 * P.Wp ? 1 : 0);
            const int j = U - ni * P.Wp - P.Pl;
            const bool ok = j >= 0 && j < P.W && (n_first + ni) < P.N && s_row[s] != SLAB_INVALID;
            goff[s] = ok ? s_row[s] + 4u * (unsigned)(P.H * j + (n_first + ni) * (P.Ctot * HW)) : SLAB_INVALID;
        }
#pragma unroll
        for (int d = 0; d < NCHMAX; ++d) {
            const unsigned soff = (unsigned)d * (unsigned)HW * 4u;
#pragma unroll
            for (int s = 0; s < EPT; ++s) {
                float v = 0.f;
                if (d < nch && s < P.EPTU) v = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(xrs, goff[s], soff, 0));
                xreg[d][s] = v;
            }
        }
    };
    auto store_chunk = [&](int buf) {
        float *yb = ybuf + buf * (TK * PCHP);
        int *tb = tabbuf + buf * PCH;
        float *xb = xbuf + buf * P.XS;
#pragma unroll
        for (int s = 0; s < KPT; ++s)
            if (kb + KSTEP * s < TK) yb[(kb + KSTEP * s) * PCHP + pl] = yreg[s];
        if (tid < PCH) tb[(pl & 1) * STEPS + (pl >> 1)] = tabreg;     // [half][step]
#pragma unroll
        for (int d = 0; d < NCHMAX; ++d)
#pragma unroll
            for (int s = 0; s < EPT; ++s)
                if (d < nch && s < P.EPTU && s_lds[s] >= 0) xb[d * CP + s_lds[s]] = xreg[d][s];
    };

    if (q_lo < q_hi) {
        load_chunk(q_lo);
        store_chunk(0);
    }
    __syncthreads();

    int buf = 0;
    for (int qa = q_lo; qa < q_hi; qa += PCH) {
        const bool more = qa + PCH < q_hi;
        if (more) load_chunk(qa + PCH);
        const float *yb = ybuf + buf * (TK * PCHP) + aoff;
        const int *tb = tabbuf + buf * PCH + half * STEPS;
        const float *xb = xbuf + buf * P.XS;
        int tab[STEPS];
#pragma unroll
        for (int t = 0; t < STEPS; ++t) tab[t] = tb[t];
        // LDS reads of step t+1 are issued before the MFMAs of step t
        float a[2][MK], bb[2][MR];
        auto fetch = [&](int t, int slot) {
#pragma unroll
            for (int mk = 0; mk < MK; ++mk) a[slot][mk] = yb[mk * 32 * PCHP + 2 * t];
#pragma unroll
            for (int mr = 0; mr < MR; ++mr) bb[slot][mr] = xb[roff[mr] + tab[t]];
        };
        fetch(0, 0);
#pragma unroll
        for (int t = 0; t < STEPS; ++t) {
            if (t + 1 < STEPS) fetch(t + 1, (t + 1) & 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int mk = 0; mk < MK; ++mk)
#pragma unroll
                for (int mr = 0; mr < MR; ++mr)
                    acc[mk][mr] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[t & 1][mk], bb[t & 1][mr], acc[mk][mr], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (more) store_chunk(buf ^ 1);
        __syncthreads();
        buf ^= 1;
    }

    // epilogue: lane holds coefficient r (lane&31) of each r tile and 16 filters of each filter tile
    float *dst = outp + (P.direct_out ? (size_t)0 : (size_t)split_id * P.Ktot * P.R);
#pragma unroll
    for (int mr = 0; mr < MR; ++mr) {
        const int r = r_lo + (wr * MR + mr) * 32 + l32;
        if (r < P.R) {
#pragma unroll
            for (int mk = 0; mk < MK; ++mk)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int kl = (wk * MK + mk) * 32 + (v >> 2) * 8 + half * 4 + (v & 3);
                    if (kl < klim) dst[(size_t)(g * P.Kg + kt * TK + kl) * P.R + r] = acc[mk][mr][v];
                }
        }
    }
}

// dzdw[e] = sum over splits, in split order
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const float *__restrict__ part, float *__restrict__ dzdw,
                                                           int total, int splits) {
    int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    float acc = 0.f;
    for (int s = 0; s < splits; ++s) acc += part[(size_t)s * total + e];
    dzdw[e] = acc;
}

}  // namespace mcn
