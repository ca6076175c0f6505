// Filter derivative on the fp32 matrix cores, as a persistent split-K implicit GEMM.
//
// MatConvNet manual (arXiv 1412.4564) Sec. 6.1: dz/dF = phi(x)^T dz/dY, summed over
// the batch, i.e.
//   dzdw[fi,fj,c,k] = sum_{n,jo,io} x[Sh*io+fi-Pt, Sw*jo+fj-Pl, g*Cg+c, n] * dzdy[io,jo,k,n].
// GEMM view:  OUT[k][r] = sum_p DY[k][p] * PATCH[r][p],  r = fi + Hf*(fj + Wf*c)  (the memory order
// of one filter), p = output pixel.  The reduction runs over pixels, two per
// v_mfma_f32_32x32x2_f32.  A tile is TK filters x TR coefficients; its reduction is cut into
// units of PCH pixels.  For a unit the block stages in LDS the dzdy tile [k][pixel] and, per
// input channel of the tile's r range, the slab of x that those pixels read (no im2row
// buffer), plus a table pixel -> slab offset.  Lanes run along r, so the final stores are
// coalesced.
//
// Scheduling is the same as in the forward kernel: all (tile, unit) pairs are cut into
// nblocks equal contiguous ranges, one per resident block; a block writes its piece of a
// tile to a workspace and wgrad_fixup_kernel sums the pieces of each tile in block order,
// so results do not depend on scheduling (no float atomics).  Global -> LDS loads bypass the
// registers and run one unit ahead.
//
// Pixels are numbered as in the forward kernel: rows are cut into row blocks of TI rows,
// and inside a row block q = ii + TI*(jo + Wo*n).
//
// With a 1x1 view this kernel is a plain GEMM  OUT[k][c] = sum_p A[k][p] B[c][p]  with both
// operands contiguous along the reduction, which is what the forward pass of a
// fully-connected layer needs (Sec. 4.1, "fully connected" case): there p runs over the filter
// coefficients, k over images and c over filters, and `rbias` adds the bias per c.
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
    int EPT;             // slab positions per thread: ceil(SRP*SC / threads)
    int KT, RT;          // filter tiles per group, r tiles
    int QN;              // TI*Wo*N
    int PCH, PCHP;       // pixels per unit (multiple of 4), LDS pitch of a dzdy row (odd)
    int CPR;             // units per row block: ceil(QN / PCH)
    int NU;              // units per tile = RB * CPR
    int R;               // Hf*Wf*Cg
    int XS;              // floats per slab buffer (max channels of an r tile * CP)
    int tiles, nblocks;
};

template <int WK, int WR, int MK, int MR, int WPE>
__global__ __launch_bounds__(64 * WK * WR, WPE) void wgrad_sk_kernel(WgradParams P, const float *__restrict__ x,
                                                                     const float *__restrict__ dzdy,
                                                                     const float *__restrict__ rbias,
                                                                     float *__restrict__ out,
                                                                     float *__restrict__ part) {
    constexpr int NT = 64 * WK * WR;
    constexpr int NW = WK * WR;
    constexpr int TK = WK * MK * 32;
    constexpr int TR = WR * MR * 32;
    const int PCH = P.PCH, PCHP = P.PCHP;
    const int NSEG = (PCH + 63) >> 6;
    const int YS = TK * PCHP;
    const int CP = P.CP, SRP = P.SRP;
    const int T = P.Hf * P.Wf;

    extern __shared__ __align__(16) float lds[];
    float *ybuf = lds;                                        // [2][TK*PCHP]
    float *xbuf = lds + 2 * YS;                               // [2][XS]
    int *tabbuf = reinterpret_cast<int *>(xbuf + 2 * P.XS);   // [2][NSEG*64] pixel -> slab offset
    int *etab = tabbuf + 2 * NSEG * 64;                       // [EPT][NT] slab position -> (col, row), private per thread

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, l32 = lane & 31;
    const int wk = wave % WK, wr = wave / WK;
    const int HW = P.H * P.W, HoWo = P.Ho * P.Wo;

    const int vb = sk_virtual_block(blockIdx.x, P.nblocks);
    const long long total = (long long)P.tiles * P.NU;
    const long long ub = sk_begin(total, P.nblocks, vb), ue = sk_begin(total, P.nblocks, vb + 1);
    if (ub >= ue) return;

    // slab position e = col*SRP + r  ->  (col, r); r >= SR is pitch padding
    for (int s = 0; s < P.EPT; ++s) {
        const int e = tid + NT * s;
        const int col = e / SRP;
        const int r = e - col * SRP;
        etab[s * NT + tid] = (col < P.SC && r < P.SR) ? (col << 16 | r) : -1;
    }

    // ---- load side -------------------------------------------------------------------------
    __amdgpu_buffer_rsrc_t xrs = __builtin_amdgcn_make_buffer_rsrc((void *)x, 0, 0x7fffffff, BUFFER_FLAGS);
    __amdgpu_buffer_rsrc_t yrs = xrs;
    int l_klim = 0, l_nch = 0;
    auto setup_load = [&](int t) {
        const int rt = t % P.RT; t /= P.RT;
        const int kt = t % P.KT;
        const int g = t / P.KT;
        const int r_lo = rt * TR;
        const int r_hi = min(r_lo + TR, P.R);
        const int c_lo = r_lo / T;
        l_nch = (r_hi - 1) / T - c_lo + 1;
        l_klim = min(P.Kg - kt * TK, TK);
        xrs = __builtin_amdgcn_make_buffer_rsrc((void *)(x + ((size_t)g * P.Cg + c_lo) * HW), 0, 0x7fffffff, BUFFER_FLAGS);
        yrs = __builtin_amdgcn_make_buffer_rsrc((void *)(dzdy + ((size_t)g * P.Kg + (size_t)kt * TK) * HoWo), 0,
                                                0x7fffffff, BUFFER_FLAGS);
    };
    auto issue_loads = [&](int uu, int b) {
        float *yb = ybuf + b * YS;
        float *xb = xbuf + b * P.XS;
        int *tb = tabbuf + b * NSEG * 64;
        const int rb = uu / P.CPR;
        const int qa = (uu - rb * P.CPR) * PCH;
        const int q_hi = min(qa + PCH, P.QN);
        // unit geometry (uniform)
        const int c_first = qa / P.TI;
        const int n_first = c_first / P.Wo;
        const int u0 = (c_first - n_first * P.Wo) * P.Sw;
        // dzdy tile: one wave instruction = 64 pixels of one filter
        for (int seg = 0; seg < NSEG; ++seg) {
            const int pl = seg * 64 + lane;
            const int q = qa + pl;
            const int c = q / P.TI;
            const int ii = q - c * P.TI;
            const int n = c / P.Wo;
            const int jo = c - n * P.Wo;
            const int io = rb * P.TI + ii;
            const bool pok = q < q_hi && io < P.Ho;
            const unsigned yoff = pok ? 4u * (unsigned)(io + P.Ho * jo + n * (P.Ktot * HoWo)) : SLAB_INVALID;
            if (wave == 0) tb[pl] = pok ? ii * P.Sh + SRP * (jo * P.Sw + (n - n_first) * P.Wp - u0) : 0;
            if (pl < PCH) {
                for (int k = wave; k < l_klim; k += NW)
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(yrs, MCN_LDS_PTR(yb + k * PCHP + seg * 64), 4, yoff,
                                                             (unsigned)k * (unsigned)HoWo * 4u, 0, 0);
            }
        }
        // x slab of the tile's channels
        const int row0 = rb * P.TI * P.Sh - P.Pt;
        const int ntot = SRP * P.SC;
        for (int s = 0; s < P.EPT; ++s) {
            const int e0 = wave * 64 + NT * s;
            if (e0 >= ntot) break;
            const int cr = etab[s * NT + tid];
            const int col = cr >> 16, r = cr & 0xffff;
            const int U = u0 + col;
            const int ni = U / P.Wp;
            const int j = U - ni * P.Wp - P.Pl;
            const int i = row0 + r;
            const bool ok = cr >= 0 && i >= 0 && i < P.H && j >= 0 && j < P.W && (n_first + ni) < P.N;
            const unsigned go = ok ? 4u * (unsigned)(i + P.H * j + (n_first + ni) * (P.Ctot * HW)) : SLAB_INVALID;
            if (e0 + lane < ntot) {
                for (int d = 0; d < l_nch; ++d)
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(xrs, MCN_LDS_PTR(xb + d * CP + e0), 4, go,
                                                             (unsigned)d * (unsigned)HW * 4u, 0, 0);
            }
        }
    };

    // ---- compute side ----------------------------------------------------------------------
    int roff[MR];
    int c_rt = 0, c_kt = 0, c_g = 0;
    floatx16 acc[MK][MR];
    auto setup_compute = [&](int t) {
        const int rt = t % P.RT; t /= P.RT;
        const int kt = t % P.KT;
        const int g = t / P.KT;
        c_rt = rt; c_kt = kt; c_g = g;
        const int r_lo = rt * TR;
        const int c_lo = r_lo / T;
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
#pragma unroll
        for (int mk = 0; mk < MK; ++mk)
#pragma unroll
            for (int mr = 0; mr < MR; ++mr)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[mk][mr][v] = 0.f;
    };
    const int aoff = (wk * MK * 32 + l32) * PCHP + half;
    auto compute = [&](int b) {
        const float *yb = ybuf + b * YS + aoff;
        const float *xb = xbuf + b * P.XS;
        const int *tb = tabbuf + b * NSEG * 64 + half;
        const int steps = PCH >> 1;             // even
        float a0[MK], b0[MR], a1[MK], b1[MR];
        auto fetch = [&](float *a, float *bq, int t, int tv) {
#pragma unroll
            for (int mk = 0; mk < MK; ++mk) a[mk] = yb[mk * 32 * PCHP + 2 * t];
#pragma unroll
            for (int mr = 0; mr < MR; ++mr) bq[mr] = xb[roff[mr] + tv];
        };
        auto mma = [&](const float *a, const float *bq) {
#pragma unroll
            for (int mk = 0; mk < MK; ++mk)
#pragma unroll
                for (int mr = 0; mr < MR; ++mr)
                    acc[mk][mr] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[mk], bq[mr], acc[mk][mr], 0, 0, 0);
        };
        int t0 = tb[0], t1 = tb[2];
        fetch(a0, b0, 0, t0);
        for (int t = 0; t < steps; t += 2) {
            const int t0n = tb[2 * min(t + 2, steps - 1)];
            const int t1n = tb[2 * min(t + 3, steps - 1)];
            fetch(a1, b1, t + 1, t1);
            __builtin_amdgcn_sched_barrier(0);
            mma(a0, b0);
            __builtin_amdgcn_sched_barrier(0);
            if (t + 2 < steps) fetch(a0, b0, t + 2, t0n);
            __builtin_amdgcn_sched_barrier(0);
            mma(a1, b1);
            __builtin_amdgcn_sched_barrier(0);
            t0 = t0n; t1 = t1n;
        }
        (void)t0;
    };
    // lane holds coefficient r (lane&31) of each r tile and 16 filters of each filter tile
    auto store_tile = [&]() {
        const int klim = min(P.Kg - c_kt * TK, TK);
#pragma unroll
        for (int mr = 0; mr < MR; ++mr) {
            const int r = c_rt * TR + (wr * MR + mr) * 32 + l32;
            if (r < P.R) {
                const float rb = rbias ? rbias[r] : 0.f;
#pragma unroll
                for (int mk = 0; mk < MK; ++mk)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int kl = (wk * MK + mk) * 32 + (v >> 2) * 8 + half * 4 + (v & 3);
                        if (kl < klim) out[(size_t)(c_g * P.Kg + c_kt * TK + kl) * P.R + r] = acc[mk][mr][v] + rb;
                    }
            }
        }
    };
    auto store_partial = [&](int slot) {
        float *dst = part + (size_t)slot * (TK * TR);
#pragma unroll
        for (int mr = 0; mr < MR; ++mr)
#pragma unroll
            for (int mk = 0; mk < MK; ++mk)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int kloc = (wk * MK + mk) * 32 + (v >> 2) * 8 + half * 4 + (v & 3);
                    dst[kloc * TR + (wr * MR + mr) * 32 + l32] = acc[mk][mr][v];
                }
    };

    // ---- the block's range of units --------------------------------------------------------
    const int NU = P.NU;
    int t_c = (int)(ub / NU);
    int uu_c = (int)(ub - (long long)t_c * NU);
    int t_l = t_c, uu_l = uu_c;
    bool first_segment = true;
    auto segment_is_whole = [&](int t, int uu) { return uu == 0 && (long long)(t + 1) * NU <= ue; };
    setup_load(t_l);
    issue_loads(uu_l, 0);
    bool whole = segment_is_whole(t_c, uu_c);
    setup_compute(t_c);

    const int nunits = (int)(ue - ub);
    for (int it = 0; it < nunits; ++it) {
        __builtin_amdgcn_s_waitcnt(WAIT_VMCNT0);
        __syncthreads();
        if (it + 1 < nunits) {
            if (++uu_l == NU) { uu_l = 0; ++t_l; setup_load(t_l); }
            issue_loads(uu_l, (it + 1) & 1);
        }
        compute(it & 1);
        const bool last = it + 1 == nunits;
        if (uu_c + 1 == NU || last) {
            if (whole) store_tile();
            else store_partial(2 * vb + (first_segment ? 0 : 1));
            first_segment = false;
            if (!last) {
                ++t_c; uu_c = 0;
                whole = segment_is_whole(t_c, 0);
                setup_compute(t_c);
            }
        } else {
            ++uu_c;
        }
    }
}

// Sum the pieces of every tile shared between blocks, in block order, and write the tile.
template <int TK, int TR>
__global__ __launch_bounds__(256) void wgrad_fixup_kernel(WgradParams P, const float *__restrict__ part,
                                                          const float *__restrict__ rbias, float *__restrict__ out) {
    const int j = blockIdx.x + 1;
    const long long total = (long long)P.tiles * P.NU;
    const long long B = sk_begin(total, P.nblocks, j);
    const int t = (int)(B / P.NU);
    const long long t_lo = (long long)t * P.NU, t_hi = t_lo + P.NU;
    if (B == t_lo) return;
    if (sk_begin(total, P.nblocks, j - 1) > t_lo) return;
    int tt = t;
    const int rt = tt % P.RT; tt /= P.RT;
    const int kt = tt % P.KT;
    const int g = tt / P.KT;
    const int klim = min(P.Kg - kt * TK, TK);
    // blocks that hold a piece of this tile: j-1 .. b_last
    int b_last = j;
    while (b_last + 1 < P.nblocks && sk_begin(total, P.nblocks, b_last + 1) < t_hi) ++b_last;
    const bool first_is_head = sk_begin(total, P.nblocks, j - 1) >= t_lo;
    for (int e = blockIdx.y * 256 + threadIdx.x; e < TK * TR; e += gridDim.y * 256) {
        const int kloc = e / TR, rl = e - kloc * TR;
        const int r = rt * TR + rl;
        if (kloc >= klim || r >= P.R) continue;
        float acc = part[(size_t)(2 * (j - 1) + (first_is_head ? 0 : 1)) * (TK * TR) + e];
        for (int b = j; b <= b_last; ++b) acc += part[(size_t)(2 * b) * (TK * TR) + e];
        if (rbias) acc += rbias[r];
        out[(size_t)(g * P.Kg + kt * TK + kloc) * P.R + r] = acc;
    }
}

}  // namespace mcn
