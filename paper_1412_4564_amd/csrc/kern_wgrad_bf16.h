// Filter derivative on the bf16 matrix cores (v_mfma_f32_32x32x16_bf16): the "operands rounded
// to bf16 on chip, fp32 accumulation" variant of kern_wgrad.h, for vertical stride 1.
//
// MatConvNet manual (arXiv 1412.4564) Sec. 6.1, dz/dF = phi(x)^T dz/dY summed over the batch:
//   dzdw[fi,fj,c,k] = sum_{n,jo,io} x[io+fi-Pt, Sw*jo+fj-Pl, g*Cg+c, n] * dzdy[io,jo,k,n],
// with every x and dzdy rounded to bf16 (round to nearest even) before the products are formed.
// GEMM view as in kern_wgrad.h: OUT[k][r] = sum_p DY[k][p] * PATCH[r][p], r = fi + Hf*(fj + Wf*c).
//
// One MFMA consumes 16 pixels: lane l holds 8 consecutive rows (an "octet") of one column for
// filter or coefficient l%32; the lower half-wave takes column dc, the upper one column dc+1.
// Arrays in memory stay fp32, rows contiguous, so an octet is 32 contiguous bytes in memory and
// one 16-byte word in LDS:
//   dzdy tile  [k][column][octet]                          one word = 8 rows of dzdy
//   x slab     [channel][fi][slab column][octet]           one word = x rows i0+fi+8*octet .. +7
// i.e. the slab is stored Hf times, shifted by one row each, so that the operand of filter row
// fi is an aligned word whatever fi is (a 16-byte LDS read cannot start at an odd row).
// Staging goes through registers (load fp32, convert, write words), one unit ahead of the MFMAs.
//
// A unit is a patch of TI rows x MC columns of ONE image; units are ordered image-fastest, so
// everything that depends on the patch (which elements are padding or lie outside the plane) is
// recomputed only when the patch changes, and from unit to unit only scalar offsets change.
//
// Scheduling: the reduction of every tile is cut into `nchunks` equal ranges of units and block
// (tile, chunk) sums one range.  Blocks are numbered chunk-major and mapped so that the blocks of
// one chunk -- which read the same dzdy and x at the same time -- sit on one XCD and share its L2:
// memory then delivers each operand about once although every r tile reads all of dzdy.  The
// pieces of a tile are added by wgrad_bf16_fixup_kernel in a fixed order (no float atomics).
#pragma once
#include "kern_igemm_bf16.h"

namespace mcn {

struct WgradBfParams {
    int H, W, N, Ctot, Cg;
    int Ho, Wo, Ktot, Kg, G;
    int Hf, Wf, Sw, Pt, Pl;    // vertical stride is 1
    int TI, RB, TIG;           // rows per patch, patches per column, octets per patch column = ceil(TI/8)
    int MC, CC;                // columns per patch (even), patches per row of patches
    int SC;                    // slab columns: (MC-1)*Sw + Wf
    int PW, PYW;               // words per dzdy row: TIG*MC, and its LDS pitch (odd)
    int RGP, CPF, CPC;         // slab pitches in words: per column, per shifted copy, per channel
    int NCH;                   // channels an r tile can touch
    int KT, RT, R;             // filter tiles per group, r tiles, Hf*Wf*Cg
    int NU;                    // units per tile: RB*CC*N
    int tiles, nchunks, nblocks;   // nblocks = tiles*nchunks
};

constexpr int WGB_YT = 4;      // dzdy words a thread stages per unit, at most
constexpr int WGB_XT = 2;      // slab (channel, column, octet) positions a thread stages per unit, at most

// Blocks on consecutive hardware ids land on different XCDs: give XCD x the virtual blocks
// [x*per, (x+1)*per).  The grid is padded to a multiple of 8; padding blocks do nothing.
__device__ __host__ inline int wgb_grid(int nblocks) { return nblocks < 8 ? nblocks : (nblocks + 7) / 8 * 8; }
__device__ inline int wgb_virtual_block(int b, int grid) { return grid % 8 == 0 ? (b % 8) * (grid / 8) + b / 8 : b; }

template <int WK, int WR, int MK, int MR, int HF>
__global__ __launch_bounds__(64 * WK * WR, 2) void wgrad_bf16_kernel(WgradBfParams P, const float *__restrict__ x,
                                                                     const float *__restrict__ dzdy,
                                                                     float *__restrict__ out,
                                                                     float *__restrict__ part) {
    constexpr int NT = 64 * WK * WR;
    constexpr int TK = WK * MK * 32;
    constexpr int TR = WR * MR * 32;
    constexpr int NE = 8 + HF - 1;             // rows a slab position loads: one octet for each of the HF shifts
    const int YS = TK * P.PYW;                 // words per dzdy buffer
    const int XS = P.NCH * P.CPC;              // words per slab buffer
    const int T = P.Hf * P.Wf;

    extern __shared__ __align__(16) float lds[];
    uintx4 *ybuf = reinterpret_cast<uintx4 *>(lds);      // [2][YS]
    uintx4 *xbuf = ybuf + 2 * YS;                        // [2][XS]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, l32 = lane & 31;
    const int wk = wave % WK, wr = wave / WK;
    const int HW = P.H * P.W, HoWo = P.Ho * P.Wo;

    const int vb = wgb_virtual_block(blockIdx.x, gridDim.x);
    if (vb >= P.nblocks) return;
    const int tile = vb % P.tiles, chunk = vb / P.tiles;
    const int u_begin = (int)((long long)P.NU * chunk / P.nchunks);
    const int u_end = (int)((long long)P.NU * (chunk + 1) / P.nchunks);
    if (u_begin >= u_end) return;              // cannot happen: nchunks <= NU

    const int rt = tile % P.RT, kt = (tile / P.RT) % P.KT, g = tile / (P.RT * P.KT);
    const int r_lo = rt * TR;
    const int r_hi = min(r_lo + TR, P.R);
    const int c_lo = r_lo / T;
    const int nch = (r_hi - 1) / T - c_lo + 1;
    const int klim = min(P.Kg - kt * TK, TK);

    // the arrays from the tile's first filter / channel of an image on; the buffer resources are built per unit at
    // the unit's image, so offsets stay inside one image (under 2^31 bytes: checked on the host) whatever the batch
    const size_t ybase = ((size_t)g * P.Kg + (size_t)kt * TK) * HoWo;
    const size_t xbase = ((size_t)g * P.Cg + c_lo) * HW;
    const int yleft = (int)(((size_t)P.Ktot * HoWo - ybase) * 4), xleft = (int)(((size_t)P.Ctot * HW - xbase) * 4);

    // ---- what this thread stages, fixed for the whole kernel -----------------------------------
    int y_k[WGB_YT], y_dc[WGB_YT], y_rg[WGB_YT], y_lds[WGB_YT];
#pragma unroll
    for (int s = 0; s < WGB_YT; ++s) {
        const int q = tid + NT * s;
        const int k = q / P.PW, w = q - k * P.PW;
        y_k[s] = q < TK * P.PW ? k : -1;
        y_dc[s] = w / P.TIG;
        y_rg[s] = w - y_dc[s] * P.TIG;
        y_lds[s] = k * P.PYW + w;
    }
    int x_c[WGB_XT], x_col[WGB_XT], x_rg[WGB_XT], x_lds[WGB_XT];
#pragma unroll
    for (int s = 0; s < WGB_XT; ++s) {
        const int q = tid + NT * s;
        const int per_c = P.SC * P.TIG;
        const int c = q / per_c, rem = q - c * per_c;
        x_c[s] = q < P.NCH * per_c ? c : -1;
        x_col[s] = rem / P.TIG;
        x_rg[s] = rem - x_col[s] * P.TIG;
        x_lds[s] = c * P.CPC + x_col[s] * P.RGP + x_rg[s];
    }

    // ---- per patch: where the staged elements are in memory (or out of range = zero) -----------
    unsigned y_vo[WGB_YT];
    int y_nv[WGB_YT];                 // valid rows of the octet (8 except in a patch's last, partial octet)
    unsigned x_vo[WGB_XT][NE];
    bool partial_rows = false;
    auto setup_patch = [&](int pp) {
        const int jc = pp / P.RB, rb = pp - jc * P.RB;
        const int io0 = rb * P.TI, jo0 = jc * P.MC;
        const int rows = min(P.TI, P.Ho - io0), cols = min(P.MC, P.Wo - jo0);
        partial_rows = (rows & 7) != 0;
#pragma unroll
        for (int s = 0; s < WGB_YT; ++s) {
            const int nv = min(8, rows - 8 * y_rg[s]);
            const bool ok = y_k[s] >= 0 && y_k[s] < klim && y_dc[s] < cols && nv > 0;
            y_nv[s] = ok ? nv : 0;
            y_vo[s] = ok ? 4u * (unsigned)(io0 + 8 * y_rg[s] + P.Ho * (jo0 + y_dc[s]) + y_k[s] * HoWo) : SLAB_INVALID;
        }
        const int i0 = io0 - P.Pt, j0 = jo0 * P.Sw - P.Pl;
#pragma unroll
        for (int s = 0; s < WGB_XT; ++s) {
            const int j = j0 + x_col[s];
            const int ibase = i0 + 8 * x_rg[s];
            const bool okc = x_c[s] >= 0 && x_c[s] < nch && j >= 0 && j < P.W;
            const unsigned base = 4u * (unsigned)(ibase + P.H * j + x_c[s] * HW);
#pragma unroll
            for (int e = 0; e < NE; ++e)
                x_vo[s][e] = (okc && (unsigned)(ibase + e) < (unsigned)P.H) ? base + 4u * e : SLAB_INVALID;
        }
    };

    // ---- staging registers ---------------------------------------------------------------------
    uintx4 y_lo[WGB_YT], y_hi[WGB_YT];
    float x_dat[WGB_XT][NE];
    auto issue_loads = [&](int n) {
        const __amdgpu_buffer_rsrc_t yrs = __builtin_amdgcn_make_buffer_rsrc(
            (void *)(dzdy + ybase + (size_t)n * P.Ktot * HoWo), 0, yleft, BUFFER_FLAGS);
        const __amdgpu_buffer_rsrc_t xrs = __builtin_amdgcn_make_buffer_rsrc(
            (void *)(x + xbase + (size_t)n * P.Ctot * HW), 0, xleft, BUFFER_FLAGS);
        const unsigned ysoff = 0u, xsoff = 0u;
#pragma unroll
        for (int s = 0; s < WGB_YT; ++s) {
            if (s * NT < TK * P.PW) {          // block-uniform
                y_lo[s] = __builtin_bit_cast(uintx4, __builtin_amdgcn_raw_buffer_load_b128(yrs, y_vo[s], ysoff, 0));
                y_hi[s] = __builtin_bit_cast(uintx4, __builtin_amdgcn_raw_buffer_load_b128(yrs, y_vo[s], ysoff + 16u, 0));
            }
        }
#pragma unroll
        for (int s = 0; s < WGB_XT; ++s) {
            if (s * NT < P.NCH * P.SC * P.TIG) {
#pragma unroll
                for (int e = 0; e < NE; ++e)
                    x_dat[s][e] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(xrs, x_vo[s][e], xsoff, 0));
            }
        }
    };
    auto write_lds = [&](int b) {
#pragma unroll
        for (int s = 0; s < WGB_YT; ++s) {
            if (s * NT < TK * P.PW && y_k[s] >= 0) {
                uintx4 lo = y_lo[s], hi = y_hi[s];
                uintx4 v;
                v.x = pack_bf16x2(__uint_as_float(lo.x), __uint_as_float(lo.y));
                v.y = pack_bf16x2(__uint_as_float(lo.z), __uint_as_float(lo.w));
                v.z = pack_bf16x2(__uint_as_float(hi.x), __uint_as_float(hi.y));
                v.w = pack_bf16x2(__uint_as_float(hi.z), __uint_as_float(hi.w));
                if (partial_rows) {
                    // rows past the patch's last one belong to the next column: they must not count
                    const int nv = y_nv[s];
                    auto keep = [&](unsigned word, int first) {
                        return nv >= first + 2 ? word : nv == first + 1 ? (word & 0xffffu) : 0u;
                    };
                    v.x = keep(v.x, 0); v.y = keep(v.y, 2); v.z = keep(v.z, 4); v.w = keep(v.w, 6);
                }
                ybuf[b * YS + y_lds[s]] = v;
            }
        }
#pragma unroll
        for (int s = 0; s < WGB_XT; ++s) {
            if (s * NT < P.NCH * P.SC * P.TIG && x_c[s] >= 0) {
#pragma unroll
                for (int fi = 0; fi < HF; ++fi) {
                    uintx4 v;
                    v.x = pack_bf16x2(x_dat[s][fi + 0], x_dat[s][fi + 1]);
                    v.y = pack_bf16x2(x_dat[s][fi + 2], x_dat[s][fi + 3]);
                    v.z = pack_bf16x2(x_dat[s][fi + 4], x_dat[s][fi + 5]);
                    v.w = pack_bf16x2(x_dat[s][fi + 6], x_dat[s][fi + 7]);
                    xbuf[b * XS + x_lds[s] + fi * P.CPF] = v;
                }
            }
        }
    };

    // ---- compute side --------------------------------------------------------------------------
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
            o = (c - c_lo) * P.CPC + fi * P.CPF + fj * P.RGP;
        }
        roff[mr] = o + half * P.Sw * P.RGP;           // the upper half-wave takes the next column
    }
    floatx16 acc[MK][MR];
#pragma unroll
    for (int mk = 0; mk < MK; ++mk)
#pragma unroll
        for (int mr = 0; mr < MR; ++mr)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mk][mr][v] = 0.f;
    const int aoff = (wk * MK * 32 + l32) * P.PYW + half * P.TIG;
    const int a_pair = P.TIG;                         // from the end of a column pair to the next pair
    const int x_pair = 2 * P.Sw * P.RGP - P.TIG;
    auto compute = [&](int b) {
        int ya[MK], xr[MR];
#pragma unroll
        for (int mk = 0; mk < MK; ++mk) ya[mk] = b * YS + aoff + mk * 32 * P.PYW;
#pragma unroll
        for (int mr = 0; mr < MR; ++mr) xr[mr] = b * XS + roff[mr];
        const int nsteps = (P.MC >> 1) * P.TIG;
        bf16x8 a0[MK], b0[MR], a1[MK], b1[MR];
        int rg = 0;
        auto fetch = [&](bf16x8 *a, bf16x8 *bq) {
#pragma unroll
            for (int mk = 0; mk < MK; ++mk) a[mk] = __builtin_bit_cast(bf16x8, ybuf[ya[mk]]);
#pragma unroll
            for (int mr = 0; mr < MR; ++mr) bq[mr] = __builtin_bit_cast(bf16x8, xbuf[xr[mr]]);
            // advance to the next step: next octet, or the first octet of the next column pair
            const bool wrap = ++rg == P.TIG;
            if (wrap) rg = 0;
            const int da = wrap ? 1 + a_pair : 1, dx = wrap ? 1 + x_pair : 1;
#pragma unroll
            for (int mk = 0; mk < MK; ++mk) ya[mk] += da;
#pragma unroll
            for (int mr = 0; mr < MR; ++mr) xr[mr] += dx;
        };
        auto mma = [&](const bf16x8 *a, const bf16x8 *bq) {
#pragma unroll
            for (int mk = 0; mk < MK; ++mk)
#pragma unroll
                for (int mr = 0; mr < MR; ++mr)
                    acc[mk][mr] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mk], bq[mr], acc[mk][mr], 0, 0, 0);
        };
        // no branches inside the loop, so that the waits inserted for the LDS reads are exact
        fetch(a0, b0);
        for (int s = 2; s < nsteps; s += 2) {        // steps s-2 and s-1, with s-1 and s in flight
            fetch(a1, b1);
            __builtin_amdgcn_sched_barrier(0);
            mma(a0, b0);
            __builtin_amdgcn_sched_barrier(0);
            fetch(a0, b0);
            __builtin_amdgcn_sched_barrier(0);
            mma(a1, b1);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (nsteps & 1) {
            mma(a0, b0);
        } else {
            fetch(a1, b1);
            __builtin_amdgcn_sched_barrier(0);
            mma(a0, b0);
            mma(a1, b1);
        }
    };

    // ---- the block's range of units: unit = image + N * patch ----------------------------------
    int pp = u_begin / P.N, n = u_begin - pp * P.N;
    setup_patch(pp);
    issue_loads(n);
    write_lds(0);
    const int nunits = u_end - u_begin;
    for (int it = 0; it < nunits; ++it) {
        lds_barrier();                 // buffer it&1 is complete, and the other one is free
        const bool more = it + 1 < nunits;
        if (more) {
            if (++n == P.N) { n = 0; ++pp; setup_patch(pp); }
            issue_loads(n);
        }
        __builtin_amdgcn_sched_barrier(0);
        compute(it & 1);
        __builtin_amdgcn_sched_barrier(0);
        if (more) write_lds((it + 1) & 1);
    }

    // lane holds coefficient r (lane&31) of each r tile and 16 filters of each filter tile
    const bool direct = P.nchunks == 1;
    float *dst = direct ? out : part + (size_t)vb * (TK * TR);
#pragma unroll
    for (int mr = 0; mr < MR; ++mr) {
        const int rl = (wr * MR + mr) * 32 + l32;
        const int r = r_lo + rl;
#pragma unroll
        for (int mk = 0; mk < MK; ++mk)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int kl = (wk * MK + mk) * 32 + (v >> 2) * 8 + half * 4 + (v & 3);
                if (direct) {
                    if (r < P.R && kl < klim) dst[(size_t)(g * P.Kg + kt * TK + kl) * P.R + r] = acc[mk][mr][v];
                } else {
                    dst[kl * TR + rl] = acc[mk][mr][v];
                }
            }
    }
}

// Sum the nchunks pieces of every tile and write the tile.  The order of the additions is
// fixed: piece i goes to partial sum i mod 8, the partial sums are added as a balanced tree.
// blockIdx.x = tile; one block = 64 results x 8 partial sums.
template <int TK, int TR>
__global__ __launch_bounds__(512) void wgrad_bf16_fixup_kernel(WgradBfParams P, const float *__restrict__ part,
                                                               float *__restrict__ out) {
    const int t = blockIdx.x;
    const int rt = t % P.RT, kt = (t / P.RT) % P.KT, g = t / (P.RT * P.KT);
    const int klim = min(P.Kg - kt * TK, TK);
    __shared__ float red[8][64];
    const int el = threadIdx.x & 63, pg = threadIdx.x >> 6;
    for (int e0 = blockIdx.y * 64; e0 < TK * TR; e0 += gridDim.y * 64) {
        const int e = e0 + el;
        float acc = 0.f;
        for (int i = pg; i < P.nchunks; i += 8) acc += part[((size_t)i * P.tiles + t) * (TK * TR) + e];
        red[pg][el] = acc;
        __syncthreads();
        if (pg == 0) {
            const int kloc = e / TR, rl = e - kloc * TR;
            const int r = rt * TR + rl;
            if (kloc < klim && r < P.R)
                out[(size_t)(g * P.Kg + kt * TK + kloc) * P.R + r] =
                    ((red[0][el] + red[1][el]) + (red[2][el] + red[3][el])) +
                    ((red[4][el] + red[5][el]) + (red[6][el] + red[7][el]));
        }
        __syncthreads();
    }
}

}  // namespace mcn
