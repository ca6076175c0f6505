// Filter derivative on the fp32 matrix cores, as a persistent split-K implicit GEMM.
//
// MatConvNet manual (arXiv 1412.4564) Sec. 6.1: dz/dF = phi(x)^T dz/dY, summed over
// the batch, i.e.
//   dzdw[fi,fj,c,k] = sum_{n,jo,io} x[Sh*io+fi-Pt, Sw*jo+fj-Pl, g*Cg+c, n] * dzdy[io,jo,k,n].
// GEMM view:  OUT[k][r] = sum_p DY[k][p] * PATCH[r][p],  r = fi + Hf*(fj + Wf*c)  (the memory order
// of one filter), p = output pixel.  The reduction runs over pixels, two per
// v_mfma_f32_32x32x2_f32.  A tile is TK filters x TR coefficients; its reduction is cut into
// units.  A unit is a patch of TI rows x MC columns of one image's output plane (pixel
// p = ii + TIE*dc of the patch, TIE = TI rounded up to even so that the two pixels of an MFMA
// step lie in one column), so everything that depends on the lane -- which pixel, which slab
// element -- is the same for every unit, and only scalar base offsets change from unit to
// unit; inside a column both operands advance by a constant stride from step to step, so the
// MFMA loop addresses LDS with immediate offsets.  For a unit the block stages in LDS the dzdy tile [k][pixel] and, per input
// channel of the tile's r range, the slab of x that the patch reads (no im2row buffer).  Lanes
// run along r, so the final stores are coalesced.
//
// Scheduling is the same as in the forward kernel: all (tile, unit) pairs are cut into
// nblocks equal contiguous ranges, one per resident block; a block writes its piece of a
// tile to a workspace and wgrad_fixup_kernel sums the pieces of each tile in block order,
// so results do not depend on scheduling (no float atomics).  Global -> LDS loads bypass the
// registers and run one unit ahead.
//
// The matrix core and the vector ALU share issue cycles, so the code around the MFMA loop is
// written to need few vector instructions: per-lane quantities are precomputed once per block,
// unit-dependent quantities are scalar.
//
// 3x3 filters at stride 1 (template flag WINO): the three row taps of a filter column are obtained for two
// output rows at a time from four products instead of six (the transpose of the minimal-filtering identity
// F(2,3) that the forward kernel uses: with d0..d3 the four input rows a pair of output rows reads and e0, e1
// the two rows of dzdy,
//   m0 = e0 (d0-d2),  m1 = (e0+e1)(d1+d2),  m2 = (e0-e1)(d2-d1),  m3 = e1 (d1-d3),
//   dzdw[0] = m0 + (m1+m2)/2,  dzdw[1] = (m1-m2)/2,  dzdw[2] = (m1+m2)/2 - m3,
// each m summed over all pairs of rows, columns and images on the matrix core).  A lane of the B operand
// is then a (filter column, channel) pair r' = fj + 3c, a pixel of the GEMM a pair of output rows, there are
// four sets of accumulators, and the combination above is applied once, when a tile is written.
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
    int TI, RB;          // rows per patch, patches per column (row blocks)
    int TIE;             // TI rounded up to even: pixel pitch of a patch column
    int MC, CC;          // columns per patch, patches per row of patches: ceil(Wo / MC)
    int SR, SRP, SC;     // slab rows, padded row pitch, columns
    int CP;              // slab channel pitch
    int EPT;             // slab positions per thread: ceil(SRP*SC / threads)
    int KT, RT;          // filter tiles per group, r tiles
    int PCH, PCHP;       // pixels per unit = TIE*MC, LDS pitch of a dzdy row (odd)
    int NU;              // units per tile = N * RB * CC
    int R;               // Hf*Wf*Cg
    int XS;              // floats per slab buffer (max channels of an r tile * CP)
    int tiles, nblocks;
    int relu;            // 1: results are written as max(0, .)  (forward pass of a fully-connected layer + ReLU)
    int nchunks;         // 0: blocks share the list of all (tile, unit) pairs in equal contiguous ranges;
                         // > 0: block (tile, chunk) sums chunk `chunk` of nchunks ranges of the tile's units
    // Chunk sizes: a chunk computed by one of the first n_first blocks (hardware ids; the blocks dispatched
    // first, one per compute unit) weighs w_first, any other w_later.  Of the two blocks resident on a
    // compute unit the one dispatched first gets more of the matrix core; with equal chunks it finishes
    // early and leaves the other to run alone, which uses the core less well.
    int n_first, w_first, w_later;
    // deal = 1 (one tile, equal chunk weights, a grid that is a multiple of 8): the chunks of the blocks on one XCD
    // cover a contiguous range of the tile's units between them, and the blocks take its units in turn (block i
    // of the XCD's n: units i, n + i, 2n + i, ... of the range) instead of a contiguous chunk each.  Units that
    // are adjacent in the plane, which share memory lines (half a line of dzdy per 16-row column run, the halo
    // rows and columns of x), are then fetched by the XCD's blocks at the same time and meet in its L2.
    int deal;
    // WINO kernels: TIE is TI rounded up to a multiple of 4 (two pairs of rows per MFMA step) and SRP, CP, PCHP
    // are even (8-byte LDS reads); tiles are counted in (filter column, channel) pairs, TR of them = 3*TR
    // coefficients.
};

// Chunked schedule: blocks are numbered chunk-major (virtual block = tile + tiles*chunk) and the virtual
// numbers are dealt to the XCDs in contiguous runs (consecutive hardware block ids land on different
// XCDs), so the tiles of one chunk, which read the same dzdy and x at the same time, share one L2 and
// memory delivers each operand about once.  The grid is padded to a multiple of 8; padding blocks do nothing.
__device__ __host__ inline int wg_chunk_grid(int nblocks) { return nblocks < 8 ? nblocks : (nblocks + 7) / 8 * 8; }
__device__ inline int wg_chunk_virtual_block(int b, int grid) { return grid % 8 == 0 ? (b % 8) * (grid / 8) + b / 8 : b; }

// Waves beyond the WK*WR computing ones only fetch.  A wave that issues global -> LDS loads is held at
// each one until the memory pipeline takes it (measured: in proportion to the bytes, some 20-130 cycles
// per 256-byte instruction depending on the access pattern and on how many waves load at once), and a
// computing wave held there feeds no MFMAs: with the fetches in waves of their own, the computing waves
// run from barrier to barrier without a stall, and the fetching waves have a whole unit's time to issue.
constexpr int WGRAD_LOADER_WAVES = 4;

// S1: vertical stride 1 (the slab rows of consecutive pixels are adjacent)
// BIAS (WINO kernels, chunked schedule): the bias derivative of Sec. 4.1's y = x*w + b, dzdb[k] = sum of dzdy[.,.,k,.],
// falls out of this kernel's operands: the second A operand of a step is e0 + e1, the sum of the two rows of dzdy
// that a lane holds, so the waves of the first B tile of the first coefficient tile add it up per filter (one
// vector addition per step) and leave one partial sum per filter and block in `bpart` ([2*block][TK], beside the
// partial tiles); wgrad_bias_final_kernel adds the blocks' sums in block order.
template <int WK, int WR, int MK, int MR, bool S1, int WPE, bool WINO = false, bool BIAS = false>
__global__ __launch_bounds__(64 * (WK * WR + WGRAD_LOADER_WAVES), WPE) void wgrad_sk_kernel(WgradParams P, const float *__restrict__ x,
                                                                     const float *__restrict__ dzdy,
                                                                     const float *__restrict__ rbias,
                                                                     float *__restrict__ out,
                                                                     float *__restrict__ part,
                                                                     float *__restrict__ bpart = nullptr) {
    static_assert(!BIAS || WINO, "the bias derivative is a by-product of the WINO kernels only");
    constexpr int NT = 64 * WK * WR;           // computing threads
    constexpr int NW = WK * WR;
    constexpr int LW = WGRAD_LOADER_WAVES;
    constexpr int NTB = NT + 64 * LW;          // threads of the block
    constexpr int TK = WK * MK * 32;
    constexpr int TR = WR * MR * 32;           // lanes of the B operand per tile: coefficients, or (WINO) column-channel pairs
    constexpr int NX = WINO ? 4 : 1;           // sets of accumulators
    constexpr int TRO = WINO ? 3 * TR : TR;    // coefficients per tile
    static_assert(!WINO || S1, "WINO: stride 1");
    constexpr int NSEGMAX = 2;                 // PCH <= 128
    const int PCH = P.PCH, PCHP = P.PCHP;
    const int NSEG = (PCH + 63) >> 6;
    const int YS = TK * PCHP;
    const int CP = P.CP, SRP = P.SRP;
    const int T = WINO ? P.Wf : P.Hf * P.Wf;   // B lanes per channel
    const int RL = T * P.Cg;                   // B lanes in all

    extern __shared__ __align__(16) float lds[];
    float *ybuf = lds;                                        // [2][TK*PCHP]
    float *xbuf = lds + 2 * YS;                               // [2][XS]
    int *etab = reinterpret_cast<int *>(xbuf + 2 * P.XS);     // [EPT*NT] slab position -> (row | column << 16)

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, l32 = lane & 31;
    const bool loader = wave >= NW;            // scalar: whole waves
    const int wk = wave % WK, wr = (wave / WK) % WR;
    const int HW = P.H * P.W, HoWo = P.Ho * P.Wo;

    int vb;
    long long ub, ue;
    DealSplit deal = {};
    if (P.nchunks > 0) {
        vb = wg_chunk_virtual_block(blockIdx.x, gridDim.x);
        if (vb >= P.nblocks) return;
        const int tile = vb % P.tiles, chunk = vb / P.tiles;
        // weight of the tile's chunks before this one, of this one, and of all of them
        const int G8 = (int)gridDim.x >> 3;
        long long w_before = 0, w_all = 0;
        int w_mine = P.w_later;
        for (int c = 0; c < P.nchunks; ++c) {
            const int v = tile + P.tiles * c;
            const int b = gridDim.x % 8 == 0 ? 8 * (v % G8) + v / G8 : v;      // hardware id of virtual block v
            const int w = b < P.n_first ? P.w_first : P.w_later;
            if (c < chunk) w_before += w;
            if (c == chunk) w_mine = w;
            w_all += w;
        }
        ub = (long long)tile * P.NU + (long long)P.NU * w_before / w_all;
        ue = (long long)tile * P.NU + (long long)P.NU * (w_before + w_mine) / w_all;
        if (P.deal) deal = make_deal(P.NU, P.nchunks, G8, vb);      // one tile: the chunk is vb
    } else {
        vb = sk_virtual_block(blockIdx.x, P.nblocks);
        const long long total = (long long)P.tiles * P.NU;
        ub = sk_begin(total, P.nblocks, vb);
        ue = sk_begin(total, P.nblocks, vb + 1);
    }
    if (ub >= ue) return;

    // ---- per-lane quantities that hold for every unit ------------------------------------------
    // slab position e = col*SRP + r
    for (int e = tid; e < P.EPT * NT; e += NTB) {
        const int col = e / SRP;
        const int r = e - col * SRP;
        const bool ok = col < P.SC && r < P.SR;
        etab[e] = ok ? (r | col << 16) : 0x7fff;       // pitch padding: any row will do, it is never read
    }
    __syncthreads();                                   // the fetching waves read every entry
    // pixel p = ii + TIE*dc of the patch
    int p_ii[NSEGMAX], p_dc[NSEGMAX];
    unsigned p_off[NSEGMAX];
#pragma unroll
    for (int seg = 0; seg < NSEGMAX; ++seg) {
        const int p = seg * 64 + lane;
        const int dc = p / P.TIE;
        const int ii = p - dc * P.TIE;
        const bool ok = ii < P.TI && dc < P.MC;
        p_ii[seg] = ok ? ii : 0x40000000;
        p_dc[seg] = dc;
        p_off[seg] = 4u * (unsigned)(ii + P.Ho * dc);
    }

    // ---- load side -------------------------------------------------------------------------
    // The buffer resources are rebuilt per unit, at the unit's image: offsets then stay inside one image (the
    // host checks that an image of x and of dzdy is under 2^31 bytes), whatever the batch size.
    int l_klim = 0, l_nch = 0;
    int l_xch = 0, l_ych = 0;      // first channel of x / of dzdy that the tile reads
    auto setup_load = [&](int t) {
        const int rt = t % P.RT; t /= P.RT;
        const int kt = t % P.KT;
        const int g = t / P.KT;
        const int r_lo = rt * TR;
        const int r_hi = min(r_lo + TR, RL);
        const int c_lo = r_lo / T;
        l_nch = (r_hi - 1) / T - c_lo + 1;
        l_klim = min(P.Kg - kt * TK, TK);
        l_xch = g * P.Cg + c_lo;
        l_ych = g * P.Kg + kt * TK;
    };
    // LDS byte addresses as 32-bit scalars: no 64-bit pointer arithmetic per load, and pinned to scalar registers
    // here so that none of the per-load additions lands on the vector ALU, where a fetching wave would queue
    // behind the matrix instructions of the computing waves
    const unsigned ybuf_lds = __builtin_amdgcn_readfirstlane(lds_address(ybuf));
    const unsigned xbuf_lds = __builtin_amdgcn_readfirstlane(lds_address(xbuf));
    auto issue_loads = [&](int uu, int b) {
        const unsigned yb = __builtin_amdgcn_readfirstlane(ybuf_lds + (unsigned)(b * YS) * 4u);
        const unsigned xb = __builtin_amdgcn_readfirstlane(xbuf_lds + (unsigned)(b * P.XS) * 4u);
        // unit -> image, patch (all scalar)
        const int per_image = P.RB * P.CC;
        const int n = uu / per_image;
        const int rem = uu - n * per_image;
        const int jc = rem / P.RB, rb = rem - jc * P.RB;
        const int io0 = rb * P.TI, jo0 = jc * P.MC;
        const int rows = min(P.TI, P.Ho - io0), cols = min(P.MC, P.Wo - jo0);
        const buffer_rsrc xrs = make_rsrc(x + ((size_t)n * P.Ctot + l_xch) * HW, 0x7fffffffu);
        const buffer_rsrc yrs = make_rsrc(dzdy + ((size_t)n * P.Ktot + l_ych) * HoWo, 0x7fffffffu);
        // dzdy tile: one wave instruction = 64 pixels of one filter
        const unsigned ybase = 4u * (unsigned)(io0 + P.Ho * jo0);
        for (int seg = 0; seg < NSEG; ++seg) {
            const unsigned yoff = (p_ii[seg] < rows && p_dc[seg] < cols) ? p_off[seg] + ybase : SLAB_INVALID;
            if (seg * 64 + lane < PCH) {
                for (int k = wave - NW; k < l_klim; k += LW)
                    load_to_lds_b32(yb + (unsigned)(k * PCHP + seg * 64) * 4u, yoff, yrs, (unsigned)k * (unsigned)HoWo * 4u);
            }
        }
        // x slab of the tile's channels: rows i0 + r, columns j0 + col of image n
        const int i0 = io0 * P.Sh - P.Pt, j0 = jo0 * P.Sw - P.Pl;
        const int xbase = 4 * (i0 + P.H * j0);
        const int ntot = SRP * P.SC;
        // The fetching waves share the (chunk of 64 positions, channel) pairs.  With at least LW channels every
        // wave walks all chunks and takes every LW-th channel of each, starting one channel further per chunk
        // (equal shares whatever the chunk count); with fewer channels (depthwise-like tiles with large slabs)
        // a wave takes every LW-th chunk with all its channels, so that no wave computes addresses it does not use.
        const bool by_chunk = l_nch < LW;
        const int lw = wave - NW;
        for (int chunk = by_chunk ? lw : 0; chunk * 64 < ntot; chunk += by_chunk ? LW : 1) {
            const int e0 = chunk * 64;
            const int rc = etab[e0 + lane];
            const int r = rc & 0xffff, col = rc >> 16;
            const int rel = 4 * (r + P.H * col);
            const bool ok = (unsigned)(r + i0) < (unsigned)P.H && (unsigned)(col + j0) < (unsigned)P.W;
            const unsigned go = ok ? (unsigned)(rel + xbase) : SLAB_INVALID;
            if (e0 + lane < ntot) {
                for (int d = by_chunk ? 0 : (lw + chunk) % LW; d < l_nch; d += by_chunk ? 1 : LW)
                    load_to_lds_b32(xb + (unsigned)(d * CP + e0) * 4u, go, xrs, (unsigned)d * (unsigned)HW * 4u);
            }
        }
    };

    // ---- compute side ----------------------------------------------------------------------
    int roff[MR];
    int c_rt = 0, c_kt = 0, c_g = 0;
    floatx16 acc[NX][MK][MR];
    float bsum[MK];          // BIAS: this lane's sum of dzdy over the pairs of rows it has held, per filter tile
    bool bias_on = false;    // BIAS: this wave sums (first B tile of the block, first coefficient tile)
    float bias_w = 0.f;      // 1 in those waves, 0 in the others
    auto setup_compute = [&](int t) {
        const int rt = t % P.RT; t /= P.RT;
        const int kt = t % P.KT;
        const int g = t / P.KT;
        c_rt = rt; c_kt = kt; c_g = g;
        bias_on = BIAS && wr == 0 && rt == 0;
        bias_w = bias_on ? 1.f : 0.f;
#pragma unroll
        for (int mk = 0; mk < MK; ++mk) bsum[mk] = 0.f;
        const int r_lo = rt * TR;
        const int c_lo = r_lo / T;
#pragma unroll
        for (int mr = 0; mr < MR; ++mr) {
            const int r = r_lo + (wr * MR + mr) * 32 + l32;
            int o = 0;
            if (r < RL) {
                const int c = r / T;
                const int tap = r - c * T;
                const int fj = WINO ? tap : tap / P.Hf;
                const int fi = WINO ? 0 : tap - fj * P.Hf;
                o = (c - c_lo) * CP + fj * SRP + fi;
            }
            // the upper half-wave takes the odd pixel (WINO: the odd pair of rows) of a step
            roff[mr] = o + half * (WINO ? 2 : P.Sh);
        }
#pragma unroll
        for (int x = 0; x < NX; ++x)
#pragma unroll
            for (int mk = 0; mk < MK; ++mk)
#pragma unroll
                for (int mr = 0; mr < MR; ++mr)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[x][mk][mr][v] = 0.f;
    };
    const int aoff = (wk * MK * 32 + l32) * PCHP + half;
    // all steps of the unit in buffer b: columns of the patch, two pixels per step
    auto compute = [&](int b) {
        if constexpr (WINO) {
            // One step = two pairs of output rows (one per half-wave).  Per filter tile an 8-byte read gives the
            // pair's two rows of dzdy, per B tile two give the four input rows; every index below is in units of
            // 8 bytes (all pitches are even).
            const float2 *y2 = reinterpret_cast<const float2 *>(ybuf);
            const float2 *x2 = reinterpret_cast<const float2 *>(xbuf);
            int ya[MK], xr[MR];
#pragma unroll
            for (int mk = 0; mk < MK; ++mk) ya[mk] = ((b * YS + (wk * MK * 32 + mk * 32 + l32) * PCHP) >> 1) + half;
#pragma unroll
            for (int mr = 0; mr < MR; ++mr) xr[mr] = (b * P.XS + roff[mr]) >> 1;
            const int steps_col = P.TIE >> 2;
            const int xcol = (SRP - P.TIE) >> 1;          // from the end of a column to the start of the next
            float2 e[2][MK], lo[2][MR], hi[2][MR];
            auto fetch = [&](int slot) {
#pragma unroll
                for (int mk = 0; mk < MK; ++mk) { e[slot][mk] = y2[ya[mk]]; ya[mk] += 2; }
#pragma unroll
                for (int mr = 0; mr < MR; ++mr) { lo[slot][mr] = x2[xr[mr]]; hi[slot][mr] = x2[xr[mr] + 1]; xr[mr] += 2; }
            };
            auto step = [&](int slot) {
                float av[4][MK], bv[4][MR];
#pragma unroll
                for (int mk = 0; mk < MK; ++mk) {
                    const float2 q = e[slot][mk];
                    av[0][mk] = q.x; av[1][mk] = q.x + q.y; av[2][mk] = q.x - q.y; av[3][mk] = q.y;
                    if constexpr (BIAS) bsum[mk] = fmaf(bias_w, av[1][mk], bsum[mk]);      // no branch in the MFMA loop
                }
#pragma unroll
                for (int mr = 0; mr < MR; ++mr) {
                    const float2 l = lo[slot][mr], h = hi[slot][mr];
                    bv[0][mr] = l.x - h.x; bv[1][mr] = l.y + h.x; bv[2][mr] = h.x - l.y; bv[3][mr] = l.y - h.y;
                }
#pragma unroll
                for (int x = 0; x < 4; ++x)
#pragma unroll
                    for (int mk = 0; mk < MK; ++mk)
#pragma unroll
                        for (int mr = 0; mr < MR; ++mr)
                            acc[x][mk][mr] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[x][mk], bv[x][mr], acc[x][mk][mr], 0, 0, 0);
            };
            for (int dc = 0; dc < P.MC; ++dc) {
                fetch(0);
                int t = 0;
                for (; t + 2 <= steps_col; t += 2) {
                    fetch(1);
                    step(0);
                    if (t + 2 < steps_col) fetch(0);
                    step(1);
                }
                if (t < steps_col) step(0);
#pragma unroll
                for (int mr = 0; mr < MR; ++mr) xr[mr] += xcol;
            }
            return;
        }
        // running LDS indices (floats) of the lane's operands
        int ya[MK], xr[MR];
#pragma unroll
        for (int mk = 0; mk < MK; ++mk) ya[mk] = b * YS + aoff + mk * 32 * PCHP;
#pragma unroll
        for (int mr = 0; mr < MR; ++mr) xr[mr] = b * P.XS + roff[mr];
        const int steps_col = P.TIE >> 1;
        const int xstep = 2 * P.Sh;                                   // floats between the slab rows of steps t and t+1
        const int xcol = SRP * P.Sw - P.TIE * P.Sh;                   // from the end of a column to the start of the next
        auto mma = [&](const float *a, const float *bq) {
#pragma unroll
            for (int mk = 0; mk < MK; ++mk)
#pragma unroll
                for (int mr = 0; mr < MR; ++mr)
                    acc[0][mk][mr] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[mk], bq[mr], acc[0][mk][mr], 0, 0, 0);
        };
        for (int dc = 0; dc < P.MC; ++dc) {
            int t = 0;
            for (; t + 4 <= steps_col; t += 4) {
                float a[4][MK], bq[4][MR];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
#pragma unroll
                    for (int mk = 0; mk < MK; ++mk) a[j][mk] = ybuf[ya[mk] + 2 * j];
#pragma unroll
                    for (int mr = 0; mr < MR; ++mr)
                        bq[j][mr] = xbuf[xr[mr] + (S1 ? 2 * j : xstep * j)];
                }
#pragma unroll
                for (int mk = 0; mk < MK; ++mk) ya[mk] += 8;
#pragma unroll
                for (int mr = 0; mr < MR; ++mr) xr[mr] += S1 ? 8 : 4 * xstep;
#pragma unroll
                for (int j = 0; j < 4; ++j) mma(a[j], bq[j]);
            }
            for (; t < steps_col; ++t) {
                float a[MK], bq[MR];
#pragma unroll
                for (int mk = 0; mk < MK; ++mk) { a[mk] = ybuf[ya[mk]]; ya[mk] += 2; }
#pragma unroll
                for (int mr = 0; mr < MR; ++mr) { bq[mr] = xbuf[xr[mr]]; xr[mr] += S1 ? 2 : xstep; }
                mma(a, bq);
            }
#pragma unroll
            for (int mr = 0; mr < MR; ++mr) xr[mr] += xcol;
        }
    };
    // lane holds coefficient r (lane&31) of each r tile and 16 filters of each filter tile
    // WINO: the three row taps of the lane's (filter column, channel) pair from the four sums
    auto taps = [&](int mk, int mr, int v, float *w3) {
        const float m1 = acc[NX > 1 ? 1 : 0][mk][mr][v], m2 = acc[NX > 2 ? 2 : 0][mk][mr][v];
        const float hs = 0.5f * (m1 + m2);
        w3[0] = acc[0][mk][mr][v] + hs;
        w3[1] = 0.5f * (m1 - m2);
        w3[2] = hs - acc[NX > 3 ? 3 : 0][mk][mr][v];
    };
    auto store_tile = [&]() {
        const int klim = min(P.Kg - c_kt * TK, TK);
        if constexpr (WINO) {
#pragma unroll
            for (int mr = 0; mr < MR; ++mr) {
                const int rl = c_rt * TR + (wr * MR + mr) * 32 + l32;
                if (rl >= RL) continue;
#pragma unroll
                for (int mk = 0; mk < MK; ++mk)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int kl = (wk * MK + mk) * 32 + (v >> 2) * 8 + half * 4 + (v & 3);
                        if (kl < klim) {
                            float w3[3];
                            taps(mk, mr, v, w3);
                            float *o = out + (size_t)(c_g * P.Kg + c_kt * TK + kl) * P.R + 3 * rl;
#pragma unroll
                            for (int fi = 0; fi < 3; ++fi) {
                                float val = w3[fi] + (rbias ? rbias[3 * rl + fi] : 0.f);
                                if (P.relu) val = fmaxf(val, 0.f);
                                o[fi] = val;
                            }
                        }
                    }
            }
            return;
        }
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
                        if (kl < klim) {
                            float val = acc[0][mk][mr][v] + rb;
                            if (P.relu) val = fmaxf(val, 0.f);
                            out[(size_t)(c_g * P.Kg + c_kt * TK + kl) * P.R + r] = val;
                        }
                    }
            }
        }
    };
    // BIAS: the two half-waves hold different pairs of rows of the same filters
    auto store_bias = [&](int slot) {
        if constexpr (BIAS) {
            if (!bias_on) return;
#pragma unroll
            for (int mk = 0; mk < MK; ++mk) {
                const float v = bsum[mk] + __shfl_xor(bsum[mk], 32);
                if (half == 0) bpart[(size_t)slot * TK + (wk * MK + mk) * 32 + l32] = v;
            }
        }
    };
    // a piece of a shared tile, [filter][coefficient] (WINO: combined into coefficients first, which is linear)
    auto store_partial = [&](int slot) {
        float *dst = part + (size_t)slot * (TK * TRO);
#pragma unroll
        for (int mr = 0; mr < MR; ++mr)
#pragma unroll
            for (int mk = 0; mk < MK; ++mk)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int kloc = (wk * MK + mk) * 32 + (v >> 2) * 8 + half * 4 + (v & 3);
                    const int rl = (wr * MR + mr) * 32 + l32;
                    if constexpr (WINO) {
                        float w3[3];
                        taps(mk, mr, v, w3);
#pragma unroll
                        for (int fi = 0; fi < 3; ++fi) dst[kloc * TRO + 3 * rl + fi] = w3[fi];
                    } else {
                        dst[kloc * TR + rl] = acc[0][mk][mr][v];
                    }
                }
    };

    // ---- the block's range of units --------------------------------------------------------
    const int NU = P.NU;
    int t_c = (int)(ub / NU);
    int uu_c = (int)(ub - (long long)t_c * NU);
    int t_l = t_c, uu_l = uu_c;
    bool first_segment = true;
    auto segment_is_whole = [&](int t, int uu) { return uu == 0 && (long long)(t + 1) * NU <= ue; };
    const int nunits = (int)(ue - ub);
    if (loader) {
        // Fetching wave: unit it+1 goes into the buffer that the computing waves left at the barrier of
        // iteration it; its own loads have landed before it joins the next barrier.  One barrier per unit,
        // the same number as the computing waves pass.
        setup_load(t_l);
        issue_loads(P.deal ? dealt_unit(deal, 0) : uu_l, 0);
        for (int it = 0; it < nunits; ++it) {
            __builtin_amdgcn_s_waitcnt(WAIT_VMCNT0);
            lds_barrier();
            if (it + 1 < nunits) {
                if (P.deal) {
                    issue_loads(dealt_unit(deal, it + 1), (it + 1) & 1);
                } else {
                    if (++uu_l == NU) { uu_l = 0; ++t_l; setup_load(t_l); }
                    issue_loads(uu_l, (it + 1) & 1);
                }
            }
        }
        return;
    }
    bool whole = segment_is_whole(t_c, uu_c);
    setup_compute(t_c);

    for (int it = 0; it < nunits; ++it) {
        lds_barrier();          // unit it is in LDS (the fetching waves waited for it); results stored earlier drain on their own
        const bool more = it + 1 < nunits;
        compute(it & 1);
        const bool last = !more;
        if (uu_c + 1 == NU || last) {
            if (whole) store_tile();
            else store_partial(2 * vb + (first_segment ? 0 : 1));
            store_bias(2 * vb + (first_segment ? 0 : 1));
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

// Sum the pieces of every tile shared between blocks and write the tile.  blockIdx.x = tile, blockIdx.y = a
// slice of the tile's results.  The order of the additions is fixed by the plan: with G = 512 / Q partial sums
// per result (a power of two chosen on the host from the number of pieces), piece i goes to partial sum i mod G
// and the G sums are added as a balanced tree.  A thread handles four consecutive coefficients of one filter
// (one 16-byte load per piece, four pieces in flight); rows and columns of the tile beyond the filters and
// coefficients that exist are skipped, so a layer whose coefficients fill a fraction of a tile reads that
// fraction of every piece.
// CHUNKED: the pieces of tile t are the first slots of blocks t + tiles*i, i < nchunks; else those of the blocks
// whose equal ranges of units overlap the tile.
template <int TK, int TR, bool CHUNKED>
__global__ __launch_bounds__(512) void wgrad_fixup_kernel(WgradParams P, const float *__restrict__ part,
                                                          const float *__restrict__ rbias, float *__restrict__ out,
                                                          int G) {
    const int t = blockIdx.x;
    int npieces, slot0 = 0, b0 = 0;
    if constexpr (CHUNKED) {
        npieces = P.nchunks;
    } else {
        // Block b holds the units [total*b/nblocks, total*(b+1)/nblocks).  The first and the last block with units
        // of this tile follow from two divisions (and at most a step of correction each); one thread finds them.
        __shared__ int found[3];
        if (threadIdx.x == 0) {
            const long long total = (long long)P.tiles * P.NU;
            const long long t_lo = (long long)t * P.NU, t_hi = t_lo + P.NU;
            const SkSplit split = sk_split(total, P.nblocks);
            int first = (int)(t_lo * P.nblocks / total);
            while (first + 1 < P.nblocks && sk_begin(split, first + 1) <= t_lo) ++first;
            while (first > 0 && sk_begin(split, first) > t_lo) --first;
            int last = (int)((t_hi - 1) * P.nblocks / total);
            while (last + 1 < P.nblocks && sk_begin(split, last + 1) < t_hi) ++last;
            while (last > first && sk_begin(split, last) >= t_hi) --last;
            found[0] = first;
            found[1] = last - first + 1;
            // the first block's piece is its first one if it starts with this tile, else its last; the others start inside the tile
            found[2] = 2 * first + (sk_begin(split, first) >= t_lo ? 0 : 1);
        }
        __syncthreads();
        b0 = found[0]; npieces = found[1]; slot0 = found[2];
        if (npieces < 2) return;      // computed by one block alone: already written
    }
    auto slot_of = [&](int i) { return CHUNKED ? 2 * (t + P.tiles * i) : (i == 0 ? slot0 : 2 * (b0 + i)); };
    int tt = t;
    const int rt = tt % P.RT; tt /= P.RT;
    const int kt = tt % P.KT;
    const int g = tt / P.KT;
    const int klim = min(P.Kg - kt * TK, TK);
    const int rlim = min(P.R - rt * TR, TR);           // coefficients of the tile that exist
    const int C4 = (rlim + 3) >> 2;                     // 16-byte words per filter row that hold any of them
    const int nwords = klim * C4;
    const int Q = 512 / G;                              // words per block and pass
    const int q = threadIdx.x % Q, pg = threadIdx.x / Q;
    __shared__ float4 red[512];
    for (int w0 = blockIdx.y * Q; w0 < nwords; w0 += gridDim.y * Q) {
        const int w = w0 + q;
        const bool valid = w < nwords;
        const int kloc = valid ? w / C4 : 0, c4 = valid ? w - kloc * C4 : 0;
        const float *src = part + (size_t)kloc * TR + 4 * c4;
        float4 acc = {0.f, 0.f, 0.f, 0.f};
        if (valid) {
            int i = pg;
            for (; i + 3 * G < npieces; i += 4 * G) {
                const float4 v0 = *reinterpret_cast<const float4 *>(src + (size_t)slot_of(i) * (TK * TR));
                const float4 v1 = *reinterpret_cast<const float4 *>(src + (size_t)slot_of(i + G) * (TK * TR));
                const float4 v2 = *reinterpret_cast<const float4 *>(src + (size_t)slot_of(i + 2 * G) * (TK * TR));
                const float4 v3 = *reinterpret_cast<const float4 *>(src + (size_t)slot_of(i + 3 * G) * (TK * TR));
                acc.x += v0.x; acc.y += v0.y; acc.z += v0.z; acc.w += v0.w;
                acc.x += v1.x; acc.y += v1.y; acc.z += v1.z; acc.w += v1.w;
                acc.x += v2.x; acc.y += v2.y; acc.z += v2.z; acc.w += v2.w;
                acc.x += v3.x; acc.y += v3.y; acc.z += v3.z; acc.w += v3.w;
            }
            for (; i < npieces; i += G) {
                const float4 v = *reinterpret_cast<const float4 *>(src + (size_t)slot_of(i) * (TK * TR));
                acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
            }
        }
        red[pg * Q + q] = acc;
        // balanced tree over the G partial sums: the sums pg and pg + h are added, h = G/2, G/4, ..., 1
        for (int h = G >> 1; h >= 1; h >>= 1) {
            __syncthreads();
            if (pg < h) {
                const float4 a = red[pg * Q + q], c = red[(pg + h) * Q + q];
                red[pg * Q + q] = float4{a.x + c.x, a.y + c.y, a.z + c.z, a.w + c.w};
            }
        }
        __syncthreads();
        if (pg == 0 && valid) {
            const float4 v4 = red[q];
            const float vv[4] = {v4.x, v4.y, v4.z, v4.w};
            float *o = out + (size_t)(g * P.Kg + kt * TK + kloc) * P.R + rt * TR;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int rl = 4 * c4 + j;
                if (rl < rlim) {
                    float v = vv[j];
                    if (rbias) v += rbias[rt * TR + rl];
                    if (P.relu) v = fmaxf(v, 0.f);
                    o[rl] = v;
                }
            }
        }
        __syncthreads();
    }
}

// BIAS: dzdb[k] = the sum over the chunks of the partial sums that the blocks of the first coefficient tile
// (rt = 0) of k's filter tile left in bpart.  One block of 1024 threads per (group, filter tile); thread (k, j) adds
// the chunks i = j, j + NS, ... (NS = 1024 / TK independent streams of loads), the NS sums are then added in order.
template <int TK>
__global__ __launch_bounds__(1024) void wgrad_bias_final_kernel(WgradParams P, const float *__restrict__ bpart,
                                                                float *__restrict__ dzdb) {
    constexpr int NS = 1024 / TK;
    const int kt = blockIdx.x % P.KT, g = blockIdx.x / P.KT;
    const int t0 = P.RT * (kt + P.KT * g);
    const int k = threadIdx.x % TK, j = threadIdx.x / TK;
    __shared__ float red[NS][TK];
    float acc = 0.f;
    for (int i = j; i < P.nchunks; i += NS) acc += bpart[(size_t)(2 * (t0 + P.tiles * i)) * TK + k];
    red[j][k] = acc;
    __syncthreads();
    if (j == 0 && kt * TK + k < P.Kg) {
        float v = red[0][k];
        for (int i = 1; i < NS; ++i) v += red[i][k];
        dzdb[g * P.Kg + kt * TK + k] = v;
    }
}

}  // namespace mcn
