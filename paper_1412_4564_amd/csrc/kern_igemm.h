// Implicit-GEMM convolution on the fp32 matrix cores (v_mfma_f32_32x32x2_f32),
// as a persistent kernel that shares the reduction between blocks ("stream-K").
//
// Computes the sum of Sec. 4.1 of the MatConvNet manual (arXiv 1412.4564),
//   out[io,jo,k,n] = bias[k] + sum_{fi,fj,c} wt(k,c,fi,fj) * in[Sh*io+fi-Pt, Sw*jo+fj-Pl, g*Cg+c, n],
// for one "view" of a convolution.  The forward pass uses it directly; the
// derivative with respect to the input (Sec. 6.1, dz/dX = phi*(dz/dY F^T)) is the
// same kind of sum over dzdy with the filter flipped and the roles of input
// channels and filters exchanged (one such sum per stride phase), and the passes
// of a fully-connected layer are 1x1 views; all of them run here with a
// different weight packing.
//
// Mapping to the GEMM  OUT[k][pixel] = sum_r WT[k][r] * PATCH[r][pixel]:
//  * matrix A (32 filters x 2 reduction elements) comes from a packed copy of the
//    weights, matrix B (2 reduction elements x 32 pixels) from an LDS copy of the
//    input ("slab") -- never from an im2row buffer in HBM.  Lanes run along pixels,
//    which are contiguous in memory (first array index), so slab loads, B reads and
//    the final stores are coalesced.
//  * pixels of one tile: rows are cut into row blocks of TI rows; inside a row
//    block the pixels are numbered q = ii + TI*(jo + Wo*n), i.e. columns of all
//    images are chained, and a tile takes TQ consecutive q.  The slab holds, per
//    channel, every input column/row those pixels read, so filter tap (fi,fj) of
//    pixel q is the slab element at  base(q) + fi + SRP*fj.
//  * reduction: a tile's reduction is cut into NU units of DC channels x TC taps.
//    One unit = NS steps of one MFMA per accumulator; a step consumes either two
//    channels of one tap (pair_mode 0) or two taps of one channel (pair_mode 1).
//  * scheduling: every resident block first computes floor(tiles / nblocks) whole
//    tiles of its own; the (tile, unit) pairs of the left-over tiles are cut into
//    nblocks equal contiguous ranges, so every compute unit gets the same amount of
//    matrix work whatever the number of tiles.  A block that computes a whole tile
//    writes it to `out`; pieces of a tile shared between blocks go to a workspace
//    and are summed in block order by igemm_fixup_kernel (no float atomics: results
//    do not depend on scheduling).
//  * input derivative with a stride: one launch per stride phase, or -- few channels
//    per group -- all phases in one launch, side by side in the filter dimension
//    (IgemmParams::mD).
//  * staging: global -> LDS loads bypass the registers (buffer_load ... lds),
//    double-buffered one unit ahead; padding is produced by the out-of-range rule of
//    buffer loads (reads as zero).
//  * 3x3 filters at stride 1 (template flag WINO): the sum over the three filter rows is evaluated for two
//    output rows at a time with four products instead of six (the minimal-filtering identity F(2,3):
//    with d0..d3 the four input rows that the pair of output rows reads and g0..g2 the filter rows,
//      m0 = (d0-d2) g0,  m1 = (d1+d2) (g0+g1+g2)/2,  m2 = (d2-d1) (g0-g1+g2)/2,  m3 = (d1-d3) g2,
//      y0 = m0 + m1 + m2,  y1 = m1 - m2 - m3).
//    The sum over channels and filter columns is taken inside each m, on the matrix core; a "pixel" of
//    the GEMM is then a pair of output rows, the slab is that of a stride-2 view with four taps per
//    column, the packed weights hold the four row combinations, and there are four sets of
//    accumulators.  Two thirds of the MFMAs for the same result, up to rounding order.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>
#include "fastdiv.h"
#include "streamk.h"

namespace mcn {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned uintx2 __attribute__((ext_vector_type(2)));

#define MCN_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))

constexpr unsigned SLAB_INVALID = 0x80000000u;   // >= any buffer size used here: reads as 0
constexpr int BUFFER_FLAGS = 0x00020000;         // raw buffer, 32-bit elements
constexpr int BUFFER_FLAGS_WORD3 = 0x00020000;
constexpr int WAIT_VMCNT0 = 0x0F70;              // s_waitcnt vmcnt(0) only

// ---- global -> LDS loads that bypass the registers ------------------------------------------
// buffer_load ... lds writes lane l's element at LDS address M0 + 4*l (16*l for the 128-bit
// form); out-of-range lanes write zero; lanes that are switched off write nothing.  They are
// issued through inline assembly so that the compiler's wait-count insertion does not know about
// them (it would otherwise wait for them before unrelated LDS reads and serialise the
// prefetch); the kernels wait for them explicitly with s_waitcnt vmcnt(0) before the barrier
// that publishes the buffer.
typedef int buffer_rsrc __attribute__((ext_vector_type(4)));
__device__ inline buffer_rsrc make_rsrc(const void *base, unsigned bytes) {
    const unsigned long long a = (unsigned long long)base;
    buffer_rsrc r = {(int)(unsigned)a, (int)((a >> 32) & 0xffffu), (int)bytes, BUFFER_FLAGS_WORD3};
    // the resource must live in scalar registers
    r.x = __builtin_amdgcn_readfirstlane(r.x); r.y = __builtin_amdgcn_readfirstlane(r.y);
    r.z = __builtin_amdgcn_readfirstlane(r.z); r.w = __builtin_amdgcn_readfirstlane(r.w);
    return r;
}
__device__ inline unsigned lds_address(const void *p) { return (unsigned)(size_t)MCN_LDS_PTR(p); }
// lds_addr: wave-uniform LDS byte address of lane 0's element.  M0 is saved and restored around the load, so the
// statement leaves no register changed that the compiler may be keeping a value in (the loads are issued by the
// fetching waves, whose scalar instructions cost the computing waves nothing).
__device__ inline void load_to_lds_b32(unsigned lds_addr, unsigned voffset, buffer_rsrc rsrc, unsigned soffset) {
    lds_addr = __builtin_amdgcn_readfirstlane(lds_addr);      // wave-uniform by construction; keeps it in a scalar register
    unsigned saved_m0;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tbuffer_load_dword %2, %3, %4 offen lds\n\ts_mov_b32 m0, %0"
                 : "=&s"(saved_m0) : "s"(lds_addr), "v"(voffset), "s"(rsrc), "s"(soffset) : "memory");
}
__device__ inline void load_to_lds_b128(unsigned lds_addr, unsigned voffset, buffer_rsrc rsrc, unsigned soffset) {
    lds_addr = __builtin_amdgcn_readfirstlane(lds_addr);
    unsigned saved_m0;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tbuffer_load_dwordx4 %2, %3, %4 offen lds\n\ts_mov_b32 m0, %0"
                 : "=&s"(saved_m0) : "s"(lds_addr), "v"(voffset), "s"(rsrc), "s"(soffset) : "memory");
}


// Workgroup barrier that orders LDS traffic only: unlike __syncthreads() it does not wait for
// this wave's outstanding global stores, so a finished tile drains to memory while the next one
// is computed.  Loads into LDS are waited for explicitly (vmcnt) where they are consumed.
__device__ inline void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

struct IgemmParams {
    int H, W, N;        // input plane size, batch
    int Ctot, Cg;       // channels in the input array / per group (reduction depth)
    int Ho, Wo;         // output plane size of this view (rows/columns actually computed)
    int Ktot, Kg, G;    // channels in the output array / per group, groups
    int Hf, Wf, Sh, Sw;
    int Pt, Pl;         // top/left pad (negative = crop)
    int TI, RB;         // rows per row block, number of row blocks
    int Wp;             // columns reserved per image in the chained padded-column index
    int SR, SRP;        // slab rows used / row pitch
    int CP;             // slab channel pitch (floats), a multiple of 64
    int EPT;            // slab elements per thread: ceil(CP / threads)
    int KT, PT;         // filter tiles per group, pixel tiles per row block
    int QN;             // TI*Wo*N: chained pixels per row block
    int DC, TC, NTR;    // channels per unit, taps per unit, tap ranges
    int NU;             // units per tile = ceil(Cg/DC) * NTR
    int NS;             // steps per unit (even)
    int WSZ;            // floats of packed weights per unit: NS*2*TK rounded up to a multiple of 256
    int pair_mode;      // 0: a step pairs two channels, 1: a step pairs two taps
    int tiles;          // G*RB*PT*KT
    int nblocks;        // resident blocks sharing tiles*NU units
    // where output pixel (io, jo) of this view lands in the output array (stride phases of dzdx)
    int OH, OW;         // plane size of the output array
    int oi0, osi, oj0, osj;   // row = oi0 + osi*io, column = oj0 + osj*jo
    unsigned packed_bytes;    // size of the packed weights of this view
    int relu;                 // 1: results are written as max(0, .)  (fused ReLU block, Sec. 4.4 of the manual)
    // Merged stride phases of an input derivative (mD > 0): "filter" kl of a group is channel kl % mD of
    // stride phase kl / mD (phase = pi + osi*pj); its results go to rows i0 + osi*io, columns j0 + osj*jo
    // of that channel, i0 = (pi - mPt) mod osi, j0 = (pj - mPl) mod osj, where they exist.
    int mD, mPt, mPl;
    // Schedule: every block first computes `own` whole tiles of its own (tiles vb*own .. vb*own+own-1); only
    // the tiles left over, own*nblocks .. tiles-1, are cut into equal contiguous ranges of units and shared.
    // own = 0 shares everything.
    int own;
    // Blocks that share the left-over tiles: all of them (nshare = nblocks), or the nshare = nblocks / 2 blocks with
    // the lowest hardware ids.  Of the two blocks resident on a compute unit the one dispatched first (the lower
    // id) gets more of the matrix core and would finish some 10 % earlier on equal work; it takes the left-over
    // units, the other only its own tiles, and half as many partial tiles go through the workspace.
    int nshare;
    // WINO kernels: the view's real number of output rows (Ho, TI, QN, Sh, Hf and osi above then describe pairs of
    // rows: Ho = ceil(wino_Ho / 2), Sh = 2, Hf = 4, osi = twice the row step of the output array); 0 otherwise
    int wino_Ho;
    int wino_pairs;     // WINO: 1 = both rows of a pair go out in one 8-byte store (rows adjacent in memory, every such
                        // address a multiple of 8: output pointer aligned to 8 bytes and an even number of rows per plane)
    Div32 dTI, dWo, dWp, dSRP, dKT, dRB, dPT;   // reciprocals of the fields of these names
};

// Merged phases: channel, and placement of output pixel (0,0), of merged filter kl
struct MergedFilter {
    int c, i0, j0;
};
__device__ __host__ inline MergedFilter merged_filter(const IgemmParams &P, int kl) {
    MergedFilter f;
    const int p = kl / P.mD;
    f.c = kl - p * P.mD;
    const int pj = p / P.osi, pi = p - pj * P.osi;
    f.i0 = ((pi - P.mPt) % P.osi + P.osi) % P.osi;
    f.j0 = ((pj - P.mPl) % P.osj + P.osj) % P.osj;
    return f;
}

// Tile order: filter tiles fastest (they share the slab), then the row blocks of one strip of
// columns (vertically adjacent tiles share the cache lines their halo rows touch), then the
// strips, then the groups.
__device__ inline void decode_tile(const IgemmParams &P, int t, int *kt, int *pt, int *rb, int *g) {
    int q = div32(t, P.dKT);
    *kt = t - q * P.KT; t = q;
    q = div32(t, P.dRB);
    *rb = t - q * P.RB; t = q;
    q = div32(t, P.dPT);
    *pt = t - q * P.PT;
    *g = q;
}

// ---- reduction order of a unit ------------------------------------------------------------
// element (s, h) of tap range tr: local channel cl and tap, or tap = -1 if it is padding
__device__ inline void unit_element(int pair_mode, int DC, int TC, int T, int tr, int s, int h, int *cl, int *tap) {
    int c, t;
    if (pair_mode == 0) {
        const int dp = s / TC;
        c = 2 * dp + h;
        t = tr * TC + (s - dp * TC);
    } else {
        const int hp = TC / 2;
        c = s / hp;
        t = tr * TC + 2 * (s - c * hp) + h;
    }
    if (c >= DC || t >= T || t >= (tr + 1) * TC) t = -1;
    *cl = c;
    *tap = t;
}

// ---- weight packing ------------------------------------------------------------------
// packed[g][kt][unit][s][h][kk] = wt(k = kt*TK+kk, c = cg*DC + cl, tap), 0 where padded; one unit
// takes WSZ floats.
// mode 0 (forward):        wt(k,c,fi,fj) = w[fi, fj, c, g*Kg + k]
// mode 1 (input derivative, Kg = D', Cg = K/G; one call per stride phase (pi, pj)):
//     view tap (ti,tj) is filter tap fi = pi + Sh*(Hfv-1-ti), fj = pj + Sw*(Wfv-1-tj):
//                          wt(k,c,ti,tj) = w[fi, fj, k, g*Cg + c]
// mode 2 (1x1 view whose weights are a transposed matrix, used for the filter derivative of a
//     fully-connected layer):  wt(k,c) = w[k + ldk*c]
// mode 3 (input derivative, all stride phases merged; Kg = D'*Sh*Sw "filters", see IgemmParams::mD):
//     filter k = channel k % mD of phase (pi, pj); along the rows the phase has A = ceil((Hf-pi)/Sh)
//     taps fi = pi + Sh*a, a = 0..A-1, which meet dzdy row m + b0 - a for output row i0 + Sh*m
//     (b0 = (i0 + Pt - pi)/Sh).  All phases share one window of the view: view tap ti stands for
//     t = Hfv-1-ti, dzdy row m + B0 - t, so a = t - (B0 - b0); taps a phase does not have are zero.
struct PackParams {
    int Hf, Wf;            // taps of the view
    int HfA, WfA, DfA;     // shape of the caller's filter array (modes 0, 1)
    int Kg, Cg, G, KT, NU, NTR, NS, WSZ, TK, DC, TC, pair_mode, mode;
    int Sh, Sw, pi, pj;    // mode 1
    int ldk;               // mode 2
    int mD, Pt, Pl, B0i, B0j;   // mode 3: channels per phase, pads of the convolution, largest b0 per direction
    int planes;            // bf16 packing: 1 = values rounded to bf16, 2 = hi and lo planes (kern_igemm_bf16.h)
    int MK;                // fp32 packing: 32-filter blocks per computing wave (see packed_filter_slot)
    int wino;              // modes 0, 1 with a 3x3 filter: Hf = 4 and view tap (ti, tj) is row combination ti of column tj
                           // (packed by igemm_pack_wino_kernel)
    int total;
};

// Where filter kk of a tile sits among the TK values of one reduction element of a step.  A wave of the fp32
// kernels owns MK blocks of 32 filters (filter = (wave*MK + block)*32 + lane).  With two blocks per wave a lane's
// two values are stored side by side, so they come with ONE 8-byte LDS read whose offset is an immediate of the
// instruction (16 bits: any step of the unit); as two 4-byte values 128 bytes apart they came with a two-address
// read, whose 8-bit offsets the compiler had to rebase with a vector addition every other step.
__device__ __host__ inline int packed_filter_slot(int kk, int MK) {
    if (MK != 2) return kk;
    return (((kk >> 6) << 5) + (kk & 31)) * 2 + ((kk >> 5) & 1);
}

// one direction of mode 3: filter tap of view tap ti for phase pi, or -1
__device__ __host__ inline int merged_tap(int ti, int Hfv, int HfA, int S, int Pt, int B0, int pi) {
    const int A = pi < HfA ? (HfA - pi + S - 1) / S : 0;
    const int i0 = ((pi - Pt) % S + S) % S;
    const int b0 = (i0 + Pt - pi) / S;
    const int a = (Hfv - 1 - ti) - (B0 - b0);
    return (a >= 0 && a < A) ? pi + S * a : -1;
}

__global__ __launch_bounds__(256) void igemm_pack_weights_kernel(const float *__restrict__ w, float *__restrict__ packed,
                                                                 PackParams Q) {
    int p = blockIdx.x * 256 + threadIdx.x;
    if (p >= Q.total) return;
    int t = p / Q.WSZ;
    int within = p - t * Q.WSZ;
    if (within >= Q.NS * 2 * Q.TK) { packed[p] = 0.f; return; }     // pitch padding
    const int kk = within % Q.TK; within /= Q.TK;
    const int h = within & 1;
    const int s = within >> 1;
    p += packed_filter_slot(kk, Q.MK) - kk;         // pitch padding aside, the threads of a step permute its slots
    const int uu = t % Q.NU; t /= Q.NU;
    const int kt = t % Q.KT;
    const int g = t / Q.KT;
    const int cg = uu / Q.NTR, tr = uu - cg * Q.NTR;
    int cl, tap;
    unit_element(Q.pair_mode, Q.DC, Q.TC, Q.Hf * Q.Wf, tr, s, h, &cl, &tap);
    const int k = kt * Q.TK + kk;
    const int c = cg * Q.DC + cl;
    float v = 0.f;
    if (tap >= 0 && k < Q.Kg && c < Q.Cg) {
        const int ti = tap % Q.Hf, tj = tap / Q.Hf;
        if (Q.mode == 0) {
            v = w[ti + Q.HfA * (tj + Q.WfA * (c + (size_t)Q.DfA * (g * Q.Kg + k)))];
        } else if (Q.mode == 1) {
            const int fi = Q.pi + Q.Sh * (Q.Hf - 1 - ti), fj = Q.pj + Q.Sw * (Q.Wf - 1 - tj);
            v = w[fi + Q.HfA * (fj + Q.WfA * (k + (size_t)Q.DfA * (g * Q.Cg + c)))];
        } else if (Q.mode == 2) {
            v = w[k + (size_t)Q.ldk * c];
        } else {
            const int ph = k / Q.mD, cch = k - ph * Q.mD;
            const int pj = ph / Q.Sh, pi = ph - pj * Q.Sh;
            const int fi = merged_tap(ti, Q.Hf, Q.HfA, Q.Sh, Q.Pt, Q.B0i, pi);
            const int fj = merged_tap(tj, Q.Wf, Q.WfA, Q.Sw, Q.Pl, Q.B0j, pj);
            if (fi >= 0 && fj >= 0) v = w[fi + Q.HfA * (fj + Q.WfA * (cch + (size_t)Q.DfA * (g * Q.Cg + c)))];
        }
    }
    packed[p] = v;
}

// The packing for the WINO kernels (PackParams::wino, modes 0 and 1; same layout), four results per thread: a
// thread reads the three row taps of one (filter, channel, filter column) once and writes their four combinations
//   g0,  (g0+g1+g2)/2,  (g0-g1+g2)/2,  g2      (input derivative: of the flipped filter).
// One unit takes exactly NS*2*TK floats (no pitch padding: NS = 48).  Thread index: kk fastest, then h, fj, channel pair, unit, filter tile, group.
__global__ __launch_bounds__(256) void igemm_pack_wino_kernel(const float *__restrict__ w, float *__restrict__ packed,
                                                              PackParams Q) {
    int p = blockIdx.x * 256 + threadIdx.x;
    if (p >= Q.total / 4) return;
    const int kk = p % Q.TK; p /= Q.TK;
    const int h = p & 1; p >>= 1;
    const int fj = p % 3; p /= 3;
    const int dp = p % (Q.DC / 2); p /= (Q.DC / 2);
    const int uu = p % Q.NU; p /= Q.NU;
    const int kt = p % Q.KT;
    const int g = p / Q.KT;
    const int k = kt * Q.TK + kk;
    const int c = uu * Q.DC + 2 * dp + h;
    float g0 = 0.f, g1 = 0.f, g2 = 0.f;
    if (k < Q.Kg && c < Q.Cg) {
        const float *src = Q.mode == 0 ? w + 3 * (fj + 3 * (c + (size_t)Q.DfA * (g * Q.Kg + k)))
                                       : w + 3 * ((2 - fj) + 3 * (k + (size_t)Q.DfA * (g * Q.Cg + c)));
        g0 = src[0]; g1 = src[1]; g2 = src[2];
        if (Q.mode != 0) { const float t = g0; g0 = g2; g2 = t; }      // input derivative: the flipped filter
    }
    float *dst = packed + ((size_t)((g * Q.KT + kt) * Q.NU + uu) * Q.NS + (size_t)(dp * 3 + fj) * 4) * 2 * Q.TK + h * Q.TK + packed_filter_slot(kk, Q.MK);
    dst[0] = g0;
    dst[2 * Q.TK] = 0.5f * (g0 + g1 + g2);
    dst[4 * Q.TK] = 0.5f * (g0 - g1 + g2);
    dst[6 * Q.TK] = g2;
}

// ---- main kernel -----------------------------------------------------------------------
// WK x WP waves; each wave owns MK x MP tiles of 32 filters x 32 pixels.
// HF, WF > 0: filter size and DCF channels per unit known at compile time (pair_mode 0, one tap
// range, fully unrolled); HF = 0: everything read from the parameters, offsets from a table.
// WPE: waves per SIMD the register allocation must allow.
// LW: that many more waves only fetch.  A wave that issues global -> LDS loads is held at each one until
// the memory pipeline takes it, and a computing wave held there feeds no MFMAs; fetching waves have a whole
// unit's time to issue, and the computing waves run from barrier to barrier.
// WINO: two output rows per GEMM pixel, four row combinations per filter column (HF = 4, WF = 3; see the top).
template <int WK, int WP, int MK, int MP, int HF, int WF, int DCF, int WPE, int LW, bool WINO = false>
__global__ __launch_bounds__(64 * (WK * WP + LW), WPE) void igemm_sk_kernel(IgemmParams P, const float *__restrict__ in,
                                                                     const float *__restrict__ wpk,
                                                                     const float *__restrict__ bias,
                                                                     float *__restrict__ out,
                                                                     float *__restrict__ part) {
    constexpr int NT = 64 * WK * WP;               // computing threads
    constexpr int NTB = NT + 64 * LW;              // threads of the block
    static_assert(LW > 0, "the computing waves do not fetch");
    constexpr int NL = 64 * LW;                    // fetching threads
    constexpr int NLW = LW;                        // fetching waves
    constexpr int TK = WK * MK * 32;
    constexpr int TQ = WP * MP * 32;
    constexpr bool FIXED = HF > 0;
    constexpr int NX = WINO ? 4 : 1;               // sets of accumulators
    static_assert(!WINO || (HF == 4 && WF == 3 && DCF % 4 == 0), "WINO: four row combinations of a 3x3 filter");
    static_assert(NLW * 64 >= TK, "the fetching waves stage one bias value per lane");
    const int DC = FIXED ? DCF : P.DC;
    const int NS = FIXED ? (DCF / 2) * HF * WF : P.NS;
    const int NU = P.NU;
    const int WSZ = FIXED ? (((DCF / 2) * HF * WF * 2 * TK + 255) & ~255) : P.WSZ;   // floats of packed weights per unit
    const int CP = P.CP, SRP = P.SRP;
    const int XSZ = DC * CP;

    extern __shared__ __align__(16) float lds[];
    float *wbuf = lds;                                   // [2][WSZ]
    float *xbuf = lds + 2 * WSZ;                         // [2][DC*CP]
    int *gtab = reinterpret_cast<int *>(xbuf + 2 * XSZ); // [EPT][NL]: entry (s, t) is private to fetching thread t
    float *blds = reinterpret_cast<float *>(gtab + P.EPT * NL);   // [2][TK] bias of the tile, slots used in turn
    int *otab = reinterpret_cast<int *>(blds + 2 * TK);           // table mode: [NTR][NS][2] slab offsets

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int half = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wk = wave % WK, wp = (wave / WK) % WP;
    const bool loader = wave >= WK * WP;                    // whole waves
    const int ltid = tid - NT;                              // index among the fetching threads
    const int lwave = wave - WK * WP;
    const int HW = P.H * P.W;
    const int OHW = P.OH * P.OW;

    const int vb = sk_virtual_block(blockIdx.x, P.nblocks);
    const int tile_s0 = P.own * P.nblocks;                          // first shared tile
    const long long total = (long long)(P.tiles - tile_s0) * NU;    // units of the shared tiles
    const int rank = sk_share_rank(P.nblocks, P.nshare, vb);
    const long long ub = rank < 0 ? 0 : sk_begin(total, P.nshare, rank), ue = rank < 0 ? 0 : sk_begin(total, P.nshare, rank + 1);
    const int n_own = P.own * NU;                                    // units of this block's own tiles
    const int nunits = n_own + (int)(ue - ub);
    if (nunits == 0) return;

    if constexpr (!FIXED) {
        const int T = P.Hf * P.Wf;
        for (int idx = tid; idx < P.NTR * NS * 2; idx += NTB) {
            const int h = idx & 1;
            const int s = (idx >> 1) % NS;
            const int tr = (idx >> 1) / NS;
            int cl, tap;
            unit_element(P.pair_mode, DC, P.TC, T, tr, s, h, &cl, &tap);
            otab[idx] = tap >= 0 ? cl * CP + (tap / P.Hf) * SRP + tap % P.Hf : 0;
        }
    }

    const buffer_rsrc wrs = make_rsrc(wpk, P.packed_bytes);
    const buffer_rsrc brs = make_rsrc(bias, bias ? (unsigned)P.Ktot * 4u : 0u);
    const buffer_rsrc zrs = make_rsrc(in, 0);   // reads as zero
    const unsigned lane16 = (unsigned)lane * 16u;

    // ---- load side: tile whose units are being fetched ------------------------------------
    buffer_rsrc xrs = wrs;
    unsigned wtile_off = 0;        // byte offset of the tile's packed weights
    int l_kt = 0, l_g = 0;
    int l_seq = -1, c_seq = -1;    // how many tiles the load / the compute side has started: picks the bias slot
    auto setup_load = [&](int t) {
        ++l_seq;
        int kt, pt, rb, g;
        decode_tile(P, t, &kt, &pt, &rb, &g);
        const int q0 = pt * TQ;
        const int c_first = div32(q0, P.dTI);
        const int n_first = div32(c_first, P.dWo);
        const int u0 = (c_first - n_first * P.Wo) * P.Sw;   // chained column of the slab's first column
        const int row0 = rb * P.TI * P.Sh - P.Pt;           // input row of slab row 0
        const size_t in_base = ((size_t)n_first * P.Ctot + (size_t)g * P.Cg) * HW;
        size_t in_left = ((size_t)P.N * P.Ctot * HW - in_base) * 4;
        if (in_left > 0x7fffffffull) in_left = 0x7fffffffull;
        xrs = make_rsrc(in + in_base, (unsigned)in_left);
        wtile_off = (unsigned)((size_t)(g * P.KT + kt) * NU * WSZ * 4);
        l_kt = kt; l_g = g;
        for (int s = 0; s < P.EPT; ++s) {
            const int e = ltid + NL * s;
            const int col = div32(e, P.dSRP);
            const int r = e - col * SRP;
            const int U = u0 + col;
            const int ni = div32(U, P.dWp);          // image relative to n_first
            const int j = U - ni * P.Wp - P.Pl;
            const int i = row0 + r;
            const bool ok = e < CP && r < P.SR && i >= 0 && i < P.H && j >= 0 && j < P.W && (n_first + ni) < P.N;
            gtab[s * NL + ltid] = ok ? (int)(4u * (unsigned)(i + P.H * j + ni * P.Ctot * HW)) : (int)SLAB_INVALID;
        }
    };
    // LDS byte addresses as 32-bit scalars: arithmetic on generic pointers would cost every load a 64-bit
    // addition and a null check.  The per-unit bases are pinned to scalar registers: an addition that lands on
    // the vector ALU makes a fetching wave queue behind the matrix instructions of the computing waves.
    const unsigned wbuf_lds = __builtin_amdgcn_readfirstlane(lds_address(wbuf));
    const unsigned xbuf_lds = __builtin_amdgcn_readfirstlane(lds_address(xbuf));
    // fetch unit uu of the load-side tile into buffer b
    auto issue_loads = [&](int uu, int b) {
        const unsigned wb = __builtin_amdgcn_readfirstlane(wbuf_lds + (unsigned)(b * WSZ) * 4u);
        const unsigned xb = __builtin_amdgcn_readfirstlane(xbuf_lds + (unsigned)(b * XSZ + lwave * 64) * 4u);    // this wave's first element
        const unsigned woff = wtile_off + (unsigned)uu * (unsigned)WSZ * 4u;
        for (int e0 = lwave * 256; e0 < WSZ; e0 += NLW * 256)     // one wave instruction = 256 floats, 16 bytes per lane
            load_to_lds_b128(wb + (unsigned)e0 * 4u, lane16, wrs, woff + (unsigned)e0 * 4u);
        if (bias && uu == 0 && lwave * 64 < TK) {
            // the tile's bias: start value of the accumulators of a tile this block owns entirely
            const int kl = l_kt * TK + lwave * 64 + lane;
            const int bidx = P.mD ? l_g * P.mD + kl % P.mD : l_g * P.Kg + kl;
            if (lwave * 64 + lane < TK)
                load_to_lds_b32(lds_address(blds + (l_seq & 1) * TK + lwave * 64),
                                kl < P.Kg ? (unsigned)bidx * 4u : SLAB_INVALID, brs, 0);
        }
        const int cg = (FIXED || P.NTR == 1) ? uu : uu / P.NTR;
        const int c0 = cg * DC;
        // up to four table entries per wait: a slab of one or two channels with many elements per thread would
        // otherwise pay one LDS round trip per load, and the fetching waves would set the pace of the block
        const int ept = min(P.EPT, (CP - lwave * 64 + NL - 1) / NL);     // rows of the table with elements of this wave
        auto batch = [&](auto count, int s) {
            constexpr int Q = decltype(count)::value;
            unsigned go[Q];
#pragma unroll
            for (int q = 0; q < Q; ++q) go[q] = (unsigned)gtab[(s + q) * NL + ltid];
            for (int d = 0; d < DC; ++d) {
                const int c = c0 + d;
                // channels past the group's last one read as zero (their weights are zero too)
                const buffer_rsrc rs = ((FIXED && !WINO) || c < P.Cg) ? xrs : zrs;
                const unsigned soff = (unsigned)c * (unsigned)HW * 4u;
#pragma unroll
                for (int q = 0; q < Q; ++q)
                    load_to_lds_b32(xb + (unsigned)(d * CP + NL * (s + q)) * 4u, go[q], rs, soff);
            }
        };
        int s = 0;
        for (; s + 4 <= ept; s += 4) batch(std::integral_constant<int, 4>{}, s);
        if (ept - s == 3) { batch(std::integral_constant<int, 3>{}, s); s += 3; }
        for (; s < ept; ++s) batch(std::integral_constant<int, 1>{}, s);   // one or two rows: all channels of a row in turn
    };

    // ---- compute side: tile whose accumulators are live -----------------------------------
    int bbase[MP];   // slab offset (floats) of the pixel's window origin (+ channel half when FIXED)
    unsigned ooff[MP];   // byte offset of the lane's first result of the tile relative to the tile's output
                         // window (filter k0 + 4*half of image n_first), or SLAB_INVALID
    unsigned ooff1[MP];  // WINO: the same for the second row of the pair, SLAB_INVALID if the view has no such row
    bool last_row[MP], last_col[MP];   // merged phases: the pixel is in the view's last row / column
    __amdgpu_buffer_rsrc_t ors = __builtin_amdgcn_make_buffer_rsrc((void *)out, 0, 0, BUFFER_FLAGS);   // the tile's output window
    int c_kt = 0, c_g = 0;
    bool need_init = true;
    floatx16 acc[NX][MK][MP];
    auto setup_compute = [&](int t) {
        ++c_seq;
        int kt, pt, rb, g;
        decode_tile(P, t, &kt, &pt, &rb, &g);
        c_kt = kt; c_g = g;
        const int q0 = pt * TQ;
        const int qend = min(q0 + TQ, P.QN);
        const int c_first = div32(q0, P.dTI);
        const int n_first = div32(c_first, P.dWo);
        const int u0 = (c_first - n_first * P.Wo) * P.Sw;
#pragma unroll
        for (int mp = 0; mp < MP; ++mp) {
            const int q = q0 + (wp * MP + mp) * 32 + (lane & 31);
            const int c = div32(q, P.dTI);
            const int ii = q - c * P.TI;
            const int n = div32(c, P.dWo);
            const int jo = c - n * P.Wo;
            const int io = rb * P.TI + ii;
            const bool ok = q < qend && io < P.Ho;
            const int ucol = jo * P.Sw + (n - n_first) * P.Wp - u0;
            bbase[mp] = (ok ? ii * P.Sh + SRP * ucol : 0) + (FIXED ? half * CP : 0);
            ooff[mp] = ok ? 4u * (unsigned)((P.oi0 + P.osi * io) + P.OH * (P.oj0 + P.osj * jo) +
                                            OHW * (P.Ktot * (n - n_first) + (P.mD ? 0 : 4 * half)))
                          : SLAB_INVALID;
            last_row[mp] = io == P.Ho - 1;
            last_col[mp] = jo == P.Wo - 1;
            if constexpr (WINO)
                ooff1[mp] = ok && 2 * io + 1 < P.wino_Ho ? ooff[mp] + 4u * (unsigned)(P.osi >> 1) : SLAB_INVALID;
        }
        (void)ooff1;
        const size_t out_base = (size_t)n_first * P.Ktot * OHW;
        size_t out_left = ((size_t)P.N * P.Ktot * OHW - out_base) * 4;
        if (out_left > 0x7fffffffull) out_left = 0x7fffffffull;
        ors = __builtin_amdgcn_make_buffer_rsrc((void *)(out + out_base), 0, (int)out_left, BUFFER_FLAGS);
        need_init = true;
    };
    // start value of the accumulators: the bias for a tile this block owns entirely (staged in LDS with the
    // tile's first unit), zero for a piece of a shared tile (the fix-up pass adds the bias)
    auto init_acc = [&](bool with_bias) {
        const float *bl = blds + (c_seq & 1) * TK;
#pragma unroll
        for (int mk = 0; mk < MK; ++mk)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int kloc = (wk * MK + mk) * 32 + (v >> 2) * 8 + half * 4 + (v & 3);
                const float bv = with_bias ? bl[kloc] : 0.f;
#pragma unroll
                for (int mp = 0; mp < MP; ++mp) {
                    acc[0][mk][mp][v] = bv;
                    if constexpr (WINO) {
                        // y0 = m0 + m1 + m2, y1 = m1 - m2 - m3: the bias enters both rows through m0 and -m3
                        acc[1][mk][mp][v] = 0.f; acc[2][mk][mp][v] = 0.f; acc[3][mk][mp][v] = -bv;
                    }
                }
            }
    };
    // the lane's first weight of a step (packed_filter_slot: with MK == 2 its two values are adjacent)
    const int aoff = half * TK + (MK == 2 ? (wk * 32 + (lane & 31)) * 2 : wk * MK * 32 + (lane & 31));
    auto read_a = [&](float *a, const float *wstep) {         // wstep: wl + step * 2 * TK
        if constexpr (MK == 2) {
            const float2 v = *reinterpret_cast<const float2 *>(wstep);
            a[0] = v.x; a[1] = v.y;
        } else {
#pragma unroll
            for (int mk = 0; mk < MK; ++mk) a[mk] = wstep[mk * 32];
        }
    };
    // steps [part*NS/2, (part+1)*NS/2) of unit uu, operands in buffer b
    auto compute = [&](auto PART, int uu, int b) {
        constexpr int part = decltype(PART)::value;
        const float *wl = wbuf + b * WSZ + aoff;
        const float *xl = xbuf + b * XSZ;
        if constexpr (WINO) {
            // One macro-step per (channel pair, filter column): the four input rows of the lane's pair of
            // output rows come as two 8-byte reads (every term of the address is even), are combined
            // into the four B operands, and meet the four row combinations of the weights.  Rows of the
            // next macro-step and the weights of the next step are read ahead of the MFMAs.
            constexpr int NM = (DCF / 2) * 3;
            constexpr int M0 = part * (NM / 2), M1 = part ? NM : NM / 2;
            const float2 *xl2 = reinterpret_cast<const float2 *>(xl);
            const int CP2 = CP, SRP2 = SRP >> 1;          // pitches of a channel pair and of a column, in float2
            float2 d[2][MP][2];
            float a[2][MK];
            const float2 *xq[MP];                          // the lane's window origin: one vector addition per macro-step
#pragma unroll
            for (int mp = 0; mp < MP; ++mp) xq[mp] = xl2 + (bbase[mp] >> 1);
            auto fetch_d = [&](int m, int slot) {
                const int dp = m / 3, fj = m % 3;
                const int o = dp * CP2 + fj * SRP2;
#pragma unroll
                for (int mp = 0; mp < MP; ++mp) {
                    d[slot][mp][0] = xq[mp][o];
                    d[slot][mp][1] = xq[mp][o + 1];
                }
            };
            auto fetch_a = [&](int st, int slot) {
                read_a(a[slot], wl + st * 2 * TK);
            };
            fetch_d(M0, M0 & 1);
            fetch_a(M0 * 4, 0);
#pragma unroll
            for (int m = M0; m < M1; ++m) {
                if (m + 1 < M1) fetch_d(m + 1, (m + 1) & 1);
                float bv[MP][4];
#pragma unroll
                for (int mp = 0; mp < MP; ++mp) {
                    const float2 lo = d[m & 1][mp][0], hi = d[m & 1][mp][1];
                    bv[mp][0] = lo.x - hi.x;
                    bv[mp][1] = lo.y + hi.x;
                    bv[mp][2] = hi.x - lo.y;
                    bv[mp][3] = lo.y - hi.y;
                }
#pragma unroll
                for (int xi = 0; xi < 4; ++xi) {
                    const int st = m * 4 + xi;
                    if (st + 1 < M1 * 4) fetch_a(st + 1, (st + 1) & 1);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int mk = 0; mk < MK; ++mk)
#pragma unroll
                        for (int mp = 0; mp < MP; ++mp)
                            acc[xi][mk][mp] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[st & 1][mk], bv[mp][xi], acc[xi][mk][mp], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        } else if constexpr (FIXED) {
            // the (channel pair, tap) steps of a unit form one flat, fully unrolled list; the LDS
            // reads of step s+1 are issued before the MFMAs of step s.
            constexpr int TT = HF * WF;
            constexpr int NSTEP = (DCF / 2) * TT;
            constexpr int S0 = part * (NSTEP / 2), S1 = part ? NSTEP : NSTEP / 2;
            float a[2][MK], bb[2][MP];
            auto fetch = [&](int s, int slot) {
                const int dp = s / TT, tap = s % TT;
                const int fj = tap / HF, fi = tap % HF;
                read_a(a[slot], wl + s * 2 * TK);
#pragma unroll
                for (int mp = 0; mp < MP; ++mp) bb[slot][mp] = xl[bbase[mp] + dp * 2 * CP + fj * SRP + fi];
            };
            fetch(S0, S0 & 1);
#pragma unroll
            for (int s = S0; s < S1; ++s) {
                if (s + 1 < S1) fetch(s + 1, (s + 1) & 1);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int mk = 0; mk < MK; ++mk)
#pragma unroll
                    for (int mp = 0; mp < MP; ++mp)
                        acc[0][mk][mp] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[s & 1][mk], bb[s & 1][mp], acc[0][mk][mp], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
            const int tr = P.NTR == 1 ? 0 : uu % P.NTR;
            const int *ot = otab + tr * NS * 2 + half;
            const int mid = (NS >> 2) << 1;                 // even
            const int s0 = part ? mid : 0, s1 = part ? NS : mid;
            if (s0 >= s1) return;
            float a0[MK], b0[MP], a1[MK], b1[MP];
            int o0 = ot[2 * s0], o1 = ot[2 * s0 + 2];
            auto fetch = [&](float *a, float *bq, int s, int o) {
                read_a(a, wl + s * 2 * TK);
#pragma unroll
                for (int mp = 0; mp < MP; ++mp) bq[mp] = xl[bbase[mp] + o];
            };
            auto mma = [&](const float *a, const float *bq) {
#pragma unroll
                for (int mk = 0; mk < MK; ++mk)
#pragma unroll
                    for (int mp = 0; mp < MP; ++mp)
                        acc[0][mk][mp] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[mk], bq[mp], acc[0][mk][mp], 0, 0, 0);
            };
            fetch(a0, b0, s0, o0);
            for (int s = s0; s < s1; s += 2) {
                const int o0n = ot[2 * min(s + 2, NS - 1)];
                const int o1n = ot[2 * min(s + 3, NS - 1)];
                fetch(a1, b1, s + 1, o1);
                __builtin_amdgcn_sched_barrier(0);
                mma(a0, b0);
                __builtin_amdgcn_sched_barrier(0);
                // no branch here (the last pass fetches a step again, for nothing): with one the compiler makes the
                // products below wait for these reads too, and the wave sits out an LDS round trip every two steps
                fetch(a0, b0, min(s + 2, s1 - 1), o0n);
                __builtin_amdgcn_sched_barrier(0);
                mma(a1, b1);
                __builtin_amdgcn_sched_barrier(0);
                o0 = o0n; o1 = o1n;
            }
            (void)o0;
        }
    };
    // lane holds pixel (lane&31) of each pixel tile and 16 filters of each filter tile
    // Buffer stores: the filter part of the address is a scalar offset, pixels that do not exist
    // carry an out-of-range offset and are dropped by the hardware, so no per-store vector arithmetic.
    // (No vector arithmetic per store on the usual path: every vector instruction here is issued between the
    // MFMAs of the block that shares the compute unit.)
    auto store_tile_as = [&](auto RELU) {
        constexpr bool relu = decltype(RELU)::value;
        const bool pairs = WINO && P.wino_pairs, odd_rows = WINO && (P.wino_Ho & 1);     // block-wide
        (void)pairs; (void)odd_rows;
        unsigned olow[MP];      // offsets for a store of which only the lower half-wave's filter exists
#pragma unroll
        for (int mp = 0; mp < MP; ++mp) olow[mp] = half == 0 ? ooff[mp] : SLAB_INVALID;
#pragma unroll
        for (int mk = 0; mk < MK; ++mk) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int kl0 = c_kt * TK + (wk * MK + mk) * 32 + (v >> 2) * 8 + (v & 3);   // filter of the lower half-wave
                const int left = P.Kg - kl0;
                if (left <= 0) continue;
                const unsigned soff = (unsigned)(c_g * P.Kg + kl0) * (unsigned)OHW * 4u;
                // the upper half-wave holds filter kl0 + 4
                if constexpr (WINO) {
#pragma unroll
                    for (int mp = 0; mp < MP; ++mp) {
                        const float m1 = acc[1][mk][mp][v], m2 = acc[2][mk][mp][v];
                        float y0 = acc[0][mk][mp][v] + m1 + m2, y1 = m1 - m2 - acc[3][mk][mp][v];
                        if (relu) { y0 = fmaxf(y0, 0.f); y1 = fmaxf(y1, 0.f); }
                        const bool both = left > 4 || half == 0;
                        if (pairs) {
                            // both rows in one store; a pair without a second row (odd number of rows) goes alone
                            const bool two_rows = ooff1[mp] != SLAB_INVALID;
                            uintx2 yy;
                            yy.x = __float_as_uint(y0); yy.y = __float_as_uint(y1);
                            __builtin_amdgcn_raw_buffer_store_b64(yy, ors, both && two_rows ? ooff[mp] : SLAB_INVALID, soff, 0);
                            if (odd_rows)
                                __builtin_amdgcn_raw_buffer_store_b32(yy.x, ors, both && !two_rows ? ooff[mp] : SLAB_INVALID, soff, 0);
                        } else {
                            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(y0), ors, both ? ooff[mp] : SLAB_INVALID, soff, 0);
                            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(y1), ors, both ? ooff1[mp] : SLAB_INVALID, soff, 0);
                        }
                    }
                } else if (left > 4) {
#pragma unroll
                    for (int mp = 0; mp < MP; ++mp) {
                        const float val = relu ? fmaxf(acc[0][mk][mp][v], 0.f) : acc[0][mk][mp][v];
                        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(val), ors, ooff[mp], soff, 0);
                    }
                } else {
#pragma unroll
                    for (int mp = 0; mp < MP; ++mp) {
                        const float val = relu ? fmaxf(acc[0][mk][mp][v], 0.f) : acc[0][mk][mp][v];
                        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(val), ors, olow[mp], soff, 0);
                    }
                }
            }
        }
    };
    auto store_tile = [&]() {
        if (P.relu) store_tile_as(std::true_type{});
        else store_tile_as(std::false_type{});
    };
    // Merged phases: the two half-waves hold filters of different phases, so the filter part of the address
    // and the "does this pixel exist in this phase" test are per half-wave.
    auto store_tile_merged = [&]() {
#pragma unroll
        for (int mk = 0; mk < MK; ++mk) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int kl0 = c_kt * TK + (wk * MK + mk) * 32 + (v >> 2) * 8 + (v & 3);
                if (kl0 >= P.Kg) continue;
                unsigned foff[2];
                bool short_row[2], short_col[2], none[2];
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int kl = kl0 + 4 * h;
                    none[h] = kl >= P.Kg;
                    const MergedFilter f = merged_filter(P, none[h] ? 0 : kl);
                    foff[h] = 4u * (unsigned)((c_g * P.mD + f.c) * OHW + f.i0 + P.OH * f.j0);
                    short_row[h] = f.i0 + P.osi * (P.Ho - 1) >= P.OH;      // this phase has no last row
                    short_col[h] = f.j0 + P.osj * (P.Wo - 1) >= P.OW;
                }
                const unsigned fo = half ? foff[1] : foff[0];
                const bool sr = half ? short_row[1] : short_row[0];
                const bool sc = half ? short_col[1] : short_col[0];
                const bool no = half ? none[1] : none[0];
#pragma unroll
                for (int mp = 0; mp < MP; ++mp) {
                    const bool drop = no || (sr && last_row[mp]) || (sc && last_col[mp]) || ooff[mp] == SLAB_INVALID;
                    const unsigned vo = drop ? SLAB_INVALID : ooff[mp] + fo;
                    float val = acc[0][mk][mp][v];
                    if (P.relu) val = fmaxf(val, 0.f);
                    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(val), ors, vo, 0, 0);
                }
            }
        }
    };
    // a piece of a shared tile, [filter][pixel]; WINO: in the output domain (the combination of the four sums
    // is linear), pixel = 2 * pair + row, so that the fix-up pass sees an ordinary tile of 2*TQ pixels
    auto store_partial = [&](int slot) {
        float *dst = part + (size_t)slot * (TK * TQ * (WINO ? 2 : 1));
#pragma unroll
        for (int mk = 0; mk < MK; ++mk)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int kloc = (wk * MK + mk) * 32 + (v >> 2) * 8 + half * 4 + (v & 3);
#pragma unroll
                for (int mp = 0; mp < MP; ++mp) {
                    const int ql = (wp * MP + mp) * 32 + (lane & 31);
                    if constexpr (WINO) {
                        const float m1 = acc[1][mk][mp][v], m2 = acc[2][mk][mp][v];
                        float2 y;
                        y.x = acc[0][mk][mp][v] + m1 + m2;
                        y.y = m1 - m2 - acc[3][mk][mp][v];
                        *reinterpret_cast<float2 *>(dst + kloc * (2 * TQ) + 2 * ql) = y;
                    } else {
                        dst[kloc * TQ + ql] = acc[0][mk][mp][v];
                    }
                }
            }
    };

    // ---- the block's range of units --------------------------------------------------------
    // position = (tile, unit); `done` = units consumed so far.  After the block's own tiles comes its range
    // of the shared ones, which may start in the middle of a tile.
    const int t_s = tile_s0 + (int)(ub / NU), uu_s = (int)(ub - (ub / NU) * NU);
    auto advance = [&](int &t, int &uu, int done) {
        if (done == n_own) { t = t_s; uu = uu_s; }
        else if (++uu == NU) { uu = 0; ++t; }
    };
    // The whole tiles of a block are numbered vb*own .. vb*own + own - 1; which tiles those are is dealt among the
    // blocks of an XCD (block i of the XCD's G takes the tiles i, G + i, 2G + i, ... of the XCD's run): tiles that
    // are neighbours in the plane, which read the same halo rows and the same weights, are then in flight on one
    // XCD at the same time and meet in its L2.  The left-over tiles keep their numbers.
    auto tile_of = [&](int t) {
        if (t >= tile_s0 || (P.nblocks & 7) != 0) return t;
        const int b = t / P.own, j = t - b * P.own;
        const int G = P.nblocks >> 3, x = b / G, i = b - x * G;
        return (x * G) * P.own + j * G + i;
    };
    int t_c = n_own ? vb * P.own : t_s;   // compute-side tile and unit
    int uu_c = n_own ? 0 : uu_s;
    int t_l = t_c, uu_l = uu_c;           // the load side runs one unit ahead
    bool first_segment = true;
    // the segment starting at unit uu of tile t covers the tile iff the tile is the block's own, or it
    // starts at 0 and the block's shared range reaches the tile's end
    auto segment_is_whole = [&](int t, int uu) {
        return t < tile_s0 || (uu == 0 && (long long)(t - tile_s0 + 1) * NU <= ue);
    };
    if (loader) {
        // Fetching wave: unit it+1 goes into the buffer that the computing waves left at the barrier of
        // iteration it; its own loads have landed before it joins the next barrier.  One barrier per
        // unit, as many as the computing waves pass.
        setup_load(tile_of(t_l));
        issue_loads(uu_l, 0);
        for (int it = 0; it < nunits; ++it) {
            __builtin_amdgcn_s_waitcnt(WAIT_VMCNT0);
            lds_barrier();
            if (it + 1 < nunits) {
                const int t_prev = t_l;
                advance(t_l, uu_l, it + 1);
                if (t_l != t_prev) setup_load(tile_of(t_l));
                issue_loads(uu_l, (it + 1) & 1);
            }
        }
        return;
    }
    bool whole = segment_is_whole(t_c, uu_c);
    setup_compute(tile_of(t_c));

    for (int it = 0; it < nunits; ++it) {
        lds_barrier();      // unit it is in LDS (the fetching waves waited for it) and the other buffer is free; results
                            // stored earlier drain on their own
        if (need_init) { init_acc(whole && bias != nullptr); need_init = false; }
        // the unit's steps in two halves (two unrolled lists)
        compute(std::integral_constant<int, 0>{}, uu_c, it & 1);
        compute(std::integral_constant<int, 1>{}, uu_c, it & 1);
        const bool last = it + 1 == nunits;
        if (uu_c + 1 == NU || last) {
            if (whole) { if (P.mD) store_tile_merged(); else store_tile(); }
            else store_partial(2 * vb + (first_segment ? 0 : 1));
            first_segment = it + 1 == n_own;      // the shared range starts with a "first" segment again
            if (!last) {
                advance(t_c, uu_c, it + 1);
                whole = segment_is_whole(t_c, uu_c);
                setup_compute(tile_of(t_c));
            }
        } else {
            ++uu_c;
        }
    }
}

// Sum the pieces of every tile that was shared between blocks, in block order, add the bias,
// and write the tile.  Grid: (left-over tiles, slices of a tile).
template <int TK, int TQ>
__global__ __launch_bounds__(256) void igemm_fixup_kernel(IgemmParams P, const float *__restrict__ part,
                                                          const float *__restrict__ bias, float *__restrict__ out) {
    const int ts = blockIdx.x;                       // shared tile (the grid has one row of blocks per shared tile)
    const int tile_s0 = P.own * P.nblocks;           // the shared tiles start here; unit numbers are relative to them
    const int t = tile_s0 + ts;
    // The tile's pieces, in block order.  Sharing block of rank r holds the units [total*r/nshare, total*(r+1)/nshare):
    // the first rank with units of this tile follows from one division (and a step of correction); its piece is
    // its first segment if its range starts in this tile, else its second; the following ranks' pieces are first
    // segments.  One thread lists them.
    constexpr int MAX_PIECES = 1024;
    __shared__ int slots[MAX_PIECES];
    __shared__ int npieces;
    if (threadIdx.x == 0)
        npieces = sk_tile_pieces((long long)(P.tiles - tile_s0) * P.NU, P.NU, P.nblocks, P.nshare, ts, slots, MAX_PIECES);
    __syncthreads();
    if (npieces == 0) return;
    int kt, pt, rb, g;
    decode_tile(P, t, &kt, &pt, &rb, &g);
    const int OHW = P.OH * P.OW;
    const int np = npieces;
    // a thread takes four consecutive pixels of one filter: one 16-byte load per piece, up to four pieces in flight
    constexpr int Q4 = TQ / 4;
    for (int e4 = blockIdx.y * 256 + threadIdx.x; e4 < TK * Q4; e4 += gridDim.y * 256) {
        const int kloc = e4 / Q4, ql = 4 * (e4 - kloc * Q4);
        const int kl = kt * TK + kloc;
        if (kl >= P.Kg || pt * TQ + ql >= P.QN) continue;
        int och = g * P.Kg + kl, fi0 = 0, fj0 = 0;
        if (P.mD) {
            const MergedFilter f = merged_filter(P, kl);
            fi0 = f.i0; fj0 = f.j0; och = g * P.mD + f.c;
        }
        const float bv = bias ? bias[och] : 0.f;
        const float *src = part + (size_t)kloc * TQ + ql;
        float4 acc = {bv, bv, bv, bv};
        int i = 0;
        for (; i + 3 < np; i += 4) {                  // four pieces in flight, added in piece order
            float4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = *reinterpret_cast<const float4 *>(src + (size_t)slots[i + u] * (TK * TQ));
#pragma unroll
            for (int u = 0; u < 4; ++u) { acc.x += v[u].x; acc.y += v[u].y; acc.z += v[u].z; acc.w += v[u].w; }
        }
        for (; i + 1 < np; i += 2) {
            const float4 v0 = *reinterpret_cast<const float4 *>(src + (size_t)slots[i] * (TK * TQ));
            const float4 v1 = *reinterpret_cast<const float4 *>(src + (size_t)slots[i + 1] * (TK * TQ));
            acc.x += v0.x; acc.y += v0.y; acc.z += v0.z; acc.w += v0.w;
            acc.x += v1.x; acc.y += v1.y; acc.z += v1.z; acc.w += v1.w;
        }
        if (i < np) {
            const float4 v0 = *reinterpret_cast<const float4 *>(src + (size_t)slots[i] * (TK * TQ));
            acc.x += v0.x; acc.y += v0.y; acc.z += v0.z; acc.w += v0.w;
        }
        const float vv[4] = {acc.x, acc.y, acc.z, acc.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int q = pt * TQ + ql + j;
            const int c = div32(q, P.dTI);
            const int ii = q - c * P.TI;
            const int n = div32(c, P.dWo);
            const int jo = c - n * P.Wo;
            const int io = rb * P.TI + ii;
            if (q >= P.QN || io >= P.Ho) continue;
            const int oi = P.oi0 + P.osi * io + fi0, oj = P.oj0 + P.osj * jo + fj0;
            if (P.mD && (oi >= P.OH || oj >= P.OW)) continue;
            float v = vv[j];
            if (P.relu) v = fmaxf(v, 0.f);
            out[(size_t)(oi + P.OH * (oj + P.OW * (P.Ktot * n))) + (size_t)OHW * och] = v;
        }
    }
}

}  // namespace mcn
