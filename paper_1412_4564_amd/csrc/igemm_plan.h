// Host-side planning for the implicit-GEMM kernel: which instantiation, how the
// pixels are cut into row blocks and tiles, how the reduction is cut into units,
// how large the LDS buffers are, and how many resident blocks share the work.
#pragma once
#include <stdint.h>
#include <stddef.h>
#include <stdlib.h>
#include "geom.h"
#include "kern_igemm.h"
#include "kern_igemm_bf16.h"

namespace mcn {

// One convolution "view": the sum the kernel evaluates (see kern_igemm.h).
struct ConvView {
    int H, W, N, Ctot, Cg;          // input array of the view
    int Ho, Wo, Ktot, Kg, G;        // output pixels computed, output channels
    int Hf, Wf, Sh, Sw, Pt, Pl;
    int OH, OW, oi0, osi, oj0, osj; // placement of the view's output pixels in the output array
    // weight packing (PackParams): mode, shape of the caller's filter array, stride phase
    int pack_mode, HfA, WfA, DfA, pSh, pSw, pi, pj, ldk;
    // all stride phases of an input derivative merged into one view (pack mode 3; kern_igemm.h)
    int mD, mPt, mPl, B0i, B0j;
};

inline ConvView forward_view(const Geom &g) {
    ConvView v = {};
    v.H = g.H; v.W = g.W; v.N = g.N; v.Ctot = g.D; v.Cg = g.Df;
    v.Ho = g.Ho; v.Wo = g.Wo; v.Ktot = g.K; v.Kg = g.Kg; v.G = g.G;
    v.Hf = g.Hf; v.Wf = g.Wf; v.Sh = g.Sh; v.Sw = g.Sw; v.Pt = g.Pt; v.Pl = g.Pl;
    v.OH = g.Ho; v.OW = g.Wo; v.oi0 = 0; v.osi = 1; v.oj0 = 0; v.osj = 1;
    v.pack_mode = 0; v.HfA = g.Hf; v.WfA = g.Wf; v.DfA = g.Df;
    return v;
}

// Input derivative, one stride phase (pi, pj), 0 <= pi < Sh, 0 <= pj < Sw  (Sec. 6.1 dz/dX, in the
// gather form of Sec. 6.2):  dzdx[i,j] = sum_{fi,fj,k} w[fi,fj,.,k] dzdy[(i+Pt-fi)/Sh, (j+Pl-fj)/Sw, k]
// over the taps for which the divisions are exact.  Rows i = i0 + Sh*m with i0 = (pi-Pt) mod Sh
// only see taps fi = pi + Sh*a; with t = A-1-a this is a stride-1 sum over dzdy with A taps and top
// pad A-1-b0, b0 = (i0+Pt-pi)/Sh.  Returns false if the phase has no taps or no rows (nothing to do:
// those samples of dzdx are zero).
inline bool backward_data_view(const Geom &g, int pi, int pj, ConvView *out) {
    const int A = pi < g.Hf ? (g.Hf - pi + g.Sh - 1) / g.Sh : 0;
    const int Bt = pj < g.Wf ? (g.Wf - pj + g.Sw - 1) / g.Sw : 0;
    const int i0 = ((pi - g.Pt) % g.Sh + g.Sh) % g.Sh;
    const int j0 = ((pj - g.Pl) % g.Sw + g.Sw) % g.Sw;
    const int Mi = i0 < g.H ? (g.H - i0 + g.Sh - 1) / g.Sh : 0;
    const int Mj = j0 < g.W ? (g.W - j0 + g.Sw - 1) / g.Sw : 0;
    if (A == 0 || Bt == 0 || Mi == 0 || Mj == 0) return false;
    const int b0 = (i0 + g.Pt - pi) / g.Sh, d0 = (j0 + g.Pl - pj) / g.Sw;   // exact divisions
    ConvView v = {};
    v.H = g.Ho; v.W = g.Wo; v.N = g.N; v.Ctot = g.K; v.Cg = g.Kg;
    v.Ho = Mi; v.Wo = Mj; v.Ktot = g.D; v.Kg = g.Df; v.G = g.G;
    v.Hf = A; v.Wf = Bt; v.Sh = 1; v.Sw = 1; v.Pt = A - 1 - b0; v.Pl = Bt - 1 - d0;
    v.OH = g.H; v.OW = g.W; v.oi0 = i0; v.osi = g.Sh; v.oj0 = j0; v.osj = g.Sw;
    v.pack_mode = 1; v.HfA = g.Hf; v.WfA = g.Wf; v.DfA = g.Df; v.pSh = g.Sh; v.pSw = g.Sw; v.pi = pi; v.pj = pj;
    *out = v;
    return true;
}

// Input derivative with all Sh*Sw stride phases in ONE view: the phases read the same dzdy, so they can
// share the slab and sit side by side in the "filter" dimension of the GEMM (merged filter = channel
// + D' * phase).  Worth it when a phase alone would leave most of a 32-row MFMA tile empty (few
// channels per group, e.g. the derivative with respect to an image with 3 channels).  Per direction
// the phases' tap ranges are put into one window: output row i0 + Sh*m of phase pi meets dzdy rows
// m + b0 - a, a = 0..A-1; with B0 = max b0 the window covers rows m + B0 - t, t = 0..TH-1.  Phases
// without taps (stride larger than the filter) are all-zero filters, so nothing is left to fill.
inline bool merged_backward_data_view(const Geom &g, ConvView *out) {
    if (g.Sh * g.Sw < 2 || g.Df > 16 || g.Df * g.Sh * g.Sw > 1024) return false;
    int B0[2] = {0, 0}, TH[2] = {1, 1};
    const int Hf[2] = {g.Hf, g.Wf}, S[2] = {g.Sh, g.Sw}, Pd[2] = {g.Pt, g.Pl};
    for (int d = 0; d < 2; ++d) {
        bool any = false;
        for (int pi = 0; pi < S[d]; ++pi) {
            if (pi >= Hf[d]) continue;
            const int i0 = ((pi - Pd[d]) % S[d] + S[d]) % S[d];
            const int b0 = (i0 + Pd[d] - pi) / S[d];
            if (!any || b0 > B0[d]) B0[d] = b0;
            any = true;
        }
        for (int pi = 0; pi < S[d]; ++pi) {
            if (pi >= Hf[d]) continue;
            const int A = (Hf[d] - pi + S[d] - 1) / S[d];
            const int i0 = ((pi - Pd[d]) % S[d] + S[d]) % S[d];
            const int b0 = (i0 + Pd[d] - pi) / S[d];
            if (A + B0[d] - b0 > TH[d]) TH[d] = A + B0[d] - b0;
        }
    }
    ConvView v = {};
    v.H = g.Ho; v.W = g.Wo; v.N = g.N; v.Ctot = g.K; v.Cg = g.Kg;
    v.Ho = (g.H + g.Sh - 1) / g.Sh; v.Wo = (g.W + g.Sw - 1) / g.Sw;
    v.Ktot = g.D; v.Kg = g.Df * g.Sh * g.Sw; v.G = g.G;
    v.Hf = TH[0]; v.Wf = TH[1]; v.Sh = 1; v.Sw = 1; v.Pt = TH[0] - 1 - B0[0]; v.Pl = TH[1] - 1 - B0[1];
    v.OH = g.H; v.OW = g.W; v.oi0 = 0; v.osi = g.Sh; v.oj0 = 0; v.osj = g.Sw;
    v.pack_mode = 3; v.HfA = g.Hf; v.WfA = g.Wf; v.DfA = g.Df; v.pSh = g.Sh; v.pSw = g.Sw;
    v.mD = g.Df; v.mPt = g.Pt; v.mPl = g.Pl; v.B0i = B0[0]; v.B0j = B0[1];
    *out = v;
    return true;
}

// Fully-connected case (Sec. 4.1: a filter as large as the input, one output sample per image,
// no padding, one group).  With R = H*W*D the three passes are plain matrix products of
// X (R x N), F (R x K) and dY (K x N), all stored with their first index fastest:
//   Y = F^T X + b,   dX = F dY,   dF = X dY^T.
inline bool is_fully_connected(const Geom &g) {
    return g.G == 1 && g.H == g.Hf && g.W == g.Wf && g.Pt == 0 && g.Pb == 0 && g.Pl == 0 && g.Pr == 0;
}
inline ConvView fc_view_1x1(int64_t R, int C, int K) {
    ConvView v = {};
    v.H = (int)R; v.W = 1; v.N = 1; v.Ctot = C; v.Cg = C;
    v.Ho = (int)R; v.Wo = 1; v.Ktot = K; v.Kg = K; v.G = 1;
    v.Hf = 1; v.Wf = 1; v.Sh = 1; v.Sw = 1; v.Pt = 0; v.Pl = 0;
    v.OH = (int)R; v.OW = 1; v.oi0 = 0; v.osi = 1; v.oj0 = 0; v.osj = 1;
    v.pack_mode = 0; v.HfA = 1; v.WfA = 1; v.DfA = C;
    return v;
}
// Y[k][n] = sum_r F[r][k] X[r][n]: the split-K kernel with the coefficients r as "pixels", the
// images as "filters" and the filters as "channels" (both operands contiguous along r).
inline ConvView fc_forward_view(const Geom &g) { return fc_view_1x1((int64_t)g.H * g.W * g.D, g.K, g.N); }
// dX[r][n] = sum_k F[r][k] dY[k][n]: a 1x1 convolution over the "image" F with R pixels and K
// channels, whose N filters are the columns of dY.
inline ConvView fc_backward_data_view(const Geom &g) { return fc_view_1x1((int64_t)g.H * g.W * g.D, g.K, g.N); }
// dF[r][k] = sum_n X[r][n] dY[k][n]: a 1x1 convolution over the "image" X with R pixels and N
// channels, whose K filters are the rows of dY (read transposed by the packing pass).
inline ConvView fc_backward_filter_view(const Geom &g) {
    ConvView v = fc_view_1x1((int64_t)g.H * g.W * g.D, g.N, g.K);
    v.pack_mode = 2; v.ldk = g.K;
    return v;
}

// IG_W*: the WINO kernels (filters x pairs of output rows)
// IG_96x256: eight waves of 96 filters x 32 pixels each, for 65 to 96 filters per group (a quarter fewer MFMAs than 128-filter tiles)
enum IgemmShape { IG_128x256 = 0, IG_64x512 = 1, IG_32x256 = 2, IG_64x256 = 3, IG_W128x128 = 4, IG_W64x256 = 5, IG_96x256 = 6,
                  IG_NONE = -1 };

struct IgemmPlan {
    int shape;          // IgemmShape
    bool bf16;          // operands rounded to bf16 (kern_igemm_bf16.h); sizes below are then in 32-bit words
    int planes;         // bf16: 1, or 2 = operands split into hi and lo bf16 planes, three products each
    int fixed;          // index into IGEMM_FIXED: an instantiation with compile-time filter size (0 = none)
    int TK, TQ, NT;
    IgemmParams P;
    PackParams Q;
    size_t lds_bytes;
    size_t packed_floats;
    size_t partial_floats;   // 2 slots of TK*TQ per resident block
    double score;            // the planner's cost figure of the chosen row-block height (lower is better)
};

constexpr size_t IGEMM_LDS_LIMIT = 160 * 1024;
constexpr int IGEMM_LOADER_WAVES = 4;     // fetching waves per block
// Instantiations with a compile-time filter size and channel count per unit: every LDS offset of
// the MFMA loop is then an immediate or one of a few hoisted sums, against an offset-table read and
// several address instructions per step in the general kernel.
struct IgemmFixed { int HF, WF, DC; };
constexpr IgemmFixed IGEMM_FIXED[] = {{0, 0, 0}, {3, 3, 8}, {1, 1, 32}, {5, 5, 4}};
constexpr int IGEMM_N_FIXED = 4;
constexpr IgemmFixed IGEMM_WINO = {4, 3, 8};      // the WINO kernels: four row combinations x three columns, 8 channels per unit

// exact number of slab columns the worst pixel tile needs
inline int slab_columns(const ConvView &v, int TI, int TQ, int Wp) {
    const int64_t QN = (int64_t)TI * v.Wo * v.N;
    int best = 0;
    for (int64_t q0 = 0; q0 < QN; q0 += TQ) {
        int64_t qe = q0 + TQ < QN ? q0 + TQ : QN;
        int64_t c0 = q0 / TI, c1 = (qe - 1) / TI;
        int64_t n0 = c0 / v.Wo, n1 = c1 / v.Wo;
        int64_t u0 = (c0 - n0 * v.Wo) * v.Sw;
        int64_t ul = (c1 - n1 * v.Wo) * v.Sw + (n1 - n0) * Wp + v.Wf - 1;
        int sc = (int)(ul - u0 + 1);
        if (sc > best) best = sc;
    }
    return best;
}

// How a tile's reduction is cut into units.  Returns false if nothing fits.
struct UnitCut { int pair_mode, DC, TC, NTR, NS; };

inline bool cut_units(const ConvView &v, int TK, int64_t CP, size_t lds_left, UnitCut *uc) {
    const int T = v.Hf * v.Wf;
    double best = 1e30;
    bool found = false;
    for (int mode = 0; mode < 2; ++mode) {
        for (int NTR = 1; NTR <= T; ++NTR) {
            int TC = (T + NTR - 1) / NTR;
            if (mode == 1) TC += TC & 1;                         // tap pairs: even capacity
            if ((int64_t)(NTR - 1) * TC >= T) continue;          // an empty last range
            for (int DC = 1; DC <= 64; ++DC) {
                if (mode == 0 && (DC & 1)) continue;
                if (DC > 1 && DC - (mode == 0 ? 2 : 1) >= v.Cg) break;   // more padding channels than needed
                int NS = mode == 0 ? (DC / 2) * TC : DC * (TC / 2);
                NS += NS & 1;
                if (NS > 80) continue;
                const size_t lds = (2 * ((size_t)NS * 2 * TK + 255) + 2 * (size_t)DC * CP) * 4;
                if (lds > lds_left) continue;
                // work actually issued per tile / useful work
                const int NCG = (v.Cg + DC - 1) / DC;
                const double issued = (double)NCG * NTR * NS * 2;
                const double useful = (double)v.Cg * T;
                // prefer little padding, then ~40 steps per unit, then few slab reloads (NTR small)
                const double score = issued / useful * (1.0 + 0.002 * (NS > 40 ? NS - 40 : 40 - NS)) *
                                     (1.0 + 0.01 * (NTR - 1));
                if (score < best) { best = score; found = true; uc->pair_mode = mode; uc->DC = DC; uc->TC = TC; uc->NTR = NTR; uc->NS = NS; }
            }
        }
    }
    return found;
}

// bf16 kernel: a unit is 16 channels x TC taps, one MFMA step per tap; the fewest tap ranges whose
// double-buffered weights (TC*2*TK 16-byte words) and slab (2*CP words) fit.
inline bool cut_units_bf16(const ConvView &v, int TK, int64_t CP, size_t lds_left, UnitCut *uc, int planes = 1) {
    const int T = v.Hf * v.Wf;
    for (int NTR = 1; NTR <= T; ++NTR) {
        const int TC = (T + NTR - 1) / NTR;
        if ((int64_t)(NTR - 1) * TC >= T) continue;
        const size_t lds = 2 * ((size_t)TC * 2 * TK + 2 * (size_t)CP) * 16 * planes;
        if (lds > lds_left) continue;
        uc->pair_mode = 0; uc->DC = BF_DC; uc->TC = TC; uc->NTR = NTR; uc->NS = TC;
        return true;
    }
    return false;
}

// wino: `v` is the stride-2, four-tap view of pairs of output rows (wino_view) and wino_Ho the real number of rows
inline bool plan_igemm_kind(const ConvView &v, int n_cu, IgemmPlan *pl, bool bf16, int fixed, bool two = false,
                            int wino_Ho = 0, int planes = 1) {
    const int T = v.Hf * v.Wf;
    const bool wino = wino_Ho > 0;
    const IgemmFixed FX = wino ? IGEMM_WINO : IGEMM_FIXED[fixed];
    int shape, WK, WP, MK, MP;
    // `two`: blocks of four waves, two of them resident per compute unit (half the LDS each): while one is
    // at its barrier or writes a tile, the other keeps the matrix cores busy
    const size_t lds_limit = two ? IGEMM_LDS_LIMIT / 2 : IGEMM_LDS_LIMIT;
    const int resident = two ? 2 * n_cu : n_cu;
    if (wino && v.Kg > 64) { shape = IG_W128x128; WK = 2; WP = 4; MK = 2; MP = 1; }
    else if (wino) { shape = IG_W64x256; WK = 1; WP = 8; MK = 2; MP = 1; }
    else if (two && v.Kg > 32) { shape = IG_64x256; WK = 1; WP = 4; MK = 2; MP = 2; }
    else if (!bf16 && v.Kg > 64 && v.Kg <= 96) { shape = IG_96x256; WK = 1; WP = 8; MK = 3; MP = 1; }
    else if (v.Kg > 64) { shape = IG_128x256; WK = 2; WP = 4; MK = 2; MP = 2; }
    else if (v.Kg > 32) { shape = IG_64x512; WK = 1; WP = 8; MK = 2; MP = 2; }
    else { shape = IG_32x256; WK = 1; WP = 4; MK = 1; MP = 2; }
    const int TK = WK * MK * 32, TQ = WP * MP * 32, NT = 64 * WK * WP;
    const int NL = 64 * IGEMM_LOADER_WAVES;      // threads of the fetching (bf16: staging) waves
    const int Wp = (v.Wo - 1) * v.Sw + v.Wf;
    // candidates for the row-block height
    int cand[48];
    int nc = 0;
    cand[nc++] = v.Ho;
    for (int parts = 2; parts <= 16; ++parts) cand[nc++] = (v.Ho + parts - 1) / parts;
    for (int t = 32; t <= 256; t += 32) cand[nc++] = t;
    for (int t = 1; t <= 16; t *= 2) cand[nc++] = t;
    const bool input_streams = 4.0 * v.H * v.W * (double)v.Ctot * v.N > 32.0 * 1024 * 1024;
    double best_score = 1e30;
    int bestTI = 0, bestSC = 0;
    UnitCut best_uc = {};
    for (int a = 0; a < nc; ++a) {
        const int TI = cand[a];
        if (TI < 1 || TI > v.Ho) continue;
        const int64_t SR = (int64_t)(TI - 1) * v.Sh + v.Hf;
        if (SR > 8192) continue;
        if ((int64_t)TI * v.Wo * v.N >= ((int64_t)1 << 30)) continue;
        const int SC = slab_columns(v, TI, TQ, Wp);
        const int64_t CP = (SR * SC + 63) / 64 * 64;
        if (CP > (bf16 ? bf_ept_max(NL) : 32) * NL) continue;
        // an image crossing inside a tile moves the window by whole images: keep offsets in range
        const int64_t span = (int64_t)SC / Wp + 2;
        if ((double)span * v.Ctot * v.H * v.W * 4.0 >= 2147483647.0) continue;
        if ((double)(span + 1) * v.Ktot * v.OH * v.OW * 4.0 >= 2147483647.0) continue;   // and inside its output window
        const int EPT = (int)((CP + NL - 1) / NL);
        const size_t fixed_lds = ((size_t)EPT * NL + 2 * TK + 4) * 4;
        UnitCut uc;
        if (bf16) {
            if (fixed_lds + 64 > lds_limit) continue;
            if (!cut_units_bf16(v, TK, CP, lds_limit - fixed_lds - 64, &uc, planes)) continue;
        } else if (fixed || wino) {
            uc.pair_mode = 0; uc.DC = FX.DC; uc.TC = T; uc.NTR = 1; uc.NS = (FX.DC / 2) * T;
            if ((2 * ((size_t)uc.NS * 2 * TK + 255) + 2 * (size_t)uc.DC * CP) * 4 + fixed_lds > lds_limit) continue;
        } else {
            if (fixed_lds + 4096 + 16384 > lds_limit) continue;
            // the offset table needs NTR*NS*2 ints: reserve 16 KB for it up front
            if (!cut_units(v, TK, CP, lds_limit - fixed_lds - 16384, &uc)) continue;
            if ((size_t)uc.NTR * uc.NS * 2 * 4 > 16384) continue;
        }
        const int RB = (v.Ho + TI - 1) / TI;
        const int64_t QN = (int64_t)TI * v.Wo * v.N;
        const int64_t PT = (QN + TQ - 1) / TQ;
        // rows of pixel tiles and of filter tiles that compute nothing
        const double mfma_waste = (double)RB * PT * TQ / ((double)v.Ho * v.Wo * v.N) *
                                  (double)((v.Kg + TK - 1) / TK * TK) / (double)v.Kg;
        const int NCG = (v.Cg + uc.DC - 1) / uc.DC;
        const double red_waste = (double)NCG * uc.NTR * uc.NS * (bf16 ? BF_DC : 2) / ((double)v.Cg * T);
        // when the input streams from memory, short slab rows waste most of every 128-byte line they touch
        // results are stored in column runs of TI samples: short runs are partial memory lines
        double score = mfma_waste * red_waste * (1.0 + 0.05 * (double)CP / TQ) *
                       (input_streams ? 1.0 + 4.0 / (double)SR : 1.0) * (1.0 + 2.0 / (double)TI);
        // bf16 kernels: every tap range of a group of channels is a unit of its own (a barrier, a prologue of LDS
        // reads); a smaller slab that leaves room for more taps per unit is worth a less regular row block
        // (measured with split operands, same box: layer 4a with one tap range 0.41 against 0.50 ms with three;
        // 4b with two 0.378 against 0.40 with three)
        if (bf16) score *= 1.0 + 0.5 * (uc.NTR - 1);
        if (wino) {
            // The row-pair kernels issue fewer MFMAs per staged byte and per stored line, and what was measured on
            // them weighs differently: short slab rows cost little, column runs of results (2*TI samples) that are
            // whole 128-byte lines are worth some 5 % (layer 4a: 32-row runs 0.74 ms, 112-row runs 0.78, 28-row 0.80).
            const double run_bytes = 8.0 * TI;
            const bool whole_lines = (8 * TI) % 128 == 0 && ((int64_t)v.OH * 4) % 128 == 0;
            score = mfma_waste * red_waste * (1.0 + 0.05 * (double)CP / TQ) *
                    (input_streams ? 1.0 + 1.0 / (double)SR : 1.0) * (1.0 + (whole_lines ? 0.0 : 0.25 * 128.0 / run_bytes));
        }
        if (score < best_score) { best_score = score; bestTI = TI; bestSC = SC; best_uc = uc; }
    }
    if (!bestTI) return false;

    IgemmParams &P = pl->P;
    P = IgemmParams{};
    P.H = v.H; P.W = v.W; P.N = v.N; P.Ctot = v.Ctot; P.Cg = v.Cg;
    P.Ho = v.Ho; P.Wo = v.Wo; P.Ktot = v.Ktot; P.Kg = v.Kg; P.G = v.G;
    P.Hf = v.Hf; P.Wf = v.Wf; P.Sh = v.Sh; P.Sw = v.Sw; P.Pt = v.Pt; P.Pl = v.Pl;
    P.TI = bestTI; P.RB = (v.Ho + bestTI - 1) / bestTI;
    P.Wp = Wp;
    P.SR = (bestTI - 1) * v.Sh + v.Hf; P.SRP = P.SR;
    P.CP = (P.SRP * bestSC + 63) / 64 * 64;
    P.EPT = (P.CP + NL - 1) / NL;
    P.KT = (v.Kg + TK - 1) / TK;
    P.QN = bestTI * v.Wo * v.N;
    P.PT = (P.QN + TQ - 1) / TQ;
    P.DC = best_uc.DC; P.TC = best_uc.TC; P.NTR = best_uc.NTR; P.NS = best_uc.NS; P.pair_mode = best_uc.pair_mode;
    P.NU = ((v.Cg + P.DC - 1) / P.DC) * P.NTR;
    const int64_t tiles = (int64_t)v.G * P.RB * P.PT * P.KT;
    if (tiles >= ((int64_t)1 << 30)) return false;
    P.tiles = (int)tiles;
    const int64_t total = tiles * P.NU;
    P.nblocks = (int)(total < resident ? total : resident);
    // whole tiles first, one share of the left-over tiles after (see IgemmParams::own): fewer tiles go through
    // the workspace and the fix-up pass than when everything is shared
    P.own = (int)(tiles / P.nblocks);
    if (!bf16 && 2 * tiles >= resident && tiles < resident) {
        // Somewhat fewer tiles than compute units: sharing every tile keeps all units busy but sends every tile through
        // the workspace and the fix-up pass; one whole tile per block leaves some units idle and needs neither.
        // Times in microseconds: a unit's MFMAs at about 80 % of the matrix core's rate (two waves per SIMD with
        // 512 threads or two resident blocks), the fix-up as a launch plus its traffic at about 4 TB/s.
        const double unit_us = (two ? 2 : NT / 256) * (double)P.NS * MK * MP * 64.0 / 0.8 / 2400.0;
        const double fix_us = 6.0 + (double)P.nblocks * TK * TQ * (wino ? 16.0 : 8.0) / 4.0e6;
        const double shared_us = (double)((total + P.nblocks - 1) / P.nblocks) * unit_us + fix_us;
        if ((double)P.NU * unit_us <= shared_us) {
            P.nblocks = (int)tiles;
            P.own = 1;
        }
    }
    // two blocks per compute unit, whole tiles for every block and some left over: the blocks dispatched
    // first take the left-over units (see IgemmParams::nshare)
    P.nshare = P.nblocks;
    if (two && P.own >= 1 && (int64_t)P.own * P.nblocks != tiles && P.nblocks == resident && P.nblocks % 16 == 0)
        P.nshare = P.nblocks / 2;
    P.OH = v.OH; P.OW = v.OW; P.oi0 = v.oi0; P.osi = v.osi; P.oj0 = v.oj0; P.osj = v.osj;
    P.mD = v.mD; P.mPt = v.mPt; P.mPl = v.mPl;
    P.wino_Ho = wino_Ho;
    P.dTI = make_div32(P.TI); P.dWo = make_div32(P.Wo); P.dWp = make_div32(P.Wp); P.dSRP = make_div32(P.SRP);
    P.dKT = make_div32(P.KT); P.dRB = make_div32(P.RB); P.dPT = make_div32(P.PT);
    // packed weights per unit, in 32-bit words: bf16 steps hold 2 octets x TK filters x 16 bytes
    const size_t wsz = bf16 ? (size_t)P.NS * planes * 2 * TK * 4 : ((size_t)P.NS * 2 * TK + 255) / 256 * 256;
    P.WSZ = (int)wsz;
    pl->packed_floats = (size_t)v.G * P.KT * P.NU * wsz;
    if (pl->packed_floats * 4 >= 2147483647ull) return false;
    P.packed_bytes = (unsigned)(pl->packed_floats * 4);
    // no workspace for partial tiles when no tile is shared
    pl->partial_floats = P.nblocks > 1 && (int64_t)P.own * P.nblocks != tiles ? (size_t)2 * P.nblocks * TK * TQ * (wino ? 2 : 1) : 0;
    pl->shape = shape; pl->bf16 = bf16; pl->planes = bf16 ? planes : 1; pl->fixed = fixed; pl->TK = TK; pl->TQ = TQ; pl->NT = NT;
    pl->score = best_score;
    if (bf16)
        pl->lds_bytes = (2 * wsz + 2 * (size_t)planes * 2 * P.CP * 4 + (size_t)P.EPT * NL + 2 * TK + 4) *
                        sizeof(float);
    else
        pl->lds_bytes = (2 * wsz + 2 * (size_t)P.DC * P.CP + (size_t)P.EPT * NL + 2 * TK +
                         (fixed || wino ? 0 : (size_t)P.NTR * P.NS * 2) + 4) * sizeof(float);
    if (pl->lds_bytes > lds_limit) return false;

    PackParams &Q = pl->Q;
    Q = PackParams{};
    Q.Hf = v.Hf; Q.Wf = v.Wf; Q.HfA = v.HfA; Q.WfA = v.WfA; Q.DfA = v.DfA;
    Q.Kg = v.Kg; Q.Cg = v.Cg; Q.G = v.G; Q.KT = P.KT; Q.NU = P.NU; Q.NTR = P.NTR; Q.NS = P.NS; Q.WSZ = P.WSZ; Q.TK = TK; Q.MK = MK;
    Q.DC = P.DC; Q.TC = P.TC; Q.pair_mode = P.pair_mode; Q.mode = v.pack_mode;
    Q.Sh = v.pSh; Q.Sw = v.pSw; Q.pi = v.pi; Q.pj = v.pj; Q.ldk = v.ldk;
    Q.mD = v.mD; Q.Pt = v.mPt; Q.Pl = v.mPl; Q.B0i = v.B0i; Q.B0j = v.B0j;
    Q.wino = wino ? 1 : 0;
    Q.planes = bf16 ? planes : 1;
    Q.total = (int)pl->packed_floats;
    return true;
}

// 3x3 filters at stride 1 with at least 16 channels per group: the view of pairs of output rows that the
// WINO kernels compute (kern_igemm.h).  Its rows are pairs, its four "taps" per column the four input rows a
// pair reads; results go to rows oi0 + osi * (2 * pair + {0, 1}) of the output array.
inline bool wino_view(const ConvView &v, ConvView *out) {
    if (v.Hf != 3 || v.Wf != 3 || v.Sh != 1 || v.Sw != 1 || v.mD || v.pack_mode > 1) return false;
    if (v.HfA != 3 || v.WfA != 3 || (v.pack_mode == 1 && (v.pSh != 1 || v.pSw != 1))) return false;
    if (v.Cg < 2 * IGEMM_WINO.DC || v.Ho < 2) return false;      // channels are padded to units of 8 (zero weights, slab reads as zero)
    if (v.Kg <= 32) return false;      // the WINO tiles are 64 or 128 filters wide; narrower layers keep the 32-filter tiles
    ConvView p = v;
    p.Hf = 4; p.Sh = 2; p.Ho = (v.Ho + 1) / 2; p.osi = 2 * v.osi;
    *out = p;
    return true;
}
inline bool wino_enabled() {
    // process-wide override for benchmarks; a caller chooses per call with MCN_PREC_FP32_PLAIN
    static const bool off = getenv("MCN_NO_WINO") != nullptr;
    return !off;
}

// The instantiation with this view's filter size if there is one, its channels divide into the
// fixed units and a plan fits; the general kernel otherwise.
// row_pairs: 3x3 stride-1 views may take the kernels that compute two output rows from four products per
// filter column (the caller asks for the plain order of summation with MCN_PREC_FP32_PLAIN).
// planes (bf16 only): 2 = split operands (kern_igemm_bf16.h)
inline bool plan_igemm(const ConvView &v, int n_cu, IgemmPlan *pl, bool bf16 = false, bool row_pairs = true, int planes = 1) {
    if (bf16) return plan_igemm_kind(v, n_cu, pl, true, 0, false, 0, planes);
    ConvView pv;
    if (row_pairs && wino_enabled() && wino_view(v, &pv) && plan_igemm_kind(pv, n_cu, pl, false, 0, false, v.Ho)) return true;
    // the instantiation with this view's filter size, if there is one and the channels divide into its units
    int fixed = 0;
    for (int f = 1; f < IGEMM_N_FIXED; ++f) {
        const IgemmFixed FX = IGEMM_FIXED[f];
        if (v.Hf == FX.HF && v.Wf == FX.WF && v.Cg >= 2 * FX.DC && v.Cg % FX.DC == 0) fixed = f;
    }
    for (int f = fixed;; f = 0) {
        // With more than 32 filters per group: two resident blocks of four waves rather than one of eight,
        // unless half the LDS forces a much worse row-block height on it (the scores are comparable).
        // Up to 32 filters the block has four computing waves either way; two of them per compute unit pay when
        // there are more tiles than compute units (layer 2a, 400 tiles: every block one whole tile, no fix-up
        // pass, forward 20 -> 17 us), not when tiles are shared anyway (layer 2b, 100 tiles in 512 pieces: +23 %).
        IgemmPlan one, two;
        const bool ok1 = plan_igemm_kind(v, n_cu, &one, false, f);
        bool ok2 = plan_igemm_kind(v, n_cu, &two, false, f, true);
        if (ok2 && v.Kg <= 32 && two.P.tiles <= n_cu) ok2 = false;
        if (ok2 && (!ok1 || two.score <= 1.15 * one.score)) { *pl = two; return true; }
        if (ok1) { *pl = one; return true; }
        if (f == 0) return false;
    }
}

}  // namespace mcn

// ---- filter derivative (kern_wgrad.h) ---------------------------------------------------
#include "kern_wgrad.h"
namespace mcn {

// WG_W*: the WINO kernels (filters x (filter column, channel) pairs)
// WG_96x128, WG_96x384: 65 to 96 filters per group; the second on 12 computing waves, for filters of more than 256
// coefficients per group (one tile then holds 384 of them and dzdy is staged once for all)
enum WgradShape { WG_128x128 = 0, WG_64x192 = 1, WG_32x256 = 2, WG_W128x128 = 3, WG_W64x192 = 4, WG_96x128 = 5, WG_96x384 = 6 };

struct WgradPlan {
    int shape;
    int TK, TR, NT;
    WgradParams P;
    size_t lds_bytes;
    int occupancy;           // resident blocks per compute unit
    size_t partial_floats;   // 2 slots of TK*TR per resident block
    bool wino;               // kern_wgrad.h, template flag WINO; TR then counts coefficients (3 per B lane)
};

// wino: the WINO kernels (3x3 filters at stride 1, more than 32 filters per group): tiles of 128 filters x 128
// (filter column, channel) pairs on 8 computing waves, or, up to 64 filters per group, 64 x 192 on 12 computing
// waves (one 32 x 32 tile with its four sets of accumulators each), which holds all of a 64-channel layer.
inline bool plan_wgrad(const ConvView &v, int n_cu, WgradPlan *pl, bool wino = false) {
    if (wino && (v.Hf != 3 || v.Wf != 3 || v.Sh != 1 || v.Sw != 1 || v.Ho < 2 || v.Kg <= 32)) return false;
    // A filter row that meets no input row at all (planes of one or two rows under large pads) has a derivative of
    // exactly zero; the WINO kernel would form it as a difference of sums that cancel only up to rounding.
    if (wino && (v.H + v.Pt < 3 || v.Ho - 1 < v.Pt)) return false;
    // Each of its sums also holds the products of the neighbouring row of dzdy, which cancel up to rounding; over a
    // handful of terms one small factor can leave that rounding large against the result's own terms.
    if (wino && (int64_t)v.N * v.Ho * v.Wo < 64) return false;
    const int T = wino ? v.Wf : v.Hf * v.Wf;             // B lanes per channel
    if ((int64_t)v.Hf * v.Wf * v.Cg >= ((int64_t)1 << 30)) return false;
    const int R = T * v.Cg;                              // B lanes in all
    // byte offsets into x and dzdy are 32-bit and relative to the start of an image
    if ((double)v.H * v.W * v.Ctot * 4 >= 2147483647.0) return false;
    if ((double)v.Ho * v.Wo * v.Ktot * 4 >= 2147483647.0) return false;
    int shape, WK, WR, MK, MR;
    if (wino && v.Kg > 64) { shape = WG_W128x128; WK = 2; WR = 4; MK = 2; MR = 1; }
    else if (wino) { shape = WG_W64x192; WK = 2; WR = 6; MK = 1; MR = 1; }     // 12 computing waves, one tile each per set
    else if (v.Kg > 64 && v.Kg <= 96 && R > 256) { shape = WG_96x384; WK = 3; WR = 4; MK = 1; MR = 3; }
    else if (v.Kg > 64 && v.Kg <= 96) { shape = WG_96x128; WK = 1; WR = 4; MK = 3; MR = 1; }
    else if (v.Kg > 64) { shape = WG_128x128; WK = 2; WR = 2; MK = 2; MR = 2; }
    else if (v.Kg > 32) { shape = WG_64x192; WK = 2; WR = 2; MK = 1; MR = 3; }
    else { shape = WG_32x256; WK = 1; WR = 4; MK = 1; MR = 2; }
    const int TK = WK * MK * 32, TR = WR * MR * 32, NT = 64 * WK * WR;
    const int RT = (R + TR - 1) / TR;
    int nch_max = 0;
    for (int rt = 0; rt < RT; ++rt) {
        const int lo = rt * TR, hi = (lo + TR < R ? lo + TR : R);
        const int n = (hi - 1) / T - lo / T + 1;
        if (n > nch_max) nch_max = n;
    }
    const int klim = v.Kg < TK ? v.Kg : TK;

    // a unit is a patch of TI rows x MC columns of one image's output plane, at most 128 pixels
    double best = 1e30;
    int bestTI = 0, bestMC = 0, bestSRP = 0, bestCP = 0, bestOcc = 0, bestPCHP = 0;
    size_t bestLds = 0;
    for (int TI = 1; TI <= v.Ho && TI <= 128; ++TI) {
        const int RB = (v.Ho + TI - 1) / TI;
        if (TI > 1 && TI < v.Ho && (v.Ho + TI - 2) / (TI - 1) == RB) continue;   // a smaller TI gives the same row blocks
        const int TIE = wino ? (TI + 3) & ~3 : (TI + 1) & ~1;
        const int64_t SR = (int64_t)(TIE - 1) * v.Sh + v.Hf;     // rows the padding pixel of an odd TI reads are staged too
        if (SR > 16384) continue;
        // pitches chosen so that the 32 coefficients a half-wave reads fall in 32 different LDS banks:
        // bank(r) = fi + SRP*fj + CP*c  ==  r  (mod 32)
        // (WINO: 8-byte reads at SRP/2 * fj + CP/2 * c, in units of 8 bytes: SRP/2 odd and CP = 3 SRP (mod 64)
        // make that SRP/2 * (fj + 3c), different for the lanes of a half-wave)
        int SRP = (int)SR;
        if (wino) while (SRP % 4 != 2) ++SRP;
        else while (SRP % 32 != v.Hf % 32) ++SRP;
        for (int MC = 1; MC <= v.Wo && TIE * MC <= 128; ++MC) {
            const int CC = (v.Wo + MC - 1) / MC;
            if (MC > 1 && MC < v.Wo && (v.Wo + MC - 2) / (MC - 1) == CC) continue;
            const int PCH = TIE * MC;
            const int64_t SC = (int64_t)(MC - 1) * v.Sw + v.Wf;
            if (SC >= 32768) continue;
            int64_t CP = (int64_t)SRP * SC;
            if (wino) while (CP % 64 != (3 * SRP) % 64) ++CP;
            else while (CP % 32 != T % 32) ++CP;
            const int64_t XS = (int64_t)nch_max * CP;
            int PCHP = PCH | 1;
            if (wino) { PCHP = PCH; while (PCHP % 4 != 2) ++PCHP; }
            const int EPT = (int)(((int64_t)SRP * SC + NT - 1) / NT);
            const int64_t lds = (2 * (int64_t)TK * PCHP + 2 * XS + (int64_t)EPT * NT + 4) * 4;
            if (lds > (int64_t)IGEMM_LDS_LIMIT) continue;
            int occ = (int)((int64_t)IGEMM_LDS_LIMIT / lds);
            if (occ > 2) occ = 2;   // the kernels are compiled for two waves per SIMD
            if (NT >= 512) occ = 1; // 8 or 12 computing + 4 fetching waves: one block per compute unit
            // cost of a unit in matrix-core cycles: its MFMAs plus what staging it costs beside them
            // (fitted to measurements: a fixed part and a part per staged element, about twice as
            // much when only one block fits a compute unit and nothing else hides it)
            const double units = (double)v.N * RB * CC;
            const double mfma = wino ? (double)(PCH / 4) * 4 * MK * MR * 64.0 : (double)(PCH / 2) * MK * MR * 64.0;
            const double elems = (double)klim * PCH + (double)nch_max * (double)(SRP * SC);
            // row runs that do not start on 128-byte lines cost extra memory transactions (a patch of whole
            // columns is one contiguous run of dzdy)
            const bool aligned = TI == v.Ho || (TI * 4) % 128 == 0;
            const double ovh = (1700.0 + 0.18 * elems) * (occ >= 2 ? 1.0 : 2.0) * (aligned ? 1.0 : 1.25);
            const double score = units * (mfma + ovh);
            if (score < best) {
                best = score; bestTI = TI; bestMC = MC; bestSRP = SRP; bestCP = (int)CP; bestOcc = occ;
                bestLds = (size_t)lds; bestPCHP = PCHP;
            }
        }
    }
    if (!bestTI) return false;

    WgradParams &P = pl->P;
    P = WgradParams{};
    P.H = v.H; P.W = v.W; P.N = v.N; P.Ctot = v.Ctot; P.Cg = v.Cg;
    P.Ho = v.Ho; P.Wo = v.Wo; P.Ktot = v.Ktot; P.Kg = v.Kg; P.G = v.G;
    P.Hf = v.Hf; P.Wf = v.Wf; P.Sh = v.Sh; P.Sw = v.Sw; P.Pt = v.Pt; P.Pl = v.Pl;
    P.TI = bestTI; P.RB = (v.Ho + bestTI - 1) / bestTI;
    P.MC = bestMC; P.CC = (v.Wo + bestMC - 1) / bestMC;
    P.TIE = wino ? (bestTI + 3) & ~3 : (bestTI + 1) & ~1;
    P.SR = (P.TIE - 1) * v.Sh + v.Hf;
    P.SRP = bestSRP; P.SC = (bestMC - 1) * v.Sw + v.Wf; P.CP = bestCP;
    P.EPT = (bestSRP * P.SC + NT - 1) / NT;
    P.KT = (v.Kg + TK - 1) / TK; P.RT = RT;
    P.PCH = P.TIE * bestMC; P.PCHP = bestPCHP;
    const int64_t NU = (int64_t)v.N * P.RB * P.CC;
    if (NU >= ((int64_t)1 << 30)) return false;
    P.NU = (int)NU;
    P.R = v.Hf * v.Wf * v.Cg;
    P.XS = nch_max * bestCP;
    const int64_t tiles = (int64_t)v.G * P.KT * RT;
    if (tiles >= ((int64_t)1 << 30)) return false;
    P.tiles = (int)tiles;
    const int64_t total = tiles * NU;
    const int64_t want = (int64_t)n_cu * bestOcc;
    P.nblocks = (int)(total < want ? total : want);
    P.nchunks = 0;
    // Arrays that stream from memory: the chunked schedule (kern_wgrad.h) reads them about once instead of
    // once per tile, if it keeps the compute units about as busy as equal ranges would (rounds of `want`
    // resident blocks, each block a chunk plus a fixed part).  It costs about 1 % of time on the large
    // layers (a few idle blocks, chunks that differ by a unit) and saves 2-10x of their memory traffic.
    if (4.0 * ((double)v.H * v.W * v.Ctot + (double)v.Ho * v.Wo * v.Ktot) * v.N > 64.0 * 1024 * 1024) {
        int best_nch = 0;
        double best_time = 1e300;
        for (int64_t nch = 1; nch <= NU && nch * tiles <= 4 * want; ++nch) {
            const int64_t rounds = (nch * tiles + want - 1) / want;
            const double time = (double)rounds * ((double)((NU + nch - 1) / nch) + 2.0);
            if (time < best_time * 0.9999999) { best_time = time; best_nch = (int)nch; }
        }
        if (best_nch > 0 && ((double)total / (double)want) / best_time >= 0.95) {
            P.nchunks = best_nch;
            P.nblocks = (int)(tiles * best_nch);
        }
    }
    // chunk weights (WgradParams::n_first): uneven only when two blocks share each compute unit and every
    // chunk has units to spare
    P.n_first = n_cu; P.w_first = 1; P.w_later = 1;
    if (P.nchunks > 0 && bestOcc == 2 && P.nblocks > n_cu && NU / P.nchunks >= 16) {
        P.w_first = 3; P.w_later = 2;      // measured on layers 4a/4b: 11:9 -1.5 %, 3:2 -2.2 %, 13:7 +1 %
    }
    // one tile, cut into a chunk per block: the blocks of an XCD take the units of their common range in turn
    // (WgradParams::deal; remainders in 32 bits: NU < 2^30 and rem * chunk < nchunks^2)
    P.deal = (P.nchunks >= 16 && P.tiles == 1 && P.nchunks % 8 == 0 && P.w_first == P.w_later && P.nchunks <= 32768) ? 1 : 0;
    pl->occupancy = bestOcc;
    pl->wino = wino;
    pl->partial_floats = P.nblocks > 1 ? (size_t)2 * P.nblocks * TK * TR * (wino ? 3 : 1) : 0;
    pl->shape = shape; pl->TK = TK; pl->TR = wino ? 3 * TR : TR; pl->NT = NT;
    pl->lds_bytes = bestLds;
    return true;
}

}  // namespace mcn

// ---- filter derivative with bf16 operands (kern_wgrad_bf16.h) ---------------------------------
#include "kern_wgrad_bf16.h"
namespace mcn {

enum WgradBfShape { WGB_128x256 = 0, WGB_64x256 = 1 };
constexpr int WGB_MAX_HF = 5;      // filter heights with an instantiation

struct WgradBfPlan {
    int shape;
    int TK, TR, NT;
    WgradBfParams P;
    size_t lds_bytes;
    size_t partial_floats;   // one TK*TR piece per block when a tile's reduction is shared
};

// Slab pitches (in 16-byte words): lane r of an operand read addresses word
// fi*CPF + fj*RGP + c*CPC (+ the same for all lanes); eight consecutive r should fall into eight
// different 16-byte bank groups.  Smallest pitches with the fewest collisions.
inline void wgb_pitches(int Hf, int Wf, int TIG, int SC, int *RGP, int *CPF, int *CPC) {
    const int T = Hf * Wf;
    long best_cost = -1;
    for (int a = 0; a < 8; ++a)
        for (int b = 0; b < 8; ++b)
            for (int c = 0; c < 8; ++c) {
                const int rgp = TIG + a, cpf = SC * rgp + b, cpc = Hf * cpf + c;
                int coll = 0;
                for (int r0 = 0; r0 < 8 * T; r0 += 8) {
                    unsigned seen = 0;
                    for (int r = r0; r < r0 + 8; ++r) {
                        const int ch = r / T, tap = r % T, fj = tap / Hf, fi = tap % Hf;
                        seen |= 1u << ((fi * cpf + fj * rgp + ch * cpc) & 7);
                    }
                    coll += 8 - __builtin_popcount(seen);
                }
                const long cost = (long)coll * 100000 + cpc;
                if (best_cost < 0 || cost < best_cost) { best_cost = cost; *RGP = rgp; *CPF = cpf; *CPC = cpc; }
            }
}

inline bool plan_wgrad_bf16(const ConvView &v, int n_cu, WgradBfPlan *pl) {
    if (v.Sh != 1 || v.Hf > WGB_MAX_HF || v.Kg <= 32) return false;
    const int T = v.Hf * v.Wf;
    const int64_t R64 = (int64_t)T * v.Cg;
    if (R64 >= ((int64_t)1 << 30)) return false;
    const int R = (int)R64;
    if ((double)v.H * v.W * v.Ctot * 4 >= 2147483647.0) return false;      // 32-bit byte offsets inside an image
    if ((double)v.Ho * v.Wo * v.Ktot * 4 >= 2147483647.0) return false;
    const int shape = v.Kg > 64 ? WGB_128x256 : WGB_64x256;
    const int TK = v.Kg > 64 ? 128 : 64, TR = 256, NT = 512;
    const int RT = (R + TR - 1) / TR;
    int NCH = 0;
    for (int rt = 0; rt < RT; ++rt) {
        const int lo = rt * TR, hi = (lo + TR < R ? lo + TR : R);
        const int n = (hi - 1) / T - lo / T + 1;
        if (n > NCH) NCH = n;
    }
    int cand[40], nc = 0;
    cand[nc++] = v.Ho;
    for (int parts = 2; parts <= 8; ++parts) cand[nc++] = (v.Ho + parts - 1) / parts;
    for (int t = 8; t <= 128; t += 8) cand[nc++] = t;
    const bool streams_from_memory =
        4.0 * ((double)v.H * v.W * v.Ctot + (double)v.Ho * v.Wo * v.Ktot) * v.N > 64.0 * 1024 * 1024;
    double best = 1e300;
    WgradBfParams B = {};
    for (int a = 0; a < nc; ++a) {
        const int TI = cand[a];
        if (TI < 1 || TI > v.Ho) continue;
        const int TIG = (TI + 7) / 8;
        for (int MC = 2; MC <= 32; MC += 2) {
            const int PW = TIG * MC;
            if ((int64_t)TK * PW > (int64_t)WGB_YT * NT) break;
            const int SC = (MC - 1) * v.Sw + v.Wf;
            if ((int64_t)NCH * SC * TIG > (int64_t)WGB_XT * NT) break;
            int RGP, CPF, CPC;
            wgb_pitches(v.Hf, v.Wf, TIG, SC, &RGP, &CPF, &CPC);
            const int PYW = PW | 1;
            const size_t lds = 2 * ((size_t)TK * PYW + (size_t)NCH * CPC) * 16;
            if (lds > IGEMM_LDS_LIMIT) break;
            const int RB = (v.Ho + TI - 1) / TI, CC = (v.Wo + MC - 1) / MC;
            const double units = (double)RB * CC * v.N;
            const double steps = (double)(MC / 2) * TIG;
            // a unit costs about three steps of set-up; when the arrays do not fit the caches, short
            // column segments waste most of every 128-byte line they touch
            const double cost = units * (steps + 3.0) * (streams_from_memory ? 1.0 + 16.0 / TI : 1.0);
            if (cost < best) {
                best = cost;
                B.TI = TI; B.RB = RB; B.TIG = TIG; B.MC = MC; B.CC = CC; B.SC = SC;
                B.PW = PW; B.PYW = PYW; B.RGP = RGP; B.CPF = CPF; B.CPC = CPC;
            }
        }
    }
    if (best >= 1e300) return false;
    WgradBfParams &P = pl->P;
    P = B;
    P.H = v.H; P.W = v.W; P.N = v.N; P.Ctot = v.Ctot; P.Cg = v.Cg;
    P.Ho = v.Ho; P.Wo = v.Wo; P.Ktot = v.Ktot; P.Kg = v.Kg; P.G = v.G;
    P.Hf = v.Hf; P.Wf = v.Wf; P.Sw = v.Sw; P.Pt = v.Pt; P.Pl = v.Pl;
    P.NCH = NCH;
    P.KT = (v.Kg + TK - 1) / TK; P.RT = RT; P.R = R;
    const int64_t NU = (int64_t)P.RB * P.CC * v.N;
    const int64_t tiles = (int64_t)v.G * P.KT * RT;
    if (NU >= ((int64_t)1 << 30) || tiles >= ((int64_t)1 << 20)) return false;
    P.NU = (int)NU; P.tiles = (int)tiles;
    // chunks per tile: fill the compute units in as few, as full rounds as possible
    int best_nch = 1;
    double best_eff = 0.0;
    const int64_t max_nch = NU < 4 * (int64_t)n_cu ? NU : 4 * (int64_t)n_cu;
    for (int64_t nch = 1; nch <= max_nch && nch * tiles <= 4 * (int64_t)n_cu; ++nch) {
        const int64_t nb = nch * tiles;
        const int64_t rounds = (nb + n_cu - 1) / n_cu;
        // a round of chunks costs its units plus a fixed part (set-up, writing the piece)
        const double time = (double)rounds * ((double)((NU + nch - 1) / nch) + 8.0);
        const double eff = 1.0 / time;
        if (eff > best_eff * 1.0000001) { best_eff = eff; best_nch = (int)nch; }
    }
    P.nchunks = best_nch;
    P.nblocks = (int)(tiles * best_nch);
    pl->shape = shape; pl->TK = TK; pl->TR = TR; pl->NT = NT;
    pl->lds_bytes = 2 * ((size_t)TK * P.PYW + (size_t)NCH * P.CPC) * 16;
    pl->partial_floats = P.nchunks > 1 ? (size_t)P.nblocks * TK * TR : 0;
    return true;
}

}  // namespace mcn
