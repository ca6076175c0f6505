// Host-side planning for the implicit-GEMM kernel: which instantiation, how the
// pixels are cut into row blocks and tiles, how large the LDS slab is.
#pragma once
#include <stdint.h>
#include <stddef.h>
#include "geom.h"
#include "kern_igemm.h"

namespace mcn {

// One convolution "view": the sum the kernel evaluates (see kern_igemm.h).
struct ConvView {
    int H, W, N, Ctot, Cg;
    int Ho, Wo, Ktot, Kg, G;
    int Hf, Wf, Sh, Sw, Pt, Pl;
    int pack_mode;   // 0 forward, 1 input derivative (flipped, transposed filters)
};

inline ConvView forward_view(const Geom &g) {
    ConvView v;
    v.H = g.H; v.W = g.W; v.N = g.N; v.Ctot = g.D; v.Cg = g.Df;
    v.Ho = g.Ho; v.Wo = g.Wo; v.Ktot = g.K; v.Kg = g.Kg; v.G = g.G;
    v.Hf = g.Hf; v.Wf = g.Wf; v.Sh = g.Sh; v.Sw = g.Sw; v.Pt = g.Pt; v.Pl = g.Pl;
    v.pack_mode = 0;
    return v;
}

// Stride-1 only: dzdx[i,j] = sum_{fi,fj,k} w[fi,fj,.,k] dzdy[i+Pt-fi, j+Pl-fj, k]; substituting
// fi' = Hf-1-fi turns it into the forward sum over dzdy with top pad Hf-1-Pt (Sec. 6.1, dz/dX).
inline ConvView backward_data_view(const Geom &g) {
    ConvView v;
    v.H = g.Ho; v.W = g.Wo; v.N = g.N; v.Ctot = g.K; v.Cg = g.Kg;
    v.Ho = g.H; v.Wo = g.W; v.Ktot = g.D; v.Kg = g.Df; v.G = g.G;
    v.Hf = g.Hf; v.Wf = g.Wf; v.Sh = 1; v.Sw = 1; v.Pt = g.Hf - 1 - g.Pt; v.Pl = g.Wf - 1 - g.Pl;
    v.pack_mode = 1;
    return v;
}

enum IgemmShape { IG_128x256 = 0, IG_64x512 = 1, IG_32x256 = 2, IG_NONE = -1 };

struct IgemmPlan {
    int shape;          // IgemmShape
    bool fixed33;       // 3x3 filter instantiation
    int DC;             // channels per chunk
    int TK, TQ, NT;
    IgemmParams P;
    size_t lds_bytes;
    size_t packed_floats;
    int blocks;
};

constexpr int IGEMM_EPT = 2;
constexpr int IGEMM_TMAX = 25;
constexpr size_t IGEMM_LDS_LIMIT = 160 * 1024;

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

inline bool plan_igemm(const ConvView &v, IgemmPlan *pl) {
    const int T = v.Hf * v.Wf;
    if (T > IGEMM_TMAX) return false;
    int shape, WK, WP, MK, MP;
    if (v.Kg > 64) { shape = IG_128x256; WK = 2; WP = 4; MK = 2; MP = 2; }
    else if (v.Kg > 32) { shape = IG_64x512; WK = 1; WP = 8; MK = 2; MP = 2; }
    else { shape = IG_32x256; WK = 1; WP = 4; MK = 1; MP = 2; }
    const int TK = WK * MK * 32, TQ = WP * MP * 32, NT = 64 * WK * WP;
    const bool fixed33 = (v.Hf == 3 && v.Wf == 3);
    int DC = fixed33 ? 8 : 4;
    if (!fixed33 && T > 16 && TK == 128) DC = 4;
    const int Wp = (v.Wo - 1) * v.Sw + v.Wf;
    const size_t wchunk = (size_t)DC * T * TK;

    // candidates for the row-block height
    int cand[40];
    int nc = 0;
    cand[nc++] = v.Ho;
    for (int parts = 2; parts <= 16; ++parts) cand[nc++] = (v.Ho + parts - 1) / parts;
    for (int t = 32; t <= 256; t += 32) cand[nc++] = t;
    double best_score = 1e30;
    int bestTI = 0, bestSC = 0;
    for (int a = 0; a < nc; ++a) {
        const int TI = cand[a];
        if (TI < 1 || TI > v.Ho) continue;
        const int64_t SR = (int64_t)(TI - 1) * v.Sh + v.Hf;
        if (SR > 4096) continue;
        if ((int64_t)TI * v.Wo * v.N >= ((int64_t)1 << 30)) continue;
        const int SC = slab_columns(v, TI, TQ, Wp);
        const int64_t CP = SR * SC;
        if (CP > (int64_t)IGEMM_EPT * NT) continue;
        const size_t lds = (2 * wchunk + 2 * (size_t)DC * CP) * sizeof(float);
        if (lds > IGEMM_LDS_LIMIT) continue;
        const int RB = (v.Ho + TI - 1) / TI;
        const int64_t QN = (int64_t)TI * v.Wo * v.N;
        const int64_t PT = (QN + TQ - 1) / TQ;
        const double mfma_waste = (double)RB * PT * TQ / ((double)v.Ho * v.Wo * v.N);
        const double score = mfma_waste * (1.0 + 0.05 * (double)CP / TQ);
        if (score < best_score) { best_score = score; bestTI = TI; bestSC = SC; }
    }
    if (!bestTI) return false;

    IgemmParams &P = pl->P;
    P.H = v.H; P.W = v.W; P.N = v.N; P.Ctot = v.Ctot; P.Cg = v.Cg;
    P.Ho = v.Ho; P.Wo = v.Wo; P.Ktot = v.Ktot; P.Kg = v.Kg; P.G = v.G;
    P.Hf = v.Hf; P.Wf = v.Wf; P.Sh = v.Sh; P.Sw = v.Sw; P.Pt = v.Pt; P.Pl = v.Pl;
    P.TI = bestTI; P.RB = (v.Ho + bestTI - 1) / bestTI;
    P.Wp = Wp;
    P.SR = (bestTI - 1) * v.Sh + v.Hf; P.SRP = P.SR;
    P.CP = P.SRP * bestSC;
    P.KT = (v.Kg + TK - 1) / TK;
    P.NCH = (v.Cg + DC - 1) / DC;
    P.QN = bestTI * v.Wo * v.N;
    P.PT = (P.QN + TQ - 1) / TQ;
    const int64_t blocks = (int64_t)v.G * P.RB * P.PT * P.KT;
    if (blocks >= ((int64_t)1 << 31)) return false;
    pl->shape = shape; pl->fixed33 = fixed33; pl->DC = DC; pl->TK = TK; pl->TQ = TQ; pl->NT = NT;
    pl->lds_bytes = (2 * wchunk + 2 * (size_t)DC * P.CP) * sizeof(float);
    pl->packed_floats = (size_t)v.G * P.KT * P.NCH * wchunk;
    pl->blocks = (int)blocks;
    return true;
}

}  // namespace mcn

// ---- filter derivative (kern_wgrad.h) ---------------------------------------------------
#include "kern_wgrad.h"
namespace mcn {

enum WgradShape { WG_128x128 = 0, WG_64x192 = 1, WG_32x256 = 2 };

struct WgradPlan {
    int shape;
    int PCH;             // pixels per chunk
    int TK, TR, NT;
    WgradParams P;
    size_t lds_bytes;
    int splits;          // RB * SPR
    size_t partial_floats;
    int blocks;
};

inline bool plan_wgrad(const Geom &g, WgradPlan *pl) {
    ConvView v = forward_view(g);
    const int T = v.Hf * v.Wf;
    const int R = T * v.Cg;
    if ((double)numel_x(g) * 4 >= 2147483647.0 || (double)numel_y(g) * 4 >= 2147483647.0) return false;
    int shape, WK, WR, MK, MR, EPT, NCHMAX, WGRAD_PCH;
    if (v.Kg > 64) { shape = WG_128x128; WK = 2; WR = 2; MK = 2; MR = 2; EPT = 2; NCHMAX = 16; WGRAD_PCH = 32; }
    else if (v.Kg > 32) { shape = WG_64x192; WK = 2; WR = 2; MK = 1; MR = 3; EPT = 2; NCHMAX = 24; WGRAD_PCH = 64; }
    else { shape = WG_32x256; WK = 1; WR = 4; MK = 1; MR = 2; EPT = 2; NCHMAX = 32; WGRAD_PCH = 32; }
    const int TK = WK * MK * 32, TR = WR * MR * 32, NT = 64 * WK * WR;
    const int RT = (R + TR - 1) / TR;
    int nch_max = 0;
    for (int rt = 0; rt < RT; ++rt) {
        const int lo = rt * TR, hi = (lo + TR < R ? lo + TR : R);
        const int n = (hi - 1) / T - lo / T + 1;
        if (n > nch_max) nch_max = n;
    }
    if (nch_max > NCHMAX) return false;
    const int Wp = (v.Wo - 1) * v.Sw + v.Wf;

    int cand[40];
    int nc = 0;
    cand[nc++] = v.Ho;
    for (int parts = 2; parts <= 16; ++parts) cand[nc++] = (v.Ho + parts - 1) / parts;
    for (int t = 32; t <= 256; t += 32) cand[nc++] = t;
    double best = 1e30;
    int bestTI = 0, bestSC = 0;
    for (int a = 0; a < nc; ++a) {
        const int TI = cand[a];
        if (TI < 1 || TI > v.Ho) continue;
        const int64_t SR = (int64_t)(TI - 1) * v.Sh + v.Hf;
        if (SR > 4096) continue;
        const int64_t QN = (int64_t)TI * v.Wo * v.N;
        if (QN >= ((int64_t)1 << 30)) continue;
        const int SC = slab_columns(v, TI, WGRAD_PCH, Wp);
        if (SC > 2 * Wp) continue;                       // at most two image crossings per chunk
        if (SR * SC > (int64_t)EPT * NT) continue;
        const int RB = (v.Ho + TI - 1) / TI;
        const double chunks = (double)RB * (double)((QN + WGRAD_PCH - 1) / WGRAD_PCH);
        const double score = chunks * (1.0 + 0.002 * (double)(SR * SC));
        if (score < best) { best = score; bestTI = TI; bestSC = SC; }
    }
    if (!bestTI) return false;

    WgradParams &P = pl->P;
    P.H = v.H; P.W = v.W; P.N = v.N; P.Ctot = v.Ctot; P.Cg = v.Cg;
    P.Ho = v.Ho; P.Wo = v.Wo; P.Ktot = v.Ktot; P.Kg = v.Kg; P.G = v.G;
    P.Hf = v.Hf; P.Wf = v.Wf; P.Sh = v.Sh; P.Sw = v.Sw; P.Pt = v.Pt; P.Pl = v.Pl;
    P.TI = bestTI; P.RB = (v.Ho + bestTI - 1) / bestTI;
    P.Wp = Wp;
    P.SR = (bestTI - 1) * v.Sh + v.Hf;
    P.SC = bestSC;
    // pitches chosen so that the 32 coefficients a half-wave reads fall in 32 different LDS banks:
    // bank(r) = fi + SRP*fj + CP*c  ==  r  (mod 32)
    int SRP = P.SR;
    while (SRP % 32 != v.Hf % 32) ++SRP;
    int CP = SRP * bestSC;
    while (CP % 32 != T % 32) ++CP;
    P.SRP = SRP; P.CP = CP;
    P.KT = (v.Kg + TK - 1) / TK; P.RT = RT;
    P.QN = bestTI * v.Wo * v.N;
    P.R = R;
    P.XS = nch_max * CP;
    P.EPTU = (P.SR * bestSC + NT - 1) / NT;
    pl->PCH = WGRAD_PCH;
    const int64_t base_blocks = (int64_t)v.G * P.KT * RT * P.RB;
    const int64_t chunks = (P.QN + WGRAD_PCH - 1) / WGRAD_PCH;
    int64_t spr = (768 + base_blocks - 1) / base_blocks;
    if (spr > chunks) spr = chunks;
    if (spr < 1) spr = 1;
    int64_t qs = ((chunks + spr - 1) / spr) * WGRAD_PCH;
    spr = (P.QN + qs - 1) / qs;
    P.QS = (int)qs; P.SPR = (int)spr;
    pl->splits = (int)(P.RB * spr);
    P.direct_out = pl->splits == 1;
    pl->partial_floats = pl->splits > 1 ? (size_t)pl->splits * (size_t)numel_w(g) : 0;
    if (pl->partial_floats * 4 > ((size_t)3 << 30)) return false;
    const int64_t blocks = base_blocks * spr;
    if (blocks >= ((int64_t)1 << 31)) return false;
    pl->blocks = (int)blocks;
    pl->shape = shape; pl->TK = TK; pl->TR = TR; pl->NT = NT;
    pl->lds_bytes = (size_t)(2 * TK * (WGRAD_PCH + 1) + 2 * WGRAD_PCH + 2 * P.XS) * sizeof(float);
    if (pl->lds_bytes > IGEMM_LDS_LIMIT) return false;
    return true;
}

}  // namespace mcn
