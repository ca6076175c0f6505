// Implicit-GEMM convolution on the fp32 matrix cores (v_mfma_f32_32x32x2_f32).
//
// Computes the sum of Sec. 4.1 of the MatConvNet manual (arXiv 1412.4564),
//   out[io,jo,k,n] = bias[k] + sum_{fi,fj,c} wt(k,c,fi,fj) * in[Sh*io+fi-Pt, Sw*jo+fj-Pl, g*Cg+c, n],
// for one "view" of a convolution.  The forward pass uses it directly; the
// derivative with respect to the input (Sec. 6.1, dz/dX = phi*(dz/dY F^T)) of a
// stride-1 convolution is the same sum over dzdy with the filter flipped and the
// roles of input channels and filters exchanged, so it runs on this kernel too with
// a different weight packing (Pt, Pl may then be negative = cropping).
//
// Mapping to the GEMM  OUT[k][pixel] = sum_r WT[k][r] * PATCH[r][pixel]:
//  * matrix A (32 filters x 2 channels) comes from a packed copy of the weights,
//    matrix B (2 channels x 32 pixels) from an LDS copy of the input ("slab") --
//    never from an im2row buffer in HBM.  Lanes run along pixels, which are
//    contiguous in memory (first array index), so B reads and the final stores
//    are coalesced.
//  * pixels of one block: rows are cut into row blocks of TI rows; inside a row
//    block the pixels are numbered q = ii + TI*(jo + Wo*n), i.e. columns of all
//    images are chained, and a block takes TQ consecutive q.  The slab holds, per
//    channel, every input column/row those pixels read, so filter tap (fi,fj) of
//    pixel q is the slab element at  base(q) + fi + SRP*fj.
//  * reduction: channels in chunks of DC, double-buffered in LDS; inside a chunk
//    all taps; one MFMA consumes two channels of one tap.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mcn {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

struct IgemmParams {
    int H, W, N;        // input plane size, batch
    int Ctot, Cg;       // channels in the input array / per group (reduction depth)
    int Ho, Wo;         // output plane size
    int Ktot, Kg, G;    // channels in the output array / per group, groups
    int Hf, Wf, Sh, Sw;
    int Pt, Pl;         // top/left pad (negative = crop)
    int TI, RB;         // rows per row block, number of row blocks
    int Wp;             // columns reserved per image in the chained padded-column index
    int SR, SRP;        // slab rows used / row pitch
    int CP;             // slab channel pitch (floats)
    int KT, NCH, PT;    // filter tiles per group, channel chunks, pixel tiles per row block
    int QN;             // TI*Wo*N: chained pixels per row block
};

constexpr unsigned SLAB_INVALID = 0x80000000u;   // >= any per-block buffer size: reads as 0

// ---- weight packing ------------------------------------------------------------------
// packed[g][kt][ch][dp][tap][half][kk] = wt(k = kt*TK+kk, c = ch*DC + 2*dp + half, tap), 0 outside.
// mode 0 (forward):        wt(k,c,fi,fj) = w[fi, fj, c, g*Kg + k]
// mode 1 (input derivative of a stride-1 convolution, Kg = D', Cg = K/G):
//                          wt(k,c,fi,fj) = w[Hf-1-fi, Wf-1-fj, k, g*Cg + c]
__global__ __launch_bounds__(256) void igemm_pack_weights_kernel(const float *__restrict__ w, float *__restrict__ packed,
                                                                 int Hf, int Wf, int Df, int Kg, int Cg, int G, int KT,
                                                                 int NCH, int TK, int DC, int mode, int total) {
    int p = blockIdx.x * 256 + threadIdx.x;
    if (p >= total) return;
    const int T = Hf * Wf;
    int t = p;
    const int kk = t % TK; t /= TK;
    const int half = t & 1; t >>= 1;
    const int tap = t % T; t /= T;
    const int dp = t % (DC / 2); t /= (DC / 2);
    const int ch = t % NCH; t /= NCH;
    const int kt = t % KT;
    const int g = t / KT;
    const int k = kt * TK + kk;
    const int c = ch * DC + 2 * dp + half;
    float v = 0.f;
    if (k < Kg && c < Cg) {
        const int fi = tap % Hf, fj = tap / Hf;
        if (mode == 0)
            v = w[fi + Hf * (fj + Wf * (c + (size_t)Df * (g * Kg + k)))];
        else
            v = w[(Hf - 1 - fi) + Hf * ((Wf - 1 - fj) + Wf * (k + (size_t)Df * (g * Cg + c)))];
    }
    packed[p] = v;
}

// ---- main kernel -----------------------------------------------------------------------
// WK x WP waves; each wave owns MK x MP tiles of 32 filters x 32 pixels.
// HF, WF > 0: filter size known at compile time; 0: read from the parameters (T <= TMAX).
template <int WK, int WP, int MK, int MP, int DC, int HF, int WF, int TMAX, int EPT>
__global__ __launch_bounds__(64 * WK * WP) void igemm_conv_kernel(IgemmParams P, const float *__restrict__ in,
                                                                  const float *__restrict__ wpk,
                                                                  const float *__restrict__ bias,
                                                                  float *__restrict__ out) {
    constexpr int NT = 64 * WK * WP;
    constexpr int TK = WK * MK * 32;
    constexpr int TQ = WP * MP * 32;
    constexpr int WPT = (DC * TMAX * TK / 4 + NT - 1) / NT;   // float4 weight loads per thread per chunk
    const int Hf = HF ? HF : P.Hf;
    const int Wf = WF ? WF : P.Wf;
    const int T = Hf * Wf;
    const int wchunk = DC * T * TK;        // floats of packed weights per chunk
    const int wchunk4 = wchunk / 4;
    const int CP = P.CP, SRP = P.SRP;

    extern __shared__ __align__(16) float lds[];
    float *wbuf0 = lds;
    float *wbuf1 = lds + wchunk;
    float *xbuf0 = lds + 2 * wchunk;
    float *xbuf1 = xbuf0 + DC * CP;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wk = wave % WK, wp = wave / WK;

    int b = blockIdx.x;
    const int kt = b % P.KT; b /= P.KT;
    const int pt = b % P.PT; b /= P.PT;
    const int rb = b % P.RB;
    const int g = b / P.RB;

    const int q0 = pt * TQ;
    const int qend = min(q0 + TQ, P.QN);
    const int c_first = q0 / P.TI;
    const int n_first = c_first / P.Wo;
    const int u0 = (c_first - n_first * P.Wo) * P.Sw;      // chained column of the slab's first column, relative to image n_first
    const int row0 = rb * P.TI * P.Sh - P.Pt;              // input row of slab row 0
    const int HW = P.H * P.W;

    // input window of this block: images n_first.. ; channel 0 of group g
    const size_t in_base = ((size_t)n_first * P.Ctot + (size_t)g * P.Cg) * HW;
    const size_t in_total = (size_t)P.N * P.Ctot * HW;
    size_t in_left = (in_total - in_base) * 4;
    if (in_left > 0x7fffffffull) in_left = 0x7fffffffull;
    __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)(in + in_base), 0, (int)in_left, 0x00020000);

    // slab elements of this thread: byte offset (channel 0) or SLAB_INVALID
    unsigned goff[EPT];
#pragma unroll
    for (int s = 0; s < EPT; ++s) {
        const int e = tid + NT * s;
        const int col = e / SRP;
        const int r = e - col * SRP;
        const int U = u0 + col;
        const int ni = U / P.Wp;                 // image relative to n_first
        const int j = U - ni * P.Wp - P.Pl;
        const int i = row0 + r;
        const bool ok = e < CP && r < P.SR && i >= 0 && i < P.H && j >= 0 && j < P.W && (n_first + ni) < P.N;
        goff[s] = ok ? 4u * (unsigned)(i + P.H * j + ni * P.Ctot * HW) : SLAB_INVALID;
    }

    // pixels of this lane
    int bbase[MP];   // slab offset (floats) of the pixel's window origin, plus this lane's channel half
    int ooff[MP];    // output offset of (io, jo, k=0 of the array, n), or -1
#pragma unroll
    for (int mp = 0; mp < MP; ++mp) {
        const int q = q0 + (wp * MP + mp) * 32 + (lane & 31);
        const int ii = q % P.TI;
        const int c = q / P.TI;
        const int n = c / P.Wo;
        const int jo = c - n * P.Wo;
        const int io = rb * P.TI + ii;
        const bool ok = q < qend && io < P.Ho;
        const int ucol = jo * P.Sw + (n - n_first) * P.Wp - u0;
        bbase[mp] = (ok ? ii * P.Sh + SRP * ucol : 0) + (lane >> 5) * CP;
        ooff[mp] = ok ? io + P.Ho * (jo + P.Wo * (P.Ktot * n)) : -1;
    }

    // accumulators start at the bias of their filter (lane holds 16 filters of each filter tile)
    floatx16 acc[MK][MP];
#pragma unroll
    for (int mk = 0; mk < MK; ++mk)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int kl = kt * TK + (wk * MK + mk) * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
            const float bv = (bias && kl < P.Kg) ? bias[g * P.Kg + kl] : 0.f;
#pragma unroll
            for (int mp = 0; mp < MP; ++mp) acc[mk][mp][v] = bv;
        }

    const float *wsrc = wpk + ((size_t)(g * P.KT + kt) * P.NCH) * wchunk;
    floatx4 wreg[WPT];
    float xreg[DC][EPT];

    auto load_chunk = [&](int ch) {
        const floatx4 *src = reinterpret_cast<const floatx4 *>(wsrc + (size_t)ch * wchunk);
#pragma unroll
        for (int s = 0; s < WPT; ++s) {
            const int idx = tid + NT * s;
            if (idx < wchunk4) wreg[s] = src[idx];
        }
#pragma unroll
        for (int d = 0; d < DC; ++d) {
            const int c = ch * DC + d;
            const unsigned soff = (unsigned)c * (unsigned)HW * 4u;
#pragma unroll
            for (int s = 0; s < EPT; ++s) {
                float v = 0.f;
                if (c < P.Cg) v = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrc, goff[s], soff, 0));
                xreg[d][s] = v;
            }
        }
    };
    auto store_chunk = [&](float *wb, float *xb) {
        floatx4 *dst = reinterpret_cast<floatx4 *>(wb);
#pragma unroll
        for (int s = 0; s < WPT; ++s) {
            const int idx = tid + NT * s;
            if (idx < wchunk4) dst[idx] = wreg[s];
        }
#pragma unroll
        for (int d = 0; d < DC; ++d)
#pragma unroll
            for (int s = 0; s < EPT; ++s) {
                const int e = tid + NT * s;
                if (e < CP) xb[d * CP + e] = xreg[d][s];
            }
    };

    load_chunk(0);
    store_chunk(wbuf0, xbuf0);
    __syncthreads();

    const int aoff = (lane >> 5) * TK + wk * MK * 32 + (lane & 31);
    for (int ch = 0; ch < P.NCH; ++ch) {
        const bool more = ch + 1 < P.NCH;
        if (more) load_chunk(ch + 1);
        const float *wl = ((ch & 1) ? wbuf1 : wbuf0) + aoff;
        const float *xl = (ch & 1) ? xbuf1 : xbuf0;
        if constexpr (HF > 0) {
            // filter size known: the (channel pair, tap) steps of a chunk form one flat, fully unrolled
            // list; the LDS reads of step s+1 are issued before the MFMAs of step s.
            constexpr int TT = HF * WF;
            constexpr int NSTEP = (DC / 2) * TT;
            float a[2][MK], bb[2][MP];
            auto fetch = [&](int s, int slot) {
                const int dp = s / TT, tap = s % TT;
                const int fj = tap / HF, fi = tap % HF;
#pragma unroll
                for (int mk = 0; mk < MK; ++mk) a[slot][mk] = wl[((dp * TT + tap) * 2) * TK + mk * 32];
#pragma unroll
                for (int mp = 0; mp < MP; ++mp) bb[slot][mp] = xl[bbase[mp] + dp * 2 * CP + fj * SRP + fi];
            };
            fetch(0, 0);
#pragma unroll
            for (int s = 0; s < NSTEP; ++s) {
                if (s + 1 < NSTEP) fetch(s + 1, (s + 1) & 1);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int mk = 0; mk < MK; ++mk)
#pragma unroll
                    for (int mp = 0; mp < MP; ++mp)
                        acc[mk][mp] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[s & 1][mk], bb[s & 1][mp], acc[mk][mp], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
#pragma unroll
            for (int dp = 0; dp < DC / 2; ++dp) {
                for (int fj = 0; fj < Wf; ++fj) {
                    for (int fi = 0; fi < Hf; ++fi) {
                        const int tap = fi + Hf * fj;
                        float a[MK], bb[MP];
#pragma unroll
                        for (int mk = 0; mk < MK; ++mk) a[mk] = wl[((dp * T + tap) * 2) * TK + mk * 32];
#pragma unroll
                        for (int mp = 0; mp < MP; ++mp) bb[mp] = xl[bbase[mp] + dp * 2 * CP + fj * SRP + fi];
#pragma unroll
                        for (int mk = 0; mk < MK; ++mk)
#pragma unroll
                            for (int mp = 0; mp < MP; ++mp)
                                acc[mk][mp] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[mk], bb[mp], acc[mk][mp], 0, 0, 0);
                    }
                }
            }
        }
        if (more) store_chunk((ch & 1) ? wbuf0 : wbuf1, (ch & 1) ? xbuf0 : xbuf1);
        __syncthreads();
    }

    // epilogue: lane holds pixel (lane&31) of each pixel tile and 16 filters of each filter tile
    const int HoWo = P.Ho * P.Wo;
#pragma unroll
    for (int mk = 0; mk < MK; ++mk) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int kl = kt * TK + (wk * MK + mk) * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
            if (kl < P.Kg) {
                const int k = g * P.Kg + kl;
#pragma unroll
                for (int mp = 0; mp < MP; ++mp)
                    if (ooff[mp] >= 0) out[(size_t)ooff[mp] + (size_t)HoWo * k] = acc[mk][mp][v];
            }
        }
    }
}

}  // namespace mcn
