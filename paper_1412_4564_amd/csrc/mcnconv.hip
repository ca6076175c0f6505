// C-ABI entry points of the convolution library and the host-side dispatcher:
// argument checks, kernel choice, workspace layout, launches.  See include/mcnconv.h
// for the contract of every function.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <mutex>

#include "../../include/mcnconv.h"
#include "geom.h"
#include "kern_direct.h"
#include "kern_igemm.h"
#include "igemm_plan.h"
#include "kern_pool.h"
#include "kern_probe.h"

using namespace mcn;

namespace {

thread_local int g_last_hip_error = 0;

inline int check_launch() {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        g_last_hip_error = (int)e;
        return MCN_HIP_ERROR;
    }
    return MCN_OK;
}

inline unsigned cdiv(int64_t a, int64_t b) { return (unsigned)((a + b - 1) / b); }

// ---- bias derivative plan --------------------------------------------------
struct BiasPlan {
    bool rows;   // small output plane: threads run along the K*HoWo values of one image
    int chunks;  // chunks of BIAS_CHUNK samples per (n, k) plane
    int S;       // partial sums per filter (rows: per value of the image row)
    size_t ws_floats;
};

// dzdy is HoWo x K x N (plane, channels, images)
BiasPlan plan_bias(int64_t HoWo, int K, int N) {
    BiasPlan p;
    p.rows = HoWo < 64;
    if (p.rows) {
        const int64_t row = HoWo * K;
        int64_t want = 1024 / ((row + 255) / 256);     // aim for ~1024 blocks in all
        if (want > N) want = N;
        if (want < 1) want = 1;
        p.chunks = 0;
        p.S = (int)want;
        p.ws_floats = (size_t)p.S * (size_t)row;
        return p;
    }
    p.chunks = (int)((HoWo + BIAS_CHUNK - 1) / BIAS_CHUNK);
    const int64_t units = (int64_t)N * p.chunks;
    int64_t want = (2048 + K - 1) / K;   // aim for ~2048 blocks in all
    if (want > units) want = units;
    if (want < 1) want = 1;
    if (want > 65535) want = 65535;
    p.S = (int)want;
    p.ws_floats = (size_t)K * p.S;
    return p;
}
BiasPlan plan_bias(const Geom &g) { return plan_bias((int64_t)g.Ho * g.Wo, g.K, g.N); }

// ---- implicit-GEMM dispatch -------------------------------------------------
bool igemm_enabled() {
    static const bool off = getenv("MCN_FORCE_DIRECT") != nullptr;   // benchmarking / debugging override
    return !off;
}

// Number of compute units of the current device (the persistent kernels run one block per
// unit).  Falls back to the MI355X figure when no device can be asked, so that size queries
// work on a machine without a GPU.
int compute_units() {
    static int n = 0;
    if (n == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
            n = v;
        else
            n = 256;
        (void)hipGetLastError();
    }
    return n;
}

constexpr int MAX_PHASES = 64;
// blocks per shared tile in igemm_fixup_kernel (8 to 32 take the same time: the pass moves the pieces once)
constexpr int IGEMM_FIXUP_SLICES = 16;

// Plans depend only on the descriptor; planning walks candidate tilings, so the last few
// descriptors' plans are remembered per host thread (host memory only, no device state).
struct PlanEntry {
    mcn_conv_desc d;
    bool used;
    bool fwd_ok, bwd_ok, wg_ok;
    IgemmPlan fwd;
    int n_bwd;                 // stride phases of the input derivative that have work
    bool bwd_fill;             // some samples of dzdx belong to no phase with work: zero-fill first
    IgemmPlan bwd[MAX_PHASES];
    WgradPlan wg;
    bool wgb_ok;               // filter derivative on the bf16 kernel
    WgradBfPlan wgb;
    bool fc;                   // fully-connected layer: the three passes run as plain matrix products
    WgradPlan fc_fwd;
    IgemmPlan fc_bwd, fc_wg;
};
constexpr int PLAN_CACHE = 8;
thread_local PlanEntry g_plans[PLAN_CACHE];
thread_local int g_plan_next = 0;

inline size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

const PlanEntry *plans_for(const mcn_conv_desc *d, const Geom &g) {
    for (int i = 0; i < PLAN_CACHE; ++i)
        if (g_plans[i].used && memcmp(&g_plans[i].d, d, sizeof(*d)) == 0) return &g_plans[i];
    PlanEntry &e = g_plans[g_plan_next];
    g_plan_next = (g_plan_next + 1) % PLAN_CACHE;
    e.d = *d;
    e.used = true;
    const bool on = igemm_enabled();
    const int ncu = compute_units();
    // bf16 operands: the bf16 kernel where a view has at least one full MFMA depth of channels;
    // other views (and the filter derivative) compute in fp32, which meets the same error bound
    // the bf16 matrix core: operands rounded to bf16, or (MCN_PREC_FP32_BF16X3) split into two bf16 planes
    const bool bf = d->precision == MCN_PREC_BF16 || d->precision == MCN_PREC_FP32_BF16X3;
    const int planes = d->precision == MCN_PREC_FP32_BF16X3 ? 2 : 1;
    const bool pairs = d->precision != MCN_PREC_FP32_PLAIN;     // the row-pair kernels for 3x3 stride-1 layers
    auto plan_view = [&](const ConvView &v, IgemmPlan *pl) {
        if (bf && !v.mD && v.Cg >= BF_DC && plan_igemm(v, ncu, pl, true, true, planes)) return true;    // merged phases: fp32 kernel only
        return plan_igemm(v, ncu, pl, false, pairs);
    };
    e.fwd_ok = on && plan_view(forward_view(g), &e.fwd);
    e.bwd_ok = on && g.Sh * g.Sw <= MAX_PHASES;
    e.n_bwd = 0;
    e.bwd_fill = false;
    ConvView mv;
    if (on && merged_backward_data_view(g, &mv) && plan_view(mv, &e.bwd[0])) {
        e.bwd_ok = true;       // one launch computes every stride phase
        e.n_bwd = 1;
    } else if (e.bwd_ok) {
        for (int pj = 0; pj < g.Sw && e.bwd_ok; ++pj)
            for (int pi = 0; pi < g.Sh && e.bwd_ok; ++pi) {
                ConvView v;
                if (!backward_data_view(g, pi, pj, &v)) {
                    // no taps in this phase: its samples (if it has any) are zero
                    e.bwd_fill = true;
                    continue;
                }
                e.bwd_ok = plan_view(v, &e.bwd[e.n_bwd++]);
            }
    }
    e.wg_ok = on && ((pairs && wino_enabled() && plan_wgrad(forward_view(g), ncu, &e.wg, true)) ||
                     plan_wgrad(forward_view(g), ncu, &e.wg));
    e.wgb_ok = on && d->precision == MCN_PREC_BF16 && plan_wgrad_bf16(forward_view(g), ncu, &e.wgb);
    e.fc = on && is_fully_connected(g) && (int64_t)g.H * g.W * g.D < ((int64_t)1 << 30) &&
           plan_wgrad(fc_forward_view(g), ncu, &e.fc_fwd) && plan_igemm(fc_backward_data_view(g), ncu, &e.fc_bwd) &&
           plan_igemm(fc_backward_filter_view(g), ncu, &e.fc_wg);
    return &e;
}

// every block has four more waves that only fetch; blocks of four computing waves (IG_64x256) run two to a
// compute unit (16 waves per unit: the registers of a wave are capped at 128)
template <int WK, int WP, int MK, int MP, int HF, int WF, int DCF>
int launch_igemm_inst(const IgemmPlan &pl, const float *in, const float *wpk, const float *bias, float *out,
                      float *part, hipStream_t s, int relu) {
    IgemmParams P = pl.P;
    P.relu = relu;
    constexpr int LW = IGEMM_LOADER_WAVES;
    // waves per SIMD the registers must allow: two blocks of 4 + 4 waves (IG_64x256), else one of 8 + 4 or 4 + 4
    constexpr int WPE = (WK * WP == 4 && MK == 2) ? 4 : (WK * WP == 8 ? 3 : 2);
    auto kern = igemm_sk_kernel<WK, WP, MK, MP, HF, WF, DCF, WPE, LW>;
    if (pl.lds_bytes > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)pl.lds_bytes);
        if (e != hipSuccess) { g_last_hip_error = (int)e; return MCN_HIP_ERROR; }
    }
    hipLaunchKernelGGL(kern, dim3(P.nblocks), dim3(64 * (WK * WP + LW)), pl.lds_bytes, s, P, in, wpk, bias, out, part);
    int st = check_launch();
    // no tile is shared; tiles of a single unit cannot be cut, so every block's range holds whole tiles
    if (st || P.nblocks < 2 || P.own * P.nblocks == P.tiles || P.NU == 1) return st;
    constexpr int TK = WK * MK * 32, TQ = WP * MP * 32;
    hipLaunchKernelGGL((igemm_fixup_kernel<TK, TQ>), dim3(P.tiles - P.own * P.nblocks, IGEMM_FIXUP_SLICES), dim3(256), 0, s, P, part, bias, out);
    return check_launch();
}

// The WINO kernels (pairs of output rows, kern_igemm.h): 8 computing + 4 fetching waves, 128 accumulator
// registers per lane.  The fix-up pass sees the shared tiles in the output domain: rows instead of pairs.
template <int WK, int WP, int MK>
int launch_igemm_wino(const IgemmPlan &pl, const float *in, const float *wpk, const float *bias, float *out,
                      float *part, hipStream_t s, int relu) {
    IgemmParams P = pl.P;
    P.relu = relu;
    P.wino_pairs = P.osi == 2 && P.OH % 2 == 0 && ((uintptr_t)out & 7) == 0;
    constexpr int LW = IGEMM_LOADER_WAVES;
    auto kern = igemm_sk_kernel<WK, WP, MK, 1, IGEMM_WINO.HF, IGEMM_WINO.WF, IGEMM_WINO.DC, 3, LW, true>;
    if (pl.lds_bytes > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)pl.lds_bytes);
        if (e != hipSuccess) { g_last_hip_error = (int)e; return MCN_HIP_ERROR; }
    }
    hipLaunchKernelGGL(kern, dim3(P.nblocks), dim3(64 * (WK * WP + LW)), pl.lds_bytes, s, P, in, wpk, bias, out, part);
    int st = check_launch();
    if (st || P.nblocks < 2 || P.own * P.nblocks == P.tiles) return st;      // no tile is shared
    constexpr int TK = WK * MK * 32, TQ = WP * 32;
    IgemmParams F = P;
    F.TI = 2 * P.TI; F.QN = 2 * P.QN; F.Ho = P.wino_Ho; F.osi = P.osi / 2;
    F.dTI = make_div32(F.TI);
    hipLaunchKernelGGL((igemm_fixup_kernel<TK, 2 * TQ>), dim3(P.tiles - P.own * P.nblocks, IGEMM_FIXUP_SLICES), dim3(256), 0, s, F, part, bias, out);
    return check_launch();
}

// workspace of one view: [packed weights][partial tiles]
size_t igemm_ws_bytes(const IgemmPlan &pl) {
    return align256(pl.packed_floats * sizeof(float)) + pl.partial_floats * sizeof(float);
}

template <int WK, int WP, int MK, int MP, int PL = 1>
int launch_igemm_bf16_inst(const IgemmPlan &pl, const float *in, const float *wpk, const float *bias, float *out,
                           float *part, hipStream_t s, int relu) {
    if (PL == 1 && pl.planes == 2) return launch_igemm_bf16_inst<WK, WP, MK, MP, 2>(pl, in, wpk, bias, out, part, s, relu);
    IgemmParams P = pl.P;
    P.relu = relu;
    // one block per compute unit: 8 computing + 4 staging waves (3 per SIMD), or 4 + 4
    constexpr int LW = IGEMM_LOADER_WAVES;
    auto kern = igemm_bf16_kernel<WK, WP, MK, MP, WK * WP == 8 ? 3 : 2, LW, PL>;
    if (pl.lds_bytes > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)pl.lds_bytes);
        if (e != hipSuccess) { g_last_hip_error = (int)e; return MCN_HIP_ERROR; }
    }
    hipLaunchKernelGGL(kern, dim3(P.nblocks), dim3(64 * (WK * WP + LW)), pl.lds_bytes, s, P, in, wpk, bias, out, part);
    int st = check_launch();
    // no tile is shared; tiles of a single unit cannot be cut, so every block's range holds whole tiles
    if (st || P.nblocks < 2 || P.own * P.nblocks == P.tiles || P.NU == 1) return st;
    constexpr int TK = WK * MK * 32, TQ = WP * MP * 32;
    hipLaunchKernelGGL((igemm_fixup_kernel<TK, TQ>), dim3(P.tiles - P.own * P.nblocks, IGEMM_FIXUP_SLICES), dim3(256), 0, s, P, part, bias, out);
    return check_launch();
}

// one block shape, every instantiation of IGEMM_FIXED
template <int WK, int WP, int MK, int MP>
int launch_igemm_fixed(const IgemmPlan &pl, const float *in, const float *wpk, const float *bias, float *out,
                       float *part, hipStream_t s, int relu) {
    static_assert(IGEMM_N_FIXED == 4, "one case per entry of IGEMM_FIXED");
    switch (pl.fixed) {
        case 0: return launch_igemm_inst<WK, WP, MK, MP, 0, 0, 0>(pl, in, wpk, bias, out, part, s, relu);
        case 1: return launch_igemm_inst<WK, WP, MK, MP, IGEMM_FIXED[1].HF, IGEMM_FIXED[1].WF, IGEMM_FIXED[1].DC>(
                    pl, in, wpk, bias, out, part, s, relu);
        case 2: return launch_igemm_inst<WK, WP, MK, MP, IGEMM_FIXED[2].HF, IGEMM_FIXED[2].WF, IGEMM_FIXED[2].DC>(
                    pl, in, wpk, bias, out, part, s, relu);
        case 3: return launch_igemm_inst<WK, WP, MK, MP, IGEMM_FIXED[3].HF, IGEMM_FIXED[3].WF, IGEMM_FIXED[3].DC>(
                    pl, in, wpk, bias, out, part, s, relu);
        default: return MCN_BAD_ARG;
    }
}

int launch_igemm(const IgemmPlan &pl, const float *in, const float *w, const float *bias, float *out, void *ws,
                 hipStream_t s, int relu = 0) {
    float *packed = (float *)ws;
    float *part = (float *)((char *)ws + align256(pl.packed_floats * sizeof(float)));
    if (pl.bf16) {
        hipLaunchKernelGGL(igemm_pack_weights_bf16_kernel, dim3(cdiv(pl.Q.total, 256)), dim3(256), 0, s, w,
                           (unsigned *)packed, pl.Q);
        int st = check_launch();
        if (st) return st;
        switch (pl.shape) {
            case IG_128x256: return launch_igemm_bf16_inst<2, 4, 2, 2>(pl, in, packed, bias, out, part, s, relu);
            case IG_64x512: return launch_igemm_bf16_inst<1, 8, 2, 2>(pl, in, packed, bias, out, part, s, relu);
            case IG_32x256: return launch_igemm_bf16_inst<1, 4, 1, 2>(pl, in, packed, bias, out, part, s, relu);
            default: return MCN_BAD_ARG;
        }
    }
    if (pl.Q.wino && pl.P.WSZ != pl.Q.NS * 2 * pl.Q.TK) return MCN_BAD_ARG;      // the planner never pads these units
    if (pl.Q.wino)
        hipLaunchKernelGGL(igemm_pack_wino_kernel, dim3(cdiv(pl.Q.total / 4, 256)), dim3(256), 0, s, w, packed, pl.Q);
    else
        hipLaunchKernelGGL(igemm_pack_weights_kernel, dim3(cdiv(pl.Q.total, 256)), dim3(256), 0, s, w, packed, pl.Q);
    int st = check_launch();
    if (st) return st;
    switch (pl.shape) {
        case IG_128x256: return launch_igemm_fixed<2, 4, 2, 2>(pl, in, packed, bias, out, part, s, relu);
        case IG_64x512: return launch_igemm_fixed<1, 8, 2, 2>(pl, in, packed, bias, out, part, s, relu);
        case IG_32x256: return launch_igemm_fixed<1, 4, 1, 2>(pl, in, packed, bias, out, part, s, relu);
        case IG_64x256: return launch_igemm_fixed<1, 4, 2, 2>(pl, in, packed, bias, out, part, s, relu);
        case IG_96x256: return launch_igemm_fixed<1, 8, 3, 1>(pl, in, packed, bias, out, part, s, relu);
        case IG_W128x128: return launch_igemm_wino<2, 4, 2>(pl, in, packed, bias, out, part, s, relu);
        case IG_W64x256: return launch_igemm_wino<1, 8, 2>(pl, in, packed, bias, out, part, s, relu);
        default: return MCN_BAD_ARG;
    }
}

// The pass that adds the pieces of the tiles shared between blocks (kern_wgrad.h).  G partial sums per result: about
// the number of pieces per tile, at most 32; about 1024 blocks in all, none without work.
template <int TK, int TR>
int launch_wgrad_fixup(const WgradParams &P, const float *part, const float *rbias, float *out, hipStream_t s) {
    const bool chunked = P.nchunks > 0;
    const long long pieces = chunked ? P.nchunks : ((long long)P.nblocks + P.tiles - 1) / P.tiles + 1;
    int G = 2;
    while (G < 32 && G < pieces) G *= 2;
    const int Q = 512 / G;
    const int klim = P.Kg < TK ? P.Kg : TK, rlim = P.R < TR ? P.R : TR;
    const int passes = (klim * ((rlim + 3) / 4) + Q - 1) / Q;      // of the largest tile
    int fy = 1024 / P.tiles;
    if (fy < 1) fy = 1;
    if (fy > passes) fy = passes;
    if (chunked)
        hipLaunchKernelGGL((wgrad_fixup_kernel<TK, TR, true>), dim3(P.tiles, fy), dim3(512), 0, s, P, part, rbias, out, G);
    else
        hipLaunchKernelGGL((wgrad_fixup_kernel<TK, TR, false>), dim3(P.tiles, fy), dim3(512), 0, s, P, part, rbias, out, G);
    return check_launch();
}

// dzdb != NULL (BIAS instantiations only): the bias derivative is computed on the way (kern_wgrad.h); its partial
// sums follow the partial tiles in the workspace
template <int WK, int WR, int MK, int MR, bool S1, bool WINO = false, int WPE = 4, bool BIAS = false>
int launch_wgrad_inst2(const WgradPlan &pl, const float *x, const float *dzdy, const float *rbias, float *out,
                       float *part, hipStream_t s, int relu, float *dzdb = nullptr) {
    WgradParams P = pl.P;
    P.relu = relu;
    // WPE = waves per SIMD the registers must allow: 4 for two blocks of 4 + 4 waves per compute unit or one of 12 + 4,
    // 3 for one block of 8 + 4
    auto kern = wgrad_sk_kernel<WK, WR, MK, MR, S1, WPE, WINO, BIAS>;
    float *bpart = part + pl.partial_floats;
    if (pl.lds_bytes > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)pl.lds_bytes);
        if (e != hipSuccess) { g_last_hip_error = (int)e; return MCN_HIP_ERROR; }
    }
    const bool chunked = P.nchunks > 0;
    hipLaunchKernelGGL(kern, dim3(chunked ? wg_chunk_grid(P.nblocks) : P.nblocks),
                       dim3(64 * (WK * WR + WGRAD_LOADER_WAVES)), pl.lds_bytes, s, P,
                       x, dzdy, rbias, out, part, bpart);
    int st = check_launch();
    if constexpr (BIAS) {
        if (st) return st;
        hipLaunchKernelGGL((wgrad_bias_final_kernel<WK * MK * 32>), dim3(P.G * P.KT), dim3(1024), 0, s, P, bpart, dzdb);
        st = check_launch();
    }
    if (st || P.nblocks < 2 || P.nchunks == 1) return st;
    constexpr int TK = WK * MK * 32, TR = WR * MR * 32 * (WINO ? 3 : 1);     // coefficients per tile
    return launch_wgrad_fixup<TK, TR>(P, part, rbias, out, s);
}

template <int WK, int WR, int MK, int MR>
int launch_wgrad_inst(const WgradPlan &pl, const float *x, const float *dzdy, const float *rbias, float *out,
                      float *part, hipStream_t s, int relu) {
    return pl.P.Sh == 1 ? launch_wgrad_inst2<WK, WR, MK, MR, true>(pl, x, dzdy, rbias, out, part, s, relu)
                        : launch_wgrad_inst2<WK, WR, MK, MR, false>(pl, x, dzdy, rbias, out, part, s, relu);
}

// The filter derivative can leave the bias derivative as a by-product: the WINO kernels on the chunked schedule
// (every block then holds one piece of one tile)
bool wgrad_gives_bias(const WgradPlan &pl) { return pl.wino && pl.P.nchunks > 0; }
size_t wgrad_bias_floats(const WgradPlan &pl) { return (size_t)2 * pl.P.nblocks * pl.TK; }

int launch_wgrad(const WgradPlan &pl, const float *x, const float *dzdy, const float *rbias, float *out, void *ws,
                 hipStream_t s, int relu = 0, float *dzdb = nullptr) {
    float *part = (float *)ws;
    if (dzdb) {
        if (!wgrad_gives_bias(pl)) return MCN_BAD_ARG;
        if (pl.shape == WG_W128x128)
            return launch_wgrad_inst2<2, 4, 2, 1, true, true, 3, true>(pl, x, dzdy, rbias, out, part, s, relu, dzdb);
        return launch_wgrad_inst2<2, 6, 1, 1, true, true, 4, true>(pl, x, dzdy, rbias, out, part, s, relu, dzdb);
    }
    switch (pl.shape) {
        case WG_128x128: return launch_wgrad_inst<2, 2, 2, 2>(pl, x, dzdy, rbias, out, part, s, relu);
        case WG_64x192: return launch_wgrad_inst<2, 2, 1, 3>(pl, x, dzdy, rbias, out, part, s, relu);
        case WG_32x256: return launch_wgrad_inst<1, 4, 1, 2>(pl, x, dzdy, rbias, out, part, s, relu);
        case WG_96x128: return launch_wgrad_inst<1, 4, 3, 1>(pl, x, dzdy, rbias, out, part, s, relu);
        case WG_96x384: return launch_wgrad_inst<3, 4, 1, 3>(pl, x, dzdy, rbias, out, part, s, relu);
        case WG_W128x128: return launch_wgrad_inst2<2, 4, 2, 1, true, true, 3>(pl, x, dzdy, rbias, out, part, s, relu);
        case WG_W64x192: return launch_wgrad_inst2<2, 6, 1, 1, true, true, 4>(pl, x, dzdy, rbias, out, part, s, relu);
        default: return MCN_BAD_ARG;
    }
}

template <int WK, int WR, int MK, int MR, int HF>
int launch_wgrad_bf16_inst(const WgradBfPlan &pl, const float *x, const float *dzdy, float *out, float *part,
                           hipStream_t s) {
    auto kern = wgrad_bf16_kernel<WK, WR, MK, MR, HF>;
    if (pl.lds_bytes > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)pl.lds_bytes);
        if (e != hipSuccess) { g_last_hip_error = (int)e; return MCN_HIP_ERROR; }
    }
    hipLaunchKernelGGL(kern, dim3(wgb_grid(pl.P.nblocks)), dim3(64 * WK * WR), pl.lds_bytes, s, pl.P, x, dzdy, out, part);
    int st = check_launch();
    if (st || pl.P.nchunks < 2) return st;
    constexpr int TK = WK * MK * 32, TR = WR * MR * 32;
    int fy = 2048 / pl.P.tiles;          // about 2048 blocks in all
    if (fy < 1) fy = 1;
    if (fy > TK * TR / 64) fy = TK * TR / 64;
    hipLaunchKernelGGL((wgrad_bf16_fixup_kernel<TK, TR>), dim3(pl.P.tiles, fy), dim3(512), 0, s, pl.P, part, out);
    return check_launch();
}

template <int WK, int WR, int MK, int MR>
int launch_wgrad_bf16_shape(const WgradBfPlan &pl, const float *x, const float *dzdy, float *out, float *part,
                            hipStream_t s) {
    switch (pl.P.Hf) {
        case 1: return launch_wgrad_bf16_inst<WK, WR, MK, MR, 1>(pl, x, dzdy, out, part, s);
        case 2: return launch_wgrad_bf16_inst<WK, WR, MK, MR, 2>(pl, x, dzdy, out, part, s);
        case 3: return launch_wgrad_bf16_inst<WK, WR, MK, MR, 3>(pl, x, dzdy, out, part, s);
        case 4: return launch_wgrad_bf16_inst<WK, WR, MK, MR, 4>(pl, x, dzdy, out, part, s);
        case 5: return launch_wgrad_bf16_inst<WK, WR, MK, MR, 5>(pl, x, dzdy, out, part, s);
        default: return MCN_BAD_ARG;
    }
}

int launch_wgrad_bf16(const WgradBfPlan &pl, const float *x, const float *dzdy, float *out, void *ws, hipStream_t s) {
    float *part = (float *)ws;
    switch (pl.shape) {
        case WGB_128x256: return launch_wgrad_bf16_shape<2, 4, 2, 2>(pl, x, dzdy, out, part, s);
        case WGB_64x256: return launch_wgrad_bf16_shape<2, 4, 1, 2>(pl, x, dzdy, out, part, s);
        default: return MCN_BAD_ARG;
    }
}

size_t workspace_bytes(const mcn_conv_desc *d, const Geom &g, int op) {
    const PlanEntry *e = plans_for(d, g);
    switch (op) {
        case MCN_OP_BACKWARD_BIAS: {
            return plan_bias(g).ws_floats * sizeof(float);
        }
        case MCN_OP_FORWARD:
            if (e->fc) return e->fc_fwd.partial_floats * sizeof(float);
            return e->fwd_ok ? igemm_ws_bytes(e->fwd) : 0;
        case MCN_OP_BACKWARD_DATA: {
            if (e->fc) return igemm_ws_bytes(e->fc_bwd);
            // the phases run one after the other on the stream and share one region
            size_t m = 0;
            if (e->bwd_ok)
                for (int i = 0; i < e->n_bwd; ++i) { size_t b = igemm_ws_bytes(e->bwd[i]); if (b > m) m = b; }
            return m;
        }
        case MCN_OP_BACKWARD_FILTER:
            if (e->fc) return igemm_ws_bytes(e->fc_wg);
            if (e->wgb_ok) return e->wgb.partial_floats * sizeof(float);
            return e->wg_ok ? e->wg.partial_floats * sizeof(float) : 0;
        case MCN_OP_BACKWARD_FILTER_BIAS: {
            // fused: the filter derivative's scratch and the partial bias sums; otherwise the two passes one
            // after the other in the same region
            const size_t f = workspace_bytes(d, g, MCN_OP_BACKWARD_FILTER), b = workspace_bytes(d, g, MCN_OP_BACKWARD_BIAS);
            if (!e->fc && !e->wgb_ok && e->wg_ok && wgrad_gives_bias(e->wg)) return f + wgrad_bias_floats(e->wg) * sizeof(float);
            return f > b ? f : b;
        }
        default:
            return 0;
    }
}

// ---- the four passes on a validated geometry ---------------------------------------------

int run_forward(const mcn_conv_desc *desc, const Geom &g, const float *x, const float *w, const float *b, float *y,
                void *ws, size_t ws_bytes, hipStream_t s, int relu = 0) {
    if (!x || !w || !y) return MCN_BAD_ARG;
    const size_t need = workspace_bytes(desc, g, MCN_OP_FORWARD);
    if (ws_bytes < need || (!ws && need)) return MCN_WORKSPACE_TOO_SMALL;
    const PlanEntry *pe = plans_for(desc, g);
    if (pe->fc) return launch_wgrad(pe->fc_fwd, w, x, b, y, ws, s, relu);
    if (pe->fwd_ok) return launch_igemm(pe->fwd, x, w, b, y, ws, s, relu);
    const int total = (int)numel_y(g);
    hipLaunchKernelGGL(direct_forward_kernel, dim3(cdiv(total, 256)), dim3(256), 0, s, g, x, w, b, y, total, relu);
    return check_launch();
}

// dzdx = (input derivative) + bias[channel of x]; the bias (may be NULL) is what turns this pass
// into the forward pass of the convolution transpose.
int run_backward_data(const mcn_conv_desc *desc, const Geom &g, const float *w, const float *dzdy, const float *bias,
                      float *dzdx, void *ws, size_t ws_bytes, hipStream_t s) {
    if (!w || !dzdy || !dzdx) return MCN_BAD_ARG;
    const size_t need = workspace_bytes(desc, g, MCN_OP_BACKWARD_DATA);
    if (ws_bytes < need || (!ws && need)) return MCN_WORKSPACE_TOO_SMALL;
    const PlanEntry *pe = plans_for(desc, g);
    const int total = (int)numel_x(g);
    int st;
    if (pe->bwd_ok && !pe->fc) {
        if (pe->bwd_fill) {
            if (bias)
                hipLaunchKernelGGL(bias_fill_kernel, dim3(cdiv(total, 1024)), dim3(256), 0, s, dzdx, bias, g.H * g.W, g.D, total);
            else
                hipLaunchKernelGGL(zero_fill_kernel, dim3(cdiv(total, 1024)), dim3(256), 0, s, dzdx, total);
            st = check_launch();
            if (st) return st;
        }
        for (int i = 0; i < pe->n_bwd; ++i) {
            st = launch_igemm(pe->bwd[i], dzdy, w, bias, dzdx, ws, s);
            if (st) return st;
        }
        return MCN_OK;
    }
    if (pe->fc) {
        st = launch_igemm(pe->fc_bwd, w, dzdy, nullptr, dzdx, ws, s);
    } else {
        hipLaunchKernelGGL(direct_backward_data_kernel, dim3(cdiv(total, 256)), dim3(256), 0, s, g, w, dzdy, dzdx, total);
        st = check_launch();
    }
    if (st || !bias) return st;
    hipLaunchKernelGGL(bias_add_kernel, dim3(cdiv(total, 1024)), dim3(256), 0, s, dzdx, bias, g.H * g.W, g.D, total);
    return check_launch();
}

int run_backward_filter(const mcn_conv_desc *desc, const Geom &g, const float *x, const float *dzdy, float *dzdw,
                        void *ws, size_t ws_bytes, hipStream_t s) {
    if (!x || !dzdy || !dzdw) return MCN_BAD_ARG;
    const size_t need = workspace_bytes(desc, g, MCN_OP_BACKWARD_FILTER);
    if (ws_bytes < need || (!ws && need)) return MCN_WORKSPACE_TOO_SMALL;
    const PlanEntry *pe = plans_for(desc, g);
    if (pe->fc) return launch_igemm(pe->fc_wg, x, dzdy, nullptr, dzdw, ws, s);
    if (pe->wgb_ok) return launch_wgrad_bf16(pe->wgb, x, dzdy, dzdw, ws, s);
    if (pe->wg_ok) return launch_wgrad(pe->wg, x, dzdy, nullptr, dzdw, ws, s);
    const int total = (int)numel_w(g);
    hipLaunchKernelGGL(direct_backward_filter_kernel, dim3(cdiv(total, 4)), dim3(256), 0, s, g, x, dzdy, dzdw, total);
    return check_launch();
}

int run_backward_bias(int plane, int K, int N, const float *dzdy, float *dzdb, void *ws, size_t ws_bytes,
                      hipStream_t s, const float *y = nullptr, float *dzdp = nullptr);

// dzdw and dzdb in one call: one kernel where the filter derivative's kernel sums dzdy on the way, else the two passes
int run_backward_filter_bias(const mcn_conv_desc *desc, const Geom &g, const float *x, const float *dzdy, float *dzdw,
                             float *dzdb, void *ws, size_t ws_bytes, hipStream_t s) {
    if (!x || !dzdy || !dzdw || !dzdb) return MCN_BAD_ARG;
    const size_t need = workspace_bytes(desc, g, MCN_OP_BACKWARD_FILTER_BIAS);
    if (ws_bytes < need || (!ws && need)) return MCN_WORKSPACE_TOO_SMALL;
    const PlanEntry *pe = plans_for(desc, g);
    if (!pe->fc && !pe->wgb_ok && pe->wg_ok && wgrad_gives_bias(pe->wg))
        return launch_wgrad(pe->wg, x, dzdy, nullptr, dzdw, ws, s, 0, dzdb);
    const int st = run_backward_filter(desc, g, x, dzdy, dzdw, ws, ws_bytes, s);
    if (st) return st;
    return run_backward_bias(g.Ho * g.Wo, g.K, g.N, dzdy, dzdb, ws, ws_bytes, s, nullptr, nullptr);
}

// dzdb[k] = sum of the plane x K x N array dzdy over its plane and its images.  With y (and dzdp):
// dzdp = [y > 0] * dzdy is written in the same pass and summed instead.
int run_backward_bias(int plane, int K, int N, const float *dzdy, float *dzdb, void *ws, size_t ws_bytes,
                      hipStream_t s, const float *y, float *dzdp) {
    if (!dzdy || !dzdb) return MCN_BAD_ARG;
    const BiasPlan p = plan_bias(plane, K, N);
    const size_t need = p.ws_floats * sizeof(float);
    if (ws_bytes < need || (!ws && need)) return MCN_WORKSPACE_TOO_SMALL;
    float *part = (float *)ws;
    int st;
    if (p.rows) {
        const int row = K * plane;
        if (y)
            hipLaunchKernelGGL(relu_bias_rows_partial_kernel, dim3(cdiv(row, 256), p.S), dim3(256), 0, s, y, dzdy, dzdp, part, row, N, p.S);
        else
            hipLaunchKernelGGL(bias_rows_partial_kernel, dim3(cdiv(row, 256), p.S), dim3(256), 0, s, dzdy, part, row, N, p.S);
        st = check_launch();
        if (st) return st;
        hipLaunchKernelGGL(bias_rows_final_kernel, dim3(cdiv(K, 4)), dim3(256), 0, s, part, dzdb, plane, K, p.S);
        return check_launch();
    }
    if (y)
        hipLaunchKernelGGL(relu_bias_partial_kernel, dim3(K, p.S), dim3(256), 0, s, y, dzdy, dzdp, part, plane, K, N, p.chunks, p.S);
    else if (plane % 4 == 0 && plane >= 1024 && ((uintptr_t)dzdy & 15) == 0)     // planes that fill a block's 16-byte loads
        hipLaunchKernelGGL(bias_partial_v4_kernel, dim3(K, p.S), dim3(256), 0, s, dzdy, part, plane, K, N, p.chunks, p.S);
    else
        hipLaunchKernelGGL(bias_partial_kernel, dim3(K, p.S), dim3(256), 0, s, dzdy, part, plane, K, N, p.chunks, p.S);
    st = check_launch();
    if (st) return st;
    hipLaunchKernelGGL(bias_final_kernel, dim3(cdiv(K, 256)), dim3(256), 0, s, part, dzdb, K, p.S);
    return check_launch();
}

// Convolution transpose (Sec. 4.2): validate the descriptor and write the "conjugate"
// convolution, the one that maps an array of y's shape to one of x's shape with the same bank
// (stride = upsampling, pads = crops).  In the conjugate's terms its input is H'' x W'' x
// groups*K', its bank has D filters of depth K', and its output is H x W x D.
int conjugate_convolution(const mcn_convt_desc *t, mcn_conv_desc *c, Geom *g) {
    if (!t) return MCN_BAD_ARG;
    if (t->H < 1 || t->W < 1 || t->D < 1 || t->N < 1) return MCN_BAD_ARG;
    if (t->Hf < 1 || t->Wf < 1 || t->Kf < 1 || t->groups < 1) return MCN_BAD_ARG;
    if (t->up_h < 1 || t->up_w < 1) return MCN_BAD_ARG;
    if (t->crop_top < 0 || t->crop_bottom < 0 || t->crop_left < 0 || t->crop_right < 0) return MCN_BAD_ARG;
    if (t->precision < MCN_PREC_FP32 || t->precision > MCN_PREC_FP32_BF16X3) return MCN_BAD_ARG;
    if (t->D % t->groups != 0) return MCN_BAD_GROUPS;
    const int64_t lim = (int64_t)1 << 31;
    const int64_t Ho = (int64_t)t->up_h * (t->H - 1) + t->Hf - t->crop_top - t->crop_bottom;
    const int64_t Wo = (int64_t)t->up_w * (t->W - 1) + t->Wf - t->crop_left - t->crop_right;
    if (Ho < 1 || Wo < 1) return MCN_CROP_TOO_LARGE;
    if (Ho >= lim || Wo >= lim || (int64_t)t->groups * t->Kf >= lim) return MCN_UNSUPPORTED;
    memset(c, 0, sizeof(*c));
    c->H = (int32_t)Ho; c->W = (int32_t)Wo; c->D = t->groups * t->Kf; c->N = t->N;
    c->Hf = t->Hf; c->Wf = t->Wf; c->Df = t->Kf; c->K = t->D;
    c->stride_h = t->up_h; c->stride_w = t->up_w;
    c->pad_top = t->crop_top; c->pad_bottom = t->crop_bottom; c->pad_left = t->crop_left; c->pad_right = t->crop_right;
    c->precision = t->precision;
    return make_geom(c, g);
}

}  // namespace

extern "C" {

int mcn_conv_output_size(const mcn_conv_desc *desc, int32_t *Ho, int32_t *Wo) {
    Geom g;
    int st = make_geom(desc, &g);
    if (st) return st;
    if (Ho) *Ho = g.Ho;
    if (Wo) *Wo = g.Wo;
    return MCN_OK;
}

int mcn_conv_workspace_size(const mcn_conv_desc *desc, int op, size_t *bytes) {
    Geom g;
    int st = make_geom(desc, &g);
    if (st) return st;
    if (!bytes || op < MCN_OP_FORWARD || op > MCN_OP_BACKWARD_FILTER_BIAS) return MCN_BAD_ARG;
    *bytes = workspace_bytes(desc, g, op);
    return MCN_OK;
}

static const char *igemm_name(const IgemmPlan &pl) {
    return pl.bf16 ? (pl.planes == 2 ? "igemm_bf16x3" : "igemm_bf16") : pl.P.wino_Ho ? "igemm_f23" : "igemm";
}

const char *mcn_conv_kernel_name(const mcn_conv_desc *desc, int op) {
    Geom g;
    if (make_geom(desc, &g)) return NULL;
    const PlanEntry *e = plans_for(desc, g);
    switch (op) {
        case MCN_OP_FORWARD:
            return e->fc ? "fc_gemm" : e->fwd_ok ? igemm_name(e->fwd) : "direct";
        case MCN_OP_BACKWARD_DATA:
            return e->fc ? "fc_gemm" : e->bwd_ok ? (e->n_bwd ? igemm_name(e->bwd[0]) : "igemm") : "direct";
        case MCN_OP_BACKWARD_FILTER:
            if (e->fc) return "fc_gemm";
            if (e->wgb_ok) return "wgrad_bf16";
            if (!e->wg_ok) return "direct";
            // "_chunked": the schedule for arrays that stream from memory (kern_wgrad.h, WgradParams::nchunks)
            if (e->wg.P.nchunks > 0) return e->wg.wino ? "wgrad_f23_chunked" : "wgrad_igemm_chunked";
            return e->wg.wino ? "wgrad_f23" : "wgrad_igemm";
        case MCN_OP_BACKWARD_BIAS: return plan_bias(g).rows ? "reduce_rows" : "reduce2";
        case MCN_OP_BACKWARD_FILTER_BIAS:
            return !e->fc && !e->wgb_ok && e->wg_ok && wgrad_gives_bias(e->wg) ? "wgrad_f23+bias" : "two passes";
        default: return NULL;
    }
}

int mcn_conv_forward(const mcn_conv_desc *desc, const float *x, const float *w, const float *b, float *y,
                     void *ws, size_t ws_bytes, void *stream) {
    Geom g;
    int st = make_geom(desc, &g);
    if (st) return st;
    return run_forward(desc, g, x, w, b, y, ws, ws_bytes, (hipStream_t)stream);
}

int mcn_conv_backward_data(const mcn_conv_desc *desc, const float *w, const float *dzdy, float *dzdx,
                           void *ws, size_t ws_bytes, void *stream) {
    Geom g;
    int st = make_geom(desc, &g);
    if (st) return st;
    return run_backward_data(desc, g, w, dzdy, nullptr, dzdx, ws, ws_bytes, (hipStream_t)stream);
}

int mcn_conv_backward_filter(const mcn_conv_desc *desc, const float *x, const float *dzdy, float *dzdw,
                             void *ws, size_t ws_bytes, void *stream) {
    Geom g;
    int st = make_geom(desc, &g);
    if (st) return st;
    return run_backward_filter(desc, g, x, dzdy, dzdw, ws, ws_bytes, (hipStream_t)stream);
}

int mcn_conv_backward_filter_bias(const mcn_conv_desc *desc, const float *x, const float *dzdy, float *dzdw,
                                  float *dzdb, void *ws, size_t ws_bytes, void *stream) {
    Geom g;
    int st = make_geom(desc, &g);
    if (st) return st;
    return run_backward_filter_bias(desc, g, x, dzdy, dzdw, dzdb, ws, ws_bytes, (hipStream_t)stream);
}

int mcn_conv_backward_bias(const mcn_conv_desc *desc, const float *dzdy, float *dzdb, void *ws, size_t ws_bytes,
                           void *stream) {
    Geom g;
    int st = make_geom(desc, &g);
    if (st) return st;
    return run_backward_bias(g.Ho * g.Wo, g.K, g.N, dzdy, dzdb, ws, ws_bytes, (hipStream_t)stream);
}

// ---- the bias derivative for callers that cannot allocate ------------------------------------
// Its partial sums go to an array that is part of the library's code object, so that the call needs neither a
// workspace argument nor an allocation.  In host code the array's name is only a handle: its address on the
// current device is asked once per device (hipGetSymbolAddress) and kept.
static __device__ __align__(256) float scratch[MCN_STATIC_SCRATCH_BYTES / sizeof(float)];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
float *g_scratch_ptr[MAX_DEVICES];      // per device: where `scratch` lives there (NULL until first asked)

// Address of `scratch` on the current device; NULL (and the HIP error recorded) on failure.
float *static_scratch() {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess && (dev < 0 || dev >= MAX_DEVICES)) e = hipErrorInvalidDevice;
    if (e != hipSuccess) { g_last_hip_error = (int)e; return nullptr; }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) { g_last_hip_error = (int)(e != hipSuccess ? e : hipErrorInvalidSymbol); return nullptr; }
        g_scratch_ptr[dev] = (float *)p;
    }
    return g_scratch_ptr[dev];
}
}  // namespace

int mcn_conv_backward_bias_static(const mcn_conv_desc *desc, const float *dzdy, float *dzdb, void *stream) {
    Geom g;
    int st = make_geom(desc, &g);
    if (st) return st;
    if (!dzdy || !dzdb) return MCN_BAD_ARG;
    if (plan_bias(g).ws_floats * sizeof(float) > (size_t)MCN_STATIC_SCRATCH_BYTES) return MCN_STATIC_SCRATCH_EXCEEDED;
    float *ptr = static_scratch();
    if (!ptr) return MCN_HIP_ERROR;
    // every partial sum the second stage reads is written by the first: nothing in the array needs clearing
    return run_backward_bias(g.Ho * g.Wo, g.K, g.N, dzdy, dzdb, ptr, MCN_STATIC_SCRATCH_BYTES, (hipStream_t)stream);
}

// ---- convolution + ReLU ------------------------------------------------------------------

int mcn_conv_relu_forward(const mcn_conv_desc *desc, const float *x, const float *w, const float *b, float *y,
                          void *ws, size_t ws_bytes, void *stream) {
    Geom g;
    int st = make_geom(desc, &g);
    if (st) return st;
    return run_forward(desc, g, x, w, b, y, ws, ws_bytes, (hipStream_t)stream, 1);
}

int mcn_conv_relu_backward_bias(const mcn_conv_desc *desc, const float *y, const float *dzdy, float *dzdp, float *dzdb,
                                void *ws, size_t ws_bytes, void *stream) {
    Geom g;
    int st = make_geom(desc, &g);
    if (st) return st;
    if (!y || !dzdp) return MCN_BAD_ARG;
    return run_backward_bias(g.Ho * g.Wo, g.K, g.N, dzdy, dzdb, ws, ws_bytes, (hipStream_t)stream, y, dzdp);
}

// ---- convolution transpose: the same kernels with the roles of the arrays exchanged ----------

int mcn_convt_output_size(const mcn_convt_desc *desc, int32_t *Ho, int32_t *Wo) {
    mcn_conv_desc c;
    Geom g;
    int st = conjugate_convolution(desc, &c, &g);
    if (st) return st;
    if (Ho) *Ho = c.H;
    if (Wo) *Wo = c.W;
    return MCN_OK;
}

int mcn_convt_workspace_size(const mcn_convt_desc *desc, int op, size_t *bytes) {
    mcn_conv_desc c;
    Geom g;
    int st = conjugate_convolution(desc, &c, &g);
    if (st) return st;
    if (!bytes || op < MCN_OP_FORWARD || op > MCN_OP_BACKWARD_BIAS) return MCN_BAD_ARG;
    switch (op) {
        case MCN_OP_FORWARD: *bytes = workspace_bytes(&c, g, MCN_OP_BACKWARD_DATA); break;
        case MCN_OP_BACKWARD_DATA: *bytes = workspace_bytes(&c, g, MCN_OP_FORWARD); break;
        case MCN_OP_BACKWARD_FILTER: *bytes = workspace_bytes(&c, g, MCN_OP_BACKWARD_FILTER); break;
        default: *bytes = plan_bias((int64_t)g.H * g.W, g.D, g.N).ws_floats * sizeof(float); break;
    }
    return MCN_OK;
}

const char *mcn_convt_kernel_name(const mcn_convt_desc *desc, int op) {
    mcn_conv_desc c;
    Geom g;
    if (conjugate_convolution(desc, &c, &g)) return NULL;
    switch (op) {
        case MCN_OP_FORWARD: return mcn_conv_kernel_name(&c, MCN_OP_BACKWARD_DATA);
        case MCN_OP_BACKWARD_DATA: return mcn_conv_kernel_name(&c, MCN_OP_FORWARD);
        case MCN_OP_BACKWARD_FILTER: return mcn_conv_kernel_name(&c, MCN_OP_BACKWARD_FILTER);
        case MCN_OP_BACKWARD_BIAS: return plan_bias((int64_t)g.H * g.W, g.D, g.N).rows ? "reduce_rows" : "reduce2";
        default: return NULL;
    }
}

int mcn_convt_forward(const mcn_convt_desc *desc, const float *x, const float *f, const float *b, float *y,
                      void *ws, size_t ws_bytes, void *stream) {
    mcn_conv_desc c;
    Geom g;
    int st = conjugate_convolution(desc, &c, &g);
    if (st) return st;
    // y = M^T x + b: the input derivative of the conjugate convolution, taken at "dzdy" = x
    return run_backward_data(&c, g, f, x, b, y, ws, ws_bytes, (hipStream_t)stream);
}

int mcn_convt_backward_data(const mcn_convt_desc *desc, const float *f, const float *dzdy, float *dzdx,
                            void *ws, size_t ws_bytes, void *stream) {
    mcn_conv_desc c;
    Geom g;
    int st = conjugate_convolution(desc, &c, &g);
    if (st) return st;
    // dzdx = M dzdy: the conjugate convolution itself, without a bias
    return run_forward(&c, g, dzdy, f, nullptr, dzdx, ws, ws_bytes, (hipStream_t)stream);
}

int mcn_convt_backward_filter(const mcn_convt_desc *desc, const float *x, const float *dzdy, float *dzdf,
                              void *ws, size_t ws_bytes, void *stream) {
    mcn_conv_desc c;
    Geom g;
    int st = conjugate_convolution(desc, &c, &g);
    if (st) return st;
    // <dzdy, M^T x> = <M dzdy, x>: the filter derivative of the conjugate convolution whose input is
    // dzdy and whose output derivative is x
    return run_backward_filter(&c, g, dzdy, x, dzdf, ws, ws_bytes, (hipStream_t)stream);
}

int mcn_convt_backward_bias(const mcn_convt_desc *desc, const float *dzdy, float *dzdb, void *ws, size_t ws_bytes,
                            void *stream) {
    mcn_conv_desc c;
    Geom g;
    int st = conjugate_convolution(desc, &c, &g);
    if (st) return st;
    return run_backward_bias(g.H * g.W, g.D, g.N, dzdy, dzdb, ws, ws_bytes, (hipStream_t)stream);
}

// ---- spatial pooling -------------------------------------------------------------------

static int make_pool_geom(const mcn_pool_desc *d, PoolGeom *g) {
    if (!d) return MCN_BAD_ARG;
    if (d->H < 1 || d->W < 1 || d->D < 1 || d->N < 1) return MCN_BAD_ARG;
    if (d->Hp < 1 || d->Wp < 1 || d->stride_h < 1 || d->stride_w < 1) return MCN_BAD_ARG;
    if (d->pad_top < 0 || d->pad_bottom < 0 || d->pad_left < 0 || d->pad_right < 0) return MCN_BAD_ARG;
    if (d->method != MCN_POOL_MAX && d->method != MCN_POOL_AVG) return MCN_BAD_ARG;
    if (d->pad_top > d->Hp - 1 || d->pad_bottom > d->Hp - 1 || d->pad_left > d->Wp - 1 || d->pad_right > d->Wp - 1)
        return MCN_PAD_TOO_LARGE;
    const int64_t hp = (int64_t)d->H + d->pad_top + d->pad_bottom, wp = (int64_t)d->W + d->pad_left + d->pad_right;
    if (hp < d->Hp || wp < d->Wp) return MCN_FILTER_TOO_LARGE;
    const int64_t Ho = (hp - d->Hp) / d->stride_h + 1, Wo = (wp - d->Wp) / d->stride_w + 1;
    const double lim = 2147483648.0;
    if ((double)d->H * d->W * d->D * d->N >= lim || (double)Ho * Wo * d->D * d->N >= lim) return MCN_UNSUPPORTED;
    // window and stride sizes the kernels' 32-bit index arithmetic is written for
    if (d->Hp >= 32768 || d->Wp >= 32768 || d->stride_h >= 32768 || d->stride_w >= 32768) return MCN_UNSUPPORTED;
    g->H = d->H; g->W = d->W; g->D = d->D; g->N = d->N;
    g->Hp = d->Hp; g->Wp = d->Wp; g->Sh = d->stride_h; g->Sw = d->stride_w; g->Pt = d->pad_top; g->Pl = d->pad_left;
    g->Ho = (int)Ho; g->Wo = (int)Wo; g->method = d->method;
    g->dH = make_div32(d->H); g->dHo = make_div32((int)Ho);
    g->dSh = make_div32(d->stride_h); g->dSw = make_div32(d->stride_w);
    g->dIn = make_fastdiv64((unsigned)(d->H * d->W)); g->dOut = make_fastdiv64((unsigned)(Ho * Wo));
    return MCN_OK;
}

int mcn_pool_output_size(const mcn_pool_desc *desc, int32_t *Ho, int32_t *Wo) {
    PoolGeom g;
    int st = make_pool_geom(desc, &g);
    if (st) return st;
    if (Ho) *Ho = g.Ho;
    if (Wo) *Wo = g.Wo;
    return MCN_OK;
}

int mcn_pool_forward(const mcn_pool_desc *desc, const float *x, float *y, void *stream) {
    PoolGeom g;
    int st = make_pool_geom(desc, &g);
    if (st) return st;
    if (!x || !y) return MCN_BAD_ARG;
    const unsigned total = (unsigned)g.Ho * g.Wo * g.D * g.N;
    const dim3 grid(cdiv(total, 256));
    if (g.Hp == 2 && g.Wp == 2)
        hipLaunchKernelGGL((pool_forward_kernel<2, 2>), grid, dim3(256), 0, (hipStream_t)stream, g, x, y, total);
    else if (g.Hp == 3 && g.Wp == 3)
        hipLaunchKernelGGL((pool_forward_kernel<3, 3>), grid, dim3(256), 0, (hipStream_t)stream, g, x, y, total);
    else
        hipLaunchKernelGGL((pool_forward_kernel<0, 0>), grid, dim3(256), 0, (hipStream_t)stream, g, x, y, total);
    return check_launch();
}

// max pooling with 2x2 or 3x3 windows that do not overlap: derivative in one pass (kern_pool.h)
static bool pool_disjoint(const PoolGeom &g) {
    return g.method == MCN_POOL_MAX && g.Sh == g.Hp && g.Sw == g.Wp && g.Hp == g.Wp && (g.Hp == 2 || g.Hp == 3);
}
// one byte per window for the position of its maximum, if a byte can hold it and the two-pass form is used
static size_t pool_ws_bytes(const PoolGeom &g) {
    return (g.method == MCN_POOL_MAX && g.Hp * g.Wp <= 256 && !pool_disjoint(g)) ? (size_t)g.Ho * g.Wo * g.D * g.N : 0;
}

int mcn_pool_workspace_size(const mcn_pool_desc *desc, size_t *bytes) {
    PoolGeom g;
    int st = make_pool_geom(desc, &g);
    if (st) return st;
    if (!bytes) return MCN_BAD_ARG;
    *bytes = pool_ws_bytes(g);
    return MCN_OK;
}

int mcn_pool_backward(const mcn_pool_desc *desc, const float *x, const float *dzdy, float *dzdx, void *ws,
                      size_t ws_bytes, void *stream) {
    PoolGeom g;
    int st = make_pool_geom(desc, &g);
    if (st) return st;
    if (!dzdy || !dzdx || (g.method == MCN_POOL_MAX && !x)) return MCN_BAD_ARG;
    const size_t need = pool_ws_bytes(g);
    if (ws_bytes < need || (!ws && need)) return MCN_WORKSPACE_TOO_SMALL;
    hipStream_t s = (hipStream_t)stream;
    const unsigned n_in = (unsigned)g.H * g.W * g.D * g.N, n_out = (unsigned)g.Ho * g.Wo * g.D * g.N;
    if (pool_disjoint(g)) {
        if (g.Hp == 2)
            hipLaunchKernelGGL((pool_backward_max_disjoint_kernel<2, 2>), dim3(cdiv(n_out, 256)), dim3(256), 0, s, g, x, dzdy, dzdx, n_out);
        else
            hipLaunchKernelGGL((pool_backward_max_disjoint_kernel<3, 3>), dim3(cdiv(n_out, 256)), dim3(256), 0, s, g, x, dzdy, dzdx, n_out);
        return check_launch();
    }
    if (need) {
        const dim3 go(cdiv(n_out, 256));
        if (g.Hp == 2 && g.Wp == 2)
            hipLaunchKernelGGL((pool_argmax_kernel<2, 2>), go, dim3(256), 0, s, g, x, (unsigned char *)ws, n_out);
        else if (g.Hp == 3 && g.Wp == 3)
            hipLaunchKernelGGL((pool_argmax_kernel<3, 3>), go, dim3(256), 0, s, g, x, (unsigned char *)ws, n_out);
        else
            hipLaunchKernelGGL((pool_argmax_kernel<0, 0>), go, dim3(256), 0, s, g, x, (unsigned char *)ws, n_out);
        st = check_launch();
        if (st) return st;
        // windows that can hold one sample, per direction
        const int nh = (g.Hp + g.Sh - 1) / g.Sh, nw = (g.Wp + g.Sw - 1) / g.Sw;
        const int nmax = nh > nw ? nh : nw;
        const dim3 gi(cdiv(n_in, 256));
        const unsigned char *code = (const unsigned char *)ws;
        if (nmax == 1)
            hipLaunchKernelGGL((pool_backward_max_coded_kernel<1, 1>), gi, dim3(256), 0, s, g, code, dzdy, dzdx, n_in);
        else if (nmax == 2)
            hipLaunchKernelGGL((pool_backward_max_coded_kernel<2, 2>), gi, dim3(256), 0, s, g, code, dzdy, dzdx, n_in);
        else if (nmax == 3)
            hipLaunchKernelGGL((pool_backward_max_coded_kernel<3, 3>), gi, dim3(256), 0, s, g, code, dzdy, dzdx, n_in);
        else
            hipLaunchKernelGGL((pool_backward_max_coded_kernel<0, 0>), gi, dim3(256), 0, s, g, code, dzdy, dzdx, n_in);
        return check_launch();
    }
    hipLaunchKernelGGL(pool_backward_kernel, dim3(cdiv(n_in, 256)), dim3(256), 0, s, g, x, dzdy, dzdx, n_in);
    return check_launch();
}

int mcn_probe_mfma(int precision, int32_t iters, float *sink, size_t sink_floats, double *flops, void *stream) {
    if (!sink || iters < 1 || (precision != MCN_PREC_FP32 && precision != MCN_PREC_BF16)) return MCN_BAD_ARG;
    if (sink_floats < (size_t)MCN_PROBE_SINK_FLOATS) return MCN_WORKSPACE_TOO_SMALL;
    static_assert(MCN_PROBE_SINK_FLOATS == PROBE_BLOCKS * PROBE_THREADS, "sink size");
    hipStream_t s = (hipStream_t)stream;
    const double per_mfma = precision == MCN_PREC_BF16 ? 2.0 * 32 * 32 * 16 : 2.0 * 32 * 32 * 2;
    if (flops) *flops = per_mfma * PROBE_ACC * (double)iters * (PROBE_THREADS / 64) * PROBE_BLOCKS;
    if (precision == MCN_PREC_BF16)
        hipLaunchKernelGGL(probe_mfma_kernel<1>, dim3(PROBE_BLOCKS), dim3(PROBE_THREADS), 0, s, sink, iters, 1.0f);
    else
        hipLaunchKernelGGL(probe_mfma_kernel<0>, dim3(PROBE_BLOCKS), dim3(PROBE_THREADS), 0, s, sink, iters, 1.0f);
    return check_launch();
}

int mcn_probe_copy(const float *src, float *dst, size_t n, void *stream) {
    if (!src || !dst || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15)) return MCN_BAD_ARG;
    if (n == 0) return MCN_OK;
    const size_t words = (n >> 2) + 1;
    const unsigned blocks = (unsigned)(words < (size_t)PROBE_BLOCKS * PROBE_THREADS
                                           ? (words + PROBE_THREADS - 1) / PROBE_THREADS : PROBE_BLOCKS * 4);
    hipLaunchKernelGGL(probe_copy_kernel, dim3(blocks), dim3(PROBE_THREADS), 0, (hipStream_t)stream, src, dst, n);
    return check_launch();
}

const char *mcn_status_string(int status) {
    switch (status) {
        case MCN_OK: return "ok";
        case MCN_BAD_ARG: return "bad argument";
        case MCN_BAD_GROUPS: return "filter depth does not divide the input depth, or groups do not divide the filters";
        case MCN_FILTER_TOO_LARGE: return "padded input is smaller than the filter";
        case MCN_WORKSPACE_TOO_SMALL: return "workspace too small";
        case MCN_UNSUPPORTED: return "array too large for 32-bit element offsets";
        case MCN_HIP_ERROR: return "HIP launch error";
        case MCN_CROP_TOO_LARGE: return "crops leave no output";
        case MCN_PAD_TOO_LARGE: return "pooling pad larger than window - 1";
        case MCN_STATIC_SCRATCH_EXCEEDED: return "the call needs more scratch than the library's static buffer holds";
        default: return "unknown status";
    }
}

int mcn_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
