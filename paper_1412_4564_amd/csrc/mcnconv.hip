// C-ABI entry points of the convolution library and the host-side dispatcher:
// argument checks, kernel choice, workspace layout, launches.  See include/mcnconv.h
// for the contract of every function.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#include "../../include/mcnconv.h"
#include "geom.h"
#include "kern_direct.h"
#include "kern_igemm.h"
#include "igemm_plan.h"

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
    int chunks;  // chunks of BIAS_CHUNK samples per (n, k) plane
    int S;       // partial sums per filter
};

BiasPlan plan_bias(const Geom &g) {
    BiasPlan p;
    const int64_t HoWo = (int64_t)g.Ho * g.Wo;
    p.chunks = (int)((HoWo + BIAS_CHUNK - 1) / BIAS_CHUNK);
    const int64_t units = (int64_t)g.N * p.chunks;
    int64_t want = (2048 + g.K - 1) / g.K;   // aim for ~2048 blocks in all
    if (want > units) want = units;
    if (want < 1) want = 1;
    if (want > 65535) want = 65535;
    p.S = (int)want;
    return p;
}

// ---- implicit-GEMM dispatch -------------------------------------------------
bool igemm_enabled() {
    static const bool off = getenv("MCN_FORCE_DIRECT") != nullptr;   // benchmarking / debugging override
    return !off;
}

// Plans depend only on the descriptor; planning walks candidate tilings, so the last few
// descriptors' plans are remembered per host thread (host memory only, no device state).
struct PlanEntry {
    mcn_conv_desc d;
    bool used;
    bool fwd_ok, bwd_ok, wg_ok;
    IgemmPlan fwd, bwd;
    WgradPlan wg;
};
constexpr int PLAN_CACHE = 16;
thread_local PlanEntry g_plans[PLAN_CACHE];
thread_local int g_plan_next = 0;

const PlanEntry *plans_for(const mcn_conv_desc *d, const Geom &g) {
    for (int i = 0; i < PLAN_CACHE; ++i)
        if (g_plans[i].used && memcmp(&g_plans[i].d, d, sizeof(*d)) == 0) return &g_plans[i];
    PlanEntry &e = g_plans[g_plan_next];
    g_plan_next = (g_plan_next + 1) % PLAN_CACHE;
    e.d = *d;
    e.used = true;
    const bool on = igemm_enabled();
    e.fwd_ok = on && plan_igemm(forward_view(g), &e.fwd);
    e.bwd_ok = on && g.Sh == 1 && g.Sw == 1 && plan_igemm(backward_data_view(g), &e.bwd);
    e.wg_ok = on && plan_wgrad(g, &e.wg);
    return &e;
}

template <int WK, int WP, int MK, int MP, int DC, int HF, int WF, int TMAX>
int launch_igemm_inst(const IgemmPlan &pl, const float *in, const float *wpk, const float *bias, float *out,
                      hipStream_t s) {
    auto kern = igemm_conv_kernel<WK, WP, MK, MP, DC, HF, WF, TMAX, IGEMM_EPT>;
    if (pl.lds_bytes > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)pl.lds_bytes);
        if (e != hipSuccess) { g_last_hip_error = (int)e; return MCN_HIP_ERROR; }
    }
    hipLaunchKernelGGL(kern, dim3(pl.blocks), dim3(64 * WK * WP), pl.lds_bytes, s, pl.P, in, wpk, bias, out);
    return check_launch();
}

int launch_igemm(const IgemmPlan &pl, const ConvView &v, const float *in, const float *w, const float *bias,
                 float *out, float *packed, hipStream_t s) {
    const int total = (int)pl.packed_floats;
    // for the packing kernel the weight array is always the caller's w : Hf x Wf x Df x K
    const int Df = v.pack_mode == 0 ? v.Cg : v.Kg;
    hipLaunchKernelGGL(igemm_pack_weights_kernel, dim3(cdiv(total, 256)), dim3(256), 0, s, w, packed, v.Hf, v.Wf, Df,
                       v.Kg, v.Cg, v.G, pl.P.KT, pl.P.NCH, pl.TK, pl.DC, v.pack_mode, total);
    int st = check_launch();
    if (st) return st;
    switch (pl.shape) {
        case IG_128x256:
            return pl.fixed33 ? launch_igemm_inst<2, 4, 2, 2, 8, 3, 3, 9>(pl, in, packed, bias, out, s)
                              : launch_igemm_inst<2, 4, 2, 2, 4, 0, 0, IGEMM_TMAX>(pl, in, packed, bias, out, s);
        case IG_64x512:
            return pl.fixed33 ? launch_igemm_inst<1, 8, 2, 2, 8, 3, 3, 9>(pl, in, packed, bias, out, s)
                              : launch_igemm_inst<1, 8, 2, 2, 4, 0, 0, IGEMM_TMAX>(pl, in, packed, bias, out, s);
        case IG_32x256:
            return pl.fixed33 ? launch_igemm_inst<1, 4, 1, 2, 8, 3, 3, 9>(pl, in, packed, bias, out, s)
                              : launch_igemm_inst<1, 4, 1, 2, 4, 0, 0, IGEMM_TMAX>(pl, in, packed, bias, out, s);
        default:
            return MCN_BAD_ARG;
    }
}

template <int WK, int WR, int MK, int MR, int PCH, int EPT, int NCHMAX>
int launch_wgrad_inst(const WgradPlan &pl, const float *x, const float *dzdy, float *outp, hipStream_t s) {
    if (pl.PCH != PCH) return MCN_BAD_ARG;
    auto kern = wgrad_kernel<WK, WR, MK, MR, PCH, EPT, NCHMAX>;
    if (pl.lds_bytes > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)pl.lds_bytes);
        if (e != hipSuccess) { g_last_hip_error = (int)e; return MCN_HIP_ERROR; }
    }
    hipLaunchKernelGGL(kern, dim3(pl.blocks), dim3(64 * WK * WR), pl.lds_bytes, s, pl.P, x, dzdy, outp);
    return check_launch();
}

int launch_wgrad(const WgradPlan &pl, const Geom &g, const float *x, const float *dzdy, float *dzdw, float *ws,
                 hipStream_t s) {
    float *outp = pl.splits > 1 ? ws : dzdw;
    int st;
    switch (pl.shape) {
        case WG_128x128: st = launch_wgrad_inst<2, 2, 2, 2, 32, 2, 16>(pl, x, dzdy, outp, s); break;
        case WG_64x192: st = launch_wgrad_inst<2, 2, 1, 3, 64, 2, 24>(pl, x, dzdy, outp, s); break;
        case WG_32x256: st = launch_wgrad_inst<1, 4, 1, 2, 32, 2, 32>(pl, x, dzdy, outp, s); break;
        default: return MCN_BAD_ARG;
    }
    if (st || pl.splits == 1) return st;
    const int total = (int)numel_w(g);
    hipLaunchKernelGGL(wgrad_reduce_kernel, dim3(cdiv(total, 256)), dim3(256), 0, s, ws, dzdw, total, pl.splits);
    return check_launch();
}

size_t workspace_bytes(const mcn_conv_desc *d, const Geom &g, int op) {
    const PlanEntry *e = plans_for(d, g);
    switch (op) {
        case MCN_OP_BACKWARD_BIAS: {
            BiasPlan p = plan_bias(g);
            return (size_t)g.K * p.S * sizeof(float);
        }
        case MCN_OP_FORWARD: return e->fwd_ok ? e->fwd.packed_floats * sizeof(float) : 0;
        case MCN_OP_BACKWARD_DATA: return e->bwd_ok ? e->bwd.packed_floats * sizeof(float) : 0;
        case MCN_OP_BACKWARD_FILTER: return e->wg_ok ? e->wg.partial_floats * sizeof(float) : 0;
        default:
            return 0;
    }
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
    if (!bytes || op < MCN_OP_FORWARD || op > MCN_OP_BACKWARD_BIAS) return MCN_BAD_ARG;
    *bytes = workspace_bytes(desc, g, op);
    return MCN_OK;
}

const char *mcn_conv_kernel_name(const mcn_conv_desc *desc, int op) {
    Geom g;
    if (make_geom(desc, &g)) return NULL;
    const PlanEntry *e = plans_for(desc, g);
    switch (op) {
        case MCN_OP_FORWARD: return e->fwd_ok ? "igemm" : "direct";
        case MCN_OP_BACKWARD_DATA: return e->bwd_ok ? "igemm" : "direct";
        case MCN_OP_BACKWARD_FILTER: return e->wg_ok ? "wgrad_igemm" : "direct";
        case MCN_OP_BACKWARD_BIAS: return "reduce2";
        default: return NULL;
    }
}

int mcn_conv_forward(const mcn_conv_desc *desc, const float *x, const float *w, const float *b, float *y,
                     void *ws, size_t ws_bytes, void *stream) {
    Geom g;
    int st = make_geom(desc, &g);
    if (st) return st;
    if (!x || !w || !y) return MCN_BAD_ARG;
    const size_t need = workspace_bytes(desc, g, MCN_OP_FORWARD);
    if (ws_bytes < need || (!ws && need)) return MCN_WORKSPACE_TOO_SMALL;
    const PlanEntry *pe = plans_for(desc, g);
    hipStream_t s = (hipStream_t)stream;
    if (pe->fwd_ok) return launch_igemm(pe->fwd, forward_view(g), x, w, b, y, (float *)ws, s);
    const int total = (int)numel_y(g);
    hipLaunchKernelGGL(direct_forward_kernel, dim3(cdiv(total, 256)), dim3(256), 0, s, g, x, w, b, y, total);
    return check_launch();
}

int mcn_conv_backward_data(const mcn_conv_desc *desc, const float *w, const float *dzdy, float *dzdx,
                           void *ws, size_t ws_bytes, void *stream) {
    Geom g;
    int st = make_geom(desc, &g);
    if (st) return st;
    if (!w || !dzdy || !dzdx) return MCN_BAD_ARG;
    const size_t need = workspace_bytes(desc, g, MCN_OP_BACKWARD_DATA);
    if (ws_bytes < need || (!ws && need)) return MCN_WORKSPACE_TOO_SMALL;
    const PlanEntry *pe = plans_for(desc, g);
    hipStream_t s = (hipStream_t)stream;
    if (pe->bwd_ok) return launch_igemm(pe->bwd, backward_data_view(g), dzdy, w, nullptr, dzdx, (float *)ws, s);
    const int total = (int)numel_x(g);
    hipLaunchKernelGGL(direct_backward_data_kernel, dim3(cdiv(total, 256)), dim3(256), 0, s, g, w, dzdy, dzdx, total);
    return check_launch();
}

int mcn_conv_backward_filter(const mcn_conv_desc *desc, const float *x, const float *dzdy, float *dzdw,
                             void *ws, size_t ws_bytes, void *stream) {
    Geom g;
    int st = make_geom(desc, &g);
    if (st) return st;
    if (!x || !dzdy || !dzdw) return MCN_BAD_ARG;
    const size_t need = workspace_bytes(desc, g, MCN_OP_BACKWARD_FILTER);
    if (ws_bytes < need || (!ws && need)) return MCN_WORKSPACE_TOO_SMALL;
    const PlanEntry *pe = plans_for(desc, g);
    hipStream_t s = (hipStream_t)stream;
    if (pe->wg_ok) return launch_wgrad(pe->wg, g, x, dzdy, dzdw, (float *)ws, s);
    const int total = (int)numel_w(g);
    hipLaunchKernelGGL(direct_backward_filter_kernel, dim3(cdiv(total, 4)), dim3(256), 0, s, g, x, dzdy, dzdw, total);
    return check_launch();
}

int mcn_conv_backward_bias(const mcn_conv_desc *desc, const float *dzdy, float *dzdb, void *ws, size_t ws_bytes,
                           void *stream) {
    Geom g;
    int st = make_geom(desc, &g);
    if (st) return st;
    if (!dzdy || !dzdb) return MCN_BAD_ARG;
    const size_t need = workspace_bytes(desc, g, MCN_OP_BACKWARD_BIAS);
    if (ws_bytes < need || (!ws && need)) return MCN_WORKSPACE_TOO_SMALL;
    hipStream_t s = (hipStream_t)stream;
    BiasPlan p = plan_bias(g);
    float *part = (float *)ws;
    hipLaunchKernelGGL(bias_partial_kernel, dim3(g.K, p.S), dim3(256), 0, s, dzdy, part, g.Ho * g.Wo, g.K, g.N,
                       p.chunks, p.S);
    st = check_launch();
    if (st) return st;
    hipLaunchKernelGGL(bias_final_kernel, dim3(cdiv(g.K, 256)), dim3(256), 0, s, part, dzdb, g.K, p.S);
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
        default: return "unknown status";
    }
}

int mcn_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
