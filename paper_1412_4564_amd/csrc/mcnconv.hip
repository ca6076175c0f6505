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

size_t workspace_bytes(const Geom &g, int op) {
    switch (op) {
        case MCN_OP_BACKWARD_BIAS: {
            BiasPlan p = plan_bias(g);
            return (size_t)g.K * p.S * sizeof(float);
        }
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
    *bytes = workspace_bytes(g, op);
    return MCN_OK;
}

const char *mcn_conv_kernel_name(const mcn_conv_desc *desc, int op) {
    Geom g;
    if (make_geom(desc, &g)) return NULL;
    switch (op) {
        case MCN_OP_FORWARD: return "direct";
        case MCN_OP_BACKWARD_DATA: return "direct";
        case MCN_OP_BACKWARD_FILTER: return "direct";
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
    if (ws_bytes < workspace_bytes(g, MCN_OP_FORWARD) || (!ws && workspace_bytes(g, MCN_OP_FORWARD)))
        return MCN_WORKSPACE_TOO_SMALL;
    hipStream_t s = (hipStream_t)stream;
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
    if (ws_bytes < workspace_bytes(g, MCN_OP_BACKWARD_DATA) || (!ws && workspace_bytes(g, MCN_OP_BACKWARD_DATA)))
        return MCN_WORKSPACE_TOO_SMALL;
    hipStream_t s = (hipStream_t)stream;
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
    if (ws_bytes < workspace_bytes(g, MCN_OP_BACKWARD_FILTER) || (!ws && workspace_bytes(g, MCN_OP_BACKWARD_FILTER)))
        return MCN_WORKSPACE_TOO_SMALL;
    hipStream_t s = (hipStream_t)stream;
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
    const size_t need = workspace_bytes(g, MCN_OP_BACKWARD_BIAS);
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
