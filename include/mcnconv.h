/*
 * mcnconv -- the convolution block (function vl_nnconv) and the convolution
 * transpose block (vl_nnconvt) of the MatConvNet manual (arXiv 1412.4564) for
 * AMD MI355X (gfx950): forward and backward.
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 * Arrays.  The manual's 4-D arrays are stored FIRST INDEX FASTEST (the vec()
 * order of Sec. 2.3.1), fp32:
 *     x    : H  x W  x D  x N     x[i,j,d,n]   at  i + H *(j + W *(d + D *n))
 *     w    : H' x W' x D' x D''   w[i',j',d',k] at i'+ H'*(j'+ W'*(d'+ D'*k))
 *     y    : H''x W''x D''x N     (same rule; D'' is called K below)
 *     b    : K values
 * Derivative arrays (dzdx, dzdw, dzdb, dzdy) have the shape of what they
 * differentiate (Sec. 4, introduction).
 *
 * Geometry (Sec. 4.1).  stride = (S_h, S_w) vertical then horizontal; pads =
 * (top, bottom, left, right), any value >= 0; H'' = floor((H - H' + top +
 * bottom)/S_h) + 1 and likewise W''.  Filter groups: D' must divide D, giving
 * g = D/D' groups; K must be a multiple of g; filters m*K/g .. (m+1)*K/g - 1
 * form group m and read input channels m*D' .. (m+1)*D' - 1.
 *
 * Pointers.  EVERY data pointer (x, w, b, y, dzdy, dzdx, dzdw, dzdb, ws) is a
 * DEVICE pointer owned by the caller, 16-byte aligned (any hipMalloc or
 * PyTorch allocation is).  The descriptor and the int32 out-parameters are
 * HOST pointers.  `stream` is a hipStream_t passed as void* (NULL = the null
 * stream).  The library allocates no device memory, keeps no state between
 * calls, never synchronises, and launches all work on `stream`.
 *
 * Workspace.  Each operation may need scratch memory: ask
 * mcn_conv_workspace_size() and pass a buffer of at least that many bytes
 * (ws may be NULL when the size is 0).  Its contents are garbage afterwards.
 *
 * Results are WRITTEN, never accumulated into (the manual's blocks return
 * derivatives; summing them along a network is the caller's business,
 * Sec. 2.3.3).  Inputs are not modified.  Outputs must not overlap inputs.
 *
 * Errors.  Every function returns an mcn_status; 0 is success.  All argument
 * and geometry checks happen on the host before anything is launched, so a
 * failed call has done no GPU work.  Nothing prints, throws or aborts.
 */
#ifndef MCNCONV_H
#define MCNCONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mcn_conv_desc {
    int32_t H, W, D, N;         /* x : H x W x D x N                               */
    int32_t Hf, Wf, Df, K;      /* w : H' x W' x D' x K;  groups g = D / Df         */
    int32_t stride_h, stride_w; /* S_h, S_w >= 1                                    */
    int32_t pad_top, pad_bottom, pad_left, pad_right; /* P_h^-, P_h^+, P_w^-, P_w^+ */
    int32_t precision;          /* MCN_PREC_*                                       */
} mcn_conv_desc;

/* Arithmetic of the three matrix-core passes (forward, dzdx, dzdw); the bias derivative is
 * always a plain fp32 sum.  The manual fixes the result of the sum of Sec. 4.1, not the order
 * of its additions, so every mode below returns that sum up to fp32 rounding.
 *
 * MCN_PREC_FP32 (default): fp32 operands and accumulation.  Layers with 3x3 filters at stride 1
 *   (more than 32 filters and at least 16 channels per group) take two output rows at a time
 *   and evaluate the three filter rows with four products instead of six (the minimal-filtering
 *   identity F(2,3), exact in real arithmetic; mcn_conv_kernel_name says "igemm_f23" /
 *   "wgrad_f23").  Each result is then a signed combination of four sums, each of which also
 *   holds products of the neighbouring output row that cancel between the sums.  Its rounding
 *   error therefore scales with the sum of |w||x| over the FOUR input rows that the pair of
 *   output rows reads (dzdw: over both rows of dzdy of a pair), not over the result's own
 *   three-row field: a result whose own terms are tiny beside its neighbour row's terms loses
 *   relative accuracy (graded magnitudes along rows), and a result that is exactly zero
 *   because of zeros in the DATA may come out as rounding noise (zeros that come from padding
 *   stay exact).  For inputs of one scale (the workloads here) the error equals that of the
 *   plain order, about 1e-7 of the sum of |w||x|.
 * MCN_PREC_FP32_PLAIN: fp32 operands and accumulation, every product of the sum of Sec. 4.1
 *   formed as written and added one by one ("igemm" / "wgrad_igemm"): error bound n * 2^-24
 *   of the result's own sum of |w||x|; 3x3 stride-1 layers run about 1.3 times slower.
 * MCN_PREC_BF16: operands (x, w, dzdy) rounded to bf16 on chip, round to nearest even,
 *   products accumulated in fp32; arrays in memory stay fp32.  Normalised error <= 1e-2.
 *   Geometries the bf16 kernels do not cover (fewer than 16 channels per group,
 *   fully-connected layers, the filter derivative with a vertical stride, more than 5 filter
 *   rows or at most 32 filters per group) compute in fp32, which meets the same bound.
 * MCN_PREC_FP32_BF16X3: fp32 arrays, fp32 accumulation, and every operand of the forward pass and of
 *   dzdx held on chip as TWO bf16 values, hi = bf16(v) and lo = bf16(v - hi) (16 bits of v's
 *   significand), with each product formed as w_hi*x_hi + w_hi*x_lo + w_lo*x_hi on the bf16 matrix core
 *   ("igemm_bf16x3").  Error per product below 1.2e-5 of |w||x| in the worst case, so the normalised
 *   error stays under the fp32 bars (1e-4 forward, 1e-3 backward) with a margin of eight or more, and
 *   measures 5e-7 to 6e-6; the two passes run 1.5 to 1.8 times as fast as under MCN_PREC_FP32 on the
 *   3x3 layers of the benchmark (staging, not the matrix core, bounds them).  For callers who would otherwise trade fp32 for
 *   bf16 operands: this keeps 16 instead of 8 significant bits.  dzdw, dzdb and the geometries the bf16
 *   kernels do not cover compute as under MCN_PREC_FP32.
 * The environment variable MCN_NO_WINO=1 (read once per process) makes MCN_PREC_FP32 behave as
 * MCN_PREC_FP32_PLAIN; it exists for benchmarks. */
enum { MCN_PREC_FP32 = 0, MCN_PREC_BF16 = 1, MCN_PREC_FP32_PLAIN = 2, MCN_PREC_FP32_BF16X3 = 3 };

typedef enum mcn_status {
    MCN_OK = 0,
    MCN_BAD_ARG = 1,             /* NULL descriptor/pointer, dim < 1, stride < 1, pad < 0,
                                    unknown precision or operation                      */
    MCN_BAD_GROUPS = 2,          /* Df does not divide D, or D/Df does not divide K     */
    MCN_FILTER_TOO_LARGE = 3,    /* H + top + bottom < H'  or  W + left + right < W'
                                    (Sec. 4.1, "Output size": the padded input must be
                                    at least as large as the filter)                    */
    MCN_WORKSPACE_TOO_SMALL = 4,
    MCN_UNSUPPORTED = 5,         /* an array has 2^31 elements or more                  */
    MCN_HIP_ERROR = 6,           /* a launch failed; see mcn_last_hip_error()           */
    MCN_CROP_TOO_LARGE = 7,      /* convolution transpose: the crops leave no output     */
    MCN_PAD_TOO_LARGE = 8,       /* pooling: a pad exceeds window - 1 (Sec. 5.2.1)       */
    MCN_STATIC_SCRATCH_EXCEEDED = 9  /* mcn_conv_backward_bias_static: the geometry needs more
                                    than MCN_STATIC_SCRATCH_BYTES of scratch            */
} mcn_status;

enum { MCN_OP_FORWARD = 0, MCN_OP_BACKWARD_DATA = 1, MCN_OP_BACKWARD_FILTER = 2, MCN_OP_BACKWARD_BIAS = 3,
       MCN_OP_BACKWARD_FILTER_BIAS = 4 /* convolution block only: mcn_conv_backward_filter_bias */ };

/* Sec. 4.1 "Output size" (derived in Sec. 5.2): writes H'' and W''.
 * Validates the whole descriptor; Ho / Wo may be NULL.  Host only. */
int mcn_conv_output_size(const mcn_conv_desc *desc, int32_t *Ho, int32_t *Wo);

/* Bytes of scratch that operation `op` (MCN_OP_*) needs for this descriptor.
 * Returns an mcn_status; the size is written to *bytes.  Host only. */
int mcn_conv_workspace_size(const mcn_conv_desc *desc, int op, size_t *bytes);

/* Sec. 4.1, "Padding and stride":
 *   y[i'',j'',k,n] = b[k] + sum_{i',j',d'} w[i',j',d',k] *
 *                    x[S_h(i''-1)+i'-top, S_w(j''-1)+j'-left, group(k)*D'+d', n]
 * with x read as zero outside its support.  b == NULL means no bias
 * (the manual's vl_nnconv(x,f,[])).  Writes all of y. */
int mcn_conv_forward(const mcn_conv_desc *desc, const float *x, const float *w, const float *b,
                     float *y, void *ws, size_t ws_bytes, void *stream);

/* Sec. 2.3.2 eq. (projected) applied to the sum above; Sec. 6.1 boxed formula
 * dz/dX = phi*(dz/dY F^T):  dzdx = d<dzdy, y>/dx.  Samples of x that no filter
 * window reads get exactly 0.  Writes all of dzdx. */
int mcn_conv_backward_data(const mcn_conv_desc *desc, const float *w, const float *dzdy,
                           float *dzdx, void *ws, size_t ws_bytes, void *stream);

/* Sec. 6.1 boxed formula dz/dF = phi(x)^T dz/dY, summed over the batch:
 * dzdw = d<dzdy, y>/dw.  Writes all of dzdw. */
int mcn_conv_backward_filter(const mcn_conv_desc *desc, const float *x, const float *dzdy,
                             float *dzdw, void *ws, size_t ws_bytes, void *stream);

/* Sec. 2.3.2: the block's backward mode returns dzdw and dzdb together.  Both of the two
 * results above in one call, same arguments and meaning; workspace that of
 * MCN_OP_BACKWARD_FILTER_BIAS.  Where the filter derivative's kernel can sum dzdy on
 * the way (3x3 filters at stride 1, more than 32 filters per group, arrays that
 * stream from memory; mcn_conv_kernel_name says "wgrad_f23+bias") dzdy is read once
 * for both; otherwise the two passes run one after the other ("two passes"). */
int mcn_conv_backward_filter_bias(const mcn_conv_desc *desc, const float *x, const float *dzdy,
                                  float *dzdw, float *dzdb, void *ws, size_t ws_bytes, void *stream);

/* y is affine in b with coefficient one, so
 * dzdb[k] = sum_{i'',j'',n} dzdy[i'',j'',k,n].  Writes K values. */
int mcn_conv_backward_bias(const mcn_conv_desc *desc, const float *dzdy, float *dzdb,
                           void *ws, size_t ws_bytes, void *stream);

/* For callers that cannot allocate device memory or hold a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The same result as
 * mcn_conv_backward_bias, bit for bit (same kernels, same order of additions), with the partial
 * sums kept in a buffer of MCN_STATIC_SCRATCH_BYTES that is part of the library's code object on
 * every GPU it runs on (held until the process ends).  The call allocates nothing and frees
 * nothing; its first call on a device looks the buffer's address up (no allocation either;
 * make that call outside a graph capture).  Geometries that need more scratch (K * H''W'' above
 * 262144 for output planes under 64 samples, or more than about 260000 filters) return
 * MCN_STATIC_SCRATCH_EXCEEDED before any GPU work.  All calls on one GPU share the one buffer:
 * calls that may overlap there (different streams, different threads) race; calls on one
 * stream are ordered and safe.  Nothing in the buffer has to be cleared between calls. */
#define MCN_STATIC_SCRATCH_BYTES (1 << 20)
int mcn_conv_backward_bias_static(const mcn_conv_desc *desc, const float *dzdy, float *dzdb, void *stream);

/* ------------------------------------------------------------------------
 * Convolution followed by the ReLU block (Sec. 4.4, y = max{0, p}), fused
 * ------------------------------------------------------------------------
 * A network that follows a convolution by a ReLU otherwise writes the
 * convolution's output, reads it back and writes it again; these two calls
 * save that pass in each direction.
 *
 * Forward:  y = max(0, x * w + b), i.e. mcn_conv_forward with the maximum
 * applied as the results are written.  Same arguments, workspace and errors
 * as mcn_conv_forward. */
int mcn_conv_relu_forward(const mcn_conv_desc *desc, const float *x, const float *w, const float *b,
                          float *y, void *ws, size_t ws_bytes, void *stream);

/* Backward through that ReLU, fused with the bias derivative (Sec. 6.4.1:
 * dz/dp = [p > 0] dz/dy, and y > 0 exactly where p > 0):
 *     dzdp[i'',j'',k,n] = dzdy[i'',j'',k,n] if y[i'',j'',k,n] > 0, else 0
 *     dzdb[k]           = sum_{i'',j'',n} dzdp[i'',j'',k,n]
 * y is the array mcn_conv_relu_forward wrote, dzdy the derivative with
 * respect to it; dzdp (same shape) is what mcn_conv_backward_data and
 * mcn_conv_backward_filter then take as their dzdy.  dzdp may be the same
 * array as dzdy (in place).  Workspace: that of MCN_OP_BACKWARD_BIAS. */
int mcn_conv_relu_backward_bias(const mcn_conv_desc *desc, const float *y, const float *dzdy,
                                float *dzdp, float *dzdb, void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------
 * Convolution transpose (Sec. 4.2; derivation Sec. 6.2; output size Sec. 5.3)
 * ------------------------------------------------------------------------
 * Arrays (first index fastest, fp32, device pointers, as above):
 *     x : H  x W  x D x N
 *     f : H' x W' x K' x D       filter k is the slice f[:,:,k,:] (Sec. 4.2): the
 *                                 THIRD index runs over output channels of a
 *                                 group, the FOURTH over all input channels
 *     y : H''x W''x (groups*K') x N,    b : groups*K' values
 * Geometry: up = (S_h, S_w) input upsampling factors, crops = (top, bottom,
 * left, right) >= 0 removed from the output;
 *     H'' = S_h (H - 1) + H' - top - bottom,   W'' likewise,
 * the smallest size whose convolution (filter H' x W', stride = up, pads =
 * crops) has size H x W.  MCN_CROP_TOO_LARGE if H'' < 1 or W'' < 1.
 * Groups (the manual is silent; this is the transpose of the grouped
 * convolution of Sec. 4.1 run from y's shape to x's): `groups` must divide D;
 * input channels m*D/groups .. (m+1)*D/groups - 1 feed output channels
 * m*K' .. (m+1)*K' - 1.
 * Workspace, stream, results-are-written and error rules are those of the
 * convolution block; `op` is the same MCN_OP_* enumeration. */
typedef struct mcn_convt_desc {
    int32_t H, W, D, N;          /* x : H x W x D x N                                  */
    int32_t Hf, Wf, Kf, groups;  /* f : H' x W' x K' x D;  y has groups*K' channels    */
    int32_t up_h, up_w;          /* S_h, S_w >= 1                                      */
    int32_t crop_top, crop_bottom, crop_left, crop_right;
    int32_t precision;           /* MCN_PREC_*                                         */
} mcn_convt_desc;

/* Sec. 4.2 / Sec. 5.3: writes H'' and W''.  Validates the whole descriptor;
 * Ho / Wo may be NULL.  Host only. */
int mcn_convt_output_size(const mcn_convt_desc *desc, int32_t *Ho, int32_t *Wo);

/* Bytes of scratch that operation `op` needs for this descriptor.  Host only. */
int mcn_convt_workspace_size(const mcn_convt_desc *desc, int op, size_t *bytes);

/* Sec. 4.2: vec y = M^T vec x (+ b), M being the matrix of the convolution
 * block that maps y's shape to x's shape with bank f, stride = up, pads =
 * crops.  Sample by sample (Sec. 6.2 in two dimensions, 1-based):
 *   y[i'',j'',m*K'+k,n] = b[m*K'+k] + sum_{i,j,d in group m}
 *        f[i''-S_h(i-1)+top, j''-S_w(j-1)+left, k, d] * x[i,j,d,n]
 * with f read as zero outside its support.  b == NULL means no bias.
 * Writes all of y. */
int mcn_convt_forward(const mcn_convt_desc *desc, const float *x, const float *f, const float *b,
                      float *y, void *ws, size_t ws_bytes, void *stream);

/* dzdx = d<dzdy, y>/dx = M dzdy: the convolution of dzdy with the bank f
 * (Sec. 4.2: the block is the transpose of convolution).  Writes all of dzdx. */
int mcn_convt_backward_data(const mcn_convt_desc *desc, const float *f, const float *dzdy,
                            float *dzdx, void *ws, size_t ws_bytes, void *stream);

/* dzdf = d<dzdy, y>/df, summed over the batch (Sec. 2.3.2 eq. (projected)
 * applied to the sum above).  Writes all of dzdf. */
int mcn_convt_backward_filter(const mcn_convt_desc *desc, const float *x, const float *dzdy,
                              float *dzdf, void *ws, size_t ws_bytes, void *stream);

/* dzdb[c] = sum_{i'',j'',n} dzdy[i'',j'',c,n].  Writes groups*K' values. */
int mcn_convt_backward_bias(const mcn_convt_desc *desc, const float *dzdy, float *dzdb,
                            void *ws, size_t ws_bytes, void *stream);

/* Name of the kernel family the dispatcher picks; NULL on a bad descriptor. */
const char *mcn_convt_kernel_name(const mcn_convt_desc *desc, int op);

/* ------------------------------------------------------------------------
 * Spatial pooling (Sec. 4.3; geometry Sec. 5.2; derivative Sec. 6.3)
 * ------------------------------------------------------------------------
 * x : H x W x D x N  ->  y : H'' x W'' x D x N, each channel pooled on its own
 * over windows of H' x W' samples placed like the filters of the convolution
 * block (stride, four pads, the same output-size rule).  A window that
 * straddles the boundary is cropped: the maximum is taken over, and the
 * average divided by the number of, the samples inside the array.  Pads may
 * not exceed window - 1 (MCN_PAD_TOO_LARGE), so every window holds a sample;
 * MCN_FILTER_TOO_LARGE if the padded input is smaller than the window.
 * Results are written, inputs are not modified.  Only the backward pass of
 * max pooling takes a workspace (one byte per output sample). */
enum { MCN_POOL_MAX = 0, MCN_POOL_AVG = 1 };

typedef struct mcn_pool_desc {
    int32_t H, W, D, N;          /* x : H x W x D x N                                 */
    int32_t Hp, Wp;              /* window H' x W'                                     */
    int32_t stride_h, stride_w;
    int32_t pad_top, pad_bottom, pad_left, pad_right;
    int32_t method;              /* MCN_POOL_MAX or MCN_POOL_AVG                       */
} mcn_pool_desc;

/* Writes H'' and W'' (either may be NULL); validates the descriptor.  Host only. */
int mcn_pool_output_size(const mcn_pool_desc *desc, int32_t *Ho, int32_t *Wo);

/* Bytes of scratch mcn_pool_backward needs for this descriptor.  Host only. */
int mcn_pool_workspace_size(const mcn_pool_desc *desc, size_t *bytes);

/* y[i'',j'',d,n] = max, or mean, of x[i,j,d,n] over the cropped window. */
int mcn_pool_forward(const mcn_pool_desc *desc, const float *x, float *y, void *stream);

/* dzdx = S(x)^T dzdy (Sec. 6.3).  Max: each window hands its dzdy to the
 * sample it selected, the first maximum in memory order (rows fastest) where
 * a window holds its maximum more than once; x is the forward input.
 * Average: each window hands dzdy / (samples inside) to every sample inside;
 * x is not read and may be NULL.  Writes all of dzdx. */
int mcn_pool_backward(const mcn_pool_desc *desc, const float *x, const float *dzdy, float *dzdx,
                      void *ws, size_t ws_bytes, void *stream);

/* Static description of a status code. */
const char *mcn_status_string(int status);

/* The hipError_t (as int) behind the most recent MCN_HIP_ERROR of this thread, else 0. */
int mcn_last_hip_error(void);

/* Name of the kernel family the dispatcher picks for this descriptor and
 * operation ("direct", "igemm", "igemm_f23" / "wgrad_f23" = the matrix-core kernels
 * that take pairs of output rows of a 3x3 stride-1 layer with four products per filter
 * column, ...); for reports and tests.  Returns NULL on a bad descriptor.  Host only. */
const char *mcn_conv_kernel_name(const mcn_conv_desc *desc, int op);

/* ---- Measurement aids (no part of the paper's blocks) ---------------------------------
 * The rates this GPU sustains on the two resources the kernels above are priced against,
 * so that a benchmark can quote a fraction of the measured ceiling beside the fraction
 * of the published one.  Both are asynchronous on `stream`; time them with HIP events. */

/* Floats `sink` of mcn_probe_mfma must hold. */
#define MCN_PROBE_SINK_FLOATS (2048 * 256)

/* Register-only matrix-core loop: 2048 blocks of 4 waves, each wave issuing 4 * iters
 * independent 32x32 MFMAs with no memory, LDS or barrier in the loop.
 * precision MCN_PREC_FP32 -> v_mfma_f32_32x32x2_f32, MCN_PREC_BF16 -> v_mfma_f32_32x32x16_bf16.
 * sink (device, MCN_PROBE_SINK_FLOATS floats, overwritten) keeps the loop alive;
 * *flops (host, may be NULL) receives the floating-point operations the launch performs.
 * MCN_BAD_ARG for a NULL sink, iters < 1 or an unknown precision; MCN_WORKSPACE_TOO_SMALL
 * when sink_floats < MCN_PROBE_SINK_FLOATS. */
int mcn_probe_mfma(int precision, int32_t iters, float *sink, size_t sink_floats, double *flops,
                   void *stream);

/* dst[0..n) = src[0..n) (device pointers, both 16-byte aligned, not overlapping) with
 * 16-byte loads and stores: one read stream and one write stream, 8 * n bytes of traffic.
 * MCN_BAD_ARG for NULL or misaligned pointers; n = 0 launches nothing. */
int mcn_probe_copy(const float *src, float *dst, size_t n, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MCNCONV_H */
