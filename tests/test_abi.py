"""Host-side checks of the C-ABI library: it loads, exports every function the
header declares, and turns every bad geometry into a status code before any GPU
work (so these run without a GPU)."""
import ctypes
import os
import re

import pytest

from paper_1412_4564_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = []
    inc = os.path.join(ROOT, "include")
    for fn in sorted(os.listdir(inc)):
        if not fn.endswith(".h"):
            continue
        text = open(os.path.join(inc, fn)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names += re.findall(r"\b(mcn_[a-z0-9_]+)\s*\(", text)
    return sorted(set(names))


def test_library_exports_every_declared_function():
    names = declared_functions()
    assert set(names) == set(B.EXPORTS), names
    L = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(L, n), n


def desc(**kw):
    base = dict(xshape=(2, 4, 9, 8), wshape=(6, 2, 3, 3), stride=(1, 1), pad=(0, 0, 0, 0))
    base.update(kw)
    return B.make_desc(**base)


def test_output_size_closed_form():
    # Sec. 4.1 "Output size": floor((H - H' + Pt + Pb)/Sh) + 1
    assert B.mcn_conv_output_size(desc()) == (6, 7)
    assert B.mcn_conv_output_size(desc(stride=(2, 3), pad=(1, 0, 2, 1))) == ((8 - 3 + 1) // 2 + 1, (9 - 3 + 3) // 3 + 1)
    assert B.mcn_conv_output_size(B.make_desc((4, 16, 53, 37), (24, 16, 5, 3), (2, 3), (1, 0, 2, 1))) == (18, 18)
    assert B.mcn_conv_output_size(B.make_desc((128, 3, 227, 227), (96, 3, 11, 11), (4, 4))) == (55, 55)


@pytest.mark.parametrize("kw,code", [
    (dict(stride=(0, 1)), B.MCN_BAD_ARG),
    (dict(stride=(1, -1)), B.MCN_BAD_ARG),
    (dict(pad=(0, -1, 0, 0)), B.MCN_BAD_ARG),
    (dict(xshape=(0, 4, 9, 8)), B.MCN_BAD_ARG),
    (dict(wshape=(6, 2, 3, 0)), B.MCN_BAD_ARG),
    (dict(precision=7), B.MCN_BAD_ARG),
    (dict(precision=4), B.MCN_BAD_ARG),
    (dict(wshape=(6, 3, 3, 3)), B.MCN_BAD_GROUPS),       # D' = 3 does not divide D = 4
    (dict(wshape=(5, 2, 3, 3)), B.MCN_BAD_GROUPS),       # 2 groups do not divide 5 filters
    (dict(wshape=(6, 2, 3, 9)), B.MCN_FILTER_TOO_LARGE),  # H = 8 < H' = 9
    (dict(wshape=(6, 2, 11, 3), pad=(0, 0, 1, 0)), B.MCN_FILTER_TOO_LARGE),
    (dict(xshape=(1 << 20, 64, 9, 8), wshape=(6, 64, 3, 3)), B.MCN_UNSUPPORTED),   # x has >= 2^31 elements
])
def test_bad_geometry_is_a_status_code_everywhere(kw, code):
    d = desc(**kw)
    L = B.lib()
    assert L.mcn_conv_output_size(ctypes.byref(d), None, None) == code
    n = ctypes.c_size_t(0)
    assert L.mcn_conv_workspace_size(ctypes.byref(d), 0, ctypes.byref(n)) == code
    # non-null dummy pointers: validation must reject before touching them
    p = 4096
    assert B.mcn_conv_forward(d, p, p, p, p, None, 0, None) == code
    assert B.mcn_conv_backward_data(d, p, p, p, None, 0, None) == code
    assert B.mcn_conv_backward_filter(d, p, p, p, None, 0, None) == code
    assert B.mcn_conv_backward_bias(d, p, p, None, 0, None) == code
    assert B.mcn_conv_relu_forward(d, p, p, p, p, None, 0, None) == code
    assert B.mcn_conv_relu_backward_bias(d, p, p, p, p, None, 0, None) == code
    assert B.mcn_conv_kernel_name(d, 0) is None


def test_null_pointers_and_small_workspace_are_rejected():
    d = desc()
    p = 4096
    L = B.lib()
    assert L.mcn_conv_output_size(None, None, None) == B.MCN_BAD_ARG
    assert L.mcn_conv_workspace_size(ctypes.byref(d), 9, ctypes.byref(ctypes.c_size_t(0))) == B.MCN_BAD_ARG
    assert L.mcn_conv_workspace_size(ctypes.byref(d), 0, None) == B.MCN_BAD_ARG
    assert B.mcn_conv_forward(d, None, p, p, p, None, 0, None) == B.MCN_BAD_ARG
    assert B.mcn_conv_forward(d, p, None, p, p, None, 0, None) == B.MCN_BAD_ARG
    assert B.mcn_conv_forward(d, p, p, p, None, None, 0, None) == B.MCN_BAD_ARG
    assert B.mcn_conv_backward_data(d, p, None, p, None, 0, None) == B.MCN_BAD_ARG
    assert B.mcn_conv_backward_filter(d, p, p, None, None, 0, None) == B.MCN_BAD_ARG
    assert B.mcn_conv_backward_bias(d, None, p, None, 0, None) == B.MCN_BAD_ARG
    for bad in range(4):
        args = [p, p, p, p]
        args[bad] = None
        assert B.mcn_conv_backward_filter_bias(d, *args, None, 0, None) == B.MCN_BAD_ARG
    assert B.mcn_conv_relu_forward(d, p, p, p, None, None, 0, None) == B.MCN_BAD_ARG
    for bad in range(4):
        args = [p, p, p, p]
        args[bad] = None
        assert B.mcn_conv_relu_backward_bias(d, *args, None, 0, None) == B.MCN_BAD_ARG
    for op, call in [(B.MCN_OP_BACKWARD_BIAS, lambda ws, n: B.mcn_conv_backward_bias(d, p, p, ws, n, None)),
                     (B.MCN_OP_BACKWARD_BIAS, lambda ws, n: B.mcn_conv_relu_backward_bias(d, p, p, p, p, ws, n, None)),
                     (B.MCN_OP_FORWARD, lambda ws, n: B.mcn_conv_forward(d, p, p, p, p, ws, n, None)),
                     (B.MCN_OP_FORWARD, lambda ws, n: B.mcn_conv_relu_forward(d, p, p, p, p, ws, n, None)),
                     (B.MCN_OP_BACKWARD_DATA, lambda ws, n: B.mcn_conv_backward_data(d, p, p, p, ws, n, None)),
                     (B.MCN_OP_BACKWARD_FILTER, lambda ws, n: B.mcn_conv_backward_filter(d, p, p, p, ws, n, None)),
                     (B.MCN_OP_BACKWARD_FILTER_BIAS, lambda ws, n: B.mcn_conv_backward_filter_bias(d, p, p, p, p, ws, n, None))]:
        need = B.mcn_conv_workspace_size(d, op)
        if need:
            assert call(p, need - 1) == B.MCN_WORKSPACE_TOO_SMALL
            assert call(None, need) == B.MCN_WORKSPACE_TOO_SMALL


def test_one_call_filter_and_bias_workspace_covers_both_passes():
    # host logic: the scratch of the one-call filter + bias derivative is never smaller than that of either pass,
    # and where one kernel gives both (layers 4a, 4b) it also holds the partial bias sums
    from paper_1412_4564_amd import synth
    for name, L in synth.LAYERS.items():
        d = B.make_desc(synth.x_shape(L), synth.w_shape(L), L["stride"], L["pad"])
        both = B.mcn_conv_workspace_size(d, B.MCN_OP_BACKWARD_FILTER_BIAS)
        f, b = B.mcn_conv_workspace_size(d, B.MCN_OP_BACKWARD_FILTER), B.mcn_conv_workspace_size(d, B.MCN_OP_BACKWARD_BIAS)
        fused = B.mcn_conv_kernel_name(d, B.MCN_OP_BACKWARD_FILTER_BIAS) == "wgrad_f23+bias"
        assert fused == (name in ("4a", "4b")), name
        assert both > f if fused else both == max(f, b), (name, both, f, b)


def test_status_strings():
    L = B.lib()
    seen = set()
    for code in range(0, 9):
        s = L.mcn_status_string(code).decode()
        assert s and s not in seen
        seen.add(s)
    assert "unknown" in L.mcn_status_string(99).decode()
    for op in range(4):
        assert B.mcn_conv_kernel_name(desc(), op)
    assert B.mcn_conv_kernel_name(desc(), 17) is None


# ---- convolution transpose ----
def tdesc(**kw):
    base = dict(xshape=(2, 4, 5, 6), fshape=(4, 3, 3, 4), upsample=(2, 2), crop=(1, 0, 0, 1), groups=2)
    base.update(kw)
    return B.make_convt_desc(**base)


def test_convt_output_size_closed_form():
    # Sec. 4.2: H'' = S_h (H - 1) + H' - top - bottom
    assert B.mcn_convt_output_size(tdesc()) == (2 * 5 + 4 - 1, 2 * 4 + 3 - 1)
    assert B.mcn_convt_output_size(tdesc(upsample=(1, 3), crop=(0, 0, 2, 2))) == (5 + 4, 3 * 4 + 3 - 4)
    # 32x bilinear upsampling of a 16x16 map with a 64-tap filter and 16 cropped on each side
    assert B.mcn_convt_output_size(B.make_convt_desc((1, 21, 16, 16), (21, 1, 64, 64), (32, 32), (16, 16, 16, 16), 21)) == (512, 512)


@pytest.mark.parametrize("kw,code", [
    (dict(upsample=(0, 1)), B.MCN_BAD_ARG),
    (dict(upsample=(1, -2)), B.MCN_BAD_ARG),
    (dict(crop=(0, 0, -1, 0)), B.MCN_BAD_ARG),
    (dict(xshape=(0, 4, 5, 6)), B.MCN_BAD_ARG),
    (dict(fshape=(4, 0, 3, 4)), B.MCN_BAD_ARG),
    (dict(groups=0), B.MCN_BAD_ARG),
    (dict(precision=9), B.MCN_BAD_ARG),
    (dict(groups=3), B.MCN_BAD_GROUPS),                    # 3 groups do not divide D = 4
    (dict(crop=(7, 7, 0, 0)), B.MCN_CROP_TOO_LARGE),       # 14 rows before cropping
    (dict(crop=(0, 0, 11, 0)), B.MCN_CROP_TOO_LARGE),      # 11 columns before cropping
    (dict(xshape=(1 << 18, 4, 64, 64), fshape=(4, 64, 3, 3)), B.MCN_UNSUPPORTED),   # y has >= 2^31 elements
])
def test_convt_bad_geometry_is_a_status_code_everywhere(kw, code):
    d = tdesc(**kw)
    L = B.lib()
    assert L.mcn_convt_output_size(ctypes.byref(d), None, None) == code
    n = ctypes.c_size_t(0)
    assert L.mcn_convt_workspace_size(ctypes.byref(d), 0, ctypes.byref(n)) == code
    p = 4096
    assert B.mcn_convt_forward(d, p, p, p, p, None, 0, None) == code
    assert B.mcn_convt_backward_data(d, p, p, p, None, 0, None) == code
    assert B.mcn_convt_backward_filter(d, p, p, p, None, 0, None) == code
    assert B.mcn_convt_backward_bias(d, p, p, None, 0, None) == code
    assert B.mcn_convt_kernel_name(d, 0) is None


def test_convt_null_pointers_and_small_workspace_are_rejected():
    d = tdesc()
    p = 4096
    L = B.lib()
    assert L.mcn_convt_output_size(None, None, None) == B.MCN_BAD_ARG
    assert L.mcn_convt_workspace_size(ctypes.byref(d), 4, ctypes.byref(ctypes.c_size_t(0))) == B.MCN_BAD_ARG
    assert L.mcn_convt_workspace_size(ctypes.byref(d), 0, None) == B.MCN_BAD_ARG
    assert B.mcn_convt_forward(d, None, p, p, p, None, 0, None) == B.MCN_BAD_ARG
    assert B.mcn_convt_forward(d, p, None, p, p, None, 0, None) == B.MCN_BAD_ARG
    assert B.mcn_convt_forward(d, p, p, p, None, None, 0, None) == B.MCN_BAD_ARG
    assert B.mcn_convt_backward_data(d, None, p, p, None, 0, None) == B.MCN_BAD_ARG
    assert B.mcn_convt_backward_filter(d, p, p, None, None, 0, None) == B.MCN_BAD_ARG
    assert B.mcn_convt_backward_bias(d, p, None, None, 0, None) == B.MCN_BAD_ARG
    for op, call in [(B.MCN_OP_BACKWARD_BIAS, lambda ws, n: B.mcn_convt_backward_bias(d, p, p, ws, n, None)),
                     (B.MCN_OP_FORWARD, lambda ws, n: B.mcn_convt_forward(d, p, p, p, p, ws, n, None)),
                     (B.MCN_OP_BACKWARD_DATA, lambda ws, n: B.mcn_convt_backward_data(d, p, p, p, ws, n, None)),
                     (B.MCN_OP_BACKWARD_FILTER, lambda ws, n: B.mcn_convt_backward_filter(d, p, p, p, ws, n, None))]:
        need = B.mcn_convt_workspace_size(d, op)
        if need:
            assert call(p, need - 1) == B.MCN_WORKSPACE_TOO_SMALL
            assert call(None, need) == B.MCN_WORKSPACE_TOO_SMALL
    for op in range(4):
        assert B.mcn_convt_kernel_name(d, op)
    assert B.mcn_convt_kernel_name(d, 4) is None


# ---- spatial pooling ----
def pdesc(**kw):
    base = dict(xshape=(2, 3, 9, 8), window=(3, 2), stride=(2, 1), pad=(1, 0, 0, 1), method=B.MCN_POOL_MAX)
    base.update(kw)
    return B.make_pool_desc(**base)


def test_pool_output_size_closed_form():
    assert B.mcn_pool_output_size(pdesc()) == ((8 - 3 + 1) // 2 + 1, (9 - 2 + 1) // 1 + 1)
    assert B.mcn_pool_output_size(B.make_pool_desc((128, 96, 55, 55), (3, 3), (2, 2))) == (27, 27)
    assert B.mcn_pool_output_size(B.make_pool_desc((100, 32, 32, 32), (3, 3), (2, 2), (0, 1, 0, 1))) == (16, 16)


@pytest.mark.parametrize("kw,code", [
    (dict(window=(0, 2)), B.MCN_BAD_ARG),
    (dict(stride=(1, 0)), B.MCN_BAD_ARG),
    (dict(pad=(0, 0, -1, 0)), B.MCN_BAD_ARG),
    (dict(xshape=(2, 0, 9, 8)), B.MCN_BAD_ARG),
    (dict(method=2), B.MCN_BAD_ARG),
    (dict(pad=(3, 0, 0, 0)), B.MCN_PAD_TOO_LARGE),          # window height 3: pads <= 2
    (dict(pad=(0, 0, 0, 2)), B.MCN_PAD_TOO_LARGE),          # window width 2: pads <= 1
    (dict(xshape=(2, 3, 9, 1), window=(3, 2), pad=(0, 0, 0, 0)), B.MCN_FILTER_TOO_LARGE),
    (dict(xshape=(1 << 20, 64, 9, 8)), B.MCN_UNSUPPORTED),
])
def test_pool_bad_geometry_is_a_status_code_everywhere(kw, code):
    d = pdesc(**kw)
    L = B.lib()
    assert L.mcn_pool_output_size(ctypes.byref(d), None, None) == code
    p = 4096
    assert B.mcn_pool_forward(d, p, p, None) == code
    assert B.mcn_pool_backward(d, p, p, p, None, 0, None) == code
    assert L.mcn_pool_workspace_size(ctypes.byref(d), ctypes.byref(ctypes.c_size_t(0))) == code


def test_pool_null_pointers_are_rejected():
    d, p = pdesc(), 4096
    assert B.lib().mcn_pool_output_size(None, None, None) == B.MCN_BAD_ARG
    assert B.mcn_pool_forward(d, None, p, None) == B.MCN_BAD_ARG
    assert B.mcn_pool_forward(d, p, None, None) == B.MCN_BAD_ARG
    need = B.mcn_pool_workspace_size(d)
    assert need == 2 * 3 * 4 * 9      # one byte per output sample (4 x 9 per plane)
    assert B.mcn_pool_backward(d, None, p, p, p, need, None) == B.MCN_BAD_ARG       # max pooling needs x
    assert B.mcn_pool_backward(d, p, None, p, p, need, None) == B.MCN_BAD_ARG
    assert B.mcn_pool_backward(d, p, p, None, p, need, None) == B.MCN_BAD_ARG
    assert B.mcn_pool_backward(d, p, p, p, p, need - 1, None) == B.MCN_WORKSPACE_TOO_SMALL
    assert B.mcn_pool_backward(d, p, p, p, None, need, None) == B.MCN_WORKSPACE_TOO_SMALL
    assert B.mcn_pool_workspace_size(pdesc(method=B.MCN_POOL_AVG)) == 0
    assert B.lib().mcn_pool_workspace_size(ctypes.byref(d), None) == B.MCN_BAD_ARG


def test_probe_arguments_are_checked():
    # bad arguments come back as status codes before anything is launched
    sink = 4096
    assert B.mcn_probe_mfma(B.MCN_PREC_FP32, 1, None, B.MCN_PROBE_SINK_FLOATS, None)[0] == B.MCN_BAD_ARG
    assert B.mcn_probe_mfma(B.MCN_PREC_FP32, 0, sink, B.MCN_PROBE_SINK_FLOATS, None)[0] == B.MCN_BAD_ARG
    assert B.mcn_probe_mfma(5, 1, sink, B.MCN_PROBE_SINK_FLOATS, None)[0] == B.MCN_BAD_ARG
    assert B.mcn_probe_mfma(B.MCN_PREC_BF16, 1, sink, B.MCN_PROBE_SINK_FLOATS - 1, None)[0] == B.MCN_WORKSPACE_TOO_SMALL
    assert B.mcn_probe_copy(None, 4096, 16, None) == B.MCN_BAD_ARG
    assert B.mcn_probe_copy(4096, None, 16, None) == B.MCN_BAD_ARG
    assert B.mcn_probe_copy(4096 + 4, 8192, 16, None) == B.MCN_BAD_ARG       # misaligned source
    assert B.mcn_probe_copy(4096, 8192 + 8, 16, None) == B.MCN_BAD_ARG       # misaligned destination
    assert B.mcn_probe_copy(4096, 8192, 0, None) == B.MCN_OK                 # nothing to copy, nothing launched
    hdr = open(os.path.join(ROOT, "include", "mcnconv.h")).read()
    assert re.search(r"#define\s+MCN_PROBE_SINK_FLOATS\s+\(2048 \* 256\)", hdr)
    assert B.MCN_PROBE_SINK_FLOATS == 2048 * 256


def test_planner_puts_every_workload_layer_on_the_matrix_core_kernels():
    # host logic only: kernel choice and workspace sizes need no GPU (the planner assumes 256 compute units then)
    from paper_1412_4564_amd import synth
    for name, L in synth.LAYERS.items():
        for prec in (B.MCN_PREC_FP32, B.MCN_PREC_BF16):
            d = B.make_desc(synth.x_shape(L), synth.w_shape(L), L["stride"], L["pad"], prec)
            names = [B.mcn_conv_kernel_name(d, op) for op in range(4)]
            assert "direct" not in names, (name, names)
            sizes = [B.mcn_conv_workspace_size(d, op) for op in range(4)]
            assert all(0 <= s < (1 << 28) for s in sizes), (name, sizes)       # scratch stays below 256 MiB
    d = B.make_desc(synth.x_shape(synth.LAYERS["5a"]), synth.w_shape(synth.LAYERS["5a"]))
    assert [B.mcn_conv_kernel_name(d, op) for op in range(3)] == ["fc_gemm"] * 3
    # the 3x3 stride-1 layers: forward and input derivative on the kernel that computes pairs of output rows
    for name in ("4a", "4b", "4c"):
        L = synth.LAYERS[name]
        d = B.make_desc(synth.x_shape(L), synth.w_shape(L), L["stride"], L["pad"])
        wg = "wgrad_f23" if name == "4c" else "wgrad_f23_chunked"      # 4a, 4b stream from memory: chunked schedule
        assert [B.mcn_conv_kernel_name(d, op) for op in range(3)] == ["igemm_f23", "igemm_f23", wg], name
        # the plain order of summation, chosen per call
        d = B.make_desc(synth.x_shape(L), synth.w_shape(L), L["stride"], L["pad"], B.MCN_PREC_FP32_PLAIN)
        assert [B.mcn_conv_kernel_name(d, op) for op in range(3)] == ["igemm", "igemm", wg.replace("f23", "igemm")], name
    # bf16 operands: the deep layers on the bf16 kernels, the 3-channel first layers on the fp32 ones
    for name, expect in (("4b", ["igemm_bf16", "igemm_bf16", "wgrad_bf16"]), ("3a", ["igemm", "igemm", "wgrad_igemm"])):
        L = synth.LAYERS[name]
        d = B.make_desc(synth.x_shape(L), synth.w_shape(L), L["stride"], L["pad"], B.MCN_PREC_BF16)
        got = [B.mcn_conv_kernel_name(d, op).replace("_chunked", "") for op in range(3)]      # whichever schedule
        assert got == expect, name


def test_planner_handles_odd_geometries_on_the_host():
    # a sweep of descriptors through the size and workspace queries: every valid one must plan (or fall back)
    # without error, and the answers must not depend on the order of the queries (plans are cached per thread)
    import itertools
    seen = {}
    for H, Hf, S, P, D, K in itertools.product((1, 7, 30), (1, 3, 5), (1, 2, 3), (0, 2), (1, 3, 16, 40), (1, 24, 96)):
        if H + 2 * P < Hf:
            continue
        d = B.make_desc((3, D, H + 2, H), (K, D, Hf, Hf), (S, S), (P, P, P, 0))
        seen[(H, Hf, S, P, D, K)] = [B.mcn_conv_workspace_size(d, op) for op in range(4)]
    for key in list(seen)[::7]:
        H, Hf, S, P, D, K = key
        d = B.make_desc((3, D, H + 2, H), (K, D, Hf, Hf), (S, S), (P, P, P, 0))
        assert [B.mcn_conv_workspace_size(d, op) for op in range(4)] == seen[key], key


def test_environment_override_of_the_summation_order():
    """MCN_NO_WINO=1 (read once per process, for benchmarks) makes the default precision behave as
    MCN_PREC_FP32_PLAIN; without it the choice is the descriptor's, per call."""
    import os
    import subprocess
    import sys
    script = ("import sys; sys.path.insert(0, sys.argv[1])\n"
              "from paper_1412_4564_amd import binding as B, synth\n"
              "L = synth.LAYERS['4b']\n"
              "d = B.make_desc(synth.x_shape(L), synth.w_shape(L), L['stride'], L['pad'])\n"
              "print(','.join(B.mcn_conv_kernel_name(d, op) for op in range(3)))\n")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, "-c", script, root], env=dict(os.environ, MCN_NO_WINO="1"), capture_output=True,
                       text=True, timeout=120)
    assert r.returncode == 0 and r.stdout.strip() == "igemm,igemm,wgrad_igemm_chunked", (r.stdout, r.stderr[-500:])


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    """mcn_conv_backward_bias_static checks the descriptor, the pointers and the size of its fixed buffer on the host,
    before anything touches a GPU."""
    # 1x1 output planes with 300000 filters: one row of K values per partial sum exceeds the 1 MiB buffer
    d = B.make_desc((4, 2, 1, 1), (300000, 2, 1, 1))
    assert B.mcn_conv_workspace_size(d, B.MCN_OP_BACKWARD_BIAS) > B.MCN_STATIC_SCRATCH_BYTES
    assert B.mcn_conv_backward_bias_static(d, 16, 16, None) == B.MCN_STATIC_SCRATCH_EXCEEDED
    d = B.make_desc((4, 2, 8, 8), (6, 2, 3, 3))
    assert B.mcn_conv_backward_bias_static(d, None, 16, None) == B.MCN_BAD_ARG
    d.stride_h = 0
    assert B.mcn_conv_backward_bias_static(d, 16, 16, None) == B.MCN_BAD_ARG
    assert b"static buffer" in B.lib().mcn_status_string(B.MCN_STATIC_SCRATCH_EXCEEDED)


def test_split_operand_precision_picks_the_bf16_matrix_core_for_forward_and_dzdx_only():
    from paper_1412_4564_amd import synth
    for name in ("4a", "4b", "4c"):
        L = synth.LAYERS[name]
        d = B.make_desc(synth.x_shape(L), synth.w_shape(L), L["stride"], L["pad"], B.MCN_PREC_FP32_BF16X3)
        names = [B.mcn_conv_kernel_name(d, op) for op in range(3)]
        assert names[:2] == ["igemm_bf16x3", "igemm_bf16x3"] and names[2].startswith("wgrad_f23"), (name, names)
        assert B.mcn_conv_workspace_size(d, 0) < (1 << 28)
    L = synth.LAYERS["3a"]      # 3 channels: fp32 kernels
    d = B.make_desc(synth.x_shape(L), synth.w_shape(L), L["stride"], L["pad"], B.MCN_PREC_FP32_BF16X3)
    assert B.mcn_conv_kernel_name(d, 0) == "igemm"
