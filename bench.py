#!/usr/bin/env python3
"""Benchmark of the convolution block on one MI355X.

A "step" is one pass of the whole hot path -- forward, input derivative, filter
derivative and bias derivative -- over every layer of the workload, with all
operands already resident in HBM.  The default workload is the deep 3x3 stack
(224x224x64->64, 56x56x256->256, 14x14x512->512; stride 1, pad 1, N=32, fp32)
on which the headline metric is quoted.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload vgg3x3|<layer names>]

Layer names t1..t5 are shapes of the convolution transpose block (timing table only; the
headline metric is quoted on the convolution block).
"""
import argparse
import json
import os
import sys
import time

import numpy as np
import torch

from paper_1412_4564_amd import binding as B
from paper_1412_4564_amd import synth

FP32_MFMA_PEAK_TFLOPS = 157.3     # 256 CU x 256 flop/clk x 2.4 GHz
BF16_MFMA_PEAK_TFLOPS = 2500.0    # dense bf16 MFMA (kernels named *_bf16 run on it)
HBM_PEAK_GBS = 8000.0

WORKLOADS = {"vgg3x3": ["4a", "4b", "4c"]}
ROOT = os.path.dirname(os.path.abspath(__file__))
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "vgg3x3_hbm_traffic.txt")
MFMA_FILE = os.path.join(ROOT, "profiles", "vgg3x3_mfma_counters.txt")

FUSED_AWAY = "(with backward_filter)"      # 'kernel' of a call that is not made: its result came with another's

# The roof that bounds each layer's three matrix passes (the bias derivative is always a stream from memory): the
# 3-channel first layers, the 1x1 layer and the tiny irregular layer move more bytes than the matrix core can be
# kept busy with; the fully-connected layer is priced against both.
BOUND = {"1": "hbm", "2a": "hbm", "3a": "hbm", "5b": "hbm", "5c": "hbm"}


def sources_id():
    """Identifies the kernel sources a counter summary under profiles/ was taken from: the summaries carry the
    same figure, and a summary of other sources is not quoted."""
    import hashlib
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_1412_4564_amd", "csrc")
    for name in sorted(os.listdir(d)):
        if name.endswith((".h", ".hip")):
            with open(os.path.join(d, name), "rb") as f:
                h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def profile_lines(path):
    """Lines of a committed counter summary, or [] if it is absent or was taken from other kernel sources
    (line 'SOURCES <id>')."""
    try:
        with open(path) as f:
            lines = [l.split() for l in f]
    except OSError:
        return []
    if not any(len(t) == 2 and t[0] == "SOURCES" and t[1] == sources_id() for t in lines):
        return []
    return lines


def issued_share(kernel):
    """Flops the matrix core executes per flop of the plain sum, by arithmetic: the *_f23 kernels take the three
    row taps of a 3x3 filter for two output rows with four products instead of six; the bf16x3 kernels form every
    product from three bf16 products.  (Padding of channel and filter counts to tile sizes comes on top; the
    counter summary, where there is one, has the measured figure.)"""
    return 2.0 / 3.0 if "_f23" in kernel else 3.0 if "bf16x3" in kernel else 1.0


def measured_mfma(call):
    """(flops the matrix core executed, its busy fraction) for one call, from the committed summary of a
    rocprofv3 --pmc run of this benchmark (lines 'CALL <layer>.<operation> <mfma flops> <busy fraction>'),
    or None."""
    for t in profile_lines(MFMA_FILE):
        if len(t) == 4 and t[0] == "CALL" and t[1] == call:
            return float(t[2]), float(t[3])
    return None


def measured_traffic(call):
    """HBM bytes (fetch + write) of one call, from the committed summary of the two rocprofv3 --pmc
    runs of this benchmark (lines 'TOTAL <layer>.<operation> <fetch bytes> <write bytes>'); None if
    the summary does not hold the call or is stale."""
    for t in profile_lines(TRAFFIC_FILE):
        if len(t) == 4 and t[0] == "TOTAL" and t[1] == call:
            return int(float(t[2]) + float(t[3]))
    return None


OPS = ["forward", "backward_data", "backward_filter", "backward_bias"]


def layer_macs(L, ho, wo):
    return ho * wo * L["K"] * L["N"] * L["Hf"] * L["Wf"] * L["Df"]


class LayerState:
    op_names = OPS

    def __init__(self, name, L, precision, rotate_mb=0):
        self.name, self.L = name, L
        self.st, self.pad, self.prec = L["stride"], L["pad"], precision
        self.x = synth.make_x(L).cuda()
        self.w = synth.make_w(L).cuda()
        self.b = synth.make_b(L).cuda()
        desc = B.make_desc(self.x.shape, self.w.shape, self.st, self.pad, precision)
        self.desc = desc
        self.ho, self.wo = B.mcn_conv_output_size(desc)
        self.p = synth.make_dzdy(L, self.ho, self.wo).cuda()
        self.y = torch.empty_like(self.p)
        self.dx = torch.empty_like(self.x)
        self.dw = torch.empty_like(self.w)
        self.db = torch.empty_like(self.b)
        # optional rotation through several copies of the activations, so that repeated launches are
        # not served from the 256 MB last-level cache (for the memory-bound layers)
        self.sets = [(self.x, self.p, self.y, self.dx)]
        if rotate_mb > 0:
            per_set = 4 * (2 * self.x.numel() + 2 * self.p.numel())
            n_sets = min(256, max(1, -(-rotate_mb * (1 << 20) // per_set)))
            for _ in range(n_sets - 1):
                self.sets.append((self.x.clone(), self.p.clone(), torch.empty_like(self.p), torch.empty_like(self.x)))
        self.turn = 0
        self.macs = layer_macs(L, self.ho, self.wo)
        self.kernels = [B.mcn_conv_kernel_name(desc, op) for op in range(4)]
        # dzdw and dzdb from one kernel where the library has one (the backward mode returns both): the step then
        # calls mcn_conv_backward_filter_bias for the two, and the bias derivative's own call is not made
        self.fused_bias = B.mcn_conv_kernel_name(desc, B.MCN_OP_BACKWARD_FILTER_BIAS) == "wgrad_f23+bias"
        if self.fused_bias:
            self.kernels[2], self.kernels[3] = "wgrad_f23+bias", FUSED_AWAY
        ws = max(B.mcn_conv_workspace_size(desc, op) for op in range(5))
        self.ws = torch.empty(max(ws, 16), dtype=torch.uint8, device="cuda")
        # algorithmic bytes per operation: each operand once
        nx, nw, ny = self.x.numel(), self.w.numel(), self.p.numel()
        self.bytes = [4 * (nx + nw + ny), 4 * (ny + nw + nx), 4 * (nx + ny + nw), 4 * (ny + L["K"])]

    def shape_info(self):
        L = self.L
        return {"x_HWDN": [L["H"], L["W"], L["D"], L["N"]], "w_HWDK": [L["Hf"], L["Wf"], L["Df"], L["K"]]}

    def with_precision(self, precision):
        """The same layer on the same device arrays under another MCN_PREC_* value."""
        import copy
        o = copy.copy(self)
        o.prec = precision
        o.desc = B.make_desc(self.x.shape, self.w.shape, self.st, self.pad, precision)
        o.kernels = [B.mcn_conv_kernel_name(o.desc, op) for op in range(4)]
        o.fused_bias = B.mcn_conv_kernel_name(o.desc, B.MCN_OP_BACKWARD_FILTER_BIAS) == "wgrad_f23+bias"
        if o.fused_bias:
            o.kernels[2], o.kernels[3] = "wgrad_f23+bias", FUSED_AWAY
        ws = max(B.mcn_conv_workspace_size(o.desc, op) for op in range(5))
        o.ws = torch.empty(max(ws, 16), dtype=torch.uint8, device="cuda")
        return o

    def run(self, op, stream):
        d, ws, n = self.desc, self.ws.data_ptr(), self.ws.numel()
        x, p, y, dx = self.sets[self.turn % len(self.sets)]
        if op == 3:
            self.turn += 1
        if op == 0:
            st = B.mcn_conv_forward(d, x.data_ptr(), self.w.data_ptr(), self.b.data_ptr(), y.data_ptr(), ws, n, stream)
        elif op == 1:
            st = B.mcn_conv_backward_data(d, self.w.data_ptr(), p.data_ptr(), dx.data_ptr(), ws, n, stream)
        elif op == 2 and self.fused_bias:
            st = B.mcn_conv_backward_filter_bias(d, x.data_ptr(), p.data_ptr(), self.dw.data_ptr(), self.db.data_ptr(),
                                                 ws, n, stream)
        elif op == 2:
            st = B.mcn_conv_backward_filter(d, x.data_ptr(), p.data_ptr(), self.dw.data_ptr(), ws, n, stream)
        elif self.fused_bias:
            st = 0          # dzdb came with dzdw
        else:
            st = B.mcn_conv_backward_bias(d, p.data_ptr(), self.db.data_ptr(), ws, n, stream)
        if st:
            raise B.McnError(st, OPS[op])


class ConvtLayerState:
    """The convolution transpose block on one of the synth.CONVT_LAYERS shapes (same interface)."""
    op_names = OPS

    def __init__(self, name, L, precision, rotate_mb=0):
        self.name, self.L, self.prec = name, L, precision
        self.x = synth.make_tx(L).cuda()
        self.w = synth.make_tf(L).cuda()
        self.b = synth.make_tb(L).cuda()
        desc = B.make_convt_desc(self.x.shape, self.w.shape, L["up"], L["crop"], L["groups"], precision)
        self.desc = desc
        self.ho, self.wo = B.mcn_convt_output_size(desc)
        self.p = synth.make_tdzdy(L, self.ho, self.wo).cuda()
        self.y = torch.empty_like(self.p)
        self.dx = torch.empty_like(self.x)
        self.dw = torch.empty_like(self.w)
        self.db = torch.empty_like(self.b)
        # every input sample meets every filter tap once per output channel of its group
        self.macs = L["H"] * L["W"] * L["D"] * L["N"] * L["Hf"] * L["Wf"] * L["Kf"]
        self.kernels = [B.mcn_convt_kernel_name(desc, op) for op in range(4)]
        ws = max(B.mcn_convt_workspace_size(desc, op) for op in range(4))
        self.ws = torch.empty(max(ws, 16), dtype=torch.uint8, device="cuda")
        nx, nw, ny = self.x.numel(), self.w.numel(), self.p.numel()
        self.bytes = [4 * (nx + nw + ny), 4 * (ny + nw + nx), 4 * (nx + ny + nw), 4 * (ny + self.b.numel())]

    def shape_info(self):
        L = self.L
        return {"block": "convt", "x_HWDN": [L["H"], L["W"], L["D"], L["N"]], "f_HWKD": [L["Hf"], L["Wf"], L["Kf"], L["D"]],
                "groups": L["groups"], "up": list(L["up"]), "crop": list(L["crop"])}

    def run(self, op, stream):
        d, ws, n = self.desc, self.ws.data_ptr(), self.ws.numel()
        if op == 0:
            st = B.mcn_convt_forward(d, self.x.data_ptr(), self.w.data_ptr(), self.b.data_ptr(), self.y.data_ptr(), ws, n, stream)
        elif op == 1:
            st = B.mcn_convt_backward_data(d, self.w.data_ptr(), self.p.data_ptr(), self.dx.data_ptr(), ws, n, stream)
        elif op == 2:
            st = B.mcn_convt_backward_filter(d, self.x.data_ptr(), self.p.data_ptr(), self.dw.data_ptr(), ws, n, stream)
        else:
            st = B.mcn_convt_backward_bias(d, self.p.data_ptr(), self.db.data_ptr(), ws, n, stream)
        if st:
            raise B.McnError(st, "convt " + OPS[op])


def fused_relu_report(layers, stream_obj, steps):
    """Per layer: conv+ReLU forward fused (one call) against conv forward followed by a separate in-place
    ReLU pass, and the fused mask+bias backward against a separate masking pass followed by the bias
    derivative.  The separate passes are torch's elementwise kernels: they only stand for 'one more
    read and write of y' in the comparison."""
    stream = stream_obj.cuda_stream

    def timed(fn):
        # warm-up: at least 20 ms of this very call, so that the clock has left its idle state
        t0 = time.perf_counter()
        while True:
            for _ in range(2):
                fn()
            torch.cuda.synchronize()
            if time.perf_counter() - t0 > 0.02:
                break
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream_obj)
        for _ in range(steps):
            fn()
        b.record(stream_obj)
        torch.cuda.synchronize()
        return a.elapsed_time(b) / steps

    out = {}
    for Ls in layers:
        if not isinstance(Ls, LayerState):
            continue
        d, ws, n = Ls.desc, Ls.ws.data_ptr(), Ls.ws.numel()
        x, w, b, y, p = Ls.x, Ls.w, Ls.b, Ls.y, Ls.p
        dzdp = torch.empty_like(p)
        zero = torch.zeros((), dtype=torch.float32, device="cuda")

        def check(st):
            if st:
                raise B.McnError(st, "fused relu")

        def fwd_fused():
            check(B.mcn_conv_relu_forward(d, x.data_ptr(), w.data_ptr(), b.data_ptr(), y.data_ptr(), ws, n, stream))

        def fwd_unfused():
            check(B.mcn_conv_forward(d, x.data_ptr(), w.data_ptr(), b.data_ptr(), y.data_ptr(), ws, n, stream))
            torch.relu_(y)

        def bwd_fused():
            check(B.mcn_conv_relu_backward_bias(d, y.data_ptr(), p.data_ptr(), dzdp.data_ptr(), Ls.db.data_ptr(), ws, n, stream))

        def bwd_unfused():
            torch.where(y > 0, p, zero, out=dzdp)
            check(B.mcn_conv_backward_bias(d, dzdp.data_ptr(), Ls.db.data_ptr(), ws, n, stream))

        t_ff, t_fu = timed(fwd_fused), timed(fwd_unfused)
        fwd_fused()
        t_bf, t_bu = timed(bwd_fused), timed(bwd_unfused)
        ybytes = 4 * p.numel()
        out[Ls.name] = {"forward_fused_ms": round(t_ff, 4), "forward_separate_relu_ms": round(t_fu, 4),
                        "mask_bias_fused_ms": round(t_bf, 4), "mask_then_bias_ms": round(t_bu, 4),
                        "mask_bias_fused_GBps": round(3 * ybytes / t_bf / 1e6, 1),     # reads y, dzdy; writes dzdp
                        "frac_of_hbm_peak": round(3 * ybytes / t_bf / 1e6 / HBM_PEAK_GBS, 4)}
    return out


class PoolLayerState:
    """The spatial pooling block on one of the synth.POOL_LAYERS shapes: forward and backward."""
    op_names = ["forward", "backward"]

    def __init__(self, name, L, precision, rotate_mb=0):
        self.name, self.L = name, L
        self.method = B.MCN_POOL_MAX if L["method"] == "max" else B.MCN_POOL_AVG
        self.x = synth.make_px(L).cuda()
        self.desc = B.make_pool_desc(self.x.shape, L["window"], L["stride"], L["pad"], self.method)
        self.ho, self.wo = B.mcn_pool_output_size(self.desc)
        self.p = synth.make_pdzdy(L, self.ho, self.wo).cuda()
        self.sets = [(self.x, self.p, torch.empty_like(self.p), torch.empty_like(self.x))]
        if rotate_mb > 0:
            per_set = 4 * (2 * self.x.numel() + 2 * self.p.numel())
            for _ in range(min(256, max(1, -(-rotate_mb * (1 << 20) // per_set))) - 1):
                self.sets.append((self.x.clone(), self.p.clone(), torch.empty_like(self.p), torch.empty_like(self.x)))
        self.turn = 0
        self.macs = 0
        self.ws = torch.empty(max(B.mcn_pool_workspace_size(self.desc), 16), dtype=torch.uint8, device="cuda")
        self.kernels = ["pool_forward", "pool_backward"]
        nx, ny = self.x.numel(), self.p.numel()
        # algorithmic bytes: forward reads x, writes y; backward reads dzdy (and x for max), writes dzdx
        self.bytes = [4 * (nx + ny), 4 * (ny + nx + (nx if L["method"] == "max" else 0))]

    def shape_info(self):
        L = self.L
        return {"block": "pool", "x_HWDN": [L["H"], L["W"], L["D"], L["N"]], "window": list(L["window"]),
                "stride": list(L["stride"]), "pad": list(L["pad"]), "method": L["method"]}

    def run(self, op, stream):
        x, p, y, dx = self.sets[self.turn % len(self.sets)]
        if op == 0:
            st = B.mcn_pool_forward(self.desc, x.data_ptr(), y.data_ptr(), stream)
        else:
            st = B.mcn_pool_backward(self.desc, x.data_ptr(), p.data_ptr(), dx.data_ptr(), self.ws.data_ptr(),
                                     self.ws.numel(), stream)
            self.turn += 1
        if st:
            raise B.McnError(st, "pool " + self.op_names[op])


def make_state(name, precision, rotate_mb):
    if name in synth.POOL_LAYERS:
        return PoolLayerState(name, synth.POOL_LAYERS[name], precision, rotate_mb)
    if name in synth.CONVT_LAYERS:
        return ConvtLayerState(name, synth.CONVT_LAYERS[name], precision, rotate_mb)
    return LayerState(name, synth.LAYERS[name], precision, rotate_mb)


def measured_ceilings(stream_obj):
    """What this GPU sustains, measured here with HIP events: the register-only MFMA loops of the
    library (no memory, LDS or barrier in the loop) and a plain copy of 512 MiB (read + write = 1 GiB
    of traffic, larger than the last-level cache)."""
    stream = stream_obj.cuda_stream
    sink = torch.empty(B.MCN_PROBE_SINK_FLOATS, dtype=torch.float32, device="cuda")

    def timed(fn, reps=3):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream_obj)
        for _ in range(reps):
            fn()
        e1.record(stream_obj)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    out = {}
    for key, prec in (("mfma_f32_TFLOPs", B.MCN_PREC_FP32), ("mfma_bf16_TFLOPs", B.MCN_PREC_BF16)):
        flops = []

        def loop():
            st, f = B.mcn_probe_mfma(prec, 8000, sink.data_ptr(), sink.numel(), stream)
            if st:
                raise B.McnError(st, "mcn_probe_mfma")
            flops.append(f)
        ms = timed(loop)
        out[key] = round(flops[0] / ms / 1e9, 1)
    n = 128 * 1024 * 1024
    src = torch.ones(n, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)

    def copy():
        st = B.mcn_probe_copy(src.data_ptr(), dst.data_ptr(), n, stream)
        if st:
            raise B.McnError(st, "mcn_probe_copy")
    out["copy_GBps"] = round(8.0 * n / timed(copy) / 1e6, 1)
    return out


def cpu_baseline(names):
    """The oracle as it stands, timed on this machine's host cores on a bounded sample
    of the same workload: the same layers at a reduced batch."""
    import oracle
    sample_n = {"4a": 12, "4b": 12, "4c": 24}      # about 10-20 s of host time in all
    flops, secs, desc = 0.0, 0.0, []
    for name in names:
        L = synth.with_batch(synth.LAYERS[name], sample_n.get(name, 1))
        st, pad = L["stride"], L["pad"]
        x = synth.make_x(L).numpy().astype(np.float64)
        w = synth.make_w(L).numpy().astype(np.float64)
        b = synth.make_b(L).numpy().astype(np.float64)
        ho, wo = oracle.output_size(x.shape, w.shape, st, pad)
        p = synth.make_dzdy(L, ho, wo).numpy().astype(np.float64)
        t0 = time.perf_counter()
        oracle.forward(x, w, b, st, pad)
        oracle.backward_data(x.shape, w, p, st, pad)
        oracle.backward_filter(x, w.shape, p, st, pad)
        oracle.backward_bias(x.shape, w.shape, p, st, pad)
        secs += time.perf_counter() - t0
        flops += 3 * 2.0 * layer_macs(L, ho, wo)
        desc.append("%s at N=%d" % (name, L["N"]))
    return {"value": flops / secs / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "fwd+bwd of layers " + ", ".join(desc) + " (fp64 loop nest, %.1f s)" % secs}


def time_calls(layers, stream_obj, steps, warmup):
    """(seconds per step, ms per call [layer, op]) for the step 'every operation of every layer': `warmup` untimed
    steps, exactly `steps` timed ones between two synchronisations, then the same steps again with an event after
    every call (a separate pass, so that the event records do not perturb the first figure)."""
    stream = stream_obj.cuda_stream
    calls = [(li, op) for li, Ls in enumerate(layers) for op in range(len(Ls.op_names))]

    def step(events=None):
        for li, op in calls:
            layers[li].run(op, stream)
            if events is not None:
                ev = torch.cuda.Event(enable_timing=True)
                ev.record(stream_obj)
                events.append(ev)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    per = np.zeros((len(layers), 4))
    for _ in range(steps):
        start = torch.cuda.Event(enable_timing=True)
        start.record(stream_obj)
        evs = []
        step(evs)
        torch.cuda.synchronize()
        prev = start
        for (li, op), ev in zip(calls, evs):
            per[li, op] += prev.elapsed_time(ev)
            prev = ev
    return elapsed / steps, per / steps


def call_report(Ls, op, ms):
    """One call: kernel, time, the rates of the plain sum and of what the matrix core executes, and the fraction
    of the roof that bounds it."""
    kernel = Ls.kernels[op]
    e = {"kernel": kernel, "ms": round(float(ms), 4)}
    if kernel == FUSED_AWAY:
        return e
    e["GBps"] = round(Ls.bytes[op] / ms / 1e6, 1)
    matrix_pass = op < 3 and Ls.macs and len(Ls.op_names) == 4
    if matrix_pass:
        tf = 2.0 * Ls.macs / ms / 1e9
        e["TFLOPs"] = round(tf, 2)
        e["issued_TFLOPs"] = round(issued_share(kernel) * tf, 2)
    bound = "mfma" if matrix_pass and BOUND.get(Ls.name, "mfma") == "mfma" else "hbm"
    e["bound"] = bound
    if bound == "mfma":
        peak = BF16_MFMA_PEAK_TFLOPS if "bf16" in kernel else FP32_MFMA_PEAK_TFLOPS
        e["frac"] = round(e["issued_TFLOPs"] / peak, 4)
    else:
        e["frac"] = round(e["GBps"] / HBM_PEAK_GBS, 4)
    return e


def all_layers_report(stream_obj, precision, have, reps=10):
    """Every layer of the synthetic workloads, one call at a time, outside the timed region: `reps` launches of the
    call between two events.  Activations rotate through copies of at least 600 MiB in all (the last-level cache
    holds 256 MB), so a launch is not served from the cache by the launch before it."""
    stream = stream_obj.cuda_stream
    out = {}
    for name in synth.LAYERS:
        Ls = have.get(name)
        mine = Ls is None
        if mine:
            Ls = LayerState(name, synth.LAYERS[name], precision, rotate_mb=600)
        for op in range(4):
            if Ls.kernels[op] == FUSED_AWAY:
                out["%s.%s" % (name, OPS[op])] = {"kernel": FUSED_AWAY}
                continue
            # warm-up: at least 20 ms of this very call, so that the clock has left its idle state (the layer's
            # inputs were just generated on the host; the first launches after a pause run some 15 % slower)
            t0 = time.perf_counter()
            while True:
                for _ in range(5):
                    Ls.run(op, stream); Ls.turn += 1
                torch.cuda.synchronize()
                if time.perf_counter() - t0 > 0.02:
                    break
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream_obj)
            for _ in range(reps):
                Ls.run(op, stream); Ls.turn += 1
            e1.record(stream_obj)
            torch.cuda.synchronize()
            out["%s.%s" % (name, OPS[op])] = call_report(Ls, op, e0.elapsed_time(e1) / reps)
        if mine:
            del Ls
            torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="vgg3x3", help="vgg3x3 or comma-separated layer names (e.g. 2b,3b)")
    ap.add_argument("--precision", default="fp32", choices=["fp32", "fp32-plain", "bf16", "bf16x3"],
                    help="fp32: the library's default order of summation; fp32-plain: MCN_PREC_FP32_PLAIN")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--rotate-mb", type=int, default=0,
                    help="rotate each layer's activations through copies totalling at least this many MiB "
                         "(cold-cache timing of the memory-bound layers)")
    ap.add_argument("--fused-relu", action="store_true",
                    help="also time the fused conv+ReLU calls against their unfused sequences (extra object "
                         "'fused_relu' in the JSON line)")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip the measured ceilings (register-only MFMA loops, plain copy) in 'measured_ceilings'")
    ap.add_argument("--no-all-layers", action="store_true",
                    help="skip the per-call table of all twelve workload layers ('all_layers')")
    ap.add_argument("--no-plain-leg", action="store_true",
                    help="skip the second timed leg in the plain order of summation ('value_plain_order')")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB elementwise copy three times, so that a counter run "
                         "(rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE) holds a kernel of known traffic to scale by")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU; --gpus %d is not supported (across GPUs the path would shard "
                 "over the batch, with one all-reduce of dzdw and dzdb)" % args.gpus)
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    torch.cuda.set_device(0)
    names = WORKLOADS.get(args.workload) or args.workload.split(",")
    prec = {"fp32": B.MCN_PREC_FP32, "fp32-plain": B.MCN_PREC_FP32_PLAIN, "bf16": B.MCN_PREC_BF16,
            "bf16x3": B.MCN_PREC_FP32_BF16X3}[args.precision]
    fp32 = prec != B.MCN_PREC_BF16
    headline = args.workload == "vgg3x3"
    layers = [make_state(n, prec, args.rotate_mb) for n in names]
    stream_obj = torch.cuda.current_stream()

    sec_per_step, per = time_calls(layers, stream_obj, args.steps, args.warmup)

    flops_step = sum(3 * 2.0 * Ls.macs for Ls in layers)      # pooling layers count no flops
    ms_per_step = 1e3 * sec_per_step
    value = flops_step / sec_per_step / 1e12

    # dominant kernel: the call that takes the most time per step
    li, op = np.unravel_index(np.argmax(per), per.shape)
    dom = layers[li]
    detail = {}
    issued_step = 0.0        # flops the matrix core executes per step (see issued_share)
    for i, Ls in enumerate(layers):
        for o in range(len(Ls.op_names)):
            detail["%s.%s" % (Ls.name, Ls.op_names[o])] = call_report(Ls, o, per[i, o])
            if o < 3 and Ls.macs and Ls.kernels[o] != FUSED_AWAY:
                issued_step += issued_share(Ls.kernels[o]) * 2.0 * Ls.macs
    dom_call = "%s.%s" % (dom.name, dom.op_names[op])
    traffic = measured_traffic(dom_call) if headline and prec == B.MCN_PREC_FP32 else None
    if op < 3 and dom.macs:
        # 'achieved' = the flops the matrix core executes for the call (what its peak bounds); 'algorithmic_equiv' =
        # the flops of the sum as the paper writes it, 2 * MACs (the *_f23 kernels execute two thirds of them)
        equiv = 2.0 * dom.macs / per[li, op] / 1e9
        peak = BF16_MFMA_PEAK_TFLOPS if "bf16" in dom.kernels[op] else FP32_MFMA_PEAK_TFLOPS
        ach, source = issued_share(dom.kernels[op]) * equiv, "arithmetic (2/3 of 2*MACs for *_f23 kernels, else all)"
        counters = measured_mfma(dom_call) if headline and prec == B.MCN_PREC_FP32 else None
        if counters:
            ach, source = counters[0] / per[li, op] / 1e9, "profiles/vgg3x3_mfma_counters.txt (SQ_INSTS_VALU_MFMA_MOPS_F32)"
        roof = {"bound": "mfma", "achieved": round(ach, 2), "peak": peak, "unit": "TFLOP/s", "frac": round(ach / peak, 4),
                "achieved_source": source, "algorithmic_equiv": round(equiv, 2), "traffic": traffic,
                "kernel": "%s (%s)" % (dom_call, dom.kernels[op])}
        if counters:
            roof["profiled_mfma_util"] = counters[1]
    else:
        ach = dom.bytes[op] / per[li, op] / 1e6
        roof = {"bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": traffic, "kernel": "%s (%s)" % (dom_call, dom.kernels[op])}

    issued_tflops = issued_step / sec_per_step / 1e12
    out = {
        "metric": "conv fwd+bwd TFLOP/s (%s) on VGG-style 3x3 layers" % ("fp32" if fp32 else "bf16 operands, fp32 accumulation"),
        "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": ("f32" if prec != B.MCN_PREC_FP32_BF16X3 else "f32 arrays, bf16x3 products, f32 accumulation") if fp32 else "bf16-in/f32-acc",
        "data": "synthetic",
        "config": {"workload": "conv fwd+bwd (dzdx, dzdw, dzdb) of layers " + ",".join(names) +
                               " (3x3 stride 1 pad 1, N=32)" if headline else
                               "conv fwd+bwd of layers " + ",".join(names),
                   "summation_order": "plain" if prec == B.MCN_PREC_FP32_PLAIN else "default",
                   "layers": {Ls.name: Ls.shape_info() for Ls in layers}},
        # 'value' counts 2 * MACs of the plain sum; the matrix core executes fewer flops for it in the *_f23 kernels:
        "mfma_issued_TFLOPs": round(issued_tflops, 3),
        "mfma_issued_frac_of_peak": round(issued_tflops / (FP32_MFMA_PEAK_TFLOPS if fp32 else BF16_MFMA_PEAK_TFLOPS), 4),
        "roofline": roof,
        "calls": detail,
    }
    if prec == B.MCN_PREC_FP32 and not args.no_plain_leg and all(n in synth.LAYERS for n in names):
        # second timed leg: the same step with every product of the paper's sum formed and added one by one
        plain = [Ls.with_precision(B.MCN_PREC_FP32_PLAIN) for Ls in layers]
        sec_plain, per_plain = time_calls(plain, stream_obj, args.steps, args.warmup)
        out["value_plain_order"] = round(flops_step / sec_plain / 1e12, 3)
        out["ms_per_step_plain_order"] = round(1e3 * sec_plain, 4)
        out["plain_order_frac_of_peak"] = round(flops_step / sec_plain / 1e12 / FP32_MFMA_PEAK_TFLOPS, 4)
        out["calls_plain_order"] = {"%s.%s" % (Ls.name, Ls.op_names[o]): call_report(Ls, o, per_plain[i, o])
                                    for i, Ls in enumerate(plain) for o in range(4)}
        del plain
        # third timed leg: fp32 arrays with the operands of forward / dzdx split into two bf16 planes on chip
        # (MCN_PREC_FP32_BF16X3: three bf16 MFMAs per product, 16 significant bits, fp32 accumulation)
        split = [Ls.with_precision(B.MCN_PREC_FP32_BF16X3) for Ls in layers]
        sec_split, per_split = time_calls(split, stream_obj, args.steps, args.warmup)
        out["value_bf16x3_operands"] = round(flops_step / sec_split / 1e12, 3)
        out["ms_per_step_bf16x3_operands"] = round(1e3 * sec_split, 4)
        out["calls_bf16x3_operands"] = {"%s.%s" % (Ls.name, Ls.op_names[o]): call_report(Ls, o, per_split[i, o])
                                        for i, Ls in enumerate(split) for o in range(4)}
        del split
    if not args.no_ceilings:
        # outside the timed region: what the chip sustains, so that the fraction of the published peak in
        # 'roofline' can be read beside the fraction of a ceiling measured on this very GPU
        ceil = measured_ceilings(stream_obj)
        out["measured_ceilings"] = ceil
        top = (ceil["copy_GBps"] if roof["bound"] == "hbm" else
               ceil["mfma_bf16_TFLOPs"] if roof["peak"] == BF16_MFMA_PEAK_TFLOPS else ceil["mfma_f32_TFLOPs"])
        roof["frac_of_measured_ceiling"] = round(roof["achieved"] / top, 4)
    if args.fused_relu:
        out["fused_relu"] = fused_relu_report(layers, stream_obj, args.steps)
    if not args.no_all_layers and headline and fp32:
        # layers whose activations exceed the last-level cache need no rotation: their state is reused
        big = {Ls.name: Ls for Ls in layers if 4 * (Ls.x.numel() + Ls.p.numel()) >= (256 << 20)}
        out["all_layers"] = all_layers_report(stream_obj, prec, big)
    if args.copy_calibration:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)      # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
    if not args.no_cpu_baseline and all(n in synth.LAYERS for n in names):
        out["cpu_baseline"] = cpu_baseline(names)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
