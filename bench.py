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
TRAFFIC_FILE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "vgg3x3_hbm_traffic.txt")


FUSED_AWAY = "(with backward_filter)"      # 'kernel' of a call that is not made: its result came with another's


def issued_share(kernel):
    """Flops the matrix core executes per flop of the plain sum: the *_f23 kernels take the three row taps of a
    3x3 filter for two output rows with four products instead of six."""
    return 2.0 / 3.0 if "_f23" in kernel else 1.0


def measured_traffic(call):
    """HBM bytes (fetch + write) of one call, from the committed summary of the two rocprofv3 --pmc
    runs of this benchmark (lines 'TOTAL <layer>.<operation> <fetch bytes> <write bytes>'); None if
    the summary does not hold the call."""
    try:
        with open(TRAFFIC_FILE) as f:
            for line in f:
                t = line.split()
                if len(t) == 4 and t[0] == "TOTAL" and t[1] == call:
                    return int(float(t[2]) + float(t[3]))
    except OSError:
        pass
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
        for _ in range(2):
            fn()
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="vgg3x3", help="vgg3x3 or comma-separated layer names (e.g. 2b,3b)")
    ap.add_argument("--precision", default="fp32", choices=["fp32", "bf16"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--rotate-mb", type=int, default=0,
                    help="rotate each layer's activations through copies totalling at least this many MiB "
                         "(cold-cache timing of the memory-bound layers)")
    ap.add_argument("--fused-relu", action="store_true",
                    help="also time the fused conv+ReLU calls against their unfused sequences (extra object "
                         "'fused_relu' in the JSON line)")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip the measured ceilings (register-only MFMA loops, plain copy) in 'measured_ceilings'")
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
    prec = B.MCN_PREC_BF16 if args.precision == "bf16" else B.MCN_PREC_FP32
    layers = [make_state(n, prec, args.rotate_mb) for n in names]
    stream_obj = torch.cuda.current_stream()
    stream = stream_obj.cuda_stream

    calls = [(li, op) for li, Ls in enumerate(layers) for op in range(len(Ls.op_names))]

    def step(events=None):
        for li, op in calls:
            layers[li].run(op, stream)
            if events is not None:
                ev = torch.cuda.Event(enable_timing=True)
                ev.record(stream_obj)
                events.append(ev)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # timed region: exactly --steps steps
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    # per-call durations with events on the launch stream (a second, separately timed pass of the same steps,
    # so that the event records do not perturb the headline number)
    per = np.zeros((len(layers), 4))
    for _ in range(args.steps):
        start = torch.cuda.Event(enable_timing=True)
        start.record(stream_obj)
        evs = []
        step(evs)
        torch.cuda.synchronize()
        prev = start
        for (li, op), ev in zip(calls, evs):
            per[li, op] += prev.elapsed_time(ev)
            prev = ev
    per /= args.steps     # ms per call

    flops_step = sum(3 * 2.0 * Ls.macs for Ls in layers)      # pooling layers count no flops
    ms_per_step = 1e3 * elapsed / args.steps
    value = flops_step / (elapsed / args.steps) / 1e12

    # dominant kernel: the call that takes the most time per step
    li, op = np.unravel_index(np.argmax(per), per.shape)
    dom = layers[li]
    detail = {}
    issued_step = 0.0        # flops the matrix core executes per step (see issued_share)
    for i, Ls in enumerate(layers):
        for o in range(len(Ls.op_names)):
            ms = per[i, o]
            e = {"kernel": Ls.kernels[o], "ms": round(float(ms), 4)}
            if Ls.kernels[o] != FUSED_AWAY:
                e["GBps"] = round(Ls.bytes[o] / ms / 1e6, 1)
            if o < 3 and Ls.macs:
                e["TFLOPs"] = round(2.0 * Ls.macs / ms / 1e9, 2)
                if issued_share(Ls.kernels[o]) != 1.0:
                    e["issued_TFLOPs"] = round(issued_share(Ls.kernels[o]) * 2.0 * Ls.macs / ms / 1e9, 2)
                issued_step += issued_share(Ls.kernels[o]) * 2.0 * Ls.macs
            detail["%s.%s" % (Ls.name, Ls.op_names[o])] = e
    OPS_dom = dom.op_names
    if op < 3 and dom.macs:
        ach = 2.0 * dom.macs / per[li, op] / 1e9
        peak = BF16_MFMA_PEAK_TFLOPS if "bf16" in dom.kernels[op] else FP32_MFMA_PEAK_TFLOPS
        # 'achieved' counts the flops of the sum as the paper writes it; 'issued' those the MFMAs of this kernel
        # execute for it (two thirds in the *_f23 kernels), which is what the matrix core's peak bounds
        share = issued_share(dom.kernels[op])
        roof = {"bound": "mfma", "achieved": round(ach, 2), "peak": peak, "unit": "TFLOP/s",
                "frac": round(ach / peak, 4), "issued": round(share * ach, 2), "frac_issued": round(share * ach / peak, 4),
                "traffic": measured_traffic("%s.%s" % (dom.name, OPS_dom[op])) if args.workload == "vgg3x3" and prec == B.MCN_PREC_FP32 else None,
                "kernel": "%s.%s (%s)" % (dom.name, OPS_dom[op], dom.kernels[op])}
    else:
        ach = dom.bytes[op] / per[li, op] / 1e6
        roof = {"bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(ach / HBM_PEAK_GBS, 4),
                "traffic": measured_traffic("%s.%s" % (dom.name, OPS_dom[op])) if args.workload == "vgg3x3" and prec == B.MCN_PREC_FP32 else None,
                "kernel": "%s.%s (%s)" % (dom.name, OPS_dom[op], dom.kernels[op])}

    out = {
        "metric": "conv fwd+bwd TFLOP/s (%s) on VGG-style 3x3 layers" % ("fp32" if prec == B.MCN_PREC_FP32 else "bf16 operands, fp32 accumulation"),
        "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if prec == B.MCN_PREC_FP32 else "bf16-in/f32-acc", "data": "synthetic",
        "config": {"workload": "conv fwd+bwd (dzdx, dzdw, dzdb) of layers " + ",".join(names) +
                               " (3x3 stride 1 pad 1, N=32)" if args.workload == "vgg3x3" else
                               "conv fwd+bwd of layers " + ",".join(names),
                   "layers": {Ls.name: Ls.shape_info() for Ls in layers}},
        "frac_of_fp32_mfma_peak": round(value / FP32_MFMA_PEAK_TFLOPS, 4) if prec == B.MCN_PREC_FP32 else None,
        "mfma_issued_TFLOPs": round(issued_step / (elapsed / args.steps) / 1e12, 3),
        "roofline": roof,
        "calls": detail,
    }
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
