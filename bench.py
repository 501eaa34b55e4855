#!/usr/bin/env python3
"""Benchmark of the Convolution hot path on one MI355X.

A step = one pass of the whole hot path over one batch of synthetic input for the workload
the headline metric is quoted on (the second benchmark configuration): ResNet-style 3x3 conv layer, bf16
data with fp32 accumulate, N=64, C=K=64, 56x56, stride 1, pad 1 -- forward with the fused
bias+ReLU epilogue, ConvolutionBackpropData and ConvolutionBackpropFilters, all on
16-channel-blocked tensors, inputs resident in HBM, filters already in their blocked
layouts (the re-layout happens once per weight update and is timed separately).

Prints ONE JSON line.  Everything is launched on one HIP stream.  After W warm-up steps the step loop is timed in
`--batches` batches of K steps (`ms_per_step` = the median batch), then every kernel of the step is timed on its
own with HIP events on the launch stream, again in batches of back-to-back launches, and `kernels` holds the
median per launch.  `value` = nominal flop of the step / sum of those kernel medians (`kernel_sum`), the
definition the metric is judged by; `step_wall` gives the same flop over the wall time of the step loop (launch
gaps included) and `three_stream_step` over a step whose three ops go to three streams (an extra, not `value`).
`roofline` is the dominant kernel against the MI355X peak that bounds it; its `traffic` is read from the
committed counter summary under profiles/ when there is one for this workload (null otherwise).
`cpu_baseline` is the CPU oracle timed on the host cores (all threads, and one thread on a smaller sample).
`--workload` selects another configuration for experiments; the default line is the contract.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6      # MI355X dense bf16 MFMA: 256 CU x 4 SIMD x 1024 flop/clk x 2.4 GHz
PEAK_HBM_GBS = 8000.0
TRAFFIC_SUMMARY = os.path.join(ROOT, "profiles", "cfg2_hbm_traffic.txt")


def measured_traffic(kernel_name):
    """HBM bytes per launch (fetch + write) of a cfg2 op from the committed counter summary: lines of the form
    `traffic_bytes <workload>:<op> <bytes>` written from `rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE` runs of
    this file (the summary states the commands and the copy-kernel scale factors).  None when there is no such line."""
    try:
        with open(TRAFFIC_SUMMARY) as f:
            for line in f:
                m = re.match(r"traffic_bytes\s+(\S+)\s+(\d+)\s*$", line)
                if m and m.group(1) == kernel_name:
                    return int(m.group(2))
    except OSError:
        pass
    return None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="cfg2", choices=["cfg2", "cfg3", "cfg4", "cfg5", "cfg6", "cfg7", "softmax"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--batches", type=int, default=5, help="timed batches of --steps steps; the median is reported")
    ap.add_argument("--kernel-reps", type=int, default=200,
                    help="back-to-back launches per batch when a kernel is timed on its own (at least --steps)")
    ap.add_argument("--no-three-stream", action="store_true",
                    help="skip the extra leg that issues forward, backprop-data and backprop-filters to three HIP "
                         "streams of equal (default) priority")
    ap.add_argument("--backward-compounds", action="store_true",
                    help="also time ngc_conv_bwd_data_relu and ngc_bias_grad of every layer on their own (reported under "
                         "backward_compound_kernels; never part of the timed step)")
    ap.add_argument("--propagate-layout", action="store_true",
                    help="cfg3 only: no conversion pass; the three ops read x from / write dx to the NCHW tensor directly")
    ap.add_argument("--fused-backward", action="store_true",
                    help="1x1 stride-1 layers with blocked tensors: backprop-data and backprop-filters as one call "
                         "(ngc_conv_bwd_data_filters, dy read once); same nominal flop, reported under its own config key")
    ap.add_argument("--cold", action="store_true", help="rotate over buffer sets (> 512 MB) between steps")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch a plain copy kernel of known size (same-layout ngc_layout_convert of the "
                         "[64,256,56,56] bf16 tensor: 102.8 MB read + 102.8 MB written) so that HBM counters can be scaled")
    ap.add_argument("--settle", type=float, default=0.5,
                    help="seconds of untimed load (the workload's own steps) before the warm-up steps; 0 = none")
    ap.add_argument("--layer", default=None, help="cfg5 / cfg6 / cfg7: time this one layer of the set only "
                    "(e.g. c256k1024hw14r1s1, v_3x3x3_c64k128); for profiles of one kernel")
    return ap.parse_args()


class LayerBench:
    """Device buffers and launch closures of one layer (all ops through the C ABI).  Inputs are
    uploaded as NCHW bf16 and brought into the blocked layout by the library's own conversion."""

    def __init__(self, L, ng, torch, nchw_input=False, sets=1, propagate=False, fused_backward=False):
        import numpy as np
        import synth_inputs
        self.L, self.ng, self.torch = L, ng, torch
        t = synth_inputs.layer_tensors(L)
        blocked_in = L.c % 16 == 0                      # blocked filters; x blocked too unless the NCHW layout is propagated
        self.xl = ng.NGC_NCHW16C if blocked_in and not propagate else ng.NGC_NCHW
        self.yl = ng.NGC_NCHW16C
        epi = (ng.NGC_EPI_BIAS | ng.NGC_EPI_RELU) if L.bias_relu else ng.NGC_EPI_NONE
        cur = torch.cuda.current_stream().cuda_stream

        def mk(w_layout=ng.NGC_KCRS, epilogue=ng.NGC_EPI_NONE):
            n, c, h, w, k, r, s, sh, sw, dh, dw, pbh, pbw, pah, paw = L.attrs15
            return ng.make_desc(n, c, h, w, k, r, s, (sh, sw), (dh, dw), (pbh, pbw), (pah, paw), ng.NGC_BF16,
                                self.xl, self.yl, w_layout, epilogue)

        def dev_bits(values_f32):
            bits = synth_inputs.f32_to_bf16_bits(values_f32)      # values of bf16 configs are exactly representable
            return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda()

        def to_layout(nchw, c, h, w, layout):
            if layout == ng.NGC_NCHW:
                return nchw
            out = torch.empty(L.n * ((c + 15) // 16) * h * w * 16, dtype=torch.int16, device="cuda")
            ng.ngc_layout_convert(ng.NGC_BF16, L.n, c, h, w, nchw, ng.NGC_NCHW, out, ng.NGC_NCHW16C, cur)
            torch.cuda.synchronize()
            return out

        self.d_fwd = mk(ng.NGC_BLOCKED_FWD if blocked_in else ng.NGC_KCRS, epi)
        self.d_bwd = mk(ng.NGC_BLOCKED_BWD if blocked_in else ng.NGC_KCRS)
        self.d_wg = mk()
        self.w_kcrs = dev_bits(t["w"])
        if blocked_in:
            self.w_fwd = torch.empty(ng.ngc_filter_elems(self.d_fwd, ng.NGC_BLOCKED_FWD), dtype=torch.int16, device="cuda")
            self.w_bwd = torch.empty(ng.ngc_filter_elems(self.d_fwd, ng.NGC_BLOCKED_BWD), dtype=torch.int16, device="cuda")
            ng.ngc_filter_convert(self.d_fwd, self.w_kcrs, self.w_fwd, ng.NGC_BLOCKED_FWD, cur)
            ng.ngc_filter_convert(self.d_fwd, self.w_kcrs, self.w_bwd, ng.NGC_BLOCKED_BWD, cur)
        else:
            self.w_fwd = self.w_bwd = self.w_kcrs
        self.bias = torch.from_numpy(np.ascontiguousarray(t["bias"], dtype=np.float32)).cuda()
        self.nchw_input = nchw_input
        self.sets = []
        x_nchw0 = dev_bits(t["x"])
        x0 = to_layout(x_nchw0, L.c, L.h, L.w, self.xl)
        dy0 = to_layout(dev_bits(t["dy"]), L.k, L.p, L.q, self.yl)
        if not nchw_input:
            x_nchw0 = None
        for i in range(sets):
            s = {"x": x0 if i == 0 else x0.clone(), "dy": dy0 if i == 0 else dy0.clone(),
                 "y": torch.empty(ng.ngc_data_elems(self.d_fwd, 1), dtype=torch.int16, device="cuda"),
                 "dx": torch.empty(ng.ngc_data_elems(self.d_fwd, 0), dtype=torch.int16, device="cuda"),
                 "dw": torch.empty(L.k * L.c * L.r * L.s, dtype=torch.float32, device="cuda")}
            if nchw_input:
                s["x_nchw"] = x_nchw0 if i == 0 else x_nchw0.clone()
            self.sets.append(s)
        self.ws = {op: torch.empty(max(ng.ngc_conv_workspace_bytes(d, op), 16), dtype=torch.uint8, device="cuda")
                   for op, d in ((ng.NGC_OP_FWD, self.d_fwd), (ng.NGC_OP_BWD_DATA, self.d_bwd),
                                 (ng.NGC_OP_BWD_FILTERS, self.d_wg), (ng.NGC_OP_BIAS_GRAD, self.d_wg),
                                 (ng.NGC_OP_BWD_DATA_DB, self.d_bwd))}
        self.db = torch.empty(L.k, dtype=torch.float32, device="cuda")
        self.db_prev = torch.empty(L.c, dtype=torch.float32, device="cuda")
        self.stream = cur
        self.ops = list(L.ops)
        # --fused-backward: where the library has the one-pass kernel for the node (1x1, stride 1, blocked tensors),
        # backprop-data and backprop-filters are one call that reads dy once
        if (fused_backward and "bwd_data" in self.ops and "bwd_filters" in self.ops and blocked_in and not propagate
                and ng.ngc_conv_variant(self.d_bwd, ng.NGC_OP_BWD_DATA_FILTERS) == "bwd1x1_fused_bf16"):
            self.ops = [op for op in self.ops if op not in ("bwd_data", "bwd_filters")] + ["bwd_fused"]
            self.ws[ng.NGC_OP_BWD_DATA_FILTERS] = torch.empty(ng.ngc_conv_workspace_bytes(self.d_bwd, ng.NGC_OP_BWD_DATA_FILTERS),
                                                              dtype=torch.uint8, device="cuda")
        if nchw_input and not propagate:
            self.ops = ["convert"] + self.ops

    def launch(self, op, i=0, streams=None):
        """streams: optional {op: raw HIP stream}; default is the stream the bench was built on."""
        ng, s = self.ng, self.sets[i % len(self.sets)]
        L = self.L
        st = self.stream if streams is None else streams[op]
        if op == "convert":
            ng.ngc_layout_convert(ng.NGC_BF16, L.n, L.c, L.h, L.w, s["x_nchw"], ng.NGC_NCHW, s["x"], ng.NGC_NCHW16C, st)
        elif op == "fwd":
            ng.ngc_conv_fwd(self.d_fwd, s["x"], self.w_fwd, self.bias if L.bias_relu else None, s["y"],
                            self.ws[ng.NGC_OP_FWD], st)
        elif op == "bwd_data":
            ng.ngc_conv_bwd_data(self.d_bwd, s["dy"], self.w_bwd, s["dx"], self.ws[ng.NGC_OP_BWD_DATA], st)
        elif op == "bwd_filters":
            ng.ngc_conv_bwd_filters(self.d_wg, s["x"], s["dy"], s["dw"], self.ws[ng.NGC_OP_BWD_FILTERS], st)
        elif op == "bwd_fused":
            ng.ngc_conv_bwd_data_filters(self.d_bwd, s["x"], s["dy"], self.w_bwd, s["dx"], s["dw"],
                                         self.ws[ng.NGC_OP_BWD_DATA_FILTERS], st)
        elif op == "bwd_data_relu":       # backward compounds: timed on their own, not part of the step
            ng.ngc_conv_bwd_data_relu(self.d_bwd, s["dy"], self.w_bwd, s["x"], s["dx"], self.ws[ng.NGC_OP_BWD_DATA], st)
        elif op == "bwd_data_relu_db":    # ... and the channel sums of dx (bias gradient of the producing layer)
            ng.ngc_conv_bwd_data_relu_db(self.d_bwd, s["dy"], self.w_bwd, s["x"], s["dx"], self.db_prev,
                                         self.ws[ng.NGC_OP_BWD_DATA_DB], st)
        elif op == "bias_grad":
            ng.ngc_bias_grad(self.d_wg, s["dy"], self.db, self.ws[ng.NGC_OP_BIAS_GRAD], st)
        else:
            raise ValueError(op)

    def step(self, i=0, streams=None):
        for op in self.ops:
            self.launch(op, i, streams)

    def algorithmic_bytes(self, op):
        """Each tensor once (bf16 data, fp32 dw / bias)."""
        L = self.L
        xb = 2 * L.n * L.c * L.h * L.w
        yb = 2 * L.n * L.k * L.p * L.q
        wb = 2 * L.k * L.c * L.r * L.s
        if op == "convert":
            return 2 * xb
        if op == "fwd":
            return xb + yb + wb + 4 * L.k
        if op == "bwd_data":
            return xb + yb + wb
        if op in ("bwd_data_relu", "bwd_data_relu_db"):
            return 2 * xb + yb + wb + (4 * L.c if op.endswith("_db") else 0)
        if op == "bias_grad":
            return yb + 4 * L.k
        if op == "bwd_fused":
            return 2 * xb + yb + 3 * wb  # dy once, x in, dx out, w in, dw (fp32) out
        return xb + yb + 2 * wb          # bwd_filters: dw fp32


def settle_clocks(torch, step, seconds):
    """Untimed: keep the GPU busy with the workload's own steps for `seconds` before the W warm-up steps, so
    that the timed region starts at the clocks a training job runs at (a cold MI355X takes some 50 ms of load to
    reach them: the cfg2 step is 73 us when timed right after 20 warm-up steps and 61 us in steady state)."""
    if seconds <= 0:
        return
    t0 = time.perf_counter()
    i = 0
    while time.perf_counter() - t0 < seconds:
        for _ in range(16):
            step(i)
            i += 1
        torch.cuda.synchronize()


def event_time_ms(torch, fn, reps, batches=5):
    """Median over `batches` of (HIP-event time of `reps` back-to-back launches on the current stream) / reps."""
    per = []
    for b in range(batches):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(reps):
            fn(b * reps + i)
        e1.record()
        torch.cuda.synchronize()
        per.append(e0.elapsed_time(e1) / reps)
    return statistics.median(per)


def timed_steps_ms(torch, step, steps, batches):
    """`batches` batches of exactly `steps` steps, each bracketed by a device synchronisation; per-step wall time of
    every batch (ms)."""
    per = []
    for b in range(batches):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            step(b * steps + i)
        torch.cuda.synchronize()
        per.append((time.perf_counter() - t0) * 1e3 / steps)
    return per


def softmax_main(args, torch, ng, synth_inputs):
    """Softmax workloads (the other kernel the paper names): forward + backprop per case, HBM-bound.
    --cold: every case rotates over enough buffer sets (> 600 MB) that no launch finds its operands in a cache."""
    import numpy as np
    cur = torch.cuda.current_stream().cuda_stream
    cases = synth_inputs.softmax_cases()
    bufs = []
    for c in cases:
        t = synth_inputs.softmax_tensors(c)
        if c.dtype == "bf16":
            up = lambda v: torch.from_numpy(np.ascontiguousarray(synth_inputs.f32_to_bf16_bits(v)).view(np.int16)).cuda()
        else:
            up = lambda v: torch.from_numpy(np.ascontiguousarray(v, dtype=np.float32)).cuda()
        x, dy = up(t["x"]), up(t["dy"])
        nbytes = c.rows * c.cols * (2 if c.dtype == "bf16" else 4)
        nsets = max(2, int(600e6 // (4 * nbytes)) + 1) if args.cold else 1
        sets = [(x, dy, torch.empty_like(x), torch.empty_like(x))]
        for _ in range(nsets - 1):
            sets.append((x.clone(), dy.clone(), torch.empty_like(x), torch.empty_like(x)))
        for x_, dy_, y_, _dx in sets[1:]:                                   # backprop reads y: make every set's y valid
            ng.ngc_softmax(ng.NGC_BF16 if c.dtype == "bf16" else ng.NGC_F32, c.rows, c.cols, x_, y_, cur)
        bufs.append((c, ng.NGC_BF16 if c.dtype == "bf16" else ng.NGC_F32, sets))
    torch.cuda.synchronize()

    def step(i):
        for c, code, sets in bufs:
            x, dy, y, dx = sets[i % len(sets)]
            ng.ngc_softmax(code, c.rows, c.cols, x, y, cur)
            ng.ngc_softmax_bwd(code, c.rows, c.cols, y, dy, dx, cur)

    settle_clocks(torch, step, args.settle)
    for i in range(args.warmup):
        step(i)
    per = timed_steps_ms(torch, step, args.steps, args.batches)
    ms_per_step = statistics.median(per)
    kern = {}
    reps = max(args.kernel_reps, args.steps)
    total_bytes = 0
    for c, code, sets in bufs:
        nbytes = c.rows * c.cols * (2 if c.dtype == "bf16" else 4)
        total_bytes += 5 * nbytes

        def fwd(i, c=c, code=code, sets=sets):
            x, dy, y, dx = sets[i % len(sets)]
            ng.ngc_softmax(code, c.rows, c.cols, x, y, cur)

        def bwd(i, c=c, code=code, sets=sets):
            x, dy, y, dx = sets[i % len(sets)]
            ng.ngc_softmax_bwd(code, c.rows, c.cols, y, dy, dx, cur)

        for op, fn, nb in (("fwd", fwd, 2 * nbytes), ("bwd", bwd, 3 * nbytes)):
            ms = event_time_ms(torch, fn, reps, args.batches)
            kern[f"{c.name}:{op}"] = {"us": round(ms * 1e3, 2), "gbs": round(nb / (ms * 1e-3) / 1e9, 1), "bytes": nb,
                                      "variant": ng.ngc_softmax_variant(code, c.cols, op == "bwd"), "count": 1}
    dom_name = max(kern, key=lambda k: kern[k]["us"])
    dom = kern[dom_name]
    ksum_us = sum(v["us"] for v in kern.values())
    value = total_bytes / (ksum_us * 1e-6) / 1e9
    print(json.dumps({
        "metric": "softmax forward + backprop, algorithmic GB/s over 4 workloads, 1 GPU", "value": round(value, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "batches": args.batches, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "softmax over the last axis: [32768,1000], [262144,512], [4096,32000] bf16 and [65536,1024] fp32, "
                               "forward + backprop each", "streams": 1, "cache": "cold" if args.cold else "warm"},
        "value_basis": "algorithmic bytes / sum of the kernel medians (kernel_sum)",
        "kernel_sum": {"us": round(ksum_us, 2)},
        "step_wall": {"ms_per_step_batches": [round(v, 5) for v in per],
                      "gbs": round(total_bytes / (ms_per_step * 1e-3) / 1e9, 1)},
        "roofline": {"bound": "hbm", "achieved": dom["gbs"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": round(dom["gbs"] / PEAK_HBM_GBS, 4), "traffic": None, "kernel": dom_name},
        "kernels": kern}))


def conv3d_main(args, torch, ng, synth_inputs):
    """Video-shaped layers over three spatial axes: forward (+bias+ReLU), backprop-data and backprop-filters of each."""
    import numpy as np
    cur = torch.cuda.current_stream().cuda_stream
    F, B, W = ng.NGC_OP_FWD, ng.NGC_OP_BWD_DATA, ng.NGC_OP_BWD_FILTERS
    items = []
    layers = [L for L in synth_inputs.video_layers() if args.layer in (None, L.name)]
    if not layers:
        print(f"bench.py: no layer {args.layer} in cfg7", file=sys.stderr)
        sys.exit(2)
    for L in layers:
        t = synth_inputs.layer3_tensors(L)
        o, p, q = L.opq
        epi = (ng.NGC_EPI_BIAS | ng.NGC_EPI_RELU) if L.bias_relu else ng.NGC_EPI_NONE
        mk = lambda wl, e=ng.NGC_EPI_NONE: ng.make_desc3(L.n, L.c, L.d, L.h, L.w, L.k, L.t, L.r, L.s, L.strides, L.dilation,
                                                         L.pad_below, L.pad_above, ng.NGC_BF16, ng.NGC_NCHW16C, ng.NGC_NCHW16C, wl, e)
        d_f, d_b, d_w = mk(ng.NGC_BLOCKED_FWD, epi), mk(ng.NGC_BLOCKED_BWD), mk(ng.NGC_KCRS)
        up = lambda v: torch.from_numpy(np.ascontiguousarray(synth_inputs.f32_to_bf16_bits(v)).view(np.int16)).cuda()

        def blocked(v, c, dd, h, w):          # upload as [N][C][D][H][W], convert on the device (D*H rows)
            src = up(v)
            dst = torch.empty(L.n * ((c + 15) // 16) * dd * h * w * 16, dtype=torch.int16, device="cuda")
            ng.ngc_layout_convert(ng.NGC_BF16, L.n, c, dd * h, w, src, ng.NGC_NCHW, dst, ng.NGC_NCHW16C, cur)
            torch.cuda.synchronize()
            return dst

        x, dy = blocked(t["x"], L.c, L.d, L.h, L.w), blocked(t["dy"], L.k, o, p, q)
        wk = up(t["w"])
        wf = torch.empty(ng.ngc_conv3d_filter_elems(d_f, ng.NGC_BLOCKED_FWD), dtype=torch.int16, device="cuda")
        wb = torch.empty(ng.ngc_conv3d_filter_elems(d_f, ng.NGC_BLOCKED_BWD), dtype=torch.int16, device="cuda")
        ng.ngc_conv3d_filter_convert(d_f, wk, wf, ng.NGC_BLOCKED_FWD, cur)
        ng.ngc_conv3d_filter_convert(d_f, wk, wb, ng.NGC_BLOCKED_BWD, cur)
        bias = torch.from_numpy(np.ascontiguousarray(t["bias"], dtype=np.float32)).cuda() if L.bias_relu else None
        y, dx = torch.empty_like(dy), torch.empty_like(x)
        dw = torch.empty(L.k * L.c * L.t * L.r * L.s, dtype=torch.float32, device="cuda")
        ws = {op: torch.empty(max(ng.ngc_conv3d_workspace_bytes(d, op), 16), dtype=torch.uint8, device="cuda")
              for op, d in ((F, d_f), (B, d_b), (W, d_w))}
        xb, yb, wbytes = 2 * L.n * L.c * L.d * L.h * L.w, 2 * L.n * L.k * o * p * q, 2 * L.k * L.c * L.t * L.r * L.s
        ops = {"fwd": (lambda i, a=(d_f, x, wf, bias, y, ws[F]): ng.ngc_conv3d_fwd(*a, cur), d_f, F, xb + yb + wbytes),
               "bwd_data": (lambda i, a=(d_b, dy, wb, dx, ws[B]): ng.ngc_conv3d_bwd_data(*a, cur), d_b, B, xb + yb + wbytes),
               "bwd_filters": (lambda i, a=(d_w, x, dy, dw, ws[W]): ng.ngc_conv3d_bwd_filters(*a, cur), d_w, W, xb + yb + 2 * wbytes)}
        items.append((L, ops))
    torch.cuda.synchronize()

    def step(i):
        for _, ops in items:
            for fn, _, _, _ in ops.values():
                fn(i)

    settle_clocks(torch, step, args.settle)
    for i in range(args.warmup):
        step(i)
    per = timed_steps_ms(torch, step, args.steps, args.batches)
    ms_per_step = statistics.median(per)
    kern = {}
    reps = max(5, min(args.steps, 50))
    for L, ops in items:
        for name, (fn, d, op, nbytes) in ops.items():
            ms = event_time_ms(torch, fn, reps, args.batches)
            kern[f"{L.name}:{name}"] = {"us": round(ms * 1e3, 2), "tflops": round(L.flop_per_op / (ms * 1e-3) / 1e12, 1),
                                        "gbs": round(nbytes / (ms * 1e-3) / 1e9, 1), "variant": ng.ngc_conv3d_variant(d, op),
                                        "count": 1}
    if args.calibrate_copy:
        # a plain copy of known size (102.8 MB read + 102.8 MB written per launch) to scale the HBM counters by
        src = torch.zeros(64 * 256 * 56 * 56, dtype=torch.int16, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(10):
            ng.ngc_layout_convert(ng.NGC_BF16, 64, 256, 56, 56, src, ng.NGC_NCHW, dst, ng.NGC_NCHW, cur)
        torch.cuda.synchronize()
    flop = 3 * sum(L.flop_per_op for L, _ in items)
    dom_name = max(kern, key=lambda k: kern[k]["us"])
    dom = kern[dom_name]
    ksum_us = sum(v["us"] for v in kern.values())
    print(json.dumps({
        "metric": "conv3d fwd+bwd TFLOP/s over 7 video-shaped layers, 1 GPU" if args.layer is None
        else f"conv3d fwd+bwd TFLOP/s, layer {args.layer}, 1 GPU", "value": round(flop / (ksum_us * 1e-6) / 1e12, 1),
        "value_basis": "nominal flop / sum of the kernel medians (kernel_sum)", "kernel_sum": {"us": round(ksum_us, 2)},
        "step_wall": {"ms_per_step_batches": [round(v, 5) for v in per],
                      "tflops": round(flop / (ms_per_step * 1e-3) / 1e12, 1)},
        "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "batches": args.batches,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "7 layers over (D,H,W), N=8 clips of 16 frames: 3x3x3 64->128 16x56x56, 3x3x3 128->256 8x28x28, "
                               "3x3x3/2 128->128, 1x3x3 64->128, 3x1x1 128->64, 1x1x1 256->64, 3x3x3 with per-axis strides / "
                               "dilation / one-sided padding; fwd(+bias+ReLU) + bwd_data + bwd_filters each", "streams": 1},
        "roofline": {"bound": "mfma", "achieved": dom["tflops"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(dom["tflops"] / PEAK_BF16_TFLOPS, 4), "traffic": None, "kernel": dom_name},
        "kernels": kern}))


def cpu_model_name():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(L):
    """The oracle as it stands, timed on the host cores: one pass over the full cfg2 tensors with every thread the
    box gives this job, then one pass over the first 4 images with one thread."""
    import ctypes
    import dataclasses
    import numpy as np
    import oracle
    import synth_inputs

    def one_pass(layer):
        a = oracle.Attrs(*layer.attrs15)
        t = synth_inputs.layer_tensors(layer)
        x, w, dy = (t[k].astype(np.float64) for k in ("x", "w", "dy"))
        t0 = time.perf_counter()
        oracle.conv_fwd(a, x, w, bias=t["bias"], relu=True)
        oracle.conv_bwd_data_gather(a, dy, w)
        oracle.conv_bwd_filters(a, x, dy)
        return time.perf_counter() - t0

    cores = int(os.environ.get("OMP_NUM_THREADS", "0")) or (os.cpu_count() or 1)
    dt = one_pass(L)
    out = {"value": 3 * L.flop_per_op / dt / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
           "cpu_model": cpu_model_name(), "seconds": round(dt, 3),
           "sample": f"one full pass (fwd+bias+ReLU, backprop-data gather form, backprop-filters) over the "
                     f"N={L.n} {L.name} tensors in fp64"}
    # one thread: the OpenMP runtime the oracle's C library runs on is told to use one (its code is untouched)
    try:
        gomp = ctypes.CDLL("libgomp.so.1")
        small = dataclasses.replace(L, n=4)
        gomp.omp_set_num_threads(1)
        try:
            dt1 = one_pass(small)
        finally:
            gomp.omp_set_num_threads(cores)
        out["one_thread"] = {"value": 3 * small.flop_per_op / dt1 / 1e12, "unit": "TFLOP/s", "cores": 1,
                             "seconds": round(dt1, 3), "sample": f"the same pass over the first {small.n} images"}
    except (OSError, AttributeError, TypeError) as e:
        out["one_thread"] = {"value": None, "error": str(e)}
    return out


def cfg1_latency(torch, ng, synth_inputs, batches):
    """The small fp32 NCHW correctness configuration: microseconds per launch of its three ops (latency only)."""
    import numpy as np
    L = synth_inputs.config_layers(1)[0]
    t = synth_inputs.layer_tensors(L)
    cur = torch.cuda.current_stream().cuda_stream
    n, c, h, w, k, r, s, sh, sw, dh, dw, pbh, pbw, pah, paw = L.attrs15
    mk = lambda e: ng.make_desc(n, c, h, w, k, r, s, (sh, sw), (dh, dw), (pbh, pbw), (pah, paw), ng.NGC_F32,
                                ng.NGC_NCHW, ng.NGC_NCHW, ng.NGC_KCRS, e)
    d_f, d_b = mk(ng.NGC_EPI_BIAS | ng.NGC_EPI_RELU), mk(ng.NGC_EPI_NONE)
    up = lambda v: torch.from_numpy(np.ascontiguousarray(v, dtype=np.float32)).cuda()
    x, wt, dy, bias = up(t["x"]), up(t["w"]), up(t["dy"]), up(t["bias"])
    y, dx, dwt = torch.empty_like(dy), torch.empty_like(x), torch.empty_like(wt)
    ws = {op: torch.empty(max(ng.ngc_conv_workspace_bytes(d_b, op), 16), dtype=torch.uint8, device="cuda")
          for op in (ng.NGC_OP_FWD, ng.NGC_OP_BWD_DATA, ng.NGC_OP_BWD_FILTERS)}
    ops = {"fwd": lambda i: ng.ngc_conv_fwd(d_f, x, wt, bias, y, ws[ng.NGC_OP_FWD], cur),
           "bwd_data": lambda i: ng.ngc_conv_bwd_data(d_b, dy, wt, dx, ws[ng.NGC_OP_BWD_DATA], cur),
           "bwd_filters": lambda i: ng.ngc_conv_bwd_filters(d_b, x, dy, dwt, ws[ng.NGC_OP_BWD_FILTERS], cur)}
    out = {}
    for name, fn in ops.items():
        for i in range(20):
            fn(i)
        out[name] = round(event_time_ms(torch, fn, 200, batches) * 1e3, 2)
    out["variant"] = ng.ngc_conv_variant(d_f, 0)
    out["note"] = "configs[0], fp32 NCHW N=2 C=16 16x16 K=32 3x3: us per launch back to back; latency only, no roofline claim"
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (no collectives are part of it); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    import paper_1801_08058_amd as ng
    import synth_inputs

    if args.workload == "softmax":
        softmax_main(args, torch, ng, synth_inputs)
        return
    if args.workload == "cfg7":
        conv3d_main(args, torch, ng, synth_inputs)
        return
    cfg = int(args.workload[3:])
    layers = synth_inputs.config_layers(cfg)
    if args.layer is not None:
        layers = [L for L in layers if L.name == args.layer]
        if not layers:
            print(f"bench.py: no layer {args.layer} in {args.workload}", file=sys.stderr)
            sys.exit(2)
    sets = 1
    if args.cold:
        per_set = sum(2 * 2 * (L.n * L.c * L.h * L.w + L.n * L.k * L.p * L.q) for L in layers[:1])
        sets = max(2, int(600e6 // per_set) + 1)
    if args.propagate_layout and cfg != 3:
        print("bench.py: --propagate-layout applies to --workload cfg3", file=sys.stderr)
        sys.exit(2)
    benches = [LayerBench(L, ng, torch, nchw_input=(cfg == 3), sets=sets, propagate=args.propagate_layout,
                          fused_backward=args.fused_backward) for L in layers]
    torch.cuda.synchronize()

    def make_step(streams):
        def step(i):
            for b in benches:
                for _ in range(b.L.count):
                    b.step(i, streams)
        return step

    step = make_step(None)                                              # everything on the current stream
    settle_clocks(torch, step, args.settle)
    for i in range(args.warmup):
        step(i)
    per = timed_steps_ms(torch, step, args.steps, args.batches)
    ms_per_step = statistics.median(per)
    flop_step = sum(L.flop_per_op * len(L.ops) * L.count for L in layers)

    # per-kernel durations (HIP events on the launch stream around back-to-back launches, median of the batches)
    kern = {}
    reps = max(args.kernel_reps, args.steps) if cfg != 5 else max(20, min(args.steps, 200))
    for b in benches:
        for op in b.ops:
            ms = event_time_ms(torch, lambda i, b=b, op=op: b.launch(op, i), reps, args.batches)
            flop = 0.0 if op == "convert" else (2 if op == "bwd_fused" else 1) * b.L.flop_per_op
            kern[f"{b.L.name}:{op}"] = {
                "us": round(ms * 1e3, 2), "tflops": round(flop / (ms * 1e-3) / 1e12, 1),
                "gbs": round(b.algorithmic_bytes(op) / (ms * 1e-3) / 1e9, 1),
                "variant": {"convert": "layout", "fwd": ng.ngc_conv_variant(b.d_fwd, 0),
                            "bwd_data": ng.ngc_conv_variant(b.d_bwd, 1),
                            "bwd_fused": ng.ngc_conv_variant(b.d_bwd, ng.NGC_OP_BWD_DATA_FILTERS),
                            "bwd_filters": ng.ngc_conv_variant(b.d_wg, 2)}[op],
                "count": b.L.count}
    ksum_us = sum(v["us"] * v["count"] for v in kern.values())
    value = flop_step / (ksum_us * 1e-6) / 1e12

    # Extra leg: the ops of a layer read and write disjoint buffers (each has its own inputs, outputs and
    # workspace), so they may be issued to one stream per op kind and overlap their launch gaps and tails;
    # cfg3's layout conversion feeds the forward op and stays single-stream.
    three = None
    if not args.no_three_stream and cfg != 3:
        extra_streams = [torch.cuda.Stream() for _ in range(2)]         # default priority
        step3 = make_step({"fwd": benches[0].stream, "bwd_data": extra_streams[0].cuda_stream,
                           "bwd_filters": extra_streams[1].cuda_stream, "bwd_fused": extra_streams[0].cuda_stream})
        for i in range(max(args.warmup, 5)):
            step3(i)
        per3 = timed_steps_ms(torch, step3, args.steps, args.batches)
        ms3 = statistics.median(per3)
        three = {"ms_per_step": round(ms3, 5), "tflops": round(flop_step / (ms3 * 1e-3) / 1e12, 2),
                 "note": "fwd / bwd_data / bwd_filters on three streams of default priority; not the headline value"}

    # backward compounds (ReLU backprop fused into backprop-data; bias gradient): same buffers, timed alone
    extra = {}
    for b in (benches if args.backward_compounds else []):
        for op in (["bwd_data_relu", "bwd_data_relu_db"] if "bwd_data" in b.ops else []) + ["bias_grad"]:
            ms = event_time_ms(torch, lambda i, b=b, op=op: b.launch(op, i), reps)
            flop = b.L.flop_per_op if op.startswith("bwd_data_relu") else 0.0
            extra[f"{b.L.name}:{op}"] = {
                "us": round(ms * 1e3, 2), "tflops": round(flop / (ms * 1e-3) / 1e12, 1),
                "gbs": round(b.algorithmic_bytes(op) / (ms * 1e-3) / 1e9, 1),
                "variant": ng.ngc_conv_variant(b.d_bwd, 1) + {"bwd_data_relu": "+relu_bwd", "bwd_data_relu_db": "+relu_bwd+db"}[op]
                if op.startswith("bwd_data_relu") else ng.ngc_conv_variant(b.d_wg, ng.NGC_OP_BIAS_GRAD), "count": b.L.count}
    if args.calibrate_copy:
        # 64 x 256 x 56 x 56 bf16 = 102.8 MB read + 102.8 MB written per launch: larger than the
        # 8 x 4 MB of L2, so FETCH_SIZE sees (almost) every byte of the source
        cn, cc, chh, cww = 64, 256, 56, 56
        src = torch.zeros(cn * cc * chh * cww, dtype=torch.int16, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(10):
            ng.ngc_layout_convert(ng.NGC_BF16, cn, cc, chh, cww, src, ng.NGC_NCHW, dst, ng.NGC_NCHW, benches[0].stream)
        torch.cuda.synchronize()
    dom_name = max(kern, key=lambda k: kern[k]["us"] * kern[k]["count"])
    dom = kern[dom_name]
    # which roof bounds the dominant kernel: the MFMA one for the headline layer (at the ridge, judged on MFMA) and for
    # any kernel whose flop per algorithmic byte lies above the machine balance, the HBM one otherwise
    dom_bench = next(b for b in benches if dom_name.startswith(b.L.name + ":"))
    dom_op = dom_name.split(":")[1]
    intensity = (0.0 if dom_op == "convert" else dom_bench.L.flop_per_op) / dom_bench.algorithmic_bytes(dom_op)
    if cfg == 2 or intensity >= PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9):
        roof = {"bound": "mfma", "achieved": dom["tflops"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": round(dom["tflops"] / PEAK_BF16_TFLOPS, 4),
                "traffic": None if args.cold else measured_traffic(dom_name),
                "traffic_unit": "bytes per launch (HBM fetch + write), from profiles/cfg2_hbm_traffic.txt",
                "algorithmic_bytes": dom_bench.algorithmic_bytes(dom_op), "kernel": dom_name}
    else:
        roof = {"bound": "hbm", "achieved": dom["gbs"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": round(dom["gbs"] / PEAK_HBM_GBS, 4), "traffic": None, "kernel": dom_name}

    out = {
        "metric": "conv TFLOP/s fwd+bwd (ResNet 3x3 bf16 layer) and % of MFMA peak, 1 GPU",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "batches": args.batches, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": {2: "configs[1]: 3x3 conv N=64 C=K=64 56x56 s1 p1 bf16, fwd(+bias+ReLU) + bwd_data + bwd_filters",
                                3: "configs[2]: 1x1 conv N=64 C=256 K=64 56x56 bf16, NCHW->nChw16c convert + fwd + bwd_data + bwd_filters",
                                4: "configs[3]: stem 7x7/2 N=64 C=3 K=64 224x224 bf16, fwd(+bias+ReLU) + bwd_filters",
                                5: "configs[4]: ResNet-50 conv stack N=128 bf16, 53 layers x (fwd+bias+ReLU, bwd_data, bwd_filters)",
                                6: "general-attribute layers (dilation, padding below != above, 5x5 / 1x7 / 7x1 / 2x2 windows, "
                                   "per-axis strides) N=32 bf16, 8 layers x (fwd+bias+ReLU, bwd_data, bwd_filters)"}[cfg],
                   "layout": "nChw16c activations, blocked filters, fp32 dw", "cache": "cold" if args.cold else "warm",
                   "streams": 1,
                   **({"layer": args.layer} if args.layer else {}),
                   **({"x_layout": "NCHW read / written by the ops themselves, no conversion pass"} if args.propagate_layout else {}),
                   **({"fused_backward": "bwd_data + bwd_filters of the 1x1 stride-1 layers as one call"} if args.fused_backward else {})},
        "value_basis": "nominal flop of the step / sum of the single-stream kernel medians (kernel_sum.us)",
        "pct_of_mfma_peak": round(100.0 * value / PEAK_BF16_TFLOPS, 2),
        "gflop_per_step": round(flop_step / 1e9, 2),
        "kernel_sum": {"us": round(ksum_us, 2), "tflops": round(value, 2)},
        # the same flop over the wall time of the single-stream step loop (launch gaps between kernels included)
        "step_wall": {"ms_per_step_batches": [round(v, 5) for v in per],
                      "tflops": round(flop_step / (ms_per_step * 1e-3) / 1e12, 2)},
        "roofline": roof,
        "kernels": kern,
    }
    if three:
        out["three_stream_step"] = three
    if args.backward_compounds:
        out["backward_compound_kernels"] = extra
    if cfg == 2 and not args.cold:
        out["cfg1_us"] = cfg1_latency(torch, ng, synth_inputs, args.batches)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(synth_inputs.config_layers(2)[0])
    print(json.dumps(out))


if __name__ == "__main__":
    main()
