#!/usr/bin/env python3
"""Benchmark of the glowmi hot path on one MI355X.

A step is one pass of the whole hot path -- contraction + bias + Relu (+ requantize), one fused
kernel per layer -- over every layer of a workload, inputs resident in HBM.

The default run times EVERY baseline configuration: the headline (`value`, `ms_per_step`, `roofline`,
`cpu_baseline`, `layers`) is the largest single-GPU one, the VGG-19-shaped fp32 stack at batch 16 plus
its FC layers; the ResNet-50 fp32 set (batch 1 and 32), the ResNet-50 int8 set (batch 32) and the FC
sweep in fp32 and int8 follow under the extra key `workloads`, each with the same block.  Every
workload is timed with the same --steps / --warmup.

Prints ONE JSON line.  Per layer: eager time per launch (events on the launch stream), TFLOP/s or
TOP/s, GB/s of algorithmic bytes, fraction of the layer's MFMA/HBM roofline, and
  * `llc`: "warm" when the layer reruns on the same buffers and those fit the 256 MB last-level cache
    (its HBM figure is then a cache figure), "cold" when the tensors exceed it; for every HBM-bound
    layer `us_cold` is the time per launch when the launches rotate over copies of the tensors that
    together exceed 512 MB, so that every launch streams from HBM;
  * `us_graph`: for layers under 16 us, the time per launch of 100 back-to-back launches replayed as
    one HIP graph (launch-amortised figure).
The top-level key `launch_floor_us` times the library's smallest kernel (16 elements of
glowmi_dequantize, one workgroup) the same ways -- per launch between events, back to back, and as 100
launches in one graph: what any single launch costs on this machine whatever it computes, so that the gap
of a microsecond-scale layer to its roofline can be attributed.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--only] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import copy
import json
import re
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X published peaks (dense)
PEAK_FP32_MFMA = 157.3e12      # FLOP/s, fp32 matrix
PEAK_INT8_MFMA = 5.0e15        # OP/s
PEAK_F16_MFMA = 2.5e15         # FLOP/s, fp16 and bf16 matrix (the large fp32 kernels multiply fp16 or bf16 pieces)
F16_PRODUCTS = 3               # fp16 piece products per fp32 multiply-add (two pieces per operand)
BF16_PRODUCTS = 6              # bf16 piece products per fp32 multiply-add (three pieces per operand)


def _mfma_peak(dtype, variant=""):
    """(published peak of the matrix-core dtype the kernel multiplies in, matrix-core products per algorithmic
    multiply-add).  The large fp32 kernels run on the fp16 cores with three piece products per fp32 product, the
    pointwise and first-layer ones on the bf16 cores with six."""
    if dtype != "f32":
        return PEAK_INT8_MFMA, 1
    if "igemm_f32_p3" in variant or "f16x3" in variant:
        return PEAK_F16_MFMA, F16_PRODUCTS
    if "bf16x6" in variant:
        return PEAK_F16_MFMA, BF16_PRODUCTS
    return PEAK_FP32_MFMA, 1
PEAK_HBM = 8.0e12              # B/s
LLC_BYTES = 256 << 20          # last-level (Infinity) cache
COLD_ROTATION_BYTES = 512 << 20
GRAPH_LAUNCHES = 100
SMALL_LAYER_US = 16.0

WORKLOADS = ["vgg19_fp32", "resnet50_fp32", "resnet50_int8", "fc_sweep_fp32", "fc_sweep_int8",
             "resnet50_tail_fp32", "resnet50_tail_int8", "resnet50_block_fp32", "resnet50_block_int8",
             "depthwise_fp32", "depthwise_int8"]
HEADLINE = "vgg19_fp32"        # largest single-GPU baseline configuration
ALSO = ["resnet50_fp32", "resnet50_int8", "fc_sweep_fp32", "fc_sweep_int8"]   # the other baseline configurations
CHAINED = {"resnet50_block_fp32", "resnet50_block_int8"}   # layers feed each other: run as one sequence


def _kernel_of(variant):
    """The kernel a variant name stands for: the 3x3 kernel whose pixel tile is shaped per layer reports the shape
    (conv_k3_f32_f16x3_14x16, .._8x28: one kernel, launched with different tile extents)."""
    return re.sub(r"^(conv_k3_f32_f16x3)_\d+x\d+((?:_add)?)$", r"\1\2", variant)


def _build_workload(name):
    from paper_1805_00907_amd import workloads as wl
    if name == "resnet50_fp32":     # config 2 of the baseline: batch 1 and batch 32
        return "f32", 1, wl.resnet50_layers(1) + wl.resnet50_layers(32)
    if name == "vgg19_fp32":        # config 3
        return "f32", 2, wl.vgg19_conv_layers(16) + wl.vgg19_fc_layers(16)
    if name == "resnet50_int8":     # config 4
        return "i8", 3, wl.resnet50_layers(32)
    if name == "fc_sweep_fp32":     # config 5
        return "f32", 4, wl.fc_sweep_layers()
    if name == "fc_sweep_int8":
        return "i8", 4, wl.fc_sweep_layers()
    if name == "resnet50_tail_fp32":   # block tails: 1x1 expand + residual add + Relu in one kernel
        return "f32", 5, wl.resnet50_block_tails(32)
    if name == "resnet50_tail_int8":
        return "i8", 5, wl.resnet50_block_tails(32)
    if name == "resnet50_block_fp32":  # a whole bottleneck block back to back out of one planned arena
        return "f32", 6, wl.resnet50_bottleneck(32)
    if name == "resnet50_block_int8":
        return "i8", 6, wl.resnet50_bottleneck(32)
    if name == "depthwise_fp32":       # one 3x3 filter per channel: nine products per output, a stream through HBM
        return "f32", 7, wl.depthwise_layers(32)
    if name == "depthwise_int8":
        return "i8", 7, wl.depthwise_layers(32)
    raise SystemExit(f"unknown workload {name}; choose from {WORKLOADS}")


class Layer:
    """One layer resident on the device plus the closure that launches it."""

    TENSORS = ("x", "w", "b", "y", "add", "ws")

    def __init__(self, spec, dtype, seed, torch, glowmi):
        from paper_1805_00907_amd import workloads as wl
        self.spec = spec
        self.dtype = dtype
        self.is_conv = isinstance(spec, wl.ConvLayer)
        dev = "cuda:0"
        to = lambda a: torch.from_numpy(a).to(dev)
        elem = 4 if dtype == "f32" else 1
        self.ops = spec.ops
        self.bytes = spec.alg_bytes(elem)
        self.set_variant("")
        if self.is_conv:
            self.desc = glowmi.ConvDesc(spec.n, spec.h, spec.w, spec.c, spec.k, spec.r, spec.s, spec.stride,
                                        spec.stride, spec.pad, spec.pad, spec.pad, spec.pad, spec.groups)
            yshape = (spec.n, spec.oh, spec.ow, spec.k)
        else:
            yshape = (spec.M, spec.N)
        if dtype == "f32":
            gen = wl.conv_inputs_f32 if self.is_conv else wl.fc_inputs_f32
            x, w, b = gen(spec, seed)          # timing does not depend on the value distribution
            self.x, self.w, self.b = to(x), to(w), to(b)
            self.y = torch.empty(yshape, dtype=torch.float32, device=dev)
            self.add = to(wl.addend_f32(spec, seed)) if getattr(spec, "add", False) else None
            if self.is_conv:
                nws = glowmi.conv2d_workspace_bytes(self.desc)
            else:
                nws = glowmi.fc_workspace_bytes(spec.M, spec.K, spec.N)
        else:
            gen = wl.conv_inputs_q if self.is_conv else wl.fc_inputs_q
            x, w, b, qp = gen(spec, seed)
            self.x, self.w, self.b = to(x), to(w), to(b)
            self.qp = (glowmi.QParam(qp.x_scale, qp.x_off), glowmi.QParam(qp.w_scale, qp.w_off),
                       glowmi.QParam(qp.y_scale, qp.y_off))
            self.y = torch.empty(yshape, dtype=torch.int8, device=dev)
            self.add = None
            if getattr(spec, "add", False):
                codes, r_scale, r_off = wl.addend_q(spec, seed, qp.y_scale)
                self.add, self.add_q = to(codes), glowmi.QParam(r_scale, r_off)
            if self.is_conv:
                nws = glowmi.qconv2d_workspace_bytes(self.desc)
            else:
                nws = glowmi.qfc_workspace_bytes(spec.M, spec.K, spec.N)
        self.ws = torch.empty(nws, dtype=torch.uint8, device=dev) if nws else None
        self.glowmi = glowmi
        self.variant = ""
        self.planes = None
        self.variant_packed = ""

    def pack_filter(self, torch, stream):
        """The paper's compile-time step (Section 5.3: a filter's memory layout is changed once, for the kernel
        that reads it): cut the constant fp32 weights into the fp16 planes, outside every timed region.
        Returns the time it took in microseconds, None when this layer's shape has no plane form."""
        g, s = self.glowmi, self.spec
        if self.dtype != "f32":
            return None
        nbytes = g.conv2d_filter_planes_bytes(self.desc) if self.is_conv else g.fc_filter_planes_bytes(s.K, s.N)
        if nbytes == 0:
            return None
        self.planes = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
        nws = g.conv2d_packed_workspace_bytes(self.desc) if self.is_conv else g.fc_packed_workspace_bytes(s.M, s.K, s.N)
        self.ws_packed = torch.empty(nws, dtype=torch.uint8, device="cuda:0") if nws else None
        t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for _ in range(2):                # the second run is the one reported (first touch of the buffer aside)
            t0.record(stream)
            if self.is_conv:
                g.conv2d_pack_filter(self.w, self.desc, self.planes, stream)
            else:
                g.fc_pack_filter(self.w, s.K, s.N, self.planes, stream)
            t1.record(stream)
        torch.cuda.synchronize()
        return t0.elapsed_time(t1) * 1e3

    def launch_packed(self, stream):
        """launch() with the weights' planes made ahead of time; layers without a plane form launch as usual."""
        g, s = self.glowmi, self.spec
        if self.planes is None:
            return self.launch(stream)
        if self.is_conv:
            g.conv2d_packed(self.x, self.w, self.planes, self.b, self.y, self.desc, self.add, s.act, self.ws_packed,
                            stream)
        else:
            g.fc_packed(self.x, self.w, self.planes, self.b, self.y, s.M, s.K, s.N, s.act, self.ws_packed, stream)

    def set_variant(self, variant):
        """The roofline of a layer depends on which matrix cores its kernel multiplies on."""
        self.variant = variant
        self.mfma_peak, self.products = _mfma_peak(self.dtype, variant)
        t_mfma, t_hbm = self.ops / self.mfma_peak, self.bytes / PEAK_HBM
        self.bound = "mfma" if t_mfma >= t_hbm else "hbm"
        self.t_roof = max(t_mfma, t_hbm)

    def device_bytes(self):
        return sum(t.numel() * t.element_size() for t in (getattr(self, n) for n in self.TENSORS) if t is not None)

    def clone(self):
        """The same layer on its own copies of every tensor (for the cold-cache rotation)."""
        other = copy.copy(self)
        for n in self.TENSORS:
            t = getattr(self, n)
            setattr(other, n, None if t is None else t.clone())
        return other

    def launch(self, stream):
        g, s = self.glowmi, self.spec
        if self.dtype == "f32":
            if self.is_conv and self.add is not None:
                g.conv2d_chain(self.x, self.w, self.b, self.y, self.desc, self.add, s.act, self.ws, stream)
            elif self.is_conv:
                g.conv2d(self.x, self.w, self.b, self.y, self.desc, s.act, self.ws, stream)
            else:
                g.fc(self.x, self.w, self.b, self.y, s.M, s.K, s.N, s.act, self.ws, stream)
        else:
            xq, wq, yq = self.qp
            if self.is_conv and self.add is not None:
                g.qconv2d_chain(self.x, xq, self.w, wq, self.b, self.y, yq, self.desc, self.add, self.add_q,
                                s.act, self.ws, stream)
            elif self.is_conv:
                g.qconv2d(self.x, xq, self.w, wq, self.b, self.y, yq, self.desc, s.act, self.ws, stream)
            else:
                g.qfc(self.x, xq, self.w, wq, self.b, self.y, yq, s.M, s.K, s.N, s.act, self.ws, stream)


class Sequence:
    """A chain of layers launched with ONE glowmi_seq_* call: activations live in a single arena whose
    regions are planned up front; presented to the timing code as one layer."""

    class _Spec:
        def __init__(self, name, gemm):
            self.name, self.gemm = name, gemm

    def __init__(self, layers, dtype, torch, glowmi, name):
        self.parts, self.dtype, self.glowmi = layers, dtype, glowmi
        self.spec = Sequence._Spec(name, (0, 0, 0))
        self.ops = sum(l.ops for l in layers)
        # algorithmic bytes of the block: its input, filters and biases, its output; intermediates
        # are the block's own business
        elem = 4 if dtype == "f32" else 1
        first, last = layers[0].spec, layers[-1].spec
        self.bytes = (first.n * first.h * first.w * first.c + last.n * last.oh * last.ow * last.k) * elem + \
            sum(l.spec.k * l.spec.r * l.spec.s * (l.spec.c // l.spec.groups) * elem + 4 * l.spec.k for l in layers)
        peak = PEAK_FP32_MFMA if dtype == "f32" else PEAK_INT8_MFMA
        t_mfma, t_hbm = self.ops / peak, self.bytes / PEAK_HBM
        self.bound = "mfma" if t_mfma >= t_hbm else "hbm"
        self.t_roof = max(t_mfma, t_hbm)
        self.x = layers[0].x
        self.y = layers[-1].y
        if dtype == "f32":
            tuples = [(l.desc, l.w, l.b, l.spec.act, l.spec.add) for l in layers]
        else:
            tuples = [(l.desc, l.w, l.b, l.spec.act, l.spec.add, l.qp[1], l.qp[2]) for l in layers]
            self.xq = layers[0].qp[0]
        self.arr = glowmi.seq_layers(tuples)
        nbytes = glowmi.seq_arena_bytes(self.arr, dtype != "f32")
        self.arena = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
        self.variant = "sequence"

    def device_bytes(self):
        return LLC_BYTES * 4          # never rotated

    def launch(self, stream):
        if self.dtype == "f32":
            self.glowmi.seq_conv2d(self.x, self.arr, self.y, self.arena, stream)
        else:
            self.glowmi.seq_qconv2d(self.x, self.xq, self.arr, self.y, self.arena, stream)


def _cpu_baseline(workload, dtype, cfg_index, unit_scale, budget_s):
    """The oracle as it stands, timed on this machine's host cores on a bounded sample."""
    import oracle
    from paper_1805_00907_amd import workloads as wl
    import dataclasses

    _, _, specs = _build_workload(workload)

    def rows_of(s):
        return s.n if isinstance(s, wl.ConvLayer) else s.M

    def shrink(s, rows):
        if isinstance(s, wl.ConvLayer):
            return s.with_batch(max(1, min(s.n, rows)))
        return dataclasses.replace(s, M=max(1, min(s.M, rows)))

    def run(specs_):
        ops, t = 0, 0.0
        for i, s in enumerate(specs_):
            seed = wl.layer_seed(cfg_index, i)
            if isinstance(s, wl.ConvLayer):
                st, pd = (s.stride, s.stride), (s.pad,) * 4
                if dtype == "f32":
                    x, w, b = wl.conv_inputs_f32(s, seed)
                    r = wl.addend_f32(s, seed) if s.add else None
                    t0 = time.perf_counter(); oracle.conv2d_f32_add(x, w, b, r, st, pd, s.groups, act=s.act)
                else:
                    x, w, b, qp = wl.conv_inputs_q(s, seed)
                    r, r_scale, r_off = wl.addend_q(s, seed, qp.y_scale) if s.add else (None, 1.0, 0)
                    t0 = time.perf_counter()
                    oracle.qconv2d_add(x, qp.x_scale, qp.x_off, w, qp.w_scale, qp.w_off, b, r, r_scale, r_off,
                                       qp.y_scale, qp.y_off, st, pd, s.groups, act=s.act)
            else:
                if dtype == "f32":
                    a, w, b = wl.fc_inputs_f32(s, seed)
                    t0 = time.perf_counter(); oracle.fc_f32(a, w, b, act=s.act)
                else:
                    a, w, b, qp = wl.fc_inputs_q(s, seed)
                    t0 = time.perf_counter()
                    oracle.qfc(a, qp.x_scale, qp.x_off, w, qp.w_scale, qp.w_off, b, qp.y_scale, qp.y_off, act=s.act)
            t += time.perf_counter() - t0
            ops += s.ops
        return ops, t

    # probe every layer at batch/rows 1 to learn the host's rate, then run the largest sample of
    # the workload (all layers, batch/rows capped) that fits the time budget
    ops1, t1 = run([shrink(s, 1) for s in specs])
    rate = ops1 / max(t1, 1e-4)
    cap = max(rows_of(s) for s in specs)
    while cap > 1 and sum(shrink(s, cap).ops for s in specs) / rate > budget_s:
        cap //= 2
    sample = [shrink(s, cap) for s in specs]
    ops, t = run(sample)
    passes = 1
    # the probe at one row underrates the host, so the capped sample often ends well inside the budget: a budget of
    # ten seconds and more (the headline's) is filled to two thirds with further passes over the same sample
    while budget_s >= 10 and t < budget_s * 2 / 3 and passes < 16:
        o2, t2 = run(sample)
        ops, t, passes = ops + o2, t + t2, passes + 1
    full = cap >= max(rows_of(s) for s in specs)
    times = "once" if passes == 1 else f"{passes} times"
    desc = (f"every layer of {workload} {times} at full size" if full
            else f"every layer of {workload} {times}, batch/rows capped at {cap}")
    return {"value": ops / t / unit_scale, "unit": "TFLOP/s" if dtype == "f32" else "TOP/s",
            "cores": oracle.num_threads(), "kind": "oracle", "sample": desc, "seconds": round(t, 2)}


def _median(v):
    v = sorted(v)
    return v[len(v) // 2]


def _time_graph_amortised(layer, torch):
    """us per launch of GRAPH_LAUNCHES back-to-back launches of one layer replayed as one HIP graph."""
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        layer.launch(side)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            for _ in range(GRAPH_LAUNCHES):
                layer.launch(side)
    torch.cuda.synchronize()
    graph.replay()
    torch.cuda.synchronize()
    times = []
    for _ in range(5):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        graph.replay()
        e1.record()
        torch.cuda.synchronize()
        times.append(e0.elapsed_time(e1))
    return _median(times) * 1e3 / GRAPH_LAUNCHES


def _time_cold(layer, stream, torch):
    """us per launch when consecutive launches rotate over copies of the layer's tensors that together
    exceed COLD_ROTATION_BYTES: nothing a launch reads is left in the last-level cache by the previous one."""
    per = max(layer.device_bytes(), 1)
    copies = min(96, max(2, -(-COLD_ROTATION_BYTES // per)))
    ring = [layer] + [layer.clone() for _ in range(copies - 1)]
    for l in ring:
        l.launch(stream)
    torch.cuda.synchronize()
    rounds = 3 if copies >= 8 else 8
    ev = []
    for _ in range(rounds):
        for l in ring:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            l.launch(stream)
            e1.record(stream)
            ev.append((e0, e1))
    torch.cuda.synchronize()
    return _median([a.elapsed_time(b) for a, b in ev]) * 1e3, copies


class _Floor:
    """The smallest launch the library has (one workgroup, 16 elements), timed like a layer."""

    def __init__(self, torch, glowmi):
        self.q = torch.zeros(16, dtype=torch.int8, device="cuda:0")
        self.x = torch.empty(16, dtype=torch.float32, device="cuda:0")
        self.qp = glowmi.QParam(0.5, 0)
        self.glowmi = glowmi

    def launch(self, stream):
        self.glowmi.dequantize(self.q, self.x, self.qp, stream=stream)


def launch_floor(torch, glowmi):
    stream = torch.cuda.current_stream()
    f = _Floor(torch, glowmi)
    for _ in range(20):
        f.launch(stream)
    torch.cuda.synchronize()
    ev = []
    for _ in range(50):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        f.launch(stream)
        e1.record(stream)
        ev.append((e0, e1))
    torch.cuda.synchronize()
    eager = _median([a.elapsed_time(b) for a, b in ev]) * 1e3
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(200):
        f.launch(stream)
    e1.record(stream)
    torch.cuda.synchronize()
    back_to_back = e0.elapsed_time(e1) * 1e3 / 200
    return {"eager_events": round(eager, 2), "eager_back_to_back": round(back_to_back, 2),
            "graph": round(_time_graph_amortised(f, torch), 2),
            "what": "glowmi_dequantize of 16 elements (one workgroup)"}


def run_workload(name, args, torch, glowmi, cpu_budget_s):
    from paper_1805_00907_amd import workloads as wl
    stream = torch.cuda.current_stream()
    dtype, cfg_index, specs = _build_workload(name)
    layers = [Layer(s, dtype, wl.layer_seed(cfg_index, i), torch, glowmi) for i, s in enumerate(specs)]
    if name in CHAINED:
        layers = [Sequence(layers, dtype, torch, glowmi, f"{name}@b{specs[0].n} ({len(specs)} launches)")]
    unit = "TFLOP/s" if dtype == "f32" else "TOP/s"
    total_ops = sum(l.ops for l in layers)

    def step():
        for l in layers:
            l.launch(stream)

    for l in layers:                      # first touch + variant names
        l.launch(stream)
        if isinstance(l, Sequence):
            l.variant = "sequence:" + glowmi.last_variant()
        else:
            l.set_variant(glowmi.last_variant())
    torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # ---- per-layer calibration (untimed part of the report): events around every launch
    cal_steps = max(5, min(20, args.steps))
    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in layers]
          for _ in range(cal_steps)]
    for s in range(cal_steps):
        for i, l in enumerate(layers):
            ev[s][i][0].record(stream)
            l.launch(stream)
            ev[s][i][1].record(stream)
    torch.cuda.synchronize()
    per_layer_ms = [_median([ev[s][i][0].elapsed_time(ev[s][i][1]) for s in range(cal_steps)])
                    for i in range(len(layers))]
    by_variant = {}
    for l, ms in zip(layers, per_layer_ms):
        by_variant[_kernel_of(l.variant)] = by_variant.get(_kernel_of(l.variant), 0.0) + ms
    dominant = max(by_variant, key=by_variant.get)
    dom_idx = [i for i, l in enumerate(layers) if _kernel_of(l.variant) == dominant]

    # ---- timed region: exactly `steps` steps, events only around the dominant kernel's launches
    dom_ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in dom_idx]
              for _ in range(args.steps)]
    torch.cuda.synchronize()
    if args.graph:
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            step_on = lambda st: [l.launch(st) for l in layers]
            step_on(side)
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                step_on(side)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    else:
        t0 = time.perf_counter()
        for s in range(args.steps):
            j = 0
            for i, l in enumerate(layers):
                if j < len(dom_idx) and dom_idx[j] == i:
                    dom_ev[s][j][0].record(stream)
                    l.launch(stream)
                    dom_ev[s][j][1].record(stream)
                    j += 1
                else:
                    l.launch(stream)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = total_ops / (ms_per_step * 1e-3) / 1e12

    if args.graph:   # no events inside a captured graph: the dominant kernel's figure is the calibration pass's
        dom_ms = [per_layer_ms[i] for i in dom_idx]
    else:
        dom_ms = [dom_ev[s][j][0].elapsed_time(dom_ev[s][j][1]) for s in range(args.steps) for j in range(len(dom_idx))]
    avg_launch_s = sum(dom_ms) / len(dom_ms) * 1e-3
    dom_layers = [layers[i] for i in dom_idx]
    dom_ops = sum(l.ops for l in dom_layers) / len(dom_layers)          # algorithmic ops per launch
    dom_bytes = sum(l.bytes for l in dom_layers) / len(dom_layers)
    mfma_peak, products = _mfma_peak(dtype, dominant)
    dom_bound = "mfma" if dom_ops / mfma_peak >= dom_bytes / PEAK_HBM else "hbm"
    if dom_bound == "mfma":
        achieved, peak, runit = dom_ops / avg_launch_s / 1e12, mfma_peak / 1e12, unit
    else:
        achieved, peak, runit = dom_bytes / avg_launch_s / 1e9, PEAK_HBM / 1e9, "GB/s"
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            traffic = json.load(f).get(f"{name}:{dominant}")
    roofline = {"bound": dom_bound, "achieved": round(achieved, 3), "peak": peak, "unit": runit,
                "frac": round(achieved / peak, 4), "traffic": traffic, "kernel": dominant,
                "launches_per_step": len(dom_idx), "avg_launch_us": round(avg_launch_s * 1e6, 2)}
    shapes = sorted({layers[i].variant for i in dom_idx})
    if shapes != [dominant]:
        roofline["variants"] = shapes        # the same kernel with the pixel-tile shape picked for each layer
    if products > 1 and dom_bound == "mfma":
        # `frac` is algorithmic fp32 flops against the fp16 / bf16 peak; the matrix pipes execute `products`
        # multiply-adds of pieces per algorithmic one, so their utilisation is products x frac
        roofline.update({"mfma_dtype": ("fp16" if products == F16_PRODUCTS else "bf16") + ", fp32 accumulate",
                         "products_per_mac": products,
                         "pipe_frac": round(products * achieved / peak, 4),
                         "fp32_mfma_peak": PEAK_FP32_MFMA / 1e12,
                         "frac_of_fp32_mfma_peak": round(achieved * 1e12 / PEAK_FP32_MFMA, 4)})
    if "igemm_f32_p3" in dominant:
        # one call of this kernel's layer = the range pass and the packing kernel (operands cut into fp16 planes) + the contraction;
        # the event pair brackets the call, so the packing is inside avg_launch_us (profiles/ has the kernels apart)
        roofline["launch_includes_packing"] = True

    layer_rows = []
    for l, ms in zip(layers, per_layer_ms):
        t = ms * 1e-3
        row = {"layer": l.spec.name, "gemm_mnk": list(l.spec.gemm), "kernel": l.variant,
               "us": round(ms * 1e3, 2), unit: round(l.ops / t / 1e12, 3),
               "GB/s": round(l.bytes / t / 1e9, 1), "bound": l.bound,
               "roofline_frac": round(l.t_roof / t, 4),
               "llc": "warm" if l.device_bytes() <= LLC_BYTES else "cold"}
        if getattr(l, "products", 1) > 1:
            row["pipe_frac"] = round(l.products * l.ops / l.mfma_peak / t, 4)
        if not args.quick:
            if l.bound == "hbm" and row["llc"] == "warm":
                us_cold, copies = _time_cold(l, stream, torch)
                row["us_cold"] = round(us_cold, 2)
                row["GB/s_cold"] = round(l.bytes / (us_cold * 1e-6) / 1e9, 1)
                row["roofline_frac_cold"] = round(l.t_roof / (us_cold * 1e-6), 4)
                row["cold_copies"] = copies
            if ms * 1e3 < SMALL_LAYER_US:
                us_graph = _time_graph_amortised(l, torch)
                row["us_graph"] = round(us_graph, 2)
                row["roofline_frac_graph"] = round(l.t_roof / (us_graph * 1e-6), 4)
        layer_rows.append(row)

    # ---- the same step with the filters transformed ahead of time (the paper's compile-time step), reported
    # APART: `value` above cuts the weights inside every call
    packed = None
    if dtype == "f32" and name not in CHAINED:
        pack_us = [l.pack_filter(torch, stream) for l in layers]
        if any(u is not None for u in pack_us):
            for l in layers:
                l.launch_packed(stream)
                l.variant_packed = glowmi.last_variant()
            for _ in range(max(2, args.warmup)):
                for l in layers:
                    l.launch_packed(stream)
            pev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in layers]
                   for _ in range(cal_steps)]
            for s in range(cal_steps):
                for i, l in enumerate(layers):
                    pev[s][i][0].record(stream)
                    l.launch_packed(stream)
                    pev[s][i][1].record(stream)
            torch.cuda.synchronize()
            packed_ms = [_median([pev[s][i][0].elapsed_time(pev[s][i][1]) for s in range(cal_steps)])
                         for i in range(len(layers))]
            t0 = time.perf_counter()
            for s in range(args.steps):
                for l in layers:
                    l.launch_packed(stream)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            p_ms = (t1 - t0) * 1e3 / args.steps
            packed = {"value": round(total_ops / (p_ms * 1e-3) / 1e12, 3), "unit": unit, "steps": args.steps,
                      "ms_per_step": round(p_ms, 4),
                      "pack_us_once": round(sum(u for u in pack_us if u is not None), 1),
                      "note": "same step through glowmi_*_packed: the weights' fp16 planes made once by "
                              "glowmi_*_pack_filter outside the timed region (pack_us_once, all layers); "
                              "not the headline"}
            for row, l, ms, u in zip(layer_rows, layers, packed_ms, pack_us):
                if u is not None:
                    row["us_packed"] = round(ms * 1e3, 2)
                    row["kernel_packed"] = l.variant_packed
                    row["pack_us_once"] = round(u, 1)

    block = {"value": round(value, 3), "unit": unit, "steps": args.steps, "warmup": args.warmup,
             "ms_per_step": round(ms_per_step, 4), "dtype": "f32" if dtype == "f32" else "int8",
             "config": {"workload": name, "layers": len(layers),
                        "launch": "hip graph replay" if args.graph else "eager",
                        "note": "ResNet-50/VGG-19 layer shapes, seeded synthetic values; no trained weights"},
             "roofline": roofline}
    if packed is not None:
        block["filters_packed_ahead"] = packed
    block["layers"] = layer_rows
    # the CPU oracle is timed after ALL GPU measurements (see main): its threads would otherwise compete
    # with the launching thread, and the GPU would idle and clock down between workloads
    block["_cpu_args"] = (name, dtype, cfg_index, 1e12, cpu_budget_s)
    del layers
    torch.cuda.empty_cache()
    return block


def _finish_block(block, want_cpu):
    """Attach the CPU baseline (keeping the key order value .. roofline, cpu_baseline, layers)."""
    cpu_args = block.pop("_cpu_args")
    if not want_cpu:
        return block
    layers = block.pop("layers")
    block["cpu_baseline"] = _cpu_baseline(*cpu_args)
    block["layers"] = layers
    return block


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default=HEADLINE, choices=WORKLOADS, help="the headline workload")
    ap.add_argument("--only", action="store_true",
                    help="time the headline workload only (default: the other baseline configurations follow "
                         "under the key `workloads`)")
    ap.add_argument("--quick", action="store_true",
                    help="skip the per-layer cold-cache rotation and graph-amortised measurements")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step in a HIP graph and time replays of it (launch-overhead "
                         "amortisation); the roofline figure then comes from the eager calibration pass")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain device copy of 256 MiB (a kernel of known traffic, used to "
                         "scale rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py: this build is single-GPU (one MI355X per box); run with --gpus 1. "
                         "Sharding is a design note only (batch/row split needs no exchange).")

    import torch
    import paper_1805_00907_amd as glowmi

    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU (no CPU fallback exists)")
    glowmi.library()
    torch.cuda.set_device(0)

    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        dst.copy_(src)                    # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    floor = None if args.quick else launch_floor(torch, glowmi)
    head = run_workload(args.workload, args, torch, glowmi, cpu_budget_s=15.0)
    others = {}
    if not args.only:
        others = {name: run_workload(name, args, torch, glowmi, cpu_budget_s=4.0)
                  for name in ALSO if name != args.workload}
    head = _finish_block(head, not args.no_cpu_baseline)
    others = {name: _finish_block(b, not args.no_cpu_baseline) for name, b in others.items()}
    out = {
        "metric": f"{head['unit']} per conv/FC layer set ({args.workload}), with per-layer % of MFMA/HBM roofline",
        "value": head["value"], "unit": head["unit"], "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": head["dtype"], "data": "synthetic",
        "config": head["config"], "roofline": head["roofline"],
    }
    if "cpu_baseline" in head:
        out["cpu_baseline"] = head["cpu_baseline"]
    if "filters_packed_ahead" in head:
        out["filters_packed_ahead"] = head["filters_packed_ahead"]
    if floor is not None:
        out["launch_floor_us"] = floor
    out["layers"] = head["layers"]
    if others:
        out["workloads"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
