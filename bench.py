#!/usr/bin/env python3
"""Benchmark of the Hadamard-quantised layer hot path on one MI355X.

A "step" is one pass of the whole hot path over the LDM-4-shaped layer sweep
(configuration 5: batch 16, W4A4, fp16 I/O, block-64 Hadamard): for each of the
nine layers, hq_act_hadamard_quant on the fp16 activation followed by
hq_int_conv2d / hq_int_linear on the packed codes.  Weights are quantised once,
offline, outside the timed region.  All inputs are seeded synthetic tensors,
resident in HBM before timing starts.

Prints ONE JSON line.  `value` is the aggregate integer throughput of the sweep
(2*M*N*K_total operations per layer, summed, divided by the wall time of a
step).  Consecutive steps alternate between two complete sets of activation,
code, scale and output buffers, so that the data a step touches (two sets:
about 440 MB) does not fit the 256 MB last-level cache.  `roofline` is for the
dominant kernel (the 3x3 implicit-GEMM convolutions) from HIP-event durations
taken around runs of identical launches in a second, instrumented pass, in which
every kernel rotates through as many buffer sets as it takes to exceed 288 MB.
`hadamard_quant` reports the standalone transform+quantise kernel on the largest
activation with the same kind of rotation.  `cpu_baseline` is the CPU oracle on
one whole step of the same workload (about two seconds on the host's cores).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT8_MFMA_PEAK_TOPS = 256 * 8192 * 2.4e9 / 1e12      # 5033 TOP/s dense int8, 256 CUs at 2.4 GHz
HBM_PEAK_GBS = 8000.0
CONFIG = 5


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--eager", action="store_true", help="time the Python launch loop instead of a HIP graph replay")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU; run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2512_05746_amd as hq
    import workloads

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    hq.load_library()
    torch.cuda.set_device(0)
    props = torch.cuda.get_device_properties(0)
    clock_khz = getattr(props, "clock_rate", 0) or 2400000
    layers = workloads.config_layers(CONFIG)

    # ---- resident inputs, offline weight preparation, preallocated outputs -----------------
    # Two complete buffer sets (the second a copy of the first): consecutive timed steps alternate
    # between them, so a step never finds its data in the 256 MB last-level cache.
    def new_buffers(layer, x):
        xq = torch.empty(x.shape[:-1] + (layer.k_in // 2,), dtype=torch.uint8, device="cuda")
        sx = torch.empty(x.shape[:-1], dtype=torch.float32, device="cuda")
        y = torch.empty(x.shape[:-1] + (layer.n_out,), dtype=torch.float16, device="cuda")
        return xq, sx, y

    state, state_b = [], []
    for layer in layers:
        x = torch.from_numpy(workloads.make_x(layer)).cuda()
        w = torch.from_numpy(workloads.make_w(layer)).cuda()
        wq, sw = hq.hq_quantize_weights(w, workloads.HAD_BLOCK, layer.w_bits)
        del w
        state.append((layer, x, wq, sw) + new_buffers(layer, x))
        xb2 = x.clone()
        state_b.append((layer, xb2, wq, sw) + new_buffers(layer, xb2))
    torch.cuda.synchronize()
    set_bytes = sum(sum(t.numel() * t.element_size() for t in s[1:]) for s in state)

    def run_quant(s):
        layer, x, wq, sw, xq, sx, y = s
        hq.hq_act_hadamard_quant(x, workloads.HAD_BLOCK, layer.a_bits, out=(xq, sx))

    def run_int(s):
        layer, x, wq, sw, xq, sx, y = s
        if layer.kind == "conv":
            hq.hq_int_conv2d(xq, sx, wq, sw, None, ksize=layer.ksize, y_dtype=torch.float16, out=y)
        else:
            hq.hq_int_linear(xq, sx, wq, sw, None, y_dtype=torch.float16, out=y)

    def step(which=None):
        for s in (state if which is None else which):
            run_quant(s)
            run_int(s)

    total_ops = sum(l.ops for l in layers)

    # One step = 18 launches of 5..45 us each.  They are captured once into a HIP graph (no
    # memset nodes: the kernels clear nothing) and the timed region replays it, so the step
    # time is the device's, not the Python launch loop's.  --eager times the plain loop.
    graph = None
    sets = (state, state_b)
    if not args.eager:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for st in sets:
                step(st)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = []
        for st in sets:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                step(st)
            graph.append(g)

    def run_step(i):
        if graph is not None:
            graph[i % 2].replay()
        else:
            step(sets[i % 2])

    for i in range(args.warmup):
        run_step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        run_step(i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall / args.steps * 1e3
    value = total_ops / (wall / args.steps) / 1e12

    # ---- instrumented pass: HIP events around runs of identical launches ----------------------
    # A single 5 us launch bracketed by its own events mostly measures the gap to the next
    # launch, and a Python loop cannot issue launches faster than one per 5..8 us.  So every
    # kernel of every layer is captured `reps` times back to back into a HIP graph of its own,
    # and the events bracket one replay of that graph on the stream the kernels run on.
    ev = lambda: torch.cuda.Event(enable_timing=True)
    reps = max(args.steps, 20)

    def batched_us(fn, s):
        """Mean duration of fn over `reps` back-to-back launches; s is one buffer set or a list of
        sets the launches rotate through."""
        rot = s if isinstance(s, list) else [s]
        n = max(reps, len(rot))
        if args.eager:
            fn(rot[0])
            e0, e1 = ev(), ev()
            e0.record()
            for r in range(n):
                fn(rot[r % len(rot)])
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e3 / n
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for r in range(n):
                fn(rot[r % len(rot)])
        g.replay()
        torch.cuda.synchronize()
        e0, e1 = ev(), ev()
        e0.record()
        g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / n

    # Every layer's two kernels are timed while rotating through as many copies of the layer's
    # buffers as it takes to exceed the last-level cache (288 MB of activations, codes, scales and
    # outputs), so the durations are those of a kernel that finds nothing of its own in cache.
    ROTATE_BYTES = 288 << 20
    quant_us = np.zeros(len(state))
    int_us = np.zeros(len(state))
    rot_sets = []
    for i, s in enumerate(state):
        layer, x, wq, sw = s[:4]
        one = sum(t.numel() * t.element_size() for t in (x,) + tuple(s[4:]))
        n_sets = max(2, -(-ROTATE_BYTES // one))
        rot = [s, state_b[i]]
        while len(rot) < n_sets:
            x2 = x.clone()
            rot.append((layer, x2, wq, sw) + new_buffers(layer, x2))
        for r in rot:
            run_quant(r)
        quant_us[i] = batched_us(run_quant, rot)
        int_us[i] = batched_us(run_int, rot)
        rot_sets.append(len(rot))
        del rot
    torch.cuda.synchronize()

    per_layer = []
    for i, (layer, *_r) in enumerate(state):
        out_bytes = layer.m * layer.n_out * 2
        in_bytes = layer.m * layer.k_in // 2 + layer.m * 4
        w_bytes = layer.n_out * layer.taps * layer.k_in // 2
        q_bytes = layer.m * layer.k_in * 2 + layer.m * layer.k_in // 2 + layer.m * 4
        int_tops = layer.ops / int_us[i] / 1e6
        int_gbs = (out_bytes + in_bytes + w_bytes) / int_us[i] / 1e3
        # the roof that binds the integer stage of this layer: the matrix cores when its arithmetic
        # intensity is above the machine balance (peak op/s over peak bytes/s), else the output write
        mfma_bound = layer.ops / (out_bytes + in_bytes + w_bytes) > INT8_MFMA_PEAK_TOPS * 1e3 / HBM_PEAK_GBS
        per_layer.append({
            "layer": layer.name, "gop": round(layer.ops / 1e9, 3),
            "int_us": round(float(int_us[i]), 2),
            "int_tops": round(int_tops, 1),
            "int_frac_mfma_peak": round(int_tops / INT8_MFMA_PEAK_TOPS, 4),
            "int_gbs": round(int_gbs, 1),
            "int_binding_roof": "mfma" if mfma_bound else "hbm",
            "int_frac_of_binding_roof": round(int_tops / INT8_MFMA_PEAK_TOPS if mfma_bound
                                              else int_gbs / HBM_PEAK_GBS, 4),
            "quant_us": round(float(quant_us[i]), 2),
            "quant_gbs": round(q_bytes / quant_us[i] / 1e3, 1),
            "quant_frac_hbm_peak": round(q_bytes / quant_us[i] / 1e3 / HBM_PEAK_GBS, 4),
            "rotating_buffer_sets": rot_sets[i],
        })
    # ---- every layer in ONE launch: transform, quantisation, integer stage and epilogue, the codes never
    # leaving the chip (hq_act_quant_int_conv2d / hq_act_quant_int_linear), with the same buffer rotation ---
    fused_layers = []
    for i, s in enumerate(state):
        layer, x, wq, sw = s[:4]
        if layer.kind == "conv" and layer.ksize == 3:
            def run_fused(r, layer=layer):
                hq.hq_act_quant_int_conv2d(r[1], r[2], r[3], None, a_bits=layer.a_bits, y_dtype=torch.float16, out=r[6])
        else:
            def run_fused(r, layer=layer):
                hq.hq_act_quant_int_linear(r[1], r[2], r[3], None, a_bits=layer.a_bits, y_dtype=torch.float16, out=r[6])
        try:
            run_fused(s)
        except hq.HqError:
            fused_layers.append({"layer": layer.name, "built": False})
            continue
        one = x.numel() * 2 + s[6].numel() * 2
        n_sets = max(2, -(-ROTATE_BYTES // one))
        rot = [s, state_b[i]]
        while len(rot) < n_sets:
            x2 = x.clone()
            rot.append((layer, x2, wq, sw) + new_buffers(layer, x2))
        f_us = batched_us(run_fused, rot)
        del rot
        io_bytes = x.numel() * 2 + s[6].numel() * 2 + wq.numel()
        fused_layers.append({"layer": layer.name, "built": True, "fused_us": round(f_us, 2),
                             "two_calls_us": round(float(quant_us[i] + int_us[i]), 2),
                             "tops": round(layer.ops / f_us / 1e6, 1),
                             "frac_mfma_peak": round(layer.ops / f_us / 1e6 / INT8_MFMA_PEAK_TOPS, 4),
                             "fp16_in_out_and_weight_bytes": io_bytes,
                             "gbs": round(io_bytes / f_us / 1e3, 1),
                             "frac_hbm_peak": round(io_bytes / f_us / 1e3 / HBM_PEAK_GBS, 4)})
    torch.cuda.synchronize()

    # ---- the same layers with ONE static activation scale (the paper's learned per-timestep
    # scale): no abs-max pass, and a 3x3 convolution keeps one integer sum over all taps ------
    static_layers = []
    for i, s in enumerate(state):
        layer, x, wq, sw, xq, sx, y = s
        sx1 = (0.7 * sx.float().median()).reshape(1).contiguous()

        def run_quant_static(_s, x=x, sx1=sx1, xq=xq, layer=layer):
            hq.hq_act_hadamard_quant_static(x, sx1, workloads.HAD_BLOCK, layer.a_bits, out=xq)

        def run_int_static(_s, layer=layer, xq=xq, sx1=sx1, wq=wq, sw=sw, y=y):
            if layer.kind == "conv":
                hq.hq_int_conv2d_static(xq, sx1, wq, sw, None, ksize=layer.ksize, y_dtype=torch.float16, out=y)
            else:
                hq.hq_int_linear_static(xq, sx1, wq, sw, None, y_dtype=torch.float16, out=y)

        run_quant_static(s)
        q_us = batched_us(run_quant_static, s)
        i_us = batched_us(run_int_static, s)
        static_layers.append({"layer": layer.name, "int_us": round(i_us, 2),
                              "int_tops": round(layer.ops / i_us / 1e6, 1), "quant_us": round(q_us, 2)})
        run_quant(s)   # restore the dynamic codes for anything that follows
    torch.cuda.synchronize()

    # ---- the linear / 1x1 layers in the paper's Single scheme: weights quantised without the
    # transform, the integer H_raw folded into three digit planes (three integer passes) -------
    single_layers = []
    for i, s in enumerate(state):
        layer, x, wq, sw, xq, sx, y = s
        if layer.kind == "conv" and layer.ksize != 1:
            continue
        w2 = torch.from_numpy(workloads.make_w(layer)[:, 0, :].copy()).cuda()
        wq3, sw3 = hq.hq_quantize_weights_single(w2, workloads.HAD_BLOCK, layer.w_bits)
        xq2, y2 = xq.reshape(layer.m, -1), y.reshape(layer.m, -1)

        def run_int_single(_s, xq2=xq2, sx=sx, wq3=wq3, sw3=sw3, y2=y2):
            hq.hq_int_linear_single(xq2, sx.reshape(-1), wq3, sw3, None, workloads.HAD_BLOCK,
                                    y_dtype=torch.float16, out=y2)

        run_int_single(s)
        i_us = batched_us(run_int_single, s)
        single_layers.append({"layer": layer.name, "int_us": round(i_us, 2),
                              "int_tops_useful": round(layer.ops / i_us / 1e6, 1),
                              "int_tops_issued": round(3 * layer.ops / i_us / 1e6, 1)})
    torch.cuda.synchronize()

    # ---- the 3x3 layers as the paper's width-axis convolution: activations transformed along the
    # width axis with one scale, codes taken back with the integer H_raw (three digit planes),
    # un-transformed quantised weights ----------------------------------------------------------
    width_layers = []
    for i, s in enumerate(state):
        layer, x, wq, sw, xq, sx, y = s
        if not (layer.kind == "conv" and layer.ksize == 3):
            continue
        block = min(64, x.shape[2])
        w2 = torch.from_numpy(workloads.make_w(layer)).cuda()
        wq1, sw1 = hq.hq_quantize_weights(w2, 1, layer.w_bits)
        sx1 = (2.0 * sx.float().median()).reshape(1).contiguous()
        xu3 = torch.empty((3,) + tuple(xq.shape), dtype=torch.uint8, device="cuda")

        def run_quant_width(_s, x=x, sx1=sx1, xu3=xu3, block=block, layer=layer):
            hq.hq_act_hadamard_quant_width(x, sx1, block, layer.a_bits, out=xu3)

        def run_conv_width(_s, xu3=xu3, sx1=sx1, wq1=wq1, sw1=sw1, y=y, block=block):
            hq.hq_int_conv2d_width(xu3, sx1, wq1, sw1, None, block, y_dtype=torch.float16, out=y)

        run_quant_width(s)
        run_conv_width(s)
        q_us = batched_us(run_quant_width, s)
        i_us = batched_us(run_conv_width, s)
        width_layers.append({"layer": layer.name, "block": block, "quant_us": round(q_us, 2), "int_us": round(i_us, 2),
                             "int_tops_useful": round(layer.ops / i_us / 1e6, 1),
                             "int_tops_issued": round(3 * layer.ops / i_us / 1e6, 1)})
    torch.cuda.synchronize()

    # ---- the same sweep with 8-bit codes for both operands (one int8 code per byte) ---------------
    w8a8_layers = []
    for i, s in enumerate(state):
        layer, x, wq, sw, xq, sx, y = s
        w2 = torch.from_numpy(workloads.make_w(layer)).cuda()
        wq8, sw8 = hq.hq_quantize_weights(w2, workloads.HAD_BLOCK, 8)
        xq8 = torch.empty(x.shape, dtype=torch.int8, device="cuda")

        def run_quant8(_s, x=x, xq8=xq8, sx=sx):
            hq.hq_act_hadamard_quant(x, workloads.HAD_BLOCK, 8, out=(xq8, sx))

        def run_int8(_s, layer=layer, xq8=xq8, sx=sx, wq8=wq8, sw8=sw8, y=y):
            if layer.kind == "conv":
                hq.hq_int_conv2d_i8(xq8, sx, wq8, sw8, None, ksize=layer.ksize, y_dtype=torch.float16, out=y)
            else:
                hq.hq_int_linear_i8(xq8.reshape(layer.m, -1), sx.reshape(-1), wq8, sw8, None,
                                    y_dtype=torch.float16, out=y.reshape(layer.m, -1))

        run_quant8(s)
        run_int8(s)
        q_us = batched_us(run_quant8, s)
        i_us = batched_us(run_int8, s)
        w8a8_layers.append({"layer": layer.name, "int_us": round(i_us, 2),
                            "int_tops": round(layer.ops / i_us / 1e6, 1), "quant_us": round(q_us, 2)})
        run_quant(s)   # restore the 4-bit scales for anything that follows
    torch.cuda.synchronize()

    # ---- the downsampling convolutions (3x3, stride 2, pad 1) at the sweep's first three sizes -------
    down_layers = []
    for s in state:
        layer, x, wq, sw, xq, sx, y = s
        if not (layer.kind == "conv" and layer.ksize == 3 and x.shape[1] >= 16):
            continue
        ho = (x.shape[1] - 1) // 2 + 1
        y2 = torch.empty((x.shape[0], ho, ho, layer.n_out), dtype=torch.float16, device="cuda")

        def run_down(_s, xq=xq, sx=sx, wq=wq, sw=sw, y2=y2):
            hq.hq_int_conv2d(xq, sx, wq, sw, None, ksize=3, stride=2, y_dtype=torch.float16, out=y2)

        run_down(s)
        i_us = batched_us(run_down, s)
        down_layers.append({"layer": layer.name + "_stride2", "int_us": round(i_us, 2),
                            "int_tops": round(layer.ops / 4 / i_us / 1e6, 1)})
    torch.cuda.synchronize()

    conv3 = [i for i, (l, *_r) in enumerate(state) if l.kind == "conv" and l.ksize == 3]
    conv3_ops = sum(state[i][0].ops for i in conv3)
    conv3_us = float(sum(int_us[i] for i in conv3))
    achieved = conv3_ops / conv3_us / 1e6
    int_all_tops = total_ops / float(int_us.sum()) / 1e6

    # ---- standalone transform+quantise on the largest activation, cache-defeating rotation --
    big = max(state, key=lambda s: s[1].numel())
    layer_b, xb = big[0], big[1]
    nrot = 16
    xs = [xb.clone() for _ in range(nrot)]
    outs = [(torch.empty_like(big[4]), torch.empty_like(big[5])) for _ in range(nrot)]
    q_bytes = xb.numel() * 2 + xb.numel() // 2 + layer_b.m * 4

    def time_quant(bufs, reps, outs=outs):
        def launches():
            for r in range(reps):
                j = r % len(bufs)
                hq.hq_act_hadamard_quant(bufs[j], workloads.HAD_BLOCK, layer_b.a_bits, out=outs[j])
        launches()
        torch.cuda.synchronize()
        g = None
        if not args.eager:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                launches()
            g.replay()
            torch.cuda.synchronize()
        e0, e1 = ev(), ev()
        e0.record()
        if g is not None:
            g.replay()
        else:
            launches()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / reps

    hq_us_hbm = time_quant(xs, 8 * nrot)
    # context: a plain device copy moving the same number of bytes per launch (half read, half written)
    # through the same rotation of buffers
    half = q_bytes // 4    # fp16 elements: q_bytes / 2 bytes each way
    cp_dst = [torch.empty(half, dtype=torch.float16, device="cuda") for _ in range(nrot)]

    def time_copy(reps):
        def launches():
            for r in range(reps):
                j = r % nrot
                cp_dst[j].copy_(xs[j].view(-1)[:half])
        launches()
        torch.cuda.synchronize()
        g = None
        if not args.eager:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                launches()
            g.replay()
            torch.cuda.synchronize()
        e0, e1 = ev(), ev()
        e0.record()
        if g is not None:
            g.replay()
        else:
            launches()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / reps

    copy_us = time_copy(8 * nrot)
    del cp_dst
    hq_us_cached = time_quant(xs[:1], 64)
    # the same kernel on 8 x the batch (two tensors in rotation): the launch and its ramp no longer dominate
    xl = [torch.cat(xs[:8]), torch.cat(xs[8:])]
    outl = [(torch.cat([o[0] for o in outs[:8]]), torch.cat([o[1] for o in outs[:8]])) for _ in range(2)]
    hq_us_large = time_quant(xl, 16, outl)
    del xs, outs, xl, outl

    result = {
        "metric": "w4a4_gemm_conv_tops", "value": round(value, 2), "unit": "TOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {
            "workload": "configs[4]: LDM-4-shaped UNet layer sweep, batch 16, W4A4, fp16 I/O, "
                        "block-64 Hadamard; 9 layers, act-quant + integer conv/linear each",
            "total_gop": round(total_ops / 1e9, 2), "launches_per_step": 2 * len(state),
            "launch": "hipgraph replay" if graph is not None else "eager",
            "buffer_sets": 2, "working_set_mb": round(2 * set_bytes / 1e6, 1),
            "memory": "consecutive steps alternate between two buffer sets (working set above the 256 MB "
                      "last-level cache); per-layer and roofline durations rotate each kernel over 288 MB of buffers",
        },
        "frac_int8_mfma_peak_wall": round(value / INT8_MFMA_PEAK_TOPS, 4),
        "int8_mfma_peak_tops": {"nominal_2.4GHz": round(INT8_MFMA_PEAK_TOPS, 1),
                                "at_queried_clock": round(props.multi_processor_count * 8192 * clock_khz * 1e3 / 1e12, 1),
                                "queried_clock_mhz": round(clock_khz / 1e3), "compute_units": props.multi_processor_count,
                                "fractions_use": "nominal"},
        "int_stage_tops_kernel_time": round(int_all_tops, 1),
        "frac_int8_mfma_peak_kernel_time": round(int_all_tops / INT8_MFMA_PEAK_TOPS, 4),
        "roofline": {
            "kernel": "the four 3x3 implicit-GEMM convolution launches of the sweep: " + ", ".join(
                hq.hq_int_conv2d_kernel_name(*state[i][1].shape, state[i][0].n_out) for i in conv3),
            "bound": "mfma", "achieved": round(achieved, 1), "peak": round(INT8_MFMA_PEAK_TOPS, 1),
            "unit": "TOP/s", "frac": round(achieved / INT8_MFMA_PEAK_TOPS, 4),
            "traffic": measured_traffic(),
            "traffic_unit": "HBM bytes per launch, mean over the four 3x3 launches; read from the committed "
                            "rocprofv3 FETCH_SIZE / WRITE_SIZE summary of this command "
                            "(profiles/bench_config5_hbm_traffic.txt), not measured in this run",
            "ops_per_launch": round(conv3_ops / len(conv3)), "us_per_launch": round(conv3_us / len(conv3), 2),
            "duration": "period of back-to-back launches in one graph replay (HIP events on the launch stream); "
                        "rocprofv3's per-dispatch durations of the same kernels run a few percent longer",
        },
        "hadamard_quant": {
            "kernel": "hq_act_hadamard_quant on %s fp16" % (list(xb.shape),),
            "bytes_per_launch": q_bytes,
            "us_hbm": round(hq_us_hbm, 2), "gbs_hbm": round(q_bytes / hq_us_hbm / 1e3, 1),
            "frac_hbm_peak": round(q_bytes / hq_us_hbm / 1e3 / HBM_PEAK_GBS, 4),
            "us_cache_resident": round(hq_us_cached, 2),
            "gbs_cache_resident": round(q_bytes / hq_us_cached / 1e3, 1),
            "rotating_buffers": nrot, "peak_gbs": HBM_PEAK_GBS,
            "device_copy_same_bytes": {"what": "torch copy_ of %d bytes (as many read + written as the kernel "
                                               "moves), same rotation" % (2 * half),
                                       "us_hbm": round(copy_us, 2), "gbs_hbm": round(4 * half / copy_us / 1e3, 1)},
            "batch_x8": {"bytes_per_launch": 8 * q_bytes, "us_hbm": round(hq_us_large, 2),
                         "gbs_hbm": round(8 * q_bytes / hq_us_large / 1e3, 1),
                         "frac_hbm_peak": round(8 * q_bytes / hq_us_large / 1e3 / HBM_PEAK_GBS, 4)},
        },
        "layers": per_layer,
        "fused_mode": {
            "what": "every layer in ONE launch (hq_act_quant_int_conv2d for 3x3, hq_act_quant_int_linear for 1x1 / "
                    "linear: block Hadamard + per-token quantisation inside the kernel that multiplies, codes never "
                    "written to memory) against the two calls of the timed step; bytes = fp16 in + fp16 out + weight "
                    "codes; not part of `value`",
            "layers": fused_layers,
        },
        "static_scale_mode": {
            "what": "the same sweep through hq_*_static (one caller-supplied activation scale per tensor); "
                    "not part of `value`",
            "conv3x3_tops_kernel_time": round(conv3_ops / sum(static_layers[i]["int_us"] for i in conv3) / 1e6, 1),
            "frac_int8_mfma_peak": round(conv3_ops / sum(static_layers[i]["int_us"] for i in conv3) / 1e6
                                         / INT8_MFMA_PEAK_TOPS, 4),
            "sum_kernel_us": round(sum(l["int_us"] + l["quant_us"] for l in static_layers), 1),
            "layers": static_layers,
        },
        "single_scheme_mode": {
            "what": "linear and 1x1 layers through hq_int_linear_single (un-transformed quantised weights, "
                    "integer H_raw in three digit planes); useful = 2*M*N*K, issued = three integer passes; "
                    "not part of `value`",
            "layers": single_layers,
        },
        "width_axis_mode": {
            "what": "the 3x3 layers through hq_act_hadamard_quant_width + hq_int_conv2d_width (the paper's own "
                    "convolution: transform along the width axis, one scale, integer H_raw on the codes, "
                    "un-transformed weights); useful = 2*M*N*K, issued = three integer passes; not part of `value`",
            "layers": width_layers,
        },
        "stride2_downsampling": {
            "what": "hq_int_conv2d with stride 2 on the 3x3 layers of the sweep down to 16 x 16 (a quarter of "
                    "the stride-1 operations each); not part of `value`",
            "layers": down_layers,
        },
        "w8a8_mode": {
            "what": "the same sweep with 8-bit codes for both operands (int8 straight into the matrix "
                    "instruction, no nibble expansion); not part of `value`",
            "conv3x3_tops_kernel_time": round(conv3_ops / sum(w8a8_layers[i]["int_us"] for i in conv3) / 1e6, 1),
            "frac_int8_mfma_peak": round(conv3_ops / sum(w8a8_layers[i]["int_us"] for i in conv3) / 1e6
                                         / INT8_MFMA_PEAK_TOPS, 4),
            "layers": w8a8_layers,
        },
    }

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(layers)
    print(json.dumps(result))


def measured_traffic():
    """HBM bytes per 3x3 convolution launch from the committed rocprofv3 counter summary of this
    same command (counters cannot be read from inside the process); None if it is absent."""
    path = os.path.join(ROOT, "profiles", "bench_config5_hbm_traffic.txt")
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("conv3x3_traffic_bytes_per_launch"):
                    return int(line.split("=")[1])
    except OSError:
        pass
    return None


def cpu_baseline(layers):
    """The oracle, as it stands, on the whole sweep (all 16 images of each layer)."""
    import numpy as np

    import oracle
    import workloads

    oracle.build()
    take = 16
    ops = 0
    prepared = []
    for layer in layers:
        x = workloads.make_x(layer)
        w = workloads.make_w(layer)
        if layer.kind == "conv":
            x = x[:take]
            m = take * x.shape[1] * x.shape[2]
        else:
            m = layer.m * take // 16
            x = x[:m]
        wq, sw, _ = oracle.quantize_weights(w, workloads.HAD_BLOCK, layer.w_bits)   # offline
        prepared.append((layer, x, wq, sw))
        ops += 2 * m * layer.n_out * layer.taps * layer.k_in
    t_act = t_int = 0.0
    for layer, x, wq, sw in prepared:
        t0 = time.perf_counter()
        xq, sx, _ = oracle.act_hadamard_quant(x, workloads.HAD_BLOCK, layer.a_bits)
        t1 = time.perf_counter()
        if layer.kind == "conv":
            oracle.int_conv2d(xq, sx, wq.reshape(layer.n_out, layer.ksize, layer.ksize, layer.k_in), sw,
                              None, stride=1, pad=layer.pad, want_acc=False)
        else:
            oracle.int_linear(xq, sx, wq[:, 0, :], sw, None)
        t2 = time.perf_counter()
        t_act += t1 - t0
        t_int += t2 - t1
    dt = t_act + t_int
    cores = oracle.max_threads()
    return {"value": round(ops / dt / 1e12, 5), "unit": "TOP/s", "cores": cores, "kind": "oracle",
            "seconds": round(dt, 2), "seconds_transform_quantise": round(t_act, 2),
            "seconds_integer_dequant": round(t_int, 2),
            "sample": "one whole step: %d of 16 images of every layer of the sweep (%.1f GOP), fp64/int64 "
                      "oracle with OpenMP over rows" % (take, ops / 1e9)}


if __name__ == "__main__":
    main()
