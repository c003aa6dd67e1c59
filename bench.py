#!/usr/bin/env python3
"""Benchmark of the CPO / CPS convolution hot path on one MI355X.

A step is one pass of the whole path over one layer: CPO encode + SpMV conv, CPS encode +
SpMV conv, im2col lowering + MFMA GEMM (fp32), and the per-layer selection.  Inputs are
resident in HBM before the timed region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--all-layers]

The printed line is a summary of a few KB (contract fields, roofline of the dominant kernel, CPU
baseline, the timed layer, totals of the supplements); every record measured goes to the file
--detail-json names, the per-layer table to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
FP32_VECTOR_PEAK_TFLOPS = 157.3
FP32_MFMA_PEAK_TFLOPS = 157.3
BF16_MFMA_PEAK_TFLOPS = 2500.0


def _events(torch):
    return torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)


def _time_us(torch, fn, reps):
    """Average duration in microseconds of `fn` over `reps` back-to-back calls (HIP events on
    the current stream, which is the stream the library launches on)."""
    e0, e1 = _events(torch)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1000.0 / reps


def _cold_time_us(torch, fn, reps, sweep):
    """Median duration of `fn` when every call follows a sweep over a buffer larger than the
    on-die caches (L2 and the 256 MiB memory-side cache): each call is bracketed by its own event
    pair, and what an empty pair reads after the same sweep is subtracted."""
    def one(body):
        v = []
        for _ in range(reps):
            sweep.add_(1.0)
            e0, e1 = _events(torch)
            e0.record()
            body()
            e1.record()
            torch.cuda.synchronize()
            v.append(e0.elapsed_time(e1) * 1000.0)
        v.sort()
        return v[len(v) // 2]
    return max(one(fn) - one(lambda: None), 0.0)


class LayerRun:
    """One layer resident on the device with every stage as a callable."""

    def __init__(self, api, torch, workloads, spec, m=0):
        self.api, self.spec, self.shape = api, spec, spec.shape_tuple
        act_np, w_np = workloads.make_layer(spec, m)
        self.act_np, self.w_np = act_np, w_np
        self.buf = api.LayerBuffers(self.shape)
        self.act = torch.from_numpy(act_np).cuda()
        self.w = torch.from_numpy(w_np).cuda()
        api.cpoconv_prepare_weights(self.w, self.shape, self.buf.wt)   # once per layer, untimed
        api.im2col_prepare_weights_bf16(self.w, self.shape, self.buf.wb)   # likewise for the bf16 comparator
        torch.cuda.synchronize()
        b = self.buf
        self.map16 = api.EncodedMap(self.shape, in_bits=16)   # compact map: int16 IN entries
        self.stages = {
            "cpo_encode": lambda: api.cpo_encode(self.act, self.shape, b.cpo, b.scratch),
            "cpo_conv": lambda: api.cpo_conv(b.cpo, self.shape, b.wt, b.out, b.scratch),
            "cps_encode": lambda: api.cps_encode(self.act, self.shape, b.cps, b.scratch),
            "cps_conv": lambda: api.cps_conv(b.cps, self.shape, b.wt, b.out, b.scratch),
            # a layer in one call (encode + convolution): what the selection compares with im2col
            "cpo_layer": lambda: api.cpo_encode_conv(self.act, self.shape, b.cpo, b.wt, b.out, b.scratch),
            "cps_layer": lambda: api.cps_encode_conv(self.act, self.shape, b.cps, b.wt, b.out, b.scratch),
            "cpo_layer_in16": lambda: api.cpo_encode_conv(self.act, self.shape, self.map16, b.wt, b.out, b.scratch),
            "im2col_f32": lambda: api.im2col_conv(self.act, self.shape, self.w, b.lowered, b.out, 0),
            "im2col_bf16": lambda: api.im2col_conv(self.act, self.shape, b.wb, b.lowered, b.out, 2),
        }

    def set_input(self, torch, act_np):
        self.act.copy_(torch.from_numpy(act_np))

    def lengths(self):
        for k in ("cpo_encode", "cps_encode"):
            self.stages[k]()
        h_cpo, h_cps = self.buf.cpo.header(), self.buf.cps.header()
        return {"ptr": h_cpo[0], "nnz": h_cpo[1], "in_cpo": h_cpo[2], "in_cps": h_cps[2]}


def sparse_flops(spec, act_np):
    """2 x (kernel cells every NZE meets: rows x partitions holding it) x K, counted exactly."""
    import numpy as np

    C, H, W, K, kh, kw, s, p = spec.shape_tuple[:8]
    pw = p if spec.pad_w is None else spec.pad_w

    def meets(n_in, n_out, k):
        cnt = np.zeros(n_in, np.int64)
        for o in range(n_out):
            cnt[o * s:o * s + k] += 1
        return cnt

    rows = meets(spec.Ih, spec.Oh, kh)[p:p + H]
    cols = meets(spec.Iw, spec.Ow, kw)[pw:pw + W]
    nz = (act_np.view(np.uint32) & 0x7FFFFFFF) != 0
    return 2.0 * K * float(np.einsum("chw,h,w->", nz.astype(np.int64), rows, cols))


def algorithmic_figures(spec, lens, act_np):
    """Bytes and flops the method itself must move / compute for one layer (4-byte elements)."""
    C, H, W, K, kh, kw, s, p = spec.shape_tuple[:8]
    nnz, ptr = lens["nnz"], lens["ptr"]
    out_elems = K * spec.Oh * spec.Ow
    wbytes = 4 * K * C * kh * kw
    S = spec.s_im2col
    return {
        "cpo_encode_bytes": 4 * C * H * W + 8 * nnz + 4 * ptr,
        "cps_encode_bytes": 4 * C * H * W + 4 * nnz + 4 * lens["in_cps"] + 4 * ptr,
        "cpo_conv_bytes": 8 * nnz + 4 * ptr + wbytes + 4 * out_elems,
        "cps_conv_bytes": 4 * nnz + 4 * lens["in_cps"] + 4 * ptr + wbytes + 4 * out_elems,
        "sparse_flops": sparse_flops(spec, act_np),
        "im2col_f32_bytes": 4 * C * H * W + 2 * 4 * S + wbytes + 4 * out_elems,
        "im2col_bf16_bytes": 4 * C * H * W + 2 * 2 * S + wbytes + 4 * out_elems,
        "dense_flops": float(spec.dense_flops),
        "s_im2col": S,
        "cr_cpo": S / float(ptr + 2 * nnz),
        "cr_cps": S / float(ptr + nnz + lens["in_cps"]),
        "cr_cpo_with_side_band": S / float(ptr + 2 * nnz + 3 * (C + 1)),
        "cr_cps_with_side_band": S / float(ptr + nnz + lens["in_cps"] + 3 * (C + 1)),
        # in bytes, against the fp32 lowered matrix: int32 IN entries, and the compact map's int16 ones
        "cr_bytes_cpo": 4.0 * S / (4 * ptr + 4 * nnz + 4 * nnz),
        "cr_bytes_cpo_in16": 4.0 * S / (4 * ptr + 4 * nnz + 2 * nnz),
        "cr_bytes_cps_in16": 4.0 * S / (4 * ptr + 4 * nnz + 2 * lens["in_cps"]),
    }


def stage_roofline(name, us, fig):
    """Roofline entry of one stage: the bound that binds and the achieved fraction of it."""
    t = us * 1e-6
    if name.endswith("_in16"):       # the compact map: same work, narrower IN entries
        name = name[:-len("_in16")]
    if name.endswith("_layer"):      # encode + convolution in one call: both stages' bytes, the convolution's flops
        algo = name[:3]
        b = fig[algo + "_encode_bytes"] + fig[algo + "_conv_bytes"]
        gbs, tf = b / t / 1e9, fig["sparse_flops"] / t / 1e12
        if fig["sparse_flops"] / (FP32_VECTOR_PEAK_TFLOPS * 1e12) >= b / (HBM_PEAK_GBS * 1e9):
            return {"bound": "alu", "achieved": tf, "peak": FP32_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": tf / FP32_VECTOR_PEAK_TFLOPS, "hbm_gbs": gbs}
        return {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                "alu_tflops": tf}
    if name.endswith("encode"):
        a = fig[name + "_bytes"] / t / 1e9
        return {"bound": "hbm", "achieved": a, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": a / HBM_PEAK_GBS}
    if name.endswith("conv") and name[:3] in ("cpo", "cps"):
        gbs = fig[name + "_bytes"] / t / 1e9
        tf = fig["sparse_flops"] / t / 1e12
        # the binding roof is the one that takes longer at peak
        if fig["sparse_flops"] / (FP32_VECTOR_PEAK_TFLOPS * 1e12) >= fig[name + "_bytes"] / (HBM_PEAK_GBS * 1e9):
            return {"bound": "alu", "achieved": tf, "peak": FP32_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": tf / FP32_VECTOR_PEAK_TFLOPS, "hbm_gbs": gbs}
        return {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                "alu_tflops": tf}
    peak = FP32_MFMA_PEAK_TFLOPS if name == "im2col_f32" else BF16_MFMA_PEAK_TFLOPS
    tf = fig["dense_flops"] / t / 1e12
    return {"bound": "mfma", "achieved": tf, "peak": peak, "unit": "TFLOP/s", "frac": tf / peak,
            "hbm_gbs": fig[name + "_bytes"] / t / 1e9}


def event_pair_overhead_us(torch, pairs=200):
    """What two HIP events recorded back to back on the launch stream read with nothing between
    them: the part of an event-bracketed launch that is not the kernel."""
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(pairs)]
    torch.cuda.synchronize()
    for a, b in ev:
        a.record()
        b.record()
    torch.cuda.synchronize()
    v = sorted(a.elapsed_time(b) * 1e3 for a, b in ev)
    return v[len(v) // 2]


def kernel_times(api, torch, run, reps):
    """Average duration of every kernel of every stage, from HIP events recorded by the library
    around each launch on the launch stream (cpoconv_kernel_timing)."""
    out = {}
    for stage, fn in run.stages.items():
        torch.cuda.synchronize()
        api.cpoconv_kernel_timing(True)
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        out[stage] = {k: {"avg_us": round(v[0], 3), "launches": v[1]} for k, v in api.cpoconv_kernel_timing_read().items()}
        api.cpoconv_kernel_timing(False)
    return out


def kernel_roofline(stage, kernel, us, fig, spec, lens):
    """Roofline entry of one kernel launch: algorithmic bytes or flops of the launch / duration."""
    t = us * 1e-6
    C, H, W, K, kh, kw, s, p = spec.shape_tuple[:8]
    if stage.endswith("_layer"):     # kernels of the one-call stages belong to its encode or convolution half
        stage = stage[:3] + ("_encode" if kernel.startswith("encode") else "_conv")
    out_bytes = 4 * K * spec.Oh * spec.Ow
    hbm = lambda b: {"bound": "hbm", "achieved": b / t / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": b / t / 1e9 / HBM_PEAK_GBS, "algorithmic_bytes": b}
    if kernel == "encode_count":      # layers of more than 256 channels: a first launch publishes the lengths
        return hbm(4 * C * H * W)
    if kernel == "encode":
        return hbm(fig[stage + "_bytes"])
    if kernel == "conv_prologue":
        b = 4 * lens["ptr"] + 4 * C * 2 * (spec.Ow + 1)
        if stage == "cps_conv":
            b += 4 * lens["in_cps"] + 4 * lens["nnz"]
        return hbm(b)
    if kernel.startswith("spmv_conv_"):   # runs, strip, tile or lds: whichever the layer was given
        r = stage_roofline(stage, us, fig)
        r["algorithmic_flops"] = fig["sparse_flops"]
        r["algorithmic_bytes"] = fig[stage + "_bytes"]
        return r
    if kernel == "reduce_transpose":
        return hbm(2 * out_bytes)
    if kernel.startswith("im2col_lower"):
        return hbm(4 * C * H * W + (4 if kernel.endswith("f32") else 2) * fig["s_im2col"])
    if kernel.startswith("gemm"):
        peak = FP32_MFMA_PEAK_TFLOPS if kernel == "gemm_f32" else BF16_MFMA_PEAK_TFLOPS
        tf = fig["dense_flops"] / t / 1e12
        return {"bound": "mfma", "achieved": tf, "peak": peak, "unit": "TFLOP/s", "frac": tf / peak,
                "algorithmic_flops": fig["dense_flops"]}
    return None


def measure_layer(api, torch, workloads, spec, reps, warm):
    run = LayerRun(api, torch, workloads, spec)
    lens = run.lengths()
    fig = algorithmic_figures(spec, lens, run.act_np)
    times = {}
    for name, fn in run.stages.items():
        for _ in range(warm):
            fn()
        times[name] = _time_us(torch, fn, reps)
    row = {
        "layer": spec.name, "shape": list(spec.shape_tuple), "nnz": lens["nnz"],
        "density": lens["nnz"] / float(spec.C * spec.H * spec.W),
        "us": {k: round(v, 2) for k, v in times.items()},
        "cpo_total_us": round(times["cpo_layer"], 2),
        "cps_total_us": round(times["cps_layer"], 2),
        "speedup_cpo_vs_im2col_f32": times["im2col_f32"] / times["cpo_layer"],
        "speedup_cps_vs_im2col_f32": times["im2col_f32"] / times["cps_layer"],
        "cr_cpo": fig["cr_cpo"], "cr_cps": fig["cr_cps"],
        "cr_cpo_with_side_band": fig["cr_cpo_with_side_band"],
        "cr_cps_with_side_band": fig["cr_cps_with_side_band"],
        "cr_bytes_cpo": fig["cr_bytes_cpo"], "cr_bytes_cpo_in16": fig["cr_bytes_cpo_in16"],
        "cr_bytes_cps_in16": fig["cr_bytes_cps_in16"],
        "roofline": {k: stage_roofline(k, v, fig) for k, v in times.items()},
    }
    return run, row, times, fig


def offline_selection(api, torch, workloads, run, spec, reps, m_inputs=5):
    """Section 3.5: total time of each method over M offline inputs, then the two modes."""
    t = {"im2col": [], "cpo": [], "cps": []}
    for m in range(m_inputs):
        run.set_input(torch, workloads.make_activation(spec, m))
        st = run.stages
        t["im2col"].append(_time_us(torch, st["im2col_f32"], reps))
        t["cpo"].append(_time_us(torch, st["cpo_layer"], reps))
        t["cps"].append(_time_us(torch, st["cps_layer"], reps))
    run.set_input(torch, run.act_np)
    names = {api.ALGO_IM2COL: "im2col", api.ALGO_CPO: "cpo", api.ALGO_CPS: "cps"}
    return t, {"favour_time": names[api.select_layer_algo(t["im2col"], t["cpo"], t["cps"], 0)],
               "favour_space": names[api.select_layer_algo(t["im2col"], t["cpo"], t["cps"], 1)]}


def batch_supplement(api, torch, workloads, spec, n_images, reps):
    """The same layer with n_images inputs per launch (the batched entry points): per-image times,
    and the SpMV kernel's achieved rate where launches are long enough to be throughput bound.
    A supplement: `value` and `roofline` of the bench line stay on the batch-1 workload."""
    import numpy as np

    shape = spec.shape_tuple
    acts = np.stack([workloads.make_activation(spec, m % 5) for m in range(n_images)])
    buf = api.LayerBuffers(shape, n_images=n_images)
    act, w = torch.from_numpy(acts).cuda(), torch.from_numpy(workloads.make_weights(spec)).cuda()
    api.cpoconv_prepare_weights(w, shape, buf.wt)
    api.im2col_prepare_weights_bf16(w, shape, buf.wb)
    api.cps_encode_batch(act, shape, buf.cps, buf.scratch)
    stages = {
        "cpo_encode": lambda: api.cpo_encode_batch(act, shape, buf.cpo, buf.scratch),
        "cpo_conv": lambda: api.cpo_conv_batch(buf.cpo, shape, buf.wt, buf.out, buf.scratch),
        "cps_conv": lambda: api.cps_conv_batch(buf.cps, shape, buf.wt, buf.out, buf.scratch),
        "im2col_f32": lambda: api.im2col_conv_batch(act, shape, n_images, w, buf.lowered, buf.out, 0),
        "im2col_bf16": lambda: api.im2col_conv_batch(act, shape, n_images, buf.wb, buf.lowered, buf.out, 2),
    }
    stages["cpo_encode"]()
    us = {}
    for k, fn in stages.items():
        for _ in range(3):
            fn()
        us[k] = _time_us(torch, fn, reps)
    flops = sum(sparse_flops(spec, a) for a in acts)
    nnz = int(sum(((a.view(np.uint32) & 0x7FFFFFFF) != 0).sum() for a in acts))
    enc_bytes = 4 * acts.size + 8 * nnz
    torch.cuda.synchronize()
    api.cpoconv_kernel_timing(True)
    for _ in range(5):
        stages["cpo_encode"]()
        stages["cpo_conv"]()
    torch.cuda.synchronize()
    kt = api.cpoconv_kernel_timing_read()
    api.cpoconv_kernel_timing(False)
    overhead = event_pair_overhead_us(torch)
    kern = {k: round(max(v[0] - overhead, 0.1), 2) for k, v in kt.items()}
    conv_kernel = next((k for k in kern if k.startswith("spmv_conv")), None)
    out = {
        "n_images": n_images,
        "per_image_us": {k: round(v / n_images, 3) for k, v in us.items()},
        "cpo_total_per_image_us": round((us["cpo_encode"] + us["cpo_conv"]) / n_images, 3),
        "speedup_cpo_vs_im2col_f32": round(us["im2col_f32"] / (us["cpo_encode"] + us["cpo_conv"]), 4),
        "kernel_us": kern,
        "encode_hbm_gbs": round(enc_bytes / (us["cpo_encode"] * 1e-6) / 1e9, 1),
        "encode_hbm_frac": round(enc_bytes / (us["cpo_encode"] * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
    }
    if conv_kernel:
        tf = flops / (kern[conv_kernel] * 1e-6) / 1e12
        out["spmv_kernel"] = {"kernel": conv_kernel, "bound": "alu", "achieved": round(tf, 2), "peak": FP32_VECTOR_PEAK_TFLOPS,
                              "unit": "TFLOP/s", "frac": round(tf / FP32_VECTOR_PEAK_TFLOPS, 4),
                              "algorithmic_flops": flops,
                              "algorithmic_bytes": 8 * nnz + 4 * w.numel() + 4 * buf.out.numel(),
                              # HBM bytes per launch from the rocprofv3 counter runs of this very launch shape, if recorded
                              "traffic": traffic_from_profiles("%s@%dimages" % (conv_kernel, n_images))}
    return out


def chain_supplement(api, torch, workloads, n_images, reps, m_inputs=5):
    """The sixteen 3x3 layers of workload 5 joined end to end (each layer reads the stored sums of
    the one before it and applies bias + ReLU on the way in) through cpoconv_chain_forward: time of
    the whole chain per image with one method everywhere, and with the per-layer choice of Section
    3.5 made from each layer timed alone on its own chain input over M input batches."""
    import numpy as np

    specs = workloads.chain_specs()
    shapes = [s.shape_tuple for s in specs]
    _, w_np, b_np = workloads.make_chain()
    ws = [torch.from_numpy(w).cuda() for w in w_np]
    bs = [None if b is None else torch.from_numpy(b).cuda() for b in b_np]
    L = len(specs)
    chain = api.Chain(shapes, ws, bs, [b is not None for b in b_np], [api.ALGO_IM2COL] * L, n_images=n_images)
    batches = [torch.from_numpy(np.stack([workloads.make_activation(specs[0], m * n_images + j)
                                          for j in range(n_images)])).cuda() for m in range(m_inputs)]
    codes = {"im2col": api.ALGO_IM2COL, "cpo": api.ALGO_CPO, "cps": api.ALGO_CPS}
    names = {v: k for k, v in codes.items()}
    whole, per_layer = {}, {k: [[0.0] * m_inputs for _ in range(L)] for k in codes}
    for k, code in codes.items():
        chain.set_methods([code] * L)
        for _ in range(3):
            chain.forward(batches[0])
        whole[k] = _time_us(torch, lambda: chain.forward(batches[0]), reps)
        for m, act in enumerate(batches):
            chain.forward(act)                                  # every layer's input for this batch
            for i in range(L):
                x = act if i == 0 else chain.outs[i - 1]
                chain.forward(x, first=i, count=1)
                per_layer[k][i][m] = _time_us(torch, lambda: chain.forward(x, first=i, count=1), max(reps // 2, 5))
    pick_time = [api.select_layer_algo(per_layer["im2col"][i], per_layer["cpo"][i], per_layer["cps"][i], 0) for i in range(L)]
    pick_space = [api.select_layer_algo(per_layer["im2col"][i], per_layer["cpo"][i], per_layer["cps"][i], 1) for i in range(L)]
    for label, picks in (("hybrid_favour_time", pick_time), ("hybrid_favour_space", pick_space)):
        chain.set_methods(picks)
        for _ in range(3):
            chain.forward(batches[0])
        whole[label] = _time_us(torch, lambda: chain.forward(batches[0]), reps)
    # realised zero fraction of every layer's input (first batch)
    chain.set_methods([api.ALGO_IM2COL] * L)
    chain.forward(batches[0])
    torch.cuda.synchronize()
    zeros = []
    for i in range(L):
        x = batches[0] if i == 0 else chain.outs[i - 1]
        z = x if bs[i] is None else x + bs[i][None, :, None, None]
        zeros.append(round(float((z <= 0).float().mean().item()), 3))
    not_moved = sum(2 * 4 * s.C * s.H * s.W for s in specs[1:])
    return {
        "workload": "chain: workload 5's sixteen 3x3 layers joined end to end, bias + ReLU fused into the reader",
        "n_images": n_images, "layers": L, "offline_inputs": m_inputs,
        "per_image_us": {("all_" + k if k in codes else k): round(v / n_images, 2) for k, v in whole.items()},
        # the paper's figure of merit (Section 4): (T_im2col - T_method) / T_im2col over the conv layers
        "time_saving_vs_all_im2col": {k: round(1.0 - whole[k] / whole["im2col"], 4) for k in whole if k != "im2col"},
        "selection_favour_time": [names[c] for c in pick_time],
        "selection_favour_space": [names[c] for c in pick_space],
        "layers_cpo_selected": sum(c == api.ALGO_CPO for c in pick_time),
        "layers_cps_selected": sum(c == api.ALGO_CPS for c in pick_space),
        "layer_us_per_image": {k: [round(sum(t) / len(t) / n_images, 2) for t in v] for k, v in per_layer.items()},
        "input_zero_fraction": zeros,
        "activated_map_bytes_not_moved_per_image": not_moved,
    }


def _cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def _oracle_layer_worker(args):
    """One process of the all-cores leg: the unchanged one-thread oracle on an input of its own."""
    config, m, repeats = args
    import oracle
    from paper_2104_08314_amd import workloads

    spec = workloads.layers(config)[0]
    act, w = workloads.make_activation(spec, m), workloads.make_weights(spec)
    oracle.sparse_conv(oracle.cpo_encode(act, spec.shape_tuple), w)
    t0 = time.perf_counter()
    for _ in range(repeats):
        oracle.sparse_conv(oracle.cpo_encode(act, spec.shape_tuple), w)
    return (time.perf_counter() - t0) / repeats


def cpu_baseline(spec, workloads, w_np, config, inputs=5, repeats=10):
    """The CPU oracle as it stands on the same layer: CPO encode + Algorithm 2 on the layer's
    `inputs` offline inputs, `repeats` times each, one thread (about 10 s of CPU work on config 2);
    then the same unchanged oracle in one process per usable host core, each on an input of its
    own (the oracle itself stays single-threaded: the all-cores figure is layers finished per
    second by independent copies)."""
    import oracle

    shape = spec.shape_tuple
    acts = [workloads.make_activation(spec, m) for m in range(inputs)]
    oracle.cpo_encode(acts[0], shape)                     # builds / loads the library
    enc, conv, dense = [], [], []
    for act in acts:
        for _ in range(repeats):
            t0 = time.perf_counter()
            m = oracle.cpo_encode(act, shape)
            t1 = time.perf_counter()
            oracle.sparse_conv(m, w_np)
            t2 = time.perf_counter()
            enc.append((t1 - t0) * 1e6)
            conv.append((t2 - t1) * 1e6)
        t0 = time.perf_counter()
        oracle.conv_direct(act, w_np, shape)
        dense.append((time.perf_counter() - t0) * 1e6)
    med = lambda v: sorted(v)[len(v) // 2]
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count() or 1
    cores = max(1, min(usable, int(os.environ.get("OMP_NUM_THREADS", usable) or usable)))
    all_cores = None
    if cores > 1:
        import multiprocessing as mp

        try:
            with mp.get_context("fork").Pool(cores) as pool:   # called before this process touches the GPU
                t0 = time.perf_counter()
                per = pool.map(_oracle_layer_worker, [(config, m, 4) for m in range(cores)])
                wall = time.perf_counter() - t0
            # every process finished 4 layers in about 4 * mean(per) seconds: layers per second over all cores
            rate = sum(1.0 / p for p in per)
            all_cores = {"cores": cores, "us_per_layer": round(1e6 / rate, 1),
                         "kind": "independent one-thread oracle copies, one input each", "wall_s": round(wall, 2)}
        except Exception as exc:   # the baseline is a report, never a reason to lose the bench line
            all_cores = {"cores": cores, "error": str(exc)[:120]}
    return {"value": round(med(enc) + med(conv), 1), "unit": "us", "cores": 1, "kind": "oracle",
            "cpu_model": _cpu_model(), "host_cores_usable": usable,
            "encode_us": round(med(enc), 1), "conv_us": round(med(conv), 1), "dense_7loop_us": round(med(dense), 1),
            "all_cores": all_cores,
            "sample": "the whole layer (cpo encode + Algorithm 2 conv), %d inputs x %d repeats, medians; plain C, "
                      "double accumulation, gcc -O2, one thread" % (inputs, repeats)}


def trace_avg_from_profiles(kernel, summary="bench_cfg2_128at56_all_kernels.txt"):
    """Average duration (us) of `kernel` in the committed rocprofv3 kernel trace of this workload: the
    row of the summary's kernel-trace table (kernel, calls, avg_us, ...).  The tracer lengthens every
    kernel by 1.5-3 us, so it reads above the event-timed figure."""
    path = os.path.join(ROOT, "profiles", summary)
    if not os.path.exists(path):
        return None
    with open(path) as f:
        for line in f:
            parts = line.split()
            if len(parts) >= 6 and parts[0] == kernel:
                try:
                    return float(parts[2])
                except ValueError:
                    return None
    return None


def traffic_from_profiles(kernel_key):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE / WRITE_SIZE runs), if a
    summary under profiles/ records them as a line `traffic_bytes_per_launch[<key>]: <n>`."""
    pdir = os.path.join(ROOT, "profiles")
    if not os.path.isdir(pdir):
        return None
    tag = f"traffic_bytes_per_launch[{kernel_key}]:"
    for fn in sorted(os.listdir(pdir)):
        if not fn.endswith((".txt", ".md")):
            continue
        with open(os.path.join(pdir, fn)) as f:
            for line in f:
                if line.strip().startswith(tag):
                    try:
                        return float(line.split(":", 1)[1].split()[0])
                    except ValueError:
                        return None
    return None


def compact_line(full):
    """The one printed JSON line: the contract's fields, the roofline of the dominant kernel, the
    CPU baseline and short summaries; everything else measured goes to --detail-json."""
    keep = ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
            "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline", "selection")
    out = {k: full[k] for k in keep if k in full}
    row = full["layer"]
    us = row["us"]
    r3 = lambda v: None if v is None else round(v, 3)
    out["layer"] = {
        "nnz": row["nnz"], "zeros": r3(1.0 - row["density"]),
        "us": {k: us[k] for k in ("cpo_encode", "cpo_conv", "cps_encode", "cps_conv", "cpo_layer", "cps_layer",
                                  "im2col_f32", "im2col_bf16") if k in us},
        "speedup_vs_im2col_f32": {"cpo": r3(row["speedup_cpo_vs_im2col_f32"]), "cps": r3(row["speedup_cps_vs_im2col_f32"])},
        "speedup_vs_im2col_bf16": {"cpo": r3(us["im2col_bf16"] / us["cpo_layer"]), "cps": r3(us["im2col_bf16"] / us["cps_layer"])},
        "cr": {"cpo": r3(row["cr_cpo"]), "cps": r3(row["cr_cps"]), "cpo_with_side_band": r3(row["cr_cpo_with_side_band"]),
               "cps_with_side_band": r3(row["cr_cps_with_side_band"])},
        "stage_roofline": {k: {"bound": v["bound"], "frac": round(v["frac"], 4),
                               "hbm_gbs": round(v["achieved"] if v["bound"] == "hbm" else v.get("hbm_gbs", 0.0), 1)}
                           for k, v in row["roofline"].items()
                           if k in ("cpo_encode", "cpo_conv", "cps_encode", "cps_conv", "im2col_f32", "im2col_bf16")},
    }
    if "cold_us" in row:
        out["layer"]["cold_us"] = {k: row["cold_us"][k] for k in ("cpo_layer", "cps_layer", "im2col_f32") if k in row["cold_us"]}
    out["kernels_us"] = {e["stage"] + "/" + e["kernel"]: e["avg_us"] for e in full.get("kernels", [])}
    b = full.get("batch_supplement")
    if b:
        out["batch_supplement"] = {"n_images": b["n_images"], "per_image_us": b["per_image_us"],
                                   "speedup_cpo_vs_im2col_f32": b["speedup_cpo_vs_im2col_f32"],
                                   "encode_hbm_frac": b["encode_hbm_frac"],
                                   "spmv_alu_frac": (b.get("spmv_kernel") or {}).get("frac")}
    for k in ("config5_end_to_end_us", "line_layers_us"):
        if k in full:
            out[k] = full[k]
    if "layers" in full:
        ls = full["layers"]
        out["layers_summary"] = {
            "layers": len(ls),
            "cpo_faster_than_im2col_f32": sum(l["time_saving_cpo"] > 0 for l in ls),
            "cps_faster_than_im2col_f32": sum(l["time_saving_cps"] > 0 for l in ls),
            "best_time_saving_cpo": max(l["time_saving_cpo"] for l in ls),
            "cr_cpo_min_max": [min(l["cr_cpo"] for l in ls), max(l["cr_cpo"] for l in ls)],
        }
    if "chain_supplement" in full:
        out["chain_supplement"] = [{"n_images": c["n_images"], "per_image_us": c["per_image_us"],
                                    "layers_cpo_selected": c["layers_cpo_selected"]} for c in full["chain_supplement"]]
    out["detail"] = "per-kernel, per-layer and supplement records: --detail-json file; per-layer table on stderr"
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=2, help="workload whose first layer is timed")
    ap.add_argument("--all-layers", action="store_true",
                    help="also measure every layer of the five workloads and the 1 x n / n x 1 layers (per-layer report "
                         "on stderr); a full run - one without --no-chain - does so anyway")
    ap.add_argument("--detail-json", default=os.path.join(ROOT, "gpurun_out", "bench_detail.json"),
                    help="file that receives everything measured (per-kernel entries, per-layer rows, supplements); "
                         "the printed line holds the summary only ('' to skip)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--batch", type=int, default=32,
                    help="images per launch of the batched supplement (0 to skip it)")
    ap.add_argument("--no-cold", action="store_true", help="skip the cold-cache timing of the stages")
    ap.add_argument("--no-chain", action="store_true",
                    help="skip the supplements beyond the timed layer: the chained layers and, unless --all-layers "
                         "asks for it, the per-layer table")
    ap.add_argument("--chain-only", action="store_true",
                    help="run only the chained-layers supplement, with --batch images per launch, and print it")
    ap.add_argument("--batch-only", action="store_true",
                    help="run only the batched supplement of the --config layer, with --batch images per launch, and print it")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch a plain elementwise kernel that reads and writes 256 MiB, five times: the "
                         "known-size kernel that rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (the path is a single-GPU kernel pipeline); "
                 "use --gpus 1")

    from paper_2104_08314_amd import workloads

    # the CPU oracle is timed first, before this process initialises the GPU (its all-cores leg forks)
    cpu = None
    if not (args.no_cpu_baseline or args.chain_only or args.batch_only):
        spec0 = workloads.layers(args.config)[0]
        cpu = cpu_baseline(spec0, workloads, workloads.make_weights(spec0), args.config)

    import torch

    from paper_2104_08314_amd import api

    api.lib()
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    torch.cuda.set_device(0)

    if args.calibrate_copy:
        src = torch.ones(64 << 20, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    if args.chain_only:
        print(json.dumps(chain_supplement(api, torch, workloads, max(args.batch, 1), reps=10)))
        return

    spec = workloads.layers(args.config)[0]
    if args.batch_only:
        print(json.dumps(batch_supplement(api, torch, workloads, spec, max(args.batch, 1), reps=10)))
        return
    run, row, times, fig = measure_layer(api, torch, workloads, spec, reps=max(args.steps, 20), warm=max(args.warmup, 5))
    sel_times, selection = offline_selection(api, torch, workloads, run, spec, reps=20)

    st = run.stages

    def step():
        st["cpo_layer"]()
        st["cps_layer"]()
        st["im2col_f32"]()
        api.select_layer_algo(sel_times["im2col"], sel_times["cpo"], sel_times["cps"], 0)
        api.select_layer_algo(sel_times["im2col"], sel_times["cpo"], sel_times["cps"], 1)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    # per-kernel durations (HIP events around every launch) and the dominant kernel of the step
    lens = run.lengths()
    ktimes = kernel_times(api, torch, run, reps=max(20, min(args.steps, 100)))
    overhead = event_pair_overhead_us(torch)
    kernels = []
    for stage in ("cpo_layer", "cps_layer", "im2col_f32"):
        for kname, rec in ktimes[stage].items():
            # launch duration = event-to-event time less what an empty event pair reads
            net = round(max(rec["avg_us"] - overhead, 0.1), 3)
            entry = {"stage": stage, "kernel": kname, "avg_us": net, "event_to_event_us": rec["avg_us"],
                     "launches": rec["launches"]}
            r = kernel_roofline(stage, kname, net, fig, spec, lens)
            if r:
                entry.update(r)
            kernels.append(entry)
    # the dominant kernel of the stage that `value` times
    dom = max((e for e in kernels if e["stage"] == "cpo_layer"), key=lambda e: e["avg_us"])
    roof = {k: (round(dom[k], 4) if isinstance(dom[k], float) else dom[k])
            for k in ("bound", "achieved", "peak", "unit", "frac") if k in dom}
    roof["kernel"] = dom["kernel"] + " (" + dom["stage"] + ")"
    roof["avg_launch_us"] = dom["avg_us"]
    roof["event_pair_overhead_us"] = round(overhead, 3)
    for k in ("algorithmic_bytes", "algorithmic_flops"):
        if k in dom:
            roof[k] = dom[k]
    roof["traffic"] = traffic_from_profiles(dom["kernel"])
    if args.config == 2:
        roof["rocprofv3_trace_avg_us"] = trace_avg_from_profiles(dom["kernel"])

    result = {
        "metric": "per-layer CPO/CPS conv time (us) + HBM GB/s, speedup and CR vs im2col",
        "value": round(times["cpo_layer"], 3),
        "unit": "us per layer (CPO encode + SpMV conv, one cpo_encode_conv call)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"configs[{args.config - 1}]: {spec.name} {spec.kh}x{spec.kw} s{spec.stride} p{spec.pad}, "
                               f"C={spec.C} H=W={spec.H} K={spec.K}, batch 1, "
                               f"{100 * (1 - row['density']):.1f}% zeros",
                   "step": "cpo_encode_conv+cps_encode_conv+im2col_conv(fp32)+select_layer_algo(2 modes)"},
        "layer": row,
        "selection": selection,
        "selection_times_us": {k: [round(x, 2) for x in v] for k, v in sel_times.items()},
        "roofline": roof,
        "kernels": kernels,
    }
    if not args.no_cold:
        # cold launches: a 1 GiB sweep between calls evicts inputs, streams and weights
        sweep = torch.zeros(256 << 20, dtype=torch.float32, device="cuda")
        cold = {k: round(_cold_time_us(torch, fn, 15, sweep), 2) for k, fn in st.items()}
        del sweep
        result["layer"]["cold_us"] = cold
        result["layer"]["cold_note"] = ("median of 15 single calls, each after a 1 GiB device-memory sweep, less "
                                        "an empty event pair; 'us' above are warm back-to-back averages")
    if args.batch > 0:
        result["batch_supplement"] = batch_supplement(api, torch, workloads, spec, args.batch, reps=10)
    if not args.no_chain:
        result["chain_supplement"] = [chain_supplement(api, torch, workloads, n, reps=10)
                                      for n in ([1, args.batch] if args.batch > 1 else [1])]
    if cpu is not None:
        result["cpu_baseline"] = cpu

    if args.all_layers or not args.no_chain:
        rows = []
        for s in workloads.all_layers() + workloads.line_layers():
            r, lrow, _, _ = measure_layer(api, torch, workloads, s, reps=50, warm=5)
            _, sel = offline_selection(api, torch, workloads, r, s, reps=10)
            lrow["selection"] = sel
            rows.append(lrow)
            del r
            torch.cuda.empty_cache()
            tail = ""
            if args.batch > 1:      # the same layer with --batch images per launch, per image
                bsup = batch_supplement(api, torch, workloads, s, args.batch, reps=5)
                pi = bsup["per_image_us"]
                lrow["batched"] = {"n_images": args.batch, "per_image_us": pi,
                                   "cpo_total_per_image_us": bsup["cpo_total_per_image_us"],
                                   "speedup_cpo_vs_im2col_f32": bsup["speedup_cpo_vs_im2col_f32"]}
                tail = (f" | x{args.batch}: cpo {bsup['cpo_total_per_image_us']:5.1f} im2col {pi['im2col_f32']:5.1f} "
                        f"bf16 {pi['im2col_bf16']:5.1f}")
                torch.cuda.empty_cache()
            print(f"{s.name:24s} nnz={lrow['nnz']:7d} enc {lrow['us']['cpo_encode']:6.1f} conv {lrow['us']['cpo_conv']:6.1f} "
                  f"cpo {lrow['cpo_total_us']:6.1f} cps {lrow['cps_total_us']:6.1f} im2col {lrow['us']['im2col_f32']:8.1f} bf16 {lrow['us']['im2col_bf16']:8.1f} "
                  f"CR {lrow['cr_cpo']:5.1f}/{lrow['cr_cps']:5.1f} pick {sel['favour_time']}/{sel['favour_space']}" + tail,
                  file=sys.stderr, flush=True)
        # every layer in the bench line itself: times, speed-ups, CR, the binding roofline's fraction per stage
        result["layers"] = [
            {"layer": r["layer"], "shape": r["shape"], "nnz": r["nnz"], "zeros": round(1.0 - r["density"], 4),
             "us": r["us"], "speedup_cpo_vs_im2col_f32": round(r["speedup_cpo_vs_im2col_f32"], 4),
             "speedup_cps_vs_im2col_f32": round(r["speedup_cps_vs_im2col_f32"], 4),
             "time_saving_cpo": round(1.0 - r["cpo_total_us"] / r["us"]["im2col_f32"], 4),
             "time_saving_cps": round(1.0 - r["cps_total_us"] / r["us"]["im2col_f32"], 4),
             "time_saving_cpo_batched": (round(1.0 - r["batched"]["cpo_total_per_image_us"] /
                                               r["batched"]["per_image_us"]["im2col_f32"], 4) if r.get("batched") else None),
             "cr_cpo": round(r["cr_cpo"], 3), "cr_cps": round(r["cr_cps"], 3),
             "roofline_frac": {k: [v["bound"], round(v["frac"], 5)] for k, v in r["roofline"].items()
                               if k in ("cpo_encode", "cpo_conv", "cps_conv", "im2col_f32", "im2col_bf16")},
             "selection": r["selection"], "batched": r.get("batched")}
            for r in rows]
        cfg5 = [r for r in rows if r["layer"].startswith("cfg5")]
        result["config5_end_to_end_us"] = {
            "all_im2col_f32": round(sum(r["us"]["im2col_f32"] for r in cfg5), 1),
            "hybrid_favour_time": round(sum(r["cpo_total_us"] if r["selection"]["favour_time"] == "cpo"
                                            else r["us"]["im2col_f32"] for r in cfg5), 1),
            "hybrid_favour_space": round(sum(r["cps_total_us"] if r["selection"]["favour_space"] == "cps"
                                             else r["us"]["im2col_f32"] for r in cfg5), 1),
            "layers_cpo_selected": sum(r["selection"]["favour_time"] == "cpo" for r in cfg5),
            "layers_cps_selected": sum(r["selection"]["favour_space"] == "cps" for r in cfg5),
        }
        if args.batch > 1:
            per = [(r["batched"]["cpo_total_per_image_us"], r["batched"]["per_image_us"]["im2col_f32"]) for r in cfg5]
            result["config5_end_to_end_us"]["batched"] = {
                "n_images": args.batch,
                "all_im2col_f32_per_image": round(sum(i for _, i in per), 1),
                "all_cpo_per_image": round(sum(c for c, _ in per), 1),
                "hybrid_per_image": round(sum(min(c, i) for c, i in per), 1),
                "layers_cpo_faster": sum(c < i for c, i in per),
            }
        line = [r for r in rows if r["layer"].startswith("line.")]
        result["line_layers_us"] = {
            "layers": len(line),
            "all_im2col_f32": round(sum(r["us"]["im2col_f32"] for r in line), 1),
            "all_cpo": round(sum(r["cpo_total_us"] for r in line), 1),
        }
        if args.batch > 1:
            per = [(r["batched"]["cpo_total_per_image_us"], r["batched"]["per_image_us"]["im2col_f32"]) for r in line]
            result["line_layers_us"]["batched"] = {
                "n_images": args.batch,
                "all_im2col_f32_per_image": round(sum(i for _, i in per), 1),
                "all_cpo_per_image": round(sum(c for c, _ in per), 1),
                "layers_cpo_faster": sum(c < i for c, i in per),
            }
    if args.detail_json:
        try:
            os.makedirs(os.path.dirname(os.path.abspath(args.detail_json)), exist_ok=True)
            with open(args.detail_json, "w") as f:
                json.dump(result, f, indent=1)
        except OSError as exc:
            print(f"bench.py: could not write {args.detail_json}: {exc}", file=sys.stderr)
    print(json.dumps(compact_line(result), separators=(",", ":")))


if __name__ == "__main__":
    main()
