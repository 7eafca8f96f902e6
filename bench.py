#!/usr/bin/env python3
"""Benchmark of the pattern-sparse 3x3 convolution path on one MI355X.

Default run: the nine distinct VGG-16 3x3 layers at batch 64, fp16 storage with fp32 accumulation, 8-pattern library,
connectivity keep 0.28 (the centre point of the throughput sweep), inputs resident in HBM.  A step is one pass over
the nine layers (nine pconv_conv3x3 launches, weights packed once); K steps are timed after W warm-up steps.
Prints ONE JSON line: effective GMAC/s over non-zero weights, per-layer rows, the roofline position of the dominant
kernel, the dense baseline of this library, the CPU oracle timed on the host cores of the same box, and short
measurements of the other configurations (batch-1 layer, batch-1 VGG-16 chain, ResNet-50 shapes at batch 32).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-extras]
    python bench.py --config1                                                  the batch-1 fp32 layer alone
    python bench.py --peaks                                                    measured peaks of this chip
    python bench.py --layers vgg_n1|resnet_n32|vgg_n64 [--K 8] [--keep 0.28]   per-layer table (stderr) + JSON line
    python bench.py --tune                                                     every tiling variant on the workload
    python bench.py --chain [--graph]            the 13 conv layers of VGG-16 at batch 1 (+ ReLU, max-pools) as one unit
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_VECTOR_TFLOPS = 157.3    # MI355X published fp32 vector peak (256 CUs x 2.4 GHz x 256 flop/clk/CU)
PEAK_FP16_MFMA_TFLOPS = 2500.0     # MI355X published dense fp16 matrix-core peak
PEAK_HBM_GBS = 8000.0              # MI355X published HBM3E bandwidth


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_bytes(spec, n_kept: int) -> int:
    """Bytes the method itself must move once: activations in, outputs out, four weights and a 16-bit channel
    index per kept kernel, group pointers, bias."""
    b = 2 if spec.dtype == "f16" else 4
    return (b * (spec.N * spec.C * spec.H * spec.W + spec.N * spec.F * spec.Ho * spec.Wo + 4 * n_kept)
            + 2 * n_kept + 4 * (spec.F * spec.K + 1) + 4 * spec.F)


def effective_macs(spec, n_kept: int) -> int:
    return spec.N * spec.Ho * spec.Wo * 4 * n_kept


class DeviceLayer:
    def __init__(self, spec, batch_from_one_image=False):
        import torch
        import paper_2001_07710_amd as pc
        from workloads import layers as L
        self.spec, self.pc, self.torch = spec, pc, torch
        self.w = L.gen_weights(spec)
        self.lib = spec.library()
        w32 = self.w.astype(np.float32)
        t0 = time.perf_counter()
        self.pid = L.gen_uniform_pattern_ids(spec) if spec.assign == "uniform" else pc.assign_patterns(w32, self.lib)
        t1 = time.perf_counter()
        self.mask = (L.gen_bernoulli_mask(spec) if spec.conn == "bernoulli"
                     else pc.select_connectivity(w32, self.lib, self.pid, spec.keep))
        t2 = time.perf_counter()
        self.packed = pc.pack(self.w, self.lib, self.pid, self.mask)
        t3 = time.perf_counter()
        self.host_ms = {"assign_ms": (t1 - t0) * 1e3, "select_ms": (t2 - t1) * 1e3, "pack_ms": (t3 - t2) * 1e3}
        self.n_kept = self.packed.n_kept
        self.bias = L.gen_bias(spec)
        if batch_from_one_image and spec.N > 1:
            # big batches: four seeded images repeated (values do not steer the kernel's control flow)
            base = L.gen_activations(spec, images=[0, 1, 2, 3][: min(4, spec.N)])
            reps = (spec.N + base.shape[0] - 1) // base.shape[0]
            self.x = np.concatenate([base] * reps, axis=0)[: spec.N]
        else:
            self.x = L.gen_activations(spec)
        self.dx = torch.from_numpy(self.x).cuda()
        self.db = torch.from_numpy(self.bias).cuda()
        tdt = torch.float16 if spec.dtype == "f16" else torch.float32
        self.dy = torch.empty((spec.N, spec.F, spec.Ho, spec.Wo), dtype=tdt, device="cuda")
        self.dtype_code = pc.F16 if spec.dtype == "f16" else pc.F32

    def launch(self, stream, x=None, **tuning):
        s = self.spec
        flags = self.pc.FLAG_RELU if s.relu else 0
        dx = self.dx if x is None else x
        if tuning:
            self.pc.conv3x3_tuned(dx, self.dy, self.packed, self.db, s.N, s.H, s.W, s.stride, s.pad, flags, stream,
                                  **tuning)
        else:
            self.pc.conv3x3(dx, self.dy, self.packed, self.db, s.N, s.H, s.W, s.stride, s.pad, flags, stream)

    def launch_dense(self, stream, dw):
        s = self.spec
        self.pc.dense_conv3x3(self.dx, self.dy, dw, self.db, self.dtype_code, s.N, s.C, s.F, s.H, s.W, s.stride, s.pad,
                              self.pc.FLAG_RELU if s.relu else 0, stream)


def library_dense_ms(torch, layer, dw, steps: int = 20):
    """The same dense convolution (masked weights, explicit zeros) by the vendor library that PyTorch-ROCm calls
    (MIOpen), in the layer's storage type: the dense reference a user would otherwise run.  Not part of the product."""
    s = layer.spec
    F = torch.nn.functional
    x4 = layer.dx.view(s.N, s.C, s.H, s.W)
    b = layer.db.to(dw.dtype)
    try:
        fn = lambda: F.conv2d(x4, dw, b, stride=s.stride, padding=s.pad)
        return time_launches(torch, fn, steps, 3)[1]
    except Exception as e:          # the library may not support a shape or type; the bench goes on without it
        log(f"library dense convolution skipped: {e}")
        return None


def time_launches(torch, fn, steps: int, warmup: int):
    """(wall ms per step, HIP-event ms per step) for `steps` launches after `warmup` untimed ones."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    return (t1 - t0) * 1e3 / steps, e0.elapsed_time(e1) / steps


def cpu_baseline(spec, layer, budget_s: float = 12.0):
    """The oracle as it stands, timed on the host cores, on the same layer (one image for batched workloads)."""
    import oracle
    x = layer.x[:1]
    wm = oracle.mask_weights(layer.w, layer.pid, layer.mask, layer.lib)
    oracle.conv3x3(x, wm, layer.bias, spec.stride, spec.pad, spec.relu)   # warm the pages
    runs, t0 = 0, time.perf_counter()
    while True:
        oracle.conv3x3(x, wm, layer.bias, spec.stride, spec.pad, spec.relu)
        runs += 1
        el = time.perf_counter() - t0
        if el > budget_s:
            break
    macs = spec.Ho * spec.Wo * 4 * layer.n_kept
    return {"value": macs * runs / el / 1e9, "unit": "effective GMAC/s", "cores": oracle.threads(), "kind": "oracle",
            "sample": f"{runs} runs of one image of the workload layer ({macs / 1e6:.1f} effective MMAC each), "
                      f"{el:.1f} s of wall time"}


def read_traffic(path: str):
    """HBM bytes per launch from the committed rocprofv3 counter summary, if there is one."""
    try:
        with open(path) as fh:
            for line in fh:
                if line.startswith("traffic_bytes_per_launch"):
                    return float(line.split()[1])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config1", action="store_true", help="time the batch-1 fp32 layer of config 1 alone")
    ap.add_argument("--peaks", action="store_true", help="measured peaks of this chip (copy, fp32 FMA, LDS, MFMA)")
    ap.add_argument("--no-extras", action="store_true", help="default run without the other configurations")
    ap.add_argument("--admm", action="store_true",
                    help="the selection-variable steps of the pruning framework over all kernels of VGG-16")
    ap.add_argument("--backward", action="store_true",
                    help="backward pass of the nine VGG-16 shapes at batch 64: masked weight gradient and input gradient")
    ap.add_argument("--conv1x1", action="store_true",
                    help="the 1x1 convolutions of ResNet-50's bottlenecks at batch 32, grouped into 3x3 patterns")
    ap.add_argument("--nhwc", action="store_true",
                    help="the nine VGG-16 shapes at batch 64 with channel-minor activations and outputs (PCONV_FLAG_NHWC)")
    ap.add_argument("--clustered", action="store_true",
                    help="VGG-16 shapes with clustered connectivity: filters in their own order against similarity order")
    ap.add_argument("--layers", default="")
    ap.add_argument("--K", type=int, default=8)
    ap.add_argument("--keep", type=float, default=0.28)
    ap.add_argument("--tune", nargs="?", const="all", default=None, choices=["all", "quad"],
                    help="with --layers: also time the explicit tilings (quad: only the four-column kernel's)")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--only", default="", help="with --layers: only the layer of this name")
    ap.add_argument("--kernel", default="auto", choices=["auto", "tiled", "quad"],
                    help="with --layers: the kernel the per-layer timing uses (auto: the library's choice)")
    ap.add_argument("--chain", action="store_true")
    ap.add_argument("--graph", action="store_true", help="with --chain: replay the chain as one HIP graph")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU; --gpus must be 1 (batches shard over GPUs without any exchange)")

    import torch
    import paper_2001_07710_amd as pc
    from workloads import layers as L
    pc.ensure_built()
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; there is no CPU fallback")
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream().cuda_stream

    if args.peaks:
        return peaks_bench(args, torch)
    if args.admm:
        return admm_bench(args, torch, pc, L)
    if args.nhwc and not args.conv1x1:
        return nhwc_bench(args, torch, pc, L)
    if args.clustered:
        return clustered_bench(args, torch, pc, L)
    if args.backward:
        return backward_bench(args, torch, pc, L)
    if args.conv1x1:
        return conv1x1_bench(args, torch, pc, L)
    if args.chain:
        return chain_bench(args, torch, pc, L)
    if args.layers:
        return layer_table(args, torch, pc, L, stream)
    if not args.config1 and not args.tune:
        return sweep_bench(args, torch, pc, L, stream)
    if args.steps == 50 and args.warmup == 5:
        args.steps, args.warmup = 2000, 200

    spec = L.config1()
    layer = DeviceLayer(spec)
    macs = effective_macs(spec, layer.n_kept)
    abytes = algorithmic_bytes(spec, layer.n_kept)

    if args.tune:
        for r, nf, wv, cpw, nbuf in [(7, 1, 8, 4, 1), (7, 1, 16, 2, 1), (7, 2, 8, 2, 1), (7, 2, 16, 2, 1),
                                     (7, 1, 16, 1, 2), (7, 2, 16, 1, 2), (7, 1, 8, 2, 2), (7, 2, 8, 2, 2)]:
            for ks in (1, 2, 4, 8):
                t = dict(kernel=pc.KERNEL_TILED, rows=r, filters_per_wave=nf, waves=wv, channels_per_wave=cpw,
                         channel_splits=ks, buffers=nbuf)
                try:
                    _, ev = time_launches(torch, lambda: layer.launch(stream, **t), 300, 30)
                except pc.PconvError:
                    continue
                log(f"tune rows={r} nf={nf} waves={wv} cpw={cpw} buffers={nbuf} splits={ks}: {ev * 1e3:8.2f} us  "
                    f"{macs / ev / 1e6:9.1f} GMAC/s")

    # one plain device-to-device copy of known size (256 MiB read + 256 MiB written): the calibration point for the
    # FETCH_SIZE / WRITE_SIZE counters when this command runs under rocprofv3 --pmc
    calib = torch.zeros(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
    calib2 = torch.empty_like(calib)
    calib2.copy_(calib)
    torch.cuda.synchronize()
    del calib, calib2

    wall_ms, ev_ms = time_launches(torch, lambda: layer.launch(stream), args.steps, args.warmup)

    # launch floor: an (almost) empty launch of the same entry point, for context at batch 1
    tiny = L.shrink(spec, C=1, F=1, H=3, W=3)
    tl = DeviceLayer(tiny)
    _, floor_ms = time_launches(torch, lambda: tl.launch(stream), 500, 50)

    dense = None
    if not args.no_dense:
        wm = np.where(layer.mask[:, :, None, None] != 0, layer.w, 0).astype(layer.w.dtype)
        dw = torch.from_numpy(np.ascontiguousarray(wm)).cuda()
        _, dense_ms = time_launches(torch, lambda: layer.launch_dense(stream, dw), 20, 3)
        dense = {"ms": dense_ms, "dense_GMACs": spec.N * spec.Ho * spec.Wo * 9 * spec.C * spec.F / dense_ms / 1e6,
                 "kind": "plain HIP direct convolution, fp32 vector ALU",
                 "library_ms": library_dense_ms(torch, layer, dw),
                 "library_kind": "MIOpen through torch.nn.functional.conv2d, same masked weights"}

    flops = 2.0 * macs
    achieved = flops / (ev_ms * 1e-3) / 1e12
    out = {
        "metric": "effective GMAC/s (nonzero weights), VGG-16 conv3_x-shaped 3x3 layer",
        "value": macs / (wall_ms * 1e-3) / 1e9,
        "unit": "GMAC/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": wall_ms,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "configs[1]: 3x3 conv 256->256 @56x56, batch 1, fp32, K=8 patterns, keep 0.28 "
                               f"({layer.n_kept} kept kernels)", "step": "one pconv_conv3x3 launch (weights packed once)"},
        "roofline": {"bound": "alu", "achieved": achieved, "peak": PEAK_FP32_VECTOR_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_FP32_VECTOR_TFLOPS,
                     "traffic": read_traffic(os.path.join(ROOT, "profiles", "tiled_kernel_config1_hbm_counters.txt")),
                     "kernel": "tiled_kernel", "kernel_ms": ev_ms, "flops_per_launch": flops,
                     "algorithmic_bytes_per_launch": abytes, "algorithmic_GBs": abytes / (ev_ms * 1e-3) / 1e9,
                     "hbm_frac_of_8TBs": abytes / (ev_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                     "note": "measured on this chip: plain v_fmac_f32 reaches 140-150 TFLOP/s with two or more waves per SIMD"},
        "launch_floor_ms": floor_ms,
        "host_once": layer.host_ms,
        "dense_baseline": dense,
    }
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(spec, layer)
    print(json.dumps(out), flush=True)



def executed_macs(spec, layer) -> int:
    """Multiply-adds the kernel that runs the layer really executes: the kept weights for the vector kernels, the
    dense contraction over the taps that occur for the matrix-core kernel (which multiplies the explicit zeros)."""
    if spec.dtype == "f16":
        taps = 0
        for j in np.unique(layer.pid[layer.mask != 0]):
            taps |= int(layer.lib[j])
        return spec.N * spec.Ho * spec.Wo * bin(taps).count("1") * spec.C * spec.F
    return effective_macs(spec, layer.n_kept)


def time_per_layer(torch, layers, stream, steps, warmup, dense_w=None):
    """One step = one launch of every layer, in order.  Returns (wall ms per step, [event ms per step and layer])."""
    def step(record=None):
        for i, l in enumerate(layers):
            if record:
                record[i][0].record()
            if dense_w is None:
                l.launch(stream)
            else:
                l.launch_dense(stream, dense_w[i])
            if record:
                record[i][1].record()
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    evs = [[[torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)] for _ in layers]
           for _ in range(steps)]
    t0 = time.perf_counter()
    for k in range(steps):
        step(evs[k])
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3 / steps
    per = [sum(evs[k][i][0].elapsed_time(evs[k][i][1]) for k in range(steps)) / steps for i in range(len(layers))]
    return wall, per


def short_sweep(torch, specs, stream, steps=30):
    """Total and per-layer times of a list of layers (one launch each per step)."""
    layers = [DeviceLayer(s, batch_from_one_image=True) for s in specs]
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < 0.05:
        for l in layers:
            l.launch(stream)
        torch.cuda.synchronize()
    _, per = time_per_layer(torch, layers, stream, steps, 3)
    macs = [effective_macs(s, l.n_kept) for s, l in zip(specs, layers)]
    out = {"total_us": sum(per) * 1e3, "eff_GMACs": sum(macs) / sum(per) / 1e6,
           "frac_of_fp32_vector_peak": 2 * sum(macs) / (sum(per) * 1e-3) / 1e12 / PEAK_FP32_VECTOR_TFLOPS,
           "layers": {s.name: round(t * 1e3, 2) for s, t in zip(specs, per)}}
    for l in layers:
        l.packed.free()
    return out


def sweep_bench(args, torch, pc, L, stream):
    """The default run: the nine VGG-16 shapes at batch 64 (config 4 at K = 8, keep 0.28)."""
    specs = L.config4(args.K, args.keep, 64)
    layers = [DeviceLayer(s, batch_from_one_image=True) for s in specs]
    eff = [effective_macs(s, l.n_kept) for s, l in zip(specs, layers)]
    exe = [executed_macs(s, l) for s, l in zip(specs, layers)]
    ab = [algorithmic_bytes(s, l.n_kept) for s, l in zip(specs, layers)]
    # plain device-to-device copy of known size: the calibration point of FETCH_SIZE / WRITE_SIZE under rocprofv3 --pmc
    calib = torch.zeros(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
    calib2 = torch.empty_like(calib)
    calib2.copy_(calib)
    torch.cuda.synchronize()
    del calib, calib2
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < 0.1:              # bring the clocks up
        for l in layers:
            l.launch(stream)
        torch.cuda.synchronize()
    wall_ms, per = time_per_layer(torch, layers, stream, args.steps, args.warmup)

    dense_per = None
    if not args.no_dense:
        dws = []
        for l in layers:
            wm = np.where(l.mask[:, :, None, None] != 0, l.w, 0).astype(l.w.dtype)
            dws.append(torch.from_numpy(np.ascontiguousarray(wm)).cuda())
        _, dense_per = time_per_layer(torch, layers, stream, max(3, args.steps // 5), 2, dense_w=dws)

    names = {pc.KERNEL_TILED: "tiled_kernel", pc.KERNEL_QUAD: "quad_kernel", pc.KERNEL_GENERIC: "generic_kernel",
             pc.KERNEL_MFMA: "mfma_conv_kernel"}
    rows, on_mfma = [], []
    for i, (s, l) in enumerate(zip(specs, layers)):
        t = per[i] * 1e-3
        family, shape = pc.conv3x3_choice(l.packed, s.N, s.H, s.W, s.stride, s.pad)
        hbm_frac = ab[i] / t / 1e9 / PEAK_HBM_GBS
        if family == pc.KERNEL_MFMA:
            on_mfma.append(i)
            unit, unit_frac, done = "mfma", 2 * exe[i] / t / 1e12 / PEAK_FP16_MFMA_TFLOPS, exe[i]
        else:           # the vector kernels multiply the kept weights only
            unit, unit_frac, done = "alu", 2 * eff[i] / t / 1e12 / PEAK_FP32_VECTOR_TFLOPS, eff[i]
        rows.append({"layer": s.name, "C": s.C, "F": s.F, "H": s.H, "n_kept": l.n_kept, "us": per[i] * 1e3,
                     "kernel": names.get(family, str(family)) + (f" (tile shape {shape})" if shape else ""),
                     "eff_GMACs": eff[i] / t / 1e9, "executed_TFLOPs": 2 * done / t / 1e12,
                     "bound": "hbm" if hbm_frac > unit_frac else unit, "frac": max(unit_frac, hbm_frac),
                     unit + "_frac": unit_frac, "alg_GBs": ab[i] / t / 1e9, "hbm_frac": hbm_frac,
                     "eff_frac_of_fp32_vector_peak": 2 * eff[i] / t / 1e12 / PEAK_FP32_VECTOR_TFLOPS,
                     "dense_us": None if dense_per is None else dense_per[i] * 1e3})
    tot_t = sum(per) * 1e-3
    # the dominant kernel: mfma_conv_kernel.  Its launches fall under two roofs: the matrix cores for most layers, HBM
    # for the two 224 x 224 layers (64 filters or fewer: little arithmetic per byte).  `roofline` is that of the
    # launches the matrix cores bind; the others are in `roofline_hbm_bound_launches`; the time-weighted fraction of
    # the binding roof over all of the kernel's launches is in `roofline` as well.  Per launch = the mean over them.
    all_mfma = on_mfma if on_mfma else list(range(len(specs)))
    dom = [i for i in all_mfma if rows[i]["bound"] != "hbm"] or all_mfma
    hbm_bound = [i for i in all_mfma if i not in dom]
    exe_flops = 2.0 * sum(exe[i] for i in dom) / len(dom)
    alg_flops = 2.0 * sum(eff[i] for i in dom) / len(dom)
    kernel_ms = sum(per[i] for i in dom) / len(dom)
    achieved = exe_flops / (kernel_ms * 1e-3) / 1e12
    traffic = read_traffic(os.path.join(ROOT, "profiles", "mfma_conv_kernel_vgg16_batch64_hbm_counters.txt"))
    out = {
        "metric": "effective GMAC/s (nonzero weights), VGG-16 3x3 layers",
        "value": sum(eff) / (wall_ms * 1e-3) / 1e9,
        "unit": "GMAC/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": wall_ms,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16 storage, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": f"configs[4] at K={args.K}, keep {args.keep}: the nine distinct VGG-16 3x3 conv shapes, "
                               "batch 64, fp16 storage (conv1_1 at keep 1.0)",
                   "step": "one pconv_conv3x3 launch per layer, nine launches (weights packed once)"},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": PEAK_FP16_MFMA_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_FP16_MFMA_TFLOPS, "traffic": traffic,
                     "traffic_source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this command, mean over all launches of the kernel "
                                       "(compare all_launches_of_the_kernel.algorithmic_bytes_per_launch), "
                                       "profiles/mfma_conv_kernel_vgg16_batch64_hbm_counters.txt",
                     "kernel": "mfma_conv_kernel", "kernel_ms": kernel_ms, "launches_per_step": len(dom),
                     "layers": [specs[i].name for i in dom],
                     "flops_per_launch": exe_flops, "algorithmic_flops_per_launch": alg_flops,
                     "algorithmic_achieved_TFLOPs": alg_flops / (kernel_ms * 1e-3) / 1e12,
                     "algorithmic_frac_of_fp32_vector_peak": alg_flops / (kernel_ms * 1e-3) / 1e12 / PEAK_FP32_VECTOR_TFLOPS,
                     "algorithmic_bytes_per_launch": sum(ab[i] for i in dom) / len(dom),
                     "algorithmic_GBs": sum(ab[i] for i in dom) / (kernel_ms * 1e-3 * len(dom)) / 1e9,
                     "hbm_frac_of_8TBs": sum(ab[i] for i in dom) / (kernel_ms * 1e-3 * len(dom)) / 1e9 / PEAK_HBM_GBS,
                     # per launch the time that the roof which binds it allows (executed flops at the MFMA peak or
                     # algorithmic bytes at the HBM peak, whichever is longer), summed, over the measured time
                     "frac_of_binding_roof_time_weighted":
                         sum(max(2.0 * exe[i] / (PEAK_FP16_MFMA_TFLOPS * 1e12), ab[i] / (PEAK_HBM_GBS * 1e9)) for i in all_mfma)
                         / (sum(per[i] for i in all_mfma) * 1e-3),
                     "all_launches_of_the_kernel": {
                         "layers": [specs[i].name for i in all_mfma],
                         "algorithmic_bytes_per_launch": sum(ab[i] for i in all_mfma) / len(all_mfma),
                         "executed_TFLOPs": 2.0 * sum(exe[i] for i in all_mfma) / (sum(per[i] for i in all_mfma) * 1e-3) / 1e12},
                     "note": "the kernel runs the layer as a dense fp16 contraction over its masked weights on the "
                             "matrix cores; 'achieved' counts the multiply-adds it executes (every tap that occurs, "
                             "explicit zeros included) against the published dense fp16 MFMA peak; the method's own "
                             "flops (non-zero weights only) are 'algorithmic_*', with the fp32 vector peak, which "
                             "bounds any kernel that skips the zeros, beside them"},
        "roofline_hbm_bound_launches": None if not hbm_bound else {
            "bound": "hbm", "kernel": "mfma_conv_kernel", "layers": [specs[i].name for i in hbm_bound],
            "achieved": sum(ab[i] for i in hbm_bound) / (sum(per[i] for i in hbm_bound) * 1e-3) / 1e9,
            "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "frac": sum(ab[i] for i in hbm_bound) / (sum(per[i] for i in hbm_bound) * 1e-3) / 1e9 / PEAK_HBM_GBS,
            "bytes_per_launch": sum(ab[i] for i in hbm_bound) / len(hbm_bound),
            "kernel_ms": sum(per[i] for i in hbm_bound) / len(hbm_bound)},
        "layers": rows,
        "dense_baseline": None if dense_per is None else {
            "total_us": sum(dense_per) * 1e3, "kind": "pconv_dense_conv3x3: the same matrix-core kernel on all nine "
            "taps of the masked dense tensor, including the re-ordering of the weights on every call"},
        "host_once": {k: sum(l.host_ms[k] for l in layers) for k in layers[0].host_ms},
    }
    if not args.no_cpu:
        big = max(range(len(specs)), key=lambda i: per[i])
        out["cpu_baseline"] = cpu_baseline(specs[big], layers[big])
        out["cpu_baseline"]["sample"] = f"layer {specs[big].name}: " + out["cpu_baseline"]["sample"]
    for l in layers:
        l.packed.free()
    del layers
    torch.cuda.empty_cache()
    if not args.no_extras:
        c1 = L.config1()
        l1 = DeviceLayer(c1)
        _, ev = time_launches(torch, lambda: l1.launch(stream), 500, 50)
        m1 = effective_macs(c1, l1.n_kept)
        out["other_configs"] = {
            "config1_batch1_fp32": {"us": ev * 1e3, "eff_GMACs": m1 / ev / 1e6,
                                    "frac_of_fp32_vector_peak": 2 * m1 / (ev * 1e-3) / 1e12 / PEAK_FP32_VECTOR_TFLOPS},
            "config2_vgg16_batch1_fp32_per_layer_sum": short_sweep(torch, L.config2(), stream, 50),
            "config3_resnet50_batch32_fp16": short_sweep(torch, L.config3(32), stream, 50),
            "config3_resnet50_batch1_fp16": short_sweep(torch, L.config3(1), stream, 50),
        }
        l1.packed.free()
        # what the other modes of this file time, in brief (10 launches each, no host baseline): the backward pass,
        # 1x1 layers grouped into 3x3 patterns, filter re-ordering on clustered connectivity, the channel-minor layout
        import copy
        b = copy.copy(args)
        b.steps, b.warmup, b.only, b.keep = 10, 2, "", 0.28
        out["beyond_the_forward_pass"] = {
            "backward_vgg16_batch64_fp16": backward_bench(b, torch, pc, L, brief=True),
            "clustered_connectivity_vgg16_batch64_fp16": clustered_bench(b, torch, pc, L, brief=True),
            "channel_minor_layout_vgg16_batch64_fp16": nhwc_bench(b, torch, pc, L, brief=True),
        }
        b.keep = 0.3
        b.nhwc = False
        out["beyond_the_forward_pass"]["conv1x1_resnet50_batch32_fp16"] = conv1x1_bench(b, torch, pc, L, brief=True)
        b.nhwc = True
        out["beyond_the_forward_pass"]["conv1x1_resnet50_batch32_fp16_channel_minor"] = conv1x1_bench(b, torch, pc, L, brief=True)
    print(json.dumps(out), flush=True)


def peaks_bench(args, torch):
    """Register-, LDS- and memory-only kernels of libpconv_peaks.so: what the chip delivers, next to the published
    peaks the roofline fractions are quoted against."""
    import paper_2001_07710_amd as pc
    out = {"peaks": pc.peaks(),
           "published": {"hbm_GBs": PEAK_HBM_GBS, "fp32_vector_TFLOPs": PEAK_FP32_VECTOR_TFLOPS,
                         "fp16_mfma_TFLOPs": PEAK_FP16_MFMA_TFLOPS},
           "note": "copy_GBs counts bytes read plus bytes written; per-clock figures use the nominal engine clock"}
    print(json.dumps(out), flush=True)


def admm_bench(args, torch, pc, L):
    """The per-kernel steps of the pruning framework (include/pconv_admm.h) over every 3x3 kernel of VGG-16's 13
    conv layers (1,634,496 kernels), K patterns: one proximal step with multiplier update, the argmax projection, and
    the pattern assignment from fp32 weights.  Each is one launch, bound by HBM: algorithmic bytes = what it must read
    and write once (proximal: four float vectors of K per kernel; argmax: K floats in, one int out; assignment: nine
    floats in, one int out)."""
    import oracle
    from workloads import rng
    n, K = sum(sp.C * sp.F for sp in L.config2()), args.K
    z = (rng.normal(rng.stream_seed(93, 1, K), n * K).reshape(n, K) * 0.5 + 1.0 / K).astype(np.float32)
    mu = (rng.normal(rng.stream_seed(93, 2, K), n * K).reshape(n, K) * 0.1).astype(np.float32)
    w = rng.normal(rng.stream_seed(93, 3), n * 9).reshape(n, 9).astype(np.float32)
    lib = np.array(L.drawn_library(4, K), dtype=np.uint16)
    # four copies of every buffer, used in turn: 0.6 GB per proximal launch set, so that a launch finds none of its
    # data in the 256 MB memory-side cache and the rate is that of HBM
    R = 4
    dz = [torch.from_numpy(z).cuda() for _ in range(R)]
    dmu = [torch.from_numpy(mu).cuda() for _ in range(R)]
    dw = [torch.from_numpy(w).cuda() for _ in range(R)]
    du, dm2 = [torch.empty_like(dz[0]) for _ in range(R)], [torch.empty_like(dz[0]) for _ in range(R)]
    pid = [torch.empty(n, dtype=torch.int32, device="cuda") for _ in range(R)]
    st = torch.cuda.current_stream().cuda_stream
    turn = [0]

    def rot():
        turn[0] = (turn[0] + 1) % R
        return turn[0]

    def prox():
        r = rot()
        pc.admm_proximal(dz[r], dmu[r], 0.75, n, K, du[r], dm2[r], st)

    def binz():
        r = rot()
        pc.admm_binarize(dz[r], n, K, pid[r], st)

    def asg():
        r = rot()
        pc.assign_patterns_device(dw[r], pc.F32, n, lib, pid[r], st)

    # connectivity selection on the largest VGG-16 layer (512 x 512 kernels): norms, a stable radix sort, marks
    nl = 512 * 512
    need = pc.select_connectivity_device_workspace(nl)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    dmask = torch.empty(nl, dtype=torch.uint8, device="cuda")
    pc.assign_patterns_device(dw[0], pc.F32, nl, lib, pid[0], st)

    def sel():
        pc.select_connectivity_device(dw[0], pc.F32, nl, lib, pid[0], 0.28, dmask, ws, need, st)

    rows = {}
    for name, fn, nbytes in (("proximal", prox, 16 * K * n), ("binarize", binz, (4 * K + 4) * n),
                             ("assign_patterns_device", asg, 40 * n),
                             ("select_connectivity_device_512x512", sel, 41 * nl)):
        _, ev = time_launches(torch, fn, args.steps, args.warmup)
        cnt = nl if name.startswith("select") else n
        rows[name] = {"us": ev * 1e3, "algorithmic_bytes": nbytes, "GBs": nbytes / (ev * 1e-3) / 1e9,
                      "frac_of_8TBs": nbytes / (ev * 1e-3) / 1e9 / PEAK_HBM_GBS, "kernels_per_s": cnt / (ev * 1e-3)}
    # the oracle on a bounded sample of the same vectors, timed on the host
    m = 20000
    t0 = time.perf_counter()
    oracle.proximal_step(z[:m], mu[:m], 0.75)
    el = time.perf_counter() - t0
    out = {"metric": "kernels/s, proximal step with multiplier update", "value": rows["proximal"]["kernels_per_s"],
           "unit": "kernels/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": rows["proximal"]["us"] * 1e-3, "higher_is_better": True, "dtype": "f32 storage, f64 arithmetic",
           "data": "synthetic", "config": {"workload": f"all {n} 3x3 kernels of VGG-16's 13 conv layers, K={K}"},
           "roofline": {"bound": "hbm", "achieved": rows["proximal"]["GBs"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                        "frac": rows["proximal"]["frac_of_8TBs"], "traffic": None, "kernel": "proximal_kernel"},
           "steps_table": rows,
           "cpu_baseline": {"value": m / el, "unit": "kernels/s", "cores": 1, "kind": "oracle",
                            "sample": f"the first {m} kernels, {el:.1f} s"}}
    print(json.dumps(out), flush=True)


def nhwc_bench(args, torch, pc, L, brief=False):
    """The default workload (config 4 at K, keep from the command line: nine VGG-16 shapes, batch 64, fp16) with
    channel-minor activations and outputs, x [N][H][W][C] and y [N][Ho][Wo][F] (PCONV_FLAG_NHWC), next to the same
    layers in the channel-major layout of the benchmark configuration.  The three-channel first layer is run with its
    input padded to eight channels (the added channels' kernels are removed, so the layer is the same)."""
    import oracle
    st = torch.cuda.current_stream().cuda_stream
    rows, t_nhwc, t_nchw, macs, flops = [], 0.0, 0.0, 0.0, 0.0
    sample = None
    for spec in L.config4(args.K, args.keep, 64):
        if args.only and spec.name != args.only:
            continue
        w, lib = L.gen_weights(spec), spec.library()
        w32 = w.astype(np.float32)
        pid = pc.assign_patterns(w32, lib)
        mask = pc.select_connectivity(w32, lib, pid, spec.keep)
        base = L.gen_activations(spec, images=[0, 1, 2, 3])
        C = spec.C
        if C % 8:
            C8 = (C + 7) // 8 * 8
            w = np.concatenate([w, np.zeros((spec.F, C8 - C, 3, 3), w.dtype)], axis=1)
            pid = np.concatenate([pid, np.zeros((spec.F, C8 - C), pid.dtype)], axis=1)
            mask = np.concatenate([mask, np.zeros((spec.F, C8 - C), mask.dtype)], axis=1)
            base = np.concatenate([base, np.zeros((4, C8 - C, spec.H, spec.W), base.dtype)], axis=1)
            C = C8
        p = pc.pack(w, lib, pid, mask)
        x = np.concatenate([base] * (spec.N // 4), axis=0)
        d_nchw = torch.from_numpy(x).cuda()
        d_nhwc = d_nchw.permute(0, 2, 3, 1).contiguous()
        db = torch.from_numpy(L.gen_bias(spec)).cuda()
        dy = torch.empty(spec.N * spec.F * spec.Ho * spec.Wo, dtype=torch.float16, device="cuda")
        f1 = lambda: pc.conv3x3(d_nhwc, dy, p, db, spec.N, spec.H, spec.W, 1, 1, pc.FLAG_RELU | pc.FLAG_NHWC, st)
        f0 = lambda: pc.conv3x3(d_nchw, dy, p, db, spec.N, spec.H, spec.W, 1, 1, pc.FLAG_RELU, st)
        _, ms1 = time_launches(torch, f1, args.steps, args.warmup)
        _, ms0 = time_launches(torch, f0, args.steps, args.warmup)
        nk = int(mask.sum())
        ex = 2.0 * spec.N * spec.Ho * spec.Wo * 9 * ((spec.F + 63) // 64 * 64) * ((C + 15) // 16 * 16)
        nbytes = 2.0 * spec.N * (C * spec.H * spec.W + spec.F * spec.Ho * spec.Wo)
        row = {"layer": spec.name, "C": C, "F": spec.F, "H": spec.H, "n_kept": nk, "nhwc_us": ms1 * 1e3,
               "nchw_us": ms0 * 1e3, "executed_TFLOPs": ex / ms1 / 1e9, "mfma_frac": ex / ms1 / 1e9 / PEAK_FP16_MFMA_TFLOPS,
               "alg_GBs": nbytes / ms1 / 1e6, "hbm_frac": nbytes / ms1 / 1e6 / PEAK_HBM_GBS,
               "eff_GMACs": effective_macs(spec, nk) / ms1 / 1e6}
        rows.append(row)
        log(json.dumps(row))
        t_nhwc += ms1
        t_nchw += ms0
        macs += effective_macs(spec, nk)
        if spec.C >= 64:
            flops += ex
        if spec.name == "conv1_2":
            sample = (spec, base[:1], oracle.mask_weights(w, pid, mask, lib), L.gen_bias(spec))
        p.free()
        del d_nchw, d_nhwc, dy
        torch.cuda.empty_cache()
    out = {"metric": "effective GMAC/s (nonzero weights), VGG-16 3x3 layers, channel-minor layout", "value": macs / t_nhwc / 1e6,
           "unit": "GMAC/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": t_nhwc,
           "higher_is_better": True, "dtype": "f16 storage, f32 accumulate", "data": "synthetic",
           "config": {"workload": f"configs[4] at K={args.K}, keep {args.keep}, batch 64, x and y channel-minor (NHWC)"},
           "nchw_ms_per_step": t_nchw, "layers": rows}
    if brief:
        return {"us": t_nhwc * 1e3, "channel_major_us_same_run": t_nchw * 1e3, "eff_GMACs": macs / t_nhwc / 1e6,
                "layers": {r["layer"]: round(r["nhwc_us"], 1) for r in rows}}
    if sample is not None:
        spec, x1, wm, b = sample
        t0, runs = time.perf_counter(), 0
        while time.perf_counter() - t0 < 8.0:
            oracle.conv3x3(x1, wm, b, 1, 1, True)
            runs += 1
        el = (time.perf_counter() - t0) / runs
        out["cpu_baseline"] = {"value": effective_macs(spec, int((wm != 0).any(axis=(2, 3)).sum())) / spec.N / el / 1e9,
                               "unit": "effective GMAC/s", "cores": oracle.threads(), "kind": "oracle",
                               "sample": f"{runs} runs of one image of {spec.name}, {el * runs:.1f} s"}
    print(json.dumps(out), flush=True)


def clustered_bench(args, torch, pc, L, brief=False):
    """What filter re-ordering buys on the matrix cores (pconv_filter_similarity_order + the channel lists of the
    matrix-core kernel).  Config 4's shapes from conv2_2 on at batch 64, fp16, K and keep from the command line, but
    with weights whose connectivity is clustered as in a trained, pruned model: filters in groups of 128 scattered
    over the indices, each group keeping its kernels inside its own subset of 1.25 * keep of the input channels
    (workloads.gen_clustered_weights; pattern assignment and top-k selection are the method's own steps, as always).
    Each layer is timed packed in its own filter order and packed in similarity order."""
    import oracle
    st = torch.cuda.current_stream().cuda_stream
    rows, t_nat, t_ord, macs = [], 0.0, 0.0, 0.0
    sample = None
    for spec in L.config4(args.K, args.keep, 64):
        if spec.C < 128 or (args.only and spec.name != args.only):
            continue
        clusters = max(1, spec.F // 128)
        if clusters < 2:
            continue
        w, _ = L.gen_clustered_weights(spec, clusters, min(1.0, 1.25 * spec.keep))
        lib, w32 = spec.library(), None
        w32 = w.astype(np.float32)
        pid = pc.assign_patterns(w32, lib)
        mask = pc.select_connectivity(w32, lib, pid, spec.keep)
        t0 = time.perf_counter()
        order = pc.filter_similarity_order(mask, 128)
        order_ms = (time.perf_counter() - t0) * 1e3
        base = L.gen_activations(spec, images=[0, 1, 2, 3])
        dx = torch.from_numpy(np.concatenate([base] * (spec.N // 4), axis=0)).cuda()
        bias = L.gen_bias(spec)
        dy = torch.empty((spec.N, spec.F, spec.Ho, spec.Wo), dtype=torch.float16, device="cuda")
        row = {"layer": spec.name, "C": spec.C, "F": spec.F, "H": spec.H, "n_kept": int(mask.sum()), "order_ms": order_ms}
        for tag, o in (("own_order", np.arange(spec.F)), ("similarity_order", order)):
            p = pc.pack(w[o], lib, pid[o], mask[o])
            db = torch.from_numpy(bias[o]).cuda()
            fn = lambda: pc.conv3x3(dx, dy, p, db, spec.N, spec.H, spec.W, 1, 1, pc.FLAG_RELU, st)
            _, ms = time_launches(torch, fn, args.steps, args.warmup)
            listed, dense = pc.packed_mfma_blocks(p, 128)
            row[tag] = {"us": ms * 1e3, "blocks": listed, "of": dense,
                        "eff_GMACs": effective_macs(spec, int(mask.sum())) / ms / 1e6}
            p.free()
        t_nat += row["own_order"]["us"]
        t_ord += row["similarity_order"]["us"]
        macs += effective_macs(spec, int(mask.sum()))
        rows.append(row)
        log(json.dumps(row))
        if sample is None:
            sample = (spec, base[:1], oracle.mask_weights(w, pid, mask, lib), bias)
    if brief:
        return {"own_order_us": t_nat, "similarity_order_us": t_ord, "eff_GMACs_similarity_order": macs / t_ord / 1e3,
                "layers": {r["layer"]: {"own_order_us": round(r["own_order"]["us"], 1),
                                        "similarity_order_us": round(r["similarity_order"]["us"], 1),
                                        "blocks": [r["own_order"]["blocks"], r["similarity_order"]["blocks"], r["own_order"]["of"]]}
                           for r in rows}}
    spec, x1, wm, b = sample
    t0, runs = time.perf_counter(), 0
    while time.perf_counter() - t0 < 8.0:
        oracle.conv3x3(x1, wm, b, 1, 1, True)
        runs += 1
    el = (time.perf_counter() - t0) / runs
    out = {"metric": "effective GMAC/s (nonzero weights), VGG-16 3x3 layers with clustered connectivity, similarity order",
           "value": macs / t_ord / 1e3, "unit": "GMAC/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": t_ord * 1e-3, "higher_is_better": True, "dtype": "f16 storage, f32 accumulate",
           "data": "synthetic", "config": {"workload": f"configs[4] shapes with 128 or more channels, batch 64, K={args.K}, "
                                                       f"keep {args.keep}, clustered connectivity (groups of 128 filters)"},
           "own_order_us": t_nat, "similarity_order_us": t_ord, "speedup": t_nat / t_ord, "layers": rows,
           "cpu_baseline": {"value": effective_macs(spec, int((wm != 0).any(axis=(2, 3)).sum())) / spec.N / el / 1e9,
                            "unit": "effective GMAC/s", "cores": oracle.threads(), "kind": "oracle",
                            "sample": f"{runs} runs of one image of {spec.name}, {el * runs:.1f} s"}}
    print(json.dumps(out), flush=True)


def backward_bench(args, torch, pc, L, brief=False):
    """Backward pass (include/pconv_backward.h) of config 4's nine VGG-16 shapes at batch 64, fp16 storage, K and keep
    from the command line: per layer one masked weight gradient (grad_weight_kernel + gather) and one input gradient
    (the forward kernel on the transposed layer; the first layer has none to hand back).  The weight gradient is a
    dense contraction over the pixels on the matrix cores: executed flops = 2 * pixels * 9 * F' * C' with F', C'
    rounded up to the 64 x 64 tile, against the dense fp16 MFMA peak; algorithmic bytes = x and dy read once."""
    import oracle
    st = torch.cuda.current_stream().cuda_stream
    rows, tot_gw, tot_gi, flops_sum = [], 0.0, 0.0, 0.0
    worst = None
    for spec in L.config4(args.K, args.keep, 64):
        if args.only and spec.name != args.only:
            continue
        layer = DeviceLayer(spec, batch_from_one_image=True)
        g = np.random.default_rng(1000 + spec.idx).standard_normal((4, spec.F, spec.Ho, spec.Wo)).astype(np.float16)
        dy = torch.from_numpy(np.concatenate([g] * (spec.N // 4), axis=0)).cuda()
        nbytes = pc.conv3x3_grad_weight_workspace(layer.packed, spec.N, spec.H, spec.W)
        ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device="cuda")
        dw4 = torch.empty((layer.n_kept, 4), dtype=torch.float32, device="cuda")
        gw = lambda: pc.conv3x3_grad_weight(layer.dx, dy, layer.packed, dw4, spec.N, spec.H, spec.W, 1, 1, ws, nbytes, st)
        _, gw_ms = time_launches(torch, gw, args.steps, args.warmup)
        pix = spec.N * spec.H * spec.W
        f64, c64 = (spec.F + 63) // 64 * 64, (spec.C + 63) // 64 * 64
        flops = 2.0 * pix * 9 * f64 * c64
        row = {"layer": spec.name, "C": spec.C, "F": spec.F, "H": spec.H, "n_kept": layer.n_kept,
               "grad_weight_us": gw_ms * 1e3, "executed_TFLOPs": flops / gw_ms / 1e9,
               "mfma_frac": flops / gw_ms / 1e9 / PEAK_FP16_MFMA_TFLOPS,
               "alg_GBs": 2.0 * pix * (spec.C + spec.F) / gw_ms / 1e6,
               "eff_GMACs": pix * 4.0 * layer.n_kept / gw_ms / 1e6, "workspace_MB": nbytes / 1e6}
        if spec.C >= 16:
            t = pc.packed_transpose(layer.packed)
            dxg = torch.empty_like(layer.dx)
            gi = lambda: pc.conv3x3_grad_input(dy, dxg, t, spec.N, spec.H, spec.W, st)
            _, gi_ms = time_launches(torch, gi, args.steps, args.warmup)
            row["grad_input_us"] = gi_ms * 1e3
            tot_gi += gi_ms
            t.free()
        tot_gw += gw_ms
        flops_sum += flops
        if worst is None or gw_ms > worst[1]:
            worst = (spec, gw_ms, layer.x[:1].copy(), g[:1].copy())
        rows.append(row)
        log(json.dumps(row))
        layer.packed.free()
        del layer, dy, ws, dw4
        torch.cuda.empty_cache()
    if brief:
        return {"grad_weight_us": tot_gw * 1e3, "grad_weight_executed_TFLOPs": flops_sum / tot_gw / 1e9,
                "grad_weight_frac_of_fp16_mfma_peak": flops_sum / tot_gw / 1e9 / PEAK_FP16_MFMA_TFLOPS,
                "grad_input_us": tot_gi * 1e3,
                "layers": {r["layer"]: [round(r["grad_weight_us"], 1), round(r.get("grad_input_us", 0.0), 1)] for r in rows}}
    # the oracle on one image of the slowest layer, timed on the host
    spec, _, x1, g1 = worst
    t0, runs = time.perf_counter(), 0
    while time.perf_counter() - t0 < 10.0:
        oracle.conv3x3_grad_weight(x1, g1, 1, 1)
        runs += 1
    el = (time.perf_counter() - t0) / runs
    out = {"metric": "executed TFLOP/s, masked weight gradient of VGG-16 3x3 layers", "value": flops_sum / tot_gw / 1e9,
           "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": tot_gw,
           "higher_is_better": True, "dtype": "f16 storage, f32 accumulate", "data": "synthetic",
           "config": {"workload": f"backward pass of configs[4] at K={args.K}, keep {args.keep}: nine VGG-16 shapes, batch 64"},
           "roofline": {"bound": "mfma", "achieved": flops_sum / tot_gw / 1e9, "peak": PEAK_FP16_MFMA_TFLOPS,
                        "unit": "TFLOP/s", "frac": flops_sum / tot_gw / 1e9 / PEAK_FP16_MFMA_TFLOPS, "traffic": None,
                        "kernel": "grad_weight_kernel"},
           "grad_input_total_us": tot_gi * 1e3, "layers": rows,
           "cpu_baseline": {"value": 2.0 * spec.H * spec.W * 9 * spec.F * spec.C / el / 1e12, "unit": "TFLOP/s",
                            "cores": oracle.threads(), "kind": "oracle",
                            "sample": f"{runs} runs of the dense weight gradient of one image of {spec.name}, {el * runs:.1f} s"}}
    print(json.dumps(out), flush=True)


def conv1x1_bench(args, torch, pc, L, brief=False):
    """The 1x1 convolutions of ResNet-50's bottleneck blocks (reduce and expand of each stage) at batch 32, fp16
    storage, grouped into 3x3 patterns (include/pconv_backward.h): K patterns, keep from the command line.  These
    layers move their activations once for C*F*4/9*keep multiply-adds per pixel: the roofline is HBM, algorithmic
    bytes = input + output + kept weights."""
    import oracle
    st = torch.cuda.current_stream().cuda_stream
    shapes = [("s1_reduce", 256, 64, 56), ("s1_expand", 64, 256, 56), ("s2_reduce", 512, 128, 28),
              ("s2_expand", 128, 512, 28), ("s3_reduce", 1024, 256, 14), ("s3_expand", 256, 1024, 14),
              ("s4_reduce", 2048, 512, 7), ("s4_expand", 512, 2048, 7)]
    N = 32
    lib = np.array(L.drawn_library(3, args.K), dtype=np.uint16)
    rows, tot_ms, tot_bytes, sample = [], 0.0, 0.0, None
    for i, (name, C, F, H) in enumerate(shapes):
        rng = np.random.default_rng(500 + i)
        G = (C + 8) // 9
        w = (rng.standard_normal((F, C)) * np.sqrt(2.0 / C)).astype(np.float16)
        b = (rng.standard_normal(F) * 0.1).astype(np.float32)
        x1 = np.maximum(rng.standard_normal((4, C, H, H)), 0).astype(np.float16)
        pid = rng.integers(0, args.K, size=(F, G)).astype(np.uint8)
        mask = (rng.random((F, G)) < args.keep).astype(np.uint8)
        p = pc.pack_1x1(w, lib, pid, mask)
        dx = torch.from_numpy(np.concatenate([x1] * (N // 4), axis=0)).cuda()
        db = torch.from_numpy(b).cuda()
        dy = torch.empty((N, F, H, H), dtype=torch.float16, device="cuda")
        fl = pc.FLAG_RELU
        if getattr(args, "nhwc", False):        # (--conv1x1 --nhwc: the same layers on channel-minor tensors)
            dx = dx.permute(0, 2, 3, 1).contiguous()
            dy = torch.empty((N, H, H, F), dtype=torch.float16, device="cuda")
            fl |= pc.FLAG_NHWC
        fn = lambda: pc.conv1x1(dx, dy, p, db, N, H, H, 1, fl, st)
        _, ms = time_launches(torch, fn, args.steps, args.warmup)
        nbytes = 2.0 * N * H * H * (C + F) + 2.0 * p.n_kept
        row = {"layer": name, "C": C, "F": F, "H": H, "n_kept_weights": p.n_kept, "us": ms * 1e3,
               "alg_GBs": nbytes / ms / 1e6, "hbm_frac": nbytes / ms / 1e6 / PEAK_HBM_GBS,
               "eff_GMACs": N * H * H * float(p.n_kept) / ms / 1e6,
               "executed_TFLOPs": 2.0 * N * H * H * ((C + 15) // 16 * 16) * F / ms / 1e9}
        rows.append(row)
        log(json.dumps(row))
        tot_ms += ms
        tot_bytes += nbytes
        if i == 0:
            sample = (name, x1[:1], w, pid, mask, b)
        p.free()
    if brief:
        return {"us": tot_ms * 1e3, "alg_GBs": tot_bytes / tot_ms / 1e6, "frac_of_8TBs": tot_bytes / tot_ms / 1e6 / PEAK_HBM_GBS,
                "layers": {r["layer"]: round(r["us"], 1) for r in rows}}
    name, x1, w, pid, mask, b = sample
    t0, runs = time.perf_counter(), 0
    while time.perf_counter() - t0 < 5.0:
        oracle.conv1x1(x1, w, pid, mask, lib, b, 1, True)
        runs += 1
    el = (time.perf_counter() - t0) / runs
    kept = int(oracle.group_mask_1x1(pid, mask, lib, *w.shape).sum())
    out = {"metric": "algorithmic GB/s, ResNet-50 1x1 layers grouped into 3x3 patterns", "value": tot_bytes / tot_ms / 1e6,
           "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": tot_ms,
           "higher_is_better": True, "dtype": "f16 storage, f32 accumulate", "data": "synthetic",
           "config": {"workload": f"eight 1x1 layers of ResNet-50's bottlenecks, batch 32, K={args.K}, keep {args.keep}"
                                  + (", x and y channel-minor (NHWC)" if getattr(args, "nhwc", False) else "")},
           "roofline": {"bound": "hbm", "achieved": tot_bytes / tot_ms / 1e6, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                        "frac": tot_bytes / tot_ms / 1e6 / PEAK_HBM_GBS, "traffic": None, "kernel": "mfma_conv_kernel"},
           "layers": rows,
           "cpu_baseline": {"value": x1.shape[2] * x1.shape[3] * kept / el / 1e9, "unit": "effective GMAC/s", "cores": 1,
                            "kind": "oracle", "sample": f"{runs} runs of one image of {name}, {el * runs:.1f} s"}}
    print(json.dumps(out), flush=True)


def chain_bench(args, torch, pc, L):
    """The 13 conv layers of VGG-16 at batch 1 (config 2: fused ReLU, 2x2 max-pool after each stage) launched back to
    back as one unit: eager launches, or one HIP graph replayed.  At this size the chain is bound by per-kernel
    start-up and launch gaps, which is what this mode shows."""
    specs = L.config2()
    layers = [DeviceLayer(s) for s in specs]
    pooled = [torch.empty((s.N, s.F, s.Ho // 2, s.Wo // 2), dtype=torch.float32, device="cuda") if s.pool_after else None
              for s in specs]
    macs = sum(effective_macs(s, l.n_kept) for s, l in zip(specs, layers))

    def run(stream):
        x = layers[0].dx
        for s, l, pl in zip(specs, layers, pooled):
            l.launch(stream, x=x)
            x = l.dy
            if pl is not None:
                pc.maxpool2x2(l.dy, pl, l.dtype_code, s.N, s.F, s.Ho, s.Wo, stream)
                x = pl

    side = torch.cuda.Stream()          # graph capture needs a non-default stream; default priority
    with torch.cuda.stream(side):
        st = side.cuda_stream
        for _ in range(3):
            run(st)                     # also makes the layers allocate their workspaces, outside any capture
        side.synchronize()
        fn = lambda: run(st)
        if args.graph:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                run(st)
            fn = g.replay
        _, ev = time_launches(torch, fn, 300, 30)
    out = {"chain": "VGG-16, 13 conv layers + ReLU + 5 max-pools, batch 1, fp32 (config 2)", "mode": "graph" if args.graph
           else "eager", "us_per_chain": ev * 1e3, "eff_GMACs": macs / ev / 1e6, "kernels_per_chain": 13 + sum(
               1 for q in pooled if q is not None)}
    log(" ".join(f"{k}={v:.4g}" if isinstance(v, float) else f"{k}={v}" for k, v in out.items()))
    print(json.dumps(out))


def layer_table(args, torch, pc, L, stream):
    """Per-layer timings for one of the layer sweeps (written to stderr as a table, and one JSON line)."""
    if args.layers == "vgg_n1":
        specs = L.config2()
    elif args.layers == "resnet_n32":
        specs = L.config3(32)
    elif args.layers == "resnet_n1":
        specs = L.config3(1)
    elif args.layers == "vgg_n64":
        specs = L.config4(args.K, args.keep, 64)
    else:
        sys.exit("unknown --layers")
    rows, tot_macs, tot_ms = [], 0, 0.0
    for spec in specs:
        if args.only and spec.name != args.only:
            continue
        layer = DeviceLayer(spec, batch_from_one_image=True)
        macs = effective_macs(spec, layer.n_kept)
        steps = max(10, min(1000, int(2e10 / max(macs, 1))))
        forced = {"auto": {}, "tiled": dict(kernel=pc.KERNEL_TILED), "quad": dict(kernel=pc.KERNEL_QUAD)}[args.kernel]
        t0 = time.perf_counter()
        while time.perf_counter() - t0 < 0.05:      # bring the clocks up before the first timed launch of a layer
            for _ in range(4):
                layer.launch(stream, **forced)
            torch.cuda.synchronize()
        _, ev = time_launches(torch, lambda: layer.launch(stream, **forced), steps, max(3, steps // 10))
        best = None
        if args.tune:
            for nf, wv, cpw, nbuf in [] if args.tune == "quad" else [(1, 8, 4, 1), (1, 16, 2, 1), (2, 16, 2, 1), (2, 16, 1, 1), (2, 8, 2, 1),
                                      (1, 8, 2, 1), (1, 16, 1, 2), (2, 16, 1, 2), (1, 8, 2, 2), (2, 8, 2, 2)]:
                for ks in (1, 2, 4, 8, 16):
                    t = dict(kernel=pc.KERNEL_TILED, rows=7, filters_per_wave=nf, waves=wv, channels_per_wave=cpw,
                             channel_splits=ks, buffers=nbuf)
                    try:
                        _, tv = time_launches(torch, lambda: layer.launch(stream, **t), max(5, steps // 4), 2)
                    except pc.PconvError:
                        continue
                    if best is None or tv < best[0]:
                        best = (tv, nf, wv, cpw, ks, nbuf)
            for nf, order, ks, walk in [(nf, o, ks, wk) for nf in (1, 2) for o in (1, 2) for ks in (1, 2, 4, 8, 16)
                                        for wk in ((1, 2) if ks == 1 else (1,))]:
                # the kernel with four columns per lane; walk 1: one workgroup per tile, 2: workgroups walk over the tiles
                wv = 16
                t = dict(kernel=pc.KERNEL_QUAD, filters_per_wave=nf, channel_order=order, channel_splits=ks, slot_walk=walk)
                try:
                    _, tv = time_launches(torch, lambda: layer.launch(stream, **t), max(5, steps // 4), 2)
                except pc.PconvError:
                    continue
                log(f"  quad nf{nf} order{order} ks{ks} walk{walk}: {tv * 1e3:.1f} us")
                if best is None or tv < best[0]:
                    best = (tv, nf, wv, 1, ks, "quad" + ("", "plain", "balanced")[order] + ("", "", "walk")[walk])
        ab = algorithmic_bytes(spec, layer.n_kept)
        row = {"layer": spec.name, "C": spec.C, "F": spec.F, "H": spec.H, "N": spec.N, "stride": spec.stride,
               "dtype": spec.dtype, "keep": spec.keep, "K": spec.K, "n_kept": layer.n_kept, "us": ev * 1e3,
               "eff_GMACs": macs / ev / 1e6, "alu_frac": 2 * macs / (ev * 1e-3) / 1e12 / PEAK_FP32_VECTOR_TFLOPS,
               "alg_GBs": ab / (ev * 1e-3) / 1e9, "hbm_frac": ab / (ev * 1e-3) / 1e9 / PEAK_HBM_GBS}
        if best:
            row["best_us"], row["best_cfg"] = best[0] * 1e3, f"nf{best[1]}w{best[2]}c{best[3]}s{best[4]}b{best[5]}"
        if not args.no_dense:
            wm = np.where(layer.mask[:, :, None, None] != 0, layer.w, 0).astype(layer.w.dtype)
            dw = torch.from_numpy(np.ascontiguousarray(wm)).cuda()
            _, dms = time_launches(torch, lambda: layer.launch_dense(stream, dw), 3, 1)
            row["dense_us"] = dms * 1e3
            lib_ms = library_dense_ms(torch, layer, dw, 5)
            if lib_ms is not None:
                row["miopen_us"] = lib_ms * 1e3
        rows.append(row)
        tot_macs += macs
        tot_ms += ev
        log(" ".join(f"{k}={v:.4g}" if isinstance(v, float) else f"{k}={v}" for k, v in row.items()))
        layer.packed.free()
        del layer
        torch.cuda.empty_cache()
    print(json.dumps({"layers": args.layers, "K": args.K, "keep": args.keep, "total_eff_GMACs": tot_macs / tot_ms / 1e6,
                      "total_ms": tot_ms, "rows": rows}), flush=True)


if __name__ == "__main__":
    main()
