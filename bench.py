#!/usr/bin/env python3
"""Benchmark of the hot path on ONE MI355X.

A "step" is one pass of the whole hot path over one batch of the headline workload:
the single conv block of the benchmark configuration -- Conv3d 3x3x3 (64 -> 64 channels) on a
1 x 128^3 NDHWC bf16 volume with InstanceNorm + ReLU, forward, data-gradient and weight-gradient:

    z, stats = conv3d_fwd(x, W)            (matrix-core implicit GEMM, statistics in the epilogue)
    y        = inorm_relu(z, stats)
    dz       = inorm_relu_bwd(dy, z, stats)
    dx       = conv3d_dgrad(dz, W)
    dW       = conv3d_wgrad(x, dz)         (fp32)

Inputs are synthetic (N(0,1) activations and upstream gradient, Kaiming-normal weights), resident
in HBM before the timed region.  Prints ONE JSON line.  Its top level is that headline workload
(value, roofline, cpu_baseline); the object `configs` in the same line carries the other benchmark
configurations -- the tiny fp32 net, the encoder partition at 192^3, the whole-net training step, the
large-input inference in one pass and as sliding windows -- each timed through its network entry
point, with the roofline of its dominant kernel (event-timed through the layer entry point on that
layer's shape) and the CPU oracle timed on a stated small sample of the same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline] [--no-configs]
    python bench.py --workload unet_train ...      (one network workload alone, e.g. under a profiler)
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--size", type=int, default=128, help="cubic volume side (default: the benchmark's 128)")
    ap.add_argument("--channels", type=int, default=64)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="headline workload only: skip the `configs` object")
    ap.add_argument("--config-steps", type=int, default=10, help="timed steps of each workload in `configs`")
    ap.add_argument("--config-warmup", type=int, default=5)
    ap.add_argument("--workload", default="block", choices=["block", "unet_train", "unet_infer", "sliding", "stage", "tiny", "unet_train_b64", "unet_train_b128",
                             "unet_infer_whole", "unet_train_step", "unet_train_pipeline", "se_block", "seunet_train"],
                    help="block (default): the headline conv block (config 2). The others time the network-level "
                         "entry points on the remaining configurations and report voxels/s.")
    ap.add_argument("--micro-batches", type=int, default=2, help="unet_train_pipeline: micro-batches the 2 samples are split into")
    ap.add_argument("--cut", type=int, default=2, help="unet_train_pipeline: last encoder block of partition 0")
    ap.add_argument("--graph", action="store_true",
                    help="tiny: replay the ~60 small kernels as one captured HIP graph (measured: no faster than launching "
                         "them one by one, the step is bound by the chain of small kernels on the GPU, not by the launches)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy (a kernel of known traffic) so that a counter "
                         "profile of this run can scale FETCH_SIZE / WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus N with N > 1 is not supported "
              "(the path has no collectives; it would shard data-parallel over samples, as pipeline stages "
              "after any block, or as spatial slabs with a one-voxel halo exchange).", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import lamp_synth as S
    import paper_2006_12575_amd as L

    L.lib()  # fails loudly when the HIP library is missing
    if args.workload != "block":
        out = net_bench(args.workload, args, torch, np, S, L, max(1, args.steps), max(1, args.warmup),
                        cpu=not args.no_cpu_baseline)
        print(json.dumps(out))
        return
    dev = "cuda:0"
    bf, f32 = torch.bfloat16, torch.float32
    N, D, C = 1, args.size, args.channels
    rx, rw, rg = S.streams(1002, 3)

    def normal_dev(rng, shape):
        # generated in slabs to keep host memory modest
        t = torch.empty(shape, dtype=bf, device=dev)
        for d in range(shape[1]):
            t[:, d] = torch.from_numpy(S.normal(rng, (shape[0],) + tuple(shape[2:]))).to(bf).to(dev)
        return t

    x = normal_dev(rx, (N, D, D, D, C))
    dy = normal_dev(rg, (N, D, D, D, C))
    w = torch.from_numpy(S.kaiming_conv(rw, C, C)).to(bf).to(dev)
    z = torch.empty_like(x)
    y = torch.empty_like(x)
    dz = torch.empty_like(x)
    dx = torch.empty_like(x)
    dw = torch.empty(w.shape, dtype=f32, device=dev)
    stats = torch.empty((N, C, 2), dtype=f32, device=dev)
    xd, zd = L.desc(x), L.desc(z)
    import ctypes
    need = max(L.lib().lamp_conv3d_fwd_workspace_bytes(ctypes.byref(xd), ctypes.byref(zd), 1),
               L.lib().lamp_conv3d_dgrad_workspace_bytes(ctypes.byref(zd), ctypes.byref(xd)),
               L.lib().lamp_conv3d_wgrad_workspace_bytes(ctypes.byref(xd), ctypes.byref(zd)),
               L.lib().lamp_inorm_relu_bwd_workspace_bytes(ctypes.byref(zd)))
    ws = torch.empty(int(need) + 256, dtype=torch.uint8, device=dev)

    def step():
        L.lamp_conv3d_fwd(x, w, z, stats_out=stats, ws=ws)
        L.lamp_inorm_relu(z, y, stats, stats_given=True, ws=ws)
        L.lamp_inorm_relu_bwd(dy, z, stats, dz, ws=ws)
        L.lamp_conv3d_dgrad(dz, w, dx, ws=ws)
        L.lamp_conv3d_wgrad(x, dz, dw, ws=ws)

    # the inputs were generated on the host while the GPU idled: let its clocks settle (untimed), then the W warm-up steps
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < 0.1:
        step()
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps

    V = N * D * D * D
    flops_conv = 2.0 * V * 27 * C * C
    tflops = 3 * flops_conv / dt / 1e12

    # ---- roofline of the dominant kernel: the forward implicit-GEMM conv, timed alone with
    # events on the launch stream (torch's current stream is the one the binding launches on)
    def timed(fn, reps):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e-3

    reps = max(3, args.steps)
    parts = {
        "conv3d_fwd": timed(lambda: L.lamp_conv3d_fwd(x, w, z, stats_out=stats, ws=ws), reps),
        "inorm_relu": timed(lambda: L.lamp_inorm_relu(z, y, stats, stats_given=True, ws=ws), reps),
        "inorm_relu_bwd": timed(lambda: L.lamp_inorm_relu_bwd(dy, z, stats, dz, ws=ws), reps),
        "conv3d_dgrad": timed(lambda: L.lamp_conv3d_dgrad(dz, w, dx, ws=ws), reps),
        "conv3d_wgrad": timed(lambda: L.lamp_conv3d_wgrad(x, dz, dw, ws=ws), reps),
    }
    # The dominant kernel is the implicit-GEMM conv kernel, launched twice per step (forward with the
    # statistics epilogue, data gradient without): its average launch duration is the mean of the two
    # event-timed entry points (each bracket also holds the 221 KB weight repack and, for the forward,
    # the statistics finalize: ~2 % of the time).
    t_conv = 0.5 * (parts["conv3d_fwd"] + parts["conv3d_dgrad"])
    roof = {"bound": "mfma", "kernel": f"conv3d_igemm_kernel<2, 8> (implicit GEMM {C}->{C}, {D}^3; fwd and dgrad launches)",
            "achieved": flops_conv / t_conv / 1e12, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
            "frac": flops_conv / t_conv / 1e12 / PEAK_BF16_TFLOPS, "traffic": None}
    # HBM bytes per launch of that kernel: a counter profile (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a
    # copy of known size) cannot be taken inside this run; the figure is the one of the committed profile, with
    # the commit it was taken at, and is null when that profile does not describe the workload.
    if args.size == 128 and args.channels == 64:
        roof["traffic"], roof["traffic_source"] = profile_traffic()
    # The rate of the bare matrix-core instruction stream on this chip, with zero and with normally
    # distributed operands (switching power sets the clock): context for `frac`, whose peak stays the
    # published one.
    roof.update(mfma_probe())
    if args.copy_calibration:
        a = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()

    out = {
        "metric": "Conv3d fwd+bwd TFLOP/s (% MFMA peak); whole-U-Net voxels/sec at 1 GPU",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"conv block fwd+dgrad+wgrad, bf16/fp32-acc, N=1 C={C}->{C} {D}^3 NDHWC, "
                               f"3x3x3 pad 1 + InstanceNorm + ReLU", "voxels": V,
                   "flop_per_step": 3 * flops_conv},
        "pct_mfma_peak": 100.0 * tflops / PEAK_BF16_TFLOPS,
        "voxels_per_s": V / dt,
        "ms_parts": {k: v * 1e3 for k, v in parts.items()},
        "tflops_parts": {k: flops_conv / parts[k] / 1e12 for k in ("conv3d_fwd", "conv3d_dgrad", "conv3d_wgrad")},
        "gbs_parts": {"inorm_relu": 2 * V * C * 2 / parts["inorm_relu"] / 1e9,
                      "inorm_relu_bwd": (2 * 2 + 3) * V * C * 2 / 2 / parts["inorm_relu_bwd"] / 1e9},
        "roofline": roof,
    }

    if not args.no_cpu_baseline:
        import oracle as O
        s = 48  # bounded sample: the same block on a 48^3 sub-volume, all 64 channels
        xs = x[:, :s, :s, :s, :].to(torch.float64).cpu().numpy()
        dys = dy[:, :s, :s, :s, :].to(torch.float64).cpu().numpy()
        w64 = w.to(torch.float64).cpu().numpy()
        O.num_threads()
        t0 = time.perf_counter()
        zz = O.conv3d_fwd(xs, w64)
        yy, _ = O.inorm_relu(zz)
        dzz, _, _ = O.inorm_relu_bwd(dys, zz)
        O.conv3d_dgrad(dzz, w64)
        O.conv3d_wgrad(xs, dzz)
        tc = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": 3 * 2.0 * s ** 3 * 27 * C * C / tc / 1e12, "unit": "TFLOP/s",
                               "cores": O.num_threads(), "kind": "oracle", "cpu_model": cpu_model(),
                               "sample": f"same conv block (fwd+dgrad+wgrad, fp64) on a {s}^3 sub-volume of the "
                                         f"workload, C={C}, {tc:.1f} s; a rate measured on that bounded sample, not a "
                                         f"full-size run (which would take about {tc * (D / s) ** 3:.0f} s)"}
    if not args.no_configs and args.size == 128 and args.channels == 64:
        del x, dy, z, y, dz, dx, ws
        torch.cuda.empty_cache()
        out["configs"] = {}
        for key, wl in (("cfg1_tiny", "tiny"), ("cfg3_stage", "stage"), ("cfg4_unet_train", "unet_train"),
                        ("cfg5a_unet_infer", "unet_infer"), ("cfg5b_sliding", "sliding")):
            e = net_bench(wl, args, torch, np, S, L, max(1, args.config_steps), max(1, args.config_warmup),
                          cpu=not args.no_cpu_baseline)
            out["configs"][key] = {k: e[k] for k in ("config", "ms_per_step", "steps", "warmup", "dtype", "voxels_per_s", "tflops",
                                                      "pct_mfma_peak", "roofline", "cpu_baseline", "final_loss") if k in e}
            torch.cuda.empty_cache()
        a, b = out["configs"]["cfg5a_unet_infer"], out["configs"]["cfg5b_sliding"]
        out["configs"]["cfg5_sliding_over_one_pass_time_ratio"] = b["ms_per_step"] / a["ms_per_step"]
    print(json.dumps(out))


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def profile_traffic():
    """(bytes per launch, source) of the headline conv kernel from the committed counter profile, or (None, reason)."""
    f = os.path.join(ROOT, "profiles", "conv3d_igemm_c64_128_traffic_bytes.txt")
    try:
        txt = open(f).read()
        val = float(txt.split()[0])
        src = " ".join(txt.split()[1:])
        return val, f"profiles/{os.path.basename(f)}: {src}"
    except Exception as e:  # noqa: BLE001
        return None, f"no usable profile ({e})"


def mfma_probe():
    """Bench-only helper library (its own .so: it allocates and synchronises, which the product ABI never does)."""
    import ctypes
    path = os.path.join(ROOT, "paper_2006_12575_amd", "benchprobe", "liblamp_benchprobe.so")
    out = {}
    try:
        lib = ctypes.CDLL(path)
        lib.benchprobe_mfma_rate.restype = ctypes.c_int
        lib.benchprobe_mfma_rate.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(ctypes.c_float)]
        for pat, name in ((0, "mfma_rate_zero_operands_tflops"), (1, "mfma_rate_normal_operands_tflops")):
            v = ctypes.c_float(0.0)
            if lib.benchprobe_mfma_rate(pat, 4000, ctypes.byref(v)) == 0:
                out[name] = float(v.value)
    except OSError:
        pass
    return out


def unet_flops(levels, base, in_ch, classes, n, d, h, w):
    """Model FLOPs of one forward pass (2 per multiply-add; padding taps counted)."""
    fl = 0.0
    ch = [base << l for l in range(levels)]
    vox = [n * (d >> l) * (h >> l) * (w >> l) for l in range(levels)]
    for l in range(levels):
        cin = in_ch if l == 0 else ch[l - 1]
        fl += 2.0 * vox[l] * 27 * (cin * ch[l] + ch[l] * ch[l])
    for l in range(levels - 2, -1, -1):
        fl += 2.0 * vox[l + 1] * 8 * ch[l + 1] * ch[l]              # transposed conv
        fl += 2.0 * vox[l] * 27 * (2 * ch[l] * ch[l] + ch[l] * ch[l])
    fl += 2.0 * vox[0] * ch[0] * classes
    return fl


def se_bench(args, torch, np, S, L):
    """InstanceNorm + ReLU + squeeze-and-excitation gate + residual, forward and backward, on the headline
    tensor (1 x size^3 x C, bf16).  Bandwidth-bound: the line carries an HBM roofline object."""
    dev, bf, f32 = "cuda:0", torch.bfloat16, torch.float32
    D, C = args.size, args.channels
    Cr = max(1, C // 16)
    gen = torch.Generator(dev).manual_seed(1009)
    shape = (1, D, D, D, C)
    z = (torch.randn(shape, device=dev, generator=gen) * 1.7 + 0.4).to(bf)
    dy = torch.randn(shape, device=dev, generator=gen).to(bf)
    res = torch.randn(shape, device=dev, generator=gen).to(bf)
    w1 = torch.randn((Cr, C), device=dev, generator=gen) / C ** 0.5
    b1 = torch.full((Cr,), 0.3, device=dev)
    w2 = torch.randn((C, Cr), device=dev, generator=gen) / Cr ** 0.5
    b2 = torch.zeros(C, device=dev)
    stats = torch.empty((1, C, 2), dtype=f32, device=dev)
    y, dz = torch.empty_like(z), torch.empty_like(z)
    L.lamp_inorm_relu(z, y, stats)
    save = torch.empty((1, 4 * C + Cr), dtype=f32, device=dev)
    g = dict(dw1=torch.empty_like(w1), db1=torch.empty_like(b1), dw2=torch.empty_like(w2), db2=torch.empty_like(b2))
    import ctypes
    ws = torch.empty(int(L.lib().lamp_inorm_relu_se_workspace_bytes(ctypes.byref(L.desc(z)), Cr)), dtype=torch.uint8, device=dev)

    def run():
        L.lamp_inorm_relu_se(z, stats, w1, w2, y, save, b1=b1, b2=b2, residual=res, ws=ws)
        L.lamp_inorm_relu_se_bwd(dy, z, stats, w1, w2, save, dz, ws=ws, **g)
    steps, warm = max(1, args.steps), max(1, args.warmup)
    for _ in range(warm):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        run()
    torch.cuda.synchronize()
    dtm = (time.perf_counter() - t0) / steps
    tb = z.numel() * 2
    alg = 9 * tb   # forward: z twice, residual, y; backward: dy and z twice, dz
    V = D ** 3
    return ({
        "metric": "Conv3d fwd+bwd TFLOP/s (% MFMA peak); whole-U-Net voxels/sec at 1 GPU", "value": V / dtm, "unit": "voxels/s",
        "n_gpus": 1, "steps": steps, "warmup": warm, "ms_per_step": dtm * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"InstanceNorm+ReLU+squeeze-and-excitation (ratio 16)+residual, forward+backward, 1x{D}^3x{C}",
                   "voxels": V, "algorithmic_bytes_per_step": alg},
        "roofline": {"bound": "hbm", "achieved": alg / dtm / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": alg / dtm / 1e9 / PEAK_HBM_GBS, "traffic": None}})


def unet_ideal_bytes(levels, base, in_ch, classes, n, d, h, w, es):
    """Algorithmic HBM bytes of one forward pass with every elementwise step fused into a neighbour: each conv reads
    its input and writes its output once (es bytes per element), pooling reads the fine and writes the coarse tensor,
    the transposed conv reads coarse and writes fine, the head reads C_1 channels and writes fp32 logits."""
    ch = [base << l for l in range(levels)]
    vox = [n * (d >> l) * (h >> l) * (w >> l) for l in range(levels)]
    b = 0.0
    for l in range(levels):
        cin = in_ch if l == 0 else ch[l - 1]
        b += vox[l] * es * ((cin + ch[l]) + 2 * ch[l])
        if l + 1 < levels:
            b += es * ch[l] * (vox[l] + vox[l + 1])
    for l in range(levels - 2, -1, -1):
        b += es * (vox[l + 1] * ch[l + 1] + vox[l] * ch[l])
        b += vox[l] * es * ((2 * ch[l] + ch[l]) + 2 * ch[l])
    b += vox[0] * (es * ch[0] + 4 * classes)
    return b


def conv_layer_roofline(torch, S, L, n, d, h, w, ci, co, reps, seed):
    """Roofline object of the matrix-core conv kernel on one layer shape: lamp_conv3d_fwd (statistics in the epilogue)
    on seeded N(0,1) bf16 data, timed with events on the launch stream (torch's current stream, the one the binding
    launches on).  The bracket holds the kernel, the weight repack and the statistics finalize (a few microseconds)."""
    import ctypes
    dev, bf, f32 = "cuda:0", torch.bfloat16, torch.float32
    g = torch.Generator(dev).manual_seed(seed)
    x = torch.randn((n, d, h, w, ci), device=dev, generator=g, dtype=f32).to(bf)
    rw, = S.streams(seed, 1)
    wt = torch.from_numpy(S.kaiming_conv(rw, co, ci)).to(bf).to(dev)
    z = torch.empty((n, d, h, w, co), dtype=bf, device=dev)
    st = torch.empty((n, co, 2), dtype=f32, device=dev)
    xd, zd = L.desc(x), L.desc(z)
    ws = torch.empty(int(L.lib().lamp_conv3d_fwd_workspace_bytes(ctypes.byref(xd), ctypes.byref(zd), 1)) + 256,
                     dtype=torch.uint8, device=dev)
    run = lambda: L.lamp_conv3d_fwd(x, wt, z, stats_out=st, ws=ws)
    # warm-up until the clocks have settled: after a pause (input generation on the host) the first launches
    # run 10-15 % slower than the steady state
    t0 = time.perf_counter()
    for i in range(200):
        run()
        if i >= 10 and i % 5 == 0:
            torch.cuda.synchronize()
            if time.perf_counter() - t0 > 0.08:
                break
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        run()
    e1.record()
    torch.cuda.synchronize()
    t = e0.elapsed_time(e1) / reps * 1e-3
    fl = 2.0 * n * d * h * w * 27 * ci * co
    alg = 2.0 * n * d * h * w * (ci + co)
    return {"bound": "mfma", "kernel": f"conv3d_igemm_kernel, 3x3x3 conv {ci}->{co} on {n}x{d}x{h}x{w} (the layer shape that takes the "
                                       f"largest share of this workload's time; lamp_conv3d_fwd with the statistics epilogue)",
            "achieved": fl / t / 1e12, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": fl / t / 1e12 / PEAK_BF16_TFLOPS,
            "traffic": None, "launch_ms": t * 1e3, "algorithmic_bytes": alg}


def oracle_sample(wl, np, S, levels, base, K):
    """The CPU oracle (fp64, as it stands) timed on a small sample of the workload: the same network on a 32^3 input
    (the tiny net at full size).  Returns the cpu_baseline object; the rate is per input voxel, which is what the
    work of these networks is proportional to, so it stands for the full-size rate and is labelled as extrapolated."""
    import oracle as O
    from oracle import sliding as OS
    from oracle import unet as OU
    rp, rx, rl = S.streams(4242, 3)
    p = {k: v.astype(np.float64) for k, v in S.unet_params(rp, levels, base, 1, K, False).items()}
    side = 32
    O.num_threads()
    if wl == "tiny":
        x = S.normal(rx, (1, side, side, side, 1)).astype(np.float64)
        t0 = time.perf_counter()
        OU.forward(p, x, levels)
        vox, what, extra = side ** 3, f"the whole workload at full size (1x{side}^3, forward)", False
    elif wl == "stage":
        x = S.ct_volume(rx, 1, side, side, side).astype(np.float64)
        t0 = time.perf_counter()
        (pooled, skips), cache = OU.forward(p, x, levels, first_level=1, last_level=2)
        gp = S.normal(rl, pooled.shape).astype(np.float64)
        gs = [S.normal(rl, t.shape).astype(np.float64) for t in skips]
        OU.stage_backward(p, cache, gp, gs, 1, 2, levels)
        vox, what, extra = side ** 3, f"the same partition (blocks 1-2, base {base}) forward+backward on a 1x{side}^3 volume", True
    elif wl == "unet_train":
        x = S.ct_volume(rx, 1, side, side, side).astype(np.float64)
        lab = S.organ_labels(rl, 1, side, side, side, K)
        t0 = time.perf_counter()
        OU.loss_and_grads(p, x, lab, levels)
        vox, what, extra = side ** 3, f"the same {levels}-level base-{base} net forward+backward on a 1x{side}^3 volume", True
    elif wl == "unet_infer":
        x = S.ct_volume(rx, 1, side, side, side).astype(np.float64)
        t0 = time.perf_counter()
        OU.forward(p, x, levels)
        vox, what, extra = side ** 3, f"the same {levels}-level base-{base} net forward on a 1x{side}^3 volume", True
    else:  # sliding: 32^3 windows at overlap 0.25 over a 56 x 56 x 32 volume = 2 x 2 x 1 windows
        x = S.ct_volume(rx, 1, 56, 56, side).astype(np.float64)
        t0 = time.perf_counter()
        OS.sliding_window(lambda win: OU.forward(p, win, levels)[0], x, patch=side, overlap=0.25)
        vox = 56 * 56 * side
        what, extra = f"the same net as 4 sliding windows of {side}^3 (overlap 0.25, Gaussian blend) over a 56x56x{side} volume", True
    tc = time.perf_counter() - t0
    return {"value": vox / tc, "unit": "voxels/s", "cores": O.num_threads(), "kind": "oracle", "cpu_model": cpu_model(),
            "extrapolated": extra, "sample": f"{what}, fp64, {tc:.1f} s" + ("; voxels per second of that sample, standing for the "
                                                                            "full-size rate (the work is proportional to the voxel count)" if extra else "")}


def net_bench(wl, args, torch, np, S, L, steps, warm, cpu=True):
    """Times one network-level workload through its entry point and returns its result object."""
    dev = "cuda:0"
    bf, f32 = torch.bfloat16, torch.float32
    if wl == "se_block":
        return se_bench(args, torch, np, S, L)
    cfg = {
        "tiny": dict(levels=3, base=8, in_ch=1, classes=5, dims=(1, 32, 32, 32), dtype=f32, seed=1001),
        "stage": dict(levels=3, base=64, in_ch=1, classes=10, dims=(1, 192, 192, 192), dtype=bf, seed=1003),
        "unet_train": dict(levels=5, base=32, in_ch=1, classes=10, dims=(2, 128, 128, 128), dtype=bf, seed=1004),
        "unet_infer": dict(levels=5, base=32, in_ch=1, classes=10, dims=(1, 256, 256, 160), dtype=bf, seed=1005),
        "sliding": dict(levels=5, base=32, in_ch=1, classes=10, dims=(1, 256, 256, 160), dtype=bf, seed=1005),
        # forward + backward + RMSProp update of the fp32 masters and the bf16 working copies: one optimiser step
        "unet_train_step": dict(levels=5, base=32, in_ch=1, classes=10, dims=(2, 128, 128, 128), dtype=bf, seed=1004),
        # the same mini-batch as two partitions on two streams, one sample per micro-batch, in the pipeline order
        "unet_train_pipeline": dict(levels=5, base=32, in_ch=1, classes=10, dims=(2, 128, 128, 128), dtype=bf, seed=1004),
        # the wider nets of the paper's Sec. 3 (base 64 / 128: up to 1024 / 2048 channels) and a whole
        # head-and-neck sized volume with unequal axes
        "unet_train_b64": dict(levels=5, base=64, in_ch=1, classes=10, dims=(2, 128, 128, 128), dtype=bf, seed=1006),
        "unet_train_b128": dict(levels=5, base=128, in_ch=1, classes=10, dims=(1, 128, 128, 128), dtype=bf, seed=1007),
        "unet_infer_whole": dict(levels=5, base=32, in_ch=1, classes=10, dims=(1, 352, 256, 288), dtype=bf, seed=1008),
        # the squeeze-and-excitation variant of the training net (Sec. 1; Tables 2, 3, 5)
        "seunet_train": dict(levels=5, base=32, in_ch=1, classes=10, dims=(2, 128, 128, 128), dtype=bf, seed=1010, se_ratio=16),
    }[wl]
    levels, base, K, dt = cfg["levels"], cfg["base"], cfg["classes"], cfg["dtype"]
    se_ratio = cfg.get("se_ratio", 0)
    N, D, H, W = cfg["dims"]
    rp, rx, rl = S.streams(cfg["seed"], 3)
    p = S.unet_params(rp, levels, base, 1, K, False, **({"se_ratio": se_ratio} if se_ratio else {}))
    params = [torch.from_numpy(v).to(f32 if (k.endswith(".b") or ".se." in k) else dt).to(dev) for k, v in p.items()]
    x = torch.from_numpy(S.ct_volume(rx, N, D, H, W) if wl != "tiny" else S.normal(rx, (N, D, H, W, 1))).to(dt).to(dev)
    V = N * D * H * W
    dom = None   # (n, d, h, w, ci, co) of the conv layer whose kernel dominates the workload
    if wl in ("tiny", "unet_infer", "unet_infer_whole"):
        ud = L.unet_desc(levels, base, 1, K, N, D, H, W, dt)
        logits = torch.empty((N, D, H, W, K), dtype=f32, device=dev)
        ws = torch.empty(L.lamp_unet_workspace_bytes(ud, False), dtype=torch.uint8, device=dev)
        run = lambda: L.lamp_unet_fwd(ud, params, x, logits, ws=ws)
        flops = unet_flops(levels, base, 1, K, N, D, H, W)
        what = f"{levels}-level base-{base} U-Net forward, {N}x{D}x{H}x{W}"
        dom = (N, D, H, W, base, base)
    elif wl.startswith("unet_train") or wl == "seunet_train":
        ud = L.unet_desc(levels, base, 1, K, N, D, H, W, dt, **({"se_ratio": se_ratio} if se_ratio else {}))
        lab = torch.from_numpy(S.organ_labels(rl, N, D, H, W, K)).to(dev)
        grads = [torch.empty(t.shape, dtype=f32, device=dev) for t in params]
        loss = torch.empty((), dtype=f32, device=dev)
        ws = torch.empty(L.lamp_unet_workspace_bytes(ud, True), dtype=torch.uint8, device=dev)
        flops = 3.0 * unet_flops(levels, base, 1, K, N, D, H, W)
        what = f"{levels}-level base-{base} U-Net forward+backward (softmax CE), {N}x{D}x{H}x{W}"
        if se_ratio:
            what = f"squeeze-and-excitation variant (ratio {se_ratio}) of the " + what
        dom = (N, D, H, W, base, base)
        if wl == "unet_train_step":
            masters = [t.to(f32).clone() for t in params]
            msq = [torch.zeros_like(t) for t in masters]

            def run():
                L.lamp_unet_fwd_bwd(ud, params, x, lab, loss, grads, ws=ws)
                L.lamp_rmsprop_step(masters, msq, grads, params, lr=1e-3, alpha=0.99, eps=1e-8)
            what += " + RMSProp update (lr 1e-3)"
        elif wl == "unet_train_pipeline":
            M, cut = args.micro_batches, args.cut
            if N % M:
                print("bench.py: --micro-batches must divide the mini-batch of 2", file=sys.stderr)
                sys.exit(2)
            mb = L.unet_desc(levels, base, 1, K, N // M, D, H, W, dt)
            aux = torch.cuda.Stream()
            ws = torch.empty(L.lamp_unet_pipeline_workspace_bytes(mb, cut, M), dtype=torch.uint8, device=dev)
            run = lambda: L.lamp_unet_pipeline_fwd_bwd(mb, cut, M, params, x, lab, loss, grads, aux, ws=ws)
            what += f" as 2 partitions (cut after encoder block {cut}) x {M} micro-batches on two streams"
        else:
            run = lambda: L.lamp_unet_fwd_bwd(ud, params, x, lab, loss, grads, ws=ws)
    elif wl == "sliding":
        P = 64
        cnt = L.lamp_sliding_window_count(D, H, W, P, 0.25)
        pd = L.unet_desc(levels, base, 1, K, cnt, P, P, P, dt)
        out = torch.empty((1, D, H, W, K), dtype=f32, device=dev)
        import ctypes
        ws = torch.empty(int(L.lib().lamp_sliding_window_workspace_bytes(ctypes.byref(pd), D, H, W)), dtype=torch.uint8, device=dev)
        run = lambda: L.lamp_sliding_window_fwd(pd, params, x, out, ws=ws)
        flops = unet_flops(levels, base, 1, K, cnt, P, P, P)
        what = f"{cnt} sliding windows of {P}^3 (overlap 0.25, Gaussian blend) over {D}x{H}x{W}, {levels}-level base-{base} U-Net"
        dom = (cnt, P, P, P, base, base)
    else:  # stage: encoder blocks 1-2 of a base-64 net, forward + backward
        ud = L.unet_desc(levels, base, 1, K, N, D, H, W, dt)
        sp = params[:4]
        ws = torch.empty(L.lamp_unet_stage_workspace_bytes(ud, 1, 2), dtype=torch.uint8, device=dev)
        pooled = torch.empty((N, D // 4, H // 4, W // 4, 2 * base), dtype=dt, device=dev)
        skips = [torch.empty((N, D, H, W, base), dtype=dt, device=dev),
                 torch.empty((N, D // 2, H // 2, W // 2, 2 * base), dtype=dt, device=dev)]
        gp = torch.randn(pooled.shape, device=dev, generator=torch.Generator(dev).manual_seed(1)).to(dt)
        gs = [torch.randn(t.shape, device=dev, generator=torch.Generator(dev).manual_seed(2 + i)).to(dt) for i, t in enumerate(skips)]
        grads = [torch.empty(t.shape, dtype=f32, device=dev) for t in sp]

        def run():
            L.lamp_unet_stage_fwd(ud, 1, 2, sp, x, pooled, skips, ws)
            L.lamp_unet_stage_bwd(ud, 1, 2, sp, x, skips, gp, gs, grads, ws)
        v1, v2 = V, V // 8
        fwd = 2.0 * 27 * (v1 * (1 * base + base * base) + v2 * (base * 2 * base + 4 * base * base))
        flops = 3.0 * fwd - 2.0 * 27 * v1 * base  # no data gradient for the first conv
        what = f"encoder partition (blocks 1-2, base {base}) forward+backward, {N}x{D}x{H}x{W}"
        dom = (N, D, H, W, base, base)
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < 0.1:   # clocks settle after the host-side input generation (untimed)
        run()
        torch.cuda.synchronize()
    for _ in range(warm):
        run()
    torch.cuda.synchronize()
    if wl == "tiny" and args.graph:
        # about 60 kernels of a few microseconds: the forward is captured once as a HIP graph on a side stream
        # (the library only enqueues kernels, so the call is capturable as it stands) and a step replays it
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            run()
        eager = logits.clone()
        graph.replay()
        torch.cuda.synchronize()
        if not torch.equal(logits, eager):
            print("bench.py: the captured graph does not reproduce the eager logits", file=sys.stderr)
            sys.exit(1)
        run = graph.replay
        what += " (one captured HIP graph per step)"
        for _ in range(warm):
            run()
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        run()
    torch.cuda.synchronize()
    dtm = (time.perf_counter() - t0) / steps
    out = {"metric": "Conv3d fwd+bwd TFLOP/s (% MFMA peak); whole-U-Net voxels/sec at 1 GPU", "value": V / dtm,
           "unit": "voxels/s", "n_gpus": 1, "steps": steps, "warmup": warm, "ms_per_step": dtm * 1e3,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "bf16" if dt == bf else "f32", "data": "synthetic",
           "config": {"workload": what, "voxels": V, "flop_per_step": flops},
           "voxels_per_s": V / dtm,
           "tflops": flops / dtm / 1e12, "pct_mfma_peak": 100.0 * flops / dtm / 1e12 / PEAK_BF16_TFLOPS}
    if wl.startswith("unet_train") or wl == "seunet_train":
        out["final_loss"] = float(loss.item())   # the timed steps ran on finite data (the optimiser workload moves the weights)
        if not np.isfinite(out["final_loss"]):
            print("bench.py: the loss is not finite after the timed steps", file=sys.stderr)
            sys.exit(1)
    del ws
    torch.cuda.empty_cache()
    if wl == "tiny":
        # a chain of about 60 launches on 32^3 ... 8^3 voxels: bound by per-kernel latency; stated against the HBM
        # roofline with the algorithmic bytes of the whole forward, timed through the entry point (no single
        # kernel dominates)
        alg = unet_ideal_bytes(levels, base, 1, K, N, D, H, W, 4)
        out["roofline"] = {"bound": "hbm", "kernel": "whole forward (a chain of about 60 small fp32 kernels; latency-bound, no dominant kernel)",
                           "achieved": alg / dtm / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": alg / dtm / 1e9 / PEAK_HBM_GBS,
                           "traffic": None, "algorithmic_bytes": alg}
    elif dom is not None:
        out["roofline"] = conv_layer_roofline(torch, S, L, *dom, reps=max(10, steps), seed=cfg["seed"] + 50)
        torch.cuda.empty_cache()
    if cpu and wl in ("tiny", "stage", "unet_train", "unet_infer", "sliding"):
        out["cpu_baseline"] = oracle_sample(wl, np, S, levels, base, K)
    return out


if __name__ == "__main__":
    main()
