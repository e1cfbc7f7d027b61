#!/usr/bin/env python3
"""Benchmark of the sparse-filter convolution hot path on one MI355X.

Workload (benchmark configs[3], the one the metric is quoted on): the VGG16-shaped
stack of 13 3x3 convolution layers (channels 64-64-128-128-256x3-512x3-512x3, 2x2 max-pool
between blocks), batch N=32, 224x224x3 fp32 input ~U[0,1), 95 % random unstructured weight
sparsity on every layer but the first (dense), bias + ReLU fused into each convolution.

A "step" is one pass of the whole stack over one batch: 13 fscnn_conv2d_sparse_filter launches
plus the 4 helper max-pools, input and compressed filters already resident in HBM.  The first
layer reads NCHW, the last writes NCHW, the layers in between hand each other N4
(batch-interleaved) tensors.  Effective work is F_eff = sum over layers of 2*nnz*Ho*Wo*N.

Prints ONE JSON line (see the keys below).  `--gpus N` with N > 1 is refused: this build runs
on one GPU.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
FP32_VECTOR_PEAK_TFLOPS = 157.3  # MI355X published fp32 vector peak (counts packed FMA)
FP32_UNPACKED_PEAK_TFLOPS = 78.6  # 256 CU x 4 SIMD x 16 lanes x 2 flop x 2.4 GHz, one FMA/lane/clk


def build_stack(fscnn, torch, inputs, n, keep):
    x, layers = inputs.vgg16_stack(4, n, keep)
    dev_layers = []
    t0 = time.perf_counter()
    for L in layers:
        w = torch.from_numpy(L["w"]).cuda()
        b = torch.from_numpy(L["bias"]).cuda()
        dev_layers.append(dict(w=w, bias=b, relu=L["relu"], pool=L["pool_after"], hw=L["hw"],
                               k=L["w"].shape[0], c=L["w"].shape[1]))
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for d in dev_layers:
        d["f"] = fscnn.filter_compress(d["w"])
    torch.cuda.synchronize()
    compress_ms = (time.perf_counter() - t1) * 1e3
    del t0
    return torch.from_numpy(x).cuda(), dev_layers, compress_ms


def alloc_buffers(fscnn, torch, dev_layers, n):
    """Output tensors of every layer (and pool), allocated once: the timed loop allocates nothing."""
    last = len(dev_layers) - 1
    for li, d in enumerate(dev_layers):
        hw = d["hw"]
        lay_out = fscnn.NCHW if li == last else fscnn.N4
        shape = (n, d["k"], hw, hw) if lay_out == fscnn.NCHW else fscnn.n4_shape(n, d["k"], hw, hw)
        d["y"] = torch.empty(shape, dtype=torch.float32, device="cuda")
        d["lay_in"] = fscnn.NCHW if li == 0 else fscnn.N4
        d["lay_out"] = lay_out
        if d["pool"]:
            d["p"] = torch.empty(fscnn.n4_shape(n, d["k"], hw // 2, hw // 2), dtype=torch.float32, device="cuda")


def run_step(fscnn, x, dev_layers, n, events=None):
    cur = x
    for li, d in enumerate(dev_layers):
        if events is not None:
            events[li][0].record()
        fscnn.conv2d_sparse_filter(d["f"], cur, (1, 1), (1, 1), d["bias"], d["relu"], out=d["y"],
                                   x_layout=d["lay_in"], y_layout=d["lay_out"], n=n)
        if events is not None:
            events[li][1].record()
        cur = d["y"]
        if d["pool"]:
            fscnn.maxpool2x2(cur, out=d["p"], layout=fscnn.N4, n=n)
            cur = d["p"]
    return cur


def cpu_baseline(inputs, keep, images):
    """The CPU oracle (as it stands) on a bounded sample: the same stack on `images` images."""
    import oracle
    x, layers = inputs.vgg16_stack(4, images, keep)
    feff = 0.0
    t0 = time.perf_counter()
    cur = x
    for L in layers:
        csr = oracle.filter_compress(L["w"])
        y = oracle.conv2d_sparse_filter(cur, csr, L["w"].shape, L["stride"], L["pad"], L["bias"], L["relu"])
        feff += 2.0 * int(csr[0][-1]) * y.shape[2] * y.shape[3] * images
        cur = oracle.maxpool2x2(y) if L["pool_after"] else y
    dt = time.perf_counter() - t0
    return dict(value=feff / dt / 1e9, unit="effective GFLOP/s", cores=oracle.num_threads(), kind="oracle",
                sample="same VGG16-shaped stack (config 4 weights), %d images instead of 32, %.1f s" % (images, dt))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--batch", type=int, default=32)
    ap.add_argument("--keep", type=float, default=0.05, help="weight density of layers 2..13")
    ap.add_argument("--cpu-images", type=int, default=16, help="images of the oracle-timed sample (0 = skip)")
    ap.add_argument("--traffic-calibration", action="store_true",
                    help="run only a plain copy-like kernel of known size (1 GiB read, 1 GiB written) three "
                         "times; used to scale the FETCH_SIZE / WRITE_SIZE counters of rocprofv3 --pmc")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding code); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2212_08815_amd import fscnn, inputs
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    fscnn.lib()
    torch.cuda.set_device(0)
    if args.traffic_calibration:
        src = torch.rand(64, 64, 256, 256, device="cuda")            # 2^28 floats = 1 GiB
        for _ in range(3):
            dst = fscnn.layout_convert(src, fscnn.NCHW)              # layout_convert_kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        print(json.dumps(dict(calibration_kernel="layout_convert_kernel", bytes_read=src.numel() * 4,
                              bytes_written=dst.numel() * 4, launches=3)))
        return
    n = args.batch
    x, dev_layers, compress_ms = build_stack(fscnn, torch, inputs, n, args.keep)
    alloc_buffers(fscnn, torch, dev_layers, n)

    # per-layer effective work and algorithmic bytes (x read once, y written once, compressed filter
    # and bias read once)
    feff, balg = [], []
    for d in dev_layers:
        hw = d["hw"]
        feff.append(2.0 * d["f"].nnz * hw * hw * n)
        balg.append(4.0 * n * hw * hw * (d["c"] + d["k"]) + 8.0 * d["f"].nnz + 4.0 * (d["k"] + 1) + 4.0 * d["k"])
    F, B = sum(feff), sum(balg)

    for _ in range(max(args.warmup, 1)):       # also builds every plan: the timed loop allocates nothing
        run_step(fscnn, x, dev_layers, n)
    torch.cuda.synchronize()

    events = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for _ in dev_layers] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        run_step(fscnn, x, dev_layers, n, events[s])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3

    # per-layer kernel durations (HIP events on the launch stream, inside the timed region)
    layer_ms = [float(np.mean([events[s][li][0].elapsed_time(events[s][li][1]) for s in range(args.steps)]))
                for li in range(len(dev_layers))]
    conv_ms = sum(layer_ms)
    # dominant kernel = the layer launch with the largest share of the step
    dom = int(np.argmax(layer_ms))
    dd = dev_layers[dom]
    dom_tflops = feff[dom] / (layer_ms[dom] * 1e-3) / 1e12
    roofline = dict(bound="alu", achieved=dom_tflops, peak=FP32_VECTOR_PEAK_TFLOPS, unit="TFLOP/s",
                    frac=dom_tflops / FP32_VECTOR_PEAK_TFLOPS, traffic=None,
                    kernel="conv_sf_tiled_kernel, layer %d (C=%d K=%d %dx%d N=%d, nnz=%d)" % (
                        dom + 1, dd["c"], dd["k"], dd["hw"], dd["hw"], n, dd["f"].nnz),
                    launch_ms=layer_ms[dom], flop_per_launch=feff[dom], bytes_per_launch=balg[dom],
                    peak_unpacked=FP32_UNPACKED_PEAK_TFLOPS, frac_unpacked=dom_tflops / FP32_UNPACKED_PEAK_TFLOPS,
                    hbm_gbs=balg[dom] / (layer_ms[dom] * 1e-3) / 1e9,
                    hbm_frac=balg[dom] / (layer_ms[dom] * 1e-3) / 1e9 / HBM_PEAK_GBS)
    # measured HBM bytes of that launch (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a copy
    # kernel of known size): taken from the committed summary of the same workload, else null
    traffic_file = os.path.join(ROOT, "profiles", "conv_sf_vgg16_n32_hbm_traffic.txt")
    if os.path.exists(traffic_file) and n == 32 and abs(args.keep - 0.05) < 1e-9:
        for line in open(traffic_file):
            f = line.split()
            if len(f) == 4 and f[0] == "layer_%d" % (dom + 1):
                roofline["traffic"] = float(f[3])

    out = dict(
        metric="effective GFLOP/s (2*nnz*Ho*Wo*N) + HBM GB/s fraction, VGG16-shaped stack @95%",
        value=F / (ms_per_step * 1e-3) / 1e9, unit="effective GFLOP/s", n_gpus=1, steps=args.steps,
        warmup=args.warmup, ms_per_step=ms_per_step, higher_is_better=True, scaling="weak",
        vs_baseline=None, dtype="f32", data="synthetic",
        config=dict(workload="VGG16 conv stack, 13 layers 3x3 s1 p1 + 4 max-pools, N=%d, 224x224x3, "
                             "weight density %.2f (first layer dense), bias+ReLU fused" % (n, args.keep),
                    batch=n, effective_gflop_per_step=F / 1e9, algorithmic_gbytes_per_step=B / 1e9,
                    nnz_total=int(sum(d["f"].nnz for d in dev_layers))),
        hbm=dict(algorithmic_gbs=B / (ms_per_step * 1e-3) / 1e9,
                 frac_of_peak=B / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, peak_gbs=HBM_PEAK_GBS),
        conv_kernels_ms=conv_ms, conv_only_effective_gflops=F / (conv_ms * 1e-3) / 1e9,
        layer_ms=[round(v, 4) for v in layer_ms],
        layer_effective_tflops=[round(feff[i] / (layer_ms[i] * 1e-3) / 1e12, 2) for i in range(len(layer_ms))],
        filter_compress_ms_all_layers=compress_ms,
        roofline=roofline,
    )
    if args.cpu_images > 0:
        out["cpu_baseline"] = cpu_baseline(inputs, args.keep, args.cpu_images)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
