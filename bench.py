#!/usr/bin/env python3
"""Benchmark of the sparse-filter convolution hot path on one MI355X.

Workload (the configuration the headline metric is quoted on): the VGG16-shaped
stack of 13 3x3 convolution layers (channels 64-64-128-128-256x3-512x3-512x3, 2x2 max-pool
between blocks), batch N=32, 224x224x3 fp32 input ~U[0,1), 95 % random unstructured weight
sparsity on every layer but the first (dense), bias + ReLU fused into each convolution.

A "step" is one pass of the whole stack over one batch: 13 convolution launches, input and
compressed filters already resident in HBM.  The 2x2 max-pools that follow layers 2, 4, 7, 10
(and 13) are merged into those layers' launches (merged convolution + pooling, Alg. 7);
`--separate-pool` runs them as helper kernels instead.  The first layer reads NCHW, the last
writes NCHW, the layers in between hand each other N4 (batch-interleaved) tensors.  Effective
work is F_eff = sum over layers of 2*nnz*Ho*Wo*N.

The `roofline` object describes the dominant kernel: the kernel instantiation (configuration,
layouts, pooled or not) with the largest share of the step.  Its launch duration is the mean over
its launches (several layers may share it), measured with HIP events inside the timed region.

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


def build_stack(fscnn, torch, inputs, n, keep, config_id=4):
    x, layers = inputs.vgg16_stack(config_id, n, keep)
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


def alloc_buffers(fscnn, torch, dev_layers, n, fuse_pool, n4=True):
    """Output tensors of every layer (and pool), allocated once: the timed loop allocates nothing.
    n4: tensors between the layers in the image-interleaved layout (batches of at least four);
    else NCHW throughout, and a pool is merged only where the automatic choice has a pooled form."""
    last = len(dev_layers) - 1
    for li, d in enumerate(dev_layers):
        hw = d["hw"]
        lay_out = fscnn.NCHW if li == last or not n4 else fscnn.N4
        shape = lambda h: (n, d["k"], h, h) if lay_out == fscnn.NCHW else fscnn.n4_shape(n, d["k"], h, h)
        d["y"] = torch.empty(shape(hw), dtype=torch.float32, device="cuda")
        d["lay_in"] = fscnn.NCHW if li == 0 or not n4 else fscnn.N4
        d["lay_out"] = lay_out
        fused = bool(d["pool"] and fuse_pool)
        if fused and not n4:
            fused = fscnn.sf_variant_choice(d["f"], n, hw, hw, n4=False, pool=True) > 0
        if fused:                              # the conv launch stores the pooled tensor only
            d["y"] = torch.empty(shape(hw // 2), dtype=torch.float32, device="cuda")
        elif d["pool"]:
            d["p"] = torch.empty(shape(hw // 2), dtype=torch.float32, device="cuda")
        d["fused"] = fused


def run_step(fscnn, x, dev_layers, n, events=None):
    """One pass of the stack.  events: one HIP event per layer boundary (len(dev_layers) + 1) when
    every pool is merged into its convolution, so that consecutive events bracket exactly one
    launch; with separate pools, a (start, stop) pair per layer."""
    cur = x
    shared = events is not None and len(events) == len(dev_layers) + 1
    for li, d in enumerate(dev_layers):
        if events is not None:
            (events[li] if shared else events[li][0]).record()
        fscnn.conv2d_sparse_filter(d["f"], cur, (1, 1), (1, 1), d["bias"], d["relu"], out=d["y"],
                                   x_layout=d["lay_in"], y_layout=d["lay_out"], n=n, pool=d["fused"])
        if events is not None and not shared:
            events[li][1].record()
        cur = d["y"]
        if d["pool"] and not d["fused"]:
            fscnn.maxpool2x2(cur, out=d["p"], layout=d["lay_out"], n=n)
            cur = d["p"]
    if shared:
        events[len(dev_layers)].record()
    return cur


def n4_flat(np, flat, n, k, h, w):
    """Positions, in an N4 tensor ([ceil(N/4)][K][H][W][4]), of the elements whose NCHW flat indices are `flat`."""
    ox = flat % w
    oy = (flat // w) % h
    kk = (flat // (w * h)) % k
    nn = flat // (w * h * k)
    return ((((nn // 4) * k + kk) * h + oy) * w + ox) * 4 + nn % 4


def to_host_nchw(fscnn, t, layout, n):
    """A tensor of the chain as a host N x C x H x W array (plumbing of the check, not of the path)."""
    if layout == fscnn.N4:
        t = t.permute(0, 4, 1, 2, 3).reshape(-1, t.shape[1], t.shape[2], t.shape[3])[:n]
    return t.contiguous().cpu().numpy()


def chain_samples(fscnn, torch, np, oracle, x, dev_layers, n, npts=4000, seed=4):
    """Checks the tensors the last run_step() left behind, layer by layer, against the oracle.

    For every layer yields (li, g, o, a, nmax): g = the launch's stored outputs at npts sampled
    positions plus the corners of the tensor, o = the oracle's values there computed from the
    GPU's own previous tensor (so errors do not compound), a = the oracle's sum |w||x| + |b| at
    those positions, nmax = longest filter row.  Where the 2x2 max-pool is merged into the
    launch, the oracle value is the maximum of the definition over the pooled window (bias and
    ReLU applied first, as the separate layers would)."""
    rng = np.random.default_rng(seed)
    cur, cur_layout = x, fscnn.NCHW
    for li, d in enumerate(dev_layers):
        xin = to_host_nchw(fscnn, cur, cur_layout, n)
        w = d["w"].cpu().numpy()
        b = d["bias"].cpu().numpy()
        k, hw = d["k"], d["hw"]
        oh = hw // 2 if d["fused"] else hw
        total = n * k * oh * oh
        flat = rng.choice(total, size=min(npts, total), replace=False)
        flat = np.unique(np.concatenate([flat, [0, oh - 1, total - 1, total - oh]])).astype(np.int64)
        y = d["y"]
        pos = n4_flat(np, flat, n, k, oh, oh) if d["lay_out"] == fscnn.N4 else flat
        g = y.view(-1)[torch.from_numpy(pos).cuda()].cpu().numpy()
        if d["fused"]:
            px, py = flat % oh, (flat // oh) % oh
            nk = flat // (oh * oh)
            win = np.stack([(nk * hw + 2 * py + dy) * hw + 2 * px + dx for dy in (0, 1) for dx in (0, 1)], 1)
            o4, a4 = oracle.conv2d_points(xin, w, win.ravel(), (1, 1), (1, 1), b, d["relu"], want_abs=True)
            o, a = o4.reshape(-1, 4).max(1), a4.reshape(-1, 4).max(1)
        else:
            o, a = oracle.conv2d_points(xin, w, flat, (1, 1), (1, 1), b, d["relu"], want_abs=True)
        nmax = int(np.count_nonzero(w.reshape(k, -1), axis=1).max())
        yield li, g, o, a, nmax
        cur, cur_layout = y, d["lay_out"]
        if d["pool"] and not d["fused"]:
            cur = d["p"]


def rel_err(np, g, o):
    """max |g - o| / max(|o|, rms(o)): the comparison rule of the parity tests."""
    g, o = g.astype(np.float64), o.astype(np.float64)
    tau = float(np.sqrt(np.mean(o * o)))
    return float(np.max(np.abs(g - o) / np.maximum(np.abs(o), tau if tau > 0 else 1.0)))


def probe_gather_fma(torch, iters=20000, work_groups=2048):
    """TFLOP/s the chip sustains on the hot loop's instruction mix (one LDS word per fused
    multiply-add) without sparsity, staging or barriers: the kernel of libfscnn_bench_probe.so, a
    shared object of this script's own (the library does not hold it), timed with HIP events."""
    import ctypes
    path = os.path.join(ROOT, "paper_2212_08815_amd", "libfscnn_bench_probe.so")
    if not os.path.exists(path):
        from paper_2212_08815_amd import build
        build.build()
    probe = ctypes.CDLL(path).bench_probe_gather_fma
    probe.restype = ctypes.c_int
    probe.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
    scratch = torch.ones(4, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    assert probe(scratch.data_ptr(), 100, work_groups, stream) == 0
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    assert probe(scratch.data_ptr(), iters, work_groups, stream) == 0
    b.record()
    torch.cuda.synchronize()
    return work_groups * 256.0 * iters * 32.0 / (a.elapsed_time(b) * 1e-3) / 1e12


def roof_of(flop, nbytes, ms):
    """Roofline object of one launch (or one step): the roof that takes longer at the published
    peaks binds; achieved / peak in that roof's unit."""
    t_hbm, t_alu = nbytes / (HBM_PEAK_GBS * 1e9), flop / (FP32_VECTOR_PEAK_TFLOPS * 1e12)
    if t_hbm >= t_alu:
        a = nbytes / (ms * 1e-3) / 1e9
        return dict(bound="hbm", achieved=a, peak=HBM_PEAK_GBS, unit="GB/s", frac=a / HBM_PEAK_GBS)
    a = flop / (ms * 1e-3) / 1e12
    return dict(bound="alu", achieved=a, peak=FP32_VECTOR_PEAK_TFLOPS, unit="TFLOP/s", frac=a / FP32_VECTOR_PEAK_TFLOPS)


def layer_bytes(n, c, k, hw, yhw, nnz):
    """Algorithmic bytes of one sparse-filter launch: x read once, y written once, the compressed
    filter (value + packed index per non-zero, row pointers) and the bias read once."""
    return 4.0 * n * (hw * hw * c + yhw * k) + 8.0 * nnz + 4.0 * (k + 1) + 4.0 * k


def config_rows(fscnn, torch, inputs, np, oracle, steps=20, check_points=2000):
    """The small configurations: the two single layers at N=1 and the 13-layer stack at N=1 (90 %
    weight sparsity), the stack both as 13 launches per step and as one captured HIP graph.  Every
    row is checked against the oracle before it is timed."""
    out = {}
    for name, c in (("config1_single_layer_n1_c16_k32_32x32_keep0.10", inputs.config1()),
                    ("config2_single_layer_n1_c256_k256_56x56_keep0.05", inputs.config2())):
        w, x = c["w"], c["x"]
        f = fscnn.filter_compress(torch.from_numpy(w).cuda())
        xd = torch.from_numpy(x).cuda()
        bd = None if c["bias"] is None else torch.from_numpy(c["bias"]).cuda()
        n, cc, h, wd = x.shape
        k = w.shape[0]
        y = fscnn.conv2d_sparse_filter(f, xd, c["stride"], c["pad"], bd, c["relu"])
        o, a = oracle.conv2d_sparse_filter(x, oracle.filter_compress(w), w.shape, c["stride"], c["pad"], c["bias"],
                                           c["relu"], want_abs=True)
        err = rel_err(np, y.cpu().numpy(), o)
        ms = time_gpu(torch, lambda: fscnn.conv2d_sparse_filter(f, xd, c["stride"], c["pad"], bd, c["relu"], out=y), 200)
        flop = 2.0 * f.nnz * h * wd * n
        nbytes = layer_bytes(n, cc, k, h, h * wd, f.nnz)          # square inputs
        v = fscnn.sf_variant_choice(f, n, h, wd)
        out[name] = dict(ms_per_launch=ms, effective_gflops=flop / ms / 1e6, algorithmic_gbs=nbytes / ms / 1e6,
                         max_rel_err=err, kernel=fscnn.sf_variant_name(v) if v > 0 else "direct",
                         roofline=roof_of(flop, nbytes, ms),
                         note="back-to-back launches on one stream, HIP events around 200 of them; one "
                              "image leaves most of the 256 compute units idle")
        assert err <= 1e-4, (name, err)

    # config 3: the stack at N=1, NCHW tensors throughout, plans and channel-split scratch prepared
    # beforehand on the stream that runs (and captures) it
    n = 1
    x, L, _ = build_stack(fscnn, torch, inputs, n, 0.10, config_id=3)
    alloc_buffers(fscnn, torch, L, n, True, n4=False)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for d in L:
            fscnn.filter_prepare(d["f"], n, d["hw"], d["hw"], (1, 1), (1, 1), 0, d["lay_in"], d["lay_out"], d["fused"])
        run_step(fscnn, x, L, n)
        side.synchronize()
        errs = [rel_err(np, g, o) for _, g, o, _, _ in chain_samples(fscnn, torch, np, oracle, x, L, n, check_points)]
        eager_last = L[-1]["y"].clone()
        ev = lambda: torch.cuda.Event(enable_timing=True)
        events = [[ev() for _ in range(len(L) + 1)] for _ in range(steps)]
        side.synchronize()
        t0 = time.perf_counter()
        for st in range(steps):
            run_step(fscnn, x, L, n, events[st] if all(d["fused"] or not d["pool"] for d in L) else None)
        side.synchronize()
        eager_ms = (time.perf_counter() - t0) / steps * 1e3
        shared = all(d["fused"] or not d["pool"] for d in L)
        layer_ms = ([float(np.mean([events[st][li].elapsed_time(events[st][li + 1]) for st in range(steps)]))
                     for li in range(len(L))] if shared else None)
    # one HIP graph of the same 13 (+ pool) launches: no allocation, no memset node, nothing but
    # kernel nodes.  Replayed with eager work and synchronisations in between, every replay
    # compared bit for bit with the eager result, then timed.
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run_step(fscnn, x, L, n)
    replays_equal = True
    for r in range(4):
        L[-1]["y"].fill_(-1.0)
        for d in L[:-1]:
            d["y"].zero_()                     # eager work of the program's own between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        replays_equal = replays_equal and bool(torch.equal(L[-1]["y"], eager_last))
    a, b = ev(), ev()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    a.record()
    for _ in range(steps):
        graph.replay()
    b.record()
    torch.cuda.synchronize()
    graph_wall_ms = (time.perf_counter() - t0) / steps * 1e3
    graph_ms = a.elapsed_time(b) / steps
    feff = [2.0 * d["f"].nnz * d["hw"] ** 2 * n for d in L]
    byts = [layer_bytes(n, d["c"], d["k"], d["hw"], (d["hw"] // 2) ** 2 if d["fused"] else d["hw"] ** 2, d["f"].nnz)
            for d in L]
    F, B = sum(feff), sum(byts)
    kern = []
    for d in L:
        v = fscnn.sf_variant_choice(d["f"], n, d["hw"], d["hw"], n4=False, pool=d["fused"])
        kern.append(fscnn.sf_variant_name(v) if v > 0 else "direct")
    row = dict(eager_ms_per_step=eager_ms, graph_ms_per_step=graph_ms, graph_wall_ms_per_step=graph_wall_ms,
               eager_effective_gflops=F / eager_ms / 1e6, graph_effective_gflops=F / graph_ms / 1e6,
               graph_algorithmic_gbs=B / graph_ms / 1e6, graph_replays_bit_equal_to_eager=replays_equal,
               max_rel_err=max(errs), per_layer_rel_err=errs, layer_ms=layer_ms, layer_kernel=kern,
               pools_merged=[bool(d["fused"]) for d in L if d["pool"]],
               roofline=roof_of(F, B, graph_ms),
               note="13 launches per step on one stream (plans and split scratch prepared beforehand) against "
                    "one replay of a HIP graph that holds the same launches; N=1 leaves the chip mostly idle "
                    "and the step is bound by launch and dependency latency, not by a roof")
    if layer_ms is not None:
        li = int(np.argmax(layer_ms))
        row["dominant_layer"] = dict(layer=li + 1, kernel=kern[li], ms=layer_ms[li],
                                     roofline=roof_of(feff[li], byts[li], layer_ms[li]))
    assert replays_equal and max(errs) <= 1e-4, row
    out["config3_vgg16_stack_n1_keep0.10"] = row
    return out


def time_gpu(torch, fn, iters):
    """Average milliseconds of fn() over `iters` calls (HIP events on the current stream)."""
    fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(iters):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / iters


def other_rows(fscnn, torch, inputs, np, dev_layers):
    """The steps of the path that are not inside the timed stack: filter compression and plan
    build (once per model), activation compression and the sparse-input convolution (workload:
    the conv4-shaped layer of the sparsity sweep, N=8, C=K=512, 28x28), and the sparse-filter
    kernel on that layer at the sweep's densities."""
    out = {}
    # A1-A3: compress + plan of all 13 layers (includes the two host synchronisations per layer)
    wbytes = sum(d["w"].numel() * 4 for d in dev_layers)

    def compress_all():
        for d in dev_layers:
            f = fscnn.filter_compress(d["w"])
            fscnn.filter_prepare(f, 32, d["hw"], d["hw"], (1, 1), (1, 1))
    t0 = time.perf_counter()
    compress_all()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3
    out["filter_compress_and_plan"] = dict(ms=ms, dense_weight_bytes=wbytes, gbs=wbytes / ms / 1e6,
                                           note="13 layers, wall clock incl. allocations and host syncs")
    # config 5 layer
    sweep = []
    for keep in inputs.CONFIG5_KEEP:
        c = inputs.config5(keep)
        x = torch.from_numpy(c["x"]).cuda()
        w = torch.from_numpy(c["w"]).cuda()
        b = torch.from_numpy(c["bias"]).cuda()
        f = fscnn.filter_compress(w)
        y = fscnn.conv2d_sparse_filter(f, x, (1, 1), (1, 1), b, True)
        ms = time_gpu(torch, lambda: fscnn.conv2d_sparse_filter(f, x, (1, 1), (1, 1), b, True, out=y), 10)
        feff = 2.0 * f.nnz * 28 * 28 * 8
        # the same launch on batch-interleaved (N4) tensors, as chained layers pass them
        x4 = fscnn.layout_convert(x, fscnn.NCHW)
        y4 = fscnn.conv2d_sparse_filter(f, x4, (1, 1), (1, 1), b, True, x_layout=fscnn.N4, y_layout=fscnn.N4, n=8)
        ms4 = time_gpu(torch, lambda: fscnn.conv2d_sparse_filter(f, x4, (1, 1), (1, 1), b, True, out=y4,
                                                                 x_layout=fscnn.N4, y_layout=fscnn.N4, n=8), 10)
        sweep.append(dict(keep=keep, nnz=f.nnz, ms=ms, effective_tflops=feff / ms / 1e9,
                          ms_n4=ms4, effective_tflops_n4=feff / ms4 / 1e9))
        if keep == 0.05:
            n, ch, h, wd = c["x"].shape
            ms_c = time_gpu(torch, lambda: fscnn.input_compress(x), 5)
            xs = fscnn.input_compress(x)
            out["input_compress"] = dict(ms=ms_c, nnz=xs.nnz, density=xs.nnz / x.numel(),
                                         gbs=(x.numel() * 4 + xs.nnz * 8) / ms_c / 1e6,
                                         note="N=8, C=512, 28x28, ReLU(N(-0.5,1)); incl. allocations and two host syncs")
            y2 = fscnn.conv2d_sparse_input(xs, w, (1, 1), (1, 1), b, True)
            ms_s = time_gpu(torch, lambda: fscnn.conv2d_sparse_input(xs, w, (1, 1), (1, 1), b, True, out=y2), 5)
            # effective work: (nonzero input, in-image tap, k) triples
            nzpix = (c["x"] != 0).sum(axis=1).astype(np.float64)             # N x H x W
            ty = np.full(h, 3.0); ty[0] = ty[-1] = 2.0
            tx = np.full(wd, 3.0); tx[0] = tx[-1] = 2.0
            triples = float((nzpix * ty[None, :, None] * tx[None, None, :]).sum()) * w.shape[0]
            out["conv2d_sparse_input"] = dict(ms=ms_s, effective_tflops=2.0 * triples / ms_s / 1e9,
                                              dense_equivalent_tflops=2.0 * w.numel() * h * wd * n / ms_s / 1e9,
                                              note="same layer, dense 512x512x3x3 filter bank (values of the 95 % "
                                                   "sparse weights), compressed input")
            dw = fscnn.dense_filter_prepare(w)
            ms_p = time_gpu(torch, lambda: fscnn.conv2d_sparse_input_prepared(xs, dw, (1, 1), (1, 1), b, True, out=y2), 5)
            out["conv2d_sparse_input_prepared"] = dict(
                ms=ms_p, effective_tflops=2.0 * triples / ms_p / 1e9,
                dense_equivalent_tflops=2.0 * w.numel() * h * wd * n / ms_p / 1e9,
                note="same, filter bank prepared once as a K-contiguous copy (N=8: too few patches to fill the chip)")
            # sparse output emission: the sparse-filter convolution of this layer returning its
            # ReLU output compressed (a dense temporary inside), next to the convolution alone
            ms_e = time_gpu(torch, lambda: fscnn.conv2d_sparse_filter_emit(f, x, (1, 1), (1, 1), b, True), 5)
            es = fscnn.conv2d_sparse_filter_emit(f, x, (1, 1), (1, 1), b, True)
            ms_i = time_gpu(torch, lambda: fscnn.conv2d_sparse_filter_emit(f, x, (1, 1), (1, 1), b, True, into=es), 5)
            out["conv2d_sparse_filter_emit"] = dict(
                ms=ms_i, ms_with_allocation=ms_e, conv_alone_ms=ms, nnz_out=es.nnz, density_out=es.nnz / y.numel(),
                note="same layer at 95 % weight sparsity: convolution + ReLU + compression of the result "
                     "(counted in the convolution's epilogue, one scan, one fill); ms = refilling a handle "
                     "(fscnn_conv2d_sparse_filter_emit_into), ms_with_allocation = a new handle per call "
                     "(one hipMalloc and the previous handle's hipFree)")
            x32 = torch.from_numpy(np.concatenate([c["x"]] * 4, 0)).cuda()
            xs32 = fscnn.input_compress(x32)
            y32 = fscnn.conv2d_sparse_input_prepared(xs32, dw, (1, 1), (1, 1), b, True)
            ms_q = time_gpu(torch, lambda: fscnn.conv2d_sparse_input_prepared(xs32, dw, (1, 1), (1, 1), b, True, out=y32), 5)
            out["conv2d_sparse_input_prepared_n32"] = dict(
                ms=ms_q, effective_tflops=8.0 * triples / ms_q / 1e9,
                dense_equivalent_tflops=8.0 * w.numel() * h * wd * n / ms_q / 1e9,
                note="same layer with the batch repeated four times (N=32)")
    out["sparse_filter_density_sweep_conv4_n8"] = sweep
    # Alg. 3 / Alg. 4: transposes of compressed operands of that layer (workspace brought by the caller:
    # the calls allocate nothing); bytes = rowptr + index + value arrays read once and written once
    c = inputs.config5(0.05)
    f = fscnn.filter_compress(torch.from_numpy(c["w"]).cuda())
    rp, ix, vl = fscnn.filter_export(f)
    K, CRS = c["w"].shape[0], int(np.prod(c["w"].shape[1:]))
    d_rp, d_ix, d_vl = (torch.from_numpy(rp).cuda(), torch.from_numpy(ix.view(np.int32)).cuda(),
                        torch.from_numpy(vl).cuda())
    ws = torch.empty(fscnn.sparse_transpose_workspace(CRS, f.nnz) // 4 + 1, dtype=torch.int32, device="cuda")
    ms_t = time_gpu(torch, lambda: fscnn.sparse_transpose(d_rp, d_ix, d_vl, K, CRS, workspace=ws), 20)
    out["sparse_matrix_transpose"] = dict(ms=ms_t, nnz=int(f.nnz),
                                          gbs=(16.0 * f.nnz + 4.0 * (K + CRS + 2)) / ms_t / 1e6,
                                          note="Alg. 3 on the 512 x 4608 matrix of the 95 % sparse filter bank; "
                                               "incl. the binding's output allocations")
    x0 = c["x"][0]                                                    # one image, C x H x W
    Cc, Hh, Ww = x0.shape
    rr, cc = np.nonzero(x0.reshape(Cc * Hh, Ww))
    tp = np.zeros(Cc * Hh + 1, np.int64)
    np.add.at(tp, rr + 1, 1)
    t_rp = torch.from_numpy(np.cumsum(tp).astype(np.int32)).cuda()
    t_ix = torch.from_numpy(cc.astype(np.int32)).cuda()
    t_vl = torch.from_numpy(x0.reshape(Cc * Hh, Ww)[rr, cc].astype(np.float32)).cuda()
    ws2 = torch.empty(fscnn.sparse_transpose_workspace(Ww * Hh, len(rr)) // 4 + 1, dtype=torch.int32, device="cuda")
    ms_t2 = time_gpu(torch, lambda: fscnn.sparse_tensor_transpose(t_rp, t_ix, t_vl, Ww, Hh, Cc, workspace=ws2), 20)
    out["sparse_tensor_transpose"] = dict(ms=ms_t2, nnz=int(len(rr)),
                                          gbs=(16.0 * len(rr) + 4.0 * (Cc * Hh + Ww * Hh + 2)) / ms_t2 / 1e6,
                                          note="Alg. 4 (O_whc -> O_chw) on one 28x28x512 activation of the same layer; "
                                               "incl. the binding's output allocations")
    # second workload of the paper (Sec. 6): YOLO-shaped stack = Darknet-53's 52 convolutions as a
    # chain (3x3 stride 1 and 2, 1x1, LeakyReLU 0.1), 416x416, N=32, 95 % sparse (first layer dense)
    yn = 32
    yx, ylayers = inputs.yolo_stack(yn, 0.05)
    ycur = fscnn.layout_convert(torch.from_numpy(yx).cuda(), fscnn.NCHW)
    ydev = []
    for L in ylayers:
        f = fscnn.filter_compress(torch.from_numpy(L["w"]).cuda())
        k = L["w"].shape[0]
        ho = (L["hw"] + 2 * L["pad"][0] - L["w"].shape[2]) // L["stride"][0] + 1
        ydev.append(dict(f=f, b=torch.from_numpy(L["bias"]).cuda(), L=L, ho=ho,
                         y=torch.empty(fscnn.n4_shape(yn, k, ho, ho), dtype=torch.float32, device="cuda")))

    def ystep():
        cur = ycur
        for d in ydev:
            L = d["L"]
            fscnn.conv2d_sparse_filter(d["f"], cur, L["stride"], L["pad"], d["b"], leaky=L["leaky"], out=d["y"],
                                       x_layout=fscnn.N4, y_layout=fscnn.N4, n=yn)
            cur = d["y"]
    ms_y = time_gpu(torch, ystep, 5)
    yflop = sum(2.0 * d["f"].nnz * d["ho"] * d["ho"] * yn for d in ydev)
    out["yolo_shaped_stack"] = dict(ms=ms_y, effective_tflops=yflop / ms_y / 1e9, effective_gflop=yflop / 1e9,
                                    nnz_total=int(sum(d["f"].nnz for d in ydev)),
                                    note="52 convolution layers of Darknet-53 as a chain, N=32, 416x416, weight "
                                         "density 0.05 (first layer dense), bias + LeakyReLU(0.1) fused, N4 between layers")
    return out


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
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--batch", type=int, default=32)
    ap.add_argument("--keep", type=float, default=0.05, help="weight density of layers 2..13")
    ap.add_argument("--cpu-images", type=int, default=16, help="images of the oracle-timed sample (0 = skip)")
    ap.add_argument("--separate-pool", action="store_true",
                    help="run the 4 max-pools as separate helper kernels instead of the merged conv+pool epilogue")
    ap.add_argument("--no-rows", action="store_true", help="skip the measurements outside the timed stack")
    ap.add_argument("--no-check", action="store_true",
                    help="skip the comparison of every layer's stored tensor with the CPU oracle on sampled outputs")
    ap.add_argument("--check-points", type=int, default=4000, help="sampled outputs per layer of that comparison")
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
    alloc_buffers(fscnn, torch, dev_layers, n, not args.separate_pool)

    # per-layer effective work and algorithmic bytes (x read once, y written once, compressed filter
    # and bias read once).  balg follows the per-convolution definition (full-size y) and feeds the
    # stack's HBM figure; blaunch counts what the launch itself has to move, i.e. the pooled tensor
    # where the pool is merged into the launch, and feeds the per-kernel figures.
    feff, balg, blaunch, kern = [], [], [], []
    for d in dev_layers:
        hw = d["hw"]
        feff.append(2.0 * d["f"].nnz * hw * hw * n)
        fixed = 8.0 * d["f"].nnz + 4.0 * (d["k"] + 1) + 4.0 * d["k"]
        balg.append(4.0 * n * hw * hw * (d["c"] + d["k"]) + fixed)
        yhw = (hw // 2) * (hw // 2) if d["fused"] else hw * hw
        blaunch.append(4.0 * n * (hw * hw * d["c"] + yhw * d["k"]) + fixed)
        v = fscnn.sf_variant_choice(d["f"], n, hw, hw, n4=(d["lay_in"] == fscnn.N4 or d["lay_out"] == fscnn.N4),
                                    pool=d["fused"])
        kern.append((fscnn.sf_variant_name(v) if v > 0 else "direct", d["lay_in"], d["lay_out"], d["fused"]))
    F, B = sum(feff), sum(balg)

    for _ in range(max(args.warmup, 1)):       # also builds every plan: the timed loop allocates nothing
        run_step(fscnn, x, dev_layers, n)
    torch.cuda.synchronize()

    # The tensors of the very chain that is timed below (same launches, layouts and automatic
    # configurations), compared with the oracle before the clock starts.
    check = None
    if not args.no_check:
        import oracle
        errs = []
        for li, g, o, a, nmax in chain_samples(fscnn, torch, np, oracle, x, dev_layers, n, args.check_points):
            if not np.all(np.isfinite(g)):
                errs.append(float("inf"))
                continue
            bound = (nmax + 2) * 2.0 ** -24 * 1.01 * a + 2.0 ** -24 * np.abs(o.astype(np.float64)) + 1e-45
            errs.append((rel_err(np, g, o), float(np.max(np.abs(g.astype(np.float64) - o) / bound))))
        worst = max(e[0] if isinstance(e, tuple) else e for e in errs)
        check = dict(max_rel_err=worst, tolerance=1e-4, passed=bool(worst <= 1e-4),
                     per_layer_rel_err=[e[0] if isinstance(e, tuple) else e for e in errs],
                     per_layer_share_of_fp32_summation_bound=[e[1] if isinstance(e, tuple) else None for e in errs],
                     points_per_layer=args.check_points,
                     rule="|g-o| / max(|o|, rms(o)) over sampled outputs + tensor corners of every layer, oracle fed "
                          "the GPU's previous tensor; pooled launches against the max of the definition over the window")
        if not check["passed"]:
            print("bench.py: the timed chain does NOT match the oracle: %r" % (check,), file=sys.stderr)
            sys.exit(3)

    ev = lambda: torch.cuda.Event(enable_timing=True)
    if args.separate_pool:
        events = [[(ev(), ev()) for _ in dev_layers] for _ in range(args.steps)]
    else:
        events = [[ev() for _ in range(len(dev_layers) + 1)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        run_step(fscnn, x, dev_layers, n, events[s])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3

    # per-layer kernel durations (HIP events on the launch stream, inside the timed region)
    if args.separate_pool:
        span = lambda s, li: events[s][li][0].elapsed_time(events[s][li][1])
    else:
        span = lambda s, li: events[s][li].elapsed_time(events[s][li + 1])
    layer_ms = [float(np.mean([span(s, li) for s in range(args.steps)])) for li in range(len(dev_layers))]
    layer_ms_median = [float(np.median([span(s, li) for s in range(args.steps)])) for li in range(len(dev_layers))]
    conv_ms = sum(layer_ms)
    # dominant kernel = the instantiation (configuration, layouts, pooled or not) with the largest
    # share of the step; its figures are means over its launches
    share = {}
    for li, kid in enumerate(kern):
        share.setdefault(kid, []).append(li)
    dom_id = max(share, key=lambda kid: sum(layer_ms[li] for li in share[kid]))
    dom = share[dom_id]
    dom_ms = float(np.mean([layer_ms[li] for li in dom]))
    dom_flop = float(np.mean([feff[li] for li in dom]))
    dom_bytes = float(np.mean([blaunch[li] for li in dom]))
    dom_tflops = dom_flop / (dom_ms * 1e-3) / 1e12
    lay = {fscnn.NCHW: "NCHW", fscnn.N4: "N4"}
    roofline = dict(bound="alu", achieved=dom_tflops, peak=FP32_VECTOR_PEAK_TFLOPS, unit="TFLOP/s",
                    frac=dom_tflops / FP32_VECTOR_PEAK_TFLOPS, traffic=None, traffic_source=None,
                    kernel="conv_sf_tiled_kernel %s %s->%s%s, layers %s" % (
                        dom_id[0], lay[dom_id[1]], lay[dom_id[2]], " +pool" if dom_id[3] else "",
                        ",".join(str(li + 1) for li in dom)),
                    launches_per_step=len(dom), launch_ms=dom_ms, flop_per_launch=dom_flop,
                    bytes_per_launch=dom_bytes,
                    peak_unpacked=FP32_UNPACKED_PEAK_TFLOPS, frac_unpacked=dom_tflops / FP32_UNPACKED_PEAK_TFLOPS,
                    hbm_gbs=dom_bytes / (dom_ms * 1e-3) / 1e9,
                    hbm_frac=dom_bytes / (dom_ms * 1e-3) / 1e9 / HBM_PEAK_GBS)
    # measured HBM bytes of that launch (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a copy
    # kernel of known size): taken from the committed summary of the same workload, else null
    # what the chip sustains on the hot loop's instruction mix alone (one LDS word per FMA)
    ceiling = probe_gather_fma(torch)
    roofline["measured_gather_fma_ceiling"] = ceiling
    roofline["frac_of_measured_ceiling"] = dom_tflops / ceiling
    traffic_file = os.path.join(ROOT, "profiles", "conv_sf_vgg16_n32_hbm_traffic.txt")
    if os.path.exists(traffic_file) and n == 32 and abs(args.keep - 0.05) < 1e-9:
        per_layer = {}
        measured_at = None
        for line in open(traffic_file):
            f = line.split()
            if len(f) == 4 and f[0].startswith("layer_"):
                per_layer[int(f[0][6:]) - 1] = float(f[3])
            elif len(f) >= 2 and f[0] == "commit:":
                measured_at = f[1]
        if all(li in per_layer for li in dom):
            roofline["traffic"] = float(np.mean([per_layer[li] for li in dom]))
            # not measured by this run: read from the committed counter summary, which names the
            # commit whose kernels the counters were collected on
            roofline["traffic_source"] = dict(file=os.path.relpath(traffic_file, ROOT), commit=measured_at)

    out = dict(
        metric="effective GFLOP/s (2*nnz*Ho*Wo*N) + HBM GB/s fraction, VGG16-shaped stack @95%",
        value=F / (ms_per_step * 1e-3) / 1e9, unit="effective GFLOP/s", n_gpus=1, steps=args.steps,
        warmup=args.warmup, ms_per_step=ms_per_step, higher_is_better=True, scaling="weak",
        vs_baseline=None, dtype="f32", data="synthetic",
        config=dict(workload="VGG16 conv stack, 13 layers 3x3 s1 p1 + 4 max-pools, N=%d, 224x224x3, "
                             "weight density %.2f (first layer dense), bias+ReLU fused" % (n, args.keep),
                    batch=n, effective_gflop_per_step=F / 1e9, algorithmic_gbytes_per_step=B / 1e9,
                    launched_gbytes_per_step=sum(blaunch) / 1e9,
                    nnz_total=int(sum(d["f"].nnz for d in dev_layers))),
        hbm=dict(algorithmic_gbs=B / (ms_per_step * 1e-3) / 1e9,
                 frac_of_peak=B / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, peak_gbs=HBM_PEAK_GBS),
        conv_kernels_ms=conv_ms, conv_only_effective_gflops=F / (conv_ms * 1e-3) / 1e9,
        layer_ms=[round(v, 4) for v in layer_ms],
        layer_ms_median=[round(v, 4) for v in layer_ms_median],
        layer_effective_tflops=[round(feff[i] / (layer_ms[i] * 1e-3) / 1e12, 2) for i in range(len(layer_ms))],
        # per layer: the launch's bytes over time, and the time of the roof that binds it -- HBM
        # (bytes / 8 TB/s) or the plain fp32 multiply-add rate, which is also the LDS rate of one
        # word per multiply-add (flop / 78.6 TFLOP/s) -- as a share of the measured time
        layer_launched_gbs=[round(blaunch[i] / (layer_ms[i] * 1e-3) / 1e9, 1) for i in range(len(layer_ms))],
        layer_roof=[("hbm" if blaunch[i] / (HBM_PEAK_GBS * 1e9) > feff[i] / (FP32_UNPACKED_PEAK_TFLOPS * 1e12)
                     else "alu/lds") for i in range(len(layer_ms))],
        layer_roof_frac=[round(max(blaunch[i] / (HBM_PEAK_GBS * 1e9), feff[i] / (FP32_UNPACKED_PEAK_TFLOPS * 1e12))
                               / (layer_ms[i] * 1e-3), 3) for i in range(len(layer_ms))],
        filter_compress_ms_all_layers=compress_ms,
        roofline=roofline,
        max_rel_err=None if check is None else check["max_rel_err"],
        check=check,
    )
    if not args.no_rows:
        out["other_rows"] = other_rows(fscnn, torch, inputs, np, dev_layers)
        import oracle
        out["config_rows"] = config_rows(fscnn, torch, inputs, np, oracle)
    if args.cpu_images > 0:
        out["cpu_baseline"] = cpu_baseline(inputs, args.keep, args.cpu_images)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
