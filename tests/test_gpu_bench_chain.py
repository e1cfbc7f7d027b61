"""The chain bench.py times, at its own size, against the oracle.

bench.py's build_stack / alloc_buffers / run_step are run exactly as the benchmark runs them
(config 4: N=32, NCHW into layer 1, N4 tensors between layers, the 2x2 max-pools merged into
layers 2, 4, 7, 10, automatic kernel configurations), and every layer's stored tensor is compared
with the oracle on sampled outputs plus the tensor's corners, the oracle being fed the GPU's own
previous tensor.  Rule: tests/parity.py (1e-4 relative with the RMS floor, and the element-wise
forward bound of fp32 summation)."""
import numpy as np
import pytest
import torch

import bench
import oracle
from paper_2212_08815_amd import inputs
from parity import assert_parity

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def F():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2212_08815_amd import fscnn
    fscnn.lib()
    return fscnn


@pytest.mark.parametrize("fuse_pool", [True, False])
def test_bench_chain_config4_full_size(F, fuse_pool):
    n = 32
    x, dev_layers, _ = bench.build_stack(F, torch, inputs, n, 0.05)
    bench.alloc_buffers(F, torch, dev_layers, n, fuse_pool)
    out = bench.run_step(F, x, dev_layers, n)
    torch.cuda.synchronize()
    assert tuple(out.shape) == (n, 512, 14, 14)
    seen = 0
    for li, g, o, a, nmax in bench.chain_samples(F, torch, np, oracle, x, dev_layers, n, npts=4000, seed=4):
        assert g.size >= 4000
        assert_parity(g, o, a, nmax, "bench chain layer %d (%s)" % (li + 1, "merged pool" if fuse_pool else "separate pool"))
        assert g.min() >= 0.0          # ReLU output
        seen += 1
    assert seen == 13
    # a second pass over the same buffers reproduces the first bit for bit (one writer per output)
    first = dev_layers[-1]["y"].clone()
    bench.run_step(F, x, dev_layers, n)
    torch.cuda.synchronize()
    assert torch.equal(first, dev_layers[-1]["y"])


def test_bench_chain_sampler_is_pinned_by_a_whole_tensor_case(F):
    """The sampler itself (index arithmetic for N4 and pooled tensors) against whole tensors on a
    small chain: N=5 (ragged image group), 28x28 input, three layers with a merged pool."""
    n = 5
    x, layers = inputs.vgg16_stack(4, n, 0.2, layers=3, size_div=8)
    dev_layers = []
    for L in layers:
        w = torch.from_numpy(L["w"]).cuda()
        dev_layers.append(dict(w=w, bias=torch.from_numpy(L["bias"]).cuda(), relu=L["relu"], pool=L["pool_after"],
                               hw=L["hw"], k=L["w"].shape[0], c=L["w"].shape[1], f=F.filter_compress(w)))
    bench.alloc_buffers(F, torch, dev_layers, n, True)
    xd = torch.from_numpy(x).cuda()
    bench.run_step(F, xd, dev_layers, n)
    torch.cuda.synchronize()
    cur = x
    for (li, g, o, a, nmax), L, d in zip(bench.chain_samples(F, torch, np, oracle, xd, dev_layers, n, npts=10 ** 9),
                                         layers, dev_layers):
        csr = oracle.filter_compress(L["w"])
        full = oracle.conv2d_sparse_filter(cur, csr, L["w"].shape, L["stride"], L["pad"], L["bias"], L["relu"])
        if L["pool_after"]:
            full = oracle.maxpool2x2(full)
        got = bench.to_host_nchw(F, d["y"], d["lay_out"], n)
        assert g.size == full.size            # every element was sampled
        assert np.array_equal(o, full.ravel()) and np.array_equal(g, got.ravel())
        assert_parity(g, o, a, nmax, "small chain layer %d" % li)
        cur = got


def test_bench_chain_config3_full_size_eager_and_as_one_graph(F):
    """Config 3 as bench.py's config_rows runs it: N=1, 90 % weight sparsity, NCHW tensors throughout,
    plans and channel-split scratch prepared beforehand on the stream that runs and captures it.
    The eager chain against the oracle layer by layer; then one HIP graph of the same launches,
    replayed with eager work and synchronisations in between, every replay bit-equal to the eager
    result (the channel-split layers add their parts in a fixed order)."""
    n = 1
    x, L, _ = bench.build_stack(F, torch, inputs, n, 0.10, config_id=3)
    bench.alloc_buffers(F, torch, L, n, True, n4=False)
    assert all(d["lay_in"] == F.NCHW and d["lay_out"] == F.NCHW for d in L)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for d in L:
            F.filter_prepare(d["f"], n, d["hw"], d["hw"], (1, 1), (1, 1), 0, d["lay_in"], d["lay_out"], d["fused"])
        out = bench.run_step(F, x, L, n)
        side.synchronize()
        assert tuple(out.shape) == (n, 512, 14, 14)
        seen = 0
        for li, g, o, a, nmax in bench.chain_samples(F, torch, np, oracle, x, L, n, npts=3000, seed=5):
            assert_parity(g, o, a, nmax, "config 3 chain layer %d" % (li + 1))
            seen += 1
        assert seen == 13
        eager = [d["y"].clone() for d in L]
        side.synchronize()
    free0 = torch.cuda.mem_get_info()[0]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        bench.run_step(F, x, L, n)
    for r in range(4):
        for d in L:
            d["y"].fill_(float(r) - 7.0)       # eager work between the replays; stale results cannot pass
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for li, (d, e) in enumerate(zip(L, eager)):
            assert torch.equal(d["y"], e), "replay %d, layer %d" % (r, li + 1)
    del graph
    assert torch.cuda.mem_get_info()[0] >= free0 - (64 << 20)     # capture made no large allocation
