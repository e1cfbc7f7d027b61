"""Seeded synthetic inputs shaped like the paper's workloads.

This module holds NO arithmetic of the method: it only draws random tensors
(numpy's PCG64, seeded per (config, layer, tensor)) and lists layer shapes.  It
is the one module the tests hand to both the CPU oracle and the HIP path.

The paper (Sec. 6) times VGG16 with filter densities 1..100 % and batch sizes
1..64 in 32-bit float; its trained sparse weights and images are not available,
so Bernoulli-masked Gaussian weights and random images of the same shapes stand
in for them.
"""
import numpy as np

# VGG16 convolution stack: (C_in, C_out, input height = width); all 3x3, stride
# 1, pad 1; a 2x2/2 max-pool follows the layers listed in VGG16_POOL_AFTER.
VGG16_LAYERS = [
    (3, 64, 224), (64, 64, 224),
    (64, 128, 112), (128, 128, 112),
    (128, 256, 56), (256, 256, 56), (256, 256, 56),
    (256, 512, 28), (512, 512, 28), (512, 512, 28),
    (512, 512, 14), (512, 512, 14), (512, 512, 14),
]
VGG16_POOL_AFTER = (1, 3, 6, 9)      # layer indices followed by a pool inside the conv stack

_TAGS = {"x": 1, "w": 2, "mask": 3, "bias": 4}


def _rng(config_id, layer, tag):
    return np.random.default_rng([int(config_id), int(layer), _TAGS[tag]])


def masked_normal(rng_w, rng_m, shape, std, keep):
    """N(0, std) entries, each kept with probability `keep` (i.i.d.), else exactly 0."""
    w = rng_w.standard_normal(shape, dtype=np.float32) * np.float32(std)
    if keep < 1.0:
        m = rng_m.random(shape, dtype=np.float32) < np.float32(keep)
        w = np.where(m, w, np.float32(0)).astype(np.float32)
    # a kept Gaussian draw is never exactly 0 in practice; nothing else is assumed
    return np.ascontiguousarray(w)


def config1():
    """Single small layer: N=1, C=16, K=32, 3x3, s1, p1, 32x32, 90 % zeros, seed 0."""
    rng = np.random.default_rng(0)
    x = rng.random((1, 16, 32, 32), dtype=np.float32)
    w = masked_normal(rng, rng, (32, 16, 3, 3), 0.05, 0.10)
    return dict(x=x, w=w, bias=None, relu=False, stride=(1, 1), pad=(1, 1))


def config2(n=1):
    """VGG16-shaped layer: C=K=256, 56x56, ReLU(N(0,1)) input, 95 % zeros, bias, ReLU."""
    x = np.maximum(_rng(2, 0, "x").standard_normal((n, 256, 56, 56), dtype=np.float32), 0)
    w = masked_normal(_rng(2, 0, "w"), _rng(2, 0, "mask"), (256, 256, 3, 3), 0.02, 0.05)
    b = _rng(2, 0, "bias").standard_normal(256, dtype=np.float32) * np.float32(0.01)
    return dict(x=np.ascontiguousarray(x), w=w, bias=b, relu=True, stride=(1, 1), pad=(1, 1))


def vgg16_stack(config_id, n, keep, layers=None, size_div=1):
    """Weights/biases of the 13-layer stack plus the input image batch.

    Layer 0 is dense, the others keep each weight with probability `keep`.
    Weight scale sqrt(2 / (9 * C * density)) keeps activations O(1) through the
    ReLU chain (the paper gives no scale).  `size_div` shrinks the spatial
    size (224 / size_div) for CPU-sized test cases; `layers` limits the depth.
    """
    specs = VGG16_LAYERS if layers is None else VGG16_LAYERS[:layers]
    hw0 = 224 // size_div
    x = _rng(config_id, 0, "x").random((n, 3, hw0, hw0), dtype=np.float32)
    out = []
    for li, (c, k, hw) in enumerate(specs):
        d = 1.0 if li == 0 else keep
        std = float(np.sqrt(2.0 / (9.0 * c * d)))
        w = masked_normal(_rng(config_id, li, "w"), _rng(config_id, li, "mask"), (k, c, 3, 3), std, d)
        b = _rng(config_id, li, "bias").standard_normal(k, dtype=np.float32) * np.float32(0.01)
        out.append(dict(w=w, bias=b, relu=True, stride=(1, 1), pad=(1, 1),
                        hw=hw // size_div, pool_after=li in VGG16_POOL_AFTER))
    return x, out


def config3(**kw):
    """Full VGG16 conv stack, N=1, 90 % weight sparsity (first layer dense)."""
    return vgg16_stack(3, 1, 0.10, **kw)


def config4(n=32, **kw):
    """Full VGG16 conv stack, N=32, 95 % weight sparsity (first layer dense)."""
    return vgg16_stack(4, n, 0.05, **kw)


def yolo_layers():
    """Convolution layers of the Darknet-53 feature extractor (the backbone of YOLOv3, as its
    public description lists them): (C_in, C_out, filter extent, stride), in order.  Residual
    additions, up-sampling and detection heads are not convolutions and are left out: the
    stack below is the plain chain of these 52 layers."""
    layers = [(3, 32, 3, 1)]
    c = 32
    for blocks in (1, 2, 8, 8, 4):
        layers.append((c, 2 * c, 3, 2))          # down-sampling convolution
        c *= 2
        for _ in range(blocks):
            layers.append((c, c // 2, 1, 1))     # bottleneck
            layers.append((c // 2, c, 3, 1))
    return layers


def yolo_stack(n, keep, hw0=416, width_div=1, config_id=6):
    """YOLO-shaped stack (the paper's second workload, Sec. 6): Darknet-53's 52 convolution
    layers as a chain, 3x3 (stride 1 and 2, pad 1) and 1x1 filters, LeakyReLU(0.1), first layer
    dense, the others Bernoulli(keep); batch-norm is taken as folded into weights and bias.
    `hw0` is the input size, `width_div` divides every channel count (small test cases)."""
    x = _rng(config_id, 0, "x").random((n, 3, hw0, hw0), dtype=np.float32)
    out = []
    hw = hw0
    for li, (c, k, r, st) in enumerate(yolo_layers()):
        c = c if li == 0 else max(c // width_div, 1)
        k = max(k // width_div, 1)
        d = 1.0 if li == 0 else keep
        # LeakyReLU(0.1) keeps about half of the variance: same scale rule as the VGG16 stack
        std = float(np.sqrt(2.0 / (r * r * c * d)))
        w = masked_normal(_rng(config_id, li, "w"), _rng(config_id, li, "mask"), (k, c, r, r), std, d)
        b = _rng(config_id, li, "bias").standard_normal(k, dtype=np.float32) * np.float32(0.01)
        out.append(dict(w=w, bias=b, leaky=0.1, stride=(st, st), pad=(r // 2, r // 2), hw=hw))
        hw = (hw + 2 * (r // 2) - r) // st + 1
    return x, out


CONFIG5_KEEP = (0.5, 0.2, 0.1, 0.05, 0.01)


def config5(keep, n=8, c=512, k=512, hw=28):
    """conv4-shaped layer for the sparsity sweep; input ReLU(N(-0.5,1)) (~69 % zeros)."""
    tag = int(round(keep * 1000))
    x = np.maximum(_rng(5, 0, "x").standard_normal((n, c, hw, hw), dtype=np.float32) - np.float32(0.5), 0)
    w = masked_normal(_rng(5, tag, "w"), _rng(5, tag, "mask"), (k, c, 3, 3),
                      float(np.sqrt(2.0 / (9.0 * c * keep))), keep)
    b = _rng(5, tag, "bias").standard_normal(k, dtype=np.float32) * np.float32(0.01)
    return dict(x=np.ascontiguousarray(x), w=w, bias=b, relu=True, stride=(1, 1), pad=(1, 1))


def random_layer(seed, n, c, k, h, w_, r, s, keep, x_zero_frac=0.0, integer=False, bias=True):
    """Free-form layer for edge-case tests.  integer=True draws small integers
    (|v| <= 4) so that every partial sum is exact in fp32."""
    rng = np.random.default_rng([99, int(seed)])
    if integer:
        x = rng.integers(-4, 5, (n, c, h, w_)).astype(np.float32)
        wt = rng.integers(-4, 5, (k, c, r, s)).astype(np.float32)
        b = rng.integers(-4, 5, k).astype(np.float32) if bias else None
    else:
        x = rng.standard_normal((n, c, h, w_), dtype=np.float32)
        wt = rng.standard_normal((k, c, r, s), dtype=np.float32)
        b = rng.standard_normal(k, dtype=np.float32) if bias else None
    if keep < 1.0:
        wt = np.where(rng.random(wt.shape) < keep, wt, 0).astype(np.float32)
    if x_zero_frac > 0.0:
        x = np.where(rng.random(x.shape) < x_zero_frac, 0, x).astype(np.float32)
    return np.ascontiguousarray(x), np.ascontiguousarray(wt), b
