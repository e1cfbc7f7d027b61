"""GPU parity on many small random problems: shapes, strides, paddings, layouts, densities and
epilogues drawn from a fixed seed, every one against the oracle through the C ABI.  Meant to
reach the corners the hand-picked cases miss (single rows and columns, one channel, ragged
groups of four images, tiles that are mostly padding)."""
import numpy as np
import pytest
import torch

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


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


def to_n4(x):
    n, c, h, w_ = x.shape
    g = (n + 3) // 4
    xp = np.zeros((g * 4, c, h, w_), np.float32)
    xp[:n] = x
    return np.ascontiguousarray(xp.reshape(g, 4, c, h, w_).transpose(0, 2, 3, 4, 1))


def from_n4(x4, n):
    g, c, h, w_, _ = x4.shape
    return np.ascontiguousarray(x4.transpose(0, 4, 1, 2, 3).reshape(g * 4, c, h, w_)[:n])


def draw(rng):
    """One problem: mostly the shapes the tiled kernels serve (3x3 at stride 1 or 2, 1x1), some
    that go to the direct kernel."""
    kind = rng.choice(["3x3", "3x3", "3x3s2", "1x1", "other"])
    n = int(rng.integers(1, 10))
    c = int(rng.choice([1, 2, 3, 7, 8, 9, 16, 31, 40, 70]))
    k = int(rng.choice([1, 2, 5, 16, 31, 33, 64, 70]))
    h = int(rng.choice([1, 2, 3, 7, 8, 13, 14, 17, 28, 33, 40]))
    w_ = int(rng.choice([1, 2, 3, 7, 15, 16, 17, 28, 31, 32, 33, 45]))
    if kind == "3x3":
        r = s = 3; stride = (1, 1); pad = (int(rng.integers(0, 3)),) * 2
    elif kind == "3x3s2":
        r = s = 3; stride = (2, 2); pad = (int(rng.integers(0, 2)),) * 2
    elif kind == "1x1":
        r = s = 1; stride = (1, 1); pad = (0, 0)
    else:
        r, s = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        stride = (int(rng.integers(1, 4)), int(rng.integers(1, 4)))
        pad = (int(rng.integers(0, 3)), int(rng.integers(0, 3)))
    if h + 2 * pad[0] < r or w_ + 2 * pad[1] < s:          # empty output: make the image larger
        h, w_ = h + r, w_ + s
    keep = float(rng.choice([0.02, 0.1, 0.3, 1.0]))
    act = rng.choice(["none", "relu", "leaky"])
    lay = rng.choice(["nchw", "n4", "n4in", "n4out"]) if kind != "other" else "nchw"
    return kind, n, c, k, h, w_, r, s, stride, pad, keep, act, lay


@pytest.mark.parametrize("block", range(6))
def test_random_small_problems(F, block):
    rng = np.random.default_rng([2212, block])
    for i in range(30):
        kind, n, c, k, h, w_, r, s, stride, pad, keep, act, lay = draw(rng)
        what = "block %d case %d: %s N%d C%d K%d %dx%d f%dx%d s%r p%r keep %g %s %s" % (
            block, i, kind, n, c, k, h, w_, r, s, stride, pad, keep, act, lay)
        print(what, flush=True)
        x, w, b = inputs.random_layer(1000 * block + i, n, c, k, h, w_, r, s, keep, x_zero_frac=0.3,
                                      bias=bool(rng.integers(0, 2)))
        o, a = oracle.conv2d_dense(x, w, stride, pad, b, act == "relu", want_abs=True,
                                   leaky=0.1 if act == "leaky" else None)
        f = F.filter_compress(dev(w))
        xin = dev(to_n4(x)) if lay in ("n4", "n4in") else dev(x)
        xl = F.N4 if lay in ("n4", "n4in") else F.NCHW
        yl = F.N4 if lay in ("n4", "n4out") else F.NCHW
        y = F.conv2d_sparse_filter(f, xin, stride, pad, dev(b), relu=(act == "relu"),
                                   leaky=0.1 if act == "leaky" else None, x_layout=xl, y_layout=yl, n=n)
        g = y.detach().cpu().numpy()
        g = from_n4(g, n) if yl == F.N4 else g
        nmax = int(np.count_nonzero(w.reshape(k, -1), axis=1).max())
        assert_parity(g, o, a, nmax, what)
        # merged pooling where it exists: 3x3 stride 1 through the tiled kernel, output at least 2x2
        ho, wo = o.shape[2:]
        if kind == "3x3" and act != "leaky" and ho >= 2 and wo >= 2 and i % 3 == 0:
            try:
                yp = F.conv2d_sparse_filter(f, xin, stride, pad, dev(b), relu=(act == "relu"), x_layout=xl,
                                            y_layout=yl, n=n, pool=True)
            except F.FscnnError as e:            # shapes whose kernel has no pooled form say so
                assert e.status == 4, what
                continue
            gp = yp.detach().cpu().numpy()
            gp = from_n4(gp, n) if yl == F.N4 else gp
            op = o[:, :, :ho // 2 * 2, :wo // 2 * 2].reshape(n, k, ho // 2, 2, wo // 2, 2).max(axis=(3, 5))
            ap = a[:, :, :ho // 2 * 2, :wo // 2 * 2].reshape(n, k, ho // 2, 2, wo // 2, 2).max(axis=(3, 5))
            assert_parity(gp, op, ap, nmax, what + " +pool")


@pytest.mark.parametrize("block", range(2))
def test_random_small_problems_sparse_input(F, block):
    rng = np.random.default_rng([2213, block])
    for i in range(25):
        n = int(rng.integers(1, 6))
        c = int(rng.choice([1, 3, 8, 9, 17, 40]))
        k = int(rng.choice([1, 5, 64, 70, 130, 260]))
        h = int(rng.choice([1, 2, 4, 5, 9, 14, 17]))
        w_ = int(rng.choice([1, 3, 4, 8, 13, 16, 21]))
        pad = (int(rng.integers(0, 3)),) * 2
        if h + 2 * pad[0] < 3 or w_ + 2 * pad[1] < 3:
            h, w_ = h + 3, w_ + 3
        zf = float(rng.choice([0.0, 0.5, 0.9, 1.0]))
        what = "si block %d case %d: N%d C%d K%d %dx%d p%r zeros %g" % (block, i, n, c, k, h, w_, pad, zf)
        print(what, flush=True)
        x, w, b = inputs.random_layer(5000 + 100 * block + i, n, c, k, h, w_, 3, 3, 1.0, x_zero_frac=zf)
        o, a = oracle.conv2d_dense(x, w, (1, 1), pad, b, True, want_abs=True)
        s = F.input_compress(dev(x))
        op, oc, ov = oracle.input_compress(x)
        prow, cidx, val = F.input_export(s)
        assert np.array_equal(prow, op) and np.array_equal(cidx, oc), what
        assert np.array_equal(val.view(np.uint32), ov.view(np.uint32)), what
        d = F.dense_filter_prepare(dev(w))
        for v in range(0, F.si_variant_count() + 1):
            g = F.conv2d_sparse_input_prepared(s, d, (1, 1), pad, dev(b), True, variant=v).cpu().numpy()
            assert_parity(g, o, a, c * 9, what + " variant %d" % v)
        g = F.conv2d_sparse_input(s, dev(w), (1, 1), pad, dev(b), True).cpu().numpy()
        assert_parity(g, o, a, c * 9, what + " unprepared")
