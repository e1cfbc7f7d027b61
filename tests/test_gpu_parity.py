"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element,
on the same seeded inputs.  Integer / index work must match bit for bit; fp32 results within
the rule of tests/parity.py."""
import ctypes

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
    fscnn.lib()          # raises if libfscnn.so was not built: no fallback
    return fscnn


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.detach().cpu().numpy()


def bits(a):
    return np.ascontiguousarray(a, np.float32).view(np.uint32)


def row_nmax(w):
    return int(np.count_nonzero(w.reshape(w.shape[0], -1), axis=1).max())


def gpu_conv(F, x, w, stride, pad, bias, relu, variant=0, filt=None):
    f = filt or F.filter_compress(dev(w))
    y = F.conv2d_sparse_filter(f, dev(x), stride, pad, dev(bias), relu, variant=variant)
    torch.cuda.synchronize()
    return host(y)


def tiled_variants(F, n4_only=False, extent="3x3"):
    """Kernel configurations for a filter extent that take NCHW tensors (or, with n4_only, those
    built for N4 only).  Configurations for 1x1 filters carry "_r1s1" in their name, those for
    3x3 filters at stride 2 "_st2" (extent "3x3s2")."""
    names = {v: F.sf_variant_name(v) for v in range(1, F.sf_variant_count() + 1)}
    kind = lambda nm: "1x1" if "_r1s1" in nm else "3x3s2" if "_st2" in nm else "3x3"
    return [v for v, nm in names.items() if nm.endswith("_n4only") == n4_only and kind(nm) == extent]


# ------------------------------------------------------------------ A1/A2: filter compression
@pytest.mark.parametrize("shape,keep", [((32, 16, 3, 3), 0.1), ((5, 7, 3, 3), 0.5), ((3, 2, 5, 4), 1.0),
                                        ((130, 33, 1, 1), 0.3), ((64, 300, 3, 3), 0.05), ((2, 1, 1, 1), 0.5)])
def test_filter_compress_bit_exact(F, shape, keep):
    _, w, _ = inputs.random_layer(sum(shape), 1, shape[1], shape[0], 4, 4, shape[2], shape[3], keep)
    f = F.filter_compress(dev(w))
    rp, ix, vl = F.filter_export(f)
    orp, oix, ovl = oracle.filter_compress(w)
    assert f.nnz == orp[-1]
    assert np.array_equal(rp, orp) and np.array_equal(ix, oix) and np.array_equal(bits(vl), bits(ovl))


def test_filter_compress_special_values_and_empty_rows(F):
    w = np.zeros((4, 3, 3, 3), np.float32)
    w[0, 0, 0, 1] = -0.0
    w[0, 1, 0, 0] = np.nan
    w[1, 0, 0, 2] = np.float32(1e-42)
    w[3, 2, 2, 2] = -3.5
    f = F.filter_compress(dev(w))
    rp, ix, vl = F.filter_export(f)
    orp, oix, ovl = oracle.filter_compress(w)
    assert list(rp) == list(orp) == [0, 1, 2, 2, 3]
    assert np.array_equal(ix, oix) and np.array_equal(bits(vl), bits(ovl))
    z = F.filter_compress(dev(np.zeros((3, 2, 3, 3), np.float32)))
    rp, ix, vl = F.filter_export(z)
    assert z.nnz == 0 and list(rp) == [0, 0, 0, 0] and ix.size == 0
    # an all-zero bank convolves to bias (then ReLU)
    x = np.random.default_rng(0).standard_normal((2, 2, 9, 70)).astype(np.float32)
    b = np.array([-1.0, 0.5, 2.0], np.float32)
    y = host(F.conv2d_sparse_filter(z, dev(x), (1, 1), (1, 1), dev(b), True))
    assert np.array_equal(y, np.broadcast_to(np.maximum(b, 0)[None, :, None, None], y.shape))


# ------------------------------------------------------------------ A3: regrouped plan
def test_variant_choice_names_the_kernel_that_runs(F):
    _, w, _ = inputs.random_layer(5, 1, 24, 40, 4, 4, 3, 3, keep=0.2)
    f = F.filter_compress(dev(w))
    n = F.sf_variant_count()
    for N, hw in ((32, 56), (32, 28), (32, 14), (8, 224), (1, 56), (2, 9)):
        v = F.sf_variant_choice(f, N, hw, hw)
        assert 1 <= v <= n
        assert F.filter_plan_export(f, N, hw, hw, (1, 1), (1, 1))["variant"] == v
        vp = F.sf_variant_choice(f, N, hw, hw, n4=True, pool=True)
        assert 1 <= vp <= n and not F.sf_variant_name(vp).endswith("_n4only")
    assert F.sf_variant_choice(f, 4, 56, 56, stride=(3, 3)) == -1      # stride 3: the direct kernel
    assert "_st2" in F.sf_variant_name(F.sf_variant_choice(f, 4, 56, 56, stride=(2, 2)))
    with pytest.raises(F.FscnnError):
        F.sf_variant_choice(f, 0, 56, 56)


def test_plan_regroup_decodes_to_the_canonical_rows(F):
    _, w, _ = inputs.random_layer(21, 1, 37, 70, 4, 4, 3, 3, keep=0.15)
    K, C, R, S = w.shape
    f = F.filter_compress(dev(w))
    orp, oix, ovl = oracle.filter_compress(w)
    for v in tiled_variants(F):
        p = F.filter_plan_export(f, 1, 30, 30, (1, 1), (1, 1), variant=v)
        assert not p["direct"] and p["variant"] == v
        CC, KG, NCH, NG, SL, WV = p["CC"], p["KG"], p["NCH"], p["NG"], p["SLOTS"], p["WAVES"]
        assert NCH == -(-C // CC) and NG == -(-K // KG) and KG == SL * WV
        if p["DENSE"]:
            # the taps-outer form: every tap of every chunk, SLOTS weights per tap, zeros where
            # the bank stores nothing
            T = CC * R * S
            assert p["nrec"] == NG * WV * NCH * T * SL
            off = p["rec_off"].reshape(NG, WV, NCH, T, SL)
            val = p["rec_val"].reshape(NG, WV, NCH, T, SL)
            tt = np.arange(T)
            want_off = ((((tt // (R * S)) * p["IN_ROWS"]) + (tt % (R * S)) // S) * p["PITCH"] + tt % S) * p["BV"] * 4
            assert np.array_equal(off, np.broadcast_to(want_off[None, None, None, :, None], off.shape))
            dense = np.zeros((NG * KG, NCH * CC, R, S), np.float32)
            dense[:K, :C] = w
            want = dense.reshape(NG, WV, SL, NCH, T).transpose(0, 1, 3, 4, 2)
            assert np.array_equal(bits(val), bits(want))
            continue
        seg = p["segptr"]
        assert seg[0] == 0 and np.all(np.diff(seg) >= 0) and seg[-1] == orp[-1] == p["nrec"]
        q = p["rec_off"].astype(np.int64) // (4 * p["BV"])
        assert np.all(p["rec_off"] % (4 * p["BV"]) == 0)
        s = q % p["PITCH"]
        r = (q // p["PITCH"]) % p["IN_ROWS"]
        cl = q // (p["PITCH"] * p["IN_ROWS"])
        seen = 0
        for g in range(NG):
            for wv in range(WV):
                for ci in range(NCH):
                    for j in range(SL):
                        b = ((g * WV + wv) * NCH + ci) * SL + j
                        k = g * KG + wv * SL + j
                        lo, hi = seg[b], seg[b + 1]
                        if k >= K:
                            assert lo == hi
                            continue
                        row = slice(orp[k], orp[k + 1])
                        flat = oix[row].astype(np.int64)
                        sel = (flat // (R * S)) // CC == ci        # entries of this chunk, in row order
                        got_flat = ((cl[lo:hi] + ci * CC) * R + r[lo:hi]) * S + s[lo:hi]
                        assert np.array_equal(got_flat, flat[sel])
                        assert np.all(cl[lo:hi] < CC) and np.all(r[lo:hi] < R) and np.all(s[lo:hi] < S)
                        assert np.array_equal(bits(p["rec_val"][lo:hi]), bits(ovl[row][sel]))
                        seen += hi - lo
        assert seen == orp[-1]


# ------------------------------------------------------------------ A4-A6: tiled convolution
CASES = [
    # n, c, k, h, w, keep, pad, bias, relu
    (1, 16, 32, 32, 32, 0.10, (1, 1), False, False),
    (2, 19, 37, 23, 71, 0.30, (1, 1), True, True),      # ragged everything, several tiles in x
    (1, 3, 64, 40, 130, 1.00, (1, 1), True, True),      # dense first-layer shape, 3 tiles in x
    (3, 40, 9, 14, 14, 0.20, (1, 1), True, False),
    (1, 33, 65, 17, 29, 0.05, (0, 0), True, True),      # no padding: output smaller than input
    (1, 8, 8, 9, 9, 0.50, (2, 2), False, True),         # pad wider than the halo of a 3x3
    (2, 64, 64, 28, 28, 0.05, (1, 1), True, True),
    (1, 5, 4, 3, 3, 0.60, (1, 1), True, False),         # image smaller than any tile
    (1, 2, 3, 1, 1, 1.00, (1, 1), True, False),         # 1x1 image
]


@pytest.mark.parametrize("case", CASES)
def test_conv_sparse_filter_matches_oracle_all_variants(F, case):
    n, c, k, h, w_, keep, pad, use_b, relu = case
    x, w, b = inputs.random_layer(hash(case) % 1000, n, c, k, h, w_, 3, 3, keep, bias=use_b)
    csr = oracle.filter_compress(w)
    o, a = oracle.conv2d_sparse_filter(x, csr, w.shape, (1, 1), pad, b, relu, want_abs=True)
    f = F.filter_compress(dev(w))
    for v in [0] + tiled_variants(F):
        g = gpu_conv(F, x, w, (1, 1), pad, b, relu, variant=v, filt=f)
        assert_parity(g, o, a, row_nmax(w), "case %r variant %d" % (case, v))


@pytest.mark.parametrize("n,h,w_,pad", [(1, 30, 21, (1, 1)), (1, 13, 40, (1, 1)), (2, 9, 18, (1, 1)), (1, 5, 7, (0, 0)),
                                        (1, 3, 3, (1, 1)), (2, 2, 35, (1, 1)), (1, 61, 17, (2, 2)), (2, 28, 28, (1, 1))])
def test_band_mode_for_one_or_two_images(F, n, h, w_, pad):
    # One or two images through NCHW tensors: the four-image configurations give a lane's image
    # slots to bands of the image.  Heights that do not divide into the bands, bands shorter than
    # a tile and shorter than the halo, heights below the number of bands; with and without the
    # merged pool (odd heights: the pool drops the last row), whole tensors against the oracle;
    # integer data: bit-exact.
    c, k = 21, 34
    x, w, b = inputs.random_layer(n * 1000 + h * 10 + w_, n, c, k, h, w_, 3, 3, 0.3, integer=True)
    want = oracle.conv2d_dense(x, w, (1, 1), pad, b, True)
    ho, wo = want.shape[2:]
    f = F.filter_compress(dev(w))
    banded = 0
    for v in [0] + tiled_variants(F):
        vv = v or F.sf_variant_choice(f, n, h, w_)
        for pool in (False, True):
            if pool and (ho < 2 or wo < 2):
                continue
            bands, rows = F.sf_band_choice(vv, n, ho, pool=pool) if vv > 0 else (1, ho)
            if vv > 0 and F.sf_variant_name(vv).startswith("bv4"):
                assert bands == 4 // n and bands * rows >= ho and (not pool or rows % 2 == 0)
                assert (rows - (2 if pool else 1)) * bands < ho, "the shortest bands that cover the image"
                banded += 1
            else:
                assert (bands, rows) == (1, ho)
            try:
                got = host(F.conv2d_sparse_filter(f, dev(x), (1, 1), pad, dev(b), True, variant=v, pool=pool))
            except F.FscnnError as e:
                assert e.status == 4 and v != 0 and pool
                continue
            ref = oracle.maxpool2x2(want) if pool else want
            assert np.array_equal(got, ref), "n %d %dx%d variant %d pool %d bands %d x %d rows" % (n, h, w_, v, pool, bands, rows)
    assert banded >= 8
    # 3x3 at stride 2 and 1x1 filters through their own configurations, in bands as well
    for r, stride, pd, extent in ((3, (2, 2), (1, 1), "3x3s2"), (1, (1, 1), (0, 0), "1x1")):
        xs, ws, bs = inputs.random_layer(n * 77 + h + r, n, c, k, h, w_, r, r, 0.3, integer=True)
        ref = oracle.conv2d_dense(xs, ws, stride, pd, bs, True)
        fs = F.filter_compress(dev(ws))
        for v in [0] + tiled_variants(F, extent=extent):
            vv = v or F.sf_variant_choice(fs, n, h, w_, stride=stride)
            if vv > 0:
                assert F.sf_band_choice(vv, n, ref.shape[2])[0] == 4 // n
            got = host(F.conv2d_sparse_filter(fs, dev(xs), stride, pd, dev(bs), True, variant=v))
            assert np.array_equal(got, ref), "n %d %dx%d %s variant %d" % (n, h, w_, extent, v)
    assert F.sf_band_choice(F.sf_variant_choice(f, n, h, w_, n4=True), n, ho, n4=True) == (1, ho)   # N4 tensors: no bands
    assert F.sf_band_choice(F.sf_variant_choice(f, 3, h, w_), 3, ho) == (1, ho)                     # three images: none


def test_integer_data_is_bit_exact_all_variants(F):
    # every partial sum is an exact small integer: any summation order gives the same bits
    x, w, b = inputs.random_layer(31, 2, 21, 34, 19, 67, 3, 3, keep=0.3, integer=True)
    o = oracle.conv2d_sparse_filter(x, oracle.filter_compress(w), w.shape, (1, 1), (1, 1), b, True)
    f = F.filter_compress(dev(w))
    for v in [0] + tiled_variants(F):
        g = gpu_conv(F, x, w, (1, 1), (1, 1), b, True, variant=v, filt=f)
        assert np.array_equal(g, o), "variant %d" % v


def test_impulses_pin_orientation_on_the_gpu(F):
    rng = np.random.default_rng(4)
    x = rng.standard_normal((1, 20, 11, 70)).astype(np.float32)
    for (k0, c0, r0, s0) in [(0, 0, 0, 0), (5, 17, 2, 1), (8, 19, 1, 2), (2, 16, 0, 2)]:
        w = np.zeros((9, 20, 3, 3), np.float32)
        w[k0, c0, r0, s0] = 1.0
        f = F.filter_compress(dev(w))
        for v in [0] + tiled_variants(F):
            y = gpu_conv(F, x, w, (1, 1), (1, 1), None, False, variant=v, filt=f)
            xp = np.pad(x[0, c0], 1)
            want = xp[r0:r0 + 11, s0:s0 + 70]
            assert np.array_equal(y[0, k0], want), (k0, c0, r0, s0, v)
            assert not np.delete(y[0], k0, axis=0).any()
    # single input pixel: the output patch around it is the un-flipped filter read backwards
    w = rng.standard_normal((4, 3, 3, 3)).astype(np.float32)
    xi = np.zeros((1, 3, 12, 12), np.float32)
    xi[0, 1, 6, 5] = 1.0
    y = gpu_conv(F, xi, w, (1, 1), (1, 1), None, False)
    assert np.array_equal(y[0, :, 5:8, 4:7], w[:, 1, ::-1, ::-1])


def test_dense_filter_equals_dense_convolution(F):
    x, w, b = inputs.random_layer(41, 1, 12, 10, 20, 66, 3, 3, keep=1.0)
    o, a = oracle.conv2d_dense(x, w, (1, 1), (1, 1), b, False, want_abs=True)
    f = F.filter_compress(dev(w))
    assert f.nnz == w.size
    assert_parity(gpu_conv(F, x, w, (1, 1), (1, 1), b, False, filt=f), o, a, row_nmax(w), "dense")


# ------------------------------------------------------------------ batch-interleaved (N4) tensors
def to_n4(x):
    """numpy NCHW -> the N4 array ceil(N/4) x C x H x W x 4 (pad images = 0)."""
    n, c, h, w_ = x.shape
    g = (n + 3) // 4
    xp = np.zeros((g * 4, c, h, w_), np.float32)
    xp[:n] = x
    return np.ascontiguousarray(xp.reshape(g, 4, c, h, w_).transpose(0, 2, 3, 4, 1))


def from_n4(x4, n):
    g, c, h, w_, _ = x4.shape
    return np.ascontiguousarray(x4.transpose(0, 4, 1, 2, 3).reshape(g * 4, c, h, w_)[:n])


@pytest.mark.parametrize("n", [1, 4, 6])
def test_layout_convert_and_pool_n4(F, n):
    x = np.random.default_rng(n).standard_normal((n, 5, 7, 10)).astype(np.float32)
    x4 = host(F.layout_convert(dev(x), F.NCHW))
    assert np.array_equal(x4, to_n4(x))
    assert np.array_equal(host(F.layout_convert(dev(to_n4(x)), F.N4, n=n)), x)
    p4 = host(F.maxpool2x2(dev(to_n4(x)), layout=F.N4, n=n))
    assert np.array_equal(from_n4(p4, n), oracle.maxpool2x2(x))


@pytest.mark.parametrize("case", [(6, 19, 37, 23, 71, 0.30, (1, 1)), (4, 40, 9, 14, 14, 0.20, (1, 1)),
                                  (5, 8, 70, 28, 28, 0.10, (1, 1)), (9, 3, 8, 12, 66, 1.0, (0, 0))])
def test_conv_n4_layouts_match_oracle(F, case):
    n, c, k, h, w_, keep, pad = case
    x, w, b = inputs.random_layer(sum(case[:5]), n, c, k, h, w_, 3, 3, keep)
    o, a = oracle.conv2d_sparse_filter(x, oracle.filter_compress(w), w.shape, (1, 1), pad, b, True, want_abs=True)
    f = F.filter_compress(dev(w))
    xs = {F.NCHW: dev(x), F.N4: dev(to_n4(x))}
    tested = 0
    for v in [0] + tiled_variants(F) + tiled_variants(F, n4_only=True):
        for xl in (F.NCHW, F.N4):
            for yl in (F.NCHW, F.N4):
                if xl == F.NCHW and yl == F.NCHW:
                    continue
                try:
                    y = F.conv2d_sparse_filter(f, xs[xl], (1, 1), pad, dev(b), True, variant=v,
                                               x_layout=xl, y_layout=yl, n=n)
                except F.FscnnError as e:
                    assert e.status == 4 and v != 0          # a one-image-per-lane configuration
                    continue
                torch.cuda.synchronize()
                g = host(y) if yl == F.NCHW else from_n4(host(y), n)
                assert_parity(g, o, a, row_nmax(w), "N4 case %r variant %d layouts %d->%d" % (case, v, xl, yl))
                tested += 1
    assert tested >= 6 + len(tiled_variants(F, n4_only=True))


# ------------------------------------------------------------------ channel-split mode (small problems)
@pytest.mark.parametrize("case", [(1, 200, 40, 14, 14, 0.10, True, True), (3, 130, 70, 9, 20, 0.30, True, False),
                                  (2, 512, 33, 7, 7, 0.05, False, True), (5, 96, 64, 28, 28, 0.10, True, True)])
def test_small_problems_split_the_channel_range(F, case):
    """Few work-groups and many input channels: the automatic configuration splits the channel
    chunks over several groups (a copy of the partial sums per part, added up in the order of the
    parts with bias + ReLU by a finishing pass; with one or two images the groups work on bands)."""
    n, c, k, h, w_, keep, use_b, relu = case
    x, w, b = inputs.random_layer(sum(case[:5]), n, c, k, h, w_, 3, 3, keep, bias=use_b)
    csr = oracle.filter_compress(w)
    o, a = oracle.conv2d_sparse_filter(x, csr, w.shape, (1, 1), (1, 1), b, relu, want_abs=True)
    f = F.filter_compress(dev(w))
    bd = dev(b) if use_b else None
    g = host(F.conv2d_sparse_filter(f, dev(x), (1, 1), (1, 1), bd, relu))
    assert_parity(g, o, a, row_nmax(w), "split case %r NCHW" % (case,))
    g4 = F.conv2d_sparse_filter(f, dev(to_n4(x)), (1, 1), (1, 1), bd, relu, x_layout=F.N4, y_layout=F.N4, n=n)
    assert_parity(from_n4(host(g4), n), o, a, row_nmax(w), "split case %r N4" % (case,))
    # same call twice into the same buffer: the result does not accumulate across calls
    out = F.conv2d_sparse_filter(f, dev(x), (1, 1), (1, 1), bd, relu)
    F.conv2d_sparse_filter(f, dev(x), (1, 1), (1, 1), bd, relu, out=out)
    assert_parity(host(out), o, a, row_nmax(w), "split case %r second call" % (case,))
    # integer data: exact whatever the order of the partial sums
    xi, wi, bi = inputs.random_layer(9, n, c, k, h, w_, 3, 3, keep, integer=True)
    want = oracle.conv2d_dense(xi, wi, (1, 1), (1, 1), bi, relu)
    assert np.array_equal(host(F.conv2d_sparse_filter(F.filter_compress(dev(wi)), dev(xi), (1, 1), (1, 1), dev(bi), relu)), want)


# ------------------------------------------------------------------ merged convolution + max-pool
@pytest.mark.parametrize("case", [(6, 19, 37, 23, 71, 0.30, (1, 1)), (4, 40, 9, 14, 14, 0.20, (1, 1)),
                                  (1, 8, 70, 28, 28, 0.10, (1, 1)), (5, 3, 8, 13, 66, 1.0, (0, 0))])
def test_merged_conv_pool_matches_oracle_conv_then_pool(F, case):
    n, c, k, h, w_, keep, pad = case
    x, w, b = inputs.random_layer(sum(case[:5]) + 1, n, c, k, h, w_, 3, 3, keep)
    oc, a = oracle.conv2d_sparse_filter(x, oracle.filter_compress(w), w.shape, (1, 1), pad, b, True, want_abs=True)
    o = oracle.maxpool2x2(oc)
    amax = oracle.maxpool2x2(a.astype(np.float32)).astype(np.float64) * (1 + 1e-6)   # bound of the window's worst element
    f = F.filter_compress(dev(w))
    xs = {F.NCHW: dev(x), F.N4: dev(to_n4(x))}
    tested = 0
    for v in [0] + tiled_variants(F):
        for xl in (F.NCHW, F.N4):
            for yl in (F.NCHW, F.N4):
                try:
                    y = F.conv2d_sparse_filter(f, xs[xl], (1, 1), pad, dev(b), True, variant=v, x_layout=xl,
                                               y_layout=yl, n=n, pool=True)
                except F.FscnnError as e:
                    assert e.status == 4 and v != 0
                    continue
                torch.cuda.synchronize()
                g = host(y) if yl == F.NCHW else from_n4(host(y), n)
                assert_parity(g, o, amax, row_nmax(w), "pool case %r variant %d layouts %d->%d" % (case, v, xl, yl))
                tested += 1
    assert tested >= 4
    # integer data: bit-exact against conv-then-pool
    xi, wi, bi = inputs.random_layer(7, n, c, k, h, w_, 3, 3, keep, integer=True)
    want = oracle.maxpool2x2(oracle.conv2d_dense(xi, wi, (1, 1), pad, bi, True))
    fi = F.filter_compress(dev(wi))
    exact = 0
    for v in [0] + tiled_variants(F):
        try:
            got = host(F.conv2d_sparse_filter(fi, dev(xi), (1, 1), pad, dev(bi), True, variant=v, pool=True))
        except F.FscnnError as e:
            assert e.status == 4 and v != 0
            continue
        assert np.array_equal(got, want), "integer pool case %r variant %d" % (case, v)
        exact += 1
    assert exact >= 2


# ------------------------------------------------------------------ direct kernel (any stride / extent)
@pytest.mark.parametrize("r,s,stride,pad", [(1, 1, (2, 2), (0, 0)), (3, 3, (3, 3), (1, 1)), (5, 5, (1, 1), (2, 2)),
                                            (7, 7, (2, 2), (3, 3)), (2, 4, (1, 3), (0, 2)), (3, 3, (1, 2), (1, 0))])
def test_direct_kernel_matches_oracle(F, r, s, stride, pad):
    x, w, b = inputs.random_layer(50 + r * s, 2, 10, 13, 21, 75, r, s, keep=0.3)
    o, a = oracle.conv2d_sparse_filter(x, oracle.filter_compress(w), w.shape, stride, pad, b, True, want_abs=True)
    f = F.filter_compress(dev(w))
    p = F.filter_plan_export(f, 2, 21, 75, stride, pad)
    assert p["direct"]
    assert_parity(gpu_conv(F, x, w, stride, pad, b, True, filt=f), o, a, row_nmax(w), "direct")


@pytest.mark.parametrize("case", [(2, 24, 17, 9, 70, 0.4, (0, 0)), (5, 130, 70, 28, 28, 0.05, (0, 0)),
                                  (1, 300, 33, 14, 14, 0.2, (1, 1)), (4, 64, 256, 56, 56, 0.05, (0, 0)),
                                  (3, 7, 5, 1, 1, 1.0, (0, 0))])
def test_one_by_one_tiled_matches_oracle_all_variants(F, case):
    """1x1 filters go through the tiled kernel (stride 1): every 1x1 configuration, every layout."""
    n, c, k, h, w_, keep, pad = case
    x, w, b = inputs.random_layer(sum(case[:5]) + 3, n, c, k, h, w_, 1, 1, keep)
    o, a = oracle.conv2d_sparse_filter(x, oracle.filter_compress(w), w.shape, (1, 1), pad, b, True, want_abs=True)
    f = F.filter_compress(dev(w))
    assert not F.filter_plan_export(f, n, h, w_, (1, 1), pad)["direct"]
    xs = {F.NCHW: dev(x), F.N4: dev(to_n4(x))}
    for v in [0] + tiled_variants(F, extent="1x1"):
        for xl in (F.NCHW, F.N4):
            for yl in (F.NCHW, F.N4):
                y = F.conv2d_sparse_filter(f, xs[xl], (1, 1), pad, dev(b), True, variant=v, x_layout=xl, y_layout=yl, n=n)
                g = host(y) if yl == F.NCHW else from_n4(host(y), n)
                assert_parity(g, o, a, row_nmax(w), "1x1 case %r variant %d layouts %d->%d" % (case, v, xl, yl))
    with pytest.raises(F.FscnnError) as e:            # a 3x3 configuration cannot serve a 1x1 filter
        F.conv2d_sparse_filter(f, dev(x), (1, 1), pad, dev(b), True, variant=tiled_variants(F)[0])
    assert e.value.status == 4
    xi, wi, bi = inputs.random_layer(8, n, c, k, h, w_, 1, 1, keep, integer=True)
    want = oracle.conv2d_dense(xi, wi, (1, 1), pad, bi, True)
    fi = F.filter_compress(dev(wi))
    for v in tiled_variants(F, extent="1x1"):
        assert np.array_equal(host(F.conv2d_sparse_filter(fi, dev(xi), (1, 1), pad, dev(bi), True, variant=v)), want)


@pytest.mark.parametrize("case", [(2, 19, 37, 23, 71, 0.30, (1, 1)), (5, 40, 70, 28, 28, 0.10, (1, 1)),
                                  (1, 16, 9, 14, 15, 0.5, (0, 0)), (4, 64, 128, 56, 56, 0.05, (1, 1)),
                                  (1, 3, 5, 2, 2, 1.0, (1, 1)), (3, 8, 8, 9, 9, 0.5, (2, 2)), (1, 6, 4, 1, 1, 1.0, (1, 1))])
def test_stride_two_tiled_matches_oracle_all_variants(F, case):
    """3x3 filters at stride 2 go through the tiled kernel (four input planes per channel)."""
    n, c, k, h, w_, keep, pad = case
    x, w, b = inputs.random_layer(sum(case[:5]) + 5, n, c, k, h, w_, 3, 3, keep)
    o, a = oracle.conv2d_sparse_filter(x, oracle.filter_compress(w), w.shape, (2, 2), pad, b, True, want_abs=True)
    f = F.filter_compress(dev(w))
    assert not F.filter_plan_export(f, n, h, w_, (2, 2), pad)["direct"]
    xs = {F.NCHW: dev(x), F.N4: dev(to_n4(x))}
    for v in [0] + tiled_variants(F, extent="3x3s2"):
        for xl in (F.NCHW, F.N4):
            for yl in (F.NCHW, F.N4):
                y = F.conv2d_sparse_filter(f, xs[xl], (2, 2), pad, dev(b), True, variant=v, x_layout=xl, y_layout=yl, n=n)
                g = host(y) if yl == F.NCHW else from_n4(host(y), n)
                assert_parity(g, o, a, row_nmax(w), "stride-2 case %r variant %d layouts %d->%d" % (case, v, xl, yl))
    with pytest.raises(F.FscnnError) as e:            # a stride-1 configuration cannot serve stride 2
        F.conv2d_sparse_filter(f, dev(x), (2, 2), pad, dev(b), True, variant=tiled_variants(F)[0])
    assert e.value.status == 4
    xi, wi, bi = inputs.random_layer(8, n, c, k, h, w_, 3, 3, keep, integer=True)
    want = oracle.conv2d_dense(xi, wi, (2, 2), pad, bi, True)
    fi = F.filter_compress(dev(wi))
    for v in tiled_variants(F, extent="3x3s2"):
        assert np.array_equal(host(F.conv2d_sparse_filter(fi, dev(xi), (2, 2), pad, dev(bi), True, variant=v)), want)


@pytest.mark.parametrize("case", [(2, 19, 37, 23, 71, 3, (1, 1), (1, 1), 0.1), (4, 64, 40, 28, 28, 3, (2, 2), (1, 1), 0.1),
                                  (5, 130, 70, 14, 14, 1, (1, 1), (0, 0), 0.25), (1, 200, 40, 14, 14, 3, (1, 1), (1, 1), 0.1),
                                  (2, 10, 13, 21, 30, 5, (1, 1), (2, 2), 0.01), (1, 8, 8, 9, 9, 3, (1, 1), (1, 1), 1.0)])
def test_leaky_relu_epilogue(F, case):
    """LeakyReLU on every kernel family: tiled 3x3, stride 2, 1x1, channel-split, direct."""
    n, c, k, h, w_, r, stride, pad, slope = case
    x, w, b = inputs.random_layer(sum(case[:5]) + 11, n, c, k, h, w_, r, r, 0.3)
    o = oracle.conv2d_sparse_filter(x, oracle.filter_compress(w), w.shape, stride, pad, b, False)
    want, a = oracle.conv2d_sparse_filter(x, oracle.filter_compress(w), w.shape, stride, pad, b, False, want_abs=True,
                                          leaky=slope)
    f = F.filter_compress(dev(w))
    g = host(F.conv2d_sparse_filter(f, dev(x), stride, pad, dev(b), leaky=slope))
    assert_parity(g, want, a, row_nmax(w), "leaky %r" % (case,))
    assert (g < 0).any() or slope == 1.0 or not (o < 0).any()
    if stride in ((1, 1), (2, 2)) and r in (1, 3):
        g4 = F.conv2d_sparse_filter(f, dev(to_n4(x)), stride, pad, dev(b), leaky=slope, x_layout=F.N4, y_layout=F.N4, n=n)
        assert_parity(from_n4(host(g4), n), want, a, row_nmax(w), "leaky N4 %r" % (case,))
    with pytest.raises(F.FscnnError) as e:
        F.conv2d_sparse_filter(f, dev(x), stride, pad, dev(b), leaky=-0.5)
    assert e.value.status == 2
    # slope 0 is ReLU
    gr = host(F.conv2d_sparse_filter(f, dev(x), stride, pad, dev(b), leaky=0.0))
    assert_parity(gr, np.maximum(o, 0), a, row_nmax(w), "leaky slope 0 %r" % (case,))


def test_one_by_one_is_matrix_product_on_the_gpu(F):
    x, w, _ = inputs.random_layer(61, 2, 24, 17, 9, 70, 1, 1, keep=0.4, integer=True, bias=False)
    g = gpu_conv(F, x, w, (1, 1), (0, 0), None, False)
    want = np.einsum("kc,ncp->nkp", w[:, :, 0, 0].astype(np.float64),
                     x.reshape(2, 24, -1).astype(np.float64)).reshape(2, 17, 9, 70)
    assert np.array_equal(g, want.astype(np.float32))


# ------------------------------------------------------------------ error paths with a device present
def test_error_statuses_on_the_gpu(F):
    _, w, _ = inputs.random_layer(70, 1, 4, 4, 4, 4, 3, 3, keep=0.5)
    f = F.filter_compress(dev(w))
    x = torch.zeros(1, 5, 8, 8, device="cuda")
    with pytest.raises(F.FscnnError) as e:
        F.conv2d_sparse_filter(f, x, (1, 1), (1, 1))
    assert e.value.status == 3                                     # C mismatch
    x4 = torch.zeros(1, 4, 8, 8, device="cuda")
    with pytest.raises(F.FscnnError) as e:
        F.conv2d_sparse_filter(f, x4, (2, 2), (1, 1), variant=1)   # tiled variant cannot stride
    assert e.value.status == 4
    with pytest.raises(F.FscnnError) as e:
        F.conv2d_sparse_filter(f, x4, (1, 1), (1, 1), variant=999)
    assert e.value.status == 4
    with pytest.raises(F.FscnnError) as e:
        F.conv2d_out_shape(2, 2, 3, 3)
    assert e.value.status == 2
    L = F.lib()
    h = f.handle
    f._h = None
    assert L.fscnn_filter_destroy(h) == 0
    # (a destroyed handle must not be touched again: its memory is gone)


# ------------------------------------------------------------------ workload configs
def test_config1_whole_layer(F):
    c = inputs.config1()
    o, a = oracle.conv2d_sparse_filter(c["x"], oracle.filter_compress(c["w"]), c["w"].shape, c["stride"],
                                       c["pad"], c["bias"], c["relu"], want_abs=True)
    for v in [0] + tiled_variants(F):
        g = gpu_conv(F, c["x"], c["w"], c["stride"], c["pad"], c["bias"], c["relu"], variant=v)
        assert_parity(g, o, a, row_nmax(c["w"]), "config1 v%d" % v)


def test_config2_whole_layer(F):
    c = inputs.config2()
    csr = oracle.filter_compress(c["w"])
    f = F.filter_compress(dev(c["w"]))
    rp, ix, vl = F.filter_export(f)
    assert np.array_equal(rp, csr[0]) and np.array_equal(ix, csr[1]) and np.array_equal(bits(vl), bits(csr[2]))
    o, a = oracle.conv2d_sparse_filter(c["x"], csr, c["w"].shape, c["stride"], c["pad"], c["bias"], c["relu"],
                                       want_abs=True)
    for v in [0] + tiled_variants(F):
        g = gpu_conv(F, c["x"], c["w"], c["stride"], c["pad"], c["bias"], c["relu"], variant=v, filt=f)
        assert_parity(g, o, a, row_nmax(c["w"]), "config2 v%d" % v)


def _run_stack(F, x, layers, check):
    """Runs the conv (+pool) chain on the GPU, calling check(li, x_in_host, layer, y_host)."""
    cur = dev(x)
    for li, L in enumerate(layers):
        f = F.filter_compress(dev(L["w"]))
        y = F.conv2d_sparse_filter(f, cur, L["stride"], L["pad"], dev(L["bias"]), L["relu"])
        torch.cuda.synchronize()
        check(li, host(cur), L, host(y), f)
        cur = F.maxpool2x2(y) if L["pool_after"] else y
        del f
    return cur


def test_config3_reduced_size_chain_whole_tensors(F):
    # the 13-layer VGG16-shaped stack at 56x56 input (224/4) so that the oracle runs every layer
    # in full; each layer is compared against the oracle fed the GPU's previous output, and the
    # final tensor against the oracle's own chain
    x, layers = inputs.config3(size_div=4)
    state = {"o": x}

    def check(li, xin, L, y, f):
        csr = oracle.filter_compress(L["w"])
        rp, ix, vl = F.filter_export(f)
        assert np.array_equal(rp, csr[0]) and np.array_equal(ix, csr[1]) and np.array_equal(bits(vl), bits(csr[2]))
        o, a = oracle.conv2d_sparse_filter(xin, csr, L["w"].shape, L["stride"], L["pad"], L["bias"], L["relu"],
                                           want_abs=True)
        assert_parity(y, o, a, row_nmax(L["w"]), "config3/4 layer %d (GPU-fed)" % li)
        oo = oracle.conv2d_sparse_filter(state["o"], csr, L["w"].shape, L["stride"], L["pad"], L["bias"], L["relu"])
        state["o"] = oracle.maxpool2x2(oo) if L["pool_after"] else oo
        state["last"] = oo
        state["last_gpu"] = y

    _run_stack(F, x, layers, check)
    # the whole chain against the oracle's own chain: rounding differences compound over the 13
    # layers (and can flip a ReLU), so this end-to-end figure is held to 1e-3 instead of 1e-4
    from parity import rel_err
    assert state["last"].shape == (1, 512, 3, 3)
    assert rel_err(state["last_gpu"], state["last"]) <= 1e-3


def _sampled_layer_check(F, rng, npts):
    def check(li, xin, L, y, f):
        flat = rng.choice(y.size, size=min(npts, y.size), replace=False)
        # always include the corners and the last element (tile and image borders)
        flat = np.unique(np.concatenate([flat, [0, y.shape[3] - 1, y.size - 1, y.size - y.shape[3]]]))
        o, a = oracle.conv2d_points(xin, L["w"], flat, L["stride"], L["pad"], L["bias"], L["relu"], want_abs=True)
        assert_parity(y.ravel()[flat], o, a, row_nmax(L["w"]), "layer %d sampled" % li)
        # properties that hold at any size: ReLU output is non-negative and finite everywhere
        assert np.all(np.isfinite(y)) and y.min() >= 0.0
    return check


def test_config3_full_size_sampled(F):
    x, layers = inputs.config3()
    out = _run_stack(F, x, layers, _sampled_layer_check(F, np.random.default_rng(3), 4000))
    assert tuple(out.shape) == (1, 512, 14, 14)


def test_config4_full_size_sampled(F):
    x, layers = inputs.config4(n=32)
    out = _run_stack(F, x, layers, _sampled_layer_check(F, np.random.default_rng(4), 4000))
    assert tuple(out.shape) == (32, 512, 14, 14)


@pytest.mark.parametrize("keep", inputs.CONFIG5_KEEP)
def test_config5_sparsity_sweep_sampled(F, keep):
    c = inputs.config5(keep)
    f = F.filter_compress(dev(c["w"]))
    y = host(F.conv2d_sparse_filter(f, dev(c["x"]), c["stride"], c["pad"], dev(c["bias"]), c["relu"]))
    flat = np.random.default_rng(5).choice(y.size, 3000, replace=False)
    o, a = oracle.conv2d_points(c["x"], c["w"], flat, c["stride"], c["pad"], c["bias"], c["relu"], want_abs=True)
    assert_parity(y.ravel()[flat], o, a, row_nmax(c["w"]), "config5 keep %g" % keep)


# ------------------------------------------------------------------ largest sizes
@pytest.mark.parametrize("wd,tiled", [(4095, True), (4096, False)])
def test_largest_image_the_tiled_kernel_addresses(F, wd, tiled):
    """The tiled kernel addresses the channels of four images with 32-bit byte offsets, i.e.
    C*H*W*16 below 2^31: an 8-channel 4096 x 4095 image is the last one it takes (2.1 GB per
    tensor at N=4), 4096 x 4096 goes to the direct kernel.  Sampled outputs, with the highest
    addresses of every image among them."""
    n, c, k, h = 4, 8, 8, 4096
    rng = np.random.default_rng([77, wd])
    x = rng.standard_normal((n, c, h, wd), dtype=np.float32)
    w = np.where(rng.random((k, c, 3, 3)) < 0.5, rng.standard_normal((k, c, 3, 3)), 0).astype(np.float32)
    b = rng.standard_normal(k, dtype=np.float32)
    f = F.filter_compress(dev(w))
    p = F.filter_plan_export(f, n, h, wd, (1, 1), (1, 1))
    assert p["direct"] == (not tiled)
    y = F.conv2d_sparse_filter(f, dev(x), (1, 1), (1, 1), dev(b), True)
    per = k * h * wd
    tail = np.concatenate([np.arange(per - 600, per) + i * per for i in range(n)])
    head = np.concatenate([np.arange(600) + i * per for i in range(n)])
    flat = np.unique(np.concatenate([tail, head, rng.choice(n * per, 4000, replace=False)]))
    g = host(y.view(-1)[torch.from_numpy(flat).cuda()])
    o, a = oracle.conv2d_points(x, w, flat, (1, 1), (1, 1), b, True, want_abs=True)
    assert_parity(g, o, a, row_nmax(w), "largest image, W=%d" % wd)


# ------------------------------------------------------------------ YOLO-shaped stack (second workload)
def test_batch_of_more_than_2_31_elements(F):
    # 2100 images of 16 x 256 x 256: image 2048 starts exactly 2^31 floats into x and y.  Images
    # are addressed with 64-bit offsets; the ones around the 32-bit boundaries and the last one are
    # compared whole with the oracle, for NCHW and N4 tensors, plain and with the merged pool.
    n, c, k, h = 2100, 16, 16, 256
    assert n * c * h * h > 2 ** 31
    _, w, b = inputs.random_layer(77, 1, c, k, 3, 3, 3, 3, 0.3)
    g = torch.Generator(device="cuda")
    g.manual_seed(1234)
    x = torch.empty((n, c, h, h), device="cuda").uniform_(-1.0, 1.0, generator=g)
    picks = [0, 1023, 1024, 2047, 2048, 2099]
    xs = np.stack([host(x[i]) for i in picks])
    csr = oracle.filter_compress(w)
    o, a = oracle.conv2d_sparse_filter(xs, csr, w.shape, (1, 1), (1, 1), b, True, want_abs=True)
    op = oracle.maxpool2x2(o)
    ap = oracle.maxpool2x2(a.astype(np.float32)).astype(np.float64) * (1 + 1e-6)
    f = F.filter_compress(dev(w))
    x4 = x.view(n // 4, 4, c, h, h).permute(0, 2, 3, 4, 1).contiguous()
    for xl, xin in ((F.NCHW, x), (F.N4, x4)):
        for yl in (F.NCHW, F.N4):
            for pool in (False, True):
                y = F.conv2d_sparse_filter(f, xin, (1, 1), (1, 1), dev(b), True, x_layout=xl, y_layout=yl, n=n, pool=pool)
                torch.cuda.synchronize()
                if yl == F.NCHW:
                    got = np.stack([host(y[i]) for i in picks])
                else:
                    got = np.stack([host(y[i // 4, ..., i % 4]) for i in picks])
                assert_parity(got, op if pool else o, ap if pool else a, row_nmax(w),
                              "large batch layouts %d->%d pool %d" % (xl, yl, pool))
                del y
    # the direct kernel (5x5 filters) as well
    _, w5, b5 = inputs.random_layer(78, 1, c, 4, 5, 5, 5, 5, 0.2)
    o5, a5 = oracle.conv2d_sparse_filter(xs, oracle.filter_compress(w5), w5.shape, (1, 1), (2, 2), b5, True, want_abs=True)
    y = F.conv2d_sparse_filter(F.filter_compress(dev(w5)), x, (1, 1), (2, 2), dev(b5), True)
    torch.cuda.synchronize()
    assert_parity(np.stack([host(y[i]) for i in picks]), o5, a5, row_nmax(w5), "large batch, direct kernel")


def test_yolo_shaped_stack_chain(F):
    """Darknet-53's 52 convolutions as a chain (3x3 stride 1 and 2, 1x1, LeakyReLU 0.1), reduced
    width and image size: every layer against the oracle on the GPU's own previous output, N4
    tensors handed from layer to layer, and the whole chain against the oracle's own chain."""
    n = 4
    x, layers = inputs.yolo_stack(n, 0.3, hw0=64, width_div=8)
    assert len(layers) == 52 and layers[-1]["hw"] == 2
    cur = dev(to_n4(x))
    cur_host = x
    oc = x                                        # the oracle's own chain
    kinds = set()
    for li, L in enumerate(layers):
        w, b, st, pad = L["w"], L["bias"], L["stride"], L["pad"]
        f = F.filter_compress(dev(w))
        p = F.filter_plan_export(f, n, L["hw"], L["hw"], st, pad)
        assert not p["direct"]
        kinds.add(F.sf_variant_name(p["variant"]).split("_")[-1] if "_" in F.sf_variant_name(p["variant"]) else "")
        y = F.conv2d_sparse_filter(f, cur, st, pad, dev(b), leaky=L["leaky"], x_layout=F.N4, y_layout=F.N4, n=n)
        g = from_n4(host(y), n)
        csr = oracle.filter_compress(w)
        want, a = oracle.conv2d_sparse_filter(cur_host, csr, w.shape, st, pad, b, False, want_abs=True,
                                              leaky=L["leaky"])
        assert_parity(g, want, a, row_nmax(w), "yolo layer %d" % li)
        oc = oracle.conv2d_sparse_filter(oc, csr, w.shape, st, pad, b, False, leaky=L["leaky"])
        cur, cur_host = y, g
    assert {"st2", "r1s1"} <= kinds               # stride-2 and 1x1 configurations were exercised
    # 52 layers of fp32 rounding against the double-accumulating oracle chain
    scale = float(np.sqrt(np.mean(oc.astype(np.float64) ** 2)))
    assert np.max(np.abs(cur_host - oc)) <= 2e-4 * max(scale, 1e-30)


# ------------------------------------------------------------------ A7/A8: sparse-input path
@pytest.mark.parametrize("shape,zf", [((2, 7, 5, 6), 0.7), ((1, 40, 9, 70), 0.5), ((3, 16, 1, 1), 0.0),
                                      ((1, 33, 4, 4), 1.0),
                                      ((2, 24, 120, 90), 0.6),      # 64 800 (pixel, step) pairs: tiled scan
                                      ((3, 130, 57, 61), 0.9)])     # 177 327 pairs, ragged last step
def test_input_compress_bit_exact(F, shape, zf):
    n, c, h, w_ = shape
    x, _, _ = inputs.random_layer(80 + c, n, c, 1, h, w_, 1, 1, 1.0, x_zero_frac=zf)
    if zf == 0.7:
        x[0, 0, 0, 0] = -0.0
        x[0, 1, 0, 0] = np.nan
    s = F.input_compress(dev(x))
    prow, cidx, val = F.input_export(s)
    op, oc, ov = oracle.input_compress(x)
    assert s.nnz == op[-1]
    assert np.array_equal(prow, op) and np.array_equal(cidx, oc) and np.array_equal(bits(val), bits(ov))


@pytest.mark.parametrize("case", [
    (2, 19, 37, 11, 23, 3, 3, (1, 1), (1, 1)),
    (1, 40, 70, 14, 14, 3, 3, (1, 1), (1, 1)),
    (1, 16, 64, 9, 9, 3, 3, (1, 1), (0, 0)),
    (2, 10, 13, 12, 15, 3, 3, (2, 2), (1, 1)),       # direct kernel
    (1, 6, 5, 8, 8, 1, 1, (1, 1), (0, 0)),           # direct kernel
    (1, 7, 66, 10, 9, 5, 2, (1, 2), (2, 0)),         # direct kernel
])
def test_conv_sparse_input_matches_oracle(F, case):
    n, c, k, h, w_, r, s_, stride, pad = case
    x, w, b = inputs.random_layer(90 + c + k, n, c, k, h, w_, r, s_, keep=0.5, x_zero_frac=0.7)
    csx = oracle.input_compress(x)
    o, a = oracle.conv2d_sparse_input(csx, x.shape, w, stride, pad, b, True, want_abs=True)
    s = F.input_compress(dev(x))
    g = host(F.conv2d_sparse_input(s, dev(w), stride, pad, dev(b), True))
    assert_parity(g, o, a, c * r * s_, "sparse input %r" % (case,))
    # three-way agreement: the sparse-filter path on the same data
    g2 = gpu_conv(F, x, w, stride, pad, b, True)
    assert_parity(g2, o, a, c * r * s_, "sparse filter on the same data")


def test_sparse_input_integer_bit_exact(F):
    x, w, b = inputs.random_layer(95, 2, 21, 70, 13, 18, 3, 3, keep=0.6, x_zero_frac=0.6, integer=True)
    o = oracle.conv2d_dense(x, w, (1, 1), (1, 1), b, True)
    g = host(F.conv2d_sparse_input(F.input_compress(dev(x)), dev(w), (1, 1), (1, 1), dev(b), True))
    assert np.array_equal(g, o)


@pytest.mark.parametrize("case", [
    (2, 19, 37, 11, 23, (1, 1)),        # ragged everything: K < 128, C not a multiple of 8, odd Wo
    (1, 40, 300, 14, 16, (1, 1)),       # three channel groups of 128, Wo a multiple of 4 (vector stores)
    (1, 16, 64, 9, 9, (0, 0)),          # no padding
    (3, 70, 130, 28, 28, (1, 1)),       # several tiles, several chunks
    (1, 8, 8, 5, 5, (2, 2)),            # pad wider than the halo
    (1, 3, 5, 1, 1, (1, 1)),            # 1x1 image
])
def test_conv_sparse_input_prepared_matches_oracle_all_variants(F, case):
    n, c, k, h, w_, pad = case
    x, w, b = inputs.random_layer(190 + c + k, n, c, k, h, w_, 3, 3, keep=0.5, x_zero_frac=0.7)
    csx = oracle.input_compress(x)
    o, a = oracle.conv2d_sparse_input(csx, x.shape, w, (1, 1), pad, b, True, want_abs=True)
    s = F.input_compress(dev(x))
    d = F.dense_filter_prepare(dev(w))
    for v in range(0, F.si_variant_count() + 1):
        g = host(F.conv2d_sparse_input_prepared(s, d, (1, 1), pad, dev(b), True, variant=v))
        assert_parity(g, o, a, c * 9, "prepared sparse input %r variant %d" % (case, v))
    g = host(F.conv2d_sparse_input_prepared(s, d, (1, 1), pad, None, False))     # no bias, no ReLU
    o2, a2 = oracle.conv2d_sparse_input(csx, x.shape, w, (1, 1), pad, None, False, want_abs=True)
    assert_parity(g, o2, a2, c * 9, "prepared sparse input %r plain" % (case,))
    # integer data: bit-exact in every configuration
    xi, wi, bi = inputs.random_layer(7, n, c, k, h, w_, 3, 3, keep=0.6, x_zero_frac=0.6, integer=True)
    want = oracle.conv2d_dense(xi, wi, (1, 1), pad, bi, True)
    si, di = F.input_compress(dev(xi)), F.dense_filter_prepare(dev(wi))
    for v in range(1, F.si_variant_count() + 1):
        assert np.array_equal(host(F.conv2d_sparse_input_prepared(si, di, (1, 1), pad, dev(bi), True, variant=v)), want)


def test_conv_sparse_input_prepared_rejects_what_it_cannot_serve(F):
    x, w, b = inputs.random_layer(1, 1, 6, 5, 8, 8, 3, 3, keep=0.5, x_zero_frac=0.5)
    s = F.input_compress(dev(x))
    d = F.dense_filter_prepare(dev(w))
    with pytest.raises(F.FscnnError) as e:
        F.conv2d_sparse_input_prepared(s, d, (2, 2), (1, 1))                       # stride 2
    assert e.value.status == 4
    with pytest.raises(F.FscnnError) as e:
        F.conv2d_sparse_input_prepared(s, d, (1, 1), (1, 1), variant=99)
    assert e.value.status == 4
    _, w5, _ = inputs.random_layer(2, 1, 6, 5, 8, 8, 5, 5, keep=0.5)
    with pytest.raises(F.FscnnError) as e:
        F.conv2d_sparse_input_prepared(s, F.dense_filter_prepare(dev(w5)), (1, 1), (2, 2))   # 5x5 filter
    assert e.value.status == 4
    _, w7, _ = inputs.random_layer(3, 1, 7, 5, 8, 8, 3, 3, keep=0.5)
    with pytest.raises(F.FscnnError) as e:
        F.conv2d_sparse_input_prepared(s, F.dense_filter_prepare(dev(w7)), (1, 1), (1, 1))   # C differs
    assert e.value.status == 3


def test_config5_sparse_input_point(F):
    c = inputs.config5(0.05)
    xs = F.input_compress(dev(c["x"]))
    op, oc, ov = oracle.input_compress(c["x"])
    prow, cidx, val = F.input_export(xs)
    assert np.array_equal(prow, op) and np.array_equal(cidx, oc) and np.array_equal(bits(val), bits(ov))
    assert 0.29 < xs.nnz / c["x"].size < 0.33          # ReLU(N(-0.5,1)) keeps ~30.85 %
    y = host(F.conv2d_sparse_input(xs, dev(c["w"]), c["stride"], c["pad"], dev(c["bias"]), c["relu"]))
    flat = np.random.default_rng(6).choice(y.size, 3000, replace=False)
    o, a = oracle.conv2d_points(c["x"], c["w"], flat, c["stride"], c["pad"], c["bias"], c["relu"], want_abs=True)
    assert_parity(y.ravel()[flat], o, a, 512 * 9, "config5 sparse input")
    d = F.dense_filter_prepare(dev(c["w"]))
    for v in range(0, F.si_variant_count() + 1):
        yp = host(F.conv2d_sparse_input_prepared(xs, d, c["stride"], c["pad"], dev(c["bias"]), c["relu"], variant=v))
        assert_parity(yp.ravel()[flat], o, a, 512 * 9, "config5 prepared sparse input variant %d" % v)


def test_first_layer_form_for_banks_without_zeros(F):
    """A bank without zeros over three input channels (an RGB first layer) is served, where the launch
    fills the chip, by the form that walks taps in the outer loop and feeds every tap it reads to all
    channels of the wave.  Same sums in the same order as the record-stream forms: bit-equal to them,
    and within the rule against the oracle; layouts, merged pool, ragged sizes."""
    n, c, k, h, w_ = 16, 3, 64, 118, 130
    x, w, b = inputs.random_layer(901, n, c, k, h, w_, 3, 3, keep=1.0)
    assert np.count_nonzero(w) == w.size
    f = F.filter_compress(dev(w))
    names = {v: F.sf_variant_name(v) for v in range(1, F.sf_variant_count() + 1)}
    for n4 in (False, True):
        for pool in (False, True):
            v = F.sf_variant_choice(f, n, h, w_, n4=n4, pool=pool)
            assert "_u5_" in names[v], (n4, pool, names[v])
    o, a = oracle.conv2d_dense(x, w, (1, 1), (1, 1), b, True, want_abs=True)
    xd, bd = dev(x), dev(b)
    y = host(F.conv2d_sparse_filter(f, xd, (1, 1), (1, 1), bd, True))
    assert_parity(y, o, a, c * 9, "first-layer form, NCHW")
    other = [v for v, nm in names.items() if "_u1_" in nm and "_cc3_" in nm and not nm.endswith(("_st2", "_r1s1"))][0]
    y1 = host(F.conv2d_sparse_filter(f, xd, (1, 1), (1, 1), bd, True, variant=other))
    assert np.array_equal(bits(y), bits(y1))
    y4 = F.conv2d_sparse_filter(f, xd, (1, 1), (1, 1), bd, True, x_layout=F.NCHW, y_layout=F.N4, n=n)
    assert np.array_equal(bits(from_n4(host(y4), n)), bits(y))
    yp = F.conv2d_sparse_filter(f, dev(to_n4(x)), (1, 1), (1, 1), bd, True, x_layout=F.N4, y_layout=F.N4, n=n, pool=True)
    assert np.array_equal(bits(from_n4(host(yp), n)), bits(oracle.maxpool2x2(y)))
    # a single zero in the bank: the automatic choice goes back to the record-stream forms
    w0 = w.copy()
    w0[5, 1, 2, 0] = 0.0
    f0 = F.filter_compress(dev(w0))
    assert "_u5_" not in names[F.sf_variant_choice(f0, n, h, w_)]
    # ... and so does a bank whose channel count leaves idle channels in a work-group
    f1 = F.filter_compress(dev(w[:40]))
    assert "_u5_" not in names[F.sf_variant_choice(f1, n, h, w_)]
    # 32 channels: the four-wave form of the same loop
    f2 = F.filter_compress(dev(w[:32]))
    v2 = F.sf_variant_choice(f2, 32, h, w_)
    assert "_u5_" in names[v2] and "_w4_" in names[v2]
    x2 = np.concatenate([x, x[::-1]], 0)
    y2 = host(F.conv2d_sparse_filter(f2, dev(x2), (1, 1), (1, 1), dev(b[:32]), True))
    assert np.array_equal(bits(y2[:n]), bits(y[:, :32])) and np.array_equal(bits(y2[n:]), bits(y[::-1, :32]))


def test_channel_split_mode_is_bit_reproducible_and_matches_the_oracle(F):
    """Small problems (few work-groups) divide the input channels over several work-groups; every
    part stores its partial sums into its own copy of the output and a finishing pass adds the
    copies in the order of the parts, so two runs give the same bits (one writer per element, no
    atomics).  Config 3's deep layers at N=1 take this mode."""
    for (n, c, k, hw, lay) in [(1, 512, 512, 14, "nchw"), (1, 256, 512, 28, "nchw"), (2, 300, 70, 14, "n4"),
                               (8, 512, 512, 14, "n4")]:
        x, w, b = inputs.random_layer(400 + c + hw, n, c, k, hw, hw, 3, 3, 0.1)
        f = F.filter_compress(dev(w))
        xl = F.N4 if lay == "n4" else F.NCHW
        xd = dev(to_n4(x)) if lay == "n4" else dev(x)
        F.filter_prepare(f, n, hw, hw, (1, 1), (1, 1), x_layout=xl, y_layout=xl)
        runs = [F.conv2d_sparse_filter(f, xd, (1, 1), (1, 1), dev(b), True, x_layout=xl, y_layout=xl, n=n)
                for _ in range(4)]
        torch.cuda.synchronize()
        got = [from_n4(host(y), n) if lay == "n4" else host(y) for y in runs]
        assert all(np.array_equal(bits(g), bits(got[0])) for g in got[1:])
        o, a = oracle.conv2d_sparse_filter(x, oracle.filter_compress(w), w.shape, (1, 1), (1, 1), b, True, want_abs=True)
        assert_parity(got[0], o, a, row_nmax(w), "channel split %r" % ((n, c, k, hw, lay),))


def test_channel_split_mode_with_the_merged_pool(F):
    """The same mode where the 2x2 max-pool is merged into the call: the parts hold full-size partial
    sums and the finishing pass pools.  Against the oracle's convolution followed by its plain
    max-pool (odd sizes: the last row and column drop out), twice for the same bits."""
    for (n, c, k, h, w_, lay) in [(1, 512, 512, 28, 28, "nchw"), (1, 256, 96, 15, 17, "nchw"), (3, 300, 70, 14, 14, "n4"),
                                  (8, 512, 512, 14, 14, "n4")]:
        x, w, b = inputs.random_layer(700 + c + h, n, c, k, h, w_, 3, 3, 0.1)
        f = F.filter_compress(dev(w))
        xl = F.N4 if lay == "n4" else F.NCHW
        xd = dev(to_n4(x)) if lay == "n4" else dev(x)
        F.filter_prepare(f, n, h, w_, (1, 1), (1, 1), x_layout=xl, y_layout=xl, pool=True)
        runs = [F.conv2d_sparse_filter(f, xd, (1, 1), (1, 1), dev(b), True, x_layout=xl, y_layout=xl, n=n, pool=True)
                for _ in range(3)]
        torch.cuda.synchronize()
        got = [from_n4(host(y), n) if lay == "n4" else host(y) for y in runs]
        assert got[0].shape == (n, k, h // 2, w_ // 2)
        assert all(np.array_equal(bits(g), bits(got[0])) for g in got[1:])
        o, a = oracle.conv2d_sparse_filter(x, oracle.filter_compress(w), w.shape, (1, 1), (1, 1), b, True, want_abs=True)
        assert_parity(got[0], oracle.maxpool2x2(o), oracle.maxpool2x2(a.astype(np.float32)).astype(np.float64) * (1 + 1e-6),
                      row_nmax(w), "channel split with pool %r" % ((n, c, k, h, w_, lay),))


def test_filter_handle_serves_two_streams_at_once(F):
    """One compressed filter, two streams launching convolutions on different inputs at the same
    time (the plan is built once, under the handle's lock): both results equal the ones computed
    one after the other."""
    xa, w, b = inputs.random_layer(97, 8, 64, 96, 56, 56, 3, 3, keep=0.1)
    xb = inputs.random_layer(98, 8, 64, 96, 56, 56, 3, 3, keep=0.1)[0]
    f = F.filter_compress(dev(w))
    xad, xbd, bd = dev(xa), dev(xb), dev(b)
    torch.cuda.synchronize()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    outs = []
    for _ in range(4):
        with torch.cuda.stream(s1):
            ya = F.conv2d_sparse_filter(f, xad, (1, 1), (1, 1), bd, True)
        with torch.cuda.stream(s2):
            yb = F.conv2d_sparse_filter(f, xbd, (1, 1), (1, 1), bd, True)
        outs.append((ya, yb))
    s1.synchronize(); s2.synchronize()
    wa = host(F.conv2d_sparse_filter(f, xad, (1, 1), (1, 1), bd, True))
    wb = host(F.conv2d_sparse_filter(f, xbd, (1, 1), (1, 1), bd, True))
    for ya, yb in outs:
        assert np.array_equal(host(ya), wa) and np.array_equal(host(yb), wb)
    o, a = oracle.conv2d_dense(xa, w, (1, 1), (1, 1), b, True, want_abs=True)
    assert_parity(wa, o, a, row_nmax(w), "two streams, first input")


def test_compressed_input_is_usable_from_another_stream(F):
    """The pass that fills a compressed handle is still queued when fscnn_input_compress returns;
    a convolution launched on a different stream must be ordered behind it by the library."""
    x, w, b = inputs.random_layer(96, 4, 64, 64, 56, 56, 3, 3, keep=1.0, x_zero_frac=0.6)
    xd, wd, bd = dev(x), dev(w), dev(b)
    d = F.dense_filter_prepare(wd)
    torch.cuda.synchronize()
    want = host(F.conv2d_sparse_input_prepared(F.input_compress(xd), d, (1, 1), (1, 1), bd, True))
    other = torch.cuda.Stream()
    for _ in range(5):
        s = F.input_compress(xd)                      # made on the current stream
        with torch.cuda.stream(other):
            y = F.conv2d_sparse_input_prepared(s, d, (1, 1), (1, 1), bd, True)
        other.synchronize()
        assert np.array_equal(host(y), want)
        prow, cidx, val = F.input_export(s)           # export waits for the fill as well
        assert prow[-1] == s.nnz == cidx.size
    torch.cuda.synchronize()


def test_sparse_input_path_on_a_large_image(F):
    """4.5 M pixel rows, about 20 M stored values: compression bit-exact, the convolution on
    sampled outputs (first and last rows of the images among them), every configuration."""
    n, c, k, h, wd = 2, 16, 32, 1500, 1501
    rng = np.random.default_rng(78)
    x = np.where(rng.random((n, c, h, wd)) < 0.7, 0, rng.standard_normal((n, c, h, wd))).astype(np.float32)
    w = rng.standard_normal((k, c, 3, 3), dtype=np.float32)
    b = rng.standard_normal(k, dtype=np.float32)
    s = F.input_compress(dev(x))
    op, oc, ov = oracle.input_compress(x)
    prow, cidx, val = F.input_export(s)
    assert np.array_equal(prow, op) and np.array_equal(cidx, oc) and np.array_equal(bits(val), bits(ov))
    per = k * h * wd
    flat = np.unique(np.concatenate([np.arange(per - 500, per) + i * per for i in range(n)] +
                                    [np.arange(500) + i * per for i in range(n)] +
                                    [rng.choice(n * per, 3000, replace=False)]))
    o, a = oracle.conv2d_points(x, w, flat, (1, 1), (1, 1), b, True, want_abs=True)
    d = F.dense_filter_prepare(dev(w))
    fl = torch.from_numpy(flat).cuda()
    for v in range(0, F.si_variant_count() + 1):
        y = F.conv2d_sparse_input_prepared(s, d, (1, 1), (1, 1), dev(b), True, variant=v)
        assert_parity(host(y.view(-1)[fl]), o, a, c * 9, "large image, prepared sparse input, variant %d" % v)
    y = F.conv2d_sparse_input(s, dev(w), (1, 1), (1, 1), dev(b), True)
    assert_parity(host(y.view(-1)[fl]), o, a, c * 9, "large image, sparse input")


# ------------------------------------------------------------------ helper
def test_maxpool_helper(F):
    x = np.random.default_rng(1).standard_normal((2, 5, 13, 22)).astype(np.float32)
    assert np.array_equal(host(F.maxpool2x2(dev(x))), oracle.maxpool2x2(x))
