"""Comparison rule shared by the GPU parity tests.

fp32 criterion ("max relative error 1e-4"): with o the oracle tensor (fp64 sum rounded once
to fp32) and g the GPU tensor,

    max_i |g_i - o_i| / max(|o_i|, tau)  <=  1e-4,      tau = rms(o)

so every element at or above the tensor's RMS magnitude is within 1e-4 relative, and the
many elements that cancel to ~0 (zero-mean weights, ReLU) are held to 1e-4 of the tensor's
scale.  A floor much smaller than this is below the noise of fp32 accumulation itself:
summing n terms of magnitude m in fp32 leaves about 2.4e-8 * n * m of rounding error while
rms(o) ~ sqrt(n) * m, i.e. error/rms ~ 2.4e-8 * sqrt(n) (1.6e-6 at n = 4608, the largest
row here), so the criterion holds with more than a decade of margin for any summation
order and fails for any indexing or precision mistake.

Second, rigorous criterion where the oracle's sum_abs = sum |w||x| + |b| is available: the
standard forward bound of recursive fp32 summation with fused multiply-adds,
|g_i - o_i| <= (n + 2) * 2^-24 * sum_abs_i (+ half an ulp of o_i for the oracle's own final
rounding), n = number of stored weights of the row.
"""
import numpy as np

RTOL = 1e-4


def rel_err(g, o):
    g = np.asarray(g, np.float64)
    o = np.asarray(o, np.float64)
    tau = float(np.sqrt(np.mean(o * o)))
    if tau == 0.0:
        return float(np.max(np.abs(g - o))) if g.size else 0.0
    return float(np.max(np.abs(g - o) / np.maximum(np.abs(o), tau))) if g.size else 0.0


def assert_parity(g, o, abs_sum=None, nmax=None, what=""):
    g = np.asarray(g)
    o = np.asarray(o)
    assert g.shape == o.shape, (what, g.shape, o.shape)
    assert np.all(np.isfinite(g)), what + ": non-finite GPU output"
    e = rel_err(g, o)
    assert e <= RTOL, "%s: max relative error %.3e > %.1e" % (what, e, RTOL)
    if abs_sum is not None:
        u = 2.0 ** -24
        bound = (nmax + 2) * u * 1.01 * np.asarray(abs_sum, np.float64) + u * np.abs(o.astype(np.float64)) + 1e-45
        d = np.abs(g.astype(np.float64) - o.astype(np.float64))
        worst = float(np.max(d / bound)) if d.size else 0.0
        assert worst <= 1.0, "%s: exceeds the fp32 summation bound by %.3fx" % (what, worst)
    return e
