"""Writes tests/golden/config1_oracle.txt from the CPU oracle alone.

Run from the repository root:  python tests/golden/make_golden.py
The values are the oracle's own (config 1 of the workload list: N=1, C=16, K=32,
3x3, stride 1, pad 1, 32x32, 90 % zeros, seed 0); the paper prints no worked
numeric example (its figures are the only ones and carry no recoverable numbers),
so this fixture is a drift guard, not an external pin.  It imports nothing from
the HIP path.
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import oracle                                    # noqa: E402
from paper_2212_08815_amd import inputs          # noqa: E402  (seeded generator only)


def main():
    c = inputs.config1()
    rowptr, idx, val = oracle.filter_compress(c["w"])
    y = oracle.conv2d_sparse_filter(c["x"], (rowptr, idx, val), c["w"].shape, c["stride"], c["pad"])
    pos = np.random.default_rng(1).choice(y.size, 8, replace=False)
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "config1_oracle.txt")
    with open(out, "w") as f:
        f.write("# written by tests/golden/make_golden.py from oracle/ only (config 1, seed 0)\n")
        f.write("nnz = %d\n" % rowptr[-1])
        f.write("idx_sum = %d\n" % int(idx.astype(np.int64).sum()))
        f.write("rowptr_head = %s\n" % " ".join(str(v) for v in rowptr[:8]))
        f.write("y_probe_flat = %s\n" % " ".join(str(int(p)) for p in pos))
        f.write("y_probe = %s\n" % " ".join(repr(float(v)) for v in y.ravel()[pos]))


if __name__ == "__main__":
    main()
