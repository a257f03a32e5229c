#!/usr/bin/env python3
"""Row -> scheme assignment by weight variance (Alg. 1, else-branch; Section 3.1) on the ResNet-18
shaped layers of configs[3], against the seeded random assignment the benchmarks use.

    python -m paper_2111_00153_amd.assign_report

For every mixed layer the Fixed-8 rows are the same seeded 5 % in both cases (the paper picks them by
Hessian eigenvalue, which needs a trained model); the remaining rows are split PoT-4 : Fixed-4 = 35 : 60
either at random or by rmsmp_assign_by_variance (lowest variance -> PoT-4).  The weights are then
quantized by the library's own packer (rmsmp_pack_roundtrip_host; no GPU needed) and the squared error
of every row is taken against the fp32 weights.  Printed per scheme: mean squared error, and the same
divided by the row's variance (the error relative to the signal).
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import paper_2111_00153_amd as rm  # noqa: E402
import synth_inputs as si  # noqa: E402

NAMES = ("Fixed-4", "PoT-4", "Fixed-8")


def row_errors(W, scheme):
    rt = rm.rmsmp_pack_roundtrip_host(W, scheme)
    what = rt["wint"].astype(np.float64) * rt["rowscale"].astype(np.float64)[:, None]
    return ((W.astype(np.float64) - what) ** 2).mean(axis=1)


def main():
    tot = {k: {s: [0.0, 0.0, 0] for s in range(3)} for k in ("seeded", "variance")}
    layer_mse = {"seeded": 0.0, "variance": 0.0}
    n_weights = 0
    print("layer                  rows   | seeded: MSE F4 / P4 / F8 (x1e-6)      | by variance: MSE F4 / P4 / F8 (x1e-6)   | layer MSE ratio variance/seeded")
    for idx, (name, C, M, k, s, pad, H) in enumerate(si.RESNET18_CONVS):
        if idx == 0:
            continue  # first layer: all rows Fixed-8
        rng = si.rng_for(3, idx)
        K = C * k * k
        W = si.weights_rowscaled(rng, M, K)
        counts = rm.rmsmp_ratio_counts(M, 35, 60, 5)
        seeded = si.scheme_permutation(rng, counts)
        by_var = rm.rmsmp_assign_by_variance(W, np.where(seeded == si.FIXED8, si.FIXED8, si.FIXED4).astype(np.uint8), counts[1])
        assert tuple(np.bincount(by_var, minlength=3)) == tuple(counts)
        var = W.astype(np.float64).var(axis=1)
        line = "%-22s %5d  |" % (name, M)
        means = {}
        for key, scheme in (("seeded", seeded), ("variance", by_var)):
            err = row_errors(W, scheme)
            means[key] = err.mean()
            layer_mse[key] += err.sum() * K
            for sc in range(3):
                sel = scheme == sc
                t = tot[key][sc]
                t[0] += err[sel].sum()
                t[1] += (err[sel] / var[sel]).sum()
                t[2] += int(sel.sum())
                line += " %9.3f" % (1e6 * err[sel].mean())
            line += "        |"
        n_weights += M * K
        print(line + "  %.3f" % (means["variance"] / means["seeded"]))
    print()
    print("all 19 mixed layers, rows weighted equally:")
    for key in ("seeded", "variance"):
        print("  %-9s" % key + "".join("  %s: MSE %.3e, MSE/row variance %.4f (%d rows)" % (NAMES[sc], tot[key][sc][0] / tot[key][sc][2],
                                                                                     tot[key][sc][1] / tot[key][sc][2], tot[key][sc][2])
                                       for sc in range(3)))
    print("  mean squared error over all %d weights: seeded %.4e, by variance %.4e (ratio %.3f)"
          % (n_weights, layer_mse["seeded"] / n_weights, layer_mse["variance"] / n_weights, layer_mse["variance"] / layer_mse["seeded"]))


if __name__ == "__main__":
    main()
