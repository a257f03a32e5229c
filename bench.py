#!/usr/bin/env python3
"""Benchmark of the RMSMP hot path on one MI355X.

One step = one pass of the whole hot path over one batch: a single rmsmp_conv2d call on the
ResNet-18-shaped 3x3 layer (batch 32, 256->256 channels, 14x14, stride 1, pad 1; GEMM
M=256, K=2304, N=6272) with weight rows Fixed4:PoT4:Fixed8 = 60:35:5, unsigned 4-bit
activations resident in HBM, fused ReLU + 4-bit requantization.  Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

INT8_MFMA_PEAK_TOPS = 5000.0  # MI355X dense int8, published
HBM_PEAK_GBS = 8000.0
# HBM-side bytes per launch of the timed kernel, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE scaled by a
# 256 MiB device copy (profiles/conv_wide_kernel_configs1.md); a counter reading cannot be taken from
# inside this script, so the last measured value is carried here.
MEASURED_TRAFFIC_BYTES = 4861294


def make_conv_workload(cfg_id=1):
    import paper_2111_00153_amd as rm
    import synth_inputs as si
    c = si.CONFIGS[cfg_id]
    rng = si.rng_for(cfg_id)
    M, C, KH, KW = c["M"], c["C"], c["KH"], c["KW"]
    K = C * KH * KW
    W = si.weights_rowscaled(rng, M, K)
    counts = rm.rmsmp_ratio_counts(M, *c["ratio"])
    scheme = si.scheme_permutation(rng, counts)
    x = si.act_codes_u4(rng, (c["B"], c["H"], c["W"], C))
    return dict(cfg=c, W=W, scheme=scheme, x=x, counts=counts, K=K)


def cpu_baseline(wl, repeats=3):
    """The oracle, as it stands, on the whole batch of the same workload, `repeats` times over
    (about 20 core-seconds on 16 host threads)."""
    import oracle
    c = wl["cfg"]
    ref = oracle.quantize_rows(wl["W"], wl["scheme"])
    d = oracle.conv_desc(c["B"], c["C"], c["H"], c["W"], c["KH"], c["KW"], c["stride"], c["pad"])
    x = wl["x"].astype(np.int32)
    wint = ref["wint"].reshape(c["M"], c["C"], c["KH"], c["KW"])
    rs = oracle.rowsum(ref["wint"])
    t0 = time.perf_counter()
    for _ in range(repeats):
        acc = oracle.conv_acc(wint, x, d, 0)
        _, y, _ = oracle.epilogue(acc, rs, 0, ref["rowscale"], c["s_x"], None, True)
    t1 = time.perf_counter()
    ops = 2.0 * c["M"] * wl["K"] * acc.shape[1] * repeats
    return dict(value=ops / (t1 - t0) / 1e12, unit="TOPS", cores=oracle.num_threads(), kind="oracle",
                sample="all %d images of the same layer, %d passes (%.2f s wall on %d threads)"
                       % (c["B"], repeats, t1 - t0, oracle.num_threads())), ref, y


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (a known-size kernel to scale rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE readings with)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (--gpus 1); the path shards over output "
              "pixels with replicated weights and needs no communication", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2111_00153_amd as rm

    dev = torch.device("cuda:0")
    wl = make_conv_workload(1)
    c = wl["cfg"]
    M, K = c["M"], wl["K"]
    OH = (c["H"] + 2 * c["pad"] - c["KH"]) // c["stride"] + 1
    OW = (c["W"] + 2 * c["pad"] - c["KW"]) // c["stride"] + 1
    N = c["B"] * OH * OW

    base = None
    s_out = 0.5
    if not args.no_cpu_baseline:
        base, ref, y = cpu_baseline(wl)
        s_out = float(np.percentile(y, 99.9)) / 15.0
    inv = np.float32(1.0 / s_out)

    p = rm.rmsmp_pack_weights(wl["W"], wl["scheme"], taps=c["KH"] * c["KW"])
    X = torch.from_numpy(rm.pack_u4(wl["x"])).to(dev)
    Y = torch.empty((N, M // 2), dtype=torch.uint8, device=dev)
    d = rm.ConvDesc(c["B"], c["C"], c["H"], c["W"], c["KH"], c["KW"], c["stride"], c["pad"])
    ep = rm.make_epilogue(c["s_x"], 0, 4, None, True, rm.OUT_U4, inv)
    ws_bytes = rm.rmsmp_conv2d_workspace_size(p, d, 4)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev) if ws_bytes else None

    step = rm.conv2d_launcher(p, X, d, ep, Y, ws)  # arguments marshalled once; one call = one step
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    gpu_ms = e0.elapsed_time(e1)
    # the job's time is what the host saw between the two synchronizations
    ms_per_step = wall * 1e3 / args.steps
    ops = 2.0 * M * K * N
    tops = ops / (ms_per_step * 1e-3) / 1e12
    kern_ms = gpu_ms / args.steps
    achieved = ops / (kern_ms * 1e-3) / 1e12
    kernel, split = rm.rmsmp_debug_last_dispatch()
    kernel_name = ("rmsmp::conv_wide_kernel<9, 8, %d, %d, %d, %d, false>" % split) if kernel == "lds_resident" else kernel

    if base is not None:
        # spot check of the timed configuration against the oracle (first images)
        import oracle
        n_img = 2
        dd = oracle.conv_desc(n_img, c["C"], c["H"], c["W"], c["KH"], c["KW"], c["stride"], c["pad"])
        acc = oracle.conv_acc(ref["wint"].reshape(M, c["C"], c["KH"], c["KW"]), wl["x"][:n_img].astype(np.int32), dd, 0)
        _, _, q = oracle.epilogue(acc, oracle.rowsum(ref["wint"]), 0, ref["rowscale"], c["s_x"], None, True, inv)
        got = rm.unpack_u4(Y[: n_img * OH * OW].cpu().numpy())  # [n][grouped row]
        chk = np.empty_like(q)
        chk[p.perm] = got.T
        if not np.array_equal(chk, q):
            print("bench.py: GPU output differs from the oracle", file=sys.stderr)
            sys.exit(1)

    out = {
        "metric": "effective int TOPS of row-wise mixed-scheme GEMM (% int8 MFMA peak), 1 GPU",
        "value": round(tops, 2), "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 6), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "pct_of_int8_mfma_peak": round(100.0 * tops / INT8_MFMA_PEAK_TOPS, 2),
        "config": {"workload": "configs[1]: ResNet-18 3x3 conv via im2col, batch 32, 256->256 ch, 14x14, s1 p1 "
                               "(GEMM M=256 K=2304 N=6272), rows Fixed4:PoT4:Fixed8 = 60:35:5, uint4 activations, "
                               "fused ReLU + uint4 requant",
                   "rows_per_scheme": list(wl["counts"])},
        "roofline": {"bound": "mfma", "achieved": round(achieved, 2), "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
                     "frac": round(achieved / INT8_MFMA_PEAK_TOPS, 4), "traffic": MEASURED_TRAFFIC_BYTES,
                     "kernel": kernel_name, "avg_launch_us": round(kern_ms * 1e3, 3)},
        "cpu_baseline": base,
    }
    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
    print(json.dumps(out))
    p.free()


if __name__ == "__main__":
    main()
