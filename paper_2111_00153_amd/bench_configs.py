#!/usr/bin/env python3
"""Times the library on every benchmark configuration (synthetic inputs, one GPU) and prints a table.

    python -m paper_2111_00153_amd.bench_configs [gemm] [conv] [skinny] [sweep] [extra] [qat] [calib]

(`calib` adds one plain 256 MiB device-to-device copy: a kernel of known size to scale rocprofv3's
FETCH_SIZE / WRITE_SIZE readings with when the script runs under the profiler.)

Protocol: 20 warm-up launches, then five blocks of back-to-back launches on one stream between two
events; the median block is reported.  Throughput counts 2*M*K*N operations of the logical GEMM
whatever the row schemes or padding.  The skinny configuration (weights 4096 x 4096, 1..64
activation columns) is timed twice: "warm" launches the same packed weights every time (they stay
in the last-level cache), "cold" rotates through enough packed copies (> 512 MB) that every launch
streams its weights from HBM.  No oracle is involved here: parity is the tests' job.
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import torch  # noqa: E402

import paper_2111_00153_amd as rm  # noqa: E402
import synth_inputs as si  # noqa: E402

DEV = torch.device("cuda:0")


def time_launches(fns, iters=200, warm=20, blocks=5):
    """fns: list of zero-argument launchers used round-robin.  Returns microseconds per launch."""
    k = len(fns)
    for i in range(warm):
        fns[i % k]()
    torch.cuda.synchronize()
    res = []
    for _ in range(blocks):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(iters):
            fns[i % k]()
        e1.record()
        torch.cuda.synchronize()
        res.append(e0.elapsed_time(e1) * 1e3 / iters)
    return float(np.median(res))


def weight_bytes(p, K):
    return sum(c * K * b for c, b in zip(p.counts, (0.5, 0.5, 1.0)))


def gemm_case(cfg, M, K, N, ratio, out_kind, z=0, copies=1, label=""):
    rng = si.rng_for(cfg)
    W = si.weights_rowscaled(rng, M, K)
    scheme = si.scheme_permutation(rng, rm.rmsmp_ratio_counts(M, *ratio))
    packs = [rm.rmsmp_pack_weights(W, scheme) for _ in range(copies)]
    X = torch.from_numpy(rm.pack_u4(si.act_codes_u4(rng, (N, K)))).to(DEV)
    if out_kind == rm.OUT_U4:
        Y = torch.empty((N, M // 2), dtype=torch.uint8, device=DEV)
    else:
        Y = torch.empty((M, N), dtype=torch.float32, device=DEV)
    ep = rm.make_epilogue(0.05, z, 4, None, out_kind == rm.OUT_U4, out_kind, 2.0)
    fns = [rm.gemm_launcher(p, X, N, ep, Y) for p in packs]
    us = time_launches(fns)
    wb = weight_bytes(packs[0], K)
    kind = {rm.OUT_U4: "u4", rm.OUT_FP32: "fp32"}[out_kind]
    print("cfg%d gemm M%d K%d N%d out=%s %s: %8.2f us  %8.1f TOPS  weights %.2f MB -> %7.1f GB/s"
          % (cfg, M, K, N, kind, label, us, 2.0 * M * K * N / us / 1e6, wb / 1e6, wb / us / 1e3), flush=True)
    for p in packs:
        p.free()
    return us


def conv_case(cfg, idx, B, geom=None, M=None, ratio=(35, 60, 5), quiet=False, pack_flags=0):
    if geom is None:
        name, C, M, k, s, pad, H = si.RESNET18_CONVS[idx]
    else:
        name, C, k, s, pad, H = geom
    rng = si.rng_for(cfg, idx)
    K = C * k * k
    W = si.weights_rowscaled(rng, M, K)
    if cfg == 3 and idx == 0:  # first layer: Fixed-8 rows, signed 8-bit image
        scheme = np.full(M, 2, np.uint8)
        bits = 8
        X = torch.from_numpy(si.act_codes_i8(rng, (B, H, H, C))).to(DEV)
    else:
        scheme = si.scheme_permutation(rng, rm.rmsmp_ratio_counts(M, *ratio))
        bits = 4
        X = torch.from_numpy(rm.pack_u4(si.act_codes_u4(rng, (B, H, H, C)))).to(DEV)
    p = rm.rmsmp_pack_weights(W, scheme, taps=k * k, flags=pack_flags)
    d = rm.ConvDesc(B, C, H, H, k, k, s, pad)
    OH = (H + 2 * pad - k) // s + 1
    N = B * OH * OH
    Y = torch.empty((N, M // 2), dtype=torch.uint8, device=DEV)
    wsb = rm.rmsmp_conv2d_workspace_size(p, d, bits)
    ws = torch.empty(wsb, dtype=torch.uint8, device=DEV) if wsb else None
    f = rm.conv2d_launcher(p, X, d, rm.make_epilogue(0.05, 0, bits, None, True, rm.OUT_U4, 2.0), Y, ws)
    us = time_launches([f], iters=100, warm=10)
    ops = 2.0 * M * K * N
    if not quiet:
        print("cfg%d %-22s M%-4d K%-5d N%-7d: %9.2f us  %8.1f TOPS" % (cfg, name, M, K, N, us, ops / us / 1e6), flush=True)
    p.free()
    return us, ops


# Section 4 / Table 6 ratios, written PoT-4 : Fixed-4 : Fixed-8 as the paper does.
TABLE6_RATIOS = [(0, 100, 0), (100, 0, 0), (50, 50, 0), (60, 40, 0), (67, 33, 0), (60, 35, 5), (65, 30, 5), (35, 60, 5)]


def ratio_sweep():
    """Throughput against the scheme ratio (Table 6's rows) on configs[1] and on the ResNet-18 stack,
    with PoT rows nibble-packed (decoded in registers) and with PoT rows stored as int8.
    On matrix cores every scheme multiplies at the same rate; what changes is the decode work."""
    for ratio in TABLE6_RATIOS:
        res = []
        for flags in (0, rm.PACK_POT_AS_INT8):
            us1, ops1 = conv_case(1, 0, 32, geom=("configs[1] %d:%d:%d" % ratio, 256, 3, 1, 1, 14), M=256, ratio=ratio, quiet=True, pack_flags=flags)
            tot_us = tot_ops = 0.0
            for i in range(len(si.RESNET18_CONVS)):
                us, ops = conv_case(3, i, 64, ratio=ratio, quiet=True, pack_flags=flags)
                tot_us += us
                tot_ops += ops
            res.append((us1, ops1 / us1 / 1e6, tot_us / 1e3, tot_ops / tot_us / 1e6))
        print("sweep PoT4:Fixed4:Fixed8 = %3d:%3d:%2d   configs[1] %6.2f us %7.1f TOPS   ResNet-18 stack %.3f ms %6.1f TOPS"
              "   | PoT rows as int8: configs[1] %6.2f us %7.1f TOPS   stack %.3f ms %6.1f TOPS" % (ratio + res[0] + res[1]), flush=True)


def extra_layers():
    """The inference GEMMs of the paper's models that the five configurations do not cover."""
    gemm_case(5, 1000, 512, 64, (0, 0, 100), rm.OUT_FP32, label="ResNet-18 FC, Fixed-8 rows")
    gemm_case(5, 768, 768, 4096, (35, 60, 5), rm.OUT_U4, z=7, label="BERT-base QKV / attention-out shape")
    gemm_case(5, 768, 3072, 4096, (35, 60, 5), rm.OUT_U4, z=7, label="BERT-base FFN down-projection shape")
    gemm_case(5, 3072, 768, 512, (35, 60, 5), rm.OUT_U4, z=7, label="BERT-base FFN up-projection, 512 tokens")


def qat_kernels():
    """Weight projection (forward) and straight-through backward on a 16384 x 4096 fp32 tensor (256 MiB in,
    256 MiB out: larger than the last-level cache, so the rates are HBM rates).  Streaming kernels."""
    M, K = 16384, 4096
    rng = si.rng_for(6)
    W = torch.from_numpy(si.weights_rowscaled(rng, M, K)).to(DEV)
    G = torch.from_numpy(rng.standard_normal((M, K)).astype(np.float32)).to(DEV)
    scheme = torch.from_numpy(si.scheme_permutation(rng, rm.rmsmp_ratio_counts(M, 35, 60, 5))).to(DEV)
    out = torch.empty_like(W)
    alpha = W.abs().amax(dim=1).mul_(0.5).contiguous()
    cases = [("fake_quant_rows, alpha = row maximum", lambda: rm.rmsmp_fake_quant_rows(W, scheme, out), 8),
             ("fake_quant_rows, alpha supplied", lambda: rm.rmsmp_fake_quant_rows(W, scheme, out, alpha), 8),
             ("ste_backward, no clip (copy)", lambda: rm.rmsmp_ste_backward(G, out), 8),
             ("ste_backward, clip mask", lambda: rm.rmsmp_ste_backward(G, out, W, alpha), 12)]
    for name, fn, bpe in cases:
        us = time_launches([fn], iters=20, warm=3)
        print("qat %-40s M%d K%d: %8.2f us  %7.1f GB/s (%d algorithmic bytes per weight)"
              % (name, M, K, us, M * K * bpe / us / 1e3, bpe), flush=True)


def main():
    which = set(sys.argv[1:]) or {"gemm", "conv", "skinny"}
    print("device:", torch.cuda.get_device_name(0), flush=True)
    if "gemm" in which:
        gemm_case(0, 64, 576, 256, (35, 60, 5), rm.OUT_FP32)
        gemm_case(2, 3072, 768, 4096, (35, 60, 5), rm.OUT_U4, z=7)
        gemm_case(2, 3072, 768, 4096, (35, 60, 5), rm.OUT_FP32, z=7)
    if "conv" in which:
        conv_case(1, 0, 32, geom=("configs[1] 3x3 256->256", 256, 3, 1, 1, 14), M=256)
        tot_us = tot_ops = 0.0
        for i in range(len(si.RESNET18_CONVS)):
            us, ops = conv_case(3, i, 64)
            tot_us += us
            tot_ops += ops
        # (the sum of the 20 layers timed one by one; bench.py times the step itself, back to back)
        print("cfg3 ResNet-18 conv stack, batch 64, sum of the layers timed one by one: %.3f ms, %.1f TOPS (%.1f GOP)"
              % (tot_us / 1e3, tot_ops / tot_us / 1e6, tot_ops / 1e9), flush=True)
    if "skinny" in which:
        for N in (1, 8, 64):
            gemm_case(4, 4096, 4096, N, (40, 50, 10), rm.OUT_FP32, label="warm")
        for N in (1, 8, 64):
            gemm_case(4, 4096, 4096, N, (40, 50, 10), rm.OUT_FP32, copies=58, label="cold")
    if "sweep" in which:
        ratio_sweep()
    if "extra" in which:
        extra_layers()
    if "qat" in which:
        qat_kernels()
    if "calib" in which:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=DEV).fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()


if __name__ == "__main__":
    main()
