#!/usr/bin/env python3
"""Benchmark of the RMSMP hot path on one MI355X.

One step = one pass of the whole hot path over one batch of configs[3]: the 20 convolutions of
ResNet-18 at batch 64 and 224x224 (Section 4.2 / Table 6's workload, 232.1 GOP), each one
rmsmp_conv2d call -- conv1 with Fixed-8 rows and 8-bit activations, the others with weight rows
Fixed4:PoT4:Fixed8 = 60:35:5 and unsigned 4-bit activations resident in HBM, fused ReLU + 4-bit
requantization -- launched back to back on one stream; the first 3x3 layer of stages 2-4 and the
stage's 1x1 shortcut projection read the same tensor and go out together as one
rmsmp_conv2d_pair call (17 launches per step).  Prints one JSON line.

Besides the contract fields the line carries: per-layer times, the time share of every kernel
family, the same step with the batch cut in two halves on two streams, the other configurations (configs[1], configs[2], configs[4] with cold weights), the
measured MFMA-only and stream-copy rates of this machine, and the CPU oracle's rate.
"""
import argparse
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

INT8_MFMA_PEAK_TOPS = 5000.0  # MI355X dense int8, published
HBM_PEAK_GBS = 8000.0
BATCH = 64


def _conv_out(h, k, s, p):
    return (h + 2 * p - k) // s + 1


def make_stack(rm, si, torch, dev, batch, inv_scales=None, pack_flags=0, reuse=None):
    """Synthetic ResNet-18 conv stack: packed weights, resident inputs, output buffers, launchers.
    reuse: a stack built earlier whose input tensors this one shares (same seeds, same values)."""
    layers = []
    by_name = {}
    for idx, (name, C, M, k, s, pad, H) in enumerate(si.RESNET18_CONVS):
        rng = si.rng_for(3, idx)
        K = C * k * k
        W = si.weights_rowscaled(rng, M, K)
        if idx == 0:  # first layer: Fixed-8 rows, signed 8-bit image (Section 4: first and last layers 8-bit)
            scheme = np.full(M, 2, np.uint8)
            x, s_x = si.symmetric_i8_from_float(rng.standard_normal((batch, H, H, C)))
            bits = 8
        else:
            scheme = si.scheme_permutation(rng, rm.rmsmp_ratio_counts(M, 35, 60, 5))
            s_x, bits = 0.05, 4
            x = None if name.endswith(".downsample") or reuse is not None else si.act_codes_u4(rng, (batch, H, H, C))
        OH = _conv_out(H, k, s, pad)
        N = batch * OH * OH
        p = rm.rmsmp_pack_weights(W, scheme, taps=k * k, flags=pack_flags)
        d = rm.ConvDesc(batch, C, H, H, k, k, s, pad)
        if reuse is not None:
            x, X = reuse[idx]["x"], reuse[idx]["X"]
        elif x is None:
            # the 1x1 projection of a stage's shortcut reads the stage's input: the tensor of its first 3x3 layer
            head = by_name[name.replace(".downsample", ".conv1")]
            x, X = head["x"], head["X"]
        else:
            X = torch.from_numpy(x if bits == 8 else rm.pack_u4(x)).to(dev)
        Y = torch.empty((N, M // 2), dtype=torch.uint8, device=dev)
        inv = np.float32(2.0 if inv_scales is None else inv_scales[idx])
        ep = rm.make_epilogue(s_x, 0, bits, None, True, rm.OUT_U4, inv)
        wsb = rm.rmsmp_conv2d_workspace_size(p, d, bits)
        ws = torch.empty(wsb, dtype=torch.uint8, device=dev) if wsb else None
        layers.append(dict(idx=idx, name=name, C=C, M=M, k=k, s=s, pad=pad, H=H, OH=OH, N=N, K=K, W=W, scheme=scheme,
                           x=x, s_x=s_x, bits=bits, p=p, d=d, X=X, Y=Y, ep=ep, inv=inv, ws=ws, ops=2.0 * M * K * N,
                           launch=rm.conv2d_launcher(p, X, d, ep, Y, ws)))
        by_name[name] = layers[-1]
    return layers


def launch_units(rm, layers, stream=None, batch=None, part=0):
    """The launches of one step, in layer order: one rmsmp_conv2d per layer, except that a stage's
    first 3x3 layer and its shortcut projection (same input) go out together as one
    rmsmp_conv2d_pair.  batch / part: only images part*batch .. (part+1)*batch-1 (same buffers)."""
    units, by_name, taken = [], {L["name"]: L for L in layers}, set()

    def view(L):
        if batch is None:
            return L["d"], L["X"], L["Y"]
        n = L["N"] // (L["d"].B // batch)
        return (rm.ConvDesc(batch, L["C"], L["H"], L["H"], L["k"], L["k"], L["s"], L["pad"]),
                L["X"][part * batch:(part + 1) * batch], L["Y"][part * n:(part + 1) * n])

    for L in layers:
        if L["name"] in taken:
            continue
        side = by_name.get(L["name"].replace(".conv1", ".downsample")) if L["name"].endswith(".0.conv1") else None
        if side is not None and L["ws"] is None and side["ws"] is None:
            (da, Xa, Ya), (db, _, Yb) = view(L), view(side)
            units.append(dict(layers=[L, side], launch=rm.conv2d_pair_launcher(L["p"], da, L["ep"], Ya, side["p"], db, side["ep"], Yb, Xa, stream=stream)))
            taken.add(side["name"])
        else:
            if batch is not None and L["ws"] is not None:
                raise SystemExit("bench.py: a layer with an im2col workspace cannot be shared by two streams")
            d, X, Y = view(L)
            units.append(dict(layers=[L], launch=rm.conv2d_launcher(L["p"], X, d, L["ep"], Y, L["ws"], stream=stream)))
    return units


def kernel_of(rm, layer):
    layer["launch"]()
    kernel, split = rm.rmsmp_debug_last_dispatch()
    taps, cpt = layer["k"] * layer["k"], layer["C"] // 32
    if kernel == "lds_resident":
        return "rmsmp::conv_wide_kernel<%d, %d, %d, %d, %d, %d, false>" % ((taps, cpt) + split)
    if kernel == "first_layer":
        return "rmsmp::conv_first_kernel"
    return kernel


def oracle_reference(oracle, layer, images):
    """Oracle accumulators -> fp32 output of the given images of one layer (weights quantized by the oracle)."""
    ref = oracle.quantize_rows(layer["W"], layer["scheme"], want_levels=False)
    k, C, M = layer["k"], layer["C"], layer["M"]
    d = oracle.conv_desc(len(images), C, layer["H"], layer["H"], k, k, layer["s"], layer["pad"])
    acc = oracle.conv_acc(ref["wint"].reshape(M, C, k, k), layer["x"][images].astype(np.int32), d, 0)
    rs = oracle.rowsum(ref["wint"])
    return ref, acc, rs


def cpu_baseline(oracle, si, sample_batch=8):
    """The oracle as it stands on a bounded sample of the same workload: all 20 layers on
    `sample_batch` images (all host threads), and the deepest 3x3 layer on one image with one thread."""
    macs = 0
    t0 = time.perf_counter()
    for idx, (name, C, M, k, s, pad, H) in enumerate(si.RESNET18_CONVS):
        rng = si.rng_for(3, idx)
        W = si.weights_rowscaled(rng, M, C * k * k)
        scheme = np.full(M, 2, np.uint8) if idx == 0 else si.scheme_permutation(rng, oracle.ratio_counts(M, 35, 60, 5))
        ref = oracle.quantize_rows(W, scheme, want_levels=False)
        x = (si.act_codes_i8(rng, (sample_batch, H, H, C)) if idx == 0 else si.act_codes_u4(rng, (sample_batch, H, H, C)))
        d = oracle.conv_desc(sample_batch, C, H, H, k, k, s, pad)
        acc = oracle.conv_acc(ref["wint"].reshape(M, C, k, k), x.astype(np.int32), d, 0)
        oracle.epilogue(acc, oracle.rowsum(ref["wint"]), 0, ref["rowscale"], 0.05, None, True, np.float32(2.0))
        macs += M * C * k * k * acc.shape[1]
    t1 = time.perf_counter()
    threads = oracle.num_threads()
    # one thread, one layer (layer3.1.conv1, 115.6 MMAC per image)
    name, C, M, k, s, pad, H = si.RESNET18_CONVS[13]
    rng = si.rng_for(3, 13)
    W = si.weights_rowscaled(rng, M, C * k * k)
    ref = oracle.quantize_rows(W, si.scheme_permutation(rng, oracle.ratio_counts(M, 35, 60, 5)), want_levels=False)
    x = si.act_codes_u4(rng, (1, H, H, C))
    d = oracle.conv_desc(1, C, H, H, k, k, s, pad)
    oracle.set_threads(1)
    t2 = time.perf_counter()
    acc1 = oracle.conv_acc(ref["wint"].reshape(M, C, k, k), x.astype(np.int32), d, 0)
    t3 = time.perf_counter()
    oracle.set_threads(threads)
    single = 2.0 * M * C * k * k * acc1.shape[1] / (t3 - t2) / 1e12
    return dict(value=2.0 * macs / (t1 - t0) / 1e12, unit="TOPS", cores=threads, kind="oracle",
                sample="all 20 layers of configs[3] on %d images (%.2f s wall on %d threads); one thread alone on "
                       "layer3.1.conv1, one image: %.5f TOPS (%.2f s)" % (sample_batch, t1 - t0, threads, single, t3 - t2),
                single_thread_value=single)


def check_against_oracle(rm, oracle, torch, layers):
    """First and last image of every layer: 4-bit codes of the timed launches against the oracle."""
    for L in layers:
        imgs = [0, BATCH - 1]
        ref, acc, rs = oracle_reference(oracle, L, imgs)
        _, _, q = oracle.epilogue(acc, rs, 0, ref["rowscale"], L["s_x"], None, True, L["inv"])
        hw = L["OH"] * L["OH"]
        Y = L["Y"].view(BATCH, hw, L["M"] // 2)[torch.tensor(imgs)].reshape(2 * hw, L["M"] // 2).cpu().numpy()
        got = rm.unpack_u4(Y)  # [n][grouped row]
        chk = np.empty_like(q)
        chk[L["p"].perm] = got.T
        if not np.array_equal(chk, q):
            print("bench.py: GPU output of %s differs from the oracle" % L["name"], file=sys.stderr)
            sys.exit(1)


def time_block(torch, fns, iters, warm, reps=5):
    """Microseconds per launch: the median over reps blocks of iters back-to-back launches, each
    block between two events on the launch stream (a single block can catch a clock or power step)."""
    for i in range(warm):
        fns[i % len(fns)]()
    torch.cuda.synchronize()
    times = []
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(iters):
            fns[i % len(fns)]()
        e1.record()
        torch.cuda.synchronize()
        times.append(e0.elapsed_time(e1) * 1e3 / iters)
    return float(np.median(times))


def other_configs(rm, si, torch, dev):
    """configs[1], configs[2] (4-bit and fp32 output) and configs[4] with cold weights, timed as
    blocks of back-to-back launches between two events (no oracle: parity is the tests' job)."""
    out = {}
    # configs[1]
    c = si.CONFIGS[1]
    rng = si.rng_for(1)
    K = c["C"] * 9
    W = si.weights_rowscaled(rng, c["M"], K)
    scheme = si.scheme_permutation(rng, rm.rmsmp_ratio_counts(c["M"], *c["ratio"]))
    p = rm.rmsmp_pack_weights(W, scheme, taps=9)
    X = torch.from_numpy(rm.pack_u4(si.act_codes_u4(rng, (c["B"], 14, 14, c["C"])))).to(dev)
    N = c["B"] * 196
    Y = torch.empty((N, c["M"] // 2), dtype=torch.uint8, device=dev)
    d = rm.ConvDesc(c["B"], c["C"], 14, 14, 3, 3, 1, 1)
    f = rm.conv2d_launcher(p, X, d, rm.make_epilogue(0.05, 0, 4, None, True, rm.OUT_U4, 2.0), Y, None)
    us = time_block(torch, [f], 1000, 50)
    ops = 2.0 * c["M"] * K * N
    out["configs[1] conv 256->256 3x3 batch 32, u4 out"] = dict(us=round(us, 3), tops=round(ops / us / 1e6, 1),
                                                                frac_of_int8_peak=round(ops / us / 1e6 / INT8_MFMA_PEAK_TOPS, 4))
    p.free()
    # configs[2]
    M, K, N = 3072, 768, 4096
    rng = si.rng_for(2)
    W = si.weights_bert(rng, M, K)
    scheme = si.scheme_permutation(rng, rm.rmsmp_ratio_counts(M, 35, 60, 5))
    xq, s_x, z = si.affine_u4_from_float(rng.standard_normal((N, K)))
    p = rm.rmsmp_pack_weights(W, scheme)
    X = torch.from_numpy(rm.pack_u4(xq)).to(dev)
    ops = 2.0 * M * K * N
    for kind, label in ((rm.OUT_U4, "u4 out"), (rm.OUT_FP32, "fp32 out")):
        Y = (torch.empty((N, M // 2), dtype=torch.uint8, device=dev) if kind == rm.OUT_U4
             else torch.empty((M, N), dtype=torch.float32, device=dev))
        f = rm.gemm_launcher(p, X, N, rm.make_epilogue(s_x, z, 4, None, kind == rm.OUT_U4, kind, 2.0), Y)
        us = time_block(torch, [f], 500, 30)
        out["configs[2] BERT FFN-up 3072x768x4096, " + label] = dict(
            us=round(us, 3), tops=round(ops / us / 1e6, 1), frac_of_int8_peak=round(ops / us / 1e6 / INT8_MFMA_PEAK_TOPS, 4))
    p.free()
    # configs[4]: enough packed copies (> the 256 MB last-level cache) that every launch streams from HBM
    M = K = 4096
    rng = si.rng_for(4)
    W = si.weights_rowscaled(rng, M, K)
    scheme = si.scheme_permutation(rng, rm.rmsmp_ratio_counts(M, 40, 50, 10))
    packs = [rm.rmsmp_pack_weights(W, scheme) for _ in range(40)]
    wbytes = sum(cnt * K * b for cnt, b in zip(packs[0].counts, (0.5, 0.5, 1.0)))
    for N in (1, 8, 64):
        X = torch.from_numpy(rm.pack_u4(si.act_codes_u4(rng, (N, K)))).to(dev)
        Y = torch.empty((M, N), dtype=torch.float32, device=dev)
        ep = rm.make_epilogue(0.05, 0, 4, None, False, rm.OUT_FP32, 1.0)
        fns = [rm.gemm_launcher(pk, X, N, ep, Y) for pk in packs]
        us = time_block(torch, fns, 400, 40)
        out["configs[4] skinny 4096x4096 N=%d, cold weights" % N] = dict(
            us=round(us, 3), tops=round(2.0 * M * K * N / us / 1e6, 2), weight_gbs=round(wbytes / us / 1e3, 1),
            frac_of_hbm_peak=round(wbytes / us / 1e3 / HBM_PEAK_GBS, 4))
    for pk in packs:
        pk.free()
    return out


def two_stream_schedule(rm, torch, layers, steps, warm):
    """The same step with the batch cut in two halves that run on two streams (every image still
    passes through the layers in order; 40 launches per step).  Launches of the two streams overlap
    on the chip: one half's prologues, epilogues and launch gaps run under the other half's MFMA
    phases.  The outputs land in the same buffers and are compared byte for byte with what the
    one-stream step left there."""
    half = BATCH // 2
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    expect = [L["Y"].clone() for L in layers]
    for L in layers:
        L["Y"].zero_()
    halves = [launch_units(rm, layers, stream=streams[i], batch=half, part=i) for i in range(2)]
    launchers = list(zip(*[[u["launch"] for u in h] for h in halves]))
    torch.cuda.synchronize()

    def step():
        for pair in launchers:
            pair[0]()
            pair[1]()

    for _ in range(warm):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    same = all(bool(torch.equal(L["Y"], e)) for L, e in zip(layers, expect))
    if not same:
        raise SystemExit("bench.py: the two-stream schedule's outputs differ from the one-stream step's")
    ops = sum(L["ops"] for L in layers)
    return {"ms_per_step": round(ms, 6), "tops": round(ops / (ms * 1e-3) / 1e12, 2), "launches_per_step": 2 * len(launchers),
            "outputs_identical_to_one_stream_step": same,
            "note": "batch 64 as two halves of 32 on two streams, layer order kept per image; not the headline "
                    "(the headline is the one-stream step that the kernel trace and the per-layer times describe)"}


def pot_rows_as_int8(rm, si, torch, dev, layers, steps, warm):
    """The same one-stream step with the PoT-4 rows of every layer stored decoded, one byte per
    weight (RMSMP_PACK_POT_AS_INT8): same levels, scales and output codes, no table decode in the
    K loop, twice the bytes for those rows.  The codes of every layer are compared, in original row
    order, with what the headline step left in its buffers."""
    alt = make_stack(rm, si, torch, dev, BATCH, [L["inv"] for L in layers], rm.PACK_POT_AS_INT8, reuse=layers)
    launchers = [u["launch"] for u in launch_units(rm, alt)]

    def step():
        for f in launchers:
            f()

    def codes(L):  # [N][M] in original row order
        g = torch.stack((L["Y"] & 15, L["Y"] >> 4), dim=2).reshape(L["N"], L["M"])
        out = torch.empty_like(g)
        out[:, torch.from_numpy(np.asarray(L["p"].perm, dtype=np.int64)).to(g.device)] = g
        return out

    for _ in range(warm):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    same = all(bool(torch.equal(codes(a), codes(b))) for a, b in zip(alt, layers))
    if not same:
        raise SystemExit("bench.py: the step with PoT rows stored as int8 gives other codes than the headline step")
    ops = sum(L["ops"] for L in layers)
    wbytes = [sum(cnt * L["K"] * b for cnt, b in zip(L["p"].counts, fac)) for L in layers[1:] for fac in ((0.5, 0.5, 1.0), (0.5, 1.0, 1.0))]
    for L in alt:
        L["p"].free()
    return {"ms_per_step": round(ms, 6), "tops": round(ops / (ms * 1e-3) / 1e12, 2),
            "pct_of_int8_mfma_peak": round(100.0 * ops / (ms * 1e-3) / 1e12 / INT8_MFMA_PEAK_TOPS, 2),
            "codes_identical_to_headline_step": same,
            "weight_bytes_mixed_layers": {"nibble_storage": int(sum(wbytes[0::2])), "pot_as_int8": int(sum(wbytes[1::2]))},
            "note": "not the headline: the headline keeps both 4-bit schemes nibble-packed and decodes PoT codes in registers"}


def chained_step(rm, oracle, si, torch, dev, layers, steps, warm):
    """The same 17 launches with every layer from layer1.0.conv2 on reading the 4-bit tensor the
    layer before it wrote (a stage's first 3x3 layer and its shortcut projection read the previous
    stage's output; residual adds and pooling are outside the path, so conv1 does not feed layer1).
    A layer writes its codes in grouped row order and the next layer's weights are packed with
    in_perm = that order, so nothing is shuffled between the launches.  With the oracle at hand it
    runs the same chain on the first and the last image first -- the output scale of every layer is
    the 99.9th percentile of its own output there, so that the chain stays alive -- and the codes
    of every layer, up to 19 chained layers deep, are compared bit for bit."""
    def producer(name):
        stage, block, conv = name.split(".")
        if conv == "conv2":
            return "%s.%s.conv1" % (stage, block)
        if block == "1":
            return "%s.0.conv2" % stage
        return None if stage == "layer1" else "layer%d.1.conv2" % (int(stage[5:]) - 1)

    imgs = [0, BATCH - 1]
    want, inv_of, hist = {}, {}, None
    if oracle is not None:
        out = {}
        for L in layers[1:]:
            src = producer(L["name"])
            x = L["x"][imgs] if src is None else out[src]
            ref = oracle.quantize_rows(L["W"], L["scheme"], want_levels=False)
            k, M = L["k"], L["M"]
            d = oracle.conv_desc(len(imgs), L["C"], L["H"], L["H"], k, k, L["s"], L["pad"])
            acc = oracle.conv_acc(ref["wint"].reshape(M, L["C"], k, k), x.astype(np.int32), d, 0)
            rs = oracle.rowsum(ref["wint"])
            _, y, _ = oracle.epilogue(acc, rs, 0, ref["rowscale"], L["s_x"], None, True)
            inv = np.float32(15.0 / max(float(np.percentile(y, 99.9)), 1e-6))
            _, _, q = oracle.epilogue(acc, rs, 0, ref["rowscale"], L["s_x"], None, True, inv)
            want[L["name"]], inv_of[L["name"]] = q, inv
            out[L["name"]] = np.ascontiguousarray(q.T).reshape(len(imgs), L["OH"], L["OH"], M).astype(np.uint8)  # NHWC, original channel order
            hist = np.bincount(q.ravel(), minlength=16).tolist()

    chain = []
    for L in layers:
        src = None if L["idx"] == 0 else producer(L["name"])
        C = dict(L)
        if src is not None:
            P = next(c for c in chain if c["name"] == src)
            C["p"] = rm.rmsmp_pack_weights(L["W"], L["scheme"], taps=L["k"] * L["k"], in_perm=P["p"].perm)
            C["X"] = P["Y"].view(BATCH, L["H"], L["H"], L["C"] // 2)
            C["own_pack"] = True
        if L["name"] in inv_of:
            C["ep"] = rm.make_epilogue(L["s_x"], 0, L["bits"], None, True, rm.OUT_U4, inv_of[L["name"]])
        C["Y"] = torch.empty_like(L["Y"])
        chain.append(C)
    launchers = [u["launch"] for u in launch_units(rm, chain)]

    def step():
        for f in launchers:
            f()

    for _ in range(warm):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    checked = None
    if oracle is not None:
        for C in chain[1:]:
            q, M, hw = want[C["name"]], C["M"], C["OH"] * C["OH"]
            Y = C["Y"].view(BATCH, hw, M // 2)[torch.tensor(imgs)].reshape(len(imgs) * hw, M // 2).cpu().numpy()
            got = np.empty_like(q)
            got[C["p"].perm] = rm.unpack_u4(Y).T
            if not np.array_equal(got, q):
                raise SystemExit("bench.py: chained step: GPU output of %s differs from the oracle" % C["name"])
        checked = ("every layer of the chain equals the oracle's chain on images 0 and %d; code counts of the last layer there: %s"
                   % (BATCH - 1, hist))
    ops = sum(L["ops"] for L in layers)
    for C in chain:
        if C.get("own_pack"):
            C["p"].free()
    return {"ms_per_step": round(ms, 6), "tops": round(ops / (ms * 1e-3) / 1e12, 2), "launches_per_step": len(launchers),
            "checked": checked,
            "note": "layers 2..20 read the previous layer's 4-bit output (grouped row order, next weights packed with in_perm); "
                    "not the headline: the headline's layers read independent synthetic tensors of the workload's distribution"}


def traffic_from_profile(kernel_name):
    """HBM bytes per launch of the dominant kernel as the committed rocprofv3 counter summary of this
    workload states them (a counter cannot be read from inside this script); None when no summary
    names this kernel."""
    path = os.path.join(ROOT, "profiles", "resnet18_stack_dominant_kernel_traffic.txt")
    try:
        text = open(path).read()
    except OSError:
        return None
    m = re.search(r"^kernel:\s*(.+)$", text, re.M)
    t = re.search(r"^traffic_bytes_per_launch:\s*(\d+)", text, re.M)
    if not m or not t or m.group(1).strip() != kernel_name:
        return None
    return int(t.group(1))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle (its timing and the in-run check)")
    ap.add_argument("--no-extras", action="store_true", help="skip the other configurations and the machine peaks")
    ap.add_argument("--layer-iters", type=int, default=200, help="launches per layer in the per-layer timing pass")
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
    import synth_inputs as si

    dev = torch.device("cuda:0")
    base = None
    inv_scales = None
    if not args.no_cpu_baseline:
        import oracle
        base = cpu_baseline(oracle, si)
    layers = make_stack(rm, si, torch, dev, BATCH)
    if base is not None:
        # output scales from the oracle's own output on the first and last image: s_out = 99.9th percentile / 15
        inv_scales = []
        for L in layers:
            ref, acc, rs = oracle_reference(oracle, L, [0, BATCH - 1])
            _, y, _ = oracle.epilogue(acc, rs, 0, ref["rowscale"], L["s_x"], None, True)
            inv_scales.append(np.float32(15.0 / max(float(np.percentile(y, 99.9)), 1e-6)))
        for L, inv in zip(layers, inv_scales):
            L["inv"] = inv
            L["ep"] = rm.make_epilogue(L["s_x"], 0, L["bits"], None, True, rm.OUT_U4, inv)
            L["launch"] = rm.conv2d_launcher(L["p"], L["X"], L["d"], L["ep"], L["Y"], L["ws"])
    units = launch_units(rm, layers)
    launchers = [u["launch"] for u in units]
    total_ops = sum(L["ops"] for L in layers)

    def step():
        for f in launchers:
            f()

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
    ms_per_step = wall * 1e3 / args.steps  # the job's time is what the host saw between the two synchronizations
    tops = total_ops / (ms_per_step * 1e-3) / 1e12

    if base is not None:
        check_against_oracle(rm, oracle, torch, layers)

    # per-layer times: every layer alone, back to back, between two events (also the two layers of a pair)
    per_layer = {}
    for L in layers:
        L["kernel"] = kernel_of(rm, L)
    torch.cuda.synchronize()
    for L in layers:
        L["us"] = time_block(torch, [L["launch"]], args.layer_iters, 10)
        per_layer[L["name"]] = dict(us=round(L["us"], 3), tops=round(L["ops"] / L["us"] / 1e6, 1), kernel=L["kernel"])
    # the launches of the step, each alone; a fused pair is a kernel family of its own
    families, fused = {}, {}
    for u in units:
        if len(u["layers"]) == 2:
            u["launch"]()
            kernel, _ = rm.rmsmp_debug_last_dispatch()
            if kernel == "lds_resident_pair":
                u["kernel"] = "rmsmp::conv_wide_pair_kernel<%d>" % (u["layers"][0]["C"] // 32)
                u["us"] = time_block(torch, [u["launch"]], args.layer_iters, 10)
                a, b = u["layers"]
                fused[a["name"] + " + " + b["name"]] = dict(us=round(u["us"], 3), one_after_the_other_us=round(a["us"] + b["us"], 3),
                                                            tops=round((a["ops"] + b["ops"]) / u["us"] / 1e6, 1), kernel=u["kernel"])
                for L in u["layers"]:
                    per_layer[L["name"]]["in_the_step"] = "one launch with its partner: " + u["kernel"]
                parts = [(u["kernel"], u["us"], a["ops"] + b["ops"])]
            else:  # the library launched the two layers one after the other
                parts = [(L["kernel"], L["us"], L["ops"]) for L in u["layers"]]
        else:
            L = u["layers"][0]
            u["kernel"] = L["kernel"]
            parts = [(L["kernel"], L["us"], L["ops"])]
        for kname, us, ops in parts:
            fam = families.setdefault(kname, dict(us=0.0, ops=0.0, launches=0))
            fam["us"] += us
            fam["ops"] += ops
            fam["launches"] += 1
    sum_us = sum(v["us"] for v in families.values())
    share = {k: round(v["us"] / sum_us, 4) for k, v in sorted(families.items(), key=lambda kv: -kv[1]["us"])}
    dom_name = max(families, key=lambda k: families[k]["us"])
    dom_units = [u for u in units if u.get("kernel") == dom_name]
    # the dominant kernel's average launch duration: its launches round-robin, back to back, between two events
    dom_us = time_block(torch, [u["launch"] for u in dom_units], max(1, args.layer_iters // 2) * len(dom_units), 4 * len(dom_units))
    dom_ops = sum(L["ops"] for u in dom_units for L in u["layers"]) / len(dom_units)
    dom_layers = [L for u in dom_units for L in u["layers"]]
    achieved = dom_ops / dom_us / 1e6

    out = {
        "metric": "effective int TOPS of row-wise mixed-scheme GEMM (% int8 MFMA peak), 1 GPU",
        "value": round(tops, 2), "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 6), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "pct_of_int8_mfma_peak": round(100.0 * tops / INT8_MFMA_PEAK_TOPS, 2),
        "config": {"workload": "configs[3]: full ResNet-18 conv stack, batch 64, 224x224: 20 conv layers (232.1 GOP per step), "
                               "conv1 Fixed-8 rows x int8 activations, the others rows Fixed4:PoT4:Fixed8 = 60:35:5 x uint4 "
                               "activations, fused ReLU + uint4 requant; one rmsmp_conv2d launch per layer, except that the first 3x3 layer of "
                               "stages 2-4 and the stage's 1x1 shortcut projection (same input tensor) go out as one "
                               "rmsmp_conv2d_pair launch; back to back on one stream",
                   "gop_per_step": round(total_ops / 1e9, 2), "launches_per_step": len(units),
                   "gpu_events_ms_per_step": round(gpu_ms / args.steps, 6)},
        "roofline": {"bound": "mfma", "achieved": round(achieved, 2), "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
                     "frac": round(achieved / INT8_MFMA_PEAK_TOPS, 4), "traffic": traffic_from_profile(dom_name),
                     "kernel": dom_name, "avg_launch_us": round(dom_us, 3), "gop_per_launch": round(dom_ops / 1e9, 3),
                     "layers": [L["name"] for L in dom_layers], "time_share_by_kernel": share},
        "per_layer": per_layer,
        "fused_pairs": fused,
        "cpu_baseline": base,
    }
    if not args.no_extras:
        out["two_stream_schedule"] = two_stream_schedule(rm, torch, layers, args.steps, args.warmup)
        out["chained_step"] = chained_step(rm, oracle if base is not None else None, si, torch, dev, layers, args.steps, args.warmup)
        out["pot_rows_stored_as_int8"] = pot_rows_as_int8(rm, si, torch, dev, layers, args.steps, args.warmup)
        out["other_configs"] = other_configs(rm, si, torch, dev)
        mfma_tops, copy_gbs = rm.rmsmp_debug_measure_peaks()
        out["measured_peaks"] = {"mfma_only_int8_tops": round(mfma_tops, 1), "stream_copy_gbs": round(copy_gbs, 1),
                                 "note": "MFMA-only: 2 waves per SIMD issuing v_mfma_i32_32x32x32_i8 on registers; "
                                         "stream copy: 1 GiB read + 1 GiB written by a plain copy kernel"}
    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
    print(json.dumps(out))
    for L in layers:
        L["p"].free()


if __name__ == "__main__":
    main()
