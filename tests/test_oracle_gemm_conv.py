"""Pins for the oracle's integer GEMM, convolution and epilogue (CPU only).

Brute force in Python integers on tiny inputs, special cases that reduce to numpy /
torch library routines, invariants, and the paper's own operation count (Table 6).
"""
import os

import numpy as np
import pytest
import torch

import synth_inputs as si

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _mixed(oracle, rng, M, K, schemes=(0, 1, 2)):
    W = (rng.standard_normal((M, K)) * rng.uniform(0.01, 0.1, (M, 1))).astype(np.float32)
    sch = np.array([schemes[i % len(schemes)] for i in range(M)], np.uint8)
    return W, sch, oracle.quantize_rows(W, sch)


def test_gemm_bruteforce_python_ints(oracle):
    rng = np.random.default_rng(1)
    M, K, N = 7, 16, 5
    # every code value of every scheme appears at least once
    wint = np.zeros((M, K), np.int32)
    wint[0] = np.arange(-7, 9)[:K].clip(-7, 7)
    wint[1] = np.array([0, 1, 2, 4, 8, 16, 32, 64, -1, -2, -4, -8, -16, -32, -64, 0])
    wint[2] = rng.integers(-127, 128, K)
    wint[2, :2] = (-127, 127)
    wint[3:] = rng.integers(-7, 8, (M - 3, K))
    xq = rng.integers(0, 16, (N, K)).astype(np.int32)
    xq[0] = np.arange(16)
    acc = oracle.gemm_acc(wint, xq)
    for r in range(M):
        for n in range(N):
            s = 0
            for k in range(K):
                s += int(wint[r, k]) * int(xq[n, k])
            assert acc[r, n] == s


@pytest.mark.parametrize("schemes", [(2,), (0,), (1,), (0, 1, 2)])
def test_gemm_reduces_to_numpy_matmul(oracle, schemes):
    """All rows Fixed-8 is a plain int8 GEMM; likewise the other single-scheme layers."""
    rng = np.random.default_rng(2)
    W, sch, r = _mixed(oracle, rng, 24, 200, schemes)
    xq = rng.integers(0, 16, (33, 200)).astype(np.int32)
    ref = r["wint"].astype(np.int64) @ xq.astype(np.int64).T
    assert np.array_equal(oracle.gemm_acc(r["wint"], xq), ref.astype(np.int32))


def test_gemm_invariants(oracle):
    rng = np.random.default_rng(3)
    W, sch, r = _mixed(oracle, rng, 12, 64)
    K = 64
    ones = np.ones((4, K), np.int32)
    assert np.array_equal(oracle.gemm_acc(r["wint"], ones), np.repeat(oracle.rowsum(r["wint"])[:, None], 4, 1))
    assert not oracle.gemm_acc(r["wint"], np.zeros((4, K), np.int32)).any()
    xq = rng.integers(0, 16, (9, K)).astype(np.int32)
    acc = oracle.gemm_acc(r["wint"], xq)
    perm = rng.permutation(12)
    assert np.array_equal(oracle.gemm_acc(r["wint"][perm], xq), acc[perm])
    # a transposed operand would fail this: one-hot activation column picks out a weight column
    e = np.zeros((K, K), np.int32)
    e[np.arange(K), np.arange(K)] = 1
    assert np.array_equal(oracle.gemm_acc(r["wint"], e), r["wint"])
    # sampled evaluation agrees with the full one
    ms, ns = rng.integers(0, 12, 50), rng.integers(0, 9, 50)
    assert np.array_equal(oracle.gemm_acc_at(r["wint"], xq, ms, ns), acc[ms, ns])


def test_gemm_overflow_is_reported(oracle):
    w = np.full((1, 4), 2 ** 30, np.int32)
    x = np.full((1, 4), 2, np.int32)
    with pytest.raises(OverflowError):
        oracle.gemm_acc(w, x)


def test_rowsum_and_zero_point_identity(oracle):
    rng = np.random.default_rng(4)
    W, sch, r = _mixed(oracle, rng, 10, 80)
    xq = rng.integers(0, 16, (6, 80)).astype(np.int32)
    z = 7
    acc = oracle.gemm_acc(r["wint"], xq)
    rs = oracle.rowsum(r["wint"])
    assert np.array_equal(rs, r["wint"].sum(1))
    corr, _, _ = oracle.epilogue(acc, rs, z, r["rowscale"], 0.05)
    assert np.array_equal(corr, oracle.gemm_acc(r["wint"], xq - z))


def _torch_conv(wint, x, d, zpad):
    """float64 CPU conv on integer-valued tensors is exact: a library routine as reference."""
    xt = torch.from_numpy(x.astype(np.float64)).permute(0, 3, 1, 2)  # NHWC -> NCHW
    if d.pad:
        xt = torch.nn.functional.pad(xt, (d.pad,) * 4, value=float(zpad))
    wt = torch.from_numpy(wint.astype(np.float64))
    y = torch.nn.functional.conv2d(xt, wt, stride=d.stride)  # [B][M][OH][OW]
    M = wint.shape[0]
    return y.permute(1, 0, 2, 3).reshape(M, -1).numpy().astype(np.int64)


@pytest.mark.parametrize("geom", [(2, 8, 6, 6, 3, 3, 1, 1), (1, 3, 13, 13, 7, 7, 2, 3), (2, 16, 9, 9, 1, 1, 2, 0),
                                  (3, 4, 5, 7, 3, 3, 2, 1), (1, 6, 7, 5, 3, 2, 1, 0)])
@pytest.mark.parametrize("zpad", [0, 5])
def test_conv_matches_torch_float64(oracle, geom, zpad):
    rng = np.random.default_rng(sum(geom) + zpad)
    B, C, H, W, KH, KW, s, p = geom
    d = oracle.conv_desc(B, C, H, W, KH, KW, s, p)
    M = 5
    wint = rng.integers(-127, 128, (M, C, KH, KW)).astype(np.int32)
    x = rng.integers(0, 16, (B, H, W, C)).astype(np.int32)
    acc = oracle.conv_acc(wint, x, d, zpad)
    ref = _torch_conv(wint, x, d, zpad)
    assert np.array_equal(acc.astype(np.int64), ref)
    OH, OW = oracle.conv_out_hw(d)
    assert acc.shape == (M, B * OH * OW)
    ms, ns = rng.integers(0, M, 40), rng.integers(0, acc.shape[1], 40)
    assert np.array_equal(oracle.conv_acc_at(wint, x, d, ms, ns, zpad), acc[ms, ns])


def test_conv_1x1_is_gemm_and_im2col_is_gemm(oracle):
    rng = np.random.default_rng(9)
    B, C, H, W, M = 2, 12, 5, 4, 7
    d = oracle.conv_desc(B, C, H, W, 1, 1, 1, 0)
    wint = rng.integers(-7, 8, (M, C, 1, 1)).astype(np.int32)
    x = rng.integers(0, 16, (B, H, W, C)).astype(np.int32)
    assert np.array_equal(oracle.conv_acc(wint, x, d), oracle.gemm_acc(wint.reshape(M, C), x.reshape(-1, C)))
    # 3x3: lowering by an explicitly built im2col matrix (filter order c,kh,kw) gives the same numbers
    d = oracle.conv_desc(B, C, H, W, 3, 3, 1, 1)
    wint = rng.integers(-64, 65, (M, C, 3, 3)).astype(np.int32)
    z = 3
    xp = np.full((B, H + 2, W + 2, C), z, np.int32)
    xp[:, 1:-1, 1:-1] = x
    cols = np.empty((B * H * W, C * 9), np.int32)
    n = 0
    for b in range(B):
        for oh in range(H):
            for ow in range(W):
                cols[n] = xp[b, oh:oh + 3, ow:ow + 3, :].transpose(2, 0, 1).ravel()
                n += 1
    assert np.array_equal(oracle.conv_acc(wint, x, d, z), oracle.gemm_acc(wint.reshape(M, -1), cols))


def test_dequant_matches_plain_float64_definition(oracle):
    """rowscale*s_x*(integer sum) equals sum_k w_hat * x_hat within 1e-5 relative."""
    rng = np.random.default_rng(12)
    W, sch, r = _mixed(oracle, rng, 30, 576)
    xq = rng.integers(0, 16, (40, 576)).astype(np.int32)
    bias = (rng.standard_normal(30) * 0.1).astype(np.float32)
    for z, b, relu in [(0, None, False), (6, None, False), (0, bias, True), (9, bias, False)]:
        acc = oracle.gemm_acc(r["wint"], xq)
        _, y, _ = oracle.epilogue(acc, oracle.rowsum(r["wint"]), z, r["rowscale"], 0.05, b, relu)
        y64 = oracle.gemm_f64(r["what"], xq, np.float32(0.05), z, b, relu)
        # a value that is the small difference of a large sum and a bias cannot be relatively
        # tighter than the fp32 rounding of its terms: 1e-5 of the result plus an ulp of the bias
        tol = 1e-5 * np.abs(y64) + (4e-7 * np.abs(b).max() if b is not None else 1e-12)
        assert np.all(np.abs(y - y64) <= tol)
    # gemm_f64 itself against numpy
    xhat = np.float64(np.float32(0.05)) * (xq - 6)
    assert np.allclose(oracle.gemm_f64(r["what"], xq, np.float32(0.05), 6), r["what"] @ xhat.T, rtol=1e-12, atol=1e-12)


def test_requant_properties(oracle):
    rng = np.random.default_rng(13)
    M, N = 8, 500
    acc = rng.integers(-4000, 4000, (M, N)).astype(np.int32)
    rowscale = rng.uniform(0.001, 0.01, M).astype(np.float32)
    s_out = 0.11
    _, y, q = oracle.epilogue(acc, np.zeros(M, np.int32), 0, rowscale, 0.05, None, True, 1.0 / s_out)
    assert q.min() >= 0 and q.max() <= 15 and q.max() == 15 and q.min() == 0
    assert np.all(y >= 0)
    # monotone in y
    o = np.argsort(y.ravel(), kind="stable")
    assert np.all(np.diff(q.ravel()[o].astype(int)) >= 0)
    # nearest code: |y/s - q| <= 1/2 inside the range
    t = y.astype(np.float64) / s_out
    inside = t <= 15
    assert np.all(np.abs(t[inside] - q[inside]) <= 0.5 + 1e-4)
    assert np.all(q[~inside] == 15)
    # re-quantizing the dequantized codes with the same scale returns the codes
    y2 = (q.astype(np.float32) * np.float32(s_out))
    q2 = np.clip(np.rint(y2 * np.float32(1.0 / s_out)), 0, 15).astype(np.uint8)
    assert np.array_equal(q, q2)
    # hand-checked values, s_out = 0.5: y = 0.74 -> 1.48 -> 1 ; 0.76 -> 2 ; 1.25 -> 2.5 -> 2 (even); 1.75 -> 4
    accs = np.array([[74, 76, 125, 175, -50, 5000]], np.int32)
    _, yy, qq = oracle.epilogue(accs, np.zeros(1, np.int32), 0, np.array([0.01], np.float32), 1.0, None, True, 2.0)
    assert list(qq[0]) == [1, 2, 2, 4, 0, 15]


def test_epilogue_bias_relu_order(oracle):
    acc = np.array([[-10, 10]], np.int32)
    _, y, _ = oracle.epilogue(acc, np.zeros(1, np.int32), 0, np.array([0.5], np.float32), 1.0,
                              np.array([6.0], np.float32), True)
    assert list(y[0]) == [1.0, 11.0]  # bias is added before the ReLU
    _, y, _ = oracle.epilogue(acc, np.zeros(1, np.int32), 0, np.array([0.5], np.float32), 1.0,
                              np.array([-6.0], np.float32), True)
    assert list(y[0]) == [0.0, 0.0]


def test_table6_operation_count_pins_the_layer_table():
    """Throughput x latency in Table 6 is the per-image operation count; it must equal
    2 x MACs of the ResNet-18 layer table used for the benchmark shapes."""
    gop = 2 * si.resnet18_macs_per_image() / 1e9
    assert abs(gop - 3.63) < 0.01
    rows = [l.split() for l in open(os.path.join(GOLDEN, "table6_resnet18_fpga.txt")) if l[0] != "#"]
    assert len(rows) == 18
    for name, board, thr, lat in rows:
        per_image = float(thr) * float(lat) / 1e3
        assert abs(per_image - gop) / gop < 0.012, (name, board, per_image)
    # the headline speedups quoted in the abstract / Section 4.3 follow from the same table
    lat = {(r[0], r[1]): float(r[3]) for r in rows}
    assert abs(lat[("fixed_8bit_firstlast", "XC7Z045")] / lat[("rmsmp2_65_30_5", "XC7Z045")] - 3.65) < 0.01
    assert abs(lat[("fixed_8bit_firstlast", "XC7Z020")] / lat[("rmsmp1_60_35_5", "XC7Z020")] - 3.01) < 0.01


def test_input_recipes():
    r = si.rng_for(0)
    W = si.weights_rowscaled(r, 64, 576)
    assert W.dtype == np.float32 and W.shape == (64, 576)
    s = W.std(axis=1)
    assert 0.008 < s.min() and s.max() < 0.12
    x = si.act_codes_u4(r, (256, 576))
    assert x.min() == 0 and x.max() == 15
    sch = si.scheme_permutation(r, (39, 22, 3))
    assert np.bincount(sch, minlength=3).tolist() == [39, 22, 3]
    # same seed, same data
    assert np.array_equal(si.weights_rowscaled(si.rng_for(0), 64, 576), W)
    c, s_, z = si.affine_u4_from_float(si.rng_for(2).standard_normal((100, 64)))
    assert c.min() == 0 and c.max() == 15 and 0 <= z <= 15
    c8, s8 = si.symmetric_i8_from_float(si.rng_for(3).standard_normal((10, 10)))
    assert np.abs(c8).max() == 127
    # GEMM shapes of the layer table
    assert len(si.RESNET18_CONVS) == 20
    shapes = {(m, c * k * k, si.conv_out(h, k, s, p) ** 2) for _, c, m, k, s, p, h in si.RESNET18_CONVS}
    assert (64, 147, 112 * 112) in shapes and (256, 2304, 196) in shapes and (512, 4608, 49) in shapes
