"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element.

Integer accumulators and 4-bit codes must match bit for bit; fp32 outputs within 1e-5 relative
(the tolerance the benchmark spec states; the integer sum is exact, so the only difference allowed is the
rounding of the per-row scale product).
"""
import numpy as np
import pytest

import synth_inputs as si

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def rm():
    import paper_2111_00153_amd as m
    assert torch.cuda.is_available(), "these tests need the GPU"
    return m


DEV = "cuda:0"


def _to_dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def run_gemm(rm, p, xq, act_bits=4, **ep_kw):
    """xq: [N][K] codes (uint8 0..15 or int8).  Returns the output as numpy in the ABI's layout."""
    N = xq.shape[0]
    X = _to_dev(rm.pack_u4(xq) if act_bits == 4 else xq.astype(np.int8))
    kind = ep_kw.get("out_kind", rm.OUT_INT32)
    bias = ep_kw.pop("bias", None)
    bias_d = None if bias is None else _to_dev(bias.astype(np.float32))
    if kind == rm.OUT_U4:
        Y = torch.full((N, p.M // 2), 0xEE, dtype=torch.uint8, device=DEV)
    else:
        Y = torch.full((p.M, N), -12345, dtype=torch.int32 if kind == rm.OUT_INT32 else torch.float32, device=DEV)
    ep = rm.make_epilogue(act_bits=act_bits, bias=bias_d, **ep_kw)
    rm.rmsmp_gemm(p, X, N, ep, Y)
    torch.cuda.synchronize()
    return Y.cpu().numpy()


def oracle_outputs(oracle, W, scheme, xq, z=0, s_x=0.05, bias=None, relu=False, inv_s_out=None, alpha=None):
    ref = oracle.quantize_rows(W, scheme, alpha=alpha)
    acc = oracle.gemm_acc(ref["wint"], xq.astype(np.int32))
    return ref, oracle.epilogue(acc, oracle.rowsum(ref["wint"]), z, ref["rowscale"], s_x, bias, relu, inv_s_out)


def assert_fp32_close(got, ref):
    assert np.all(np.abs(got - ref) <= 1e-5 * np.abs(ref)), float(np.abs(got - ref).max())


def grouped_codes(rm, Yb, perm):
    """[N][M/2] bytes in grouped order -> [M][N] codes in original row order."""
    q = rm.unpack_u4(Yb)  # [N][M] grouped
    out = np.empty((q.shape[1], q.shape[0]), np.uint8)
    out[perm] = q.T
    return out


def test_config0_tiny_mixed_gemm(rm, oracle):
    """W 64x576 at Fixed4:PoT4:Fixed8 = 60:35:5, X 576x256 uint4, scale 0.05."""
    rng = si.rng_for(0)
    M, K, N = 64, 576, 256
    W = si.weights_rowscaled(rng, M, K)
    scheme = si.scheme_permutation(rng, rm.rmsmp_ratio_counts(M, 35, 60, 5))
    xq = si.act_codes_u4(rng, (N, K))
    p = rm.rmsmp_pack_weights(W, scheme)
    assert p.counts == (39, 22, 3)
    ref, (acc, y, _) = oracle_outputs(oracle, W, scheme, xq)
    assert np.array_equal(rm.rmsmp_unpack_codes(p).astype(np.int32), ref["wint"])
    assert np.array_equal(run_gemm(rm, p, xq, act_scale=0.05, out_kind=rm.OUT_INT32), acc)
    assert_fp32_close(run_gemm(rm, p, xq, act_scale=0.05, out_kind=rm.OUT_FP32), y)
    p.free()


def test_one_hot_activations_return_the_weights(rm, oracle):
    """Column n = unit vector e_n: the accumulator is the decoded weight itself, so every code
    value of every scheme is checked through the real decode path."""
    rng = np.random.default_rng(21)
    M, K = 48, 128
    W = si.weights_rowscaled(rng, M, K)
    # make sure every level occurs: rows sweep the whole range
    W[0] = np.linspace(-1, 1, K) * 0.1
    W[1] = np.sign(np.linspace(-1, 1, K)) * 0.1 * 2.0 ** (-rng.integers(0, 9, K))
    W[2] = np.linspace(-1, 1, K) * 0.1
    scheme = np.array([0, 1, 2] * (M // 3), np.uint8)
    p = rm.rmsmp_pack_weights(W, scheme)
    ref = oracle.quantize_rows(W, scheme)
    assert set(np.unique(ref["wint"][0])) == set(range(-7, 8))
    assert set(np.unique(ref["wint"][1])) == {0} | {s * 2 ** e for s in (-1, 1) for e in range(7)}
    xq = np.eye(K, dtype=np.uint8)
    assert np.array_equal(run_gemm(rm, p, xq, out_kind=rm.OUT_INT32), ref["wint"])
    p.free()


@pytest.mark.parametrize("M,K,N", [(64, 576, 256), (37, 130, 77), (16, 64, 1), (130, 1000, 65), (2, 2, 3),
                                   (272, 192, 200), (100, 2304, 129)])
@pytest.mark.parametrize("ratio", [(35, 60, 5), (100, 0, 0), (0, 100, 0), (0, 0, 100), (50, 50, 0)])
def test_gemm_ragged_shapes_and_ratios(rm, oracle, M, K, N, ratio):
    rng = np.random.default_rng(M * 7 + K * 3 + N + ratio[0])
    W = si.weights_rowscaled(rng, M, K)
    scheme = si.scheme_permutation(rng, rm.rmsmp_ratio_counts(M, *ratio))
    xq = si.act_codes_u4(rng, (N, K))
    z = int(rng.integers(0, 16))
    p = rm.rmsmp_pack_weights(W, scheme)
    ref, (acc, y, _) = oracle_outputs(oracle, W, scheme, xq, z=z, s_x=0.03)
    assert np.array_equal(run_gemm(rm, p, xq, act_scale=0.03, act_zero_point=z, out_kind=rm.OUT_INT32), acc)
    assert_fp32_close(run_gemm(rm, p, xq, act_scale=0.03, act_zero_point=z, out_kind=rm.OUT_FP32), y)
    p.free()


@pytest.mark.parametrize("M,K,N", [(64, 576, 256), (38, 130, 77), (256, 256, 100)])
def test_gemm_bias_relu_requant_grouped_output(rm, oracle, M, K, N):
    rng = np.random.default_rng(M + K + N)
    W = si.weights_rowscaled(rng, M, K)
    scheme = si.scheme_permutation(rng, rm.rmsmp_ratio_counts(M, 35, 60, 5))
    xq = si.act_codes_u4(rng, (N, K))
    bias = (rng.standard_normal(M) * 0.5).astype(np.float32)
    p = rm.rmsmp_pack_weights(W, scheme)
    ref, (acc, y, _) = oracle_outputs(oracle, W, scheme, xq, bias=bias, relu=True)
    s_out = float(np.percentile(y, 99.9)) / 15.0
    inv = np.float32(1.0 / s_out)
    _, (_, y, q) = oracle_outputs(oracle, W, scheme, xq, bias=bias, relu=True, inv_s_out=inv)
    got_y = run_gemm(rm, p, xq, act_scale=0.05, bias=bias, relu=True, out_kind=rm.OUT_FP32)
    assert_fp32_close(got_y, y)
    Yb = run_gemm(rm, p, xq, act_scale=0.05, bias=bias, relu=True, out_kind=rm.OUT_U4, out_inv_scale=inv)
    got_q = grouped_codes(rm, Yb, p.perm)
    assert np.array_equal(got_q, q)
    assert q.max() == 15 and q.min() == 0
    p.free()


@pytest.mark.parametrize("M,K,N", [(70, 64, 129), (130, 128, 300), (2000, 256, 5000), (96, 512, 1000), (333, 768, 257), (1030, 768, 4100),
                                   (33, 768, 128)])
def test_gemm_lds_resident_activation_kernel(rm, oracle, M, K, N):
    """Shapes whose K is one of the widths the LDS-resident kernel is built for (including a weight
    matrix tall enough that one work-group runs through several tile pairs, an odd tile count and
    ragged M and N), with a zero point; all three output kinds."""
    rng = np.random.default_rng(M * 11 + K * 5 + N)
    W = si.weights_rowscaled(rng, M, K)
    scheme = si.scheme_permutation(rng, rm.rmsmp_ratio_counts(M, 35, 60, 5))
    xq = si.act_codes_u4(rng, (N, K))
    z = int(rng.integers(1, 15))
    bias = (rng.standard_normal(M) * 0.5).astype(np.float32)
    p = rm.rmsmp_pack_weights(W, scheme)
    ref, (acc, y, _) = oracle_outputs(oracle, W, scheme, xq, z=z, s_x=0.03, bias=bias, relu=True)
    inv = np.float32(15.0 / float(np.percentile(y, 99.9)))
    _, (_, _, q) = oracle_outputs(oracle, W, scheme, xq, z=z, s_x=0.03, bias=bias, relu=True, inv_s_out=inv)
    kw = dict(act_scale=0.03, act_zero_point=z, bias=bias, relu=True)
    assert np.array_equal(run_gemm(rm, p, xq, act_scale=0.03, act_zero_point=z, out_kind=rm.OUT_INT32), acc)
    assert_fp32_close(run_gemm(rm, p, xq, out_kind=rm.OUT_FP32, **kw), y)
    if M % 2 == 0:
        Yb = run_gemm(rm, p, xq, out_kind=rm.OUT_U4, out_inv_scale=inv, **kw)
        assert np.array_equal(grouped_codes(rm, Yb, p.perm), q)
    p.free()


def test_gemm_int8_activations(rm, oracle):
    rng = np.random.default_rng(31)
    for M, K, N in [(64, 147, 300), (32, 256, 64)]:
        W = si.weights_rowscaled(rng, M, K)
        scheme = np.full(M, 2, np.uint8)
        xq = si.act_codes_i8(rng, (N, K))
        p = rm.rmsmp_pack_weights(W, scheme)
        ref, (acc, y, _) = oracle_outputs(oracle, W, scheme, xq, s_x=0.01)
        assert np.array_equal(run_gemm(rm, p, xq, act_bits=8, act_scale=0.01, out_kind=rm.OUT_INT32), acc)
        assert_fp32_close(run_gemm(rm, p, xq, act_bits=8, act_scale=0.01, out_kind=rm.OUT_FP32), y)
        p.free()


def run_conv(rm, oracle, geom, M, ratio, act_bits=4, z=0, relu=False, requant=False, seed=0):
    B, C, H, Wd, KH, KW, stride, pad = geom
    rng = np.random.default_rng(seed + sum(geom) + M)
    K = C * KH * KW
    Wt = si.weights_rowscaled(rng, M, K)
    scheme = si.scheme_permutation(rng, rm.rmsmp_ratio_counts(M, *ratio))
    x = si.act_codes_u4(rng, (B, H, Wd, C)) if act_bits == 4 else si.act_codes_i8(rng, (B, H, Wd, C))
    p = rm.rmsmp_pack_weights(Wt, scheme, taps=KH * KW)
    d = rm.ConvDesc(B, C, H, Wd, KH, KW, stride, pad)
    od = oracle.conv_desc(B, C, H, Wd, KH, KW, stride, pad)
    OH, OW = oracle.conv_out_hw(od)
    N = B * OH * OW
    ref = oracle.quantize_rows(Wt, scheme)
    acc = oracle.conv_acc(ref["wint"].reshape(M, C, KH, KW), x.astype(np.int32), od, zpad=z)
    rs = oracle.rowsum(ref["wint"])
    X = _to_dev(rm.pack_u4(x) if act_bits == 4 else x)
    ws_bytes = rm.rmsmp_conv2d_workspace_size(p, d, act_bits)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=DEV) if ws_bytes else None
    out = {}
    acc_c, y, _ = oracle.epilogue(acc, rs, z, ref["rowscale"], 0.05, None, relu)
    Y = torch.empty((M, N), dtype=torch.int32, device=DEV)
    rm.rmsmp_conv2d(p, X, d, rm.make_epilogue(0.05, z, act_bits, None, relu, rm.OUT_INT32), Y, ws)
    torch.cuda.synchronize()
    assert np.array_equal(Y.cpu().numpy(), acc_c)
    Yf = torch.empty((M, N), dtype=torch.float32, device=DEV)
    rm.rmsmp_conv2d(p, X, d, rm.make_epilogue(0.05, z, act_bits, None, relu, rm.OUT_FP32), Yf, ws)
    torch.cuda.synchronize()
    assert_fp32_close(Yf.cpu().numpy(), y)
    if requant:
        inv = np.float32(15.0 / max(float(np.percentile(y, 99.9)), 1e-6))
        _, _, q = oracle.epilogue(acc, rs, z, ref["rowscale"], 0.05, None, relu, inv)
        Yq = torch.empty((N, M // 2), dtype=torch.uint8, device=DEV)
        rm.rmsmp_conv2d(p, X, d, rm.make_epilogue(0.05, z, act_bits, None, relu, rm.OUT_U4, inv), Yq, ws)
        torch.cuda.synchronize()
        assert np.array_equal(grouped_codes(rm, Yq.cpu().numpy(), p.perm), q)
    p.free()
    return ws_bytes


@pytest.mark.parametrize("geom", [(2, 64, 6, 6, 3, 3, 1, 1), (1, 128, 9, 7, 3, 3, 2, 1), (3, 64, 8, 8, 1, 1, 2, 0),
                                  (2, 256, 5, 5, 3, 3, 1, 1), (2, 96, 5, 5, 3, 3, 1, 1), (1, 16, 9, 9, 5, 5, 2, 2),
                                  (2, 32, 6, 5, 3, 3, 1, 2)])
def test_conv_implicit_im2col(rm, oracle, geom):
    ws = run_conv(rm, oracle, geom, 48, (35, 60, 5), z=0, relu=True, requant=True)
    assert ws == 0
    run_conv(rm, oracle, geom, 34, (35, 60, 5), z=6, seed=1)


@pytest.mark.parametrize("geom", [(5, 64, 14, 14, 3, 3, 1, 1), (2, 128, 10, 9, 3, 3, 1, 0), (3, 64, 7, 7, 1, 1, 1, 0),
                                  (1, 64, 40, 40, 3, 3, 1, 1), (9, 128, 7, 7, 3, 3, 1, 1), (1, 64, 1, 1, 1, 1, 1, 0),
                                  (2, 512, 7, 7, 3, 3, 1, 1)])
@pytest.mark.parametrize("M", [48, 256, 90])
def test_conv_stride1_lds_patch_kernel(rm, oracle, geom, M):
    """Stride-1 layers with C % 64 == 0 take the LDS-resident patch kernel: several pixel tiles,
    tiles that straddle images, a ragged last tile, no padding, 1x1, partial weight tiles."""
    z = (sum(geom) + M) % 16
    assert run_conv(rm, oracle, geom, M, (35, 60, 5), z=z, relu=True, requant=True, seed=3) == 0
    run_conv(rm, oracle, geom, M, (100, 0, 0), z=0, seed=4)


@pytest.mark.parametrize("geom", [(2, 64, 12, 12, 3, 3, 2, 1), (3, 128, 16, 14, 3, 3, 2, 1), (1, 64, 30, 30, 1, 1, 2, 0),
                                  (2, 256, 14, 14, 3, 3, 2, 1), (2, 64, 9, 9, 3, 3, 3, 0), (40, 64, 4, 4, 1, 1, 2, 0)])
@pytest.mark.parametrize("M", [64, 90])
def test_conv_strided_lds_patch_kernel(rm, oracle, geom, M):
    """Strided layers through the LDS-resident kernel (3x3 and 1x1, stride 2 and 3): the patch of a
    pixel tile then spans several input rows and images with gaps the kernel never reads."""
    z = (sum(geom) + M) % 16
    assert run_conv(rm, oracle, geom, M, (35, 60, 5), z=z, relu=True, requant=True, seed=6) == 0


def test_config1_resnet_layer_full_size(rm, oracle):
    """configs[1] at its benchmark size, every output compared: batch 32, 256->256, 14x14, 3x3 s1 p1
    (GEMM 256 x 2304 x 6272), 60:35:5, ReLU + 4-bit requant."""
    c = si.CONFIGS[1]
    rng = si.rng_for(1)
    M, C = c["M"], c["C"]
    K = C * 9
    Wt = si.weights_rowscaled(rng, M, K)
    scheme = si.scheme_permutation(rng, rm.rmsmp_ratio_counts(M, *c["ratio"]))
    x = si.act_codes_u4(rng, (c["B"], c["H"], c["W"], C))
    p = rm.rmsmp_pack_weights(Wt, scheme, taps=9)
    assert p.counts == (153, 90, 13)
    d = rm.ConvDesc(c["B"], C, c["H"], c["W"], 3, 3, 1, 1)
    od = oracle.conv_desc(c["B"], C, c["H"], c["W"], 3, 3, 1, 1)
    N = c["B"] * c["H"] * c["W"]
    ref = oracle.quantize_rows(Wt, scheme)
    acc = oracle.conv_acc(ref["wint"].reshape(M, C, 3, 3), x.astype(np.int32), od, 0)
    rs = oracle.rowsum(ref["wint"])
    _, y, _ = oracle.epilogue(acc, rs, 0, ref["rowscale"], c["s_x"], None, True)
    inv = np.float32(15.0 / float(np.percentile(y, 99.9)))
    _, _, q = oracle.epilogue(acc, rs, 0, ref["rowscale"], c["s_x"], None, True, inv)
    X = _to_dev(rm.pack_u4(x))
    Yi = torch.empty((M, N), dtype=torch.int32, device=DEV)
    rm.rmsmp_conv2d(p, X, d, rm.make_epilogue(c["s_x"], 0, 4, None, False, rm.OUT_INT32), Yi)
    Yq = torch.empty((N, M // 2), dtype=torch.uint8, device=DEV)
    rm.rmsmp_conv2d(p, X, d, rm.make_epilogue(c["s_x"], 0, 4, None, True, rm.OUT_U4, inv), Yq)
    torch.cuda.synchronize()
    assert np.array_equal(Yi.cpu().numpy(), acc)
    assert np.array_equal(grouped_codes(rm, Yq.cpu().numpy(), p.perm), q)
    p.free()


@pytest.mark.parametrize("geom", [(2, 6, 9, 9, 3, 3, 1, 1), (1, 10, 8, 8, 5, 5, 2, 2), (2, 24, 5, 5, 3, 3, 1, 1)])
def test_conv_materialised_im2col_fallback(rm, oracle, geom):
    ws = run_conv(rm, oracle, geom, 40, (35, 60, 5), z=3, relu=True, requant=True)
    assert ws > 0


def test_conv_first_layer_int8_activations(rm, oracle):
    """ResNet conv1 shape (3 -> 64, 7x7, stride 2, pad 3) on a small image, Fixed-8 weights, int8 input."""
    run_conv(rm, oracle, (2, 3, 32, 32, 7, 7, 2, 3), 64, (0, 0, 100), act_bits=8, relu=True, requant=True)


@pytest.mark.parametrize("geom", [(2, 3, 32, 32, 7, 7, 2, 3), (3, 3, 21, 19, 7, 7, 2, 3), (1, 4, 20, 33, 3, 3, 1, 1),
                                  (2, 1, 17, 17, 5, 5, 3, 2), (1, 2, 9, 40, 8, 8, 1, 0), (2, 3, 16, 16, 3, 3, 2, 0)])
@pytest.mark.parametrize("M,ratio", [(64, (0, 0, 100)), (40, (35, 60, 5)), (160, (35, 60, 5))])
def test_conv_small_channel_int8_direct(rm, oracle, geom, M, ratio):
    """8-bit layers with at most four input channels run without an im2col matrix: output tiles that
    are ragged in both directions, strides 1..3, filters 3..8 wide, more than four weight tiles,
    every row class, a zero point."""
    z = (sum(geom) + M) % 7 - 3
    assert run_conv(rm, oracle, geom, M, ratio, act_bits=8, z=z, relu=True, requant=True, seed=5) == 0


@pytest.mark.parametrize("geom", [(2, 4, 9, 9, 3, 3, 1, 1), (1, 2, 8, 7, 3, 3, 2, 1)])
def test_conv_small_channel_u4_through_workspace(rm, oracle, geom):
    """The same storage layout with 4-bit activations goes through the materialised im2col matrix."""
    ws = run_conv(rm, oracle, geom, 40, (35, 60, 5), z=3, relu=True, requant=True)
    assert ws > 0


def test_small_channel_weights_are_conv_only(rm):
    rng = np.random.default_rng(3)
    p = rm.rmsmp_pack_weights(si.weights_rowscaled(rng, 8, 27), np.zeros(8, np.uint8), taps=9)
    X = torch.zeros((4, 27), dtype=torch.int8, device=DEV)
    Y = torch.empty((8, 4), dtype=torch.int32, device=DEV)
    with pytest.raises(rm.RmsmpError) as e:
        rm.rmsmp_gemm(p, X, 4, rm.make_epilogue(act_bits=8), Y)
    assert e.value.code == 5
    p.free()


def test_chained_layers_through_grouped_order(rm, oracle):
    """Layer 1 writes 4-bit output in grouped row order; layer 2 is packed with in_perm = that
    order and must give what the oracle gives on the original channel order."""
    rng = np.random.default_rng(77)
    M1, K1, N, M2 = 64, 128, 70, 32
    W1 = si.weights_rowscaled(rng, M1, K1)
    s1 = si.scheme_permutation(rng, rm.rmsmp_ratio_counts(M1, 35, 60, 5))
    W2 = si.weights_rowscaled(rng, M2, M1)
    s2 = si.scheme_permutation(rng, rm.rmsmp_ratio_counts(M2, 35, 60, 5))
    xq = si.act_codes_u4(rng, (N, K1))
    ref1, (_, y1, _) = oracle_outputs(oracle, W1, s1, xq, relu=True)
    inv = np.float32(15.0 / float(np.percentile(y1, 99.5)))
    _, (_, _, q1) = oracle_outputs(oracle, W1, s1, xq, relu=True, inv_s_out=inv)
    ref2 = oracle.quantize_rows(W2, s2)
    acc2 = oracle.gemm_acc(ref2["wint"], q1.T.astype(np.int32))  # layer-2 columns = layer-1 outputs
    p1 = rm.rmsmp_pack_weights(W1, s1)
    p2 = rm.rmsmp_pack_weights(W2, s2, in_perm=p1.perm)
    X = _to_dev(rm.pack_u4(xq))
    H = torch.empty((N, M1 // 2), dtype=torch.uint8, device=DEV)
    Y = torch.empty((M2, N), dtype=torch.int32, device=DEV)
    rm.rmsmp_gemm(p1, X, N, rm.make_epilogue(0.05, relu=True, out_kind=rm.OUT_U4, out_inv_scale=inv), H)
    rm.rmsmp_gemm(p2, H, N, rm.make_epilogue(1.0 / float(inv), out_kind=rm.OUT_INT32), Y)
    torch.cuda.synchronize()
    assert np.array_equal(Y.cpu().numpy(), acc2)
    p1.free()
    p2.free()


def test_chained_convolutions_through_grouped_order(rm, oracle):
    """Three 3x3 layers and a shortcut projection chained on the GPU: every layer reads the 4-bit
    tensor the layer before it wrote (grouped row order; its weights are packed with in_perm = that
    order), the stride-2 layer and the 1x1 projection go out as one rmsmp_conv2d_pair.  The codes of
    every layer must be the oracle's, which works in the original channel order throughout."""
    rng = np.random.default_rng(4242)
    B, H = 3, 12
    spec = [("a", 64, 64, 3, 1, 1, None), ("b", 64, 128, 3, 2, 1, "a"), ("side", 64, 128, 1, 2, 0, "a"), ("c", 128, 128, 3, 1, 1, "b")]
    x0 = si.act_codes_u4(rng, (B, H, H, 64))
    ref_out, gpu = {}, {}
    for name, C, M, k, s, pad, src in spec:
        Hin = H if src in (None, "a") else H // 2
        OH = (Hin + 2 * pad - k) // s + 1
        W = si.weights_rowscaled(rng, M, C * k * k)
        scheme = si.scheme_permutation(rng, rm.rmsmp_ratio_counts(M, 35, 60, 5))
        x = x0 if src is None else ref_out[src]
        ref = oracle.quantize_rows(W, scheme)
        od = oracle.conv_desc(B, C, Hin, Hin, k, k, s, pad)
        acc = oracle.conv_acc(ref["wint"].reshape(M, C, k, k), x.astype(np.int32), od, 0)
        rs = oracle.rowsum(ref["wint"])
        _, y, _ = oracle.epilogue(acc, rs, 0, ref["rowscale"], 0.05, None, True)
        inv = np.float32(15.0 / max(float(np.percentile(y, 99.0)), 1e-6))
        _, _, q = oracle.epilogue(acc, rs, 0, ref["rowscale"], 0.05, None, True, inv)
        assert len(np.unique(q)) > 8  # the chain stays alive: most codes occur
        ref_out[name] = np.ascontiguousarray(q.T).reshape(B, OH, OH, M).astype(np.uint8)
        p = rm.rmsmp_pack_weights(W, scheme, taps=k * k, in_perm=None if src is None else gpu[src]["p"].perm)
        X = _to_dev(rm.pack_u4(x0)) if src is None else gpu[src]["Y"].view(B, Hin, Hin, C // 2)
        Y = torch.full((B * OH * OH, M // 2), 0xEE, dtype=torch.uint8, device=DEV)
        gpu[name] = dict(p=p, X=X, Y=Y, q=q, d=rm.ConvDesc(B, C, Hin, Hin, k, k, s, pad),
                         ep=rm.make_epilogue(0.05, 0, 4, None, True, rm.OUT_U4, inv))
    g = gpu
    rm.rmsmp_conv2d(g["a"]["p"], g["a"]["X"], g["a"]["d"], g["a"]["ep"], g["a"]["Y"])
    rm.rmsmp_conv2d_pair(g["b"]["p"], g["b"]["d"], g["b"]["ep"], g["b"]["Y"], g["side"]["p"], g["side"]["d"], g["side"]["ep"], g["side"]["Y"], g["b"]["X"])
    rm.rmsmp_conv2d(g["c"]["p"], g["c"]["X"], g["c"]["d"], g["c"]["ep"], g["c"]["Y"])
    torch.cuda.synchronize()
    for name in g:
        got = np.empty_like(g[name]["q"])
        got[g[name]["p"].perm] = rm.unpack_u4(g[name]["Y"].cpu().numpy()).T
        assert np.array_equal(got, g[name]["q"]), name
    for name in g:
        g[name]["p"].free()


def test_empty_and_errors(rm):
    W = np.ones((4, 8), np.float32)
    p = rm.rmsmp_pack_weights(W, np.array([0, 1, 2, 0], np.uint8))
    X = torch.zeros((16,), dtype=torch.uint8, device=DEV)
    Y = torch.zeros((4, 4), dtype=torch.int32, device=DEV)
    rm.rmsmp_gemm(p, X, 0, rm.make_epilogue(), Y)  # N = 0 is a no-op
    with pytest.raises(rm.RmsmpError) as e:
        rm.rmsmp_gemm(p, X, -1, rm.make_epilogue(), Y)
    assert e.value.code == 2
    with pytest.raises(rm.RmsmpError) as e:
        rm.rmsmp_gemm(p, X, 4, rm.make_epilogue(act_bits=5), Y)
    assert e.value.code == 1
    with pytest.raises(rm.RmsmpError) as e:
        rm.rmsmp_gemm(p, X, 4, rm.make_epilogue(act_zero_point=16), Y)
    assert e.value.code == 1
    d = rm.ConvDesc(1, 4, 3, 3, 1, 1, 1, 0)
    with pytest.raises(rm.RmsmpError) as e:  # K = 8 but C*KH*KW = 4
        rm.rmsmp_conv2d(p, X, d, rm.make_epilogue(), Y)
    assert e.value.code == 2
    p.free()
    p3 = rm.rmsmp_pack_weights(np.ones((3, 8), np.float32), np.zeros(3, np.uint8))
    with pytest.raises(rm.RmsmpError) as e:  # odd M cannot be nibble-packed
        rm.rmsmp_gemm(p3, X, 4, rm.make_epilogue(out_kind=rm.OUT_U4), Y)
    assert e.value.code == 2
    p3.free()
    pc = rm.rmsmp_pack_weights(np.ones((4, 6 * 9), np.float32), np.zeros(4, np.uint8), taps=9)
    d = rm.ConvDesc(1, 6, 5, 5, 3, 3, 1, 1)
    assert rm.rmsmp_conv2d_workspace_size(pc, d, 4) > 0
    with pytest.raises(rm.RmsmpError) as e:  # materialised im2col needs a workspace
        rm.rmsmp_conv2d(pc, torch.zeros(75, dtype=torch.uint8, device=DEV), d, rm.make_epilogue(),
                        torch.zeros((4, 25), dtype=torch.int32, device=DEV))
    assert e.value.code == 6
    pc.free()


def test_repeatable(rm, oracle):
    """Integer results are deterministic: two runs give identical bytes."""
    rng = np.random.default_rng(5)
    W = si.weights_rowscaled(rng, 96, 512)
    scheme = si.scheme_permutation(rng, rm.rmsmp_ratio_counts(96, 35, 60, 5))
    xq = si.act_codes_u4(rng, (333, 512))
    p = rm.rmsmp_pack_weights(W, scheme)
    a = run_gemm(rm, p, xq, out_kind=rm.OUT_INT32)
    b = run_gemm(rm, p, xq, out_kind=rm.OUT_INT32)
    assert np.array_equal(a, b)
    p.free()
