"""GPU parity per kernel path: every wave split of the LDS-resident kernel and the first-layer kernel,
each forced or checked through the library's dispatch test hooks, against the CPU oracle.

Integer accumulators and 4-bit codes must match bit for bit; fp32 outputs within 1e-5 relative.
"""
import numpy as np
import pytest

import synth_inputs as si

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

DEV = "cuda:0"
SPLITS = [(4, 4, 1, 1), (4, 2, 2, 1), (4, 1, 4, 1), (4, 1, 1, 4), (2, 2, 2, 1), (2, 4, 1, 1), (2, 1, 1, 4), (2, 1, 4, 1), (4, 2, 1, 2), (2, 2, 1, 2)]


@pytest.fixture(scope="module")
def rm():
    import paper_2111_00153_amd as m
    assert torch.cuda.is_available(), "these tests need the GPU"
    yield m
    m.rmsmp_debug_set_wave_split(0, 0, 0, 0)


def _to_dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _grouped_codes(rm, Yb, perm):
    q = rm.unpack_u4(Yb)
    out = np.empty((q.shape[1], q.shape[0]), np.uint8)
    out[perm] = q.T
    return out


def _check_conv(rm, oracle, geom, M, ratio, act_bits, z, with_bias, relu, seed, expect_kernel=None, expect_split=None):
    """All three output kinds of one layer against the oracle's direct convolution."""
    B, C, H, Wd, KH, KW, stride, pad = geom
    rng = np.random.default_rng(seed + sum(geom) + M)
    K = C * KH * KW
    Wt = si.weights_rowscaled(rng, M, K)
    scheme = si.scheme_permutation(rng, rm.rmsmp_ratio_counts(M, *ratio))
    x = si.act_codes_u4(rng, (B, H, Wd, C)) if act_bits == 4 else si.act_codes_i8(rng, (B, H, Wd, C))
    bias = rng.normal(0.0, 0.3, M).astype(np.float32) if with_bias else None
    bias_d = None if bias is None else _to_dev(bias)
    p = rm.rmsmp_pack_weights(Wt, scheme, taps=KH * KW)
    d = rm.ConvDesc(B, C, H, Wd, KH, KW, stride, pad)
    od = oracle.conv_desc(B, C, H, Wd, KH, KW, stride, pad)
    OH, OW = oracle.conv_out_hw(od)
    N = B * OH * OW
    ref = oracle.quantize_rows(Wt, scheme)
    acc = oracle.conv_acc(ref["wint"].reshape(M, C, KH, KW), x.astype(np.int32), od, zpad=z)
    rs = oracle.rowsum(ref["wint"])
    X = _to_dev(rm.pack_u4(x) if act_bits == 4 else x)
    assert rm.rmsmp_conv2d_workspace_size(p, d, act_bits) == 0
    acc_c, y, _ = oracle.epilogue(acc, rs, z, ref["rowscale"], 0.05, bias, relu)
    Y = torch.full((M, N), -777, dtype=torch.int32, device=DEV)
    rm.rmsmp_conv2d(p, X, d, rm.make_epilogue(0.05, z, act_bits, None, False, rm.OUT_INT32), Y)
    kernel, split = rm.rmsmp_debug_last_dispatch()
    if expect_kernel is not None:
        assert kernel == expect_kernel, (kernel, split)
    if expect_split is not None:
        assert split == expect_split, (kernel, split)
    torch.cuda.synchronize()
    assert np.array_equal(Y.cpu().numpy(), acc_c)
    Yf = torch.full((M, N), np.nan, dtype=torch.float32, device=DEV)
    rm.rmsmp_conv2d(p, X, d, rm.make_epilogue(0.05, z, act_bits, bias_d, relu, rm.OUT_FP32), Yf)
    torch.cuda.synchronize()
    got = Yf.cpu().numpy()
    assert np.all(np.abs(got - y) <= 1e-5 * np.abs(y))
    if M % 2 == 0:
        pos = y[y > 0]
        inv = np.float32(15.0 / max(float(np.percentile(pos, 99.0)) if pos.size else 1.0, 1e-6))
        _, _, q = oracle.epilogue(acc, rs, z, ref["rowscale"], 0.05, bias, relu, inv)
        Yq = torch.full((N, M // 2), 0xEE, dtype=torch.uint8, device=DEV)
        rm.rmsmp_conv2d(p, X, d, rm.make_epilogue(0.05, z, act_bits, bias_d, relu, rm.OUT_U4, inv), Yq)
        torch.cuda.synchronize()
        assert np.array_equal(_grouped_codes(rm, Yq.cpu().numpy(), p.perm), q)
    p.free()


def _fits(split, C, taps):
    """Whether a split exists for this channel count at all (a tap must hold a whole number of K
    steps per wave, and a wave needs at least two K steps)."""
    cpt = C // 32
    ks = split[1]
    return cpt % ks == 0 and taps * (cpt // ks) >= 2


@pytest.mark.parametrize("split", SPLITS)
@pytest.mark.parametrize("geom,M", [((3, 256, 14, 14, 3, 3, 1, 1), 256), ((2, 128, 20, 18, 3, 3, 2, 1), 160),
                                    ((2, 64, 33, 31, 3, 3, 1, 1), 90), ((5, 128, 9, 9, 1, 1, 1, 0), 300),
                                    ((1, 512, 7, 7, 3, 3, 1, 1), 64)])
def test_lds_resident_kernel_every_wave_split(rm, oracle, split, geom, M):
    """Each way of sharing the four waves of a work-group out (K quarters, pixel blocks side by side,
    tile pairs; 64 or 128 pixels per wave) computes the same layer: ragged pixel tiles, images
    that straddle tiles, stride 2, 1x1, a partial last weight tile, odd tile counts."""
    C, taps = geom[1], geom[4] * geom[5]
    rm.rmsmp_debug_set_wave_split(*split)
    try:
        z = (sum(geom) + M + sum(split)) % 16
        pairs = ((M + 31) // 32 + 1) // 2
        # a forced split is used wherever it fits the layer; at stride 1 and up to 128 channels every patch fits the LDS
        forced = C <= 128 and geom[6] == 1 and _fits(split, C, taps) and not (split[3] > 1 and pairs < split[3])
        _check_conv(rm, oracle, geom, M, (35, 60, 5), 4, z, True, True, 11, "lds_resident", split if forced else None)
        _check_conv(rm, oracle, geom, M, (100, 0, 0), 4, 0, False, False, 12, "lds_resident")
    finally:
        rm.rmsmp_debug_set_wave_split(0, 0, 0, 0)


@pytest.mark.parametrize("split", SPLITS)
@pytest.mark.parametrize("M,K,N", [(333, 768, 300), (96, 256, 1000), (130, 128, 129), (100, 576, 300), (70, 1152, 129)])
def test_lds_resident_kernel_gemm_every_wave_split(rm, oracle, split, M, K, N):
    """Plain GEMMs with short K run as 1x1 layers of the LDS-resident kernel, in every wave split;
    K = 576 and 1152 (nine times 64 / 128) run through the 3x3 families as convolutions over N
    images of 3x3 pixels."""
    rng = np.random.default_rng(M + K + N + sum(split))
    W = si.weights_rowscaled(rng, M, K)
    scheme = si.scheme_permutation(rng, rm.rmsmp_ratio_counts(M, 35, 60, 5))
    xq = si.act_codes_u4(rng, (N, K))
    z = 5
    ref = oracle.quantize_rows(W, scheme)
    acc = oracle.gemm_acc(ref["wint"], xq.astype(np.int32))
    acc_c, y, _ = oracle.epilogue(acc, oracle.rowsum(ref["wint"]), z, ref["rowscale"], 0.05, None, False)
    p = rm.rmsmp_pack_weights(W, scheme)
    X = _to_dev(rm.pack_u4(xq))
    rm.rmsmp_debug_set_wave_split(*split)
    try:
        Y = torch.full((M, N), -777, dtype=torch.int32, device=DEV)
        rm.rmsmp_gemm(p, X, N, rm.make_epilogue(0.05, z, 4, None, False, rm.OUT_INT32), Y)
        assert rm.rmsmp_debug_last_dispatch()[0] == "lds_resident"
        Yf = torch.full((M, N), np.nan, dtype=torch.float32, device=DEV)
        rm.rmsmp_gemm(p, X, N, rm.make_epilogue(0.05, z, 4, None, False, rm.OUT_FP32), Yf)
        torch.cuda.synchronize()
        assert np.array_equal(Y.cpu().numpy(), acc_c)
        assert np.all(np.abs(Yf.cpu().numpy() - y) <= 1e-5 * np.abs(y))
    finally:
        rm.rmsmp_debug_set_wave_split(0, 0, 0, 0)
        p.free()


@pytest.mark.parametrize("split", SPLITS)
@pytest.mark.parametrize("M,K,N", [(200, 3072, 300), (96, 1024, 130), (64, 2304, 257), (130, 4096, 70)])
def test_lds_resident_kernel_deep_gemm_every_wave_split(rm, oracle, split, M, K, N):
    """GEMMs deeper than one LDS patch: the channels are staged in equal parts (4 x 768, 2 x 512, 3 x 768,
    8 x 512) with the accumulators kept across the parts, in every wave split; 4-bit output too."""
    rng = np.random.default_rng(M + K + N + sum(split))
    W = si.weights_rowscaled(rng, M, K)
    scheme = si.scheme_permutation(rng, rm.rmsmp_ratio_counts(M, 35, 60, 5))
    xq = si.act_codes_u4(rng, (N, K))
    z = 3
    ref = oracle.quantize_rows(W, scheme)
    acc = oracle.gemm_acc(ref["wint"], xq.astype(np.int32))
    rs = oracle.rowsum(ref["wint"])
    acc_c, y, _ = oracle.epilogue(acc, rs, z, ref["rowscale"], 0.05, None, True)
    p = rm.rmsmp_pack_weights(W, scheme)
    X = _to_dev(rm.pack_u4(xq))
    rm.rmsmp_debug_set_wave_split(*split)
    try:
        Y = torch.full((M, N), -777, dtype=torch.int32, device=DEV)
        rm.rmsmp_gemm(p, X, N, rm.make_epilogue(0.05, z, 4, None, False, rm.OUT_INT32), Y)
        assert rm.rmsmp_debug_last_dispatch()[0] == "lds_resident"
        Yf = torch.full((M, N), np.nan, dtype=torch.float32, device=DEV)
        rm.rmsmp_gemm(p, X, N, rm.make_epilogue(0.05, z, 4, None, True, rm.OUT_FP32), Yf)
        pos = y[y > 0]
        inv = np.float32(15.0 / max(float(np.percentile(pos, 99.0)) if pos.size else 1.0, 1e-6))
        _, _, q = oracle.epilogue(acc, rs, z, ref["rowscale"], 0.05, None, True, inv)
        Yq = torch.full((N, M // 2), 0xEE, dtype=torch.uint8, device=DEV)
        rm.rmsmp_gemm(p, X, N, rm.make_epilogue(0.05, z, 4, None, True, rm.OUT_U4, inv), Yq)
        torch.cuda.synchronize()
        assert np.array_equal(Y.cpu().numpy(), acc_c)
        assert np.all(np.abs(Yf.cpu().numpy() - y) <= 1e-5 * np.abs(y))
        assert np.array_equal(_grouped_codes(rm, Yq.cpu().numpy(), p.perm), q)
    finally:
        rm.rmsmp_debug_set_wave_split(0, 0, 0, 0)
        p.free()


def test_lds_resident_kernel_deep_1x1_layer(rm, oracle):
    """A 1x1 layer of stride 1 with 1024 input channels (a ResNet-50 bottleneck's shape): two parts of 512."""
    _check_conv(rm, oracle, (2, 1024, 7, 9, 1, 1, 1, 0), 96, (35, 60, 5), 4, 5, True, True, 41, "lds_resident")


@pytest.mark.parametrize("geom", [(2, 3, 32, 32, 7, 7, 2, 3), (1, 3, 70, 44, 7, 7, 2, 3), (3, 3, 36, 40, 3, 3, 2, 1),
                                  (2, 3, 35, 36, 5, 5, 2, 1), (1, 3, 18, 8, 5, 5, 2, 3), (5, 3, 16, 16, 7, 7, 2, 3)])
@pytest.mark.parametrize("M,ratio", [(64, (0, 0, 100)), (40, (35, 60, 5)), (160, (35, 60, 5))])
def test_first_layer_kernel(rm, oracle, geom, M, ratio):
    """Three input channels, 8-bit activations, stride 2: the kernel that walks through 16x16 pixel
    tiles with the weights in registers.  Output sizes that are not multiples of the tile, several
    images and tiles per work-group, one to five weight tiles (three passes), every row class,
    3x3 / 5x5 / 7x7 filters with padding 1 and 3, zero points, bias, ReLU, all output kinds."""
    z = (sum(geom) + M) % 7 - 3
    _check_conv(rm, oracle, geom, M, ratio, 8, z, True, True, 21, "first_layer")
    _check_conv(rm, oracle, geom, M, ratio, 8, 0, False, True, 22, "first_layer")
    _check_conv(rm, oracle, geom, M, ratio, 8, 0, False, False, 23, "first_layer")


@pytest.mark.parametrize("B,k,pad", [(40, 7, 3), (17, 3, 1)])
def test_first_layer_kernel_several_tiles_per_work_group(rm, oracle, B, k, pad):
    """More 16x16 pixel tiles than work-groups (the launch has at most 768): work-groups walk through
    two or three tiles with double-buffered staging, and the tile counts differ by one between them."""
    geom = (B, 3, 224, 224, k, k, 2, pad)
    _check_conv(rm, oracle, geom, 64, (0, 0, 100), 8, 0, False, True, 31, "first_layer")
    _check_conv(rm, oracle, geom, 40, (35, 60, 5), 8, 2, True, True, 32, "first_layer")


def test_gemm_with_k_of_a_lowered_3x3_layer_four_bit_output(rm, oracle):
    """K = 576 = 9 x 64 through the 3x3 family, 4-bit output with bias and ReLU and without (the lean
    epilogue), ragged N."""
    rng = np.random.default_rng(576)
    M, K, N = 96, 576, 333
    W = si.weights_rowscaled(rng, M, K)
    scheme = si.scheme_permutation(rng, rm.rmsmp_ratio_counts(M, 35, 60, 5))
    xq = si.act_codes_u4(rng, (N, K))
    ref = oracle.quantize_rows(W, scheme)
    acc = oracle.gemm_acc(ref["wint"], xq.astype(np.int32))
    p = rm.rmsmp_pack_weights(W, scheme)
    X = _to_dev(rm.pack_u4(xq))
    for z, with_bias in ((0, False), (4, True)):
        bias = rng.normal(0.0, 0.3, M).astype(np.float32) if with_bias else None
        _, y, _ = oracle.epilogue(acc, oracle.rowsum(ref["wint"]), z, ref["rowscale"], 0.05, bias, True)
        inv = np.float32(15.0 / float(np.percentile(y, 99.0)))
        _, _, q = oracle.epilogue(acc, oracle.rowsum(ref["wint"]), z, ref["rowscale"], 0.05, bias, True, inv)
        Yq = torch.full((N, M // 2), 0xEE, dtype=torch.uint8, device=DEV)
        rm.rmsmp_gemm(p, X, N, rm.make_epilogue(0.05, z, 4, None if bias is None else _to_dev(bias), True, rm.OUT_U4, inv), Yq)
        assert rm.rmsmp_debug_last_dispatch()[0] == "lds_resident"
        torch.cuda.synchronize()
        assert np.array_equal(_grouped_codes(rm, Yq.cpu().numpy(), p.perm), q)
    p.free()


def test_dispatch_record_names_the_kernel(rm, oracle):
    """The dispatch hook reports the kernel family of the last launch on this thread."""
    rng = np.random.default_rng(5)
    for (M, K, N, want) in [(64, 4096, 8, "skinny"), (64, 512, 256, "lds_resident"), (64, 576, 256, "lds_resident"),
                            (37, 130, 77, "general")]:
        W = si.weights_rowscaled(rng, M, K)
        scheme = si.scheme_permutation(rng, rm.rmsmp_ratio_counts(M, 35, 60, 5))
        xq = si.act_codes_u4(rng, (N, K))
        p = rm.rmsmp_pack_weights(W, scheme)
        Y = torch.empty((M, N), dtype=torch.int32, device=DEV)
        rm.rmsmp_gemm(p, _to_dev(rm.pack_u4(xq)), N, rm.make_epilogue(0.05, 0, 4, None, False, rm.OUT_INT32), Y)
        assert rm.rmsmp_debug_last_dispatch()[0] == want
        torch.cuda.synchronize()
        ref = oracle.quantize_rows(W, scheme)
        assert np.array_equal(Y.cpu().numpy(), oracle.gemm_acc(ref["wint"], xq.astype(np.int32)))
        p.free()


@pytest.mark.parametrize("ratio", [(35, 60, 5), (100, 0, 0)])
def test_pot_rows_stored_as_int8_give_the_same_results(rm, oracle, ratio):
    """RMSMP_PACK_POT_AS_INT8: PoT-4 rows stored decoded.  Codes, scales, row sums, accumulators and
    4-bit outputs are those of the oracle (and so of the 4-bit storage) through the LDS-resident, the
    skinny and the general kernel."""
    rng = np.random.default_rng(800 + ratio[0])
    # a 3x3 layer (LDS-resident kernel)
    B, C, H, M = 3, 128, 12, 160
    K = C * 9
    Wt = si.weights_rowscaled(rng, M, K)
    scheme = si.scheme_permutation(rng, rm.rmsmp_ratio_counts(M, *ratio))
    x = si.act_codes_u4(rng, (B, H, H, C))
    ref = oracle.quantize_rows(Wt, scheme)
    p = rm.rmsmp_pack_weights(Wt, scheme, taps=9, flags=rm.PACK_POT_AS_INT8)
    p4 = rm.rmsmp_pack_weights(Wt, scheme, taps=9)
    assert p.counts == p4.counts  # the schemes are what they were; only the storage differs
    assert np.array_equal(rm.rmsmp_unpack_codes(p).astype(np.int32), ref["wint"])
    assert np.array_equal(p.rowscale, ref["rowscale"]) and np.array_equal(p.rowsum, oracle.rowsum(ref["wint"]))
    od = oracle.conv_desc(B, C, H, H, 3, 3, 1, 1)
    acc = oracle.conv_acc(ref["wint"].reshape(M, C, 3, 3), x.astype(np.int32), od, zpad=2)
    rs = oracle.rowsum(ref["wint"])
    acc_c, y, _ = oracle.epilogue(acc, rs, 2, ref["rowscale"], 0.05, None, True)
    inv = np.float32(15.0 / float(np.percentile(y, 99.0)))
    _, _, q = oracle.epilogue(acc, rs, 2, ref["rowscale"], 0.05, None, True, inv)
    X = _to_dev(rm.pack_u4(x))
    d = rm.ConvDesc(B, C, H, H, 3, 3, 1, 1)
    N = B * H * H
    Y = torch.full((M, N), -777, dtype=torch.int32, device=DEV)
    rm.rmsmp_conv2d(p, X, d, rm.make_epilogue(0.05, 2, 4, None, False, rm.OUT_INT32), Y)
    assert rm.rmsmp_debug_last_dispatch()[0] == "lds_resident"
    Yq = torch.full((N, M // 2), 0xEE, dtype=torch.uint8, device=DEV)
    rm.rmsmp_conv2d(p, X, d, rm.make_epilogue(0.05, 2, 4, None, True, rm.OUT_U4, inv), Yq)
    torch.cuda.synchronize()
    assert np.array_equal(Y.cpu().numpy(), acc_c)
    assert np.array_equal(_grouped_codes(rm, Yq.cpu().numpy(), p.perm), q)
    p.free()
    p4.free()
    # plain GEMMs: skinny (N = 8) and general (K = 130 fits no other kernel)
    for (M, K, N, want) in [(96, 1024, 8, "skinny"), (70, 130, 77, "general")]:
        Wt = si.weights_rowscaled(rng, M, K)
        scheme = si.scheme_permutation(rng, rm.rmsmp_ratio_counts(M, *ratio))
        xq = si.act_codes_u4(rng, (N, K))
        ref = oracle.quantize_rows(Wt, scheme)
        p = rm.rmsmp_pack_weights(Wt, scheme, flags=rm.PACK_POT_AS_INT8)
        Y = torch.full((M, N), -777, dtype=torch.int32, device=DEV)
        rm.rmsmp_gemm(p, _to_dev(rm.pack_u4(xq)), N, rm.make_epilogue(0.05, 0, 4, None, False, rm.OUT_INT32), Y)
        assert rm.rmsmp_debug_last_dispatch()[0] == want
        torch.cuda.synchronize()
        assert np.array_equal(Y.cpu().numpy(), oracle.gemm_acc(ref["wint"], xq.astype(np.int32)))
        p.free()
    with pytest.raises(rm.RmsmpError):
        rm.rmsmp_pack_weights(Wt, scheme, flags=6)
