"""GPU parity at the benchmark configurations' full sizes (benchmark configs 2, 3, 4; configs 0
and 1 are in test_gpu_parity.py).  Where the oracle cannot compute every output in seconds the
comparison is on sampled outputs that the oracle computes one by one, in the same launch
configuration the library uses for the full layer."""
import numpy as np
import pytest

import synth_inputs as si

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
DEV = "cuda:0"


@pytest.fixture(scope="module")
def rm():
    import paper_2111_00153_amd as m
    assert torch.cuda.is_available(), "these tests need the GPU"
    return m


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _grouped_to_rows(rm, Yb, perm):
    q = rm.unpack_u4(Yb)
    out = np.empty((q.shape[1], q.shape[0]), np.uint8)
    out[perm] = q.T
    return out


def test_config2_bert_ffn_up_projection(rm, oracle):
    """W 3072x768 (60:35:5), 4096 tokens ~N(0,1) quantized to uint4 with a zero point; every output compared."""
    rng = si.rng_for(2)
    M, K, N = 3072, 768, 4096
    W = si.weights_bert(rng, M, K)
    scheme = si.scheme_permutation(rng, rm.rmsmp_ratio_counts(M, 35, 60, 5))
    xq, s_x, z = si.affine_u4_from_float(rng.standard_normal((N, K)))
    assert 0 < z < 15
    p = rm.rmsmp_pack_weights(W, scheme)
    assert p.counts == (1843, 1075, 154)
    ref = oracle.quantize_rows(W, scheme)
    acc = oracle.gemm_acc(ref["wint"], xq.astype(np.int32))
    rs = oracle.rowsum(ref["wint"])
    acc_c, y, _ = oracle.epilogue(acc, rs, z, ref["rowscale"], s_x)
    inv = np.float32(15.0 / float(np.percentile(np.maximum(y, 0), 99.9)))
    _, _, q = oracle.epilogue(acc, rs, z, ref["rowscale"], s_x, None, True, inv)
    X = _dev(rm.pack_u4(xq))
    Yi = torch.empty((M, N), dtype=torch.int32, device=DEV)
    rm.rmsmp_gemm(p, X, N, rm.make_epilogue(s_x, z, 4, None, False, rm.OUT_INT32), Yi)
    Yf = torch.empty((M, N), dtype=torch.float32, device=DEV)
    rm.rmsmp_gemm(p, X, N, rm.make_epilogue(s_x, z, 4, None, False, rm.OUT_FP32), Yf)
    Yq = torch.empty((N, M // 2), dtype=torch.uint8, device=DEV)
    rm.rmsmp_gemm(p, X, N, rm.make_epilogue(s_x, z, 4, None, True, rm.OUT_U4, inv), Yq)
    torch.cuda.synchronize()
    assert np.array_equal(Yi.cpu().numpy(), acc_c)
    got = Yf.cpu().numpy()
    assert np.all(np.abs(got - y) <= 1e-5 * np.abs(y))
    assert np.array_equal(_grouped_to_rows(rm, Yq.cpu().numpy(), p.perm), q)
    p.free()


@pytest.mark.parametrize("N", [1, 8, 64])
def test_config4_skinny_gemm(rm, oracle, N):
    """W 4096x4096 at Fixed4:PoT4:Fixed8 = 50:40:10, activation batch N in {1, 8, 64}; every output compared."""
    rng = si.rng_for(4)
    M = K = 4096
    W = si.weights_rowscaled(rng, M, K)
    scheme = si.scheme_permutation(rng, rm.rmsmp_ratio_counts(M, 40, 50, 10))
    xq = si.act_codes_u4(rng, (64, K))[:N]
    p = rm.rmsmp_pack_weights(W, scheme)
    assert p.counts == (2048, 1638, 410)
    ref = oracle.quantize_rows(W, scheme, want_levels=False)
    acc = oracle.gemm_acc(ref["wint"], xq.astype(np.int32))
    _, y, _ = oracle.epilogue(acc, oracle.rowsum(ref["wint"]), 0, ref["rowscale"], 0.05)
    X = _dev(rm.pack_u4(xq))
    Yi = torch.empty((M, N), dtype=torch.int32, device=DEV)
    rm.rmsmp_gemm(p, X, N, rm.make_epilogue(0.05, out_kind=rm.OUT_INT32), Yi)
    Yf = torch.empty((M, N), dtype=torch.float32, device=DEV)
    rm.rmsmp_gemm(p, X, N, rm.make_epilogue(0.05, out_kind=rm.OUT_FP32), Yf)
    torch.cuda.synchronize()
    assert np.array_equal(Yi.cpu().numpy(), acc)
    assert np.all(np.abs(Yf.cpu().numpy() - y) <= 1e-5 * np.abs(y))
    p.free()


def _layer_reference(rm, oracle, idx, B, n_samples, structured=False, x=None):
    """Packed weights of layer idx of the ResNet-18 stack and the oracle's accumulators and 4-bit
    codes at sampled outputs.  x: input codes to use instead of the layer's own seeded ones (the
    shortcut projection of a stage reads the input of the stage's first 3x3 layer)."""
    name, C, M, k, s, pad, H = si.RESNET18_CONVS[idx]
    rng = si.rng_for(3, idx)
    K = C * k * k
    Wt = si.weights_rowscaled(rng, M, K)
    first = idx == 0
    if first:  # first layer: Fixed-8 rows, signed 8-bit image
        scheme = np.full(M, 2, np.uint8)
        x, s_x = si.symmetric_i8_from_float(rng.standard_normal((B, H, H, C)))
        bits = 8
    else:
        scheme = si.scheme_permutation(rng, rm.rmsmp_ratio_counts(M, 35, 60, 5))
        s_x, bits = 0.05, 4
        if x is None:
            x = si.act_codes_u4(rng, (B, H, H, C))
    p = rm.rmsmp_pack_weights(Wt, scheme, taps=k * k)
    d = rm.ConvDesc(B, C, H, H, k, k, s, pad)
    od = oracle.conv_desc(B, C, H, H, k, k, s, pad)
    OH, OW = oracle.conv_out_hw(od)
    N = B * OH * OW
    ref = oracle.quantize_rows(Wt, scheme, want_levels=False)
    wint4 = ref["wint"].reshape(M, C, k, k)
    srng = np.random.default_rng(1000 + idx)
    ms = srng.integers(0, M, n_samples)
    ns = srng.integers(0, N, n_samples)
    # make sure image borders, the first / last pixel and every row class are among the samples
    ns[:4] = (0, N - 1, OW - 1, N - OW)
    ms[:M if M < n_samples else n_samples] = np.arange(M)[:n_samples]
    if structured:
        # Whole pixel tiles of the launch geometry the library picks for this layer, every row of each:
        # the first, a middle and the last (ragged) tile, and the tiles around the first and the last
        # image boundary.  The tile width is the largest any kernel here uses (512 pixels); a narrower
        # launch tile divides it, so whole launch tiles are covered whatever the split.
        tile = 512
        n_tiles = (N + tile - 1) // tile
        hw = OH * OW
        want = {0, n_tiles // 2, n_tiles - 1, (hw - 1) // tile, hw // tile, ((B - 1) * hw - 1) // tile, ((B - 1) * hw) // tile}
        cols = np.concatenate([np.arange(t * tile, min(N, (t + 1) * tile)) for t in sorted(t for t in want if 0 <= t < n_tiles)])
        # every row of every weight tile (the padded tail of each class's last tile included)
        mm, nn = np.meshgrid(np.arange(M), cols, indexing="ij")
        ms = np.concatenate([ms, mm.ravel()])
        ns = np.concatenate([ns, nn.ravel()])
        n_samples = ms.size
    acc_s = oracle.conv_acc_at(wint4, x.astype(np.int32), od, ms, ns, 0)
    rs = oracle.rowsum(ref["wint"])
    # the oracle's epilogue works on whole rows: feed it the samples of each row in turn
    y_ref = np.empty(n_samples, np.float32)
    q_ref = np.empty(n_samples, np.uint8)
    for r in np.unique(ms):
        sel = ms == r
        _, yy, _ = oracle.epilogue(acc_s[sel][None, :], rs[r:r + 1], 0, ref["rowscale"][r:r + 1], s_x, None, True)
        y_ref[sel] = yy[0]
    inv = np.float32(15.0 / max(float(np.percentile(y_ref, 99.5)), 1e-6))
    for r in np.unique(ms):
        sel = ms == r
        _, _, qq = oracle.epilogue(acc_s[sel][None, :], rs[r:r + 1], 0, ref["rowscale"][r:r + 1], s_x, None, True, inv)
        q_ref[sel] = qq[0]
    return dict(name=name, p=p, d=d, x=x, s_x=s_x, bits=bits, M=M, N=N, ms=ms, ns=ns, acc_s=acc_s, q_ref=q_ref, inv=inv)


def _check_samples(R, Yi, Yq):
    ms, ns, M, p = R["ms"], R["ns"], R["M"], R["p"]
    got_acc = Yi[torch.from_numpy(ms).to(DEV), torch.from_numpy(ns).to(DEV)].cpu().numpy()
    assert np.array_equal(got_acc, R["acc_s"]), R["name"]
    inv_perm = np.empty(M, np.int64)
    inv_perm[p.perm] = np.arange(M)
    g = inv_perm[ms]
    bytes_ = Yq[torch.from_numpy(ns).to(DEV), torch.from_numpy(g // 2).to(DEV)].cpu().numpy()
    got_q = np.where(g % 2 == 0, bytes_ & 15, bytes_ >> 4).astype(np.uint8)
    assert np.array_equal(got_q, R["q_ref"]), R["name"]


def _resnet_layer(rm, oracle, idx, B, n_samples, structured=False):
    R = _layer_reference(rm, oracle, idx, B, n_samples, structured)
    p, d, x, s_x, bits, M, N, inv = (R[k] for k in ("p", "d", "x", "s_x", "bits", "M", "N", "inv"))
    X = _dev(rm.pack_u4(x) if bits == 4 else x)
    ws_bytes = rm.rmsmp_conv2d_workspace_size(p, d, bits)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=DEV) if ws_bytes else None
    Yi = torch.empty((M, N), dtype=torch.int32, device=DEV)
    rm.rmsmp_conv2d(p, X, d, rm.make_epilogue(s_x, 0, bits, None, False, rm.OUT_INT32), Yi, ws)
    Yq = torch.empty((N, M // 2), dtype=torch.uint8, device=DEV)
    rm.rmsmp_conv2d(p, X, d, rm.make_epilogue(s_x, 0, bits, None, True, rm.OUT_U4, inv), Yq, ws)
    torch.cuda.synchronize()
    _check_samples(R, Yi, Yq)
    p.free()
    del Yi, Yq, X, ws
    torch.cuda.empty_cache()


@pytest.mark.parametrize("head", ["layer2.0", "layer3.0", "layer4.0"])
def test_config3_stage_heads_as_one_launch_batch64_sampled(rm, oracle, head):
    """The launches bench.py makes for the head of stages 2-4 at batch 64: the stride-2 3x3
    convolution and the stride-2 1x1 shortcut projection on the same input through
    rmsmp_conv2d_pair, accumulators and 4-bit codes of both against the oracle on the same
    structured and random samples as the single layers."""
    names = [c[0] for c in si.RESNET18_CONVS]
    ia, ib = names.index(head + ".conv1"), names.index(head + ".downsample")
    A = _layer_reference(rm, oracle, ia, 64, 4000, structured=True)
    Bl = _layer_reference(rm, oracle, ib, 64, 4000, structured=True, x=A["x"])
    X = _dev(rm.pack_u4(A["x"]))
    out = {}
    for kind in (rm.OUT_INT32, rm.OUT_U4):
        Ys = []
        eps = []
        for R in (A, Bl):
            if kind == rm.OUT_INT32:
                Ys.append(torch.empty((R["M"], R["N"]), dtype=torch.int32, device=DEV))
                eps.append(rm.make_epilogue(R["s_x"], 0, 4, None, False, kind))
            else:
                Ys.append(torch.empty((R["N"], R["M"] // 2), dtype=torch.uint8, device=DEV))
                eps.append(rm.make_epilogue(R["s_x"], 0, 4, None, True, kind, R["inv"]))
        rm.rmsmp_conv2d_pair(A["p"], A["d"], eps[0], Ys[0], Bl["p"], Bl["d"], eps[1], Ys[1], X)
        assert rm.rmsmp_debug_last_dispatch()[0] == "lds_resident_pair"
        out[kind] = Ys
    torch.cuda.synchronize()
    _check_samples(A, out[rm.OUT_INT32][0], out[rm.OUT_U4][0])
    _check_samples(Bl, out[rm.OUT_INT32][1], out[rm.OUT_U4][1])
    A["p"].free()
    Bl["p"].free()
    del out, X
    torch.cuda.empty_cache()


@pytest.mark.parametrize("idx", range(len(si.RESNET18_CONVS)))
def test_config3_resnet18_layer_batch64_sampled(rm, oracle, idx):
    """Every convolution of the ResNet-18 stack at batch 64 and 224x224 input geometry against the
    oracle's direct convolution (accumulators and 4-bit codes): 4000 random outputs per layer, plus
    every row of whole pixel tiles -- the first, a middle and the last one and those that straddle
    an image boundary."""
    _resnet_layer(rm, oracle, idx, 64, 4000, structured=True)


@pytest.mark.parametrize("idx", [0, 5, 7, 12, 16])
def test_config3_resnet18_layer_small_batch_sampled_dense(rm, oracle, idx):
    """The layers that do not take the stride-1 kernel (conv1, stride-2 3x3, 1x1 downsample), batch 2,
    densely sampled."""
    _resnet_layer(rm, oracle, idx, 2, 20000)


# ---- the inference GEMMs of the paper's models that the five configurations do not cover

@pytest.mark.parametrize("name,M,K,N,ratio,bits", [
    ("resnet18_fc_fixed8_rows", 1000, 512, 64, (0, 0, 100), 4),
    ("resnet18_fc_w8a8", 1000, 512, 64, (0, 0, 100), 8),
    ("bert_qkv_shape", 768, 768, 4096, (35, 60, 5), 4),
    ("bert_ffn_down_shape", 768, 3072, 1024, (35, 60, 5), 4),
])
def test_remaining_inference_gemms(rm, oracle, name, M, K, N, ratio, bits):
    """Last layer of ResNet-18 (Fixed-8 rows; with 4-bit and with 8-bit activations: Section 4 sets
    first and last layers to 8 bits) and the BERT-base projection shapes; every output compared."""
    rng = si.rng_for(5, len(name))
    W = si.weights_bert(rng, M, K) if name.startswith("bert") else si.weights_rowscaled(rng, M, K)
    scheme = si.scheme_permutation(rng, rm.rmsmp_ratio_counts(M, *ratio))
    if bits == 4:
        xq, s_x, z = si.affine_u4_from_float(rng.standard_normal((N, K)))
        X = _dev(rm.pack_u4(xq))
    else:
        xq, s_x = si.symmetric_i8_from_float(rng.standard_normal((N, K)))
        z = 0
        X = _dev(xq)
    p = rm.rmsmp_pack_weights(W, scheme)
    ref = oracle.quantize_rows(W, scheme, want_levels=False)
    acc = oracle.gemm_acc(ref["wint"], xq.astype(np.int32))
    rs = oracle.rowsum(ref["wint"])
    acc_c, y, _ = oracle.epilogue(acc, rs, z, ref["rowscale"], s_x, None, True)
    inv = np.float32(15.0 / float(np.percentile(y, 99.9)))
    _, _, q = oracle.epilogue(acc, rs, z, ref["rowscale"], s_x, None, True, inv)
    Yi = torch.empty((M, N), dtype=torch.int32, device=DEV)
    rm.rmsmp_gemm(p, X, N, rm.make_epilogue(s_x, z, bits, None, False, rm.OUT_INT32), Yi)
    Yf = torch.empty((M, N), dtype=torch.float32, device=DEV)
    rm.rmsmp_gemm(p, X, N, rm.make_epilogue(s_x, z, bits, None, True, rm.OUT_FP32), Yf)
    Yq = torch.empty((N, M // 2), dtype=torch.uint8, device=DEV)
    rm.rmsmp_gemm(p, X, N, rm.make_epilogue(s_x, z, bits, None, True, rm.OUT_U4, inv), Yq)
    torch.cuda.synchronize()
    assert np.array_equal(Yi.cpu().numpy(), acc_c)
    assert np.all(np.abs(Yf.cpu().numpy() - y) <= 1e-5 * np.abs(y))
    assert np.array_equal(_grouped_to_rows(rm, Yq.cpu().numpy(), p.perm), q)
    p.free()


# ---- GELU epilogue of the feed-forward up-projection (out_kind 3)

@pytest.mark.parametrize("M,K,N,inv_s,z_out,with_bias", [
    (3072, 768, 4096, 2.0, 1, True),      # configs[2]'s shape: the LDS-resident kernel
    (3072, 768, 4096, 6.5, 2, False),     # a finer output scale: codes below the zero point on GELU's negative lobe
    (130, 576, 300, 6.0, 0, True),        # general kernel, ragged tiles
    (96, 1024, 8, 5.0, 1, True),          # skinny kernel
])
def test_gelu_epilogue_matches_oracle(rm, oracle, M, K, N, inv_s, z_out, with_bias):
    """BERT-base FFN up-projection with the GELU + affine 4-bit requantization fused: every 4-bit code
    against the oracle (GELU in float64 from the same fp32 pre-activation)."""
    rng = si.rng_for(2, M + N)
    W = si.weights_bert(rng, M, K)
    scheme = si.scheme_permutation(rng, rm.rmsmp_ratio_counts(M, 35, 60, 5))
    xq, s_x, z = si.affine_u4_from_float(rng.standard_normal((N, K)))
    bias = rng.normal(0.0, 0.4, M).astype(np.float32) if with_bias else None
    p = rm.rmsmp_pack_weights(W, scheme)
    ref = oracle.quantize_rows(W, scheme, want_levels=False)
    acc = oracle.gemm_acc(ref["wint"], xq.astype(np.int32))
    inv = float(np.float32(inv_s))
    _, q = oracle.epilogue_gelu(acc, oracle.rowsum(ref["wint"]), z, ref["rowscale"], s_x, bias, inv, z_out)
    assert len(np.unique(q)) >= 8, np.unique(q)  # the case spans the code range
    X = _dev(rm.pack_u4(xq))
    bias_d = None if bias is None else _dev(bias)
    Yq = torch.full((N, M // 2), 0xEE, dtype=torch.uint8, device=DEV)
    rm.rmsmp_gemm(p, X, N, rm.make_epilogue(s_x, z, 4, bias_d, False, rm.OUT_GELU_U4, inv, z_out), Yq)
    torch.cuda.synchronize()
    assert np.array_equal(_grouped_to_rows(rm, Yq.cpu().numpy(), p.perm), q)
    p.free()


def test_gelu_epilogue_conv_and_argument_errors(rm, oracle):
    """The same epilogue behind rmsmp_conv2d (1x1 and 3x3), and the argument checks of out_kind 3."""
    rng = np.random.default_rng(77)
    for (B, C, H, k, s, pad, M) in ((2, 64, 12, 3, 1, 1, 96), (3, 128, 9, 1, 1, 0, 160)):
        K = C * k * k
        W = si.weights_bert(rng, M, K)
        scheme = si.scheme_permutation(rng, rm.rmsmp_ratio_counts(M, 35, 60, 5))
        x = si.act_codes_u4(rng, (B, H, H, C))
        bias = rng.normal(0.0, 0.3, M).astype(np.float32)
        p = rm.rmsmp_pack_weights(W, scheme, taps=k * k)
        d = rm.ConvDesc(B, C, H, H, k, k, s, pad)
        od = oracle.conv_desc(B, C, H, H, k, k, s, pad)
        ref = oracle.quantize_rows(W, scheme, want_levels=False)
        acc = oracle.conv_acc(ref["wint"].reshape(M, C, k, k), x.astype(np.int32), od, zpad=7)
        _, q = oracle.epilogue_gelu(acc, oracle.rowsum(ref["wint"]), 7, ref["rowscale"], 0.02, bias, 2.5, 1)
        N = acc.shape[1]
        Yq = torch.full((N, M // 2), 0xEE, dtype=torch.uint8, device=DEV)
        rm.rmsmp_conv2d(p, _dev(rm.pack_u4(x)), d, rm.make_epilogue(0.02, 7, 4, _dev(bias), False, rm.OUT_GELU_U4, 2.5, 1), Yq)
        torch.cuda.synchronize()
        assert np.array_equal(_grouped_to_rows(rm, Yq.cpu().numpy(), p.perm), q)
        for bad in (rm.make_epilogue(0.02, 7, 4, None, True, rm.OUT_GELU_U4, 2.5, 1),      # relu with GELU
                    rm.make_epilogue(0.02, 7, 4, None, False, rm.OUT_GELU_U4, 0.0, 1),     # no scale
                    rm.make_epilogue(0.02, 7, 4, None, False, rm.OUT_GELU_U4, 2.5, 16)):   # zero point out of range
            with pytest.raises(rm.RmsmpError) as e:
                rm.rmsmp_conv2d(p, _dev(rm.pack_u4(x)), d, bad, Yq)
            assert e.value.code == 1
        p.free()


def test_variance_assigned_layer_matches_oracle(rm, oracle):
    """A configs[3] layer (layer3.1.conv1's geometry, batch 2) whose PoT-4 / Fixed-4 rows are chosen by
    weight variance (Alg. 1, else-branch) instead of the seeded permutation: the library's assignment equals
    the oracle's, and the layer computed from it matches the oracle in every accumulator and 4-bit code."""
    name, C, M, k, s, pad, H = si.RESNET18_CONVS[13]
    B = 2
    rng = si.rng_for(3, 13)
    W = si.weights_rowscaled(rng, M, C * k * k)
    counts = rm.rmsmp_ratio_counts(M, 35, 60, 5)
    seeded = si.scheme_permutation(rng, counts)
    start = np.where(seeded == si.FIXED8, si.FIXED8, si.FIXED4).astype(np.uint8)
    scheme = rm.rmsmp_assign_by_variance(W, start, counts[1])
    assert np.array_equal(scheme, oracle.assign_by_variance(W, start, counts[1]))
    assert tuple(np.bincount(scheme, minlength=3)) == tuple(counts)
    var = W.astype(np.float64).var(axis=1)
    assert var[scheme == si.POT4].max() <= var[scheme == si.FIXED4].min()
    x = si.act_codes_u4(rng, (B, H, H, C))
    p = rm.rmsmp_pack_weights(W, scheme, taps=k * k)
    d = rm.ConvDesc(B, C, H, H, k, k, s, pad)
    od = oracle.conv_desc(B, C, H, H, k, k, s, pad)
    ref = oracle.quantize_rows(W, scheme, want_levels=False)
    acc = oracle.conv_acc(ref["wint"].reshape(M, C, k, k), x.astype(np.int32), od, 0)
    rs = oracle.rowsum(ref["wint"])
    _, y, _ = oracle.epilogue(acc, rs, 0, ref["rowscale"], 0.05, None, True)
    inv = np.float32(15.0 / float(np.percentile(y, 99.9)))
    _, _, q = oracle.epilogue(acc, rs, 0, ref["rowscale"], 0.05, None, True, inv)
    N = acc.shape[1]
    X = _dev(rm.pack_u4(x))
    Yi = torch.empty((M, N), dtype=torch.int32, device=DEV)
    rm.rmsmp_conv2d(p, X, d, rm.make_epilogue(0.05, 0, 4, None, False, rm.OUT_INT32), Yi)
    Yq = torch.empty((N, M // 2), dtype=torch.uint8, device=DEV)
    rm.rmsmp_conv2d(p, X, d, rm.make_epilogue(0.05, 0, 4, None, True, rm.OUT_U4, inv), Yq)
    torch.cuda.synchronize()
    assert np.array_equal(Yi.cpu().numpy(), acc)
    assert np.array_equal(_grouped_to_rows(rm, Yq.cpu().numpy(), p.perm), q)
    p.free()
