"""GPU parity of rmsmp_conv2d_pair (two convolutions on one input, one launch where the library can)
against the CPU oracle: every output kind of both layers, the fused path and the fall-back path.

Integer accumulators and 4-bit codes must match bit for bit; fp32 outputs within 1e-5 relative.
"""
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


@pytest.fixture(scope="module")
def oracle():
    import oracle as o
    return o


def _to_dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


class _Layer:
    """One convolution of a pair: packed weights, descriptor, and the oracle's three outputs."""

    def __init__(self, rm, oracle, rng, x, z, B, C, H, W, M, k, stride, pad, with_bias, relu):
        K = C * k * k
        Wt = si.weights_rowscaled(rng, M, K)
        scheme = si.scheme_permutation(rng, rm.rmsmp_ratio_counts(M, 35, 60, 5))
        self.M = M
        self.p = rm.rmsmp_pack_weights(Wt, scheme, taps=k * k)
        self.d = rm.ConvDesc(B, C, H, W, k, k, stride, pad)
        od = oracle.conv_desc(B, C, H, W, k, k, stride, pad)
        OH, OW = oracle.conv_out_hw(od)
        self.N = B * OH * OW
        ref = oracle.quantize_rows(Wt, scheme)
        acc = oracle.conv_acc(ref["wint"].reshape(M, C, k, k), x.astype(np.int32), od, zpad=z)
        rs = oracle.rowsum(ref["wint"])
        self.bias = rng.normal(0.0, 0.3, M).astype(np.float32) if with_bias else None
        self.bias_d = None if self.bias is None else _to_dev(self.bias)
        self.relu = relu
        self.acc, self.y, _ = oracle.epilogue(acc, rs, z, ref["rowscale"], 0.05, self.bias, relu)
        pos = self.y[self.y > 0]
        self.inv = np.float32(15.0 / max(float(np.percentile(pos, 99.0)) if pos.size else 1.0, 1e-6))
        _, _, q = oracle.epilogue(acc, rs, z, ref["rowscale"], 0.05, self.bias, relu, self.inv)
        self.q = np.ascontiguousarray(q[self.p.perm].T)  # [N][M], the packed blob's row order

    def epilogue(self, rm, z, kind):
        if kind == rm.OUT_INT32:
            return rm.make_epilogue(0.05, z, 4, None, False, kind)
        return rm.make_epilogue(0.05, z, 4, self.bias_d, self.relu, kind, self.inv)

    def output(self, rm, kind):
        if kind == rm.OUT_INT32:
            return torch.full((self.M, self.N), -777, dtype=torch.int32, device=DEV)
        if kind == rm.OUT_FP32:
            return torch.full((self.M, self.N), np.nan, dtype=torch.float32, device=DEV)
        return torch.full((self.N, self.M // 2), 0xEE, dtype=torch.uint8, device=DEV)

    def check(self, rm, kind, Y):
        got = Y.cpu().numpy()
        if kind == rm.OUT_INT32:
            assert np.array_equal(got, self.acc)
        elif kind == rm.OUT_FP32:
            assert np.all(np.abs(got - self.y) <= 1e-5 * np.abs(self.y))
        else:
            assert np.array_equal(rm.unpack_u4(got), self.q)


def _pair(rm, oracle, seed, B, C, H, W, MA, MB, stride, z, bias_a=False, bias_b=True, kb=1):
    rng = np.random.default_rng(seed)
    x = si.act_codes_u4(rng, (B, H, W, C))
    A = _Layer(rm, oracle, rng, x, z, B, C, H, W, MA, 3, stride, 1, bias_a, True)
    Bl = _Layer(rm, oracle, rng, x, z, B, C, H, W, MB, kb, stride, kb // 2, bias_b, False)
    return _to_dev(rm.pack_u4(x)), A, Bl


def _run_all_kinds(rm, X, A, Bl, z, expect_kernel):
    for ka, kb in ((rm.OUT_U4, rm.OUT_U4), (rm.OUT_INT32, rm.OUT_FP32), (rm.OUT_FP32, rm.OUT_INT32), (rm.OUT_U4, rm.OUT_FP32)):
        Ya, Yb = A.output(rm, ka), Bl.output(rm, kb)
        rm.rmsmp_conv2d_pair(A.p, A.d, A.epilogue(rm, z, ka), Ya, Bl.p, Bl.d, Bl.epilogue(rm, z, kb), Yb, X)
        kernel, _ = rm.rmsmp_debug_last_dispatch()
        torch.cuda.synchronize()
        if expect_kernel is not None:
            assert kernel == expect_kernel, kernel
        A.check(rm, ka, Ya)
        Bl.check(rm, kb, Yb)


@pytest.mark.parametrize("C,MA,MB,H,W", [(64, 100, 128, 20, 18), (128, 250, 256, 14, 14), (256, 130, 96, 10, 12)])
@pytest.mark.parametrize("stride", [2, 1])
def test_pair_runs_as_one_launch_and_matches_oracle(rm, oracle, C, MA, MB, H, W, stride):
    """The three channel counts the two-layer launch exists for: ragged row counts (padding rows in the
    last weight tiles), image sizes that leave ragged pixel tiles, zero point 3, with and without bias."""
    z = 3
    X, A, Bl = _pair(rm, oracle, 1000 + C + stride, 3, C, H, W, MA, MB, stride, z)
    _run_all_kinds(rm, X, A, Bl, z, "lds_resident_pair")
    A.p.free()
    Bl.p.free()


def test_pair_of_resnet_stage_head_shapes(rm, oracle):
    """layer3.0 of ResNet-18 at a small batch (128 -> 256 channels, 28x28 -> 14x14), zero point 0,
    no bias, ReLU on the 3x3 layer only: the configuration bench.py launches."""
    X, A, Bl = _pair(rm, oracle, 77, 2, 128, 28, 28, 256, 256, 2, 0, bias_a=False, bias_b=False)
    _run_all_kinds(rm, X, A, Bl, 0, "lds_resident_pair")
    A.p.free()
    Bl.p.free()


def test_pair_falls_back_to_two_launches(rm, oracle):
    """Shapes the two-layer launch does not exist for are launched one after the other, with the
    same results: 96 channels (general kernel), and two 3x3 layers."""
    X, A, Bl = _pair(rm, oracle, 5, 2, 96, 12, 12, 64, 64, 2, 1)
    _run_all_kinds(rm, X, A, Bl, 1, None)
    kernel, _ = rm.rmsmp_debug_last_dispatch()
    assert kernel != "lds_resident_pair"
    A.p.free()
    Bl.p.free()
    X, A, Bl = _pair(rm, oracle, 6, 2, 64, 12, 12, 128, 128, 1, 0, kb=3)
    _run_all_kinds(rm, X, A, Bl, 0, "lds_resident")
    A.p.free()
    Bl.p.free()


def test_pair_argument_errors(rm, oracle):
    rng = np.random.default_rng(9)
    x = si.act_codes_u4(rng, (2, 10, 10, 64))
    X = _to_dev(rm.pack_u4(x))
    A = _Layer(rm, oracle, rng, x, 0, 2, 64, 10, 10, 128, 3, 2, 1, False, True)
    Bl = _Layer(rm, oracle, rng, x, 0, 2, 64, 10, 10, 128, 1, 2, 0, False, False)
    Ya, Yb = A.output(rm, rm.OUT_U4), Bl.output(rm, rm.OUT_U4)
    epa, epb = A.epilogue(rm, 0, rm.OUT_U4), Bl.epilogue(rm, 0, rm.OUT_U4)
    with pytest.raises(rm.RmsmpError):  # different input tensors
        rm.rmsmp_conv2d_pair(A.p, A.d, epa, Ya, Bl.p, rm.ConvDesc(2, 64, 12, 10, 1, 1, 2, 0), epb, Yb, X)
    with pytest.raises(rm.RmsmpError):  # one output buffer for both
        rm.rmsmp_conv2d_pair(A.p, A.d, epa, Ya, Bl.p, Bl.d, epb, Ya, X)
    with pytest.raises(rm.RmsmpError):  # the layers disagree on the input's zero point
        rm.rmsmp_conv2d_pair(A.p, A.d, epa, Ya, Bl.p, Bl.d, Bl.epilogue(rm, 2, rm.OUT_U4), Yb, X)
    with pytest.raises(rm.RmsmpError):  # weights of another shape
        rm.rmsmp_conv2d_pair(A.p, A.d, epa, Ya, A.p, Bl.d, epb, Yb, X)
    # a layer that needs an im2col workspace (24 channels) is refused
    x2 = si.act_codes_u4(rng, (1, 8, 8, 24))
    C2 = _Layer(rm, oracle, rng, x2, 0, 1, 24, 8, 8, 64, 3, 1, 1, False, True)
    D2 = _Layer(rm, oracle, rng, x2, 0, 1, 24, 8, 8, 64, 1, 1, 0, False, False)
    assert rm.rmsmp_conv2d_workspace_size(C2.p, C2.d, 4) > 0
    with pytest.raises(rm.RmsmpError):
        rm.rmsmp_conv2d_pair(C2.p, C2.d, C2.epilogue(rm, 0, rm.OUT_U4), C2.output(rm, rm.OUT_U4), D2.p, D2.d,
                             D2.epilogue(rm, 0, rm.OUT_U4), D2.output(rm, rm.OUT_U4), _to_dev(rm.pack_u4(x2)))
    for L in (A, Bl, C2, D2):
        L.p.free()
