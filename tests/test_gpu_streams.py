"""GPU: the hot path under the two launch patterns a serving loop uses -- launches of two streams
overlapping on the chip, and a captured graph replayed several times -- against the CPU oracle.

The library keeps no per-call device state (no scratch buffer, no counters) on these paths, so
overlapping launches must not disturb each other, and a replay must give what the eager call gives.
4-bit codes are compared bit for bit.
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


def _layer(rm, oracle, seed, B, C, H, M, k, stride, pad, act_bits=4):
    """One convolution with 4-bit output: packed weights, input codes, the oracle's codes in grouped order."""
    rng = np.random.default_rng(seed)
    K = C * k * k
    W = si.weights_rowscaled(rng, M, K)
    if act_bits == 8:
        scheme = np.full(M, 2, np.uint8)
        x = si.act_codes_i8(rng, (B, H, H, C))
    else:
        scheme = si.scheme_permutation(rng, rm.rmsmp_ratio_counts(M, 35, 60, 5))
        x = si.act_codes_u4(rng, (B, H, H, C))
    p = rm.rmsmp_pack_weights(W, scheme, taps=k * k)
    od = oracle.conv_desc(B, C, H, H, k, k, stride, pad)
    OH, OW = oracle.conv_out_hw(od)
    ref = oracle.quantize_rows(W, scheme)
    acc = oracle.conv_acc(ref["wint"].reshape(M, C, k, k), x.astype(np.int32), od, zpad=0)
    rs = oracle.rowsum(ref["wint"])
    _, y, _ = oracle.epilogue(acc, rs, 0, ref["rowscale"], 0.05, None, True)
    inv = np.float32(15.0 / max(float(np.percentile(y, 99.0)), 1e-6))
    _, _, q = oracle.epilogue(acc, rs, 0, ref["rowscale"], 0.05, None, True, inv)
    grouped = np.ascontiguousarray(q[p.perm].T)  # [N][M] in the packed blob's row order
    X = torch.from_numpy(np.ascontiguousarray(rm.pack_u4(x) if act_bits == 4 else x)).to(DEV)
    ep = rm.make_epilogue(0.05, 0, act_bits, None, True, rm.OUT_U4, inv)
    return dict(p=p, X=X, ep=ep, B=B, C=C, H=H, M=M, k=k, stride=stride, pad=pad, OH=OH, N=B * OH * OW,
                bits=act_bits, expect=grouped)


def _codes(rm, Y):
    return rm.unpack_u4(Y.cpu().numpy())


def test_two_streams_halves_of_the_batch_overlap(rm, oracle):
    """Two halves of the batch on two streams, many launches in flight at once (LDS-resident 3x3 and
    1x1 kernels and the first-layer kernel): every output equals the oracle's."""
    layers = [_layer(rm, oracle, 11, 8, 64, 28, 64, 3, 1, 1), _layer(rm, oracle, 12, 8, 128, 14, 128, 1, 2, 0),
              _layer(rm, oracle, 13, 8, 256, 14, 128, 3, 1, 1), _layer(rm, oracle, 14, 4, 3, 32, 64, 7, 2, 3, act_bits=8)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    launch = []
    for L in layers:
        half = L["B"] // 2
        n = L["N"] // 2
        L["Y"] = torch.full((L["N"], L["M"] // 2), 0xEE, dtype=torch.uint8, device=DEV)
        d = rm.ConvDesc(half, L["C"], L["H"], L["H"], L["k"], L["k"], L["stride"], L["pad"])
        assert rm.rmsmp_conv2d_workspace_size(L["p"], d, L["bits"]) == 0
        launch.append([rm.conv2d_launcher(L["p"], L["X"][i * half:(i + 1) * half], d, L["ep"], L["Y"][i * n:(i + 1) * n],
                                          None, stream=streams[i]) for i in range(2)])
    torch.cuda.synchronize()
    for rep in range(25):
        for pair in launch:
            pair[0]()
            pair[1]()
    torch.cuda.synchronize()
    for L in layers:
        assert np.array_equal(_codes(rm, L["Y"]), L["expect"]), (L["C"], L["k"])
        L["p"].free()


def test_captured_graph_replays_equal_the_eager_result(rm, oracle):
    """A chain of rmsmp_conv2d calls captured once (after one eager run, which also does the
    one-time per-kernel set-up) and replayed four times with eager work and synchronisations in
    between: every replay gives the oracle's codes."""
    layers = [_layer(rm, oracle, 21, 4, 64, 28, 64, 3, 1, 1), _layer(rm, oracle, 22, 4, 128, 14, 256, 3, 2, 1),
              _layer(rm, oracle, 23, 4, 128, 14, 128, 1, 2, 0)]
    for L in layers:
        L["Y"] = torch.zeros((L["N"], L["M"] // 2), dtype=torch.uint8, device=DEV)
        L["d"] = rm.ConvDesc(L["B"], L["C"], L["H"], L["H"], L["k"], L["k"], L["stride"], L["pad"])

    def run():
        for L in layers:
            rm.rmsmp_conv2d(L["p"], L["X"], L["d"], L["ep"], L["Y"])

    run()
    torch.cuda.synchronize()
    for L in layers:
        assert np.array_equal(_codes(rm, L["Y"]), L["expect"])
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        graph.capture_begin()
        run()
        graph.capture_end()
    torch.cuda.synchronize()
    scratch = torch.empty(1 << 20, dtype=torch.float32, device=DEV)
    for rep in range(4):
        for L in layers:
            L["Y"].fill_(0xEE)  # a fill kernel, not a memset node; eager work between the replays
        scratch.normal_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for L in layers:
            assert np.array_equal(_codes(rm, L["Y"]), L["expect"]), rep
    for L in layers:
        L["p"].free()
