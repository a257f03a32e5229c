"""Pins of the oracle's GELU epilogue (the feed-forward activation of the BERT-base workload,
Section 4.1 / Table 5) against what the mathematics fixes, without calling erf again:
the symmetry x*Phi(x) - (-x)*Phi(-x) = x, tabulated values of the normal distribution function,
a numerical integral of the Gaussian density, the location and depth of the minimum, the two
monotone branches, the asymptotes, and the affine 4-bit code on hand-checked values."""
import numpy as np

# Phi(x) from standard normal tables (Abramowitz & Stegun, Table 26.1, to 15 places)
PHI = {0.5: 0.691462461274013, 1.0: 0.841344746068543, 1.5: 0.933192798731142, 2.0: 0.977249868051821,
       3.0: 0.998650101968370}


def _gelu(oracle, y):
    return oracle.gelu_codes(np.asarray(y, np.float32), 1.0, 0)[0]


def test_tabulated_values_and_zero(oracle):
    assert _gelu(oracle, [0.0])[0] == 0.0
    for x, phi in PHI.items():
        g = _gelu(oracle, [x, -x])
        assert abs(float(g[0]) - x * phi) <= 1e-7 * x
        assert abs(float(g[1]) + x * (1.0 - phi)) <= 1e-7 * x


def test_symmetry_identity(oracle):
    """GELU(x) - GELU(-x) = x * (Phi(x) + Phi(-x)) = x."""
    x = np.linspace(0.0, 8.0, 4001, dtype=np.float32)
    g = _gelu(oracle, np.concatenate([x, -x]))
    assert np.all(np.abs((g[:x.size].astype(np.float64) - g[x.size:]) - x) <= 2e-7 * np.maximum(x, 1.0))


def test_against_an_integral_of_the_gaussian_density(oracle):
    """Phi(x) = 1/2 + int_0^x phi(t) dt by composite Simpson in float64 (independent of erf)."""
    rng = np.random.default_rng(3)
    xs = rng.uniform(-5.0, 5.0, 200).astype(np.float32)
    g = _gelu(oracle, xs)
    for x, gx in zip(xs.astype(np.float64), g):
        t = np.linspace(0.0, x, 4001)
        f = np.exp(-0.5 * t * t) / np.sqrt(2.0 * np.pi)
        h = t[1] - t[0]
        integral = h / 3.0 * (f[0] + f[-1] + 4.0 * f[1:-1:2].sum() + 2.0 * f[2:-1:2].sum())
        assert abs(gx - x * (0.5 + integral)) <= 3e-7 * max(abs(x), 1.0)


def test_minimum_branches_and_asymptotes(oracle):
    y = np.linspace(-8.0, 8.0, 160001, dtype=np.float32)
    g = _gelu(oracle, y)
    i = int(np.argmin(g))
    # d/dy [y Phi(y)] = Phi(y) + y phi(y) = 0 at y = -0.75179..., where GELU = -0.16997...
    assert abs(float(y[i]) + 0.75179) < 2e-4 and abs(float(g[i]) + 0.169971) < 1e-6
    assert np.all(np.diff(g[:i + 1]) <= 0) and np.all(np.diff(g[i:]) >= 0)
    assert np.all(g <= np.maximum(y, 0)) and np.all(g >= -0.17)
    big = np.array([6.0, 8.0, 20.0, 1e6], np.float32)
    assert np.array_equal(_gelu(oracle, big), big)          # 1 - Phi(6) < 2^-25: rounds to y
    small = _gelu(oracle, -big)
    assert np.all(small <= 0) and np.all(np.abs(small) < 1e-8)


def test_affine_four_bit_codes(oracle):
    # s_out = 0.5, zero point 1: code = clamp(rint(2 g) + 1, 0, 15)
    y = np.array([-30.0, -0.75, -0.2, 0.0, 0.3, 1.0, 2.0, 3.4, 7.1, 100.0], np.float32)
    g, q = oracle.gelu_codes(y, 2.0, 1)
    #   g:      -0     -0.17  -0.084  0    0.185 0.841 1.954 3.399 7.1  100
    #   2g:      -0    -0.34  -0.17   0    0.37  1.68  3.91  6.80  14.2 200
    assert q.tolist() == [1, 1, 1, 1, 1, 3, 5, 8, 15, 15]
    # half-way cases round to even: g = 0.25 * k for 2 g = k + 0.5
    y2 = np.array([8.25, 8.75], np.float32)                  # GELU(y) = y up there: 2 g = 16.5, 17.5
    assert oracle.gelu_codes(y2, 2.0, -10)[1].tolist() == [6, 8]
    # codes are a monotone function of g, cover 0..15 and sit in range
    ys = np.linspace(-6.0, 9.0, 30001, dtype=np.float32)
    g, q = oracle.gelu_codes(ys, 2.0, 1)
    order = np.argsort(g, kind="stable")
    assert np.all(np.diff(q[order].astype(np.int32)) >= 0)
    assert q.min() >= 0 and q.max() == 15


def test_gelu_epilogue_is_the_chain_of_its_steps(oracle):
    """The epilogue applied to accumulators equals: the plain fp32 dequant (pinned elsewhere),
    then the GELU code of that value."""
    rng = np.random.default_rng(5)
    M, N = 7, 33
    acc = rng.integers(-40000, 40000, (M, N)).astype(np.int32)
    rowsum = rng.integers(-500, 500, M).astype(np.int32)
    rowscale = rng.uniform(1e-4, 3e-4, M).astype(np.float32)
    bias = rng.normal(0, 0.5, M).astype(np.float32)
    _, y, _ = oracle.epilogue(acc, rowsum, 7, rowscale, 0.31, bias, False)
    g, q = oracle.epilogue_gelu(acc, rowsum, 7, rowscale, 0.31, bias, 3.0, 1)
    g2, q2 = oracle.gelu_codes(y, 3.0, 1)
    assert np.array_equal(g.ravel(), g2) and np.array_equal(q.ravel(), q2)
