"""Pins for the oracle's quantizers (CPU only).

Each test checks the oracle against something the paper or mathematics fixes --
the printed level sets (Eq. 1, Eq. 3), brute-force projection onto those sets,
error bounds, invariances -- never against a retyped copy of its own formula.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden_levels():
    out = {}
    for line in open(os.path.join(GOLDEN, "level_sets.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, *vals = line.split()
        out[name] = [Fraction(v) for v in vals]
    return out


def _signed(levels):
    return sorted(set(levels) | {-v for v in levels})


def _sweep(alpha, n=4001, span=1.2):
    return np.linspace(-span * alpha, span * alpha, n).astype(np.float32)


@pytest.mark.parametrize("alpha", [1.0, 0.37, 3.0])
def test_fixed4_level_set_is_eq1(oracle, alpha):
    """Dense sweep: the set of Fixed-4 outputs is exactly the 15-element set of Eq. 1."""
    g = _golden_levels()["fixed4"]
    q = oracle.fixed_codes(_sweep(alpha), alpha, 4)
    got = sorted(set(Fraction(int(v), 7) for v in q))
    assert got == _signed(g)
    assert len(got) == 15 and Fraction(0) in got


def test_fixed8_level_set_is_eq1(oracle):
    g = _golden_levels()
    q = oracle.fixed_codes(_sweep(1.0, n=200001), 1.0, 8)
    got = sorted(set(int(v) for v in q))
    assert got == list(range(-127, 128))
    assert int(g["fixed8_count_nonneg"][0]) == 128 and g["fixed8_step"][0] == Fraction(1, 127)


@pytest.mark.parametrize("m,Q", [(4, 7), (8, 127)])
def test_fixed_is_nearest_level_bruteforce(oracle, m, Q):
    """Projection onto Eq. 1's set: brute-force argmin over all levels, in exact rationals."""
    rng = np.random.default_rng(7)
    alpha = np.float32(0.8125)  # exactly representable, so w/alpha is clean to reason about
    w = (rng.uniform(-1.3, 1.3, 3000) * alpha).astype(np.float32)
    q = oracle.fixed_codes(w, float(alpha), m)
    levels = [Fraction(j, Q) for j in range(-Q, Q + 1)]
    for wi, qi in zip(w, q):
        x = np.float32(wi) / alpha  # the fp32 ratio the quantizer sees
        x = Fraction(float(min(max(x, np.float32(-1)), np.float32(1))))
        d = [abs(x - lv) for lv in levels]
        best = min(d)
        assert abs(x - Fraction(int(qi), Q)) <= best + Fraction(1, 10 ** 7), (wi, qi)


@pytest.mark.parametrize("m,Q", [(4, 7), (8, 127)])
def test_fixed_error_half_step_and_clip(oracle, m, Q):
    alpha = 0.37
    w = _sweep(alpha, n=20001, span=1.5)
    q = oracle.fixed_codes(w, alpha, m).astype(np.float64)
    what = alpha * q / Q
    inside = np.abs(w) <= np.float32(alpha)
    assert np.all(np.abs(what[inside] - w[inside]) <= alpha / (2 * Q) * (1 + 1e-5))
    # outside the clipping range the output is the extreme level and the error is |w| - alpha
    out = ~inside
    assert np.all(np.abs(q[out]) == Q)
    assert np.allclose(np.abs(what[out] - w[out]), np.abs(w[out]) - alpha, rtol=1e-5, atol=1e-7)


def test_fixed_ties_round_half_to_even(oracle):
    """Exact ties: with alpha = 2 the ratio w/alpha is exact, so Q*x lands exactly on k + 1/2."""
    # m = 4: x = 0.5 -> 3.5 -> 4 (even), both signs
    assert list(oracle.fixed_codes(np.array([1.0, -1.0], np.float32), 2.0, 4)) == [4, -4]
    # m = 8: x = 0.5 -> 63.5 -> 64 (even); x = 0.25 -> 31.75 -> 32 (no tie)
    assert list(oracle.fixed_codes(np.array([1.0, -1.0], np.float32), 2.0, 8)) == [64, -64]
    assert list(oracle.fixed_codes(np.array([0.5], np.float32), 2.0, 8)) == [32]
    # alpha = 14: w = 5 -> x*7 = 2.5 up to fp32 rounding of 5/14; w = 7 -> x = 0.5 exactly -> 3.5 -> 4
    assert list(oracle.fixed_codes(np.array([7.0], np.float32), 14.0, 4)) == [4]


@pytest.mark.parametrize("alpha", [1.0, 0.37, 5.0])
def test_pot4_level_set_is_eq3(oracle, alpha):
    """Dense sweep: outputs are exactly 0 or +-alpha*2^-k, k = 0..6 (15 levels)."""
    g = _golden_levels()["pot4"]
    w = np.concatenate([_sweep(alpha, n=40001), (_sweep(alpha, n=4001) / 50).astype(np.float32)])
    q = oracle.pot4_ints(w, alpha)
    got = sorted(set(Fraction(int(v), 64) for v in q))
    assert got == _signed(g)
    nz = np.abs(q[q != 0]).astype(np.float64)
    e = np.log2(nz / 64.0)
    assert np.all(e == np.round(e)) and e.min() == -6 and e.max() == 0


def test_pot4_rounds_the_logarithm(oracle):
    """Eq. 4 rounds log2 of the magnitude: boundary between 2^e and 2^(e+1) is sqrt(2)*2^e."""
    rng = np.random.default_rng(11)
    x = rng.uniform(2.0 ** -6.4, 1.0, 20000)
    x = x[np.abs((np.log2(x) % 1.0) - 0.5) > 1e-6]  # stay off the boundary itself
    w = (x * rng.choice([-1.0, 1.0], x.size)).astype(np.float32)
    q = oracle.pot4_ints(w, 1.0)
    a = np.abs(w.astype(np.float64))
    e = np.clip(np.round(np.log2(a)), -6, 0)
    assert np.array_equal(np.abs(q), (2.0 ** (6 + e)).astype(np.int64))
    assert np.array_equal(np.sign(q), np.sign(w).astype(np.int64))
    # a point that separates log-domain rounding from nearest-level rounding:
    # 0.72 is nearer to 0.5 on the line, but log2(0.72) = -0.47 rounds to 0 -> level 1
    assert list(oracle.pot4_ints(np.array([0.72, -0.72, 0.70], np.float32), 1.0)) == [64, -64, 32]
    # within 1/2 in the log domain wherever the exponent is not clamped
    ok = (a >= 2.0 ** -6.5)
    assert np.all(np.abs(np.log2(np.abs(q[ok]) / 64.0) - np.log2(a[ok])) <= 0.5 + 1e-9)


def test_pot4_zero_threshold_and_clamp(oracle):
    t = 2.0 ** -7
    w = np.array([0.0, t, -t, np.nextafter(np.float32(t), np.float32(1)), t * 1.2, 2.0 ** -6.6,
                  1.0, 1.7, -3.0], np.float32)
    assert list(oracle.pot4_ints(w, 1.0)) == [0, 0, 0, 1, 1, 1, 64, 64, -64]


def test_exact_boundary_sqrt2_is_decided_without_libm(oracle):
    """Floats adjacent to sqrt(2)*2^e fall on the correct side (needs an exact comparison)."""
    for e in range(-6, 0):
        s = np.float32(math.sqrt(2.0) * 2.0 ** e)
        lo = s if float(s) ** 2 < 2.0 * 4.0 ** e else np.nextafter(s, np.float32(0))
        hi = np.nextafter(lo, np.float32(2))
        assert float(lo) ** 2 < 2.0 * 4.0 ** e < float(hi) ** 2
        q = oracle.pot4_ints(np.array([lo, hi], np.float32), 1.0)
        assert list(q) == [2 ** (6 + e), 2 ** (7 + e)]


@pytest.mark.parametrize("scheme", [0, 1, 2])
def test_idempotence_symmetry_scale_invariance(oracle, scheme):
    rng = np.random.default_rng(3 + scheme)
    W = (rng.standard_normal((6, 257)) * 0.05).astype(np.float32)
    sch = np.full(6, scheme, np.uint8)
    r = oracle.quantize_rows(W, sch)
    # the element of largest magnitude sits on the extreme level when alpha = max|w|
    top = {0: 7, 1: 64, 2: 127}[scheme]
    assert np.all(np.abs(r["wint"]).max(axis=1) == top)
    # idempotent: quantizing the quantized weights with the same alpha changes nothing
    r2 = oracle.quantize_rows(r["what"].astype(np.float32), sch, alpha=r["alpha"])
    assert np.array_equal(r2["wint"], r["wint"])
    # odd symmetry
    r3 = oracle.quantize_rows(-W, sch)
    assert np.array_equal(r3["wint"], -r["wint"])
    # scaling weights (and hence alpha) by a power of two leaves the codes unchanged
    r4 = oracle.quantize_rows(W * np.float32(8.0), sch)
    assert np.array_equal(r4["wint"], r["wint"])
    assert np.array_equal(r4["rowscale"], r["rowscale"] * np.float32(8.0))


def test_levels_equal_rowscale_times_integer(oracle):
    rng = np.random.default_rng(5)
    W = (rng.standard_normal((9, 64)) * 0.1).astype(np.float32)
    sch = np.array([0, 1, 2] * 3, np.uint8)
    r = oracle.quantize_rows(W, sch)
    div = np.array([7.0, 64.0, 127.0])[sch]
    assert np.allclose(r["what"], r["alpha"][:, None].astype(np.float64) * r["wint"] / div[:, None], rtol=1e-15)
    assert np.allclose(r["rowscale"], r["alpha"] / div, rtol=2e-7)
    # PoT rowscale is exact
    p = sch == 1
    assert np.array_equal(r["rowscale"][p], r["alpha"][p] * np.float32(2.0 ** -6))


def test_zero_row_and_caller_alpha(oracle):
    W = np.zeros((2, 8), np.float32)
    W[1, 3] = 0.9
    r = oracle.quantize_rows(W, np.array([0, 1], np.uint8))
    assert r["alpha"][0] == 1.0 and not r["wint"][0].any()
    # caller alpha below max|w| -> the clip is live and saturates
    r = oracle.quantize_rows(W, np.array([0, 0], np.uint8), alpha=np.array([1.0, 0.3], np.float32))
    assert r["wint"][1, 3] == 7
    with pytest.raises(ValueError):
        oracle.quantize_rows(W, np.array([0, 3], np.uint8))


def test_shift_equals_multiply(oracle):
    """PoT weight x Fixed activation is a bit shift (Section 2.1.2)."""
    for k in range(7):
        for x in range(16):
            assert (x << (6 - k)) == x * 2 ** (6 - k)
            assert np.float32(x << (6 - k)) * np.float32(2.0 ** -6) == np.float32(x * 2.0 ** -k)
    rng = np.random.default_rng(17)
    W = (rng.standard_normal((5, 96)) * 0.05).astype(np.float32)
    sch = np.array([1, 0, 1, 2, 1], np.uint8)
    r = oracle.quantize_rows(W, sch)
    xq = rng.integers(0, 16, (7, 96)).astype(np.int32)
    full = oracle.gemm_acc(r["wint"], xq)
    sh = oracle.gemm_acc_pot_shift(r["wint"], sch, xq)
    assert np.array_equal(sh[sch == 1], full[sch == 1])


@pytest.mark.parametrize("ratio", [(35, 60, 5), (60, 35, 5), (65, 30, 5), (40, 50, 10), (100, 0, 0),
                                   (0, 100, 0), (50, 50, 0), (0, 95, 5), (0, 0, 100)])
@pytest.mark.parametrize("M", [64, 128, 256, 512, 1000, 3072, 4096, 10, 1])
def test_ratio_counts_follow_the_layer_uniform_ratio(oracle, ratio, M):
    """Per layer the row counts follow A:B:C with A+B+C = 100 (Section 4)."""
    a, b, c = ratio
    n4, npot, n8 = oracle.ratio_counts(M, a, b, c)
    assert n4 + npot + n8 == M and min(n4, npot, n8) >= 0
    assert abs(npot - M * a / 100) <= 1.0
    assert abs(n8 - M * c / 100) <= 1.0
    assert abs(n4 - M * b / 100) <= 1.5
    if c > 0:
        assert n8 >= 1
    if c == 0:
        assert n8 == 0
    if a == 0:
        assert npot == 0 or M * 0 == 0 and npot == 0
    if b == 0 and M > 1:
        assert n4 == 0


def test_ratio_counts_named_cases(oracle):
    assert oracle.ratio_counts(256, 35, 60, 5) == (153, 90, 13)
    assert oracle.ratio_counts(64, 35, 60, 5) == (39, 22, 3)
    assert oracle.ratio_counts(4096, 40, 50, 10) == (2048, 1638, 410)
    with pytest.raises(ValueError):
        oracle.ratio_counts(64, 50, 50, 5)


def test_variance_assignment(oracle):
    """Low-variance rows go to PoT-4, high-variance rows to Fixed-4; Fixed-8 rows stay (Alg. 1)."""
    rng = np.random.default_rng(23)
    M, K = 40, 200
    std = rng.permutation(np.linspace(0.01, 0.4, M))
    W = (rng.standard_normal((M, K)) * std[:, None]).astype(np.float32)
    scheme = np.zeros(M, np.uint8)
    f8 = rng.choice(M, 2, replace=False)
    scheme[f8] = 2
    out = oracle.assign_by_variance(W, scheme, 14)
    assert np.all(out[f8] == 2) and (out == 1).sum() == 14 and (out == 0).sum() == M - 16
    v = W.astype(np.float64).var(axis=1)
    assert v[out == 1].max() < v[out == 0].min()
    # numpy argsort gives the same split
    rest = np.array([r for r in range(M) if r not in set(f8)])
    low = set(rest[np.argsort(v[rest], kind="stable")[:14]])
    assert set(np.nonzero(out == 1)[0]) == low
