"""Pins for the oracle's weight projection in fp32 and the straight-through backward step
(Alg. 1 loop body, Eq. 5), against what the paper and arithmetic fix."""
import numpy as np
import pytest

import synth_inputs as si


def _case(oracle, M=24, K=200, seed=0):
    rng = np.random.default_rng(seed)
    W = si.weights_rowscaled(rng, M, K)
    scheme = si.scheme_permutation(rng, oracle.ratio_counts(M, 35, 60, 5))
    return rng, W, scheme


def test_projection_lands_on_the_level_sets(oracle):
    """Eq. 1 / Eq. 3: every projected weight is alpha times a member of its scheme's set."""
    _, W, scheme = _case(oracle)
    what, alpha = oracle.project_rows_f32(W, scheme)
    assert np.array_equal(alpha, np.abs(W).max(axis=1))
    for r in range(W.shape[0]):
        ratio = what[r].astype(np.float64) / float(alpha[r])
        if scheme[r] == 1:  # PoT-4: 0 or +-2^-k, k = 0..6
            nz = ratio[ratio != 0]
            k = -np.log2(np.abs(nz))
            assert np.allclose(k, np.rint(k), atol=1e-6) and k.min() > -1e-6 and k.max() < 6 + 1e-6
        else:
            Q = 7 if scheme[r] == 0 else 127
            j = ratio * Q
            assert np.allclose(j, np.rint(j), atol=2e-4) and np.abs(j).max() <= Q + 1e-3


def test_projection_agrees_with_the_float64_levels(oracle):
    """The fp32 value rowscale * q is within two roundings of the exact level alpha * q / Q."""
    _, W, scheme = _case(oracle, seed=1)
    what, _ = oracle.project_rows_f32(W, scheme)
    ref = oracle.quantize_rows(W, scheme)["what"]
    assert np.all(np.abs(what - ref) <= 2.0 ** -22 * np.abs(ref))


def test_projection_error_bounds(oracle):
    """Fixed: at most half a step (Eq. 1); PoT: within a factor sqrt(2) above 2^-6.5 (Eq. 4)."""
    _, W, scheme = _case(oracle, seed=2)
    what, alpha = oracle.project_rows_f32(W, scheme)
    for r in range(W.shape[0]):
        a = float(alpha[r])
        if scheme[r] == 1:
            x = np.abs(W[r].astype(np.float64)) / a
            big = x >= 2.0 ** -6.5
            assert np.all(np.abs(np.log2(np.abs(what[r][big].astype(np.float64)) / a / x[big])) <= 0.5 + 1e-6)
            assert np.all(what[r][x <= 2.0 ** -7] == 0)
        else:
            Q = 7 if scheme[r] == 0 else 127
            assert np.all(np.abs(what[r].astype(np.float64) - W[r]) <= a / (2 * Q) * (1 + 1e-5))


def test_projection_is_idempotent_and_odd(oracle):
    _, W, scheme = _case(oracle, seed=3)
    what, alpha = oracle.project_rows_f32(W, scheme)
    again, _ = oracle.project_rows_f32(what, scheme, alpha)
    assert np.array_equal(again, what)
    neg, _ = oracle.project_rows_f32(-W, scheme)
    assert np.array_equal(neg, -what)


def test_projection_with_caller_alpha_clips(oracle):
    _, W, scheme = _case(oracle, seed=4)
    alpha = (np.abs(W).max(axis=1) * 0.5).astype(np.float32)
    what, a_used = oracle.project_rows_f32(W, scheme, alpha)
    assert np.array_equal(a_used, alpha)
    clipped = np.abs(W) > alpha[:, None]
    assert clipped.any()
    assert np.allclose(np.abs(what[clipped]), np.broadcast_to(alpha[:, None], W.shape)[clipped], rtol=1e-6)
    with pytest.raises(ValueError):
        oracle.project_rows_f32(W, scheme, np.zeros(W.shape[0], np.float32))


def test_ste_backward_is_the_identity_inside_the_clip_range(oracle):
    """Eq. 5: derivative of round() taken as 1; Alg. 1: dLoss/dW <- dLoss/dproj(W)."""
    rng, W, scheme = _case(oracle, seed=5)
    g = rng.standard_normal(W.shape).astype(np.float32)
    assert np.array_equal(oracle.ste_backward(W, g), g)  # alpha = row maximum: nothing is clipped
    alpha = (np.abs(W).max(axis=1) * 0.5).astype(np.float32)
    dw = oracle.ste_backward(W, g, alpha)
    inside = np.abs(W) <= alpha[:, None]
    assert np.array_equal(dw[inside], g[inside]) and np.all(dw[~inside] == 0) and (~inside).any()


def test_ste_backward_matches_a_finite_difference_of_the_clip(oracle):
    """The backward mask is the derivative of the clip function (Section 3.1.1) wherever that
    derivative exists: compare with a central difference of clip(w) = min(max(w, -a), a)."""
    rng, W, scheme = _case(oracle, M=6, K=50, seed=6)
    alpha = (np.abs(W).max(axis=1) * 0.5).astype(np.float32)
    a = alpha[:, None].astype(np.float64)
    Wd = W.astype(np.float64)
    h = 1e-7
    fd = (np.clip(Wd + h, -a, a) - np.clip(Wd - h, -a, a)) / (2 * h)
    away = np.abs(np.abs(Wd) - a) > 1e-5  # not at the kink
    ones = np.ones_like(W)
    assert np.allclose(oracle.ste_backward(W, ones, alpha)[away], fd[away], atol=1e-6)
