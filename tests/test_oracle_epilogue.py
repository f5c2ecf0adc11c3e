"""Pins of the oracle's epilogue (bias, GELU) against what mathematics fixes."""
import math

import numpy as np
import pytest

from oracle import vnm_oracle as o


def test_gelu_known_values_and_identities():
    # Phi(1) = 0.841344746068543 (standard normal table), so GELU(1) = Phi(1), GELU(-1) = -(1 - Phi(1))
    assert o.gelu_erf(np.array([1.0]))[0] == pytest.approx(0.841344746068543, abs=1e-15)
    assert o.gelu_erf(np.array([-1.0]))[0] == pytest.approx(-0.158655253931457, abs=1e-15)
    # Phi(2) = 0.977249868051821
    assert o.gelu_erf(np.array([2.0]))[0] == pytest.approx(2 * 0.977249868051821, abs=1e-14)
    x = np.linspace(-8, 8, 3201)
    g = o.gelu_erf(x)
    assert g[1600] == 0.0
    # x Phi(x) - (-x) Phi(-x) = x (Phi(x) + Phi(-x)) = x
    assert np.allclose(g - o.gelu_erf(-x), x, atol=1e-15)
    # asymptotes and the global minimum (-0.16997 at x = -0.75179)
    assert abs(g[-1] - 8.0) < 1e-13 and abs(g[0]) < 1e-13
    assert g.min() == pytest.approx(-0.169971, abs=1e-5)
    assert x[g.argmin()] == pytest.approx(-0.75179, abs=5e-3)


def test_gelu_slope_bound_is_the_stated_constant():
    x = np.linspace(-10, 10, 400001)
    g = o.gelu_erf(x)
    slope = np.diff(g) / np.diff(x)
    assert slope.max() < o.GELU_LIPSCHITZ and slope.max() > 1.128
    assert slope.min() > -0.13
    gt = o.gelu_tanh(x)
    st = np.diff(gt) / np.diff(x)
    assert st.max() < o.GELU_LIPSCHITZ


def test_tanh_form_tracks_the_definition():
    x = np.linspace(-6, 6, 2401)
    d = np.abs(o.gelu_tanh(x) - o.gelu_erf(x))
    assert d.max() < 5e-4 and d.max() > 1e-4     # the known accuracy of the approximation
    # written out independently for three points
    for v in (-1.5, 0.3, 2.5):
        ref = 0.5 * v * (1 + math.tanh(math.sqrt(2 / math.pi) * (v + 0.044715 * v ** 3)))
        assert o.gelu_tanh(np.array([v]))[0] == pytest.approx(ref, abs=1e-15)


def test_bias_broadcasts_over_columns_and_grows_the_bound():
    C = np.arange(12, dtype=np.float64).reshape(3, 4)
    E = np.ones((3, 4))
    bias = np.array([1.0, -2.0, 0.5], dtype=np.float16).view(np.uint16)
    Y, Ey = o.epilogue_fp64(C, E, bias, "none")
    assert np.array_equal(Y, C + np.array([[1.0], [-2.0], [0.5]]))
    assert np.array_equal(Ey, E + np.array([[1.0], [2.0], [0.5]]))
    Y0, E0 = o.epilogue_fp64(C, E, None, "none")
    assert np.array_equal(Y0, C) and np.array_equal(E0, E)
    with pytest.raises(ValueError):
        o.epilogue_fp64(C, E, bias[:2], "none")
    # zero product: every row is act(bias)
    Yg, _ = o.epilogue_fp64(np.zeros((3, 4)), np.zeros((3, 4)), bias, "gelu")
    assert np.allclose(Yg, o.gelu_erf(np.array([[1.0], [-2.0], [0.5]])) * np.ones((1, 4)), atol=0)


def test_planted_mistakes_in_the_epilogue_are_caught():
    C = np.linspace(-3, 3, 20).reshape(4, 5)
    bias = np.array([0.5, -1.0, 2.0, 0.25], dtype=np.float16).view(np.uint16)
    good, _ = o.epilogue_fp64(C, np.abs(C), bias, "gelu")
    b = o.f16_bits_to_f64(bias)
    wrong_axis = o.gelu_erf(C + np.resize(b, 5)[None, :])        # bias along columns
    act_before_bias = o.gelu_erf(C) + b[:, None]
    no_half = C + b[:, None]
    for bad in (wrong_axis, act_before_bias, no_half):
        assert np.abs(bad - good).max() > 1e-2


def test_linear_layer_view_is_x_times_masked_weight_transposed():
    from paper_2310_02065_amd import inputs
    R, K, T, V, M = 32, 48, 5, 16, 6
    A, mask, _ = inputs.gen_problem(R, K, 8, V, M, 1.0, seed=21)
    rng = np.random.default_rng(4)
    X = rng.standard_normal((T, K)).astype(np.float16)
    bias = rng.standard_normal(R).astype(np.float16)
    vals, cols, meta = o.compress(A, mask, V, M)
    Y, Ey = o.linear_fp64(vals, cols, meta, R, K, V, M, X.view(np.uint16), bias.view(np.uint16), "none")
    W = np.where(mask != 0, A.view(np.float16).astype(np.float64), 0.0)          # dense masked weight, no format
    ref = np.zeros((T, R))
    for t in range(T):
        for r in range(R):
            ref[t, r] = sum(float(X[t, k]) * W[r, k] for k in range(K)) + float(bias[r])
    assert Y.shape == (T, R) and np.allclose(Y, ref, rtol=0, atol=1e-12)
    assert (Ey >= np.abs(Y) - 1e-12).all()
    Yg, _ = o.linear_fp64(vals, cols, meta, R, K, V, M, X.view(np.uint16), bias.view(np.uint16), "gelu")
    assert np.allclose(Yg, o.gelu_erf(ref), atol=1e-12)
    with pytest.raises(ValueError):
        o.linear_fp64(vals, cols, meta, R, K, V, M, X.view(np.uint16)[:, :-1])
