"""Pins of the oracle's least-squares objective (Section 5.2): finite differences, the closed form at
x = 0, the normal equations at the minimiser, and the quadratic's exact second-order expansion."""
import numpy as np
import pytest


def problem(oracle, seed, lam=0.0):
    rng = np.random.default_rng(seed)
    n, m, d = 3, 17, 6
    A = rng.standard_normal((n, m, d)).astype(np.float32)
    b = rng.standard_normal((n, m)).astype(np.float32)
    return oracle.LeastSquaresDense(A, b, lam), rng


@pytest.mark.parametrize("lam", [0.0, 0.1])
def test_gradient_matches_central_differences(oracle, lam):
    P, rng = problem(oracle, 1, lam)
    x = rng.standard_normal(P.d)
    h = 1e-6
    for i in range(P.n):
        g = P.grad_i(i, x)
        for j in range(P.d):
            e = np.zeros(P.d)
            e[j] = h
            fd = (P.loss_i(i, x + e) - P.loss_i(i, x - e)) / (2 * h)
            assert abs(fd - g[j]) <= 1e-6 * max(1.0, abs(g[j]))


def test_closed_forms(oracle):
    """At x = 0: f_i = mean(b^2), grad f_i = -(2/m) A^T b.  At the least-squares solution of worker i the
    normal equations make its gradient vanish.  f_i is a quadratic: f_i(x + h) = f_i(x) + g^T h + (1/m)|A h|^2."""
    P, rng = problem(oracle, 2)
    zero = np.zeros(P.d)
    for i in range(P.n):
        Ai, bi = P.A[i].astype(np.float64), P.b[i].astype(np.float64)
        assert np.isclose(P.loss_i(i, zero), np.mean(bi * bi), rtol=1e-14)
        assert np.allclose(P.grad_i(i, zero), -(2.0 / P.m) * Ai.T @ bi, rtol=1e-13, atol=1e-15)
        sol = np.linalg.lstsq(Ai, bi, rcond=None)[0]
        assert np.all(np.abs(P.grad_i(i, sol)) <= 1e-12)
        x, h = rng.standard_normal(P.d), rng.standard_normal(P.d)
        lhs = P.loss_i(i, x + h)
        rhs = P.loss_i(i, x) + P.grad_i(i, x) @ h + np.mean((Ai @ h) ** 2)
        assert np.isclose(lhs, rhs, rtol=1e-12)
    assert np.isclose(P.loss(zero), np.mean([P.loss_i(i, zero) for i in range(P.n)]))


def test_ef21_with_k_equal_d_descends_like_gradient_descent(oracle):
    P, rng = problem(oracle, 3)
    x0 = rng.standard_normal(P.d)
    gamma = 0.05
    st = oracle.init_state(x0, P.grads(x0), P.d, init="grad", storage_f32=False)
    x = x0.copy()
    for _ in range(10):
        x = x - gamma * P.grads(x).mean(axis=0)
        oracle.iteration(st, P.grads, P.d, gamma, order="step_first", storage_f32=False)
        assert np.allclose(st.x, x, rtol=1e-12, atol=1e-12)
    assert P.loss(st.x) < P.loss(x0)
