"""Pins for the oracle's objective and gradient (Section 5, eq. (9)): closed forms, a library
routine for the loss, central finite differences, CSR against dense.  No GPU."""
import numpy as np
import pytest

from paper_2106_05203_amd import workloads


@pytest.fixture(scope="module")
def small():
    return workloads.logreg_dense(n=3, d=12, m=40, seed=1)


def numpy_loss(A, y, x, lam):
    """eq. (9) typed with numpy's logaddexp: mean log(1+exp(-y a^T x)) + lam sum x^2/(1+x^2)."""
    z = A.astype(np.float64) @ x
    return np.logaddexp(0.0, -y.astype(np.float64) * z).mean() + lam * np.sum(x * x / (1.0 + x * x))


def test_closed_form_at_zero(oracle, small):
    """At x = 0 every sigmoid is 1/2 and the regulariser and its gradient vanish:
    f_i(0) = log 2, grad f_i(0) = -(1/(2m)) A_i^T y_i."""
    P = oracle.LogRegDense(small.A, small.y, 0.1)
    x0 = np.zeros(P.d)
    for i in range(P.n):
        assert abs(P.loss_i(i, x0) - np.log(2.0)) < 1e-15
        expect = -(small.A[i].astype(np.float64).T @ small.y[i].astype(np.float64)) / (2.0 * P.m)
        assert np.allclose(P.grad_i(i, x0), expect, rtol=1e-13, atol=1e-16)


def test_one_point_one_dim(oracle):
    """m = 1, d = 1, a = 2, y = -1, x = 0.5, lam = 0.3: f = log(1+e^{1}) + 0.3*0.25/1.25,
    f' = 2/(1+e^{-1}) + 2*0.3*0.5/1.25^2 (by hand)."""
    P = oracle.LogRegDense(np.array([[[2.0]]], np.float32), np.array([[-1.0]], np.float32), 0.3)
    x = np.array([0.5])
    assert abs(P.loss_i(0, x) - (np.log1p(np.e) + 0.3 * 0.25 / 1.25)) < 1e-15
    assert abs(P.grad_i(0, x)[0] - (2.0 / (1.0 + np.exp(-1.0)) + 2 * 0.3 * 0.5 / 1.25 ** 2)) < 1e-15


def test_regulariser_only(oracle):
    """With A = 0 the loss part is log 2 and the gradient is 2 lam x / (1+x^2)^2; at x_j = 1 that is
    lam/2, at x_j = -1 it is -lam/2, and it is odd in x."""
    d = 5
    P = oracle.LogRegDense(np.zeros((1, 3, d), np.float32), np.ones((1, 3), np.float32), 0.1)
    x = np.array([1.0, -1.0, 0.0, 2.0, -2.0])
    g = P.grad_i(0, x)
    assert np.allclose(g, [0.05, -0.05, 0.0, 2 * 0.1 * 2 / 25, -2 * 0.1 * 2 / 25], rtol=1e-15)
    assert abs(P.loss_i(0, x) - (np.log(2.0) + 0.1 * (0.5 + 0.5 + 0 + 0.8 + 0.8))) < 1e-15


def test_loss_matches_library_logaddexp(oracle, small):
    P = oracle.LogRegDense(small.A, small.y, 0.1)
    rng = np.random.default_rng(0)
    for scale in (0.1, 1.0, 30.0, 300.0):      # large scales exercise the overflow-safe branch
        x = rng.standard_normal(P.d) * scale
        for i in range(P.n):
            ref = numpy_loss(small.A[i], small.y[i], x, 0.1)
            assert abs(P.loss_i(i, x) - ref) <= 1e-13 * max(1.0, abs(ref))
    x = rng.standard_normal(P.d)
    assert abs(P.loss(x) - np.mean([numpy_loss(small.A[i], small.y[i], x, 0.1) for i in range(P.n)])) < 1e-14


def test_gradient_central_differences(oracle, small):
    P = oracle.LogRegDense(small.A, small.y, 0.1)
    rng = np.random.default_rng(2)
    x = rng.standard_normal(P.d)
    h = 1e-6
    for i in range(P.n):
        g = P.grad_i(i, x)
        fd = np.empty(P.d)
        for j in range(P.d):
            e = np.zeros(P.d)
            e[j] = h
            fd[j] = (P.loss_i(i, x + e) - P.loss_i(i, x - e)) / (2 * h)
        assert np.max(np.abs(g - fd)) <= 1e-6 * max(1.0, np.max(np.abs(g)))
        assert np.max(np.abs(g - fd)) <= 5e-9      # O(h^2) truncation + rounding, tighter in practice


def test_gradient_of_each_term_separately(oracle, small):
    """lam = 0 isolates the data term (vs numpy: -(1/m) A^T (y * sigmoid(-y z))); the difference
    between lam = 0.7 and lam = 0 isolates the regulariser term."""
    x = np.random.default_rng(4).standard_normal(small.A.shape[2])
    P0 = oracle.LogRegDense(small.A, small.y, 0.0)
    P7 = oracle.LogRegDense(small.A, small.y, 0.7)
    for i in range(P0.n):
        A = small.A[i].astype(np.float64)
        y = small.y[i].astype(np.float64)
        sig = 1.0 / (1.0 + np.exp(y * (A @ x)))
        assert np.allclose(P0.grad_i(i, x), -(A.T @ (y * sig)) / P0.m, rtol=1e-12, atol=1e-15)
        assert np.allclose(P7.grad_i(i, x) - P0.grad_i(i, x), 2 * 0.7 * x / (1 + x * x) ** 2, rtol=1e-11,
                           atol=1e-15)


def test_csr_equals_dense(oracle):
    W = workloads.logreg_csr(n=3, d=64, m=30, nnz_per_row=7, seed=3)
    dense = np.zeros((W.n * W.m, W.d), np.float32)
    for r in range(W.n * W.m):
        s, e = W.rowptr[r], W.rowptr[r + 1]
        dense[r, W.col[s:e]] = W.val[s:e]
    Pd = oracle.LogRegDense(dense.reshape(W.n, W.m, W.d), W.y, 0.1)
    Ps = oracle.LogRegCSR(W.rowptr, W.col, W.val, W.y, W.n, W.m, W.d, 0.1)
    x = np.random.default_rng(9).standard_normal(W.d)
    for i in range(W.n):
        assert abs(Pd.loss_i(i, x) - Ps.loss_i(i, x)) < 1e-14
        assert np.allclose(Pd.grad_i(i, x), Ps.grad_i(i, x), rtol=1e-12, atol=1e-16)
    assert abs(Pd.loss(x) - Ps.loss(x)) < 1e-14


def test_csr_central_differences(oracle):
    W = workloads.logreg_csr(n=2, d=40, m=25, nnz_per_row=5, seed=8)
    P = oracle.LogRegCSR(W.rowptr, W.col, W.val, W.y, W.n, W.m, W.d, 0.1)
    x = np.random.default_rng(1).standard_normal(W.d)
    h = 1e-6
    for i in range(W.n):
        g = P.grad_i(i, x)
        for j in range(W.d):
            e = np.zeros(W.d)
            e[j] = h
            fd = (P.loss_i(i, x + e) - P.loss_i(i, x - e)) / (2 * h)
            assert abs(g[j] - fd) <= 5e-9
