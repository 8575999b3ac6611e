"""Pins of the oracle's smoothness constants and of the stepsize of Theorem 1: the Lipschitz inequality on
random pairs, tightness along the top eigenvector (exact for the quadratic, in the limit at x = 0 for the
logistic loss), closed forms of the stepsize (k = d, one worker, the printed form of sqrt(beta/theta)), and
the descent the theorem promises."""
import numpy as np
import pytest

from paper_2106_05203_amd import workloads


def make(oracle, kind, seed, lam):
    rng = np.random.default_rng(seed)
    n, m, d = 3, 40, 7
    A = rng.standard_normal((n, m, d)).astype(np.float32) * np.array([1.0, 2.0, 0.5])[:, None, None].astype(np.float32)
    t = np.where(rng.random((n, m)) < 0.5, 1.0, -1.0).astype(np.float32)
    if kind == "logistic":
        return oracle.LogRegDense(A, t, lam), rng
    return oracle.LeastSquaresDense(A, t, lam), rng


@pytest.mark.parametrize("kind", ["logistic", "squares"])
@pytest.mark.parametrize("lam", [0.0, 0.3])
def test_gradients_are_lipschitz_with_these_constants(oracle, kind, lam):
    P, rng = make(oracle, kind, 1, lam)
    L = oracle.smoothness_constants(P)
    worst = np.zeros(P.n)
    for _ in range(200):
        x, y = rng.standard_normal(P.d) * rng.choice([0.01, 1.0, 5.0]), rng.standard_normal(P.d) * rng.choice([0.01, 1.0])
        for i in range(P.n):
            ratio = np.linalg.norm(P.grad_i(i, x) - P.grad_i(i, y)) / np.linalg.norm(x - y)
            assert ratio <= L[i] * (1 + 1e-12)
            worst[i] = max(worst[i], ratio)
    assert np.all(worst >= 0.2 * L)          # and they are not orders of magnitude too large


@pytest.mark.parametrize("kind", ["logistic", "squares"])
@pytest.mark.parametrize("lam", [0.0, 0.3])
def test_constant_of_f_is_a_lipschitz_constant_below_the_mean(oracle, kind, lam):
    """f = (1/n) sum f_i: its gradient (the mean of the workers') changes by at most L |x - y| on random pairs,
    L is never above the mean of the L_i (the remark before Theorem 1) and never below any bound a pair shows."""
    P, rng = make(oracle, kind, 3, lam)
    L, L_i = oracle.smoothness_constant_of_f(P), oracle.smoothness_constants(P)
    assert L <= np.mean(L_i) * (1 + 1e-12)
    assert L >= np.min(L_i) / P.n            # one worker's share of the mean alone
    worst = 0.0
    for _ in range(200):
        x, y = rng.standard_normal(P.d) * rng.choice([0.01, 1.0, 5.0]), rng.standard_normal(P.d) * rng.choice([0.01, 1.0])
        ratio = np.linalg.norm(P.grads(x).mean(axis=0) - P.grads(y).mean(axis=0)) / np.linalg.norm(x - y)
        assert ratio <= L * (1 + 1e-12)
        worst = max(worst, ratio)
    assert worst >= 0.2 * L


def test_constant_of_f_is_attained(oracle):
    """lam = 0: along the top eigenvector v of the averaged matrix the quadratic's mean gradient changes by
    exactly L |v|; the logistic loss has curvature 1/4 at margin zero, so at x = 0 the change per unit step tends
    to L.  And a regulariser adds exactly 2 lam (its curvature at 0 is 2, the largest it has)."""
    for kind in ("squares", "logistic"):
        P, _ = make(oracle, kind, 4, 0.0)
        L = oracle.smoothness_constant_of_f(P)
        S = sum(np.asarray(P.A[i], np.float64).T @ np.asarray(P.A[i], np.float64) for i in range(P.n)) / (P.n * P.m)
        v = np.linalg.eigh(S)[1][:, -1]
        h = 1.0 if kind == "squares" else 1e-4
        change = np.linalg.norm(P.grads(h * v).mean(axis=0) - P.grads(0 * v).mean(axis=0)) / h
        assert abs(change - L) <= (1e-12 if kind == "squares" else 1e-6) * L
        Q, _ = make(oracle, kind, 4, 0.3)
        assert abs(oracle.smoothness_constant_of_f(Q) - (L + 0.6)) <= 1e-12 * L
    # one worker: f is f_1
    rng = np.random.default_rng(0)
    A = rng.standard_normal((1, 30, 5)).astype(np.float32)
    P1 = oracle.LogRegDense(A, np.ones((1, 30), np.float32), 0.2)
    assert abs(oracle.smoothness_constant_of_f(P1) - oracle.smoothness_constants(P1)[0]) <= 1e-12


def test_constants_are_attained(oracle):
    """lam = 0: the quadratic's gradient changes by exactly L_i |v| along the top eigenvector v; the logistic
    loss has curvature 1/4 at margin zero, so at x = 0 the change per unit step tends to L_i."""
    for kind in ("squares", "logistic"):
        P, _ = make(oracle, kind, 2, 0.0)
        L = oracle.smoothness_constants(P)
        for i in range(P.n):
            Ai = P.A[i].astype(np.float64)
            v = np.linalg.eigh(Ai.T @ Ai)[1][:, -1]
            step = 1.0 if kind == "squares" else 1e-4
            x0 = np.full(P.d, 0.7) if kind == "squares" else np.zeros(P.d)
            ratio = np.linalg.norm(P.grad_i(i, x0 + step * v) - P.grad_i(i, x0)) / step
            assert ratio == pytest.approx(L[i], rel=1e-12 if kind == "squares" else 1e-6)


def test_regulariser_adds_two_lambda(oracle):
    P0, _ = make(oracle, "logistic", 3, 0.0)
    P1, _ = make(oracle, "logistic", 3, 0.25)
    assert np.allclose(oracle.smoothness_constants(P1) - oracle.smoothness_constants(P0), 0.5, rtol=1e-12)


def test_csr_constants_match_dense(oracle):
    n, d, m = 2, 30, 12
    W = workloads.logreg_csr(n, d, m, 6, seed=4)
    C = oracle.LogRegCSR(W.rowptr, W.col, W.val, W.y, n, m, d, 0.1)
    D = oracle.LogRegDense(oracle.densify_csr(W.rowptr, W.col, W.val, n, m, d), np.asarray(W.y).reshape(n, m), 0.1)
    assert np.allclose(oracle.smoothness_constants(C), oracle.smoothness_constants(D), rtol=1e-13)


def test_stepsize_closed_forms(oracle):
    L_i = np.array([1.0, 3.0, 2.0])
    # k = d: no compression, beta = 0, the stepsize of gradient descent 1 / L
    assert oracle.theory_stepsize(L_i, 1.0) == pytest.approx(1.0 / 2.0, rel=1e-15)
    assert oracle.theory_stepsize(L_i, 1.0, L=1.5) == pytest.approx(1.0 / 1.5, rel=1e-15)
    # the form printed after Theorem 1: sqrt(beta/theta) = (1 + sqrt(1 - alpha)) / alpha - 1
    for alpha in (0.01, 0.25, 0.9):
        r = (1.0 + np.sqrt(1.0 - alpha)) / alpha - 1.0
        lt = np.sqrt(np.mean(L_i ** 2))
        assert oracle.theory_stepsize(L_i, alpha) == pytest.approx(1.0 / (2.0 + lt * r), rel=1e-12)
    # one worker: L = Ltilde = L_1, so gamma = alpha / (L_1 (1 + sqrt(1 - alpha)))
    a = 0.3
    assert oracle.theory_stepsize([4.0], a) == pytest.approx(a / (4.0 * (1.0 + np.sqrt(1.0 - a))), rel=1e-12)
    # more compression, smaller stepsize
    g = [oracle.theory_stepsize(L_i, a) for a in (0.05, 0.1, 0.5, 1.0)]
    assert all(g[j] < g[j + 1] for j in range(3))


@pytest.mark.parametrize("kind", ["logistic", "squares"])
def test_theorem_1_holds_with_this_stepsize(oracle, kind):
    """(1/T) sum_t |grad f(x^t)|^2 <= 2 (f(x^0) - f_inf) / (gamma T) + G^0 / (theta T), f_inf >= 0 here."""
    P, rng = make(oracle, kind, 5, 0.1)
    k, T = 2, 200
    gamma = oracle.theory_stepsize(oracle.smoothness_constants(P), k / P.d)
    theta, _ = oracle.theta_beta(k / P.d)
    x0 = rng.standard_normal(P.d)
    st = oracle.init_state(x0, P.grads(x0), k, init="compressed", storage_f32=False)
    G0, f0 = oracle.distortion(st, P.grads(x0)), P.loss(x0)
    sq = []
    for t in range(T):
        sq.append(np.sum(P.grads(st.x).mean(axis=0) ** 2))
        oracle.iteration(st, P.grads, k, gamma, order="step_first", storage_f32=False)
    assert np.mean(sq) <= 2 * f0 / (gamma * T) + G0 / (theta * T)
    assert P.loss(st.x) < f0
