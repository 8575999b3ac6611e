"""Pins of the oracle's minibatch estimator and of Algorithm 5: a batch that lists every row once is the
full gradient, the average over all batches of a size is the full gradient (unbiasedness, by enumeration),
a one-row batch against the formula of that row written out, repeated rows, dense against CSR, and
Algorithm 5 with full batches against Algorithm 2."""
import itertools

import numpy as np
import pytest

from paper_2106_05203_amd import workloads


def problems(oracle, seed):
    rng = np.random.default_rng(seed)
    n, m, d = 3, 6, 5
    A = rng.standard_normal((n, m, d)).astype(np.float32)
    y = np.where(rng.random((n, m)) < 0.5, 1.0, -1.0).astype(np.float32)
    b = rng.standard_normal((n, m)).astype(np.float32)
    return oracle.LogRegDense(A, y, 0.1), oracle.LeastSquaresDense(A, b, 0.05), rng


@pytest.mark.parametrize("which", [0, 1])
def test_full_batch_is_the_gradient(oracle, which):
    P = problems(oracle, 1)[which]
    rng = np.random.default_rng(2)
    x = rng.standard_normal(P.d)
    batch = np.stack([rng.permutation(P.m) for _ in range(P.n)])
    assert np.allclose(oracle.minibatch_grads(P, x, batch), P.grads(x), rtol=1e-13, atol=1e-15)


@pytest.mark.parametrize("which", [0, 1])
@pytest.mark.parametrize("tau", [1, 2, 4])
def test_mean_over_all_batches_is_the_gradient(oracle, which, tau):
    P = problems(oracle, 3)[which]
    x = np.random.default_rng(4).standard_normal(P.d)
    subsets = list(itertools.combinations(range(P.m), tau))
    acc = np.zeros((P.n, P.d))
    for S in subsets:
        acc += oracle.minibatch_grads(P, x, np.tile(np.array(S), (P.n, 1)))
    assert np.allclose(acc / len(subsets), P.grads(x), rtol=1e-12, atol=1e-14)


def test_one_row_batches(oracle):
    """tau = 1: ghat = -y a / (1 + exp(y a^T x)) + reg'(x) for the logistic loss, 2 (a^T x - b) a + reg'(x)
    for least squares; every worker may draw another row."""
    L, Q, rng = problems(oracle, 5)
    x = rng.standard_normal(L.d)
    rows = np.array([[4], [0], [2]])
    gl, gq = oracle.minibatch_grads(L, x, rows), oracle.minibatch_grads(Q, x, rows)
    for i in range(L.n):
        a, l = L.A[i, rows[i, 0]].astype(np.float64), rows[i, 0]
        z = float(a @ x)
        reg = lambda lam: 2.0 * lam * x / (1.0 + x * x) ** 2
        assert np.allclose(gl[i], -float(L.y[i, l]) * a / (1.0 + np.exp(float(L.y[i, l]) * z)) + reg(L.lam), rtol=1e-13)
        assert np.allclose(gq[i], 2.0 * (z - float(Q.b[i, l])) * a + reg(Q.lam), rtol=1e-13)


def test_repeated_rows_count_twice(oracle):
    L, _, rng = problems(oracle, 6)
    x = rng.standard_normal(L.d)
    one = oracle.minibatch_grads(L, x, np.array([[1], [1], [1]]))
    two = oracle.minibatch_grads(L, x, np.array([[1, 1], [1, 1], [1, 1]]))
    assert np.allclose(one, two, rtol=1e-14)
    mixed = oracle.minibatch_grads(L, x, np.array([[1, 1, 3]] * 3))
    three = oracle.minibatch_grads(L, x, np.array([[3]] * 3))
    reg = 2.0 * L.lam * x / (1.0 + x * x) ** 2
    assert np.allclose(mixed - reg, (2.0 * (one - reg) + (three - reg)) / 3.0, rtol=1e-13, atol=1e-16)


def test_csr_batches_match_dense(oracle):
    n, d, m = 2, 40, 9
    W = workloads.logreg_csr(n, d, m, 7, seed=8)
    C = oracle.LogRegCSR(W.rowptr, W.col, W.val, W.y, n, m, d, 0.1)
    D = oracle.LogRegDense(oracle.densify_csr(W.rowptr, W.col, W.val, n, m, d), np.asarray(W.y).reshape(n, m), 0.1)
    rng = np.random.default_rng(9)
    x = rng.standard_normal(d)
    batch = np.stack([rng.choice(m, size=4, replace=False) for _ in range(n)])
    assert np.allclose(oracle.minibatch_grads(C, x, batch), oracle.minibatch_grads(D, x, batch), rtol=1e-12, atol=1e-15)


def test_algorithm_5_with_full_batches_is_algorithm_2(oracle):
    L, _, rng = problems(oracle, 10)
    k, gamma = 2, 0.3
    x0 = rng.standard_normal(L.d)
    a = oracle.init_state(x0, L.grads(x0), k, init="grad", storage_f32=False)
    b = a.copy()
    for t in range(8):
        oracle.iteration(a, L.grads, k, gamma, storage_f32=False)
        batch = np.stack([rng.permutation(L.m) for _ in range(L.n)])
        oracle.iteration_stochastic(b, L, batch, k, gamma, storage_f32=False)
        assert np.allclose(a.x, b.x, rtol=1e-11, atol=1e-13)
        assert np.allclose(b.g, b.g_i.mean(axis=0), rtol=1e-11, atol=1e-13)


def test_algorithm_5_keeps_the_mean_invariant_and_uses_the_batch(oracle):
    """g = mean g_i under any estimator, and the message is the Top-k of (estimator - g_i), not of the gradient."""
    L, _, rng = problems(oracle, 11)
    k, gamma = 1, 0.2
    x0 = np.zeros(L.d)
    st = oracle.init_state(x0, L.grads(x0), k, init="zero", storage_f32=False)
    batch = np.array([[0], [1], [2]])
    est = oracle.minibatch_grads(L, st.x, batch)
    oracle.iteration_stochastic(st, L, batch, k, gamma, storage_f32=False)
    for i in range(L.n):
        j = int(np.argmax(np.abs(est[i])))
        expect = np.zeros(L.d)
        expect[j] = est[i, j]
        assert np.allclose(st.g_i[i], expect, rtol=1e-14)
    assert np.allclose(st.g, st.g_i.mean(axis=0), rtol=1e-13)
