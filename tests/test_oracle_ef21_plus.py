"""Pins of the oracle's EF21+ (Algorithm 3): a hand-worked example, the distortion it must achieve
(the smaller of the two compressors', each bounded by the Top-k contraction of Section 2.1), the
k = d reduction to gradient descent, and its relation to EF21 (Algorithm 2)."""
import json
import os

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def test_hand_worked_example(oracle):
    ex = json.load(open(os.path.join(HERE, "golden", "ef21_plus_hand_example.json")))
    g_i = np.array(ex["g_i"])
    st = oracle.EF21State(np.array(ex["x"]), g_i.copy(), g_i.mean(axis=0))
    branch, B, M = oracle.iteration_plus(st, np.array(ex["grads"]), ex["k"], ex["gamma"], order="grad_first")
    want = ex["expect"]
    assert B.tolist() == want["B"] and M.tolist() == want["M"] and branch.tolist() == want["branch"]
    assert st.g_i.tolist() == want["g_i"] and st.g.tolist() == want["g"]
    assert st.msg_idx.tolist() == want["msg_idx"] and st.msg_val.tolist() == want["msg_val"]
    assert st.x.tolist() == want["x_after_step"]


@pytest.mark.parametrize("seed", range(6))
def test_new_distortion_is_the_smaller_one_and_contracts(oracle, seed):
    """After line 8, ||g_i - s||^2 = min(B, M); B <= (1 - k/d)||s||^2 and M <= (1 - k/d)||s - g_i||^2
    (Top-k is contractive with alpha = k/d, Section 2.1) up to the rounding of the fp32 update."""
    rng = np.random.default_rng(seed)
    n, d, k = 5, 40, int(rng.integers(1, 40))
    g_old = rng.standard_normal((n, d)) * rng.choice([0.0, 0.3, 3.0], size=(n, 1))
    s = rng.standard_normal((n, d))
    st = oracle.EF21State(np.zeros(d), oracle.round_storage(g_old, True), np.zeros(d))
    g_before = st.g_i.copy()
    s32 = oracle.round_storage(s, True)
    branch, B, M = oracle.plus_update(st, s32, k)
    new = np.sum((st.g_i - s32) ** 2, axis=1)
    assert np.allclose(new, np.minimum(B, M), rtol=1e-12, atol=0)
    assert np.array_equal(branch, (M > B).astype(np.int32))
    slack = 1e-6
    assert np.all(B <= (1 - k / d) * np.sum(s32 ** 2, axis=1) * (1 + slack))
    assert np.all(M <= (1 - k / d) * np.sum((s32 - g_before) ** 2, axis=1) * (1 + slack) + 1e-12)
    assert np.allclose(st.g, st.g_i.mean(axis=0), rtol=1e-6, atol=1e-7)


def test_k_equals_d_is_gradient_descent(oracle):
    """Top-d is the identity, so both branches give g_i = grad f_i(x) and the iterates are those of
    distributed gradient descent."""
    rng = np.random.default_rng(3)
    n, d, gamma = 3, 12, 0.2
    targets = rng.standard_normal((n, d))
    grads_at = lambda x: x[None, :] - targets                      # f_i = ||x - t_i||^2 / 2
    x0 = rng.standard_normal(d)
    st = oracle.init_state(x0, grads_at(oracle.round_storage(x0, True)), d, init="grad")
    x_gd = st.x.copy()
    for _ in range(15):
        x_gd = oracle.round_storage(x_gd - gamma * oracle.round_storage(grads_at(x_gd).mean(axis=0), True), True)
        oracle.iteration_plus(st, grads_at, d, gamma, order="step_first")
        assert np.allclose(st.x, x_gd, rtol=2e-6, atol=2e-7)


def test_zero_state_takes_the_markov_branch_and_equals_ef21(oracle):
    """With g_i = 0 the two compressors coincide (M = B): ties go to the Markov branch and the step
    is the EF21 step (Algorithm 2) from the same state."""
    rng = np.random.default_rng(4)
    n, d, k = 4, 50, 7
    grads = rng.standard_normal((n, d))
    a = oracle.EF21State(np.ones(d), np.zeros((n, d)), np.zeros(d))
    b = a.copy()
    branch, B, M = oracle.iteration_plus(a, grads, k, 0.1)
    oracle.iteration(b, grads, k, 0.1)
    assert not branch.any() and np.array_equal(B, M)
    assert np.array_equal(a.msg_idx, b.msg_idx) and np.array_equal(a.g_i, b.g_i)
    assert np.allclose(a.x, b.x, rtol=1e-6, atol=1e-7)


def test_never_worse_than_ef21_from_the_same_state(oracle):
    """G_i^{t+1} <= min(B, M) <= M (Section 3.5): from one state, EF21+ leaves no worker with a larger
    distortion than EF21 does."""
    rng = np.random.default_rng(5)
    n, d, k = 6, 64, 5
    grads = rng.standard_normal((n, d))
    g0 = oracle.round_storage(rng.standard_normal((n, d)) * np.linspace(0, 4, n)[:, None], True)
    a = oracle.EF21State(np.zeros(d), g0.copy(), g0.mean(axis=0))
    b = a.copy()
    branch, _, _ = oracle.plus_update(a, grads, k)
    oracle.compress_update(b, grads, k)
    s = oracle.round_storage(grads, True)
    da, db = np.sum((a.g_i - s) ** 2, axis=1), np.sum((b.g_i - s) ** 2, axis=1)
    assert np.all(da <= db * (1 + 1e-12))
    assert branch.any() and not branch.all(), "the example should exercise both branches"
