"""Pins of the oracle's classical error feedback (Algorithm 4): a hand-worked example, the telescoped
error recursion, the contraction of the error, and Theorem 3's equivalence with EF21 for a compressor
that is deterministic, positively homogeneous and additive (Top-d, the identity)."""
import json
import os

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def test_hand_worked_example(oracle):
    ex = json.load(open(os.path.join(HERE, "golden", "ef_hand_example.json")))
    st = oracle.EFState(np.array(ex["x0"]), np.zeros((ex["n"], ex["d"])))
    for r in (0, 1):
        oracle.ef_iteration(st, np.array(ex[f"grads_round{r}"]), ex["k"], ex["gamma"])
        want = ex["expect"][f"round{r}"]
        assert st.e.tolist() == want["e"] and st.x.tolist() == want["x"]
        assert st.msg_idx.tolist() == want["msg_idx"] and st.msg_val.tolist() == want["msg_val"]


@pytest.mark.parametrize("seed", range(4))
def test_messages_and_errors_telescope(oracle, seed):
    """Summing line 6 over the rounds: sum_t w_i^t = gamma sum_t grad f_i(x^t) - e_i^T, hence
    x^T = x^0 - (1/n) sum_i (gamma sum_t grad f_i(x^t) - e_i^T); and every round leaves
    ||e_i||^2 <= (1 - k/d) ||e_i_old + gamma grad||^2 with zeros where entries were kept."""
    rng = np.random.default_rng(seed)
    n, d, k, gamma = 4, 30, int(rng.integers(1, 30)), 0.3
    targets = rng.standard_normal((n, d))
    grads_at = lambda x: x[None, :] - targets
    st = oracle.EFState(rng.standard_normal(d), np.zeros((n, d)))
    x0, acc = st.x.copy(), np.zeros((n, d))
    for _ in range(12):
        g = grads_at(st.x)
        p = st.e + gamma * g
        acc += gamma * g
        oracle.ef_iteration(st, grads_at, k, gamma, storage_f32=False)
        assert np.all(np.sum(st.e ** 2, axis=1) <= (1 - k / d) * np.sum(p ** 2, axis=1) * (1 + 1e-12) + 1e-300)
        assert np.all(np.take_along_axis(st.e, st.msg_idx.astype(np.int64), axis=1) == 0.0)
    assert np.allclose(st.x, x0 - (acc - st.e).mean(axis=0), rtol=1e-12, atol=1e-12)


def test_identity_compressor_makes_ef_ef21_and_gd_coincide(oracle):
    """Theorem 3: for a deterministic, positively homogeneous and additive compressor EF and EF21
    produce the same iterates.  Top-d is such a compressor (the identity), and then both are
    gradient descent."""
    rng = np.random.default_rng(11)
    n, d, gamma = 3, 10, 0.2
    targets = rng.standard_normal((n, d))
    grads_at = lambda x: x[None, :] - targets
    x0 = rng.standard_normal(d)
    ef = oracle.EFState(x0.copy(), np.zeros((n, d)))
    ef21 = oracle.init_state(x0, grads_at(x0), d, init="compressed", storage_f32=False)
    x_gd = x0.copy()
    for _ in range(20):
        x_gd = x_gd - gamma * grads_at(x_gd).mean(axis=0)
        oracle.ef_iteration(ef, grads_at, d, gamma, storage_f32=False)
        oracle.iteration(ef21, grads_at, d, gamma, order="step_first", storage_f32=False)
        assert np.allclose(ef.x, x_gd, rtol=1e-12, atol=1e-12)
        assert np.allclose(ef21.x, x_gd, rtol=1e-12, atol=1e-12)
        assert np.all(ef.e == 0.0)
