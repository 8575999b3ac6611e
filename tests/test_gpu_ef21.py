"""GPU parity of the EF21 iteration (ef21_step through the C ABI) against the CPU oracle.

Bars: messages (positions, values) and g_i bit-exact when both sides start from the same state and
see the same gradients; g and x within 1e-5 relative per coordinate (the library sums the messages
in fp32 in worker order, the oracle in fp64); f(x^t) within 1e-4 relative over a whole run with GPU-computed gradients.
"""
import numpy as np
import pytest

from helpers import RoundingBudget, close_per_coordinate, same_bits, sampled_positions
from paper_2106_05203_amd import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    from paper_2106_05203_amd import binding
    assert torch.cuda.is_available(), "these tests need the MI355X"
    binding.load_library()
    return torch, binding


def to_gpu(torch, a, dtype=np.float32):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=dtype)).cuda()


def oracle_step(oracle, st, budget, grads, k, gamma, order="grad_first"):
    """One oracle iteration (supplied gradients or a callable), charging the rounding budget."""
    if order == "step_first":
        budget.model_step(st.x.copy(), st.g)
        oracle.model_step(st, gamma, True)
    g_before = st.g.copy()
    oracle.compress_update(st, grads(st.x) if callable(grads) else grads, k, True)
    budget.compress_update(g_before, st.msg_idx, st.msg_val)
    if order == "grad_first":
        budget.model_step(st.x.copy(), st.g)
        oracle.model_step(st, gamma, True)


def compare_state(torch, h, st, budget, msgs=True, rows=None):
    """g_i and the messages bit for bit; g and x within 1e-5 relative per coordinate plus the
    rounding budget of fp32 arithmetic (see helpers.RoundingBudget)."""
    x, g_i, g = (t.cpu().numpy() for t in h.get_state())
    rows = range(h.n) if rows is None else rows
    for i in rows:
        assert same_bits(g_i[i], st.g_i[i].astype(np.float32)), f"g_i row {i} differs"
    if msgs:
        idx, val = (t.cpu().numpy() for t in h.get_messages())
        for i in rows:
            assert np.array_equal(idx[i], st.msg_idx[i]), f"message positions of worker {i} differ"
            assert same_bits(val[i], st.msg_val[i].astype(np.float32)), f"message values of worker {i} differ"
    ok, info = budget.check(g, st.g, "g")
    assert ok, f"g: max err, #bad = {info}"
    ok, info = budget.check(x, st.x, "x")
    assert ok, f"x: max err, #bad = {info}"
    return x, g_i, g


@pytest.mark.parametrize("n,d,k", [(1, 1, 1), (4, 100, 1), (3, 1000, 1000), (7, 4099, 41), (20, 2000, 20),
                                   (5, 70001, 700), (3, 300_000, 3000), (5, 70001, 1), (3, 300_000, 1), (6, 20_000, 1)])
@pytest.mark.parametrize("order", ["grad_first", "step_first"])
def test_single_step_from_oracle_state(gpu, oracle, n, d, k, order):
    torch, binding = gpu
    print(f"step case n={n} d={d} k={k} {order}", flush=True)
    rng = np.random.default_rng(n * 1000 + d + k)
    x0 = rng.standard_normal(d).astype(np.float32)
    g_i0 = rng.standard_normal((n, d)).astype(np.float32)
    g0 = g_i0.astype(np.float64).mean(axis=0).astype(np.float32)
    gamma = 0.25
    st = oracle.EF21State(x0.astype(np.float64), g_i0.astype(np.float64), g0.astype(np.float64))
    budget = RoundingBudget(n, d, gamma)
    with binding.EF21(n, d, k, gamma) as h:
        h.set_state(to_gpu(torch, x0), to_gpu(torch, g_i0), to_gpu(torch, g0))
        for t in range(3):
            grads = (g_i0 + 0.3 * rng.standard_normal((n, d))).astype(np.float32)
            if t == 1:     # exact zeros in the difference: ties at magnitude 0
                grads[:, ::7] = st.g_i[:, ::7].astype(np.float32)
            oracle_step(oracle, st, budget, grads.astype(np.float64), k, gamma, order)
            h.step(to_gpu(torch, grads), binding.ORDER_GRAD_FIRST if order == "grad_first" else binding.ORDER_STEP_FIRST)
            torch.cuda.synchronize()
            x, g_i, g = compare_state(torch, h, st, budget)
            # resynchronise g and x to the oracle's so the next step is again a single-step comparison
            h.set_state(to_gpu(torch, st.x), None, to_gpu(torch, st.g))
            budget.reset()


def test_single_steps_on_random_shapes(gpu, oracle):
    """Thirty seeded draws of (n, d, k) across the kernels' ranges, one step each from a random state with
    supplied gradients: messages and g_i bit for bit, g and x within the rounding budget."""
    torch, binding = gpu
    rng = np.random.default_rng(5203)
    for case in range(30):
        d = int(np.exp(rng.uniform(0.0, np.log(200_000))))
        n = int(rng.integers(1, 24))
        k = int(min(d, max(1, [1, 2, rng.integers(1, 64), d // 100 + 1, d // 3 + 1, d][rng.integers(0, 6)])))
        if n * d > 3_000_000:
            n = max(1, 3_000_000 // d)
        gamma = 0.25
        print(f"random step case {case}: n={n} d={d} k={k}", flush=True)
        x0 = rng.standard_normal(d).astype(np.float32)
        g_i0 = rng.standard_normal((n, d)).astype(np.float32)
        g0 = g_i0.astype(np.float64).mean(axis=0).astype(np.float32)
        grads = (g_i0 + rng.choice([0.0, 0.3], size=(n, d)) * rng.standard_normal((n, d))).astype(np.float32)
        st = oracle.EF21State(x0.astype(np.float64), g_i0.astype(np.float64), g0.astype(np.float64))
        budget = RoundingBudget(n, d, gamma)
        order = "step_first" if case % 3 == 0 else "grad_first"
        with binding.EF21(n, d, k, gamma) as h:
            h.set_state(to_gpu(torch, x0), to_gpu(torch, g_i0), to_gpu(torch, g0))
            oracle_step(oracle, st, budget, grads.astype(np.float64), k, gamma, order)
            h.step(to_gpu(torch, grads), binding.ORDER_STEP_FIRST if order == "step_first" else binding.ORDER_GRAD_FIRST)
            torch.cuda.synchronize()
            compare_state(torch, h, st, budget)


def test_step_sequences_on_random_shapes_and_distributions(gpu, oracle):
    """Sixteen seeded sequences of five steps each on long rows (the candidate path, which remembers the threshold
    from step to step): gradients of different kinds (Gaussian, heavy-tailed, many equal magnitudes, mostly zeros,
    two halves of very different scale, magnitudes in ascending order) whose scale jumps up or down between steps,
    so that the remembered threshold is now right, now too low, now too high.  Messages and g_i bit for bit every
    step, g and x within the rounding budget (resynchronised after each step)."""
    torch, binding = gpu
    rng = np.random.default_rng(2106)
    kinds = ["normal", "student", "ties", "sparse", "halves", "ascending"]
    for case in range(16):
        d = int(rng.integers(*[(16_384, 18_000), (60_000, 70_000), (100_000, 400_000), (900_000, 1_300_000)][case % 4]))
        n = int(rng.integers(1, max(2, min(9, 2_500_000 // d + 1))))
        k = int(max(2, min(d, d * 10 ** rng.uniform(-3.5, -1.0))))
        kind = kinds[case % len(kinds)]
        gamma = 0.25
        print(f"sequence {case}: n={n} d={d} k={k} {kind}", flush=True)
        base = rng.standard_normal((n, d))
        if kind == "student":
            base = base / np.sqrt(rng.chisquare(3, (n, d)) / 3)
        elif kind == "ties":
            base = np.round(base * 2) / 2
        elif kind == "sparse":
            base[rng.random((n, d)) < 0.995] = 0.0
        elif kind == "halves":
            base[:, : d // 2] *= 1e-6
        elif kind == "ascending":
            base = np.sort(np.abs(base), axis=1)
        base = base.astype(np.float32)
        x0 = rng.standard_normal(d).astype(np.float32)
        st = oracle.EF21State(x0.astype(np.float64), np.zeros((n, d)), np.zeros(d))
        budget = RoundingBudget(n, d, gamma)
        scale = 1.0
        with binding.EF21(n, d, k, gamma) as h:
            h.set_state(to_gpu(torch, x0), to_gpu(torch, np.zeros((n, d))), to_gpu(torch, np.zeros(d)))
            for t in range(5):
                scale *= [1.0, 1.05, 3.0, 0.25, 1.0][int(rng.integers(5))]
                noise = 0.3 * rng.standard_normal((n, d)) if kind not in ("ties", "sparse") else 0.0
                grads = ((base + noise) * scale).astype(np.float32)
                oracle_step(oracle, st, budget, grads.astype(np.float64), k, gamma)
                h.step(to_gpu(torch, grads))
                torch.cuda.synchronize()
                compare_state(torch, h, st, budget)
                h.set_state(to_gpu(torch, st.x), None, to_gpu(torch, st.g))
                budget.reset()


@pytest.mark.parametrize("n,d,k", [(16, 20_000, 600), (17, 20_000, 600), (33, 70_001, 1500), (67, 16_500, 300)])
def test_step_with_many_workers_and_clustered_messages(gpu, oracle, n, d, k):
    """Sixteen workers and more take the aggregation that splits the workers over four wavefronts; the large
    differences of every worker sit in a few runs of adjacent coordinates (runs longer than a wavefront inside
    one block of 256 columns, shared by several workers), the rest of the message is scattered."""
    torch, binding = gpu
    print(f"many workers n={n} d={d} k={k}", flush=True)
    rng = np.random.default_rng(n + d + k)
    gamma = 0.25
    x0 = rng.standard_normal(d).astype(np.float32)
    g_i0 = (0.01 * rng.standard_normal((n, d))).astype(np.float32)
    g0 = g_i0.astype(np.float64).mean(axis=0).astype(np.float32)
    grads = (g_i0 + 0.01 * rng.standard_normal((n, d))).astype(np.float32)
    for i in range(n):
        for start in (1000 + 40 * (i % 3), d - 300):              # overlapping runs of 200 and 150 coordinates
            width = 200 if start < d // 2 else 150
            grads[i, start:start + width] += (1.0 + rng.random(width)).astype(np.float32) * (-1.0) ** i
    st = oracle.EF21State(x0.astype(np.float64), g_i0.astype(np.float64), g0.astype(np.float64))
    budget = RoundingBudget(n, d, gamma)
    with binding.EF21(n, d, k, gamma) as h:
        h.set_state(to_gpu(torch, x0), to_gpu(torch, g_i0), to_gpu(torch, g0))
        oracle_step(oracle, st, budget, grads.astype(np.float64), k, gamma)
        h.step(to_gpu(torch, grads))
        torch.cuda.synchronize()
        compare_state(torch, h, st, budget)


@pytest.mark.parametrize("k", [5000, 60000])
def test_step_when_the_sample_misleads(gpu, oracle, k):
    """Long rows whose large differences sit exactly on the sampled pieces: the candidate threshold
    guessed from the sample keeps fewer than k candidates and the exact per-row algorithm takes over,
    inside the step (difference, state update) for the small-k and the large-k candidate stage."""
    torch, binding = gpu
    n, d, gamma = 2, 300_000, 0.25
    print(f"misleading sample step k={k}", flush=True)
    rng = np.random.default_rng(k)
    g_i0 = (rng.standard_normal((n, d)) * 1e-3).astype(np.float32)
    x0 = rng.standard_normal(d).astype(np.float32)
    g0 = g_i0.astype(np.float64).mean(axis=0).astype(np.float32)
    grads = (g_i0 + 1e-3 * rng.standard_normal((n, d))).astype(np.float32)
    pos = sampled_positions(d)
    grads[:, pos] += (1.0 + rng.random((n, pos.size))).astype(np.float32)
    st = oracle.EF21State(x0.astype(np.float64), g_i0.astype(np.float64), g0.astype(np.float64))
    budget = RoundingBudget(n, d, gamma)
    with binding.EF21(n, d, k, gamma) as h:
        h.set_state(to_gpu(torch, x0), to_gpu(torch, g_i0), to_gpu(torch, g0))
        oracle_step(oracle, st, budget, grads.astype(np.float64), k, gamma)
        h.step(to_gpu(torch, grads))
        torch.cuda.synchronize()
        compare_state(torch, h, st, budget)


@pytest.mark.parametrize("k", [3000, 40000])
def test_steps_when_the_remembered_threshold_is_wrong(gpu, oracle, k):
    """Consecutive steps on long rows: from the second step on, the candidates are collected with the previous
    step's threshold as the guess.  The scale of the differences then jumps per row: unchanged (the guess
    holds), up by 300 (the threshold lies far beyond the guess's window), down by 1000 (fewer than k candidates
    reach the guess), back, and finally one row of equal magnitudes (a crowded bin: the exact per-row algorithm).
    Whatever the guess, every step must give the oracle's messages and state bit for bit."""
    torch, binding = gpu
    n, d, gamma = 3, 300_000, 0.25
    print(f"wrong warm start k={k}", flush=True)
    rng = np.random.default_rng(k + 1)
    x0 = rng.standard_normal(d).astype(np.float32)
    g_i0 = rng.standard_normal((n, d)).astype(np.float32)
    g0 = g_i0.astype(np.float64).mean(axis=0).astype(np.float32)
    st = oracle.EF21State(x0.astype(np.float64), g_i0.astype(np.float64), g0.astype(np.float64))
    budget = RoundingBudget(n, d, gamma)
    scales = [(1.0, 1.0, 1.0), (1.01, 0.99, 1.0), (300.0, 1e-3, 1.0), (300.0, 1e-3, 1.05), (1.0, 1.0, 0.93),
              (1e-3, 300.0, 1.0), (1.0, 1.0, 1.0), (1.0, 1.0, 1.0)]
    with binding.EF21(n, d, k, gamma) as h:
        h.set_state(to_gpu(torch, x0), to_gpu(torch, g_i0), to_gpu(torch, g0))
        for t, sc in enumerate(scales):
            noise = rng.standard_normal((n, d)) * np.array(sc)[:, None]
            if t == len(scales) - 1:
                noise[1] = np.where(rng.random(d) < 0.5, 0.5, -0.5)      # every magnitude equal
            grads = (st.g_i + noise).astype(np.float32)
            oracle_step(oracle, st, budget, grads.astype(np.float64), k, gamma)
            h.step(to_gpu(torch, grads))
            torch.cuda.synchronize()
            compare_state(torch, h, st, budget)
            h.set_state(to_gpu(torch, st.x), None, to_gpu(torch, st.g))
            budget.reset()


@pytest.mark.parametrize("kind", ["equal", "distinct"])
def test_step_with_a_crowded_threshold_bin(gpu, oracle, kind):
    """Long rows whose threshold falls into a cluster of thousands of equal (or consecutive) magnitudes, inside the
    step: two steps, so that the second starts from the first one's threshold."""
    torch, binding = gpu
    n, d, k, gamma = 3, 250_000, 3000, 0.25
    print(f"crowded bin step, {kind}", flush=True)
    rng = np.random.default_rng(9)
    x0 = rng.standard_normal(d).astype(np.float32)
    g_i0 = np.zeros((n, d), dtype=np.float32)
    st = oracle.EF21State(x0.astype(np.float64), g_i0.astype(np.float64), np.zeros(d))
    budget = RoundingBudget(n, d, gamma)
    with binding.EF21(n, d, k, gamma) as h:
        h.set_state(to_gpu(torch, x0), to_gpu(torch, g_i0), None)
        for t in range(2):
            noise = 0.1 * rng.standard_normal((n, d))
            for i in range(n):
                pos = rng.choice(d, size=6000, replace=False)
                sign = np.where(rng.random(6000) < 0.5, 1.0, -1.0)
                if kind == "equal":
                    noise[i, pos] = sign
                else:
                    bits = np.float32(1.0).view(np.uint32) + rng.permutation(6000).astype(np.uint32)
                    noise[i, pos] = bits.view(np.float32).astype(np.float64) * sign
            # differences that are exactly the planted values: the state is zero at the planted positions' scale
            grads = (noise + (st.g_i if kind == "equal" and t == 0 else 0.0)).astype(np.float32) if t == 0 else \
                    (st.g_i + noise).astype(np.float32)
            oracle_step(oracle, st, budget, grads.astype(np.float64), k, gamma)
            h.step(to_gpu(torch, grads))
            torch.cuda.synchronize()
            compare_state(torch, h, st, budget)
            h.set_state(to_gpu(torch, st.x), None, to_gpu(torch, st.g))
            budget.reset()


def test_first_pass_compresses_zero_vector(gpu, oracle):
    """g_i^0 = grad: the first grad-first pass sees v = 0; k zero-valued pairs at positions 0..k-1
    are emitted and the state does not change."""
    torch, binding = gpu
    n, d, k = 3, 5000, 50
    rng = np.random.default_rng(0)
    grads = rng.standard_normal((n, d)).astype(np.float32)
    with binding.EF21(n, d, k, 0.5) as h:
        h.set_state(None, to_gpu(torch, grads), None)
        h.step(to_gpu(torch, grads))
        torch.cuda.synchronize()
        idx, val = (t.cpu().numpy() for t in h.get_messages())
        assert np.array_equal(idx, np.tile(np.arange(k, dtype=np.int32), (n, 1)))
        assert np.all(val == 0.0)
        x, g_i, g = (t.cpu().numpy() for t in h.get_state())
        assert same_bits(g_i, grads)
        ok, info = close_per_coordinate(g, grads.astype(np.float64).mean(axis=0))
        assert ok, info


def test_k_equals_d_is_gradient_descent(gpu, oracle):
    torch, binding = gpu
    W = workloads.logreg_dense(n=4, d=64, m=50, seed=3)
    P = oracle.LogRegDense(W.A, W.y, 0.1)
    gamma = 0.5
    x = np.zeros(P.d)
    with binding.EF21(P.n, P.d, P.d, gamma) as h:
        h.set_problem_dense(to_gpu(torch, W.A), to_gpu(torch, W.y), 0.1)
        h.set_state(to_gpu(torch, x), to_gpu(torch, P.grads(x)), None)
        for t in range(20):
            h.step(None, binding.ORDER_STEP_FIRST)
            x = x - gamma * P.grads(x).mean(axis=0)
            torch.cuda.synchronize()
            got = h.get_x().cpu().numpy()
            assert np.max(np.abs(got - x)) <= 2e-6 * max(1.0, np.max(np.abs(x))), t


def run_both(gpu, oracle, P, set_problem, k, gamma, iters, order="grad_first"):
    torch, binding = gpu
    x0 = np.zeros(P.d)
    st = oracle.init_state(x0, P.grads(x0), k, init="grad", storage_f32=True)
    f_ref, f_gpu, first_set_diff = [], [], None
    with binding.EF21(P.n, P.d, k, gamma) as h:
        set_problem(h)
        h.set_state(to_gpu(torch, st.x), to_gpu(torch, st.g_i), to_gpu(torch, st.g))
        flag = binding.ORDER_GRAD_FIRST if order == "grad_first" else binding.ORDER_STEP_FIRST
        for t in range(iters):
            oracle.iteration(st, P.grads, k, gamma, order=order, storage_f32=True)
            h.step(None, flag)
            xg = h.get_x().cpu().numpy().astype(np.float64)
            f_ref.append(P.loss(st.x))
            f_gpu.append(P.loss(xg))
            if first_set_diff is None:
                idx = h.get_messages()[0].cpu().numpy()
                if not np.array_equal(idx, st.msg_idx):
                    first_set_diff = t
        xg, g_i, g = (a.cpu().numpy() for a in h.get_state())
    return np.array(f_ref), np.array(f_gpu), first_set_diff, (xg, g_i, g), st


def test_config0_hundred_steps(gpu, oracle):
    """n = 4, d = 100, m = 250, Top-1, gamma = 0.1, 100 iterations from x = 0, g_i^0 = grad f_i(0):
    f(x^t) on the GPU trajectory within 1e-4 relative of the oracle's at every t."""
    torch, binding = gpu
    c = workloads.CONFIGS["C0"]
    W = workloads.logreg_dense(c["n"], c["d"], c["m"], seed=c["seed"])
    P = oracle.LogRegDense(W.A, W.y, c["lam"])
    A, y = to_gpu(torch, W.A), to_gpu(torch, W.y)
    f_ref, f_gpu, first_diff, (xg, g_i, g), st = run_both(
        gpu, oracle, P, lambda h: h.set_problem_dense(A, y, c["lam"]), c["k"], c["gamma"], c["iters"])
    rel = np.abs(f_gpu - f_ref) / np.abs(f_ref)
    print(f"C0: max rel f diff {rel.max():.3e}, first differing message set at t={first_diff}", flush=True)
    assert rel.max() <= 1e-4
    assert f_ref[-1] < f_ref[0]
    # invariant of Section 3.3 on the GPU state
    assert np.allclose(g, g_i.astype(np.float64).mean(axis=0), rtol=1e-4, atol=1e-7)


def test_dense_medium_run(gpu, oracle):
    """Shape class of config 2 (d = 2000, k = 1 % of d) at a size the oracle runs in seconds."""
    torch, binding = gpu
    W = workloads.logreg_dense(n=6, d=2000, m=300, seed=5)
    P = oracle.LogRegDense(W.A, W.y, 0.1)
    A, y = to_gpu(torch, W.A), to_gpu(torch, W.y)
    f_ref, f_gpu, first_diff, (xg, g_i, g), st = run_both(
        gpu, oracle, P, lambda h: h.set_problem_dense(A, y, 0.1), 20, 0.5, 40)
    rel = np.abs(f_gpu - f_ref) / np.abs(f_ref)
    print(f"dense medium: max rel f diff {rel.max():.3e}, first differing message set at t={first_diff}", flush=True)
    assert rel.max() <= 1e-4
    assert np.allclose(g, g_i.astype(np.float64).mean(axis=0), rtol=1e-4, atol=1e-7)


def test_csr_medium_run(gpu, oracle):
    """Shape class of config 3 (1 % dense CSR rows, k = 1 % of d)."""
    torch, binding = gpu
    W = workloads.logreg_csr(n=8, d=5000, m=300, nnz_per_row=50, seed=6)
    P = oracle.LogRegCSR(W.rowptr, W.col, W.val, W.y, W.n, W.m, W.d, 0.1)
    rp, col, val, y = (to_gpu(torch, W.rowptr, np.int64), to_gpu(torch, W.col, np.int32), to_gpu(torch, W.val),
                       to_gpu(torch, W.y))
    f_ref, f_gpu, first_diff, (xg, g_i, g), st = run_both(
        gpu, oracle, P, lambda h: h.set_problem_csr(rp, col, val, y, W.m, 0.1), 50, 0.5, 40)
    rel = np.abs(f_gpu - f_ref) / np.abs(f_ref)
    print(f"csr medium: max rel f diff {rel.max():.3e}, first differing message set at t={first_diff}", flush=True)
    assert rel.max() <= 1e-4
    assert np.allclose(g, g_i.astype(np.float64).mean(axis=0), rtol=1e-4, atol=1e-7)


def test_config4_scaled_run(gpu, oracle):
    """Config 4 at d/100 (n = 8, d = 112000, k = 1120, gamma = 0.01), all 200 iterations with fresh
    Student-t gradients each step, from the zero state: messages and g_i bit-exact throughout."""
    torch, binding = gpu
    n, d, k, gamma = 8, 112_000, 1120, 0.01
    st = oracle.EF21State(np.zeros(d), np.zeros((n, d)), np.zeros(d))
    budget = RoundingBudget(n, d, gamma)
    with binding.EF21(n, d, k, gamma) as h:
        for t in range(200):
            grads = workloads.student_t_grads(n, d, seed=1000 + t)
            oracle_step(oracle, st, budget, grads.astype(np.float64), k, gamma)
            h.step(to_gpu(torch, grads))
            if t % 20 == 19 or t < 3:
                torch.cuda.synchronize()
                compare_state(torch, h, st, budget)
        torch.cuda.synchronize()
        compare_state(torch, h, st, budget)


@pytest.mark.timeout(600)
def test_config4_full_size_step(gpu, oracle):
    """Config 4 at full size (n = 8, d = 11.2e6, k = 112000): two steps.  First step (threshold from the sample):
    the messages and g_i rows of all eight workers one by one against the oracle.  Second step (threshold guessed
    from the first step's): three workers one by one, the rest through invariants."""
    torch, binding = gpu
    c = workloads.CONFIGS["C4"]
    n, d, k, gamma = c["n"], c["d"], c["k"], c["gamma"]
    rows = [0, 3, 7]
    g_i_ref = np.zeros((n, d), dtype=np.float32)
    budget, line6, g_prev = RoundingBudget(n, d, gamma), np.zeros(d), np.zeros(d)
    with binding.EF21(n, d, k, gamma) as h:
        for t in range(2):
            print(f"C4 full size step {t}", flush=True)
            grads = workloads.student_t_grads(n, d, seed=7 + t)
            h.step(to_gpu(torch, grads))
            torch.cuda.synchronize()
            idx, val = (a.cpu().numpy() for a in h.get_messages())
            x, g_i, g = (a.cpu().numpy() for a in h.get_state())
            for i in (range(n) if t == 0 else rows):
                v = grads[i] - g_i_ref[i]                       # fp32 subtraction, as in line 5
                ref_idx, ref_val = oracle.topk(v.astype(np.float64), k)
                assert np.array_equal(idx[i], ref_idx), f"step {t} worker {i}"
                assert same_bits(val[i], ref_val.astype(np.float32))
            # every worker: k ascending positions, values are the differences, g_i updated there only
            assert np.all(np.diff(idx.astype(np.int64), axis=1) > 0)
            v_all = grads - g_i_ref
            assert same_bits(val, np.take_along_axis(v_all, idx.astype(np.int64), axis=1))
            thr = np.abs(val).min(axis=1)
            for i in range(n):
                expect = g_i_ref[i].copy()
                expect[idx[i]] = g_i_ref[i][idx[i]] + val[i]
                assert same_bits(g_i[i], expect)
                dropped = np.ones(d, dtype=bool)
                dropped[idx[i]] = False
                assert np.abs(v_all[i][dropped]).max() <= thr[i]
            g_i_ref = g_i
            # invariant g = mean_i g_i up to the fp32 roundings made so far: those of line 8
            # (budget.g) and those of line 6 (one per kept entry, relative to the new g_i)
            budget.compress_update(g_prev, idx, val)
            line6 += 2.0 ** -24 * np.abs(g_i).astype(np.float64).mean(axis=0)
            mean = g_i.astype(np.float64).mean(axis=0)
            assert np.all(np.abs(g - mean) <= 1e-5 * np.abs(mean) + budget.g + line6)
            g_prev = g.astype(np.float64)


@pytest.mark.timeout(400)
@pytest.mark.parametrize("order", ["grad_first", "step_first"])
def test_config3_shape_single_steps(gpu, oracle, order):
    """Exactly the shape of config 3's Top-k and update (n = 100, d = 50 000, k = 500), gradients supplied: two
    consecutive steps element by element (the second collects with the first one's threshold as the guess)."""
    torch, binding = gpu
    c = workloads.CONFIGS["C3"]
    n, d, k, gamma = c["n"], c["d"], c["k"], c["gamma"]
    print(f"C3 shape single steps {order}", flush=True)
    rng = np.random.default_rng(33)
    x0 = rng.standard_normal(d).astype(np.float32)
    g_i0 = (0.1 * rng.standard_normal((n, d))).astype(np.float32)
    g0 = g_i0.astype(np.float64).mean(axis=0).astype(np.float32)
    st = oracle.EF21State(x0.astype(np.float64), g_i0.astype(np.float64), g0.astype(np.float64))
    budget = RoundingBudget(n, d, gamma)
    with binding.EF21(n, d, k, gamma) as h:
        h.set_state(to_gpu(torch, x0), to_gpu(torch, g_i0), to_gpu(torch, g0))
        for t in range(2):
            grads = (st.g_i + 0.1 * rng.standard_normal((n, d)) * rng.choice([0.2, 1.0, 3.0], size=(n, 1))).astype(np.float32)
            oracle_step(oracle, st, budget, grads.astype(np.float64), k, gamma, order)
            h.step(to_gpu(torch, grads), binding.ORDER_GRAD_FIRST if order == "grad_first" else binding.ORDER_STEP_FIRST)
            torch.cuda.synchronize()
            compare_state(torch, h, st, budget)
            h.set_state(to_gpu(torch, st.x), None, to_gpu(torch, st.g))
            budget.reset()


@pytest.mark.timeout(400)
def test_config3_shape_step_with_internal_csr_gradient(gpu, oracle):
    """ef21_step(NULL) on a CSR problem of config 3's shape (n = 100, d = 50 000, k = 500, 500 entries per row; 120
    rows per worker so that the oracle finishes in seconds).  The library's gradients of sampled workers against
    the oracle's (1e-5 and the rounding floor); then, because the last bits of a gradient may move a near-tie, the
    step itself against the oracle's lines 5, 6, 8, 3 applied to the library's own gradients: every worker's
    message and g_i row bit for bit, g and x within the budget."""
    from helpers import gradient_rounding_floor
    torch, binding = gpu
    c = workloads.CONFIGS["C3"]
    n, d, k, gamma, m, nnz = c["n"], c["d"], c["k"], c["gamma"], 120, c["nnz_per_row"]
    print("C3 shape step with CSR gradients", flush=True)
    W = workloads.logreg_csr(n, d, m, nnz, seed=11)
    P = oracle.LogRegCSR(W.rowptr, W.col, W.val, W.y, n, m, d, c["lam"])
    rng = np.random.default_rng(12)
    x0 = (0.3 * rng.standard_normal(d)).astype(np.float32)
    g_i0 = (1e-3 * rng.standard_normal((n, d))).astype(np.float32)
    g0 = g_i0.astype(np.float64).mean(axis=0).astype(np.float32)
    st = oracle.EF21State(x0.astype(np.float64), g_i0.astype(np.float64), g0.astype(np.float64))
    budget = RoundingBudget(n, d, gamma)
    import scipy.sparse as sp
    with binding.EF21(n, d, k, gamma) as h:
        h.set_problem_csr(to_gpu(torch, W.rowptr, np.int64), to_gpu(torch, W.col, np.int32), to_gpu(torch, W.val),
                          to_gpu(torch, W.y), m, c["lam"])
        h.set_state(to_gpu(torch, x0), to_gpu(torch, g_i0), to_gpu(torch, g0))
        for t in range(2):
            x_now = h.get_x()
            grads = h.local_grad(x_now).cpu().numpy()
            for i in (0, 37, 99):
                ref = P.grad_i(i, x_now.cpu().numpy().astype(np.float64))
                A_i = sp.csr_matrix((W.val[W.rowptr[i * m]:W.rowptr[(i + 1) * m]],
                                     W.col[W.rowptr[i * m]:W.rowptr[(i + 1) * m]],
                                     W.rowptr[i * m:(i + 1) * m + 1] - W.rowptr[i * m]), shape=(m, d))
                bound = 1e-5 * np.abs(ref) + gradient_rounding_floor(A_i, W.y[i], x_now.cpu().numpy(), nnz / 64 + 8, 64,
                                                                     c["lam"])
                assert np.all(np.abs(grads[i] - ref) <= bound), f"step {t}: gradient of worker {i}"
            oracle_step(oracle, st, budget, grads.astype(np.float64), k, gamma)
            h.step()
            torch.cuda.synchronize()
            compare_state(torch, h, st, budget)
            h.set_state(to_gpu(torch, st.x), None, to_gpu(torch, st.g))
            budget.reset()


@pytest.mark.timeout(400)
def test_config2_full_size_steps(gpu, oracle):
    """Config 2 at full size, the launch configuration bench.py times: five iterations with the
    library's own gradients against the oracle's: f(x^t) within 1e-4, the invariant g = mean g_i."""
    torch, binding = gpu
    c = workloads.CONFIGS["C2"]
    print("C2 full size steps", flush=True)
    W = workloads.logreg_dense(c["n"], c["d"], c["m"], seed=c["seed"])
    P = oracle.LogRegDense(W.A, W.y, c["lam"])
    A, y = to_gpu(torch, W.A), to_gpu(torch, W.y)
    f_ref, f_gpu, first_diff, (x, g_i, g), st = run_both(
        gpu, oracle, P, lambda h: h.set_problem_dense(A, y, c["lam"]), c["k"], c["gamma"], 5)
    assert np.all(np.abs(f_gpu - f_ref) <= 1e-4 * np.abs(f_ref)), (f_ref, f_gpu, first_diff)
    mean = g_i.astype(np.float64).mean(axis=0)
    assert np.all(np.abs(g - mean) <= 1e-5 * np.abs(mean) + 1e-6 * np.abs(mean).max())


@pytest.mark.timeout(600)
def test_config3_full_size_steps(gpu, oracle):
    """Config 3 at full size (CSR, 10^8 non-zeros, long-row Top-k with k = 500): three iterations."""
    torch, binding = gpu
    c = workloads.CONFIGS["C3"]
    n, d, m = c["n"], c["d"], c["m"]
    print("C3 full size steps", flush=True)
    W = workloads.logreg_csr(n, d, m, c["nnz_per_row"], seed=c["seed"])
    P = oracle.LogRegCSR(W.rowptr, W.col, W.val, W.y, n, m, d, c["lam"])
    rp, col, val, y = (to_gpu(torch, W.rowptr, np.int64), to_gpu(torch, W.col, np.int32), to_gpu(torch, W.val),
                       to_gpu(torch, W.y))
    f_ref, f_gpu, first_diff, (x, g_i, g), st = run_both(
        gpu, oracle, P, lambda h: h.set_problem_csr(rp, col, val, y, m, c["lam"]), c["k"], c["gamma"], 3)
    assert np.all(np.abs(f_gpu - f_ref) <= 1e-4 * np.abs(f_ref)), (f_ref, f_gpu, first_diff)
    mean = g_i.astype(np.float64).mean(axis=0)
    assert np.all(np.abs(g - mean) <= 1e-5 * np.abs(mean) + 1e-6 * np.abs(mean).max())


@pytest.mark.parametrize("n,d,m,k", [(5, 2000, 120, 20), (3, 99, 64, 7), (2, 8192, 40, 100), (2, 8200, 40, 100)])
def test_step_with_internal_gradient_equals_supplied_gradient(gpu, n, d, m, k):
    """ef21_step(NULL) computes the dense gradient itself; the result must be bit for bit what
    ef21_local_grad followed by ef21_step(grads) gives."""
    torch, binding = gpu
    W = workloads.logreg_dense(n, d, m, seed=d)
    A, y = to_gpu(torch, W.A), to_gpu(torch, W.y)
    x0 = torch.randn(d, device="cuda") * 0.3
    g_i0 = torch.randn(n, d, device="cuda") * 0.01
    with binding.EF21(n, d, k, 0.5) as h1, binding.EF21(n, d, k, 0.5) as h2:
        for h in (h1, h2):
            h.set_problem_dense(A, y, 0.1)
            h.set_state(x0, g_i0, None)
        for t in range(4):
            h1.step(None)
            h2.step(h2.local_grad())
            torch.cuda.synchronize()
            for a, b in zip(h1.get_state() + h1.get_messages(), h2.get_state() + h2.get_messages()):
                assert torch.equal(a.view(torch.int32), b.view(torch.int32)), t


def test_get_set_state_roundtrip_and_errors(gpu):
    torch, binding = gpu
    with binding.EF21(3, 17, 4, 0.1) as h:
        x = torch.randn(17, device="cuda")
        g_i = torch.randn(3, 17, device="cuda")
        h.set_state(x, g_i, None)
        x2, g_i2, g2 = h.get_state()
        torch.cuda.synchronize()
        assert torch.equal(x, x2) and torch.equal(g_i, g_i2)
        assert torch.allclose(g2, g_i.double().mean(0).float(), rtol=1e-6, atol=1e-7)
        with pytest.raises(binding.EF21Error) as e:
            h.step(None)                       # no problem attached
        assert e.value.code == binding.EF21_ESTATE
        with pytest.raises(binding.EF21Error) as e:
            h.local_grad()
        assert e.value.code == binding.EF21_ESTATE
        with pytest.raises(ValueError):
            h.step(torch.zeros(2, 17, device="cuda"))
    for bad in [(0, 5, 1, 0.1), (2, 5, 6, 0.1), (2, 5, 1, -1.0)]:
        with pytest.raises(binding.EF21Error):
            binding.EF21(*bad)


@pytest.mark.parametrize("case", ["dense_problem", "long_rows_large_k", "long_rows_small_k"])
def test_step_replayed_from_a_hip_graph(gpu, case):
    """ef21_step only enqueues kernels (no allocation, no memset, no host wait once the handle is warm), so
    a caller may capture it into a HIP graph.  Every replay, with eager work and synchronisations in
    between, must leave exactly the state that an eager handle has after the same number of steps."""
    torch, binding = gpu
    rng = np.random.default_rng(5)
    if case == "dense_problem":
        c = workloads.CONFIGS["C0"]
        n, d, k, gamma = c["n"], c["d"], c["k"], c["gamma"]
        W = workloads.logreg_dense(n, d, c["m"], seed=1)
        A, y = to_gpu(torch, W.A), to_gpu(torch, W.y)
        grads = None
    else:
        n, d, gamma = 3, 200_000, 0.1
        k = 40_000 if case == "long_rows_large_k" else 300
        grads = to_gpu(torch, rng.standard_normal((n, d)).astype(np.float32))

    def fresh():
        h = binding.EF21(n, d, k, gamma)
        if grads is None:
            h.set_problem_dense(A, y, 0.1)
            x0 = torch.zeros(d, device="cuda")
            h.set_state(x0, h.local_grad(x0), None)
        return h

    side = torch.cuda.Stream()
    with fresh() as eager, fresh() as replayed:
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            replayed.use_current_stream()
            replayed.step(grads)                       # warm-up: buffers and kernel attributes exist afterwards
            side.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                replayed.step(grads)
        eager.step(grads)
        torch.cuda.synchronize()
        for r in range(4):
            graph.replay()
            eager.step(grads)
            torch.cuda.synchronize()
            scratch = torch.randn(1000, device="cuda").sum().item()      # unrelated eager work between replays
            assert np.isfinite(scratch)
            got = replayed.get_state() + replayed.get_messages()     # copies on each handle's own stream
            ref = eager.get_state() + eager.get_messages()
            torch.cuda.synchronize()
            for a, b, name in zip(got, ref, ("x", "g_i", "g", "message positions", "message values")):
                assert torch.equal(a, b), f"replay {r}: {name} differ from the eager handle"
