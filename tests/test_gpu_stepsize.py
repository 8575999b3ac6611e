"""GPU parity of ef21_theory_stepsize against the oracle's exact eigenvalues: the power iteration approaches
every smoothness constant from below, to 1e-4 where the matrix has a dominant direction and to two per cent
on matrices without one (the gap of a random matrix's top eigenvalues is small), and the stepsize follows."""
import numpy as np
import pytest

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


def check(got, exact, below, what):
    got, exact = np.asarray(got), np.asarray(exact)
    assert np.all(got <= exact * (1 + 2e-6)), f"{what}: an estimate above the eigenvalue: {got} vs {exact}"
    assert np.all(got >= exact * (1 - below)), f"{what}: {got} vs {exact}"


@pytest.mark.parametrize("n,d,m,k", [(4, 100, 250, 3), (3, 333, 41, 10), (2, 4100, 29, 41)])
@pytest.mark.parametrize("loss", ["logistic", "squares"])
def test_dense_with_a_dominant_direction(gpu, oracle, n, d, m, k, loss):
    """Rows with a common offset (non-negative features, as in the paper's data sets) have one large eigenvalue."""
    torch, binding = gpu
    print(f"stepsize dense n={n} d={d} m={m} {loss}", flush=True)
    rng = np.random.default_rng(d)
    A = (rng.standard_normal((n, m, d)) / np.sqrt(d) + 0.5 * rng.random((n, 1, d)) / np.sqrt(d)).astype(np.float32)
    A *= np.linspace(0.5, 2.0, n)[:, None, None].astype(np.float32)          # workers of different scale
    t = np.where(rng.random((n, m)) < 0.5, 1.0, -1.0).astype(np.float32)
    lam = 0.1
    P = oracle.LeastSquaresDense(A, t, lam) if loss == "squares" else oracle.LogRegDense(A, t, lam)
    L_i = oracle.smoothness_constants(P)
    with binding.EF21(n, d, k, 0.1) as h:
        h.set_problem_dense(to_gpu(torch, A), to_gpu(torch, t), lam)
        if loss == "squares":
            h.set_loss(binding.LOSS_LEAST_SQUARES)
        gamma, L, got_i = h.theory_stepsize(150)
    check(got_i, L_i, 1e-4, "L_i")
    L_exact = oracle.smoothness_constant_of_f(P)
    check([L], [L_exact], 1e-4, "L")
    ref = oracle.theory_stepsize(L_i, k / d, L=L_exact)
    assert ref * (1 - 2e-6) <= gamma <= ref * (1 + 2e-4)
    assert L <= np.mean(got_i) * (1 + 1e-6)                      # the remark before Theorem 1: L <= mean L_i


def test_dense_without_a_dominant_direction(gpu, oracle):
    torch, binding = gpu
    n, d, m, k = 3, 200, 500, 2
    W = workloads.logreg_dense(n, d, m, seed=3)
    P = oracle.LogRegDense(W.A, W.y, 0.1)
    L_i = oracle.smoothness_constants(P)
    with binding.EF21(n, d, k, 0.1) as h:
        h.set_problem_dense(to_gpu(torch, W.A), to_gpu(torch, W.y), 0.1)
        few = h.theory_stepsize(5)
        many = h.theory_stepsize(300)
    check(many[2], L_i, 2e-2, "L_i after 300 steps")
    check(few[2], L_i, 0.6, "L_i after 5 steps")
    assert np.all(np.asarray(few[2]) <= np.asarray(many[2]) * (1 + 1e-6))     # the estimate grows with the steps
    ref = oracle.theory_stepsize(L_i, k / d, L=oracle.smoothness_constant_of_f(P))
    assert ref * (1 - 2e-6) <= many[0] <= ref * 1.03


@pytest.mark.parametrize("sorted_cols", [True, False])
def test_csr(gpu, oracle, sorted_cols):
    torch, binding = gpu
    n, d, m, nnz, k = 3, 3000, 150, 40, 30
    W = workloads.logreg_csr(n, d, m, nnz, seed=4)
    col, val = np.array(W.col), np.abs(np.array(W.val))           # non-negative features: a dominant direction
    if not sorted_cols:
        for r in range(n * m):
            s, e = W.rowptr[r], W.rowptr[r + 1]
            col[s:e], val[s:e] = col[s:e][::-1].copy(), val[s:e][::-1].copy()
    P = oracle.LogRegCSR(W.rowptr, col, val, W.y, n, m, d, 0.05)
    L_i = oracle.smoothness_constants(P)
    with binding.EF21(n, d, k, 0.1) as h:
        h.set_problem_csr(to_gpu(torch, W.rowptr, np.int64), to_gpu(torch, col, np.int32), to_gpu(torch, val),
                          to_gpu(torch, W.y), m, 0.05)
        gamma, L, got_i = h.theory_stepsize(200)
    check(got_i, L_i, 1e-3, "L_i")
    L_exact = oracle.smoothness_constant_of_f(P)
    check([L], [L_exact], 1e-3, "L")
    ref = oracle.theory_stepsize(L_i, k / d, L=L_exact)
    assert ref * (1 - 2e-6) <= gamma <= ref * (1 + 2e-3)


def test_stepsize_runs_ef21_downhill(gpu, oracle):
    """EF21 with the stepsize the library computes: f decreases along the run, as Theorem 1's proof shows for the
    Lyapunov function; here checked on f at the end against the start."""
    torch, binding = gpu
    n, d, m, k = 4, 100, 250, 2
    W = workloads.logreg_dense(n, d, m, seed=5)
    P = oracle.LogRegDense(W.A, W.y, 0.1)
    with binding.EF21(n, d, k, 0.1) as probe:
        probe.set_problem_dense(to_gpu(torch, W.A), to_gpu(torch, W.y), 0.1)
        gamma = probe.theory_stepsize(300)[0]
    x0 = np.random.default_rng(6).standard_normal(d).astype(np.float32)
    with binding.EF21(n, d, k, gamma) as h:
        h.set_problem_dense(to_gpu(torch, W.A), to_gpu(torch, W.y), 0.1)
        x0g = to_gpu(torch, x0)
        h.set_state(x0g, h.local_grad(x0g), None)
        for _ in range(200):
            h.step()
        assert P.loss(h.get_x().cpu().numpy().astype(np.float64)) < P.loss(x0.astype(np.float64))


def test_argument_errors(gpu):
    torch, binding = gpu
    with binding.EF21(2, 16, 2, 0.1) as h:
        with pytest.raises(binding.EF21Error):
            h.theory_stepsize(10)                                 # no problem
        A = torch.ones((2, 5, 16), device="cuda")
        h.set_problem_dense(A, torch.ones((2, 5), device="cuda"), 0.0)
        with pytest.raises(binding.EF21Error):
            h.theory_stepsize(0)
        gamma, L, L_i = h.theory_stepsize(3)                      # rank one: lambda_max = |a|^2 = 16 exactly
        assert L_i == pytest.approx([4.0, 4.0], rel=1e-6) and L == pytest.approx(4.0, rel=1e-6)
