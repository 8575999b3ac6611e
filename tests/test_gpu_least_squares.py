"""GPU parity of the least-squares objective (Section 5.2; ef21_set_loss) against the CPU oracle: gradients
within 1e-5 relative per coordinate plus the first-order rounding floor of the fp32 sums, and an EF21 run
through f(x^t) (1e-4)."""
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


def ls_rounding_floor(A, b, x, dot_depth, sum_depth):
    """First-order bound on what fp32 rounding does to (2/m) A^T (A x - b): the dot products carry
    dot_depth * u * sum_j |a_lj x_j|, the subtraction u (|z_l| + |b_l|), the sum over rows sum_depth * u per term."""
    u = 2.0 ** -24
    A = np.asarray(A, dtype=np.float64)
    z = A @ x
    dr = 2.0 * (dot_depth * u * (np.abs(A) @ np.abs(x)) + 2 * u * (np.abs(z) + np.abs(b))) + sum_depth * u * 2.0 * np.abs(z - b)
    return (np.abs(A).T @ dr) / A.shape[0]


def assert_ls_grads_close(got, ref, A, b, x, dot_depth, sum_depth, what):
    for i in range(ref.shape[0]):
        bound = 1e-5 * np.abs(ref[i]) + ls_rounding_floor(A[i], b[i].astype(np.float64), x.astype(np.float64), dot_depth, sum_depth)
        err = np.abs(got[i].astype(np.float64) - ref[i])
        assert np.all(err <= bound), f"{what}, worker {i}: max err {err.max():.3e}, {int((err > bound).sum())} bad"
        # the residuals cancel in A^T r, so the floor is larger against the gradient than for the logistic loss
        assert np.median(bound) <= 1e-3 * np.max(np.abs(ref[i])), f"{what}: tolerance too loose"


@pytest.mark.parametrize("n,d,m", [(4, 100, 250), (3, 256, 37), (2, 333, 41), (5, 2000, 301), (2, 4100, 29), (1, 1, 1)])
def test_dense_gradient(gpu, oracle, n, d, m):
    torch, binding = gpu
    print(f"least squares dense grad n={n} d={d} m={m}", flush=True)
    rng = np.random.default_rng(d + m)
    A = (rng.standard_normal((n, m, d)) / np.sqrt(d)).astype(np.float32)
    b = np.where(rng.random((n, m)) < 0.5, 1.0, -1.0).astype(np.float32)       # the paper's targets are labels
    P = oracle.LeastSquaresDense(A, b)
    with binding.EF21(n, d, 1, 0.1) as h:
        h.set_problem_dense(to_gpu(torch, A), to_gpu(torch, b), 0.0)
        h.set_loss(binding.LOSS_LEAST_SQUARES)
        for scale in (0.0, 1.0, 4.0):
            x = (rng.standard_normal(d) * scale).astype(np.float32)
            got = h.local_grad(to_gpu(torch, x))
            torch.cuda.synchronize()
            assert_ls_grads_close(got.cpu().numpy(), P.grads(x.astype(np.float64)), A, b, x, d / 64 + 8, 16, f"scale {scale}")
        # and back to the logistic loss on the same handle
        h.set_loss(binding.LOSS_LOGISTIC)
        Pl = oracle.LogRegDense(A, b, 0.0)
        x = rng.standard_normal(d).astype(np.float32)
        got = h.local_grad(to_gpu(torch, x)).cpu().numpy()
        ref = Pl.grads(x.astype(np.float64))
        assert np.all(np.abs(got - ref) <= 1e-4 * np.abs(ref).max())


def test_csr_gradient(gpu, oracle):
    torch, binding = gpu
    n, d, m, nnz = 3, 20_000, 120, 60
    W = workloads.logreg_csr(n, d, m, nnz, seed=5)
    D = oracle.densify_csr(W.rowptr, W.col, W.val, n, m, d)
    P = oracle.LeastSquaresDense(D, W.y)
    rng = np.random.default_rng(6)
    x = rng.standard_normal(d).astype(np.float32)
    with binding.EF21(n, d, 1, 0.1) as h:
        h.set_problem_csr(to_gpu(torch, W.rowptr, np.int64), to_gpu(torch, W.col, np.int32), to_gpu(torch, W.val),
                          to_gpu(torch, W.y), m, 0.0)
        h.set_loss(binding.LOSS_LEAST_SQUARES)
        got = h.local_grad(to_gpu(torch, x))
        torch.cuda.synchronize()
    assert_ls_grads_close(got.cpu().numpy(), P.grads(x.astype(np.float64)), D, W.y, x, 128 + 8, 64, "csr")


def test_ef21_run_on_least_squares(gpu, oracle):
    """Sixty EF21 iterations (k = 2 of d = 100) on a least-squares problem: f(x^t) within 1e-4 of the oracle's."""
    torch, binding = gpu
    rng = np.random.default_rng(7)
    n, d, m, k = 4, 100, 250, 2
    A = (rng.standard_normal((n, m, d)) / np.sqrt(d)).astype(np.float32)
    w = rng.standard_normal(d)
    b = (A.astype(np.float64) @ w + 0.1 * rng.standard_normal((n, m))).astype(np.float32)
    P = oracle.LeastSquaresDense(A, b)
    gamma = float(np.float32(0.25))
    x0 = np.zeros(d)
    st = oracle.init_state(x0, P.grads(x0), k, init="grad", storage_f32=True)
    with binding.EF21(n, d, k, gamma) as h:
        h.set_problem_dense(to_gpu(torch, A), to_gpu(torch, b), 0.0)
        h.set_loss(binding.LOSS_LEAST_SQUARES)
        h.set_state(to_gpu(torch, st.x), to_gpu(torch, st.g_i), to_gpu(torch, st.g))
        f0 = P.loss(x0)
        for t in range(60):
            oracle.iteration(st, P.grads, k, gamma)
            h.step()
            f_ref, f_gpu = P.loss(st.x), P.loss(h.get_x().cpu().numpy().astype(np.float64))
            assert abs(f_gpu - f_ref) <= 1e-4 * abs(f_ref), f"iteration {t}: {f_gpu} vs {f_ref}"
    assert f_ref < 0.7 * f0, "the run should make progress"


def test_unknown_loss_is_rejected(gpu):
    torch, binding = gpu
    with binding.EF21(2, 10, 3, 0.1) as h:
        with pytest.raises(binding.EF21Error):
            h.set_loss(7)
