"""GPU parity of the local gradients (ef21_local_grad through the C ABI) against the CPU oracle:
1e-5 relative per coordinate (fp32 kernels, fp64 oracle) plus the first-order rounding floor of the
fp32 sums (helpers.gradient_rounding_floor), which matters only where a coordinate cancels."""
import numpy as np
import pytest

from helpers import gradient_rounding_floor
from paper_2106_05203_amd import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    from paper_2106_05203_amd import binding
    assert torch.cuda.is_available(), "these tests need the MI355X"
    binding.load_library()
    return torch, binding


GUARD = 2e-5    # the median allowance of a gradient entry, as a share of the gradient's largest entry


def to_gpu(torch, a, dtype=np.float32):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=dtype)).cuda()


def assert_grads_close(got, ref, A_dense, y, x, dot_depth, sum_depth, what):
    """got, ref: [n][d]; A_dense: [n][m][d]."""
    for i in range(ref.shape[0]):
        bound = 1e-5 * np.abs(ref[i]) + gradient_rounding_floor(A_dense[i], y[i], x, dot_depth, sum_depth)
        err = np.abs(got[i].astype(np.float64) - ref[i])
        assert np.all(err <= bound), f"{what}, worker {i}: max err {err.max():.3e}, {int((err > bound).sum())} bad"
        # the floor must stay a floor: tiny next to the gradient's scale
        loose = np.median(bound) / np.max(np.abs(ref[i]))
        print(f"  {what}, worker {i}: worst coordinate uses {np.max(err / np.maximum(bound, 1e-300)):.3f} of its allowance; "
              f"median allowance {loose:.2e} of the largest entry", flush=True)
        assert loose <= GUARD, f"{what}: tolerance too loose"


def densify(W):
    D = np.zeros((W.n * W.m, W.d), np.float32)
    for r in range(W.n * W.m):
        s, e = W.rowptr[r], W.rowptr[r + 1]
        D[r, W.col[s:e]] = W.val[s:e]
    return D.reshape(W.n, W.m, W.d)


# d: vector path (d % 4 == 0) at each register tiling, scalar path, two-pass path for long rows
@pytest.mark.parametrize("n,d,m", [(4, 100, 250), (3, 256, 37), (2, 260, 64), (3, 1000, 130), (5, 2000, 301),
                                   (2, 4096, 50), (3, 99, 70), (2, 333, 41), (2, 2047, 33), (2, 4100, 29),
                                   (2, 6001, 21), (1, 1, 1)])
def test_dense_gradient(gpu, oracle, n, d, m):
    torch, binding = gpu
    print(f"dense grad case n={n} d={d} m={m}", flush=True)
    W = workloads.logreg_dense(n, d, m, seed=d + m)
    P = oracle.LogRegDense(W.A, W.y, 0.1)
    rng = np.random.default_rng(1)
    with binding.EF21(n, d, 1, 0.1) as h:
        h.set_problem_dense(to_gpu(torch, W.A), to_gpu(torch, W.y), 0.1)
        for scale in (0.0, 1.0, 8.0):
            x = (rng.standard_normal(d) * scale).astype(np.float32)
            got = h.local_grad(to_gpu(torch, x))
            again = h.local_grad(to_gpu(torch, x))
            torch.cuda.synchronize()
            ref = P.grads(x.astype(np.float64))
            assert_grads_close(got.cpu().numpy(), ref, W.A, W.y, x, d / 64 + 8, 16, f"scale {scale}")
            assert torch.equal(got, again), "the dense gradient is bitwise reproducible"
        # x = NULL uses the handle's iterate
        h.set_state(to_gpu(torch, x), None, None)
        assert torch.equal(h.local_grad(), got)


@pytest.mark.parametrize("n,d,m,nnz", [(3, 64, 30, 7), (4, 5000, 200, 50), (2, 50_000, 100, 500), (2, 1000, 40, 130)])
def test_csr_gradient(gpu, oracle, n, d, m, nnz):
    torch, binding = gpu
    print(f"csr grad case n={n} d={d} m={m} nnz/row={nnz}", flush=True)
    W = workloads.logreg_csr(n, d, m, nnz, seed=d + nnz)
    P = oracle.LogRegCSR(W.rowptr, W.col, W.val, W.y, n, m, d, 0.1)
    D = densify(W)
    rng = np.random.default_rng(2)
    with binding.EF21(n, d, 1, 0.1) as h:
        h.set_problem_csr(to_gpu(torch, W.rowptr, np.int64), to_gpu(torch, W.col, np.int32), to_gpu(torch, W.val),
                          to_gpu(torch, W.y), m, 0.1)
        for scale in (0.0, 1.0, 4.0):
            x = (rng.standard_normal(d) * scale).astype(np.float32)
            got = h.local_grad(to_gpu(torch, x))
            torch.cuda.synchronize()
            assert_grads_close(got.cpu().numpy(), P.grads(x.astype(np.float64)), D, W.y, x, nnz / 64 + 8, 32,
                               f"scale {scale}")


def test_csr_ragged_rows(gpu, oracle):
    """Rows of different lengths, empty rows included."""
    torch, binding = gpu
    rng = np.random.default_rng(4)
    n, m, d = 3, 50, 300
    lens = rng.integers(0, 200, size=n * m)
    lens[::9] = 0
    rowptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    col = np.concatenate([np.sort(rng.choice(d, size=L, replace=False)) for L in lens]).astype(np.int32)
    val = rng.random(col.size).astype(np.float32)
    y = np.where(rng.random((n, m)) < 0.5, 1.0, -1.0).astype(np.float32)
    P = oracle.LogRegCSR(rowptr, col, val, y, n, m, d, 0.1)
    x = rng.standard_normal(d).astype(np.float32)
    with binding.EF21(n, d, 1, 0.1) as h:
        h.set_problem_csr(to_gpu(torch, rowptr, np.int64), to_gpu(torch, col, np.int32), to_gpu(torch, val),
                          to_gpu(torch, y), m, 0.1)
        got = h.local_grad(to_gpu(torch, x))
        torch.cuda.synchronize()
    D = np.zeros((n * m, d), np.float32)
    for r in range(n * m):
        D[r, col[rowptr[r]:rowptr[r + 1]]] = val[rowptr[r]:rowptr[r + 1]]
    assert_grads_close(got.cpu().numpy(), P.grads(x.astype(np.float64)), D.reshape(n, m, d), y, x, 200 / 64 + 8, 64,
                       "ragged")


@pytest.mark.parametrize("n,m,d,always,extra", [(2, 1500, 200, (0, 5, 199), 6), (1, 17000, 70, (1,), 3),
                                                (3, 100, 13000, (12287, 12288), 40), (1, 70000, 70, (69,), 2)])
def test_csr_long_columns_many_rows(gpu, oracle, n, m, d, always, extra):
    """Columns present in every row (pieces of a column longer than a staging tile, summed by the whole
    wavefront), more rows per worker than the in-LDS coefficient vector holds, more than 16-bit row
    indices hold, columns next to a range boundary; and the sorted-CSR gradient is bitwise reproducible."""
    torch, binding = gpu
    print(f"csr long columns case n={n} m={m} d={d}", flush=True)
    rng = np.random.default_rng(m + d)
    others = np.setdiff1d(np.arange(d), np.array(always))
    rows = [np.sort(np.concatenate([np.array(always), rng.choice(others, size=extra, replace=False)]))
            for _ in range(n * m)]
    per = len(always) + extra
    rowptr = (np.arange(n * m + 1) * per).astype(np.int64)
    col = np.concatenate(rows).astype(np.int32)
    val = (rng.random(col.size) * 2 - 0.5).astype(np.float32)
    y = np.where(rng.random((n, m)) < 0.5, 1.0, -1.0).astype(np.float32)
    P = oracle.LogRegCSR(rowptr, col, val, y, n, m, d, 0.1)
    x = rng.standard_normal(d).astype(np.float32)
    with binding.EF21(n, d, 1, 0.1) as h:
        h.set_problem_csr(to_gpu(torch, rowptr, np.int64), to_gpu(torch, col, np.int32), to_gpu(torch, val),
                          to_gpu(torch, y), m, 0.1)
        got = h.local_grad(to_gpu(torch, x))
        again = h.local_grad(to_gpu(torch, x))
        torch.cuda.synchronize()
    assert torch.equal(got, again), "the gradient from sorted CSR rows is bitwise reproducible"
    D = np.zeros((n * m, d), np.float32)
    D[np.repeat(np.arange(n * m), per), col] = val
    assert_grads_close(got.cpu().numpy(), P.grads(x.astype(np.float64)), D.reshape(n, m, d), y, x, per / 64 + 8,
                       m / 64 + 32, "long columns")


def test_csr_unsorted_columns(gpu, oracle):
    """Columns in arbitrary order inside the rows: the library must notice and take its kernel that
    does not rely on ascending columns; same gradients."""
    torch, binding = gpu
    n, d, m, nnz = 3, 20_000, 60, 90
    W = workloads.logreg_csr(n, d, m, nnz, seed=12)
    rng = np.random.default_rng(5)
    col = W.col.reshape(n * m, nnz).copy()
    val = W.val.reshape(n * m, nnz).copy()
    for r in range(n * m):
        perm = rng.permutation(nnz)
        col[r], val[r] = col[r, perm], val[r, perm]
    P = oracle.LogRegCSR(W.rowptr, W.col, W.val, W.y, n, m, d, 0.1)
    x = rng.standard_normal(d).astype(np.float32)
    with binding.EF21(n, d, 1, 0.1) as h:
        h.set_problem_csr(to_gpu(torch, W.rowptr, np.int64), to_gpu(torch, col.reshape(-1), np.int32),
                          to_gpu(torch, val.reshape(-1)), to_gpu(torch, W.y), m, 0.1)
        got = h.local_grad(to_gpu(torch, x))
        torch.cuda.synchronize()
    assert_grads_close(got.cpu().numpy(), P.grads(x.astype(np.float64)), densify(W), W.y, x, nnz / 64 + 8, 64,
                       "unsorted")


@pytest.mark.timeout(400)
def test_config2_full_size_gradient(gpu, oracle):
    """Config 2 at full size (n = 20, m = 5000, d = 2000, 800 MB of rows): every worker's gradient, at
    x = 0 (closed form -A^T y / 2m inside the oracle's pins) and at a random x."""
    torch, binding = gpu
    c = workloads.CONFIGS["C2"]
    n, d, m = c["n"], c["d"], c["m"]
    print("C2 full size gradient", flush=True)
    W = workloads.logreg_dense(n, d, m, seed=c["seed"])
    P = oracle.LogRegDense(W.A, W.y, c["lam"])
    rng = np.random.default_rng(21)
    with binding.EF21(n, d, c["k"], c["gamma"]) as h:
        h.set_problem_dense(to_gpu(torch, W.A), to_gpu(torch, W.y), c["lam"])
        for x in (np.zeros(d, np.float32), rng.standard_normal(d).astype(np.float32)):
            got = h.local_grad(to_gpu(torch, x))
            again = h.local_grad(to_gpu(torch, x))
            torch.cuda.synchronize()
            assert torch.equal(got, again)
            assert_grads_close(got.cpu().numpy(), P.grads(x.astype(np.float64)), W.A, W.y, x, d / 64 + 8, 16,
                               "C2 full size")


@pytest.mark.timeout(600)
def test_config3_full_size_gradient(gpu, oracle):
    """Config 3 at full size (n = 100, m = 2000, d = 50000, 10^8 non-zeros): three workers' gradients
    coordinate by coordinate (the rounding floor needs the worker's matrix), all workers through the
    norm of the difference."""
    import scipy.sparse as sp
    torch, binding = gpu
    c = workloads.CONFIGS["C3"]
    n, d, m, nnz = c["n"], c["d"], c["m"], c["nnz_per_row"]
    print("C3 full size gradient", flush=True)
    W = workloads.logreg_csr(n, d, m, nnz, seed=c["seed"])
    P = oracle.LogRegCSR(W.rowptr, W.col, W.val, W.y, n, m, d, c["lam"])
    rng = np.random.default_rng(22)
    x = rng.standard_normal(d).astype(np.float32)
    with binding.EF21(n, d, c["k"], c["gamma"]) as h:
        h.set_problem_csr(to_gpu(torch, W.rowptr, np.int64), to_gpu(torch, W.col, np.int32), to_gpu(torch, W.val),
                          to_gpu(torch, W.y), m, c["lam"])
        got = h.local_grad(to_gpu(torch, x))
        again = h.local_grad(to_gpu(torch, x))
        torch.cuda.synchronize()
        assert torch.equal(got, again)
    got = got.cpu().numpy()
    ref = P.grads(x.astype(np.float64))
    for i in (0, 57, 99):
        lo, hi = W.rowptr[i * m], W.rowptr[(i + 1) * m]
        A_i = sp.csr_matrix((W.val[lo:hi], W.col[lo:hi], W.rowptr[i * m:(i + 1) * m + 1] - lo), shape=(m, d))
        bound = 1e-5 * np.abs(ref[i]) + gradient_rounding_floor(A_i, W.y[i], x, nnz / 64 + 8, 64)
        err = np.abs(got[i].astype(np.float64) - ref[i])
        assert np.all(err <= bound), f"worker {i}: max err {err.max():.3e}, {int((err > bound).sum())} bad"
        assert np.median(bound) <= 2e-5 * np.max(np.abs(ref[i]))
    rel = np.linalg.norm(got - ref, axis=1) / np.linalg.norm(ref, axis=1)
    assert rel.max() <= 1e-6, f"relative error of the gradients in the 2-norm: {rel.max():.3e}"
