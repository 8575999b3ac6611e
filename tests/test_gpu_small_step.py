"""The one-launch iteration of small dense problems (ef21_step with EF21_ONE_LAUNCH): bit for bit the
state and the messages of the separate gradient, Top-k and aggregation kernels, step after step, in both loop
orders and for both losses; and against the CPU oracle through f(x^t) (1e-4) and the first message."""
import numpy as np
import pytest

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


def problem(n, d, m, seed):
    rng = np.random.default_rng(seed)
    A = (rng.standard_normal((n, m, d)) / np.sqrt(d)).astype(np.float32)
    w = rng.standard_normal(d)
    y = np.sign(A.astype(np.float64) @ w + 1e-30).astype(np.float32)
    return A, y, rng


SHAPES = [(4, 100, 250, 3),      # the smallest configuration: vec4, one quarter-wave of columns
          (3, 256, 37, 5),       # vec4, a full wavefront of float4
          (2, 333, 41, 4),       # scalar columns, ragged
          (5, 1024, 301, 16),    # the widest rows the kernel takes
          (20, 123, 1628, 1),    # the shape of the paper's a9a split over 20 workers, Top-1
          (7, 68, 1579, 2),      # phishing over 7 workers
          (1, 1, 1, 1),
          (3, 512, 9, 512)]      # k = d


@pytest.mark.parametrize("n,d,m,k", SHAPES)
@pytest.mark.parametrize("order", ["grad_first", "step_first"])
def test_same_bits_as_the_separate_kernels(gpu, n, d, m, k, order):
    torch, binding = gpu
    print(f"one-launch iteration n={n} d={d} m={m} k={k} {order}", flush=True)
    A, y, rng = problem(n, d, m, d + m)
    Ag, yg = to_gpu(torch, A), to_gpu(torch, y)
    x0 = to_gpu(torch, 0.1 * rng.standard_normal(d))
    flag = binding.ORDER_STEP_FIRST if order == "step_first" else binding.ORDER_GRAD_FIRST
    with binding.EF21(n, d, k, 0.5) as one, binding.EF21(n, d, k, 0.5) as sep:
        for h in (one, sep):
            h.set_problem_dense(Ag, yg, 0.1)
            h.set_state(x0, 0.5 * h.local_grad(x0), None)
        for t in range(12):
            one.step(None, flag | binding.ONE_LAUNCH)
            sep.step(None, flag)
            a, b = one.get_state(), sep.get_state()
            for name, u, v in zip(("x", "g_i", "g"), a, b):
                assert torch.equal(u, v), f"step {t}: {name} differs"
            (ia, va), (ib, vb) = one.get_messages(), sep.get_messages()
            assert torch.equal(ia, ib) and torch.equal(va, vb), f"step {t}: messages differ"
        one.set_timing(True)
        one.step(None, flag | binding.ONE_LAUNCH)
        classes = one.get_timing(reset=True)
        one.set_timing(False)
        assert "small_step" in classes and "topk_row" not in classes and "grad_main" not in classes


def test_least_squares_same_bits(gpu):
    torch, binding = gpu
    n, d, m, k = 3, 200, 90, 7
    A, _, rng = problem(n, d, m, 5)
    b = rng.standard_normal((n, m)).astype(np.float32)
    Ag, bg = to_gpu(torch, A), to_gpu(torch, b)
    x0 = torch.zeros(d, device="cuda")
    with binding.EF21(n, d, k, 0.2) as one, binding.EF21(n, d, k, 0.2) as sep:
        for h in (one, sep):
            h.set_problem_dense(Ag, bg, 0.0)
            h.set_loss(binding.LOSS_LEAST_SQUARES)
            h.set_state(x0, torch.zeros((n, d), device="cuda"), None)
        for t in range(10):
            one.step(None, binding.ONE_LAUNCH)
            sep.step()
            for u, v in zip(one.get_state(), sep.get_state()):
                assert torch.equal(u, v), f"step {t}"


def test_against_the_oracle(gpu, oracle):
    torch, binding = gpu
    n, d, m, k = 4, 100, 250, 3
    A, y, rng = problem(n, d, m, 6)
    P = oracle.LogRegDense(A, y, 0.1)
    gamma = float(np.float32(0.5))
    x0 = np.zeros(d)
    st = oracle.init_state(x0, P.grads(x0), k, init="zero", storage_f32=True)
    with binding.EF21(n, d, k, gamma) as h:
        h.set_problem_dense(to_gpu(torch, A), to_gpu(torch, y), 0.1)
        h.set_state(to_gpu(torch, st.x), to_gpu(torch, st.g_i), to_gpu(torch, st.g))
        grads0 = h.local_grad(None).cpu().numpy()
        f0 = P.loss(x0)
        for t in range(60):
            oracle.iteration(st, P.grads, k, gamma)
            h.step(None, binding.ONE_LAUNCH)
            if t == 0:        # zero state: the message is the Top-k of the gradient the library itself reports
                idx, val = h.get_messages()
                ref_idx, ref_val = oracle.topk_rows(grads0.astype(np.float64), k)
                assert np.array_equal(idx.cpu().numpy(), ref_idx)
                assert np.array_equal(val.cpu().numpy(), ref_val.astype(np.float32))
            f_ref, f_gpu = P.loss(st.x), P.loss(h.get_x().cpu().numpy().astype(np.float64))
            assert abs(f_gpu - f_ref) <= 1e-4 * abs(f_ref), f"iteration {t}: {f_gpu} vs {f_ref}"
        assert f_ref < f0


def test_larger_problems_keep_the_separate_kernels(gpu):
    torch, binding = gpu
    n, d, m, k = 2, 2000, 40, 5          # d above the one-launch limit
    A, y, _ = problem(n, d, m, 7)
    with binding.EF21(n, d, k, 0.5) as h:
        h.set_problem_dense(to_gpu(torch, A), to_gpu(torch, y), 0.1)
        h.set_timing(True)
        h.step(None, binding.ONE_LAUNCH)
        classes = h.get_timing(reset=True)
        assert "small_step" not in classes and "grad_main" in classes
    with binding.EF21(4, 100, 3, 0.5) as h:          # and a qualifying problem takes them unless asked
        A, y, _ = problem(4, 100, 250, 8)
        h.set_problem_dense(to_gpu(torch, A), to_gpu(torch, y), 0.1)
        h.set_timing(True)
        h.step()
        classes = h.get_timing(reset=True)
        assert "small_step" not in classes and "grad_main" in classes


def test_flag_combinations(gpu):
    torch, binding = gpu
    with binding.EF21(2, 16, 2, 0.1) as h:
        g = torch.ones((2, 16), device="cuda")
        h.step(g, binding.ONE_LAUNCH)                      # supplied gradients: the flag changes nothing
        h.step(g, binding.ONE_LAUNCH | binding.PLUS | binding.ORDER_STEP_FIRST)
        h.step(g, binding.ONE_LAUNCH | binding.CLASSIC_EF)
        for bad in (16, binding.CLASSIC_EF | binding.PLUS, binding.CLASSIC_EF | binding.ORDER_STEP_FIRST):
            with pytest.raises(binding.EF21Error):
                h.step(g, bad)
