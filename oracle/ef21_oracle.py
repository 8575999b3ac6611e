"""ctypes front end of the EF21 CPU oracle (``ef21_oracle.c``) -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import this module.
It imports nothing from the HIP package and the HIP package imports nothing from here.

The iteration of Algorithm 2 (EF21, multiple nodes) is composed here from the C routines, one
call per line of the algorithm, in the order the paper states, and so are Algorithm 3 (EF21+), whose
distortions and choice are written out in numpy, and Algorithm 4 (the original EF); all state lives in fp64 numpy
arrays (``storage_f32=True`` rounds every stored value to fp32, see the C file's header).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ef21_oracle.c")
_LIB = os.path.join(_HERE, "libef21_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, -O2, single-threaded). Returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-shared", "-fPIC",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = C.CDLL(build())
        i32, i64, dbl = C.c_int32, C.c_int64, C.c_double
        p = C.c_void_p
        lib.ef21o_topk.argtypes = [p, i64, i64, p, p]
        lib.ef21o_topk.restype = C.c_int
        lib.ef21o_logreg_loss_dense.argtypes = [p, p, i64, i64, p, dbl]
        lib.ef21o_logreg_loss_dense.restype = dbl
        lib.ef21o_logreg_grad_dense.argtypes = [p, p, i64, i64, p, dbl, p]
        lib.ef21o_logreg_grad_dense.restype = None
        lib.ef21o_logreg_loss_csr.argtypes = [p, p, p, p, i64, i64, p, dbl]
        lib.ef21o_logreg_loss_csr.restype = dbl
        lib.ef21o_logreg_grad_csr.argtypes = [p, p, p, p, i64, i64, p, dbl, p]
        lib.ef21o_logreg_grad_csr.restype = None
        lib.ef21o_round_storage.argtypes = [p, i64, C.c_int]
        lib.ef21o_round_storage.restype = None
        lib.ef21o_compress_update.argtypes = [i32, i64, i64, p, p, p, p, p, C.c_int]
        lib.ef21o_compress_update.restype = C.c_int
        lib.ef21o_model_step.argtypes = [i64, dbl, p, p, C.c_int]
        lib.ef21o_model_step.restype = None
        lib.ef21o_mean_rows.argtypes = [i32, i64, p, p, C.c_int]
        lib.ef21o_mean_rows.restype = None
        _lib = lib
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


# ----------------------------------------------------------------------------- Top-k (Section 2.1)
def topk(v, k: int):
    """Top-k of one vector: (ascending int32 indices [k], float64 values [k])."""
    v = _f64(v)
    assert v.ndim == 1
    idx = np.empty(k, dtype=np.int32)
    val = np.empty(k, dtype=np.float64)
    rc = _load().ef21o_topk(_ptr(v), v.size, k, _ptr(idx), _ptr(val))
    if rc != 0:
        raise ValueError("ef21o_topk: bad arguments")
    return idx, val


def topk_rows(V, k: int):
    """Row-wise Top-k of an [n][d] array: (idx [n][k] int32, val [n][k] float64)."""
    V = _f64(V)
    out = [topk(row, k) for row in V]
    return np.stack([o[0] for o in out]), np.stack([o[1] for o in out])


def topk_dense(v, k: int) -> np.ndarray:
    """C(v) as a dense vector: the k kept entries, zeros elsewhere."""
    idx, val = topk(v, k)
    out = np.zeros(len(v), dtype=np.float64)
    out[idx] = val
    return out


# --------------------------------------------------------------- objective of Section 5, eq. (9)
class LogRegDense:
    """n workers, each with m dense fp32 rows: A [n][m][d], y [n][m] (+-1), regulariser weight lam."""

    def __init__(self, A, y, lam: float):
        self.A = np.ascontiguousarray(A, dtype=np.float32)
        self.y = np.ascontiguousarray(y, dtype=np.float32)
        self.n, self.m, self.d = self.A.shape
        assert self.y.shape == (self.n, self.m)
        self.lam = float(lam)

    def loss_i(self, i: int, x) -> float:
        x = _f64(x)
        return _load().ef21o_logreg_loss_dense(_ptr(self.A[i]), _ptr(self.y[i]), self.m, self.d, _ptr(x),
                                               self.lam)

    def grad_i(self, i: int, x) -> np.ndarray:
        x = _f64(x)
        g = np.empty(self.d, dtype=np.float64)
        _load().ef21o_logreg_grad_dense(_ptr(self.A[i]), _ptr(self.y[i]), self.m, self.d, _ptr(x), self.lam,
                                        _ptr(g))
        return g

    def loss(self, x) -> float:
        """f(x) = (1/n) sum_i f_i(x), eq. (1)."""
        return sum(self.loss_i(i, x) for i in range(self.n)) / self.n

    def grads(self, x) -> np.ndarray:
        return np.stack([self.grad_i(i, x) for i in range(self.n)])


class LogRegCSR:
    """n workers, each with m sparse rows; one CSR over all n*m rows (rowptr int64 [n*m+1])."""

    def __init__(self, rowptr, col, val, y, n: int, m: int, d: int, lam: float):
        self.rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
        self.col = np.ascontiguousarray(col, dtype=np.int32)
        self.val = np.ascontiguousarray(val, dtype=np.float32)
        self.y = np.ascontiguousarray(y, dtype=np.float32).reshape(n, m)
        self.n, self.m, self.d = n, m, d
        assert self.rowptr.size == n * m + 1
        self.lam = float(lam)

    def _rp(self, i):
        return self.rowptr[i * self.m:(i + 1) * self.m + 1]

    def loss_i(self, i: int, x) -> float:
        x = _f64(x)
        rp = np.ascontiguousarray(self._rp(i))
        return _load().ef21o_logreg_loss_csr(_ptr(rp), _ptr(self.col), _ptr(self.val), _ptr(self.y[i]), self.m,
                                             self.d, _ptr(x), self.lam)

    def grad_i(self, i: int, x) -> np.ndarray:
        x = _f64(x)
        rp = np.ascontiguousarray(self._rp(i))
        g = np.empty(self.d, dtype=np.float64)
        _load().ef21o_logreg_grad_csr(_ptr(rp), _ptr(self.col), _ptr(self.val), _ptr(self.y[i]), self.m, self.d,
                                      _ptr(x), self.lam, _ptr(g))
        return g

    def loss(self, x) -> float:
        return sum(self.loss_i(i, x) for i in range(self.n)) / self.n

    def grads(self, x) -> np.ndarray:
        return np.stack([self.grad_i(i, x) for i in range(self.n)])


# --------------------------------------------------------------- objective of Section 5.2 (least squares)
class LeastSquaresDense:
    """f_i(x) = (1/m) sum_l (a_il^T x - b_il)^2  (+ lam sum_j x_j^2 / (1 + x_j^2), zero in the paper's
    function), A [n][m][d] dense fp32 rows, b [n][m]; numpy in fp64."""

    def __init__(self, A, b, lam: float = 0.0):
        self.A = np.ascontiguousarray(A, dtype=np.float32)
        self.b = np.ascontiguousarray(b, dtype=np.float32)
        self.n, self.m, self.d = self.A.shape
        assert self.b.shape == (self.n, self.m)
        self.lam = float(lam)

    def _reg(self, x):
        return self.lam * float(np.sum(x * x / (1.0 + x * x))), 2.0 * self.lam * x / (1.0 + x * x) ** 2

    def loss_i(self, i: int, x) -> float:
        x = _f64(x)
        r = self.A[i].astype(np.float64) @ x - self.b[i].astype(np.float64)
        return float(np.mean(r * r)) + self._reg(x)[0]

    def grad_i(self, i: int, x) -> np.ndarray:
        x = _f64(x)
        Ai = self.A[i].astype(np.float64)
        r = Ai @ x - self.b[i].astype(np.float64)
        return (2.0 / self.m) * (Ai.T @ r) + self._reg(x)[1]

    def loss(self, x) -> float:
        return sum(self.loss_i(i, x) for i in range(self.n)) / self.n

    def grads(self, x) -> np.ndarray:
        return np.stack([self.grad_i(i, x) for i in range(self.n)])


def densify_csr(rowptr, col, val, n: int, m: int, d: int) -> np.ndarray:
    """[n][m][d] dense copy of a CSR matrix over n*m rows (small problems only)."""
    D = np.zeros((n * m, d), dtype=np.float32)
    for r in range(n * m):
        D[r, col[rowptr[r]:rowptr[r + 1]]] = val[rowptr[r]:rowptr[r + 1]]
    return D.reshape(n, m, d)


# --------------------------------------------------------------- stochastic gradients (Algorithm 5)
def restrict_rows(problem, i: int, rows):
    """Worker i's objective over the listed rows only (a one-worker problem of the same class): the
    minibatch estimator of Algorithm 5 is the gradient of this function.  A row listed twice counts twice."""
    rows = np.asarray(rows, dtype=np.int64)
    assert rows.ndim == 1 and rows.size > 0 and rows.min() >= 0 and rows.max() < problem.m
    if isinstance(problem, LogRegDense):
        return LogRegDense(problem.A[i][rows][None], problem.y[i][rows][None], problem.lam)
    if isinstance(problem, LeastSquaresDense):
        return LeastSquaresDense(problem.A[i][rows][None], problem.b[i][rows][None], problem.lam)
    if isinstance(problem, LogRegCSR):
        rp = [0]
        cols, vals = [], []
        for l in rows:
            p0, p1 = problem.rowptr[i * problem.m + l], problem.rowptr[i * problem.m + l + 1]
            cols.append(problem.col[p0:p1])
            vals.append(problem.val[p0:p1])
            rp.append(rp[-1] + int(p1 - p0))
        return LogRegCSR(np.array(rp), np.concatenate(cols) if cols else np.zeros(0, np.int32),
                         np.concatenate(vals) if vals else np.zeros(0, np.float32), problem.y[i][rows], 1,
                         rows.size, problem.d, problem.lam)
    raise TypeError(type(problem))


def minibatch_grads(problem, x, batch) -> np.ndarray:
    """ghat_i = (1/tau) sum over l in batch[i] of the gradient of row l's loss, plus the regulariser's
    gradient (line 5 of Algorithm 5; the experiments draw the batch without replacement).  batch: [n][tau]
    row indices in [0, m), drawn by the caller."""
    batch = np.asarray(batch, dtype=np.int64)
    assert batch.ndim == 2 and batch.shape[0] == problem.n
    return np.stack([restrict_rows(problem, i, batch[i]).grad_i(0, x) for i in range(problem.n)])


def iteration_stochastic(state: "EF21State", problem, batch, k: int, gamma: float, order: str = "grad_first",
                         storage_f32: bool = True) -> None:
    """One iteration of Algorithm 5: Algorithm 2 with the minibatch estimator in the place of the gradient."""
    iteration(state, lambda x: minibatch_grads(problem, x, batch), k, gamma, order=order, storage_f32=storage_f32)


# ------------------------------------------------------------------ Algorithm 2 (EF21, multi-node)
def round_storage(a, storage_f32: bool) -> np.ndarray:
    a = _f64(a).copy()
    _load().ef21o_round_storage(_ptr(a), a.size, int(storage_f32))
    return a


def mean_rows(g_i, storage_f32: bool) -> np.ndarray:
    g_i = _f64(g_i)
    n, d = g_i.shape
    g = np.empty(d, dtype=np.float64)
    _load().ef21o_mean_rows(n, d, _ptr(g_i), _ptr(g), int(storage_f32))
    return g


@dataclass
class EF21State:
    """State of Algorithm 2: iterate x [d], per-worker estimators g_i [n][d], their mean g [d]."""
    x: np.ndarray
    g_i: np.ndarray
    g: np.ndarray
    msg_idx: np.ndarray | None = None   # last messages c_i as (index, value) pairs, [n][k]
    msg_val: np.ndarray | None = None

    def copy(self) -> "EF21State":
        return EF21State(self.x.copy(), self.g_i.copy(), self.g.copy(),
                         None if self.msg_idx is None else self.msg_idx.copy(),
                         None if self.msg_val is None else self.msg_val.copy())


def init_state(x0, grads0, k: int, init: str = "grad", storage_f32: bool = True) -> EF21State:
    """Input line of Algorithm 2.  init="compressed": g_i^0 = C(grad f_i(x^0)) (the algorithm's
    default); init="grad": g_i^0 = grad f_i(x^0) (allowed by the remark after Theorem 2, makes
    G^0 = 0); init="zero": g_i^0 = 0 (any vector is admissible).  g^0 = mean_i g_i^0."""
    x = round_storage(x0, storage_f32)
    grads0 = round_storage(grads0, storage_f32)
    if init == "grad":
        g_i = grads0
    elif init == "compressed":
        g_i = np.stack([topk_dense(row, k) for row in grads0])
    elif init == "zero":
        g_i = np.zeros_like(grads0)
    else:
        raise ValueError(init)
    return EF21State(x, g_i, mean_rows(g_i, storage_f32))


def compress_update(state: EF21State, grads, k: int, storage_f32: bool = True) -> None:
    """Lines 5, 6 and 8 of Algorithm 2 for all workers, in place."""
    grads = round_storage(grads, storage_f32)
    n, d = state.g_i.shape
    assert grads.shape == (n, d)
    idx = np.empty((n, k), dtype=np.int32)
    val = np.empty((n, k), dtype=np.float64)
    rc = _load().ef21o_compress_update(n, d, k, _ptr(grads), _ptr(state.g_i), _ptr(state.g), _ptr(idx),
                                       _ptr(val), int(storage_f32))
    if rc != 0:
        raise ValueError("ef21o_compress_update: bad arguments")
    state.msg_idx, state.msg_val = idx, val


def model_step(state: EF21State, gamma: float, storage_f32: bool = True) -> None:
    """Line 3 of Algorithm 2, in place."""
    _load().ef21o_model_step(state.x.size, float(gamma), _ptr(state.x), _ptr(state.g), int(storage_f32))


def iteration(state: EF21State, grads_at, k: int, gamma: float, order: str = "grad_first",
              storage_f32: bool = True) -> None:
    """One pass of the loop body of Algorithm 2.

    grads_at: callable x -> [n][d] gradients, or an [n][d] array of supplied gradients
    (the stochastic variant, Algorithm 5, replaces grad f_i by any estimator).
    order="step_first" is the loop body as printed: line 3, then lines 5, 6, 8 at the new x.
    order="grad_first" is the same loop rotated by one phase: lines 5, 6, 8 at the current x,
    then line 3.  With g_i^0 = grad f_i(x^0) both produce the same iterates x^0, x^1, ...
    """
    def grads_now():
        return grads_at(state.x) if callable(grads_at) else grads_at

    if order == "step_first":
        model_step(state, gamma, storage_f32)
        compress_update(state, grads_now(), k, storage_f32)
    elif order == "grad_first":
        compress_update(state, grads_now(), k, storage_f32)
        model_step(state, gamma, storage_f32)
    else:
        raise ValueError(order)


# ------------------------------------------------------------------ Algorithm 3 (EF21+, multi-node)
def plus_update(state: EF21State, grads, k: int, storage_f32: bool = True):
    """Lines 5 to 8 and 10 of Algorithm 3 for all workers, in place, with C = Top-k and s = grad f_i(x):
         b = C(s)                                  (line 5, the plain compressor)
         m = g_i + C(s - g_i)                      (line 6, the Markov compressor)
         B = ||b - s||^2,  M = ||m - s||^2         (line 7; fp64 sums of the stored values)
         g_i <- m if M <= B else b                 (line 8)
         g   <- (1/n) sum_i g_i                    (line 10)
    The message a worker sends is the k pairs of whichever compressor it chose, kept in state.msg_*.
    Returns (branch [n] int32: 1 where the plain compressor was chosen, B [n], M [n])."""
    grads = round_storage(grads, storage_f32)
    n, d = state.g_i.shape
    assert grads.shape == (n, d)
    idx = np.empty((n, k), dtype=np.int32)
    val = np.empty((n, k), dtype=np.float64)
    branch = np.zeros(n, dtype=np.int32)
    Bs, Ms = np.empty(n), np.empty(n)
    for i in range(n):
        s, g_old = grads[i], state.g_i[i]
        ib, vb = topk(s, k)
        b = np.zeros(d)
        b[ib] = vb
        if storage_f32:      # the difference is one fp32 subtraction, the update one fp32 addition
            v = (s.astype(np.float32) - g_old.astype(np.float32)).astype(np.float64)
        else:
            v = s - g_old
        im, vm = topk(v, k)
        m = g_old.copy()
        if storage_f32:
            m[im] = (g_old[im].astype(np.float32) + vm.astype(np.float32)).astype(np.float64)
        else:
            m[im] = g_old[im] + vm
        Bs[i] = float(np.sum((b - s) ** 2))
        Ms[i] = float(np.sum((m - s) ** 2))
        if Ms[i] <= Bs[i]:
            state.g_i[i], idx[i], val[i] = m, im, vm
        else:
            state.g_i[i], idx[i], val[i], branch[i] = b, ib, vb, 1
    state.g[:] = mean_rows(state.g_i, storage_f32)
    state.msg_idx, state.msg_val = idx, val
    return branch, Bs, Ms


def iteration_plus(state: EF21State, grads_at, k: int, gamma: float, order: str = "grad_first",
                   storage_f32: bool = True):
    """One pass of the loop body of Algorithm 3 (EF21+); arguments and the two orders as in `iteration`.
    Returns what plus_update returns."""
    def grads_now():
        return grads_at(state.x) if callable(grads_at) else grads_at

    if order == "step_first":
        model_step(state, gamma, storage_f32)
        return plus_update(state, grads_now(), k, storage_f32)
    if order == "grad_first":
        out = plus_update(state, grads_now(), k, storage_f32)
        model_step(state, gamma, storage_f32)
        return out
    raise ValueError(order)


# ------------------------------------------------------------------ Algorithm 4 (EF, the original error feedback)
@dataclass
class EFState:
    """State of Algorithm 4: iterate x [d] and the workers' errors e_i [n][d]; the last messages w_i as pairs."""
    x: np.ndarray
    e: np.ndarray
    msg_idx: np.ndarray | None = None
    msg_val: np.ndarray | None = None


def ef_iteration(state: EFState, grads_at, k: int, gamma: float, storage_f32: bool = True) -> None:
    """One round of Algorithm 4 written with one gradient per round: at the current x,
         p_i = e_i + gamma grad f_i(x)        (what the worker would like to send; lines 6 and 8)
         w_i = C(p_i)                          (line 8, C = Top-k)
         e_i <- p_i - w_i                      (line 6 of the next round)
         x   <- x - (1/n) sum_i w_i            (line 4 of the next round)
    which, started from e_i = 0, produces the algorithm's x^0, x^1, ... (its line 2 is the first round)."""
    grads = round_storage(grads_at(state.x) if callable(grads_at) else grads_at, storage_f32)
    n, d = state.e.shape
    assert grads.shape == (n, d)
    idx = np.empty((n, k), dtype=np.int32)
    val = np.empty((n, k), dtype=np.float64)
    total = np.zeros(d)
    for i in range(n):
        p = round_storage(state.e[i] + gamma * grads[i], storage_f32)
        idx[i], val[i] = topk(p, k)
        w = np.zeros(d)
        w[idx[i]] = val[i]
        state.e[i] = p - w                  # exact: zero where kept, p elsewhere
        total += w                          # worker order
    state.x = round_storage(state.x - total / n, storage_f32)
    state.msg_idx, state.msg_val = idx, val


# ------------------------------------------------------------------------ theory (Section 3.4)
def theta_beta(alpha: float):
    """theta = 1 - sqrt(1 - alpha), beta = (1 - alpha) / (1 - sqrt(1 - alpha))  (before Theorem 1)."""
    r = np.sqrt(1.0 - alpha)
    return 1.0 - r, (1.0 - alpha) / (1.0 - r)


def smoothness_constants(problem) -> np.ndarray:
    """L_i of the smoothness assumption of Section 3.4 for every worker, from the definition: the gradient of
    f_i is Lipschitz with  c * lambda_max((1/m) A_i^T A_i) + 2 lam,  c the largest curvature of the per-row
    loss in its margin (1/4 for the logistic loss of eq. (9), 2 for the square of Section 5.2) and 2 the
    largest curvature of t^2 / (1 + t^2).  Exact symmetric eigenvalues (numpy); CSR problems are made dense,
    so small sizes only."""
    if isinstance(problem, LogRegCSR):
        A = densify_csr(problem.rowptr, problem.col, problem.val, problem.n, problem.m, problem.d)
        c = 0.25
    else:
        A = problem.A
        c = 2.0 if isinstance(problem, LeastSquaresDense) else 0.25
    out = np.empty(problem.n)
    for i in range(problem.n):
        Ai = A[i].astype(np.float64)
        out[i] = c * np.linalg.eigvalsh(Ai.T @ Ai / problem.m)[-1] + 2.0 * problem.lam
    return out


def smoothness_constant_of_f(problem) -> float:
    """L of the smoothness assumption of Section 3.4 for f = (1/n) sum_i f_i itself, from the definition: the
    Hessian of f is (1/(n m)) sum_i A_i^T diag(curvatures) A_i plus the regulariser's, so its gradient is Lipschitz
    with  c * lambda_max((1/(n m)) sum_i A_i^T A_i) + 2 lam  (c and 2 as in smoothness_constants).  Never above
    the mean of the L_i, the bound the text notes before Theorem 1.  Exact symmetric eigenvalues (numpy); CSR
    problems are made dense, so small sizes only."""
    if isinstance(problem, LogRegCSR):
        A = densify_csr(problem.rowptr, problem.col, problem.val, problem.n, problem.m, problem.d)
        c = 0.25
    else:
        A = problem.A
        c = 2.0 if isinstance(problem, LeastSquaresDense) else 0.25
    S = np.zeros((problem.d, problem.d))
    for i in range(problem.n):
        Ai = np.asarray(A[i], dtype=np.float64)
        S += Ai.T @ Ai
    return float(c * np.linalg.eigvalsh(S / (problem.n * problem.m))[-1] + 2.0 * problem.lam)


def theory_stepsize(L_i, alpha: float, L: float = None) -> float:
    """The largest stepsize Theorem 1 allows: 1 / (L + Ltilde sqrt(beta / theta)), Ltilde the quadratic mean of
    the L_i; L defaults to their arithmetic mean (an upper bound on the smoothness constant of f, as noted
    before the theorem).  alpha = k / d for Top-k."""
    L_i = _f64(L_i)
    theta, beta = theta_beta(alpha)
    if L is None:
        L = float(np.mean(L_i))
    return 1.0 / (L + float(np.sqrt(np.mean(L_i * L_i))) * float(np.sqrt(beta / theta)))


def distortion(state: EF21State, grads) -> float:
    """G^t = (1/n) sum_i ||g_i - grad f_i(x)||^2, eq. (8)."""
    diff = state.g_i - _f64(grads)
    return float(np.mean(np.sum(diff * diff, axis=1)))
