"""Thin Python binding of ``libef21.so`` (see ``include/ef21.h``): argument marshalling only.

PyTorch supplies device memory (``tensor.data_ptr()``) and the stream; every step of the EF21
hot path runs inside the library's HIP kernels.  There is no fallback: a missing library or a
failing call raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libef21.so")

EF21_OK, EF21_EINVAL, EF21_ENOMEM, EF21_EHIP, EF21_ESTATE = 0, -1, -2, -3, -4
ORDER_GRAD_FIRST, ORDER_STEP_FIRST, PLUS, CLASSIC_EF, ONE_LAUNCH = 0, 1, 2, 4, 8
LOSS_LOGISTIC, LOSS_LEAST_SQUARES = 0, 1

# every symbol include/ef21.h declares
SYMBOLS = (
    "ef21_last_error", "ef21_create", "ef21_destroy", "ef21_set_stream", "ef21_topk",
    "ef21_set_problem_dense", "ef21_set_problem_csr", "ef21_set_state", "ef21_get_state",
    "ef21_get_messages", "ef21_local_grad", "ef21_step", "ef21_set_timing", "ef21_get_timing", "ef21_kernel_name",
    "ef21_hbm_read", "ef21_hbm_copy", "ef21_get_choices", "ef21_set_loss", "ef21_set_minibatch", "ef21_theory_stepsize",
    "ef21_topk_static",
)
K_COUNT = 11


class EF21Error(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"libef21 error {code}: {text}")
        self.code = code


_lib = None


def load_library() -> C.CDLL:
    """Open libef21.so (built in-tree by paper_2106_05203_amd/build.py) and declare prototypes."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2106_05203_amd.build` "
            "(there is no non-HIP fallback)")
    lib = C.CDLL(LIB_PATH)
    p, i32, i64, f32, u32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.c_uint32
    lib.ef21_last_error.argtypes = []
    lib.ef21_last_error.restype = C.c_char_p
    lib.ef21_create.argtypes = [i32, i64, i64, f32]
    lib.ef21_create.restype = p
    lib.ef21_destroy.argtypes = [p]
    lib.ef21_set_stream.argtypes = [p, p]
    lib.ef21_topk.argtypes = [p, i32, i64, i64, p, p, p]
    lib.ef21_topk_static.argtypes = [p, i32, i64, i64, p, p, p]
    lib.ef21_set_problem_dense.argtypes = [p, p, p, i64, f32]
    lib.ef21_set_problem_csr.argtypes = [p, p, p, p, p, i64, f32]
    lib.ef21_set_state.argtypes = [p, p, p, p]
    lib.ef21_get_state.argtypes = [p, p, p, p]
    lib.ef21_get_messages.argtypes = [p, p, p]
    lib.ef21_local_grad.argtypes = [p, p, p]
    lib.ef21_step.argtypes = [p, p, u32]
    lib.ef21_set_timing.argtypes = [p, C.c_int]
    lib.ef21_get_timing.argtypes = [p, p, p, C.c_int]
    lib.ef21_kernel_name.argtypes = [C.c_int]
    lib.ef21_get_choices.argtypes = [p, p, p]
    lib.ef21_set_loss.argtypes = [p, C.c_int]
    lib.ef21_set_minibatch.argtypes = [p, p, C.c_int64]
    lib.ef21_theory_stepsize.argtypes = [p, C.c_int32, p, p, p]
    lib.ef21_hbm_read.argtypes = [p, C.c_int64, p, p]
    lib.ef21_hbm_copy.argtypes = [p, p, C.c_int64, p]
    for name in SYMBOLS[2:]:
        getattr(lib, name).restype = C.c_int
    lib.ef21_kernel_name.restype = C.c_char_p
    _lib = lib
    return lib


def _check(rc: int) -> None:
    if rc != EF21_OK:
        raise EF21Error(rc, load_library().ef21_last_error().decode())


def _dev(t: torch.Tensor, dtype: torch.dtype, shape=None) -> int:
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("expected a tensor in GPU memory")
    if t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"expected a contiguous {dtype} tensor, got {t.dtype} (contiguous={t.is_contiguous()})")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {tuple(t.shape)}")
    return t.data_ptr()


def _opt(t, dtype, shape=None):
    return None if t is None else _dev(t, dtype, shape)


def _current_stream_ptr() -> int:
    return torch.cuda.current_stream().cuda_stream


def ef21_topk(rows: torch.Tensor, k: int, out_idx: torch.Tensor | None = None,
              out_val: torch.Tensor | None = None, static: bool = False):
    """Batched Top-k (ef21_topk, or ef21_topk_static if `static`) of rows [n][d] on torch's current stream.
    Returns (idx [n][k] int32 ascending, val [n][k] float32)."""
    lib = load_library()
    if rows.dim() != 2:
        raise ValueError("rows must be [n][d]")
    n, d = rows.shape
    if out_idx is None:
        out_idx = torch.empty((n, max(k, 0)), dtype=torch.int32, device=rows.device)
    if out_val is None:
        out_val = torch.empty((n, max(k, 0)), dtype=torch.float32, device=rows.device)
    call = lib.ef21_topk_static if static else lib.ef21_topk
    _check(call(_dev(rows, torch.float32), n, d, k, _dev(out_idx, torch.int32), _dev(out_val, torch.float32),
                _current_stream_ptr()))
    return out_idx, out_val


def ef21_hbm_read(src: torch.Tensor, sink: torch.Tensor) -> None:
    """One plain read of `src` (ef21_hbm_read) on torch's current stream; measurement only."""
    lib = load_library()
    _check(lib.ef21_hbm_read(src.data_ptr(), src.numel() * src.element_size(), sink.data_ptr(), _current_stream_ptr()))


def ef21_hbm_copy(dst: torch.Tensor, src: torch.Tensor) -> None:
    """dst <- src by a plain copy kernel (ef21_hbm_copy) on torch's current stream; measurement only."""
    lib = load_library()
    if dst.numel() * dst.element_size() != src.numel() * src.element_size():
        raise ValueError("dst and src must have the same size in bytes")
    _check(lib.ef21_hbm_copy(dst.data_ptr(), src.data_ptr(), src.numel() * src.element_size(), _current_stream_ptr()))


class EF21:
    """Handle of the C library: state of Algorithm 2 for n workers batched on one GPU."""

    def __init__(self, n: int, d: int, k: int, gamma: float, device="cuda:0"):
        self._lib = load_library()
        self.n, self.d, self.k, self.gamma = int(n), int(d), int(k), float(gamma)
        self.device = torch.device(device)
        self._keep = []     # borrowed problem tensors stay alive with the handle
        self._batch = None  # and the rows of the minibatch
        with torch.cuda.device(self.device):
            self._h = self._lib.ef21_create(self.n, self.d, self.k, self.gamma)
        if not self._h:
            raise EF21Error(EF21_EINVAL, self._lib.ef21_last_error().decode())
        self.use_current_stream()

    # -- plumbing
    def use_current_stream(self) -> None:
        with torch.cuda.device(self.device):
            _check(self._lib.ef21_set_stream(self._h, _current_stream_ptr()))

    def close(self) -> None:
        if getattr(self, "_h", None):
            with torch.cuda.device(self.device):
                _check(self._lib.ef21_destroy(self._h))
            self._h = None
            self._keep = []

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    # -- problem
    def set_problem_dense(self, A: torch.Tensor, y: torch.Tensor, lam: float) -> None:
        n, m, d = A.shape
        if (n, d) != (self.n, self.d):
            raise ValueError("A must be [n][m][d]")
        with torch.cuda.device(self.device):
            _check(self._lib.ef21_set_problem_dense(self._h, _dev(A, torch.float32), _dev(y, torch.float32, (n, m)), m,
                                                    float(lam)))
        self._keep = [A, y]
        self._batch = None

    def set_problem_csr(self, rowptr: torch.Tensor, col: torch.Tensor, val: torch.Tensor, y: torch.Tensor, m: int,
                        lam: float) -> None:
        if rowptr.numel() != self.n * m + 1 or col.numel() != val.numel():
            raise ValueError("rowptr must have n*m+1 entries and col, val equal lengths")
        with torch.cuda.device(self.device):
            _check(self._lib.ef21_set_problem_csr(self._h, _dev(rowptr, torch.int64), _dev(col, torch.int32),
                                                  _dev(val, torch.float32), _dev(y, torch.float32, (self.n, m)), m,
                                                  float(lam)))
        self._keep = [rowptr, col, val, y]
        self._batch = None

    # -- state
    def set_state(self, x=None, g_i=None, g=None) -> None:
        with torch.cuda.device(self.device):
            _check(self._lib.ef21_set_state(self._h, _opt(x, torch.float32, (self.d,)),
                                            _opt(g_i, torch.float32, (self.n, self.d)),
                                            _opt(g, torch.float32, (self.d,))))

    def get_state(self):
        x = torch.empty(self.d, dtype=torch.float32, device=self.device)
        g_i = torch.empty((self.n, self.d), dtype=torch.float32, device=self.device)
        g = torch.empty(self.d, dtype=torch.float32, device=self.device)
        with torch.cuda.device(self.device):
            _check(self._lib.ef21_get_state(self._h, x.data_ptr(), g_i.data_ptr(), g.data_ptr()))
        return x, g_i, g

    def get_x(self) -> torch.Tensor:
        x = torch.empty(self.d, dtype=torch.float32, device=self.device)
        with torch.cuda.device(self.device):
            _check(self._lib.ef21_get_state(self._h, x.data_ptr(), None, None))
        return x

    def get_messages(self):
        idx = torch.empty((self.n, self.k), dtype=torch.int32, device=self.device)
        val = torch.empty((self.n, self.k), dtype=torch.float32, device=self.device)
        with torch.cuda.device(self.device):
            _check(self._lib.ef21_get_messages(self._h, idx.data_ptr(), val.data_ptr()))
        return idx, val

    def set_loss(self, loss: int) -> None:
        with torch.cuda.device(self.device):
            _check(self._lib.ef21_set_loss(self._h, int(loss)))

    def set_minibatch(self, rows: "torch.Tensor | None") -> None:
        """rows: int32 [n][tau] on the device (kept alive by the handle and read at every gradient), or None
        for full gradients."""
        with torch.cuda.device(self.device):
            if rows is None:
                _check(self._lib.ef21_set_minibatch(self._h, None, 0))
                self._batch = None
                return
            assert rows.dtype == torch.int32 and rows.is_cuda and rows.is_contiguous() and rows.dim() == 2
            assert rows.shape[0] == self.n
            _check(self._lib.ef21_set_minibatch(self._h, rows.data_ptr(), int(rows.shape[1])))
            self._batch = rows

    def theory_stepsize(self, iterations: int = 200):
        """(gamma, L, L_i [n]) of Theorem 1 for the attached problem, eigenvalues by power iteration on the GPU."""
        gamma, L = C.c_double(), C.c_double()
        L_i = (C.c_double * self.n)()
        with torch.cuda.device(self.device):
            _check(self._lib.ef21_theory_stepsize(self._h, int(iterations), C.byref(gamma), C.byref(L), L_i))
        return gamma.value, L.value, list(L_i)

    def get_choices(self):
        """(branch [n] int32: 1 = plain compressor chosen, distortions [n][2] float64: B_i, M_i) of the last
        step taken with PLUS."""
        branch = torch.empty(self.n, dtype=torch.int32, device=self.device)
        bm = torch.empty((self.n, 2), dtype=torch.float64, device=self.device)
        with torch.cuda.device(self.device):
            _check(self._lib.ef21_get_choices(self._h, branch.data_ptr(), bm.data_ptr()))
        return branch, bm

    # -- measurement
    def set_timing(self, enabled: bool) -> None:
        with torch.cuda.device(self.device):
            _check(self._lib.ef21_set_timing(self._h, int(bool(enabled))))

    def get_timing(self, reset: bool = True) -> dict:
        """{kernel class: (milliseconds, launches)} accumulated while timing was enabled."""
        ms = (C.c_double * K_COUNT)()
        cnt = (C.c_int64 * K_COUNT)()
        with torch.cuda.device(self.device):
            _check(self._lib.ef21_get_timing(self._h, C.addressof(ms), C.addressof(cnt), int(reset)))
        return {self._lib.ef21_kernel_name(i).decode(): (ms[i], cnt[i]) for i in range(K_COUNT) if cnt[i]}

    # -- the hot path
    def local_grad(self, x: torch.Tensor | None = None, out: torch.Tensor | None = None) -> torch.Tensor:
        if out is None:
            out = torch.empty((self.n, self.d), dtype=torch.float32, device=self.device)
        with torch.cuda.device(self.device):
            _check(self._lib.ef21_local_grad(self._h, _opt(x, torch.float32, (self.d,)),
                                             _dev(out, torch.float32, (self.n, self.d))))
        return out

    def step(self, grads: torch.Tensor | None = None, order: int = ORDER_GRAD_FIRST) -> None:
        with torch.cuda.device(self.device):
            _check(self._lib.ef21_step(self._h, _opt(grads, torch.float32, (self.n, self.d)), int(order)))
