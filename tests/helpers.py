"""Shared helpers of the GPU parity tests."""
import numpy as np


def close_per_coordinate(got, ref, rel=1e-5):
    """|got - ref| <= rel * max(|ref|, rel * max|ref|) per coordinate (ref = oracle).
    The floor keeps coordinates that cancel to (almost) zero from demanding absolute exactness."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    floor = rel * np.max(np.abs(ref)) if ref.size else 0.0
    bound = rel * np.maximum(np.abs(ref), floor)
    err = np.abs(got - ref)
    bad = err > bound
    return not bad.any(), (float(err.max()) if err.size else 0.0, int(bad.sum()))


def same_bits(a, b):
    """Bitwise equality of two float32 arrays (so -0.0 != +0.0 and equal NaNs compare equal)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    b = np.ascontiguousarray(b, dtype=np.float32)
    return a.shape == b.shape and np.array_equal(a.view(np.uint32), b.view(np.uint32))


class RoundingBudget:
    """Per-coordinate absolute error that fp32 arithmetic may put between the GPU's g, x and the
    oracle's (which computes lines 8 and 3 of Algorithm 2 in fp64 and rounds once).

    Line 8 on the GPU is n fp32 atomic additions of val * (1/n) into g_j: each addition, the
    product and the rounding of 1/n contribute at most one unit roundoff u = 2^-24 relative to the
    magnitudes involved, so |g_gpu - g_ref| grows per step by at most (n + 2) u (|g_j| + mean_i |c_ij|).
    Line 3 is one fused multiply-add: 2 u (|x_j| + gamma |g_j|) covers both sides' rounding, plus
    gamma times the error already in g.  Budgets add up over steps until `reset` (state resynchronised).
    A coordinate whose value cancels to almost zero therefore keeps a floor proportional to its
    operands instead of an unattainable relative bound.
    """
    U = 2.0 ** -24

    def __init__(self, n, d, gamma):
        self.n, self.gamma = n, gamma
        self.g = np.zeros(d)
        self.x = np.zeros(d)

    def reset(self):
        self.g[:] = 0.0
        self.x[:] = 0.0

    def compress_update(self, g_before, msg_idx, msg_val):
        mean_abs_c = np.zeros_like(self.g)
        np.add.at(mean_abs_c, np.asarray(msg_idx).reshape(-1), np.abs(np.asarray(msg_val)).reshape(-1) / self.n)
        self.g += (self.n + 2) * self.U * (np.abs(g_before) + mean_abs_c)

    def model_step(self, x_before, g_used):
        self.x += 2 * self.U * (np.abs(x_before) + self.gamma * np.abs(g_used)) + self.gamma * self.g

    def check(self, got, ref, which, rel=1e-5):
        got = np.asarray(got, dtype=np.float64)
        ref = np.asarray(ref, dtype=np.float64)
        bound = rel * np.abs(ref) + (self.g if which == "g" else self.x)
        err = np.abs(got - ref)
        bad = err > bound
        return not bad.any(), (float(err.max()), int(bad.sum()))


def gradient_rounding_floor(A, y, x, dot_depth, sum_depth, lam=0.1):
    """First-order bound on what fp32 rounding can do to one worker's logistic gradient
    grad_j = (1/m) sum_l r_l a_lj,  r_l = -y_l sigma(-y_l z_l),  z_l = a_l^T x  (A [m][d]: dense, or a
    scipy.sparse matrix):
      - z_l carries at most dot_depth * u * sum_j |a_lj x_j| (a dot product summed in `dot_depth` levels),
        which moves r_l by sigma_l (1 - sigma_l) times that;
      - the sum over rows carries at most sum_depth * u * |r_l a_lj| per term.
    Returned per coordinate; a coordinate that cancels to almost zero keeps this floor."""
    u = 2.0 ** -24
    sparse = hasattr(A, "tocsr")                       # a scipy.sparse matrix is taken as it is
    A = A.astype(np.float64) if sparse else np.asarray(A, dtype=np.float64)
    absA = abs(A)
    x = np.asarray(x, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    z = A @ x
    sig = 1.0 / (1.0 + np.exp(y * z))                 # |r_l|
    dz = dot_depth * u * (absA @ np.abs(x))
    dr = sig * (1.0 - sig) * dz + sum_depth * u * sig
    reg = 2.0 * lam * np.abs(x) / (1.0 + x * x) ** 2               # the regulariser term's own rounding
    return np.asarray(absA.T @ dr).reshape(-1) / A.shape[0] + 8 * u * reg
