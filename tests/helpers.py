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


def sampled_positions(d):
    """The entries of a long row (d > 4096) that the library's long-row Top-k samples to guess its candidate
    threshold: 64 evenly spaced pieces of 64 entries (the constants of csrc/topk_split.hip, restated here so that
    tests can build rows on which the sample misleads)."""
    return np.concatenate([(p * (d - 64)) // 63 + np.arange(64) for p in range(64)])


def same_bits(a, b):
    """Bitwise equality of two float32 arrays (so -0.0 != +0.0 and equal NaNs compare equal)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    b = np.ascontiguousarray(b, dtype=np.float32)
    return a.shape == b.shape and np.array_equal(a.view(np.uint32), b.view(np.uint32))


class RoundingBudget:
    """Per-coordinate absolute error that fp32 arithmetic may put between the GPU's g, x and the
    oracle's (which computes lines 8 and 3 of Algorithm 2 in fp64 and rounds once), to first order in the unit
    roundoff u = 2^-24.

    Line 8 on the GPU: the messages that hit coordinate j are added in fp32 in worker order (c_j of them: c_j - 1
    additions, each off by at most u times the partial sum, so at most (c_j - 1) u sum_i |c_ij| in all), then
    g_j + sum * (1/n) as one fused multiply-add with 1/n rounded to fp32 (u |sum| / n) and one rounding of the
    result (u |g_j^new|); the oracle rounds its fp64 result once more (u |g_j^new|).  With
    a_j = (1/n) sum_i |c_ij| and |g_j^new| <= |g_j| + a_j that is at most u ((c_j + 2) a_j + 2 |g_j|) per update;
    a coordinate that no message hits keeps its bits on both sides.
    Line 3 is one fused multiply-add: one rounding on each side, 2 u (|x_j| + gamma |g_j|), the stepsize held in
    fp32 by the library and in fp64 by the oracle, u gamma |g_j|, plus gamma times the error already in g.
    Budgets add up over steps until `reset` (state resynchronised).  A coordinate whose value cancels to almost
    zero therefore keeps a floor proportional to its operands instead of an unattainable relative bound.
    `check` also reports how much of the allowance (1e-5 |ref| + budget) the worst coordinate used.
    """
    U = 2.0 ** -24

    def __init__(self, n, d, gamma):
        self.n, self.gamma = n, gamma
        self.g = np.zeros(d)
        self.x = np.zeros(d)
        self.used = {}          # which -> largest err / allowance seen

    def reset(self):
        self.g[:] = 0.0
        self.x[:] = 0.0

    def compress_update(self, g_before, msg_idx, msg_val):
        mean_abs_c = np.zeros_like(self.g)
        hits = np.zeros_like(self.g)
        flat = np.asarray(msg_idx).reshape(-1)
        np.add.at(mean_abs_c, flat, np.abs(np.asarray(msg_val)).reshape(-1) / self.n)
        np.add.at(hits, flat, 1.0)
        self.g += self.U * ((hits + 2.0) * mean_abs_c + 2.0 * np.abs(g_before) * (hits > 0))

    def model_step(self, x_before, g_used):
        self.x += self.U * (2.0 * np.abs(x_before) + 3.0 * self.gamma * np.abs(g_used)) + self.gamma * self.g

    def check(self, got, ref, which, rel=1e-5):
        got = np.asarray(got, dtype=np.float64)
        ref = np.asarray(ref, dtype=np.float64)
        bound = rel * np.abs(ref) + (self.g if which == "g" else self.x)
        err = np.abs(got - ref)
        bad = err > bound
        with np.errstate(divide="ignore", invalid="ignore"):
            share = np.where(bound > 0, err / bound, np.where(err > 0, np.inf, 0.0))
        used = float(share.max()) if share.size else 0.0
        self.used[which] = max(self.used.get(which, 0.0), used)
        print(f"  {which}: worst coordinate uses {used:.3f} of its allowance (max err {err.max() if err.size else 0.0:.3e})",
              flush=True)
        return not bad.any(), (float(err.max()) if err.size else 0.0, int(bad.sum()))


def gradient_rounding_floor(A, y, x, dot_depth, sum_depth, lam=0.1):
    """First-order bound on what fp32 rounding can do to one worker's logistic gradient
    grad_j = (1/m) sum_l r_l a_lj,  r_l = -y_l sigma(-y_l z_l),  z_l = a_l^T x  (A [m][d]: dense, or a
    scipy.sparse matrix):
      - z_l carries at most dot_depth * u * sum_j |a_lj x_j| (a dot product summed in `dot_depth` levels),
        which moves r_l by sigma_l (1 - sigma_l) times that;
      - the sum over rows carries at most sum_depth * u * |r_l a_lj| per term.
    Returned per coordinate; a coordinate that cancels to almost zero keeps this floor.
    The worst case (every rounding off by a full u, all in one direction) is halved: measured over all the GPU
    tests the kernels' error stays below a tenth of the worst case, so half of it still leaves a factor of five
    while keeping the floor small next to the gradient (the tests assert: median below 2e-5 of the largest entry)."""
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
    return 0.5 * (np.asarray(absA.T @ dr).reshape(-1) / A.shape[0] + 8 * u * reg)
