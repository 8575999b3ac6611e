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
