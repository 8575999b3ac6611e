"""Pins for the oracle's Top-k against what the paper's definition fixes (Section 2.1,
Appendix F.2).  No GPU."""
import itertools
import json
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def subset_search_topk(v, k):
    """The definition, by exhaustion: the unique k-subset S such that every j outside S is
    beaten by every i inside S, where i beats j if |v_i| > |v_j| or (|v_i| == |v_j| and i < j)."""
    d = len(v)
    mag = [abs(float(t)) for t in v]

    def beats(i, j):
        return mag[i] > mag[j] or (mag[i] == mag[j] and i < j)

    hits = []
    for S in itertools.combinations(range(d), k):
        inside = set(S)
        if all(beats(i, j) for i in S for j in range(d) if j not in inside):
            hits.append(S)
    assert len(hits) == 1, "the definition with the tie rule selects exactly one subset"
    return list(hits[0])


def test_hand_examples(oracle):
    cases = json.load(open(os.path.join(GOLDEN, "topk_hand_examples.json")))["cases"]
    for c in cases:
        idx, val = oracle.topk(np.array(c["v"], dtype=np.float64), c["k"])
        assert idx.tolist() == c["idx"], c
        assert val.tolist() == [float(t) for t in c["val"]], c


def test_exhaustive_small_alphabet(oracle):
    """Every vector of length <= 5 over an alphabet with zeros, signed zeros and +-a pairs,
    every k: the oracle equals the exhaustive subset search."""
    alphabet = [0.0, -0.0, 1.0, -1.0, 2.5, -2.5]
    for d in range(1, 6):
        for v in itertools.product(alphabet, repeat=d):
            va = np.array(v, dtype=np.float64)
            for k in range(1, d + 1):
                idx, val = oracle.topk(va, k)
                assert idx.tolist() == subset_search_topk(v, k), (v, k)
                # values are the signed inputs at the kept positions (bit pattern included)
                assert np.array_equal(np.signbit(val), np.signbit(va[idx]))
                assert np.array_equal(val, va[idx])


def test_random_against_subset_search(oracle):
    rng = np.random.default_rng(5)
    for trial in range(200):
        d = int(rng.integers(1, 9))
        v = rng.integers(-3, 4, size=d).astype(np.float64) * 0.5   # many ties
        for k in range(1, d + 1):
            idx, _ = oracle.topk(v, k)
            assert idx.tolist() == subset_search_topk(v, k), (v, k)


@pytest.mark.parametrize("d,k", [(1, 1), (17, 1), (17, 5), (1000, 10), (1000, 999), (4096, 41), (5000, 5000)])
def test_definition_properties(oracle, d, k):
    rng = np.random.default_rng(d * 7919 + k)
    v = rng.standard_normal(d).astype(np.float32).astype(np.float64)
    v[rng.integers(0, d, size=max(1, d // 50))] = v[rng.integers(0, d, size=max(1, d // 50))]  # some ties
    idx, val = oracle.topk(v, k)
    assert idx.shape == (k,) and val.shape == (k,)
    assert np.all(np.diff(idx) > 0), "exactly k distinct positions, ascending"
    assert np.array_equal(val, v[idx])
    kept = np.zeros(d, dtype=bool)
    kept[idx] = True
    if k < d:
        # no dropped entry is larger than a kept one
        assert np.abs(v[~kept]).max() <= np.abs(v[kept]).min()
        # ties at the threshold go to the lower indices
        thr = np.abs(v[kept]).min()
        tied_kept = np.flatnonzero(kept & (np.abs(v) == thr))
        tied_drop = np.flatnonzero(~kept & (np.abs(v) == thr))
        if tied_drop.size:
            assert tied_kept.max() < tied_drop.min()
    # contraction: ||C(v) - v||^2 <= (1 - k/d) ||v||^2  (eq. (3) with alpha = k/d)
    dense = oracle.topk_dense(v, k)
    assert np.sum((dense - v) ** 2) <= (1.0 - k / d) * np.sum(v ** 2) * (1 + 1e-12)


def test_k_equals_d_is_identity(oracle):
    v = np.random.default_rng(0).standard_normal(257)
    assert np.array_equal(oracle.topk_dense(v, v.size), v)


def test_k1_is_first_argmax(oracle):
    rng = np.random.default_rng(3)
    for _ in range(100):
        v = rng.integers(-5, 6, size=50).astype(np.float64)
        idx, val = oracle.topk(v, 1)
        j = int(np.argmax(np.abs(v)))          # numpy returns the first maximiser
        assert idx[0] == j and val[0] == v[j]


def test_matches_library_stable_sort(oracle):
    """Same result as numpy's stable argsort on -|v| (a library routine as the sort step)."""
    rng = np.random.default_rng(11)
    for d, k in [(10_000, 100), (65_537, 3000)]:
        v = rng.standard_normal(d).astype(np.float32).astype(np.float64)
        v[::97] = v[5]
        v[1::89] = -v[5]
        order = np.argsort(-np.abs(v), kind="stable")[:k]
        idx, val = oracle.topk(v, k)
        assert np.array_equal(idx, np.sort(order).astype(np.int32))
        assert np.array_equal(val, v[idx])


def test_bad_arguments(oracle):
    v = np.zeros(4)
    for k in (0, 5, -1):
        with pytest.raises(ValueError):
            oracle.topk(v, k)
