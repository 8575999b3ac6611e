"""GPU parity of the batched Top-k (ef21_topk through the C ABI) against the CPU oracle:
positions bit-exact, values bit-exact (they are copies of the inputs)."""
import numpy as np
import pytest

from helpers import same_bits, sampled_positions
from paper_2106_05203_amd import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    from paper_2106_05203_amd import binding
    assert torch.cuda.is_available(), "these tests need the MI355X"
    binding.load_library()
    return torch, binding


def run_gpu(gpu, V, k):
    torch, binding = gpu
    t = torch.from_numpy(np.ascontiguousarray(V, dtype=np.float32)).cuda()
    idx, val = binding.ef21_topk(t, k)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), val.cpu().numpy()


def check(gpu, oracle, V, k, rows=None):
    print(f"topk case n={V.shape[0]} d={V.shape[1]} k={k}", flush=True)
    idx, val = run_gpu(gpu, V, k)
    rows = range(V.shape[0]) if rows is None else rows
    for i in rows:
        ref_idx, ref_val = oracle.topk(V[i].astype(np.float64), k)
        assert np.array_equal(idx[i], ref_idx), f"row {i}: positions differ"
        assert same_bits(val[i], ref_val.astype(np.float32)), f"row {i}: values differ"
    # properties that hold for every row at any size
    assert np.all(np.diff(idx.astype(np.int64), axis=1) > 0)
    assert np.all((idx >= 0) & (idx < V.shape[1]))
    assert same_bits(val, np.take_along_axis(V, idx.astype(np.int64), axis=1))
    return idx, val


def test_tiny_patterns(gpu, oracle):
    pats = [
        [0.0], [-3.0], [0.0, 0.0, 0.0, 0.0], [0.0, -0.0, 0.0, -0.0, 1.0],
        [1.0, -1.0, 1.0, -1.0, 1.0], [3, -5, 1, 5, -2], [5, 4, 3, 2, 1, 0, -1, -2, -3, -4, -5],
        [1e-45, -1e-45, 0.0, 2e-45], [np.inf, -np.inf, 1.0, 3e38],
    ]
    for v in pats:
        v = np.array(v, dtype=np.float32)
        for k in range(1, v.size + 1):
            check(gpu, oracle, v[None, :].repeat(3, axis=0), k)


@pytest.mark.parametrize("d", [1, 2, 63, 64, 65, 127, 1000, 1023, 1024, 1025, 4096, 5000, 16385, 40000])
def test_random_small_rows(gpu, oracle, d):
    rng = np.random.default_rng(d)
    V = rng.standard_normal((5, d)).astype(np.float32)
    V[1] = np.round(V[1] * 2) / 2                      # heavy ties
    V[2] = 0.0                                         # all equal
    V[3, ::3] = -V[3, (d // 2) % d]                    # one value repeated with flipped sign
    V[4] *= np.float32(1e-41)                          # subnormals
    for k in sorted(k for k in {1, 2, d // 100, d // 2, d - 1, d} if 1 <= k <= d):
        check(gpu, oracle, V, k)


@pytest.mark.parametrize("d", [200, 256, 257, 5000, 9000, 300_000])
@pytest.mark.parametrize("crowd", [3, 255, 256, 257, 600])
def test_threshold_inside_a_bin_of_near_equal_magnitudes(gpu, oracle, d, crowd):
    """`crowd` entries share the twelve leading key bits (values in [1, 1.0625), many of them exactly equal up
    to sign), a few are larger, the rest tiny; k runs through the crowd, so the threshold key and the tie quota
    are decided among them: by ranking them directly up to 256, by further histogram passes beyond."""
    crowd = min(crowd, d - 2)
    rng = np.random.default_rng(d * 1000 + crowd)
    V = (1e-4 * rng.standard_normal((4, d))).astype(np.float32)
    for i in range(4):
        pos = rng.choice(d, size=crowd + 2, replace=False)
        vals = 1.0 + rng.integers(0, 8, size=crowd) / 128.0            # 8 distinct magnitudes: heavy ties
        V[i, pos[:crowd]] = (vals * rng.choice([-1.0, 1.0], size=crowd)).astype(np.float32)
        V[i, pos[crowd:]] = [3.0, -2.5]
    for k in sorted({1, 2, 3, 2 + crowd // 3, 2 + crowd // 2, 1 + crowd, 2 + crowd, min(d, 3 + crowd)}):
        check(gpu, oracle, V, k)


@pytest.mark.parametrize("d", [16384, 20001, 50000, 61440, 61441])
@pytest.mark.parametrize("k", [1, 37, 1000, 1024, 1025])
def test_rows_held_in_lds_as_key_prefixes(gpu, oracle, d, k):
    """Rows of 16 384 to 61 440 entries with k <= 1024 are selected by one workgroup that keeps 16 bits of every key
    in LDS (the sizes around those limits take the other kernels).  Rows: Gaussian; heavy exact ties (the list
    of entries above the bound overflows); a crowded bin of near-equal magnitudes with ties (narrowed by four
    bits, or given up); fewer non-zeros than k (the threshold is zero); infinities and a row of one value."""
    rng = np.random.default_rng(d + k)
    V = rng.standard_normal((7, d)).astype(np.float32)
    V[1] = np.round(V[1] * 2) / 2
    V[2] = (1e-3 * rng.standard_normal(d)).astype(np.float32)
    crowd = rng.choice(d, size=3000, replace=False)
    V[2, crowd] = ((1.0 + rng.integers(0, 2000, size=3000) / 32768.0) * rng.choice([-1.0, 1.0], size=3000)).astype(np.float32)
    V[3] = 0.0
    few = rng.choice(d, size=min(k, 700) // 2 + 1, replace=False)
    V[3, few] = rng.standard_normal(few.size).astype(np.float32)
    V[4, rng.choice(d, size=5, replace=False)] = [np.inf, -np.inf, 3e38, -3e38, np.inf]
    V[5] = -2.5
    V[6] = (rng.standard_t(3, size=d) * 1e-3).astype(np.float32)
    check(gpu, oracle, V, k)


@pytest.mark.parametrize("d,k", [(70001, 700), (262144, 5), (300007, 3000), (1_000_003, 999), (70001, 1), (1_000_003, 1),
                                 (262144, 1)])
def test_long_rows_ragged(gpu, oracle, d, k):
    V = workloads.topk_rows(3, d, seed=d % 1000)
    check(gpu, oracle, V, k)
    W = workloads.force_threshold_ties(V, k, copies=8, seed=1)
    check(gpu, oracle, W, k)


def test_long_rows_degenerate(gpu, oracle):
    d = 200_000
    V = np.zeros((4, d), dtype=np.float32)
    V[1] = 1.5
    V[1, ::2] = -1.5
    V[2, 1000:] = np.float32(2.0) ** -130               # subnormal plateau
    V[3] = np.arange(d, dtype=np.float32)[::-1]
    for k in (1, 777, d // 2, d):
        check(gpu, oracle, V, k)


@pytest.mark.parametrize("k", [10000, 60000])
def test_long_rows_misleading_sample(gpu, oracle, k):
    """The long-row path guesses a candidate threshold from 64 evenly spaced pieces of 64 entries.
    Here the large values sit exactly on those pieces and nowhere else, so the guess keeps far fewer
    than k candidates and the exact per-row algorithm has to take over (both the small-k and the
    large-k variant of the candidate stage)."""
    d = 300_000
    rng = np.random.default_rng(k)
    V = (rng.standard_normal((3, d)) * 1e-3).astype(np.float32)
    pos = sampled_positions(d)
    V[:, pos] = (1.0 + rng.random((3, pos.size))).astype(np.float32)
    V[2] = np.abs(V[2])
    check(gpu, oracle, V, k)


@pytest.mark.parametrize("k", [10000, 60000])
def test_long_rows_sample_far_too_low(gpu, oracle, k):
    """The opposite mistake: the sampled pieces hold tiny values and everything else is large, so the
    guessed threshold admits every entry and the k-th largest magnitude lies far above it (above the
    window of leading digits the collect pass counts, for the large-k variant).  Same results."""
    d = 300_000
    rng = np.random.default_rng(k + 1)
    V = (1000.0 * (1.0 + rng.random((3, d)))).astype(np.float32)
    pos = sampled_positions(d)
    V[:, pos] = (rng.standard_normal((3, pos.size)) * 1e-3).astype(np.float32)
    V[1] = -V[1]
    check(gpu, oracle, V, k)


@pytest.mark.parametrize("n,d,k", [(2, 1_500_000, 100_000), (1, 2_000_001, 700_000), (3, 400_000, 399_999)])
def test_long_rows_large_k(gpu, oracle, n, d, k):
    """k large enough that the candidates are processed by many workgroups per row."""
    V = workloads.topk_rows(n, d, seed=k % 97)
    check(gpu, oracle, V, k)
    check(gpu, oracle, workloads.force_threshold_ties(V, k, copies=8, seed=3), k)


@pytest.mark.timeout(300)
@pytest.mark.parametrize("k", [1, 1000, 10000])
def test_config1_full_size(gpu, oracle, k):
    """n = 20 rows of 10^6 N(0,1) values with 1 % exact duplicates (+a / -a), the size the
    throughput is quoted on, and the variant whose threshold magnitude is tied."""
    V = workloads.topk_rows(20, 1_000_000, seed=0)
    check(gpu, oracle, V, k)
    W = workloads.force_threshold_ties(V[:4], k, copies=8, seed=2)
    check(gpu, oracle, W, k)


def test_random_shapes(gpu, oracle):
    """Sixty seeded draws of (n, d, k, kind of row) across all the kernels' ranges of d and k."""
    rng = np.random.default_rng(2106)
    for case in range(60):
        d = int(np.exp(rng.uniform(0.0, np.log(400_000))))
        n = int(rng.integers(1, 5))
        k = int(min(d, max(1, [1, 2, rng.integers(1, 64), d // 100 + 1, d // 3 + 1, d][rng.integers(0, 6)])))
        kind = int(rng.integers(0, 5))
        if kind == 0:
            V = rng.standard_normal((n, d))
        elif kind == 1:
            V = np.round(rng.standard_normal((n, d)) * 3) / 3          # heavy ties
        elif kind == 2:
            V = rng.standard_t(2, size=(n, d)) * 1e-4                  # heavy tails
        elif kind == 3:
            V = np.zeros((n, d))
            nz = rng.integers(0, d, size=max(1, d // 50))
            V[:, nz] = rng.standard_normal((n, nz.size))               # mostly zeros
        else:
            V = np.exp(rng.uniform(-80, 80, size=(n, d))) * rng.choice([-1.0, 1.0], size=(n, d))   # all exponents
        check(gpu, oracle, V.astype(np.float32), k)


def test_deterministic(gpu):
    torch, binding = gpu
    V = torch.from_numpy(workloads.topk_rows(6, 300_000, seed=9)).cuda()
    a = binding.ef21_topk(V, 3000)
    b = binding.ef21_topk(V, 3000)
    torch.cuda.synchronize()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1].view(torch.int32), b[1].view(torch.int32))


def test_error_codes(gpu):
    torch, binding = gpu
    V = torch.zeros((2, 10), device="cuda")
    for k in (0, 11):
        with pytest.raises(binding.EF21Error) as e:
            binding.ef21_topk(V, k)
        assert e.value.code == binding.EF21_EINVAL
    with pytest.raises(TypeError):
        binding.ef21_topk(V.double(), 1)


def test_calls_on_two_streams_overlap_safely(gpu, oracle):
    """ef21_topk keeps one workspace per stream: calls enqueued on two streams without any ordering between them
    (long rows, so both use a workspace) must each give their own input's selection."""
    torch, binding = gpu
    n, d, k = 6, 400_000, 4000
    A = torch.from_numpy(workloads.topk_rows(n, d, seed=21)).cuda()
    B = torch.from_numpy(workloads.topk_rows(n, d, seed=22)).cuda()
    torch.cuda.synchronize()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    outs = []
    for rep in range(6):
        with torch.cuda.stream(s1):
            ia, va = binding.ef21_topk(A, k)
        with torch.cuda.stream(s2):
            ib, vb = binding.ef21_topk(B, k + rep)
        outs.append((ia, va, ib, vb))
    torch.cuda.synchronize()
    ref_a = oracle.topk(A[2].cpu().numpy().astype(np.float64), k)
    for rep, (ia, va, ib, vb) in enumerate(outs):
        assert np.array_equal(ia[2].cpu().numpy(), ref_a[0]) and same_bits(va[2].cpu().numpy(), ref_a[1].astype(np.float32))
        ref_b = oracle.topk(B[4].cpu().numpy().astype(np.float64), k + rep)
        assert np.array_equal(ib[4].cpu().numpy(), ref_b[0]) and same_bits(vb[4].cpu().numpy(), ref_b[1].astype(np.float32))
        assert same_bits(va.cpu().numpy(), np.take_along_axis(A.cpu().numpy(), ia.cpu().numpy().astype(np.int64), axis=1))
        assert same_bits(vb.cpu().numpy(), np.take_along_axis(B.cpu().numpy(), ib.cpu().numpy().astype(np.int64), axis=1))


@pytest.mark.parametrize("kind", ["equal", "distinct"])
def test_crowded_threshold_bin_on_long_rows(gpu, oracle, kind):
    """Thousands of candidates share the histogram bin of the threshold: 6000 copies of one magnitude (no ranking
    needed: ties go to the lower positions), or 6000 consecutive floats (too many to rank: the exact per-row
    algorithm takes over).  k is chosen so that the threshold falls inside the cluster."""
    rng = np.random.default_rng(8)
    n, d = 3, 250_000
    V = (0.1 * rng.standard_normal((n, d))).astype(np.float32)
    for i in range(n):
        pos = rng.choice(d, size=6000, replace=False)
        if kind == "equal":
            V[i, pos] = np.where(rng.random(6000) < 0.5, 1.0, -1.0).astype(np.float32)
        else:
            bits = np.float32(1.0).view(np.uint32) + rng.permutation(6000).astype(np.uint32)
            V[i, pos] = bits.view(np.float32) * np.where(rng.random(6000) < 0.5, 1.0, -1.0).astype(np.float32)
    for k in (3000, 5999, 6001):
        check(gpu, oracle, V, k)
