"""ef21_topk_static (the Top-k entry point that allocates nothing: its workspace is a static device array) against
ef21_topk, through the C ABI: positions and values bit for bit, on calls that follow one another with different
shapes (the array keeps the previous call's contents), the second smaller than the first."""
import ctypes as C

import numpy as np
import pytest

from helpers import same_bits
from paper_2106_05203_amd import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    from paper_2106_05203_amd import binding
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch, binding, binding.load_library()


def both(gpu, V, k):
    """(idx, val) of ef21_topk and of ef21_topk_static on the same rows, by raw C-ABI calls."""
    torch, binding, lib = gpu
    n, d = V.shape
    rows = torch.from_numpy(np.ascontiguousarray(V, dtype=np.float32)).cuda()
    out = []
    for fn in (lib.ef21_topk, lib.ef21_topk_static):
        idx = torch.full((n, k), -7, dtype=torch.int32, device="cuda")
        val = torch.full((n, k), np.nan, dtype=torch.float32, device="cuda")
        rc = fn(C.c_void_p(rows.data_ptr()), n, d, k, C.c_void_p(idx.data_ptr()), C.c_void_p(val.data_ptr()),
                C.c_void_p(torch.cuda.current_stream().cuda_stream))
        assert rc == binding.EF21_OK, lib.ef21_last_error().decode()
        torch.cuda.synchronize()
        out.append((idx.cpu().numpy(), val.cpu().numpy()))
    return out


def agree(gpu, V, k):
    print(f"static Top-k case n={V.shape[0]} d={V.shape[1]} k={k}", flush=True)
    (idx_a, val_a), (idx_s, val_s) = both(gpu, V, k)
    assert np.array_equal(idx_a, idx_s), "positions differ between ef21_topk and ef21_topk_static"
    assert same_bits(val_a, val_s), "values differ between ef21_topk and ef21_topk_static"
    return idx_s, val_s


def test_two_calls_in_a_row_second_smaller(gpu, oracle):
    # long rows, many workgroups per row and the many-kernel candidate stages (k large), then fewer, shorter rows
    # with the one-workgroup select (k small) on the same scratch
    V1 = workloads.topk_rows(4, 300_000, seed=11)
    idx, val = agree(gpu, V1, 30_000)
    ref_idx, ref_val = oracle.topk(V1[2].astype(np.float64), 30_000)
    assert np.array_equal(idx[2], ref_idx) and same_bits(val[2], ref_val.astype(np.float32))
    V2 = workloads.topk_rows(3, 70_001, seed=12)
    idx, val = agree(gpu, V2, 700)
    for i in range(3):
        ref_idx, ref_val = oracle.topk(V2[i].astype(np.float64), 700)
        assert np.array_equal(idx[i], ref_idx) and same_bits(val[i], ref_val.astype(np.float32))
    # and back to a larger shape, k = 1 (the running-maximum kernels, which keep a word of the workspace at zero)
    V3 = workloads.topk_rows(5, 200_000, seed=13)
    agree(gpu, V3, 1)
    agree(gpu, V1, 2)


def test_shapes_without_workspace_and_ties(gpu):
    rng = np.random.default_rng(5)
    agree(gpu, rng.standard_normal((6, 5000)).astype(np.float32), 50)          # one workgroup per row
    agree(gpu, rng.standard_normal((3, 40_000)).astype(np.float32), 400)       # 16-bit prefixes in LDS
    V = np.round(rng.standard_normal((2, 100_000)) * 4).astype(np.float32) / 4  # heavy ties, long rows
    agree(gpu, V, 5000)
    agree(gpu, np.zeros((2, 66_000), dtype=np.float32), 3000)                  # all equal: the slots fill up


def test_limit_is_an_error_not_an_allocation(gpu):
    torch, binding, lib = gpu
    n, d, k = 10, 1_000_000, 2000                    # about 81 MB of workspace: beyond the static 64 MiB
    rows = torch.zeros((n, d), dtype=torch.float32, device="cuda")
    idx = torch.zeros((n, k), dtype=torch.int32, device="cuda")
    val = torch.zeros((n, k), dtype=torch.float32, device="cuda")
    rc = lib.ef21_topk_static(C.c_void_p(rows.data_ptr()), n, d, k, C.c_void_p(idx.data_ptr()),
                              C.c_void_p(val.data_ptr()), None)
    assert rc == binding.EF21_EINVAL
    assert b"static scratch" in lib.ef21_last_error()
    assert lib.ef21_topk_static(None, 1, 4, 1, C.c_void_p(idx.data_ptr()), C.c_void_p(val.data_ptr()), None) == binding.EF21_EINVAL


def test_static_entry_point_under_graph_capture(gpu):
    """One of the callers it is for: a HIP graph.  The call is captured once (after an eager call of the same shape,
    which does the per-device set-up) and replayed on new contents of the same input buffer, with eager work and
    synchronisations between the replays; every replay must equal an eager ef21_topk of the same contents."""
    torch, binding, lib = gpu
    n, d, k = 3, 150_000, 1200
    rows = torch.zeros((n, d), dtype=torch.float32, device="cuda")
    idx = torch.full((n, k), -7, dtype=torch.int32, device="cuda")
    val = torch.zeros((n, k), dtype=torch.float32, device="cuda")
    side = torch.cuda.Stream()

    def static_call(stream):
        rc = lib.ef21_topk_static(C.c_void_p(rows.data_ptr()), n, d, k, C.c_void_p(idx.data_ptr()),
                                  C.c_void_p(val.data_ptr()), C.c_void_p(stream.cuda_stream))
        assert rc == binding.EF21_OK, lib.ef21_last_error().decode()

    rows.copy_(torch.from_numpy(workloads.topk_rows(n, d, seed=20)))
    torch.cuda.synchronize()
    static_call(side)                                     # eager: set-up happens here, outside the capture
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        static_call(side)
    for seed in (21, 22, 23):
        V = workloads.topk_rows(n, d, seed=seed)
        if seed == 23:
            V = np.round(V * 2) / 2                       # many equal magnitudes
        rows.copy_(torch.from_numpy(np.ascontiguousarray(V, dtype=np.float32)))
        idx.fill_(-7)
        val.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got_idx, got_val = idx.cpu().numpy().copy(), val.cpu().numpy().copy()
        ref_idx = torch.empty_like(idx)
        ref_val = torch.empty_like(val)
        binding.ef21_topk(rows, k, ref_idx, ref_val)      # eager work between the replays
        torch.cuda.synchronize()
        print(f"graph replay of ef21_topk_static, seed {seed}", flush=True)
        assert np.array_equal(got_idx, ref_idx.cpu().numpy())
        assert same_bits(got_val, ref_val.cpu().numpy())
