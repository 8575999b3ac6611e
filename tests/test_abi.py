"""The C-ABI library loads and exports every symbol include/ef21.h declares; argument errors
that are detected before any HIP call are reported without a GPU.  No compute calls."""
import ctypes as C
import os
import re

import pytest

from paper_2106_05203_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2106_05203_amd import build
        build.build_library()
    return binding.load_library()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "ef21.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ef21_[a-z_]+)\s*\(", text)))


def test_header_symbols_exported(lib):
    names = declared_symbols()
    assert set(names) == set(binding.SYMBOLS), "binding.SYMBOLS must list exactly the header's functions"
    raw = C.CDLL(binding.LIB_PATH)
    for name in names:
        assert hasattr(raw, name), f"{name} is declared in include/ef21.h but not exported"


@pytest.mark.parametrize("compiler,std", [("gcc", "-std=c99"), ("g++", "-std=c++11")])
def test_header_is_plain_c_and_cxx(compiler, std, tmp_path):
    """include/ef21.h alone (only <stdint.h> beneath it) compiles as C99 and as C++11 without warnings."""
    import subprocess
    src = tmp_path / ("use_header.c" if compiler == "gcc" else "use_header.cpp")
    src.write_text('#include "ef21.h"\nint main(void) { return ef21_last_error() == 0 && EF21_OK; }\n')
    subprocess.check_call([compiler, std, "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only",
                           "-I", os.path.join(ROOT, "include"), str(src)])


def test_argument_errors_need_no_gpu(lib):
    buf = (C.c_float * 8)()
    ibuf = (C.c_int32 * 8)()
    ptr, iptr = C.addressof(buf), C.addressof(ibuf)
    bad = [
        (ptr, 0, 4, 1, iptr, ptr),          # n < 1
        (ptr, 1, 0, 1, iptr, ptr),          # d < 1
        (ptr, 1, 4, 0, iptr, ptr),          # k < 1
        (ptr, 1, 4, 5, iptr, ptr),          # k > d
        (ptr, 1, 2 ** 31, 1, iptr, ptr),    # d >= 2^31
        (None, 1, 4, 1, iptr, ptr),         # NULL rows
        (ptr, 1, 4, 1, None, ptr),          # NULL out_idx
        (ptr, 1, 4, 1, iptr, None),         # NULL out_val
    ]
    for rows, n, d, k, oi, ov in bad:
        assert lib.ef21_topk(rows, n, d, k, oi, ov, None) == binding.EF21_EINVAL
        assert lib.ef21_last_error() != b""
    assert not lib.ef21_create(0, 4, 1, 0.1)
    assert not lib.ef21_create(1, 4, 5, 0.1)
    assert not lib.ef21_create(1, 4, 1, 0.0)
    assert not lib.ef21_create(1, 4, 1, float("nan"))
    assert not lib.ef21_create(1, 4, 1, float("inf"))
    assert lib.ef21_destroy(None) == binding.EF21_OK
    for call in (lambda: lib.ef21_step(None, None, 0), lambda: lib.ef21_local_grad(None, None, ptr),
                 lambda: lib.ef21_set_state(None, None, None, None), lambda: lib.ef21_get_state(None, None, None, None),
                 lambda: lib.ef21_get_messages(None, None, None), lambda: lib.ef21_set_stream(None, None),
                 lambda: lib.ef21_set_problem_dense(None, ptr, ptr, 1, 0.1),
                 lambda: lib.ef21_set_problem_csr(None, ptr, ptr, ptr, ptr, 1, 0.1)):
        assert call() == binding.EF21_EINVAL


def test_binding_refuses_host_tensors(lib):
    import torch
    with pytest.raises(TypeError):
        binding.ef21_topk(torch.zeros(2, 8), 1)
