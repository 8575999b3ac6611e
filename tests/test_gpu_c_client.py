"""The C ABI used from plain C: tests/c_client.c (compiled with gcc against include/ef21.h, linked with libef21.so
and the HIP runtime, no Python and no C++ in the process) runs Top-k through both entry points and one iteration
of Algorithm 2, and checks them against a brute-force selection of its own.  This test runs the executable."""
import os
import subprocess

import pytest

from paper_2106_05203_amd import build

pytestmark = pytest.mark.gpu


def test_plain_c_client_runs_and_agrees():
    # The client is started as a child process, which must happen before this process has touched the GPU (a
    # process that has initialised the GPU should not start other programs).  pytest collects this file before the
    # other GPU tests, so in a run of the whole suite it comes first; after another GPU test, run it by itself.
    import sys
    torch = sys.modules.get("torch")
    if torch is not None and torch.cuda.is_initialized():
        pytest.skip("this process has already initialised the GPU: run tests/test_gpu_c_client.py alone")
    if not os.path.exists(build.C_CLIENT):
        build.build_c_client()
    done = subprocess.run([build.C_CLIENT], capture_output=True, text=True, timeout=120)
    print(done.stdout, done.stderr, flush=True)
    assert done.returncode == 0, f"c_client exited with {done.returncode}: {done.stdout} {done.stderr}"
    assert "all checks passed" in done.stdout
    assert "MISMATCH" not in done.stdout
