"""The boundary is a C ABI: a plain C99 program includes include/ll.h, links the shared library and
uses the host entry points (no GPU needed)."""
import os
import subprocess

import pytest

import paper_2505_23819_amd as ll

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_c99_client_builds_and_runs(tmp_path):
    exe = str(tmp_path / "abi_check")
    libdir = os.path.dirname(ll.LIBRARY_PATH)
    cmd = ["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "c", "abi_check.c"), "-o", exe, "-L", libdir, "-lll355", "-Wl,-rpath," + libdir]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    res = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, res.stderr
    assert res.stdout.strip() == "ok"


@pytest.mark.gpu
def test_c_client_on_the_gpu(tmp_path):
    """The same boundary from plain C on a GPU: HIP runtime C API for memory, ll_convert and
    ll_gather, checked against the oracle's C functions inside the C program."""
    import oracle
    exe = str(tmp_path / "gpu_client")
    libdir, odir = os.path.dirname(ll.LIBRARY_PATH), os.path.dirname(oracle.build())
    cmd = ["gcc", "-std=c99", "-O1", "-Wall", "-Wextra", "-I", os.path.join(ROOT, "include"), "-I", "/opt/rocm/include",
           os.path.join(ROOT, "tests", "c", "gpu_client.c"), "-o", exe,
           "-L", libdir, "-lll355", "-L", odir, "-lll_oracle", "-L", "/opt/rocm/lib", "-lamdhip64",
           "-Wl,-rpath," + libdir, "-Wl,-rpath," + odir, "-Wl,-rpath,/opt/rocm/lib"]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    res = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, res.stderr
    assert res.stdout.strip() == "ok"
