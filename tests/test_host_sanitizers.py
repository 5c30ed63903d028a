"""The host side of the library (F2 algebra, planners, gather chooser, options, C ABI checks) built
with g++ under AddressSanitizer and UndefinedBehaviorSanitizer against stub launchers, and driven
by a bounded, seeded fuzz through the C ABI: random layouts (arbitrary XOR columns, distributed,
broadcasting, memory, affine), element widths, axes and option sets, including option values outside
their documented domains.  Any sanitizer report, unexpected status or crash fails the test.
A second program uses shared layouts and plans from eight threads at once under ThreadSanitizer.  No GPU."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2505_23819_amd", "csrc")
HOST_SOURCES = ["f2.cpp", "plan.cpp", "plan_vec.cpp", "plan_pull.cpp", "plan_tr.cpp", "algebra.cpp", "families.cpp",
                "options.cpp", "run.cpp", "capi.cpp"]


@pytest.fixture(scope="module")
def fuzz_binary(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("san") / "host_fuzz")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-fno-omit-frame-pointer", "-Wall", "-Wextra", "-Wno-unused-parameter"]
    cmd += [os.path.join(CSRC, f) for f in HOST_SOURCES]
    cmd += [os.path.join(ROOT, "tests", "c", "launcher_stubs.cpp"), os.path.join(ROOT, "tests", "c", "host_fuzz.cpp"), "-o", exe]
    res = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    assert res.returncode == 0, res.stderr[-3000:]
    return exe


@pytest.mark.parametrize("seed,cases", [(1, 700), (2, 700), (20250527, 700)])
def test_host_fuzz_under_asan_and_ubsan(fuzz_binary, seed, cases):
    # (a preloaded library in the environment would otherwise make ASan refuse to start: it wants to come first)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([fuzz_binary, str(seed), str(cases)], capture_output=True, text=True, timeout=600, env=env)
    assert res.returncode == 0, (res.stdout[-500:], res.stderr[-3000:])
    assert res.stdout.startswith("cases %d planned" % cases)
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr and "LeakSanitizer" not in res.stderr


def test_shared_layouts_and_plans_from_many_threads_under_tsan(tmp_path):
    """Layouts (with their lock-free cache of gather choices) and plans are shared by eight threads that query,
    plan and launch against the stub launchers; every answer must equal the single-threaded one and
    ThreadSanitizer must stay silent."""
    exe = str(tmp_path / "host_threads")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=thread", "-fno-omit-frame-pointer", "-pthread", "-Wall", "-Wextra",
           "-Wno-unused-parameter"]
    cmd += [os.path.join(CSRC, f) for f in HOST_SOURCES]
    cmd += [os.path.join(ROOT, "tests", "c", "launcher_stubs.cpp"), os.path.join(ROOT, "tests", "c", "host_threads.cpp"), "-o", exe]
    res = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    assert res.returncode == 0, res.stderr[-3000:]
    env = dict(os.environ, TSAN_OPTIONS="halt_on_error=0:exitcode=66")
    res = subprocess.run([exe, "8", "30"], capture_output=True, text=True, timeout=600, env=env)
    assert res.returncode == 0, (res.stdout[-500:], res.stderr[-3000:])
    assert res.stdout.startswith("threads 8 rounds 30") and res.stdout.strip().endswith("mismatches 0")
    assert "ThreadSanitizer" not in res.stderr
