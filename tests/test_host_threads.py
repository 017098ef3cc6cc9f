"""Thread-safety of the host-side pool (paper Sec. 3.1: mutex-guarded free list, blocking acquire with timeout).

Compiles the pool's C++ together with a small stress driver under ThreadSanitizer (host code only, no GPU) and
runs it: concurrent acquire / alias / append / trim / release from six threads must neither race nor break an
invariant, and every cell must be back in the allocator at the end."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.parametrize("sanitizer", ["thread", "address,undefined"])
def test_pool_stress_under_sanitizers(tmp_path, sanitizer):
    cxx = shutil.which("g++")
    if cxx is None:
        pytest.skip("no host C++ compiler")
    exe = str(tmp_path / "pool_stress")
    cmd = [cxx, "-std=c++17", "-O1", "-g", f"-fsanitize={sanitizer}", "-pthread",
           os.path.join(ROOT, "tests", "pool_stress.cpp"),
           os.path.join(ROOT, "paper_2605_26289_amd", "csrc", "pool.cpp"), "-o", exe]
    built = subprocess.run(cmd, capture_output=True, text=True)
    if built.returncode != 0 and "sanitizer" in built.stderr.lower() and "cannot find" in built.stderr.lower():
        pytest.skip("sanitizer runtime not installed")
    assert built.returncode == 0, built.stderr[-2000:]
    env = dict(os.environ, TSAN_OPTIONS="halt_on_error=1", ASAN_OPTIONS="detect_leaks=1")
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    if run.returncode != 0 and "runtime does not come first" in run.stderr:
        pytest.skip("another preloaded library keeps the sanitizer runtime from loading first")
    assert run.returncode == 0, (run.stdout[-2000:], run.stderr[-3000:])
    assert "failures 0 held 0" in run.stdout


def test_radix_traffic_under_address_and_undefined_sanitizers(tmp_path):
    """The radix prefix cache (node splits, leaf evictions, donor hand-over) on the real pool under ASan/UBSan."""
    cxx = shutil.which("g++")
    if cxx is None:
        pytest.skip("no host C++ compiler")
    exe = str(tmp_path / "radix_stress")
    csrc = os.path.join(ROOT, "paper_2605_26289_amd", "csrc")
    cmd = [cxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-pthread",
           os.path.join(ROOT, "tests", "radix_stress.cpp"), os.path.join(csrc, "radix.cpp"),
           os.path.join(csrc, "pool.cpp"), "-o", exe]
    built = subprocess.run(cmd, capture_output=True, text=True)
    if built.returncode != 0 and "sanitizer" in built.stderr.lower() and "cannot find" in built.stderr.lower():
        pytest.skip("sanitizer runtime not installed")
    assert built.returncode == 0, built.stderr[-2000:]
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300,
                         env=dict(os.environ, ASAN_OPTIONS="detect_leaks=1"))
    if run.returncode != 0 and "runtime does not come first" in run.stderr:
        pytest.skip("another preloaded library keeps the sanitizer runtime from loading first")
    assert run.returncode == 0, (run.stdout[-2000:], run.stderr[-3000:])
    assert "failures 0" in run.stdout
