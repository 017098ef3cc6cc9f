"""The attend planner's work decomposition (host C++, no GPU): compiles the planner together with a checker
and runs it.  Every (row, key) pair must be covered by exactly one work item, rows whose keys were split must
have a merge record, and the chains the streaming kernel's workgroups walk must hold every (item, KV head)
unit exactly once and finish together, also when the XCDs differ in speed."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2605_26289_amd", "csrc")


@pytest.mark.parametrize("sanitizer", [None, "address,undefined"])
def test_plan_covers_every_row_and_key_once_and_balances_chains(tmp_path, sanitizer):
    cxx = shutil.which("g++")
    if cxx is None:
        pytest.skip("no host C++ compiler")
    exe = str(tmp_path / "plan_check")
    flags = [f"-fsanitize={sanitizer}"] if sanitizer else []
    cmd = [cxx, "-std=c++17", "-O1", "-g", "-pthread", *flags, os.path.join(ROOT, "tests", "plan_check.cpp"),
           os.path.join(CSRC, "plan.cpp"), os.path.join(CSRC, "pool.cpp"), "-o", exe]
    built = subprocess.run(cmd, capture_output=True, text=True)
    if built.returncode != 0 and sanitizer and "cannot find" in built.stderr.lower():
        pytest.skip("sanitizer runtime not installed")
    assert built.returncode == 0, built.stderr[-3000:]
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    if run.returncode != 0 and sanitizer and "runtime does not come first" in run.stderr:
        pytest.skip("another preloaded library keeps the sanitizer runtime from loading first")
    assert run.returncode == 0, (run.stdout[-3000:], run.stderr[-2000:])
    assert "failures 0" in run.stdout
