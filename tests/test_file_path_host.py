"""Host logic of the file path (reader / writer threads, bounce-buffer reuse, error propagation) on the CPU: the
library's filetier.hip is host-only C++, so it is compiled here with g++ against a stub of the HIP header and driven by
tests/host_logic/file_path_harness.cpp - once plainly and once under ThreadSanitizer."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HL = os.path.join(ROOT, "tests", "host_logic")
CSRC = os.path.join(ROOT, "paper_2509_02480_amd", "csrc")


@pytest.mark.parametrize("sanitizer", ["", "thread"])
def test_file_path_threads(tmp_path, sanitizer):
    if shutil.which("g++") is None:
        pytest.skip("no g++")
    exe = str(tmp_path / "harness")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-I", os.path.join(HL, "stubs"), "-I", CSRC, "-I",
           os.path.join(ROOT, "include"), "-x", "c++", os.path.join(HL, "file_path_harness.cpp"),
           os.path.join(CSRC, "filetier.hip"), "-o", exe, "-lpthread"]
    if sanitizer:
        cmd.insert(1, f"-fsanitize={sanitizer}")
    build = subprocess.run(cmd, capture_output=True, text=True)
    if build.returncode != 0 and sanitizer:
        pytest.skip("this toolchain cannot build with -fsanitize=" + sanitizer)
    assert build.returncode == 0, build.stderr
    out = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "all cases ok" in out.stdout and "ThreadSanitizer" not in out.stderr
