"""The C ABI from a plain C program (tests/c_abi/abi_check.c): HIP runtime only, no Python, no PyTorch in the
process.  The program is compiled here with gcc (it is plain C) against include/mlpo.h and the HIP runtime's C
header, linked with the library and with the oracle, and run as one child process."""
import os
import shutil
import subprocess

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_plain_c_program_matches_the_oracle(oracle, tmp_path):
    import oracle as oracle_pkg
    from paper_2509_02480_amd import binding as B
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    if shutil.which("gcc") is None or not os.path.exists(os.path.join(rocm, "include", "hip", "hip_runtime_api.h")):
        pytest.skip("no C compiler or no HIP headers on this machine")
    exe = str(tmp_path / "abi_check")
    libdir = os.path.dirname(B.LIB_PATH)
    oradir = os.path.dirname(oracle_pkg._LIB)
    cmd = ["gcc", "-std=c11", "-D__HIP_PLATFORM_AMD__", os.path.join(ROOT, "tests", "c_abi", "abi_check.c"),
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(rocm, "include"), "-o", exe,
           "-L", libdir, "-lmlpo", "-L", oradir, "-lmlpo_oracle", "-L", os.path.join(rocm, "lib"), "-lamdhip64", "-lm",
           f"-Wl,-rpath,{libdir}", f"-Wl,-rpath,{oradir}", f"-Wl,-rpath,{os.path.join(rocm, 'lib')}"]
    subprocess.check_call(cmd)
    out = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "abi_check ok" in out.stdout
