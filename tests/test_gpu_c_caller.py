"""The C ABI from a plain C program (no Python binding, no PyTorch in the process): device memory
from the HIP runtime, rounds through librps.so, results checked inside the program."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.dirname(os.path.abspath(__file__))


def test_plain_c_caller(tmp_path):
    lib_dir = os.path.join(ROOT, "paper_1810_07766_amd")
    assert os.path.exists(os.path.join(lib_dir, "librps.so")), "build the library first"
    exe = str(tmp_path / "c_caller")
    subprocess.run(["gcc", "-std=c99", "-O1", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(ROOT, "include"),
                    "-I", "/opt/rocm/include", os.path.join(HERE, "c_abi_round_trip.c"), "-o", exe,
                    os.path.join(lib_dir, "librps.so"), "-L/opt/rocm/lib", "-lamdhip64", "-lm",
                    f"-Wl,-rpath,{lib_dir}", "-Wl,-rpath,/opt/rocm/lib"], check=True)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and "c caller ok" in r.stdout, f"{r.stdout}\n{r.stderr}"
