"""Host-side sanitizer leg (CPU only): the CPU oracle and the host half of the HIP library's C ABI
run under AddressSanitizer and UndefinedBehaviorSanitizer.

The sanitizer runtimes are linked statically into small driver programs (tests/sanitize_*_driver.c),
so nothing has to be preloaded into the Python process.  GPU code is not instrumented (not
available on the test machines); kernels are covered by the parity tests instead."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.dirname(os.path.abspath(__file__))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def _run(exe):
    r = subprocess.run([exe], capture_output=True, text=True, env=ENV, timeout=300)
    assert r.returncode == 0, f"{exe} failed under the sanitizers:\n{r.stdout}\n{r.stderr}"
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr
    return r.stdout


def test_oracle_under_asan_and_ubsan(tmp_path):
    """Every oracle entry point over edge shapes, instrumented; same checksums as the plain build."""
    src = [os.path.join(ROOT, "oracle", "rps_oracle.c"), os.path.join(HERE, "sanitize_oracle_driver.c")]
    common = ["gcc", "-std=c11", "-O1", "-ffp-contract=off", "-fopenmp", "-Wall", "-Wextra"]
    san = str(tmp_path / "oracle_san")
    plain = str(tmp_path / "oracle_plain")
    subprocess.run(common + SAN + ["-static-libasan", "-static-libubsan"] + src + ["-o", san, "-lm"], check=True)
    subprocess.run(common + src + ["-o", plain, "-lm"], check=True)
    out_san, out_plain = _run(san), _run(plain)
    assert out_san == out_plain and out_san.count("\n") == 8, (out_san, out_plain)


def test_abi_host_paths_under_asan_and_ubsan(tmp_path):
    """The C-ABI translation unit rebuilt with the host sanitizers (device code untouched, linked with
    the regular kernel object), driven through every path that returns before the first GPU call."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    csrc = os.path.join(ROOT, "paper_1810_07766_amd", "csrc")
    kernels_o = os.path.join(csrc, "rps_kernels.o")
    if not os.path.exists(kernels_o):
        from paper_1810_07766_amd import build
        build.build()
    api_o = str(tmp_path / "rps_api_san.o")
    lib = str(tmp_path / "librps_san.so")
    host_san = []
    for flag in ("-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all"):
        host_san += ["-Xarch_host", flag]
    subprocess.run([hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-ffp-contract=off",
                    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", *host_san,
                    "-c", os.path.join(csrc, "rps_api.hip"), "-o", api_o], check=True, capture_output=True)
    subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined",
                    "-shared-libsan", kernels_o, api_o, "-o", lib], check=True, capture_output=True)
    exe = str(tmp_path / "abi_san")
    clang = os.path.join(os.path.dirname(os.path.realpath(hipcc)), "..", "lib", "llvm", "bin", "clang")
    if not os.path.exists(clang):
        clang = "/opt/rocm/lib/llvm/bin/clang"
    subprocess.run([clang, "-std=c99", "-O1", "-g", "-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all",
                    "-shared-libsan", "-I", os.path.join(ROOT, "include"), os.path.join(HERE, "sanitize_abi_driver.c"),
                    "-o", exe, lib, f"-Wl,-rpath,{tmp_path}", "-lm"], check=True, capture_output=True)
    env = dict(ENV)
    r = subprocess.run([clang, "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True)
    rt_dir = os.path.dirname(r.stdout.strip())
    env["LD_LIBRARY_PATH"] = rt_dir + os.pathsep + env.get("LD_LIBRARY_PATH", "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0"     # the HIP runtime keeps process-lifetime allocations
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, f"{run.stdout}\n{run.stderr}"
    assert "abi host paths ok" in run.stdout
    assert "runtime error" not in run.stderr and "ERROR: AddressSanitizer" not in run.stderr, run.stderr
