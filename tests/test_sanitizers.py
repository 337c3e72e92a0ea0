"""Host code under the address and undefined-behaviour sanitizers, without a GPU: the C oracle
(gcc) runs its pin tests, and the host side of the HIP library -- argument validation, launch
planning, tile map, with the kernel launchers stubbed out -- runs the ABI tests.  Each build is
loaded into a child interpreter with its sanitizer runtime preloaded; a report makes the child
fail."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run_child(env_extra, preload, tests, tmp):
    env = dict(os.environ, **env_extra)
    env["LD_PRELOAD"] = " ".join(p for p in (preload, os.environ.get("LD_PRELOAD", "")) if p)
    # leak checking would report the interpreter's own allocations
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:exitcode=77"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu"] + tests
    r = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, (r.stdout[-3000:], r.stderr[-3000:])
    assert "passed" in r.stdout


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_pins_under_asan_and_ubsan(tmp_path):
    lib = str(tmp_path / "libtess_oracle_san.so")
    subprocess.run(["gcc", "-O1", "-g", "-fopenmp", "-fPIC", "-shared", "-std=gnu11",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                    "-o", lib, os.path.join(ROOT, "oracle", "tess_oracle.c"), "-lm"], check=True)
    rt = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True, check=True).stdout.strip()
    _run_child({"TESS_ORACLE_LIB": lib}, os.path.realpath(rt), ["tests/test_oracle_pins.py"], tmp_path)


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs the ROCm compiler")
def test_host_dispatcher_under_asan_and_ubsan(tmp_path):
    lib = str(tmp_path / "libtesseract_host_san.so")
    csrc = os.path.join(ROOT, "paper_2105_14500_amd", "csrc")
    hip_root = os.path.join(os.path.dirname(os.path.realpath(shutil.which("hipcc"))), "..")
    clang = os.path.join(hip_root, "lib", "llvm", "bin", "clang++")
    if not os.path.exists(clang):
        hip_root, clang = "/opt/rocm", "/opt/rocm/llvm/bin/clang++"
    # plain C++ (no device code): the HIP runtime header is used for its host declarations only
    subprocess.run([clang, "-x", "c++", "-D__HIP_PLATFORM_AMD__", "-O1", "-g", "-std=c++17", "-fPIC", "-shared",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-shared-libsan",
                    "-I", os.path.join(hip_root, "include"), "-I", os.path.join(ROOT, "include"), "-I", csrc,
                    os.path.join(csrc, "tess_api.cpp"), os.path.join(ROOT, "tests", "host_stubs.cpp"),
                    "-o", lib, "-L" + os.path.join(hip_root, "lib"), "-lamdhip64"], check=True, capture_output=True)
    rt = subprocess.run([clang, "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True,
                        check=True).stdout.strip()
    assert os.path.exists(rt), rt
    _run_child({"TESS_LIB_PATH": lib}, rt, ["tests/test_abi_host.py", "tests/test_plan_coverage.py"], tmp_path)
