"""Address- and undefined-behaviour-sanitizer builds of the host code, run on the CPU: the C oracle
(gcc) on small ragged problems through every entry point, and the host side of the C ABI (hipcc's
host compiler; the kernel launchers replaced by stubs, since nothing here reaches a launch) through
its validation paths.  Each runs in a child process with the matching sanitizer runtime preloaded;
a finding aborts the child."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests", "sanitizer")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]


def run_child(script, lib, runtime):
    env = dict(os.environ)
    env["LD_PRELOAD"] = " ".join(x for x in (runtime, env.get("LD_PRELOAD", "")) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"       # the interpreter itself leaks by design
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    res = subprocess.run([sys.executable, os.path.join(HERE, script), lib, ROOT], env=env, stdout=subprocess.PIPE,
                         stderr=subprocess.STDOUT, text=True, timeout=600)
    assert res.returncode == 0 and "sanitizer walk done" in res.stdout, res.stdout[-4000:]
    assert "runtime error" not in res.stdout and "AddressSanitizer" not in res.stdout, res.stdout[-4000:]


def test_oracle_under_asan_and_ubsan(tmp_path):
    lib = str(tmp_path / "libpskv_oracle_san.so")
    subprocess.run(["gcc", *SAN, "-std=c11", "-fopenmp", "-fPIC", "-shared", "-fno-fast-math", "-o", lib,
                    os.path.join(ROOT, "oracle", "pskv_oracle.c"), "-lm"], check=True)
    runtime = subprocess.run(["gcc", "-print-file-name=libasan.so"], stdout=subprocess.PIPE, text=True, check=True).stdout.strip()
    if not os.path.isabs(runtime):
        pytest.skip("gcc's AddressSanitizer runtime is not installed")
    run_child("drive_oracle.py", lib, runtime)


def test_api_host_side_under_asan_and_ubsan(tmp_path):
    lib = str(tmp_path / "libpskv_api_san.so")
    # host code only: every -fsanitize goes to the host compiler (-Xarch_host); no device code is involved
    san = [x for f in SAN for x in (("-Xarch_host", f) if f.startswith("-fsanitize") or f.startswith("-fno-sanitize") else (f,))]
    cmd = [HIPCC, "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared", "-x", "hip", *san, "-o", lib,
           os.path.join(ROOT, "paper_2603_13420_amd", "csrc", "pskv_api.cpp"), os.path.join(HERE, "launch_stubs.cpp")]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout[-4000:]
    clang = os.path.join(os.path.dirname(os.path.realpath(HIPCC)), "..", "lib", "llvm", "bin", "clang")
    runtime = subprocess.run([clang, "-print-file-name=libclang_rt.asan-x86_64.so"], stdout=subprocess.PIPE, text=True,
                             check=True).stdout.strip()
    if not os.path.isabs(runtime):
        pytest.skip("clang's AddressSanitizer runtime is not installed")
    run_child("drive_api.py", lib, runtime)
