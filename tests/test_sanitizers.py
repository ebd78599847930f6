"""Host-side sanitizer runs (no GPU): the C oracle and the library's host code (argument checks,
split planning, workspace layout) built with -fsanitize=address,undefined, then the oracle's pins
and the ABI tests run against those builds in a child process with the sanitizer runtime
preloaded.  Device code is not instrumented."""
import glob
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _gcc_runtime(name):
    path = subprocess.run(["gcc", f"-print-file-name={name}"], capture_output=True, text=True).stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def _run_pytest_child(env_extra, files, select=None):
    env = dict(os.environ)
    env.update(env_extra)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:halt_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider", *files]
    if select:
        cmd += ["-k", select]
    return subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)


def test_oracle_pins_under_address_and_undefined_sanitizers(tmp_path):
    asan, ubsan = _gcc_runtime("libasan.so"), _gcc_runtime("libubsan.so")
    if not asan or not ubsan:
        pytest.skip("gcc sanitizer runtimes not installed")
    lib = str(tmp_path / "libls_oracle_san.so")
    subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-Wall", "-Wextra", "-o", lib,
                    os.path.join(ROOT, "oracle", "ls_oracle.c"), "-lm"], check=True)
    r = _run_pytest_child({"LS_ORACLE_LIB": lib, "LD_PRELOAD": f"{asan}:{ubsan}"},
                          ["tests/test_oracle_pins.py", "tests/test_oracle_accept_pins.py"])
    assert r.returncode == 0, (r.stdout[-3000:], r.stderr[-3000:])
    assert "passed" in r.stdout and "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr


def test_library_host_code_under_address_and_undefined_sanitizers(tmp_path):
    rt = glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    if not rt:
        pytest.skip("clang address-sanitizer runtime not installed")
    from paper_2502_17421_amd import build as ls_build
    lib = str(tmp_path / "libls_attn_san.so")
    flags = [f for f in ls_build.FLAGS if f != "-O3"]
    cmd = [ls_build.HIPCC, *flags, "-O1", "-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host",
           "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all", "-shared-libsan", "-o", lib,
           *ls_build.sources()]
    subprocess.run(cmd, check=True, capture_output=True)
    # (the test that links a C program against the in-tree library by name is not part of this run)
    r = _run_pytest_child({"LS_ATTN_LIB": lib, "LD_PRELOAD": rt[0]}, ["tests/test_abi.py"],
                          select="not plain_c_program")
    assert r.returncode == 0, (r.stdout[-3000:], r.stderr[-3000:])
    assert "passed" in r.stdout and "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr
