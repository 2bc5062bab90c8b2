"""The host-side C and C++ code under the address and undefined-behaviour sanitizers, on the CPU:
(1) the oracle (oracle/*.c, gcc) through its own pins, (2) the host side of libmmvseg (argument checks, workspace
layouts, tile plans: everything the C ABI does before a launch), built with hipcc with the sanitizers on the host
pass only, through the host-only ABI tests.  Each runs in a child process that has the matching sanitizer run-time
preloaded; a report of either sanitizer ends the child with a non-zero status."""
import os
import subprocess
import sys

import pytest

from conftest import ROOT


def _preload(env, lib):
    env = dict(env)
    env["LD_PRELOAD"] = lib + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:exitcode=97"      # (the interpreter itself leaks)
    env["UBSAN_OPTIONS"] = "halt_on_error=1:exitcode=98:print_stacktrace=1"
    return env


def _gcc_runtime(name):
    path = subprocess.run(["gcc", "-print-file-name=" + name], capture_output=True, text=True).stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def test_oracle_under_address_and_undefined_behaviour_sanitizers():
    asan = _gcc_runtime("libasan.so")
    if asan is None:
        pytest.skip("gcc has no libasan here")
    env = _preload(os.environ, asan)
    env["MMVSEG_ORACLE_SANITIZE"] = "1"
    res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                          "tests/test_oracle_pins.py", "tests/test_oracle_primitives.py", "tests/test_oracle_xor.py",
                          "tests/test_host_threads.py", "tests/test_formulations.py"],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=1500)
    assert res.returncode == 0, res.stdout[-3000:] + res.stderr[-3000:]
    assert "passed" in res.stdout and "ERROR: AddressSanitizer" not in res.stderr and "runtime error" not in res.stderr


def test_library_host_code_under_sanitizers(tmp_path):
    from paper_2506_23906_amd import build
    rt = None
    for root, _, files in os.walk("/opt/rocm/lib/llvm/lib/clang"):
        if "libclang_rt.asan-x86_64.so" in files:
            rt = os.path.join(root, "libclang_rt.asan-x86_64.so")
    if rt is None:
        pytest.skip("the HIP compiler ships no address sanitizer run-time here")
    lib = str(tmp_path / "libmmvseg_san.so")
    build.build(extra=["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                       "-Xarch_host", "-fno-sanitize-recover=undefined", "-shared-libsan", "-g"], out=lib)
    code = ("import sys, pytest\n"
            "from paper_2506_23906_amd import binding\n"
            "binding.LIB_PATH = %r\n"
            "sys.exit(pytest.main(['-x', '-q', '-p', 'no:cacheprovider', 'tests/test_abi.py']))\n" % lib)
    res = subprocess.run([sys.executable, "-c", code], cwd=ROOT, env=_preload(os.environ, rt), capture_output=True,
                         text=True, timeout=1500)
    assert res.returncode == 0, res.stdout[-3000:] + res.stderr[-3000:]
    assert "passed" in res.stdout and "ERROR: AddressSanitizer" not in res.stderr and "runtime error" not in res.stderr
