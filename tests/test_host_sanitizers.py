"""Host-side sanitizer runs (AddressSanitizer + UndefinedBehaviorSanitizer), CPU only.

The C oracle and the HOST code of the HIP library (argument validation, workspace and sub-layer planning, the
cost model) are built with -fsanitize=address,undefined and driven, each in a process of its own that preloads the
matching sanitizer runtime, through tests/host_sanitizer_driver.py.  No GPU sanitizer is involved and no kernel is
launched: every library call in the driver is a host-only query or stops in argument validation.
"""
import os
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
DRIVER = os.path.join(HERE, "host_sanitizer_driver.py")


def _run(kind, lib, runtime):
    if not os.path.exists(runtime):
        pytest.skip(f"sanitizer runtime {runtime} not found")
    env = dict(os.environ)
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:exitcode=99"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    r = subprocess.run([sys.executable, DRIVER, kind, lib], env=env, capture_output=True, text=True, timeout=600)
    report = r.stdout[-2000:] + r.stderr[-4000:]
    assert r.returncode == 0, report
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, report
    assert "no sanitizer report" in r.stdout


def test_oracle_under_host_sanitizers():
    from oracle import build as ob
    lib = ob.build_sanitized()
    rt = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    _run("oracle", lib, os.path.realpath(rt))


def test_library_host_code_under_host_sanitizers():
    from paper_1606_05688_amd import build as hb
    lib = hb.build_host_sanitized()
    rt = "/opt/rocm/lib/llvm/lib/clang/22/lib/linux/libclang_rt.asan-x86_64.so"
    if not os.path.exists(rt):
        import glob
        found = glob.glob("/opt/rocm*/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
        rt = found[0] if found else rt
    _run("znni", lib, rt)
