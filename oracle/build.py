"""Compile the CPU oracle (plain C, gcc) into oracle/libznni_ref.so.

Test infrastructure only: building the checker is not using it.  No -march flag is given, so the
library built in one container also runs on a host with a different CPU.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRCS = [os.path.join(HERE, "znni_ref.c"), os.path.join(HERE, "znni_ref_mpf.c")]
LIB = os.path.join(HERE, "libznni_ref.so")
LIB_SANITIZED = os.path.join(HERE, "libznni_ref_san.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(s) for s in SRCS):
        return LIB
    cmd = ["gcc", "-O3", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", LIB, *SRCS]
    subprocess.run(cmd, check=True)
    return LIB


def build_sanitized() -> str:
    """The same sources under AddressSanitizer and UndefinedBehaviorSanitizer (host checks of the oracle's indexing;
    loaded by tests/test_host_sanitizers.py in a process that preloads the sanitizer runtime)."""
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
           "-o", LIB_SANITIZED, *SRCS]
    subprocess.run(cmd, check=True)
    return LIB_SANITIZED


if __name__ == "__main__":
    print(build())
