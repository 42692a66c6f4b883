"""Compile the HIP sources under csrc/ into paper_1606_05688_amd/libznni.so for gfx950 (in-tree build)."""
import glob
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJDIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libznni.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# Packed-fp32 VALU instructions are switched off for all device code (known-bad forms on the test machines).
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


# Per-file additions.  The batch multiply-accumulate combines matrix-core results with vector instructions after
# every product; with the accumulators in the separate accumulator registers that costs one move per value each
# way (a quarter of the kernel's vector instructions), so its matrix instructions are kept in the VGPR form.
EXTRA_FLAGS = {"mac_batch.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"]}


def _compile(src: str) -> str:
    obj = os.path.join(OBJDIR, os.path.basename(src) + ".o")
    extra = EXTRA_FLAGS.get(os.path.basename(src), [])
    subprocess.run([HIPCC, *FLAGS, *extra, "-c", src, "-o", obj], check=True)
    return obj


def build(verbose: bool = False) -> str:
    os.makedirs(OBJDIR, exist_ok=True)
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        objs = list(ex.map(_compile, srcs))
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    if verbose:
        print(LIB)
    return LIB


LIB_HOST_SANITIZED = os.path.join(OBJDIR, "libznni_hostsan.so")


def build_host_sanitized() -> str:
    """The library with its HOST code (argument validation, workspace and sub-layer planning, cost model, launch
    set-up) under AddressSanitizer and UndefinedBehaviorSanitizer; device code as usual.  For host-only checks
    (tests/test_host_sanitizers.py): no GPU sanitizer is involved."""
    os.makedirs(OBJDIR, exist_ok=True)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]

    def one(src):
        obj = os.path.join(OBJDIR, os.path.basename(src) + ".san.o")
        extra = EXTRA_FLAGS.get(os.path.basename(src), [])
        subprocess.run([HIPCC, *FLAGS, *extra, *san, "-c", src, "-o", obj], check=True)
        return obj

    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        objs = list(ex.map(one, srcs))
    # (link: host sanitizer runtimes only, never the GPU one)
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-sanitize", "-fsanitize=address",
                    "-fsanitize=undefined", "-o", LIB_HOST_SANITIZED, *objs], check=True)
    return LIB_HOST_SANITIZED


if __name__ == "__main__":
    build(verbose=True)
