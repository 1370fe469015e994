"""Builds libreshard.so (plan builder + HIP kernels + swap path) for gfx950."""

from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libreshard.so")
SOURCES = ["plan.cpp", "repack.hip", "api.cpp"]


def _compile(out: str, defines, verbose: bool) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = out + ".tmp%d" % os.getpid()
    cmd = [
        hipcc, "-O3", "--offload-arch=gfx950", "-std=c++17", "-shared", "-fPIC",
        # keep the compiler from forming packed-fp32 instructions
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(HERE, "csrc"),
        "-o", tmp,
    ] + ["-D" + d for d in defines] + [os.path.join(HERE, "csrc", s) for s in SOURCES]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building " + os.path.basename(out))
    os.replace(tmp, out)
    return out


def build_library(verbose: bool = False) -> str:
    """Compiles every source with hipcc, always (no staleness check)."""
    return _compile(LIB, [], verbose)


COUNT_LIB = os.path.join(ROOT, "tests", "libreshard_count_writes.so")


def build_count_library(verbose: bool = False) -> str:
    """A TEST build of the same sources in which every store of the repack kernels counts instead of
    storing (RESHARD_COUNT_WRITES): run on zeroed shadow buffers it leaves, per destination byte, how
    often the real kernels would have written it.  Lives under tests/; the product never loads it."""
    return _compile(COUNT_LIB, ["RESHARD_COUNT_WRITES"], verbose)


C_CLIENT_SRC = os.path.join(ROOT, "tests", "c_abi_gpu_client.c")
C_CLIENT = os.path.join(ROOT, "tests", "c_abi_gpu_client")


def build_c_client() -> str:
    """The plain-C GPU client used by the GPU tests (gcc, C99; links the library and the HIP runtime)."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    tmp = C_CLIENT + ".tmp%d" % os.getpid()
    cmd = ["gcc", "-std=c99", "-O1", "-Wall", "-Wextra", "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(rocm, "include"),
           C_CLIENT_SRC, "-o", tmp, "-L" + HERE, "-l:libreshard.so", "-L" + os.path.join(rocm, "lib"), "-lamdhip64",
           "-Wl,-rpath,$ORIGIN/../paper_2507_19017_amd", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        print(res.stdout)
        print(res.stderr)
        raise RuntimeError("gcc failed building the C client")
    os.replace(tmp, C_CLIENT)
    return C_CLIENT


def ensure_built() -> None:
    """For tests, smoke() and bench.py: build what is missing, leave what is there alone.
    The binding never calls this: without a built library the product refuses to load."""
    if not os.path.exists(LIB):
        build_library()
    if not os.path.exists(C_CLIENT):
        build_c_client()
    if not os.path.exists(COUNT_LIB):
        build_count_library()


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_c_client())
    print(build_count_library())
