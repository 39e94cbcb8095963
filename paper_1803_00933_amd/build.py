"""Builds ``libapex_replay.so`` (HIP, gfx950) next to this file.  Cross-compiles without a GPU."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libapex_replay.so")
SOURCES = [os.path.join(HERE, "csrc", "apex_replay.hip")]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    # every fp32 rounding on the priority -> mass path is written out by hand
    "-ffp-contract=off",
    # keep the compiler from forming packed fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
]


LIB_HOSTSAN = os.path.join(HERE, "libapex_replay_hostsan.so")
# host code only (the -Xarch_host prefix keeps the sanitizers away from the device pass), shared runtime
HOSTSAN_FLAGS = ["-O1", "-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                 "-Xarch_host", "-fno-sanitize-recover=undefined", "-shared-libsan"]


def build_library(verbose=False, sanitize_host=False):
    """sanitize_host: a second library, same sources, whose HOST code runs under AddressSanitizer and
    UndefinedBehaviorSanitizer (for the CPU-only argument-check tests; the process that loads it needs clang's
    AddressSanitizer runtime preloaded, see asan_runtime())."""
    out = LIB_HOSTSAN if sanitize_host else LIB
    flags = [f for f in FLAGS if f != "-O3"] + HOSTSAN_FLAGS if sanitize_host else FLAGS
    tmp = out + ".tmp.%d" % os.getpid()
    cmd = [HIPCC] + flags + ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"), "-o", tmp] + SOURCES
    if verbose:
        print(" ".join(cmd))
    subprocess.check_call(cmd)
    os.replace(tmp, out)
    return out


def asan_runtime():
    """Path of the AddressSanitizer runtime that belongs to hipcc's host compiler."""
    return subprocess.check_output([HIPCC, "-print-file-name=libclang_rt.asan-x86_64.so"], text=True).strip()


if __name__ == "__main__":
    print(build_library(verbose=True))
