"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU): the oracle's C code (its pins are run
once more in a child process that loads the sanitized build) and the host side of the HIP library (the CPU-only
tests of its exports and argument checks, against a build whose host code is sanitized).  Any out-of-bounds
access, use after free, signed overflow, misaligned access or invalid shift ends the child with a report."""
import glob
import os
import subprocess
import sys

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_pins_pass_under_asan_and_ubsan():
    so = oracle.build(sanitize=True)
    assert os.path.exists(so)
    asan = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    assert os.path.isabs(asan) and os.path.exists(asan), "no AddressSanitizer runtime beside gcc"
    env = dict(os.environ)
    env[oracle.SANITIZE_ENV] = "1"
    env["LD_PRELOAD"] = ":".join(x for x in (env.get("LD_PRELOAD", ""), asan) if x)
    # the interpreter itself is not instrumented: no leak report at its exit, and other preloads may come first
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0:exitcode=99"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    files = sorted(glob.glob(os.path.join(ROOT, "tests", "test_oracle_*.py")))
    assert len(files) >= 5
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + files,
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    out = r.stdout + r.stderr
    assert "AddressSanitizer" not in out and "runtime error:" not in out, out[-4000:]
    assert r.returncode == 0, out[-4000:]
    assert " passed" in r.stdout and "libapex_oracle_san" not in out


def test_library_host_code_passes_its_cpu_tests_under_asan_and_ubsan():
    from paper_1803_00933_amd import build
    so = build.build_library(sanitize_host=True)
    asan = build.asan_runtime()
    assert os.path.isabs(asan) and os.path.exists(asan), "no AddressSanitizer runtime beside hipcc's host compiler"
    env = dict(os.environ)
    env["APEX_REPLAY_LIB"] = so
    env["LD_PRELOAD"] = ":".join(x for x in (env.get("LD_PRELOAD", ""), asan) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0:exitcode=99"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_abi.py")],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    out = r.stdout + r.stderr
    assert "AddressSanitizer" not in out and "runtime error:" not in out, out[-4000:]
    assert r.returncode == 0, out[-4000:]
    assert " passed" in r.stdout
