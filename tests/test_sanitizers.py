"""Host-side sanitizers: the CPU oracle, and the host part of the C-ABI library (argument checks,
launch logic), are rebuilt with AddressSanitizer and UndefinedBehaviorSanitizer and driven through
the existing CPU tests in a child interpreter that has the sanitizer runtime preloaded.  Any report
aborts the child.  GPU code is never instrumented (there is no GPU sanitizer on this platform)."""
import glob
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _gcc_runtime(name):
    path = subprocess.run(["gcc", "-print-file-name=" + name], capture_output=True, text=True).stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def _run(env_extra, args, timeout=900):
    env = dict(os.environ)
    env.update(env_extra)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:halt_on_error=1"      # the interpreter itself leaks by design
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *args], cwd=ROOT, env=env,
                          capture_output=True, text=True, timeout=timeout)


def test_oracle_pins_under_asan_and_ubsan():
    asan = _gcc_runtime("libasan.so")
    if asan is None:
        pytest.skip("gcc's AddressSanitizer runtime is not installed")
    files = sorted(glob.glob(os.path.join(ROOT, "tests", "test_oracle_*.py")))
    r = _run({"TA_ORACLE_SANITIZE": "1", "LD_PRELOAD": asan}, files)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
    assert " passed" in r.stdout and "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr


def test_abi_argument_checks_under_host_asan_and_ubsan():
    rts = glob.glob("/opt/rocm/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    if not rts:
        pytest.skip("clang's AddressSanitizer runtime is not installed")
    from paper_2604_11288_amd import build as lib_build
    lib = lib_build.build_lib(host_sanitizers=True)
    r = _run({"TA_LIBTA_PATH": lib, "LD_PRELOAD": rts[0]}, [os.path.join(ROOT, "tests", "test_abi.py")])
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
    assert " passed" in r.stdout and "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr
