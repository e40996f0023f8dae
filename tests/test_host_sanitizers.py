"""The host half of the library (argument checks, the launch planner, classification, cache bookkeeping)
under AddressSanitizer and UndefinedBehaviorSanitizer: the library is built a second time with the
sanitizers on the host side only (device code is untouched) and the CPU tests that call into it are run
against that build in a child process.  No GPU is needed: none of these tests launches a kernel."""
import glob
import os
import subprocess
import sys

import pytest

from paper_2601_20499_amd import build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HOST_TESTS = ["tests/test_abi.py", "tests/test_workloads_vs_oracle.py"]
SANITIZE = ["-g", "-fno-omit-frame-pointer", "-shared-libsan",
            "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
            "-Xarch_host", "-fno-sanitize-recover=undefined"]


def _asan_runtime():
    found = sorted(glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so"))
    return found[-1] if found else None


def test_host_code_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    runtime = _asan_runtime()
    if runtime is None:
        pytest.skip("the toolchain ships no shared AddressSanitizer runtime")
    lib = str(tmp_path / "libdf_hip_sanitized.so")
    subprocess.run(build.hipcc_command(out=lib, extra=SANITIZE), check=True, cwd=build.CSRC,
                   stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
    needed = subprocess.run(["ldd", lib], capture_output=True, text=True).stdout
    assert "libclang_rt.asan" in needed, "the build is not instrumented"
    env = dict(os.environ)
    # the sanitizer runtime has to come first among the preloaded libraries; whatever is there stays
    env["LD_PRELOAD"] = ":".join(x for x in (runtime, env.get("LD_PRELOAD", "")) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:halt_on_error=1"      # the interpreter itself is not leak-clean
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env["DF_HIP_LIBRARY"] = lib
    check = ("from paper_2601_20499_amd import binding as b; import sys; "
             "sys.exit(0 if b.LIB_PATH.endswith('libdf_hip_sanitized.so') and b.lib is not None else 3)")
    assert subprocess.run([sys.executable, "-c", check], env=env, cwd=ROOT).returncode == 0
    r = subprocess.run([sys.executable, "-m", "pytest", "-q", "-x", "-p", "no:cacheprovider", *HOST_TESTS],
                       env=env, cwd=ROOT, capture_output=True, text=True, timeout=900)
    report = r.stdout[-3000:] + r.stderr[-3000:]
    assert r.returncode == 0, report
    assert "runtime error" not in report and "AddressSanitizer" not in report, report
