"""AddressSanitizer + UndefinedBehaviorSanitizer builds of everything that runs on the host: the C
oracle (gcc) and the host side of the C-ABI library (hipcc, sanitizers on the host pass only; the
device code is compiled as usual and never launched here).  Each build is exercised by the CPU tests
that use it, in a child process with the sanitizer runtime preloaded; any report aborts the child."""
import glob
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run_tests(files, env_extra, preload):
    env = dict(os.environ, **env_extra)
    env["LD_PRELOAD"] = ":".join(preload)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"          # the interpreter itself leaks by design
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    p = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *files], cwd=ROOT, env=env,
                       capture_output=True, text=True, timeout=900)
    assert p.returncode == 0, p.stdout[-3000:] + p.stderr[-3000:]
    assert " passed" in p.stdout


def test_oracle_under_sanitizers(tmp_path):
    rt = [subprocess.check_output(["gcc", f"-print-file-name={n}"], text=True).strip() for n in ("libasan.so", "libubsan.so")]
    if not all(os.path.isabs(r) and os.path.exists(r) for r in rt):
        pytest.skip("gcc's sanitizer runtimes are not installed")
    lib = str(tmp_path / "libevomem_oracle_san.so")
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c11", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
                           "-fsanitize=address,undefined", "-fno-omit-frame-pointer", "-o", lib,
                           os.path.join(ROOT, "oracle", "evomem_oracle.c"), "-lm"])
    _run_tests(["tests/test_oracle_pins.py", "tests/test_parity_checker.py"], {"EVOMEM_ORACLE_LIB": lib}, rt)


def test_c_abi_host_code_under_sanitizers(tmp_path):
    rt = sorted(glob.glob("/opt/rocm/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so"))
    if not rt:
        pytest.skip("clang's sanitizer runtime is not installed")
    from paper_2603_10846_amd import binding
    lib = str(tmp_path / "libevomem_san.so")
    flags = [f for f in binding.HIPCC_FLAGS if f != "-O3"]
    subprocess.check_call(["hipcc", *flags, "-O1", "-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                           "-Xarch_host", "-fno-omit-frame-pointer", "-shared-libsan", "-o", lib, binding.SRC],
                          stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
    _run_tests(["tests/test_host_logic.py"], {"EVOMEM_LIB": lib}, rt[-1:])
