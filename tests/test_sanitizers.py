"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only; sanitizers for GPU code do not exist here).

Two builds, each exercised by the existing CPU tests in a child process that has the sanitizer runtime preloaded:
  * the C oracle (gcc), against its pins;
  * the library's host side (argument validation of every entry point, and the stateful residency pool of
    symph_pool.h), compiled by hipcc with the sanitizers applied to the host pass only, against the ABI tests and the
    pool's event-by-event parity sequences.
A sanitizer report aborts the child, which fails the test with the report in its output."""
import glob
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run_pytest_under(runtime: str, extra_env: dict, files):
    env = dict(os.environ, **extra_env)
    # the sanitizer runtime has to come first among the preloaded libraries; whatever is preloaded already stays
    env["LD_PRELOAD"] = runtime + (" " + os.environ["LD_PRELOAD"] if os.environ.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"      # the interpreter's own allocations are not ours
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *files], cwd=ROOT, env=env,
                       capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, f"under the sanitizers:\n{r.stdout[-3000:]}\n{r.stderr[-3000:]}"
    assert "passed" in r.stdout


def test_oracle_under_asan_and_ubsan(tmp_path):
    # the oracle's own source, unchanged, as a second library that only this job's child process loads
    lib = str(tmp_path / "liboracle_san.so")
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-fno-omit-frame-pointer",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-o", lib,
                           os.path.join(ROOT, "oracle", "symph_oracle.c"), "-lm"])
    runtime = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    if not os.path.isabs(runtime) or not os.path.exists(runtime):
        pytest.skip("gcc has no AddressSanitizer runtime here")
    _run_pytest_under(runtime, {"ORACLE_LIBRARY_PATH": lib}, ["tests/test_oracle_pins.py"])


def test_library_host_code_under_asan_and_ubsan(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    runtimes = glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    if not os.path.exists(hipcc) or not runtimes:
        pytest.skip("hipcc or its AddressSanitizer runtime is not installed")
    from paper_2412_16434_amd import build as hip_build
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-sanitize-recover=undefined"]
    flags = [f for f in hip_build.HIPCC_FLAGS if f != "-O3"] + ["-O1", "-g"] + san
    objs, procs = [], []
    for src in hip_build.SOURCES:
        obj = str(tmp_path / (os.path.splitext(src)[0] + ".o"))
        procs.append(subprocess.Popen([hipcc, *flags, "-I", os.path.join(ROOT, "include"), "-I", hip_build.CSRC, "-c",
                                       os.path.join(hip_build.CSRC, src), "-o", obj], stdout=subprocess.PIPE,
                                      stderr=subprocess.STDOUT, text=True))
        objs.append(obj)
    for pr in procs:
        out, _ = pr.communicate()
        assert pr.returncode == 0, out[-3000:]
    lib = str(tmp_path / "libsymph_san.so")
    subprocess.check_call([hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", *san, "-shared-libsan", "-o", lib, *objs],
                          stderr=subprocess.DEVNULL)
    _run_pytest_under(runtimes[0], {"SYMPH_LIBRARY_PATH": lib}, ["tests/test_abi.py", "tests/test_pool_parity.py"])
