"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only; no GPU code is sanitized):
  - the C oracle, built with gcc's sanitizers, runs its pins (the ones that need no torch),
  - the library's host layer (argument validation, cache handle, dispatch), built by hipcc with the sanitizers
    on the host pass only, runs the C-ABI checks that need no GPU.
Each runs in a subprocess with the matching sanitizer runtime preloaded; any report aborts it."""
import glob
import os
import subprocess
import sys
import textwrap

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ENV = {**os.environ, "ASAN_OPTIONS": "detect_leaks=0:abort_on_error=1", "UBSAN_OPTIONS": "halt_on_error=1:print_stacktrace=1"}


def run_under(runtime, script, tmp_path):
    path = tmp_path / "run.py"
    path.write_text(textwrap.dedent(script))
    res = subprocess.run([sys.executable, str(path)], env={**ENV, "LD_PRELOAD": runtime}, capture_output=True, text=True, timeout=600)
    assert res.returncode == 0, res.stdout[-3000:] + res.stderr[-3000:]
    assert "passed" in res.stdout and "ERROR: AddressSanitizer" not in res.stderr and "runtime error" not in res.stderr


def test_oracle_pins_under_asan_ubsan(tmp_path):
    runtime = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(runtime) or not os.path.exists(runtime):
        pytest.skip("gcc's libasan is not installed")
    lib = tmp_path / "liblcsa_oracle_san.so"
    subprocess.run(["gcc", "-O1", "-g", "-fsanitize=address,undefined", "-fno-omit-frame-pointer", "-fopenmp", "-fPIC", "-shared",
                    "-std=c99", "-o", str(lib), os.path.join(ROOT, "oracle", "lcsa_oracle.c"), "-lm"], check=True)
    run_under(runtime, f"""
        import sys
        sys.path.insert(0, {ROOT!r})
        import oracle
        oracle._LIB_PATH = {str(lib)!r}
        oracle.build = lambda force=False: oracle._LIB_PATH
        import pytest
        sys.exit(pytest.main(["-q", "-x", "--noconftest", "-p", "no:cacheprovider", {os.path.join(ROOT, "tests", "test_oracle_pins.py")!r},
                              "-k", "not autograd and not backward_reduces"]))
        """, tmp_path)


def test_host_layer_under_asan_ubsan(tmp_path):
    runtimes = glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    if not runtimes:
        pytest.skip("clang's shared asan runtime is not installed")
    from paper_2510_12747_amd import build as lib_build
    lib = tmp_path / "liblcsa_san.so"
    flags = [f for f in lib_build.FLAGS if f != "-O3"]
    cmd = ["/opt/rocm/bin/hipcc", *flags, "-O1", "-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-omit-frame-pointer", "-shared-libsan", "-o", str(lib),
           *[os.path.join(lib_build.CSRC, s) for s in lib_build.SOURCES]]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-3000:]
    run_under(runtimes[0], f"""
        import sys
        sys.path.insert(0, {ROOT!r})
        from paper_2510_12747_amd import binding as B
        B.LIB_PATH = {str(lib)!r}
        import pytest
        sys.exit(pytest.main(["-q", "-x", "--noconftest", "-p", "no:cacheprovider", {os.path.join(ROOT, "tests", "test_abi_host.py")!r}]))
        """, tmp_path)
