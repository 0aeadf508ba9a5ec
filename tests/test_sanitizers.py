"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only; no GPU code is instrumented):
the C oracle, and the host side of libtcr.so -- validation, the tuning table's parser and printer, the dispatch
names, the workspace bound -- each driven by a small C program of tests/sanitize/.  A sanitizer report makes the
program exit with a failure."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests", "sanitize")
CLANG = "/opt/rocm/llvm/bin/clang"
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:verify_asan_link_order=0:abort_on_error=0:halt_on_error=1",
           UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def _run(cmd, **kw):
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert proc.returncode == 0, " ".join(cmd) + "\n" + proc.stdout[-4000:]
    return proc.stdout


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_driver")
    _run(["gcc", "-O1", "-g", "-std=c11", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-o", exe,
          os.path.join(HERE, "oracle_driver.c"), os.path.join(ROOT, "oracle", "tcr_oracle.c"), "-lm"])
    assert _run([exe], env=ENV).strip().endswith("ok")


@pytest.mark.skipif(not (os.path.exists(CLANG) and shutil.which(HIPCC)), reason="needs the ROCm compilers")
def test_library_host_code_under_sanitizers(tmp_path):
    from paper_1811_09736_amd import build
    lib = str(tmp_path / "libtcr_sanitized.so")
    flags = [f for f in build.HIPCC_FLAGS if f != "-O3"]
    host = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all",
            "-Xarch_host", "-g", "-O1", "-shared-libsan"]
    _run([HIPCC] + flags + host + ["-o", lib] + build.sources())
    exe = str(tmp_path / "abi_driver")
    _run([CLANG, "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-shared-libsan", "-o", exe,
          os.path.join(HERE, "abi_driver.c"), lib, "-Wl,-rpath," + str(tmp_path),
          "-Wl,-rpath," + os.path.dirname(_runtime())])
    # leak checking off here: the HIP runtime keeps allocations of its own until the process ends
    env = dict(ENV, ASAN_OPTIONS=ENV["ASAN_OPTIONS"].replace("detect_leaks=1", "detect_leaks=0"))
    assert _run([exe], env=env).strip().endswith("ok")


def _runtime():
    out = subprocess.run([CLANG, "-print-file-name=libclang_rt.asan-x86_64.so"], stdout=subprocess.PIPE, text=True).stdout.strip()
    return out
