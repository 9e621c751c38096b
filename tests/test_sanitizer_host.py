"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU involved).

Two small C programs (tests/sanitize/) are built with -fsanitize=address,undefined and run:
  - the fp64 oracle, compiled from source together with a driver that feeds it ragged batches
    (single tokens, empty sequences, key counts of 0, negative and beyond the sequence) and
    re-checks the invariants its pins rest on (rows of P sum to one, rows of dS to zero);
  - the C ABI's host-side validation: the library is rebuilt with the sanitizers on its host
    code (the device code is compiled as usual and never runs here) and every refusal path is
    called with real host allocations of exactly the promised sizes.
The sanitizers end a run at the first finding; the programs print "ok" as their last line."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=600, **kw)
    assert r.returncode == 0, "%s\n%s\n%s" % (" ".join(cmd), r.stdout[-3000:], r.stderr[-6000:])
    return r.stdout


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not found")
def test_oracle_under_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_driver")
    run(["gcc", "-std=c11", "-fopenmp", *SAN, "-o", exe, os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"),
         os.path.join(ROOT, "oracle", "fmha_oracle.c"), "-lm"])
    out = run([exe], env=dict(ENV, ASAN_OPTIONS="detect_leaks=1"))
    assert out.strip().endswith("ok")


@pytest.mark.skipif(not os.path.exists("/opt/rocm/bin/hipcc"), reason="hipcc not found")
def test_abi_validation_under_sanitizers(tmp_path):
    from paper_2208_08124_amd import build
    lib = str(tmp_path / "libfmha_varlen_san.so")
    host_san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                "-Xarch_host", "-fno-sanitize-recover=undefined"]
    flags = [f for f in build.HIPCC_FLAGS if f != "-O3"]
    run(["/opt/rocm/bin/hipcc", *flags, "-O1", "-g", *host_san, "-o", lib, *build.sources()])
    exe = str(tmp_path / "abi_driver")
    run(["/opt/rocm/llvm/bin/clang", *SAN, "-I" + os.path.join(ROOT, "include"), "-o", exe,
         os.path.join(ROOT, "tests", "sanitize", "abi_driver.c"), lib,
         "-Wl,-rpath," + str(tmp_path), "-Wl,-rpath,/opt/rocm/lib"])
    out = run([exe], env=ENV)
    assert out.strip().endswith("ok")
