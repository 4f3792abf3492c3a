"""Host-side sanitizer builds (no GPU): the C oracle and the host half of the library's C ABI
are compiled with -fsanitize=address,undefined and driven by the two small programs under
tests/sanitize/; a third program drives the host entry points from four threads under
-fsanitize=thread. A report from any sanitizer fails the test. GPU code is not instrumented
(device sanitizers are not available); the other translation units are linked as built."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:halt_on_error=1",
           UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1", OMP_NUM_THREADS="2")


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, f"{' '.join(cmd)}\n{r.stdout}\n{r.stderr}"
    return r


def _clean(r):
    out = r.stdout + r.stderr
    assert "AddressSanitizer" not in out and "runtime error" not in out, out


def test_oracle_under_address_and_undefined_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    _run(["gcc", "-std=c99", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
          "-static-libasan", "-static-libubsan", os.path.join(ROOT, "oracle", "moc_oracle.c"),
          os.path.join(SAN, "oracle_paths.c"), "-o", exe, "-lm"])
    r = _run([exe], env=ENV)
    _clean(r)
    assert r.stdout.startswith("ok ")


@pytest.mark.skipif(shutil.which("hipcc") is None or not os.path.exists("/opt/rocm/llvm/bin/clang++"), reason="ROCm toolchain not found")
def test_abi_host_paths_under_address_and_undefined_sanitizers(tmp_path):
    from paper_2508_21058_amd import build as hb
    hb.build()                                                     # the other translation units, as built
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined"]
    obj = str(tmp_path / "moc_api_san.o")
    _run(["hipcc", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-Xclang", "-target-feature",
          "-Xclang", "-packed-fp32-ops", *san, "-c", os.path.join(hb.CSRC, "moc_api.hip"), "-o", obj])
    others = [os.path.join(hb.OBJ, u + ".o") for u in hb.UNITS if u != "moc_api"]
    exe, drv = str(tmp_path / "abi_san"), str(tmp_path / "abi_host_paths.o")
    _run(["/opt/rocm/llvm/bin/clang++", "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined",
          "-fno-sanitize-recover=undefined", "-c", os.path.join(SAN, "abi_host_paths.cpp"), "-o", drv])
    _run(["hipcc", "--offload-arch=gfx950", *san, drv, obj, *others, "-o", exe])
    r = _run([exe], env=ENV)
    _clean(r)
    assert r.stdout.startswith("ok ")


@pytest.mark.skipif(shutil.which("hipcc") is None or not os.path.exists("/opt/rocm/llvm/bin/clang++"), reason="ROCm toolchain not found")
def test_abi_host_paths_from_four_threads_under_thread_sanitizer(tmp_path):
    """The library's host state (per-thread error string, profiling records and the list-tag registry behind
    their mutexes) driven from four threads at once, host side built with -fsanitize=thread."""
    from paper_2508_21058_amd import build as hb
    hb.build()
    san = ["-Xarch_host", "-fsanitize=thread"]
    obj = str(tmp_path / "moc_api_tsan.o")
    _run(["hipcc", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-Xclang", "-target-feature",
          "-Xclang", "-packed-fp32-ops", *san, "-c", os.path.join(hb.CSRC, "moc_api.hip"), "-o", obj])
    others = [os.path.join(hb.OBJ, u + ".o") for u in hb.UNITS if u != "moc_api"]
    exe, drv = str(tmp_path / "abi_tsan"), str(tmp_path / "abi_host_threads.o")
    _run(["/opt/rocm/llvm/bin/clang++", "-O1", "-g", "-std=c++17", "-fsanitize=thread", "-c",
          os.path.join(SAN, "abi_host_threads.cpp"), "-o", drv])
    _run(["hipcc", "--offload-arch=gfx950", *san, drv, obj, *others, "-o", exe])
    r = _run([exe], env=dict(ENV, TSAN_OPTIONS="halt_on_error=1"))
    out = r.stdout + r.stderr
    assert "ThreadSanitizer" not in out, out
    assert r.stdout.startswith("ok ")
